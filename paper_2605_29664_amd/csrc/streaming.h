// Streaming kernels over the stage's flat fp32 buffers: gradient accumulation,
// the fused Adam update (which also publishes the next weight version and
// clears the gradient sum), and the publication of a version from the master.
// All are HBM-bound: 16-byte accesses, grid-stride, several independent loads
// in flight per lane.
#pragma once
#include "common.h"

namespace amdp {

constexpr int STREAM_BLOCK = 256;

// Flat buffers are allocated in multiples of 1024 floats, so every kernel
// here works on whole float4 quads: n4 = number of quads.

// Launch shape of the streaming kernels: ONE 16-byte vector per lane and as
// many small workgroups as that takes. Measured on MI355X over 3.2 GB buffers,
// this beats every grid-stride variant (2048 resident workgroups looping: 4.6
// TB/s for G += g; one vector per lane: 6.1-6.3 TB/s): the dispatcher walks
// memory strictly in address order and each workgroup retires after one
// round trip, which keeps the HBM channels evenly loaded.
constexpr int ACC_BLOCK = 64;

// G += g      (12 bytes of traffic per parameter)
__global__ __launch_bounds__(ACC_BLOCK) void accumulate_kernel(float* __restrict__ G,
                                                               const float* __restrict__ g, long n4) {
    const long i = (long)blockIdx.x * ACC_BLOCK + threadIdx.x;
    if (i >= n4) return;
    f32x4* G4 = (f32x4*)G;
    const f32x4 a = __builtin_nontemporal_load(&G4[i]);
    const f32x4 b = __builtin_nontemporal_load(&((const f32x4*)g)[i]);
    __builtin_nontemporal_store(a + b, &G4[i]);
}

struct AdamScalars {
    float lr, beta1, beta2, eps, weight_decay, grad_scale;
    float omb1, omb2;         // 1-beta1, 1-beta2, formed in double on the host
    float inv_bc1, inv_bc2;   // 1/(1-beta1^t), 1/(1-beta2^t), or 1 without bias correction
};

template <class T> struct Pack4;
template <> struct Pack4<float> { typedef f32x4 type; };
template <> struct Pack4<bf16> { typedef bf16x4 type; };

// theta, m, v updated in place from grad_scale*G; new version written in the
// stage dtype; G cleared.      (34 bytes per parameter with bf16 versions)
// Launch shape measured on 805 M parameters: one-wave workgroups with
// nontemporal loads and stores reach 5.7 TB/s, 256-lane workgroups with plain
// loads 5.35 TB/s; interleaving theta/m/v in memory made no difference.
template <class T>
__global__ __launch_bounds__(ACC_BLOCK) void adam_kernel(float* __restrict__ theta, float* __restrict__ m,
                                                            float* __restrict__ v, float* __restrict__ G,
                                                            T* __restrict__ version_out, long n4,
                                                            AdamScalars hp) {
    typedef typename Pack4<T>::type out4;
    f32x4* th4 = (f32x4*)theta;
    f32x4* m4 = (f32x4*)m;
    f32x4* v4 = (f32x4*)v;
    f32x4* G4 = (f32x4*)G;
    out4* o4 = (out4*)version_out;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    const long i = (long)blockIdx.x * ACC_BLOCK + threadIdx.x;
    if (i < n4) {
        f32x4 t = __builtin_nontemporal_load(&th4[i]), mm = __builtin_nontemporal_load(&m4[i]);
        f32x4 vv = __builtin_nontemporal_load(&v4[i]), gg = __builtin_nontemporal_load(&G4[i]);
        out4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float gh = hp.grad_scale * gg[k];
            const float mn = hp.beta1 * mm[k] + hp.omb1 * gh;
            const float vn = hp.beta2 * vv[k] + hp.omb2 * gh * gh;
            const float mh = mn * hp.inv_bc1, vh = vn * hp.inv_bc2;
            const float tn = t[k] - hp.lr * (mh / (sqrtf(vh) + hp.eps) + hp.weight_decay * t[k]);
            mm[k] = mn; vv[k] = vn; t[k] = tn;
            o[k] = (T)tn;
        }
        __builtin_nontemporal_store(t, &th4[i]);
        __builtin_nontemporal_store(mm, &m4[i]);
        __builtin_nontemporal_store(vv, &v4[i]);
        __builtin_nontemporal_store(zero, &G4[i]);
        o4[i] = o;     // the new version is read again soon: keep it cacheable
    }
}

// version_out = cast(theta)
template <class T>
__global__ __launch_bounds__(STREAM_BLOCK) void publish_kernel(const float* __restrict__ theta,
                                                               T* __restrict__ version_out, long n4) {
    typedef typename Pack4<T>::type out4;
    const long stride = (long)gridDim.x * STREAM_BLOCK;
    const f32x4* th4 = (const f32x4*)theta;
    out4* o4 = (out4*)version_out;
    for (long i = (long)blockIdx.x * STREAM_BLOCK + threadIdx.x; i < n4; i += stride) {
        f32x4 t = th4[i];
        out4 o;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = (T)t[k];
        o4[i] = o;
    }
}

// Plain device-to-device copy and zero fill, used instead of the runtime's
// memcpy/memset so that every byte the library moves is moved by a kernel that
// is ordered on the stage's stream like all its other work. n16 = number of
// 16-byte units.
// One 16-byte vector per lane, 64-lane workgroups, streaming loads and stores:
// the launch shape that measured fastest for the accumulation as well.
__global__ __launch_bounds__(ACC_BLOCK) void copy16_kernel(u32x4* __restrict__ dst,
                                                           const u32x4* __restrict__ src, long n16) {
    const long i = (long)blockIdx.x * ACC_BLOCK + threadIdx.x;
    if (i >= n16) return;
    __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}
__global__ __launch_bounds__(STREAM_BLOCK) void copy4_kernel(uint32_t* __restrict__ dst,
                                                             const uint32_t* __restrict__ src, long n4b) {
    const long stride = (long)gridDim.x * STREAM_BLOCK;
    for (long i = (long)blockIdx.x * STREAM_BLOCK + threadIdx.x; i < n4b; i += stride) dst[i] = src[i];
}
__global__ __launch_bounds__(ACC_BLOCK) void zero16_kernel(u32x4* __restrict__ dst, long n16) {
    const long i = (long)blockIdx.x * ACC_BLOCK + threadIdx.x;
    if (i >= n16) return;
    const u32x4 z = {0u, 0u, 0u, 0u};
    dst[i] = z;
}

// out (+)= partial[0] + partial[1] + ... + partial[parts-1], each of n4 float4, added in that order:
// the second stage of a product whose contraction was split over workgroups.
__global__ __launch_bounds__(ACC_BLOCK) void splitk_reduce_kernel(float* __restrict__ out,
                                                                  const float* __restrict__ partial, long n4,
                                                                  int parts, int accumulate) {
    const long i = (long)blockIdx.x * ACC_BLOCK + threadIdx.x;
    if (i >= n4) return;
    const f32x4* p4 = (const f32x4*)partial;
    f32x4 s = p4[i];
    for (int k = 1; k < parts; ++k) s += p4[(long)k * n4 + i];
    f32x4* o4 = (f32x4*)out;
    if (accumulate) s += o4[i];
    o4[i] = s;
}

// out[m][n] = bf16(partial[0][m][n] + ... + partial[parts-1][m][n] (+ bias[n]) (+ res[m][n])), eight
// columns per lane; n8 = M*N/8, N a multiple of 8, out and res row-major [M, N]. The second stage of a
// bf16-output product whose contraction was split in parts; parts are added in index order.
__global__ __launch_bounds__(ACC_BLOCK) void splitk_epilogue_kernel(bf16* __restrict__ out,
                                                                    const float* __restrict__ partial,
                                                                    const bf16* __restrict__ bias,
                                                                    const bf16* __restrict__ res, long n8, int N,
                                                                    int parts) {
    const long i = (long)blockIdx.x * ACC_BLOCK + threadIdx.x;
    if (i >= n8) return;
    const f32x4* p4 = (const f32x4*)partial;
    f32x4 lo = p4[2 * i], hi = p4[2 * i + 1];
    for (int k = 1; k < parts; ++k) {
        lo += p4[(long)k * 2 * n8 + 2 * i];
        hi += p4[(long)k * 2 * n8 + 2 * i + 1];
    }
    if (bias) {
        const bf16x8 b = *(const bf16x8*)(bias + (i * 8) % N);
#pragma unroll
        for (int k = 0; k < 4; ++k) { lo[k] += (float)b[k]; hi[k] += (float)b[4 + k]; }
    }
    if (res) {
        const bf16x8 r = ((const bf16x8*)res)[i];
#pragma unroll
        for (int k = 0; k < 4; ++k) { lo[k] += (float)r[k]; hi[k] += (float)r[4 + k]; }
    }
    bf16x8 o;
#pragma unroll
    for (int k = 0; k < 4; ++k) { o[k] = (bf16)lo[k]; o[4 + k] = (bf16)hi[k]; }
    ((bf16x8*)out)[i] = o;
}

// grid for the grid-stride helpers (copy, zero, publish)
inline int stream_grid(long n4) {
    long blocks = (n4 + STREAM_BLOCK - 1) / STREAM_BLOCK;
    const long cap = 256 * 64;
    return (int)(blocks < cap ? (blocks > 0 ? blocks : 1) : cap);
}
// grid for the one-vector-per-lane kernels
inline unsigned direct_grid(long n4, int block) { return (unsigned)((n4 + block - 1) / block); }

}  // namespace amdp
