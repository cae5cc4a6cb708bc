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

// G += g      (12 bytes of traffic per parameter)
__global__ __launch_bounds__(STREAM_BLOCK) void accumulate_kernel(float* __restrict__ G,
                                                                  const float* __restrict__ g, long n4) {
    const long stride = (long)gridDim.x * STREAM_BLOCK;
    long i = (long)blockIdx.x * STREAM_BLOCK + threadIdx.x;
    f32x4* G4 = (f32x4*)G;
    const f32x4* g4 = (const f32x4*)g;
    for (; i + 3 * stride < n4; i += 4 * stride) {
        f32x4 a0 = G4[i], a1 = G4[i + stride], a2 = G4[i + 2 * stride], a3 = G4[i + 3 * stride];
        f32x4 b0 = __builtin_nontemporal_load(&g4[i]);
        f32x4 b1 = __builtin_nontemporal_load(&g4[i + stride]);
        f32x4 b2 = __builtin_nontemporal_load(&g4[i + 2 * stride]);
        f32x4 b3 = __builtin_nontemporal_load(&g4[i + 3 * stride]);
        G4[i] = a0 + b0;
        G4[i + stride] = a1 + b1;
        G4[i + 2 * stride] = a2 + b2;
        G4[i + 3 * stride] = a3 + b3;
    }
    for (; i < n4; i += stride) G4[i] = G4[i] + g4[i];
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
template <class T>
__global__ __launch_bounds__(STREAM_BLOCK) void adam_kernel(float* __restrict__ theta, float* __restrict__ m,
                                                            float* __restrict__ v, float* __restrict__ G,
                                                            T* __restrict__ version_out, long n4,
                                                            AdamScalars hp) {
    typedef typename Pack4<T>::type out4;
    const long stride = (long)gridDim.x * STREAM_BLOCK;
    f32x4* th4 = (f32x4*)theta;
    f32x4* m4 = (f32x4*)m;
    f32x4* v4 = (f32x4*)v;
    f32x4* G4 = (f32x4*)G;
    out4* o4 = (out4*)version_out;
    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
    for (long i = (long)blockIdx.x * STREAM_BLOCK + threadIdx.x; i < n4; i += stride) {
        f32x4 t = th4[i], mm = m4[i], vv = v4[i], gg = G4[i];
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
        th4[i] = t; m4[i] = mm; v4[i] = vv; G4[i] = zero;
        o4[i] = o;
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
__global__ __launch_bounds__(STREAM_BLOCK) void copy16_kernel(u32x4* __restrict__ dst,
                                                              const u32x4* __restrict__ src, long n16) {
    const long stride = (long)gridDim.x * STREAM_BLOCK;
    long i = (long)blockIdx.x * STREAM_BLOCK + threadIdx.x;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u32x4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
        dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
    }
    for (; i < n16; i += stride) dst[i] = src[i];
}
__global__ __launch_bounds__(STREAM_BLOCK) void copy4_kernel(uint32_t* __restrict__ dst,
                                                             const uint32_t* __restrict__ src, long n4b) {
    const long stride = (long)gridDim.x * STREAM_BLOCK;
    for (long i = (long)blockIdx.x * STREAM_BLOCK + threadIdx.x; i < n4b; i += stride) dst[i] = src[i];
}
__global__ __launch_bounds__(STREAM_BLOCK) void zero16_kernel(u32x4* __restrict__ dst, long n16) {
    const long stride = (long)gridDim.x * STREAM_BLOCK;
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (long i = (long)blockIdx.x * STREAM_BLOCK + threadIdx.x; i < n16; i += stride) dst[i] = z;
}

inline int stream_grid(long n4) {
    long blocks = (n4 + STREAM_BLOCK - 1) / STREAM_BLOCK;
    const long cap = 256 * 8;   // 256 CUs x 8 workgroups
    return (int)(blocks < cap ? (blocks > 0 ? blocks : 1) : cap);
}

}  // namespace amdp
