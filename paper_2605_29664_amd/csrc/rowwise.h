// Row-wise kernels: LayerNorm forward/backward, masked softmax forward/backward,
// cross-entropy, and the column reductions that produce bias and LayerNorm
// parameter gradients. One 64-lane wavefront owns one row; reductions are
// wave shuffles, statistics and exponentials are fp32, accesses are 16-byte
// vectors along the row. No float atomics: results are run-to-run identical.
#pragma once
#include "common.h"

namespace amdp {

template <class T> struct Vec;
template <> struct Vec<float> { static constexpr int N = 4; };
template <> struct Vec<bf16> { static constexpr int N = 8; };

template <class T>
__device__ __forceinline__ void load_vec(const T* p, float (&out)[Vec<T>::N]) {
    if constexpr (sizeof(T) == 4) {
        f32x4 v = *(const f32x4*)p;
#pragma unroll
        for (int i = 0; i < 4; ++i) out[i] = v[i];
    } else {
        bf16x8 v = *(const bf16x8*)p;
#pragma unroll
        for (int i = 0; i < 8; ++i) out[i] = (float)v[i];
    }
}
template <class T>
__device__ __forceinline__ void store_vec(T* p, const float (&in)[Vec<T>::N]) {
    if constexpr (sizeof(T) == 4) {
        f32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = in[i];
        *(f32x4*)p = v;
    } else {
        bf16x8 v;
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (bf16)in[i];
        *(bf16x8*)p = v;
    }
}

constexpr int ROWS_PER_BLOCK = 4;   // 256 threads

// ------------------------------------------------------------------ LayerNorm
// y = (x - mean) * rstd * gamma + beta, biased variance; stats[2r] = mean, stats[2r+1] = rstd.
template <class T>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                     const T* __restrict__ beta, T* __restrict__ y,
                                                     float* __restrict__ stats, int N, int D, float eps) {
    constexpr int V = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= N) return;
    const T* xr = x + row * D;
    const int nv = D / V;
    float s = 0.f;
    for (int c = lane; c < nv; c += WAVE) {
        float a[V];
        load_vec<T>(xr + c * V, a);
#pragma unroll
        for (int i = 0; i < V; ++i) s += a[i];
    }
    const float mean = wave_sum(s) / (float)D;
    float q = 0.f;
    for (int c = lane; c < nv; c += WAVE) {
        float a[V];
        load_vec<T>(xr + c * V, a);
#pragma unroll
        for (int i = 0; i < V; ++i) { const float d = a[i] - mean; q += d * d; }
    }
    const float rstd = rsqrtf(wave_sum(q) / (float)D + eps);
    if (lane == 0) { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
    T* yr = y + row * D;
    for (int c = lane; c < nv; c += WAVE) {
        float a[V], gm[V], bt[V];
        load_vec<T>(xr + c * V, a);
        load_vec<T>(gamma + c * V, gm);
        load_vec<T>(beta + c * V, bt);
#pragma unroll
        for (int i = 0; i < V; ++i) a[i] = (a[i] - mean) * rstd * gm[i] + bt[i];
        store_vec<T>(yr + c * V, a);
    }
}

// dx = [res +] rstd * (dxhat - mean(dxhat) - xhat * mean(dxhat * xhat)), dxhat = dy * gamma
template <class T>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                     const float* __restrict__ stats,
                                                     const T* __restrict__ gamma, const T* res,
                                                     T* dx, int N, int D) {
    constexpr int V = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= N) return;
    const float mean = stats[2 * row], rstd = stats[2 * row + 1];
    const T* xr = x + row * D;
    const T* dyr = dy + row * D;
    const int nv = D / V;
    float s1 = 0.f, s2 = 0.f;
    for (int c = lane; c < nv; c += WAVE) {
        float a[V], d[V], gm[V];
        load_vec<T>(xr + c * V, a);
        load_vec<T>(dyr + c * V, d);
        load_vec<T>(gamma + c * V, gm);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float dxh = d[i] * gm[i];
            s1 += dxh;
            s2 += dxh * (a[i] - mean) * rstd;
        }
    }
    const float c1 = wave_sum(s1) / (float)D, c2 = wave_sum(s2) / (float)D;
    for (int c = lane; c < nv; c += WAVE) {
        float a[V], d[V], gm[V], r[V];
        load_vec<T>(xr + c * V, a);
        load_vec<T>(dyr + c * V, d);
        load_vec<T>(gamma + c * V, gm);
        if (res) load_vec<T>(res + row * D + c * V, r);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const float xh = (a[i] - mean) * rstd;
            float o = rstd * (d[i] * gm[i] - c1 - xh * c2);
            if (res) o += r[i];
            a[i] = o;
        }
        store_vec<T>(dx + row * D + c * V, a);
    }
}

// ------------------------------------------ LayerNorm, row held in registers
// The same arithmetic with ONE read of every input: a lane keeps its NV
// 16-byte vectors of the row (vector c = lane + 64 i, i < NV; D <= 64 * NV * V)
// in registers as loaded, all loads are issued before the first reduction.
template <class T> struct RawVec;
template <> struct RawVec<float> { typedef f32x4 type; };
template <> struct RawVec<bf16> { typedef bf16x8 type; };

template <class T, int NV>
__global__ __launch_bounds__(256) void ln_fwd_reg_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                         const T* __restrict__ beta, T* __restrict__ y,
                                                         float* __restrict__ stats, int N, int D, float eps) {
    constexpr int V = Vec<T>::N;
    typedef typename RawVec<T>::type raw_t;
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= N) return;
    const int nv = D / V;
    const raw_t* xr = (const raw_t*)(x + row * D);
    raw_t a[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
        if (c < nv) a[i] = xr[c];
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
        if (lane + 64 * i < nv) {
#pragma unroll
            for (int k = 0; k < V; ++k) s += (float)a[i][k];
        }
    const float mean = wave_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
        if (lane + 64 * i < nv) {
#pragma unroll
            for (int k = 0; k < V; ++k) { const float d = (float)a[i][k] - mean; q += d * d; }
        }
    const float rstd = rsqrtf(wave_sum(q) / (float)D + eps);
    if (lane == 0) { stats[2 * row] = mean; stats[2 * row + 1] = rstd; }
    raw_t* yr = (raw_t*)(y + row * D);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
        if (c < nv) {
            const raw_t gm = ((const raw_t*)gamma)[c], bt = ((const raw_t*)beta)[c];
            raw_t o;
#pragma unroll
            for (int k = 0; k < V; ++k) o[k] = (T)(((float)a[i][k] - mean) * rstd * (float)gm[k] + (float)bt[k]);
            yr[c] = o;
        }
    }
}

// Backward with the row in registers: dy, x and gamma are read once.
template <class T, int NV>
__global__ __launch_bounds__(256) void ln_bwd_reg_kernel(const T* __restrict__ dy, const T* __restrict__ x,
                                                         const float* __restrict__ stats,
                                                         const T* __restrict__ gamma, const T* res, T* dx,
                                                         int N, int D) {
    constexpr int V = Vec<T>::N;
    typedef typename RawVec<T>::type raw_t;
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= N) return;
    const int nv = D / V;
    const raw_t* xr = (const raw_t*)(x + row * D);
    const raw_t* dyr = (const raw_t*)(dy + row * D);
    raw_t a[NV], d[NV], gm[NV];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
        if (c < nv) { a[i] = xr[c]; d[i] = dyr[c]; gm[i] = ((const raw_t*)gamma)[c]; }
    }
    const float mean = stats[2 * row], rstd = stats[2 * row + 1];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
        if (lane + 64 * i < nv) {
#pragma unroll
            for (int k = 0; k < V; ++k) {
                const float dxh = (float)d[i][k] * (float)gm[i][k];
                s1 += dxh;
                s2 += dxh * ((float)a[i][k] - mean) * rstd;
            }
        }
    const float c1 = wave_sum(s1) / (float)D, c2 = wave_sum(s2) / (float)D;
    raw_t* dxr = (raw_t*)(dx + row * D);
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        const int c = lane + 64 * i;
        if (c < nv) {
            raw_t r;
            if (res) r = ((const raw_t*)(res + row * D))[c];
            raw_t o;
#pragma unroll
            for (int k = 0; k < V; ++k) {
                const float xh = ((float)a[i][k] - mean) * rstd;
                float v = rstd * ((float)d[i][k] * (float)gm[i][k] - c1 - xh * c2);
                if (res) v += (float)r[k];
                o[k] = (T)v;
            }
            dxr[c] = o;
        }
    }
}

// ----------------------------------------------------------- column reductions
// Stage 1: a block owns 64*VEC consecutive columns and one chunk of rows; its 4
// waves take rows round-robin, every lane keeps VEC column sums in registers
// (16-byte loads along the row), the waves are combined through LDS.
//   LN = false: partial[rc][c]      = sum_r dy[r][c]
//   LN = true : partial[rc][c]      = sum_r dy[r][c] * xhat[r][c]      (dgamma)
//               partial[rc][C + c]  = sum_r dy[r][c]                    (dbeta)
template <class T, bool LN>
__global__ __launch_bounds__(256) void colreduce_partial_kernel(const T* __restrict__ dy,
                                                               const T* __restrict__ x,
                                                               const float* __restrict__ stats,
                                                               float* __restrict__ partial, int N, int C,
                                                               int rows_per_chunk) {
    constexpr int V = Vec<T>::N;
    __shared__ float red[2][4][64 * V];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c0 = (blockIdx.x * 64 + lane) * V;
    const bool live = c0 < C;                       // C is a multiple of V
    const int r0 = blockIdx.y * rows_per_chunk, r1 = min(N, r0 + rows_per_chunk);
    float s[V], sg[V];
#pragma unroll
    for (int i = 0; i < V; ++i) { s[i] = 0.f; sg[i] = 0.f; }
    if (live) {
        // four rows per step: their loads are all in flight before the first addition
        // (rows are added in the same order as one at a time: the sums do not change)
        typedef typename RawVec<T>::type raw_t;
        int r = r0 + wave;
        for (; r + 12 < r1; r += 16) {
            raw_t dv[4], xv[4];
            float mean[4], rstd[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                dv[u] = *(const raw_t*)(dy + (long)(r + 4 * u) * C + c0);
                if constexpr (LN) {
                    xv[u] = *(const raw_t*)(x + (long)(r + 4 * u) * C + c0);
                    mean[u] = stats[2 * (r + 4 * u)];
                    rstd[u] = stats[2 * (r + 4 * u) + 1];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const float dd = (float)dv[u][i];
                    if constexpr (LN) sg[i] += dd * ((float)xv[u][i] - mean[u]) * rstd[u];
                    s[i] += dd;
                }
        }
        for (; r < r1; r += 4) {
            float d[V];
            load_vec<T>(dy + (long)r * C + c0, d);
            if constexpr (LN) {
                float a[V];
                load_vec<T>(x + (long)r * C + c0, a);
                const float mean = stats[2 * r], rstd = stats[2 * r + 1];
#pragma unroll
                for (int i = 0; i < V; ++i) sg[i] += d[i] * (a[i] - mean) * rstd;
            }
#pragma unroll
            for (int i = 0; i < V; ++i) s[i] += d[i];
        }
    }
#pragma unroll
    for (int i = 0; i < V; ++i) {
        red[0][wave][lane * V + i] = s[i];
        if constexpr (LN) red[1][wave][lane * V + i] = sg[i];
    }
    __syncthreads();
    const long width = LN ? 2 * (long)C : C;
    for (int j = threadIdx.x; j < 64 * V; j += 256) {
        const int c = blockIdx.x * 64 * V + j;
        if (c >= C) continue;
        const float t = red[0][0][j] + red[0][1][j] + red[0][2][j] + red[0][3][j];
        if constexpr (LN) {
            partial[blockIdx.y * width + c] = red[1][0][j] + red[1][1][j] + red[1][2][j] + red[1][3][j];
            partial[blockIdx.y * width + C + c] = t;
        } else {
            partial[blockIdx.y * width + c] = t;
        }
    }
}
// ---- several column reductions in one pair of launches ----------------------
// All bias and LayerNorm-parameter gradients of one layer's backward: up to 8
// segments, each a [N, C] matrix dy (LayerNorm segments also x and the row
// statistics) with its own output vector. The partial sums of all segments sit
// side by side in one row of `partial` per row chunk (segment i at column
// woff, width C or 2 C).
struct ColSumSeg {
    const void* dy;
    const void* x;          // null: plain column sums; else LayerNorm input
    const float* stats;
    float* out;
    int C, first_block, woff, width;
};
struct ColSumBatch {
    ColSumSeg seg[8];
    int n, N, rows_per_chunk, width;
};

template <class T>
__global__ __launch_bounds__(256) void colsum_batch_partial_kernel(ColSumBatch b, float* __restrict__ partial) {
    constexpr int V = Vec<T>::N;
    typedef typename RawVec<T>::type raw_t;
    __shared__ float red[2][4][64 * V];
    int si = 0;
    for (int i = 1; i < b.n; ++i)
        if ((int)blockIdx.x >= b.seg[i].first_block) si = i;
    const T* dy = (const T*)b.seg[si].dy;
    const T* x = (const T*)b.seg[si].x;
    const float* stats = b.seg[si].stats;
    const int C = b.seg[si].C, woff = b.seg[si].woff;
    const bool ln = x != nullptr;                   // uniform over the block
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cb = blockIdx.x - b.seg[si].first_block;
    const int c0 = (cb * 64 + lane) * V;
    const bool live = c0 < C;
    const int r0 = blockIdx.y * b.rows_per_chunk, r1 = min(b.N, r0 + b.rows_per_chunk);
    float s[V], sg[V];
#pragma unroll
    for (int i = 0; i < V; ++i) { s[i] = 0.f; sg[i] = 0.f; }
    if (live) {
        int r = r0 + wave;
        for (; r + 12 < r1; r += 16) {              // four rows' loads in flight before the first addition
            raw_t dv[4], xv[4];
            float mean[4], rstd[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                dv[u] = *(const raw_t*)(dy + (long)(r + 4 * u) * C + c0);
                if (ln) {
                    xv[u] = *(const raw_t*)(x + (long)(r + 4 * u) * C + c0);
                    mean[u] = stats[2 * (r + 4 * u)];
                    rstd[u] = stats[2 * (r + 4 * u) + 1];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int i = 0; i < V; ++i) {
                    const float dd = (float)dv[u][i];
                    if (ln) sg[i] += dd * ((float)xv[u][i] - mean[u]) * rstd[u];
                    s[i] += dd;
                }
        }
        for (; r < r1; r += 4) {
            const raw_t dv = *(const raw_t*)(dy + (long)r * C + c0);
            if (ln) {
                const raw_t xv = *(const raw_t*)(x + (long)r * C + c0);
                const float mean = stats[2 * r], rstd = stats[2 * r + 1];
#pragma unroll
                for (int i = 0; i < V; ++i) sg[i] += (float)dv[i] * ((float)xv[i] - mean) * rstd;
            }
#pragma unroll
            for (int i = 0; i < V; ++i) s[i] += (float)dv[i];
        }
    }
#pragma unroll
    for (int i = 0; i < V; ++i) {
        red[0][wave][lane * V + i] = s[i];
        red[1][wave][lane * V + i] = sg[i];
    }
    __syncthreads();
    float* prow = partial + (long)blockIdx.y * b.width + woff;
    for (int j = threadIdx.x; j < 64 * V; j += 256) {
        const int c = cb * 64 * V + j;
        if (c >= C) continue;
        const float t = red[0][0][j] + red[0][1][j] + red[0][2][j] + red[0][3][j];
        if (ln) {
            prow[c] = red[1][0][j] + red[1][1][j] + red[1][2][j] + red[1][3][j];
            prow[C + c] = t;
        } else {
            prow[c] = t;
        }
    }
}

// Second stage over the concatenated width: column j belongs to the segment whose
// [woff, woff + width) holds it and goes to that segment's output vector.
__global__ __launch_bounds__(256) void colsum_batch_final_kernel(ColSumBatch b, const float* __restrict__ partial,
                                                                 int chunks, int accumulate) {
    __shared__ float red[16][17];
    const int j = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int c = blockIdx.x * 16 + j;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (c < b.width) {
        const float* p = partial + c;
        int k = grp;
        for (; k + 48 < chunks; k += 64) {
            s0 += p[(long)k * b.width];
            s1 += p[(long)(k + 16) * b.width];
            s2 += p[(long)(k + 32) * b.width];
            s3 += p[(long)(k + 48) * b.width];
        }
        for (; k < chunks; k += 16) s0 += p[(long)k * b.width];
    }
    red[grp][j] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (grp == 0 && c < b.width) {
        float t = 0.f;
#pragma unroll
        for (int g = 0; g < 16; ++g) t += red[g][j];
        int si = 0;
        for (int i = 1; i < b.n; ++i)
            if (c >= b.seg[i].woff) si = i;
        float* o = b.seg[si].out + (c - b.seg[si].woff);
        *o = accumulate ? *o + t : t;
    }
}

// Stage 2: out[c] = sum over chunks. A block owns 16 columns; its 16 groups of
// 16 threads each sum every 16th chunk (four loads in flight per thread: the
// sums are short, so the kernel lives on memory latency), then the groups are
// added in fixed order. accumulate != 0: out[c] += that sum.
__global__ __launch_bounds__(256) void colreduce_final_kernel(const float* __restrict__ partial,
                                                             float* __restrict__ out, int width, int chunks,
                                                             int accumulate) {
    __shared__ float red[16][17];
    const int j = threadIdx.x & 15, grp = threadIdx.x >> 4;
    const int c = blockIdx.x * 16 + j;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    if (c < width) {
        const float* p = partial + c;
        int k = grp;
        for (; k + 48 < chunks; k += 64) {
            s0 += p[(long)k * width];
            s1 += p[(long)(k + 16) * width];
            s2 += p[(long)(k + 32) * width];
            s3 += p[(long)(k + 48) * width];
        }
        for (; k < chunks; k += 16) s0 += p[(long)k * width];
    }
    red[grp][j] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (grp == 0 && c < width) {
        float t = 0.f;
#pragma unroll
        for (int g = 0; g < 16; ++g) t += red[g][j];
        out[c] = accumulate ? out[c] + t : t;
    }
}

// -------------------------------------------------------------------- softmax
// In place over rows of S [batch*s, s]: P = softmax(scale * S) over the visible
// keys; hidden keys get probability exactly 0. Row r belongs to batch z = r / s,
// query q = r % s, sequence z / H. causal: keys > q hidden. valid_len != null:
// keys >= valid_len[sequence] hidden.
template <class T>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(T* S, long rows, int s, float scale, int causal,
                                                          const int32_t* __restrict__ valid_len, int H) {
    constexpr int V = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int q = (int)(row % s);
    const long z = row / s;
    int limit = s;
    if (causal) limit = q + 1;
    if (valid_len) limit = min(limit, max(0, valid_len[z / H]));
    T* p = S + row * s;
    const int nv = s / V;
    float mx = -INFINITY;
    for (int c = lane; c * V < limit; c += WAVE) {
        float a[V];
        load_vec<T>(p + c * V, a);
#pragma unroll
        for (int i = 0; i < V; ++i) if (c * V + i < limit) mx = fmaxf(mx, a[i]);
    }
    mx = wave_max(mx) * scale;
    float sum = 0.f;
    for (int c = lane; c * V < limit; c += WAVE) {
        float a[V];
        load_vec<T>(p + c * V, a);
#pragma unroll
        for (int i = 0; i < V; ++i) if (c * V + i < limit) sum += __expf(a[i] * scale - mx);
    }
    sum = wave_sum(sum);
    const float inv = sum > 0.f ? 1.0f / sum : 0.f;
    for (int c = lane; c < nv; c += WAVE) {
        float a[V];
        if (c * V < limit) load_vec<T>(p + c * V, a);
#pragma unroll
        for (int i = 0; i < V; ++i) a[i] = (c * V + i < limit) ? __expf(a[i] * scale - mx) * inv : 0.f;
        store_vec<T>(p + c * V, a);
    }
}

// In place on dP: dS = scale * P * (dP - sum_j dP_j P_j) over the visible keys, 0 elsewhere.
template <class T>
__global__ __launch_bounds__(256) void softmax_bwd_kernel(const T* __restrict__ P, T* dP, long rows, int s,
                                                          float scale, int causal,
                                                          const int32_t* __restrict__ valid_len, int H) {
    constexpr int V = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int q = (int)(row % s);
    const long z = row / s;
    int limit = s;
    if (causal) limit = q + 1;
    if (valid_len) limit = min(limit, max(0, valid_len[z / H]));
    const T* p = P + row * s;
    T* d = dP + row * s;
    const int nv = s / V;
    float dot = 0.f;
    for (int c = lane; c * V < limit; c += WAVE) {
        float a[V], b[V];
        load_vec<T>(p + c * V, a);
        load_vec<T>(d + c * V, b);
#pragma unroll
        for (int i = 0; i < V; ++i) if (c * V + i < limit) dot += a[i] * b[i];
    }
    dot = wave_sum(dot);
    for (int c = lane; c < nv; c += WAVE) {
        float a[V], b[V];
        if (c * V < limit) { load_vec<T>(p + c * V, a); load_vec<T>(d + c * V, b); }
#pragma unroll
        for (int i = 0; i < V; ++i) a[i] = (c * V + i < limit) ? scale * a[i] * (b[i] - dot) : 0.f;
        store_vec<T>(d + c * V, a);
    }
}

// -------------------------------------------------------------- cross-entropy
// Row n of logits [N, ld] (V valid columns): row_loss[n] = logsumexp - logit[target];
// logits are overwritten with d loss / d logits = (softmax - onehot) / N, pad columns 0.
template <class T>
__global__ __launch_bounds__(256) void ce_fwd_kernel(T* logits, const int32_t* __restrict__ targets,
                                                     float* __restrict__ row_loss, int N, int Vocab, long ld) {
    constexpr int V = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= N) return;
    T* p = logits + row * ld;
    const int nv = (int)(ld / V);
    const int t = targets[row];
    // maximum and sum of exponentials in ONE pass over the row: each lane keeps a
    // running maximum and rescales its running sum whenever the maximum moves
    float mx = -INFINITY, sum = 0.f, tl = 0.f;
    for (int c = lane; c * V < Vocab; c += WAVE) {
        float a[V];
        load_vec<T>(p + c * V, a);
        float vm = mx;
#pragma unroll
        for (int i = 0; i < V; ++i) if (c * V + i < Vocab) vm = fmaxf(vm, a[i]);
        sum *= (mx == vm) ? 1.f : __expf(mx - vm);   // first vector: exp(-inf) = 0 times a sum of 0
        mx = vm;
#pragma unroll
        for (int i = 0; i < V; ++i) if (c * V + i < Vocab) {
            sum += __expf(a[i] - mx);
            if (c * V + i == t) tl = a[i];
        }
    }
    {
        const float wm = wave_max(mx);
        sum *= (mx == -INFINITY) ? 0.f : __expf(mx - wm);   // a lane that saw no column contributes nothing
        mx = wm;
    }
    sum = wave_sum(sum);
    tl = wave_sum(tl);
    if (lane == 0) row_loss[row] = mx + __logf(sum) - tl;
    const float inv = 1.0f / sum, invN = 1.0f / (float)N;
    for (int c = lane; c < nv; c += WAVE) {
        float a[V];
        if (c * V < Vocab) load_vec<T>(p + c * V, a);
#pragma unroll
        for (int i = 0; i < V; ++i) {
            const int col = c * V + i;
            a[i] = col < Vocab ? (__expf(a[i] - mx) * inv - (col == t ? 1.f : 0.f)) * invN : 0.f;
        }
        store_vec<T>(p + c * V, a);
    }
}

// mean of row losses, one block, fixed order
__global__ __launch_bounds__(256) void mean_kernel(const float* __restrict__ v, float* out, int N) {
    __shared__ float sh[256];
    float s = 0.f;
    for (int i = threadIdx.x; i < N; i += 256) s += v[i];
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) sh[threadIdx.x] += sh[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = sh[0] / (float)N;
}

}  // namespace amdp
