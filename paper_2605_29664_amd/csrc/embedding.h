// First-stage input layer: x[n] = E[token[n]] + P[n mod s] (token embedding plus
// learned position embedding, the input layer of the GPT / BERT model family of
// Section 4.1), and its gradients. Token ids outside [0, V) are clamped, so
// bad device data cannot cause an out-of-range access.
#pragma once
#include "rowwise.h"

namespace amdp {

__device__ __forceinline__ int clamp_token(int t, int V) { return min(max(t, 0), V - 1); }

// One wave per token row.
template <class T>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const T* __restrict__ E, const T* __restrict__ P,
                                                       const int32_t* __restrict__ tokens, T* __restrict__ x,
                                                       int N, int s, int D, int V) {
    constexpr int VEC = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (row >= N) return;
    const T* e = E + (long)clamp_token(tokens[row], V) * D;
    const T* p = P + (row % s) * D;
    for (int c = lane; c < D / VEC; c += WAVE) {
        float a[VEC], b[VEC];
        load_vec<T>(e + c * VEC, a);
        load_vec<T>(p + c * VEC, b);
#pragma unroll
        for (int i = 0; i < VEC; ++i) a[i] += b[i];
        store_vec<T>(x + row * D + c * VEC, a);
    }
}

// gP[p][:] (+)= sum over the minibatch's sequences of dx[q*s + p][:], fixed order.
template <class T>
__global__ __launch_bounds__(256) void pos_embed_bwd_kernel(const T* __restrict__ dx, float* __restrict__ gP,
                                                           int b, int s, int D, int accumulate) {
    constexpr int VEC = Vec<T>::N;
    const int vpr = D / VEC;
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= (long)s * vpr) return;
    const long p = i / vpr, c = i % vpr;
    float acc[VEC];
#pragma unroll
    for (int k = 0; k < VEC; ++k) acc[k] = 0.f;
    for (int q = 0; q < b; ++q) {
        float a[VEC];
        load_vec<T>(dx + ((long)q * s + p) * D + c * VEC, a);
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[k] += a[k];
    }
    float* o = gP + p * D + c * VEC;
#pragma unroll
    for (int k = 0; k < VEC; ++k) o[k] = accumulate ? o[k] + acc[k] : acc[k];
}

// gE[t][:] (+)= sum of dx[n][:] over the positions n that hold token t, added in
// increasing n (no atomics: the same bits every run). One workgroup per
// position; the workgroup of a token's FIRST occurrence does all of that
// token's rows, the others find an earlier occurrence and leave. Rows of
// tokens that do not occur are not touched (the caller clears them).
// D <= 256 * VEC * MAXI columns.
template <class T, int MAXI>
__global__ __launch_bounds__(256) void tok_embed_bwd_kernel(const T* __restrict__ dx,
                                                           const int32_t* __restrict__ tokens,
                                                           float* __restrict__ gE, int N, int D, int V,
                                                           int accumulate) {
    constexpr int VEC = Vec<T>::N;
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x;
    const int t = clamp_token(tokens[n], V);
    for (int base = 0; base < n; base += 64) {                   // every wave scans alike: uniform exit
        const int pos = base + lane;
        const bool hit = pos < n && clamp_token(tokens[pos], V) == t;
        if (__ballot(hit)) return;
    }
    float acc[MAXI][VEC];
#pragma unroll
    for (int i = 0; i < MAXI; ++i)
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[i][k] = 0.f;
    for (int base = n & ~63; base < N; base += 64) {
        const int pos = base + lane;
        const bool hit = pos >= n && pos < N && clamp_token(tokens[pos], V) == t;
        unsigned long long m = __ballot(hit);
        while (m) {
            const int r = base + __builtin_ctzll(m);
            m &= m - 1;
#pragma unroll
            for (int i = 0; i < MAXI; ++i) {
                const int c = (threadIdx.x + i * 256) * VEC;
                if (c < D) {
                    float a[VEC];
                    load_vec<T>(dx + (long)r * D + c, a);
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[i][k] += a[k];
                }
            }
        }
    }
#pragma unroll
    for (int i = 0; i < MAXI; ++i) {
        const int c = (threadIdx.x + i * 256) * VEC;
        if (c < D) {
            float* o = gE + (long)t * D + c;
#pragma unroll
            for (int k = 0; k < VEC; ++k) o[k] = accumulate ? o[k] + acc[i][k] : acc[i][k];
        }
    }
}

// Both buffers end up holding their element-wise sum (the tie of the input
// embedding and the output projection: two copies of one parameter whose
// gradients add). n4 = number of float4.
__global__ __launch_bounds__(64) void tie_sum_kernel(float* __restrict__ a, float* __restrict__ b, long n4) {
    const long i = (long)blockIdx.x * 64 + threadIdx.x;
    if (i >= n4) return;
    const f32x4 s = ((f32x4*)a)[i] + ((f32x4*)b)[i];
    ((f32x4*)a)[i] = s;
    ((f32x4*)b)[i] = s;
}

}  // namespace amdp
