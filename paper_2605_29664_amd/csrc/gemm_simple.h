// Generic fully-guarded GEMM: any shape, any strides, fp32 FMA arithmetic.
// Used for the fp32 stage configuration and for bf16 shapes that are not
// multiples of the MFMA kernel's tiles.
#pragma once
#include "common.h"

namespace amdp {

constexpr int GS_TILE = 64;   // output tile edge
constexpr int GS_BK = 16;

template <class T>
__global__ __launch_bounds__(256) void gemm_simple_kernel(GemmArgs g) {
    __shared__ float As[GS_BK][GS_TILE + 1];
    __shared__ float Bs[GS_BK][GS_TILE + 1];

    const int z = blockIdx.z;
    const long zo = z / g.batch_inner, zi = z % g.batch_inner;
    const T* A = (const T*)g.A + zo * g.a_bo + zi * g.a_bi;
    const T* B = (const T*)g.B + zo * g.b_bo + zi * g.b_bi;
    const long c_off = zo * g.c_bo + zi * g.c_bi;

    const int m0 = blockIdx.y * GS_TILE, n0 = blockIdx.x * GS_TILE;
    if (g.causal == 1 && n0 > m0 + GS_TILE - 1) return;
    int k_lo = 0, k_hi = g.K;
    if (g.causal == 2) k_hi = min(g.K, m0 + GS_TILE);
    if (g.causal == 3) k_lo = (m0 / GS_BK) * GS_BK;

    const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
    float acc[4][4] = {};

    for (int k0 = k_lo; k0 < k_hi; k0 += GS_BK) {
        // 64x16 elements per operand, 256 threads: 4 each
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int idx = threadIdx.x + i * 256;
            {   // A tile: favour the contiguous direction for coalescing
                int mm, kk;
                if (g.a_cs == 1) { kk = idx % GS_BK; mm = idx / GS_BK; }
                else { mm = idx % GS_TILE; kk = idx / GS_TILE; }
                const int gm = m0 + mm, gk = k0 + kk;
                As[kk][mm] = (gm < g.M && gk < k_hi) ? to_f32(A[(long)gm * g.a_rs + (long)gk * g.a_cs]) : 0.f;
            }
            {
                int nn, kk;
                if (g.b_rs == 1) { kk = idx % GS_BK; nn = idx / GS_BK; }
                else { nn = idx % GS_TILE; kk = idx / GS_TILE; }
                const int gn = n0 + nn, gk = k0 + kk;
                Bs[kk][nn] = (gn < g.N && gk < k_hi) ? to_f32(B[(long)gk * g.b_rs + (long)gn * g.b_cs]) : 0.f;
            }
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < GS_BK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty + 16 * i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx + 16 * j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    void* C = g.epi.out_f32 ? (void*)((float*)g.C + c_off) : (void*)((T*)g.C + c_off);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty + 16 * i;
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx + 16 * j;
            if (n < g.N) epilogue_store<T>(g.epi, C, g.ldc, m, n, acc[i][j]);
        }
    }
}

template <class T>
inline hipError_t launch_gemm_simple(const GemmArgs& g, hipStream_t st) {
    if (g.M <= 0 || g.N <= 0) return hipSuccess;
    dim3 grid((g.N + GS_TILE - 1) / GS_TILE, (g.M + GS_TILE - 1) / GS_TILE, g.batch);
    hipLaunchKernelGGL(gemm_simple_kernel<T>, grid, dim3(256), 0, st, g);
    return hipGetLastError();
}

}  // namespace amdp
