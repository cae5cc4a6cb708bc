// NT GEMM (both operands k-contiguous: dX = dY W^T, logits = z E^T) with tiles
// loaded from global memory STRAIGHT INTO LDS (global_load_lds_dwordx4): no
// staging registers, no LDS-write instructions, and the data of a tile is in
// flight for a whole k-tile of matrix work.
//
// One such load moves 64 lanes x 16 bytes = 1 KB to consecutive LDS addresses
// (lane l's 16 bytes land at base + 16 l), so a tile row cannot be padded.
// A [rows][64 k] bf16 tile is 128 bytes per row = 8 chunks of 16 bytes; chunk c
// of row r is stored at chunk position c ^ ((r >> 1) & 7). A 128-bit fragment
// read by 16 consecutive rows of one chunk then touches all 64 banks once. The
// swizzle costs nothing at load time (the lane that writes position p of row r
// simply fetches chunk p ^ ((r >> 1) & 7) from memory) and four precomputed
// lane offsets per operand at read time (one per k-step).
#pragma once
#include "gemm_mfma.h"

namespace amdp {

typedef __attribute__((address_space(3))) void lds_void;

template <int BM, int BN, int WGN>
__global__ __launch_bounds__(128 * WGN) void gemm_mfma_nt_dl_kernel(GemmArgs g) {
    constexpr int NT = 128 * WGN, NW = NT / 64;
    constexpr int WM = BM / 2, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWB = MF_BK * 2;                       // 128 bytes per tile row
    constexpr int A_BYTES = BM * ROWB, B_BYTES = BN * ROWB, STAGE = A_BYTES + B_BYTES;
    constexpr int A_PW = BM / 8 / NW, B_PW = BN / 8 / NW; // 1 KB chunk loads per wave and operand
    static_assert(BM % (8 * NW) == 0 && BN % (8 * NW) == 0, "tile rows must split into whole chunk loads per wave");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    lds_u8* lds = (lds_u8*)smem_raw;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    const int tiles_m = g.M / BM, tiles_n = g.N / BN, ntiles = tiles_m * tiles_n;
    int pid = blockIdx.x;
    if (ntiles % 8 == 0) pid = (pid % 8) * (ntiles / 8) + pid / 8;
    constexpr int GROUP = 8;
    const int per_group = GROUP * tiles_n;
    const int first_m = (pid / per_group) * GROUP;
    const int gsize = min(tiles_m - first_m, GROUP);
    const int pm = first_m + (pid % per_group) % gsize;
    const int pn = (pid % per_group) / gsize;
    const int m0 = pm * BM, n0 = pn * BN;

    // ---- what this lane fetches: row 8*(wave + NW*p) + lane/8 of the tile, LDS chunk position lane%8
    const int rowl = lane >> 3, pos = lane & 7;
    const int fl = (4 * (wave & 1) + (rowl >> 1)) & 7;    // (row >> 1) & 7; NW is even, so the pass does not change it
    const char* pa = (const char*)((const bf16*)g.A + (long)(m0 + 8 * wave + rowl) * g.a_rs) + ((pos ^ fl) * 16);
    const char* pb = (const char*)((const bf16*)g.B + (long)(n0 + 8 * wave + rowl) * g.b_cs) + ((pos ^ fl) * 16);
    const long a_pass = (long)8 * NW * g.a_rs * 2, b_pass = (long)8 * NW * g.b_cs * 2;
    auto issue_tile = [&](int stage) {
#pragma unroll
        for (int p = 0; p < A_PW; ++p)
            __builtin_amdgcn_global_load_lds(pa + p * a_pass, (lds_void*)(lds + stage + (wave + NW * p) * 1024), 16, 0, 0);
#pragma unroll
        for (int p = 0; p < B_PW; ++p)
            __builtin_amdgcn_global_load_lds(pb + p * b_pass, (lds_void*)(lds + stage + A_BYTES + (wave + NW * p) * 1024), 16, 0, 0);
        pa += MF_BK * 2;
        pb += MF_BK * 2;
    };

    // ---- where this lane reads fragments: row lane%32 of a 32-row group, chunk 2*kk + lane/32
    const int fr = ((lane & 31) >> 1) & 7, half = lane >> 5;
    lds_u8* fa[4];
    lds_u8* fb[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const int off = (lane & 31) * ROWB + (((2 * kk + half) ^ fr) * 16);
        fa[kk] = lds + (wm * WM) * ROWB + off;
        fb[kk] = lds + A_BYTES + (wn * WN) * ROWB + off;
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = g.K / MF_BK;
    constexpr int NDS = TM + TN, NMF = TM * TN, NVM = A_PW + B_PW;

    bf16x8 va[2][TM], vb[2][TN];
    auto load_frags = [&](int buf, int stage, int kk) {
#pragma unroll
        for (int i = 0; i < TM; ++i) va[buf][i] = *(lds_bf16x8*)(fa[kk] + stage + i * 32 * ROWB);
#pragma unroll
        for (int j = 0; j < TN; ++j) vb[buf][j] = *(lds_bf16x8*)(fb[kk] + stage + j * 32 * ROWB);
    };
    auto mfma_step = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[buf][i], vb[buf][j], acc[i][j], 0, 0, 0);
    };
    auto interleave_reads = [&]() {
#pragma unroll
        for (int t = 0; t < NMF; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (t < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (NDS > NMF) __builtin_amdgcn_sched_group_barrier(0x100, NDS - NMF, 0);
    };

    // tiles 0 and 1 travel; tile kt+2 is issued at the barrier inside iteration kt,
    // when every wave is done with the stage it goes to
    if (nk > 0) issue_tile(0);
    if (nk > 1) issue_tile(STAGE);
    // s_waitcnt immediate: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8
    if (nk > 1) __builtin_amdgcn_s_waitcnt(0x0F70 | (NVM & 15) | ((NVM >> 4) << 14));   // vmcnt(NVM): tile 0 has landed
    else __builtin_amdgcn_s_waitcnt(0x0F70);                                           // vmcnt(0)
    __syncthreads();
    if (nk > 0) load_frags(0, 0, 0);

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = (kt & 1) * STAGE, nxt = STAGE - cur;
        load_frags(1, cur, 1);
        mfma_step(0);
        interleave_reads();
        load_frags(0, cur, 2);
        mfma_step(1);
        interleave_reads();
        load_frags(1, cur, 3);
        mfma_step(0);
        interleave_reads();
        // tile kt+1 has landed (it is the only one in flight), this wave's reads of
        // the current stage are done: after the barrier the stage can be refilled
        __builtin_amdgcn_s_waitcnt(0);                              // vmcnt(0) expcnt(0) lgkmcnt(0)
        __syncthreads();
        if (kt + 2 < nk) issue_tile(cur);
        if (kt + 1 < nk) load_frags(0, nxt, 0);
        mfma_step(1);
#pragma unroll
        for (int t = 0; t < NMF; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (t < NVM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            if (t < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
    }
    __syncthreads();

    // Epilogue through LDS, as in gemm_mfma_kernel.
    void* C = g.epi.out_f32 ? (void*)((float*)g.C) : (void*)((bf16*)g.C);
    constexpr int SW = WN + 4;
    lds_f32* strip = (lds_f32*)lds + wave * (32 * SW);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                strip[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * SW + j * 32 + (lane & 31)] = acc[i][j][v];
        __syncthreads();
        constexpr int CPR = WN / 8;
        for (int it = 0; it < WN / 16; ++it) {
            const int c = lane + 64 * it;
            const int row = c / CPR, cc = c % CPR;
            float v8[8];
            const f32x4 lo = *(lds_f32x4*)(strip + row * SW + cc * 8);
            const f32x4 hi = *(lds_f32x4*)(strip + row * SW + cc * 8 + 4);
#pragma unroll
            for (int k = 0; k < 4; ++k) { v8[k] = lo[k]; v8[4 + k] = hi[k]; }
            const long m = m0 + wm * WM + i * 32 + row;
            const long n = n0 + wn * WN + cc * 8;
            epilogue_store8(g.epi, C, g.ldc, m, n, v8);
        }
    }
}

// Conditions beyond mfma_shape_ok: plain NT problem, no batch, no causal band.
template <int BM, int BN>
inline bool mfma_dl_shape_ok(const GemmArgs& g) {
    return mfma_shape_ok<BM, BN>(g, false, false) && g.batch == 1 && g.causal == 0;
}

template <int BM, int BN, int WGN>
inline hipError_t launch_gemm_mfma_nt_dl(const GemmArgs& g, hipStream_t st) {
    constexpr size_t lds = 2 * (size_t)(BM + BN) * MF_BK * 2;
    static_assert(lds <= 160 * 1024, "tile does not fit the 160 KB LDS of a CDNA4 compute unit");
    auto kern = gemm_mfma_nt_dl_kernel<BM, BN, WGN>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3((g.M / BM) * (g.N / BN)), dim3(128 * WGN), lds, st, g);
    return hipGetLastError();
}

}  // namespace amdp
