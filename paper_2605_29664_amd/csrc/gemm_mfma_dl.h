// bf16 GEMM on the matrix cores with tiles loaded from global memory STRAIGHT
// INTO LDS (global_load_lds_dwordx4): no staging registers, no LDS-write
// instructions, and the data of a tile is in flight for a whole k-tile of
// matrix work. Same tiling, fragment double buffering, XCD-aware tile order and
// epilogue as gemm_mfma_kernel; plain problems only (no batch, no causal band).
// Measured on MI355X against the register-staged kernel: the four-wave 128x128
// tile is 7-18 % faster in every layout once more than one workgroup per compute
// unit is resident; the 256x256 tile gains 1-5 % for NT and TN and loses up to
// 18 % for NN on wide-N shapes, so the stage keeps the staged kernel there.
//
// One such load moves 64 lanes x 16 bytes = 1 KB to consecutive LDS addresses
// (lane l's 16 bytes land at base + 16 l), so a tile row cannot be padded.
// Bank conflicts are avoided by a swizzle instead, which costs nothing at load
// time (a lane simply fetches the piece of memory that belongs at the LDS
// position it writes) and a few precomputed lane offsets at read time:
//   * k-contiguous operand, tile [rows][64 k], 128 bytes per row = 8 chunks of
//     16 bytes: chunk c of row r sits at chunk position c ^ ((r >> 1) & 7); a
//     128-bit fragment read by 16 consecutive rows touches all 64 banks once;
//   * m/n-contiguous operand, tile [64 k][R], R*2 bytes per row: the 64-byte
//     block b of row k sits at block position b ^ (k & 3); the transposing read
//     of half a wave (4 consecutive k, 64 bytes each) touches all banks once.
#pragma once
#include "gemm_mfma.h"

namespace amdp {

// 16 bytes per lane from global memory to LDS: lane l's data lands at
// lds_addr + 16 l (lds_addr uniform, it travels in M0). Written as an asm
// statement on purpose: with the compiler's own builtin its wait-count pass
// puts a full vmcnt(0) wait in front of every transposing LDS read that follows
// (it cannot tell that those read the other LDS stage), which serialises the
// loads with the matrix work. The waits that are needed are written out below:
// vmcnt(0) before the barrier that publishes a stage.
// M0 is saved and restored around the load, so the statement leaves no
// register the compiler reserves changed.
__device__ __forceinline__ void load16_to_lds(const void* g, lds_u8* lds_addr) {
    unsigned saved_m0;
    asm volatile("s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
                 : "=&s"(saved_m0)
                 : "s"((unsigned)(__UINTPTR_TYPE__)lds_addr), "v"(g)
                 : "memory");
}

// One operand's tile: R rows (m or n) by 64 k. NW = waves in the workgroup.
template <int R, bool KM, int NW>
struct DlTile {
    static constexpr int BYTES = R * MF_BK * 2;
    static constexpr int ROWB = KM ? R * 2 : MF_BK * 2;       // bytes per LDS row
    static constexpr int CHUNK_ROWS = 1024 / ROWB;            // LDS rows per 1 KB load
    static constexpr int PW = BYTES / 1024 / NW;              // loads per wave
    static_assert(BYTES % (1024 * NW) == 0, "tile must split into whole 1 KB loads per wave");
    static_assert(NW % 2 == 0 && (!KM || R == 128 || R == 256), "swizzle terms assume these shapes");

    // Byte offset from the tile's first element (row 0, k 0) of what this lane
    // fetches in pass 0; rs = elements between consecutive m/n rows, ks =
    // elements between consecutive k.
    // `valid` = rows of the tile that exist (a multiple of 64; R except in a
    // ragged last tile). Rows beyond it are never stored, so their LDS content
    // may be anything: a lane that would fetch them fetches an existing row
    // instead (same address arithmetic, no access outside the matrix).
    __device__ static __forceinline__ long lane_goff(int wave, int lane, long rs, long ks, int valid = R) {
        if constexpr (!KM) {
            const int row = 8 * wave + (lane >> 3), pos = lane & 7;
            const int f = (row >> 1) & 7;
            return (long)row * rs * 2 + ((pos ^ f) * 16);
        } else {
            const int o = 16 * lane;                          // LDS byte inside the 1 KB chunk
            const int krow = CHUNK_ROWS * wave + o / ROWB, pb = o % ROWB;
            int b = (((pb >> 6) ^ (krow & 3)) << 6) | (pb & 63);
            if (b >= valid * 2) b &= 127;                     // the first 64 rows always exist
            return (long)krow * ks * 2 + b;
        }
    }
    // Pass whose global rows pass p fetches: itself, or (k-contiguous operand, rows of
    // the pass beyond `valid`) the pass that covers the same rows modulo 64.
    __device__ static __forceinline__ int source_pass(int p, int valid) {
        if constexpr (KM) return p;
        else return p * 8 * NW < valid ? p : p % (64 / (8 * NW));
    }
    // pass p adds p * pass_gstride (the swizzle terms do not change with the pass)
    __device__ static __forceinline__ long pass_gstride(long rs, long ks) {
        return KM ? (long)CHUNK_ROWS * NW * ks * 2 : (long)8 * NW * rs * 2;
    }
    __device__ static __forceinline__ long ktile_gstride(long ks) { return KM ? (long)MF_BK * ks * 2 : MF_BK * 2; }

    // Fragment addressing. `origin` = first row of the wave's part of the tile.
    // !KM: index = k-step (4 lane offsets), sub-tile j is an immediate.
    //  KM: index = sub-tile (up to 4 lane offsets), k-step is an immediate.
    __device__ static __forceinline__ int frag_off(int origin, int lane, int idx) {
        if constexpr (!KM) {
            const int r = lane & 31, f = (r >> 1) & 7, half = lane >> 5;
            return (origin + r) * ROWB + (((2 * idx + half) ^ f) * 16);
        } else {
            const int q = lane >> 4, i = lane & 15;
            const int krow = 8 * (q >> 1) + (i >> 2), sx = (i >> 2) & 3;
            const int blk = (origin + 32 * idx) * 2 / 64;
            return krow * ROWB + ((blk ^ sx) << 6) + (16 * (q & 1) + 4 * (i & 3)) * 2;
        }
    }
    // f[] = lds + operand base + frag_off(origin, lane, 0..3)
    __device__ static __forceinline__ bf16x8 frag(lds_u8* const (&f)[4], int stage, int j, int kk) {
        if constexpr (!KM) {
            return *(lds_bf16x8*)(f[kk] + stage + j * 32 * ROWB);
        } else {
            lds_u8* p = f[j] + stage + kk * 16 * ROWB;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * ROWB));
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
    }
};

// EDGE: M and N need only be multiples of 64; the last tile of a row or column
// of tiles is then ragged, loads of its missing rows are redirected (see
// DlTile::lane_goff) and the epilogue skips them.
template <int BM, int BN, bool A_KM, bool B_KM, int WGN, bool EDGE = false>
__global__ __launch_bounds__(128 * WGN) void gemm_mfma_dl_kernel(GemmArgs g) {
    constexpr int NT = 128 * WGN, NW = NT / 64;
    constexpr int WM = BM / 2, WN = BN / WGN;
    constexpr int TM = WM / 32, TN = WN / 32;
    using TA = DlTile<BM, A_KM, NW>;
    using TB = DlTile<BN, B_KM, NW>;
    constexpr int STAGE = TA::BYTES + TB::BYTES;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    lds_u8* lds = (lds_u8*)smem_raw;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WGN, wn = wave % WGN;

    const int tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN, ntiles = tiles_m * tiles_n;
    int pid = blockIdx.x;
    if (ntiles % 8 == 0) pid = (pid % 8) * (ntiles / 8) + pid / 8;
    constexpr int GROUP = 8;
    const int per_group = GROUP * tiles_n;
    const int first_m = (pid / per_group) * GROUP;
    const int gsize = min(tiles_m - first_m, GROUP);
    const int pm = first_m + (pid % per_group) % gsize;
    const int pn = (pid % per_group) / gsize;
    const int m0 = pm * BM, n0 = pn * BN;

    const int valid_m = EDGE ? min(BM, g.M - m0) : BM, valid_n = EDGE ? min(BN, g.N - n0) : BN;
    const char* pa = (const char*)((const bf16*)g.A + (long)m0 * g.a_rs) + TA::lane_goff(wave, lane, g.a_rs, g.a_cs, valid_m);
    const char* pb = (const char*)((const bf16*)g.B + (long)n0 * g.b_cs) + TB::lane_goff(wave, lane, g.b_cs, g.b_rs, valid_n);
    const long a_pass = TA::pass_gstride(g.a_rs, g.a_cs), b_pass = TB::pass_gstride(g.b_cs, g.b_rs);
    const long a_step = TA::ktile_gstride(g.a_cs), b_step = TB::ktile_gstride(g.b_rs);
    auto issue_tile = [&](int stage) {
#pragma unroll
        for (int p = 0; p < TA::PW; ++p)
            load16_to_lds(pa + (EDGE ? TA::source_pass(p, valid_m) : p) * a_pass, lds + stage + (wave + NW * p) * 1024);
#pragma unroll
        for (int p = 0; p < TB::PW; ++p)
            load16_to_lds(pb + (EDGE ? TB::source_pass(p, valid_n) : p) * b_pass, lds + stage + TA::BYTES + (wave + NW * p) * 1024);
        pa += a_step;
        pb += b_step;
    };

    lds_u8* fa[4];
    lds_u8* fb[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
        fa[x] = lds + TA::frag_off(wm * WM, lane, x);
        fb[x] = lds + TA::BYTES + TB::frag_off(wn * WN, lane, x);
    }

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nk = g.K / MF_BK;
    constexpr int NDS = TM * (A_KM ? 2 : 1) + TN * (B_KM ? 2 : 1), NMF = TM * TN, NVM = TA::PW + TB::PW;

    bf16x8 va[2][TM], vb[2][TN];
    auto load_frags = [&](int buf, int stage, int kk) {
#pragma unroll
        for (int i = 0; i < TM; ++i) va[buf][i] = TA::frag(fa, stage, i, kk);
#pragma unroll
        for (int j = 0; j < TN; ++j) vb[buf][j] = TB::frag(fb, stage, j, kk);
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

    // Tiles 0 and 1 travel first; tile kt+2 is issued at the barrier inside
    // iteration kt, when every wave is done with the stage it goes to.
    // s_waitcnt immediate: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8.
    if (nk > 0) issue_tile(0);
    if (nk > 1) {
        issue_tile(STAGE);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (NVM & 15) | ((NVM >> 4) << 14));   // vmcnt(NVM): tile 0 has landed
    } else {
        __builtin_amdgcn_s_waitcnt(0x0F70);                                     // vmcnt(0)
    }
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
        // tile kt+1 has landed (it is the only one in flight) and this wave's reads of
        // the current stage are done: after the barrier the stage can be refilled
        __builtin_amdgcn_s_waitcnt(0);                               // vmcnt(0) expcnt(0) lgkmcnt(0)
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
    void* C = g.C;
    constexpr int SW = WN + 4;
    lds_f32* strip = (lds_f32*)lds + wave * (32 * SW);
    const bool plain_f32 = epilogue_is_plain_f32(g.epi);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        __builtin_amdgcn_wave_barrier();   // wave-private strip: no workgroup barrier needed (see gemm_mfma_kernel)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                strip[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * SW + j * 32 + (lane & 31)] = acc[i][j][v];
        __builtin_amdgcn_wave_barrier();
        if (plain_f32) {
            constexpr int QPR = WN / 4;            // column quads per strip row
            for (int it = 0; it < WN / 8; ++it) {
                const int c = lane + 64 * it;
                const int row = c / QPR, cq = c % QPR;
                const f32x4 v4 = *(lds_f32x4*)(strip + row * SW + cq * 4);
                const long m = m0 + wm * WM + i * 32 + row;
                const long n = n0 + wn * WN + cq * 4;
                if (!EDGE || (m < g.M && n < g.N)) epilogue_store4_f32(g.epi, C, g.ldc, m, n, v4);
            }
            continue;
        }
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
            if (!EDGE || (m < g.M && n < g.N)) epilogue_store8(g.epi, C, g.ldc, m, n, v8);
        }
    }
}

// Conditions beyond mfma_shape_ok: a plain problem, no batch, no causal band.
template <int BM, int BN>
inline bool mfma_dl_shape_ok(const GemmArgs& g, bool a_km, bool b_km) {
    return mfma_shape_ok<BM, BN>(g, a_km, b_km) && g.batch == 1 && g.causal == 0;
}

// The EDGE instantiation's conditions: as mfma_dl_shape_ok, with M and N multiples
// of 64 instead of the tile.
inline bool mfma_dl_edge_shape_ok(const GemmArgs& g, bool a_km, bool b_km) {
    return mfma_shape_ok<64, 64>(g, a_km, b_km) && g.batch == 1 && g.causal == 0;
}

template <int BM, int BN, bool A_KM, bool B_KM, int WGN, bool EDGE = false>
inline hipError_t launch_gemm_mfma_dl(const GemmArgs& g, hipStream_t st) {
    constexpr size_t lds = 2 * (size_t)(BM + BN) * MF_BK * 2;
    static_assert(lds <= 160 * 1024, "tile does not fit the 160 KB LDS of a CDNA4 compute unit");
    constexpr auto kern = gemm_mfma_dl_kernel<BM, BN, A_KM, B_KM, WGN, EDGE>;
    if (hipError_t e = allow_dynamic_lds<kern>((int)lds); e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN)), dim3(128 * WGN), lds, st, g);
    return hipGetLastError();
}

}  // namespace amdp
