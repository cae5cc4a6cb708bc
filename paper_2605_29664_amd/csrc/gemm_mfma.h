// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32
// accumulation. Tiles are staged through LDS (double buffered); one workgroup
// = 4 wavefronts of 64 lanes arranged 2x2 over the BM x BN output tile.
//
// Operand storage, per template flag:
//   A_KM = false : A is [M][K], k contiguous        (activations, dY)
//   A_KM = true  : A is [K][M], m contiguous        (X^T in dW = X^T dY)
//   B_KM = true  : B is [K][N], n contiguous        (W in Y = X W; dY in dW)
//   B_KM = false : B is [N][K], k contiguous        (W in dX = dY W^T; K in Q K^T)
// The matrix instruction wants, per lane, 8 consecutive k of one row (A) or
// one column (B). k-contiguous operands are read from LDS with one 128-bit
// read. m/n-contiguous operands are kept in LDS as they are in memory and
// read with the transposing LDS read (ds_read_b64_tr_b16), or, with TR =
// false, element by element.
//
// Shapes must be whole tiles: M % BM == 0, N % BN == 0, K % 64 == 0, 16-byte
// aligned rows; anything else takes the generic kernel.
//
// Two main-loop pipelines, chosen by tile size from measurement: tiles up to
// 128x128 (<= 188 VGPRs, two workgroups per compute unit) keep fragments live
// across the barrier so the matrix cores work through it; the 256x256 tile
// (one wave per SIMD, 256 accumulator registers) cannot afford those extra
// live registers and uses the simpler load / compute / store / barrier order.
#pragma once
#include "common.h"

namespace amdp {

constexpr int MF_BK = 64;

// LDS pointers carry their address space so that every access is a ds_*
// instruction with an immediate offset.
typedef __attribute__((address_space(3))) unsigned char lds_u8;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
typedef __attribute__((address_space(3))) bf16x8 lds_bf16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) bf16 lds_bf16;
typedef __attribute__((address_space(3))) float lds_f32;
typedef __attribute__((address_space(3))) f32x4 lds_f32x4;

template <int R, bool KM, int NT = 256>
struct OperandTile {
    // LDS rows are padded so that consecutive rows start 16 bytes (k-contiguous
    // tile: 128-bit reads of 16 rows) or 64 bytes (transposing reads: half a
    // wave reads 4 rows x 64 bytes at a time) further round the 64 banks.
    static constexpr int PAD = KM ? 32 : 8;
    static constexpr int ROWS = KM ? MF_BK : R;
    static constexpr int COLS = (KM ? R : MF_BK) + PAD;
    static constexpr int BYTES = ROWS * COLS * 2;
    static constexpr int NV = R * 8 / NT;           // 16-byte vectors per thread per tile
    static constexpr int VPR = KM ? R / 8 : 8;      // vectors per LDS row
    static constexpr int ROWS_PER_PASS = NT / VPR;  // rows covered by the NT threads in one pass

    // Byte offset, inside the operand, of the first vector this thread loads
    // (row stride rs and k stride ks in elements).
    __device__ static __forceinline__ long thread_goff(int tid, long rs, long ks) {
        const int row = tid / VPR, c = tid % VPR;
        return KM ? ((long)row * ks + c * 8) * 2 : ((long)row * rs + c * 8) * 2;
    }
    // Byte distance between the vectors of consecutive passes.
    __device__ static __forceinline__ long pass_gstride(long rs, long ks) {
        return (KM ? (long)ROWS_PER_PASS * ks : (long)ROWS_PER_PASS * rs) * 2;
    }
    // Byte distance between consecutive k-tiles.
    __device__ static __forceinline__ long ktile_gstride(long ks) { return (KM ? (long)MF_BK * ks : MF_BK) * 2; }
    __device__ static __forceinline__ int thread_loff(int tid) {
        const int row = tid / VPR, c = tid % VPR;
        return (row * COLS + c * 8) * 2;
    }
    static constexpr int PASS_LSTRIDE = ROWS_PER_PASS * COLS * 2;

    __device__ static __forceinline__ void load(u32x4 (&reg)[NV], const char* p, long pass_stride) {
#pragma unroll
        for (int i = 0; i < NV; ++i) reg[i] = *(const u32x4*)(p + i * pass_stride);
    }
    __device__ static __forceinline__ void store(const u32x4 (&reg)[NV], lds_u8* p) {
#pragma unroll
        for (int i = 0; i < NV; ++i) *(lds_u32x4*)(p + i * PASS_LSTRIDE) = reg[i];
    }

    // Per-lane byte offset of this lane's fragment data inside the tile, for the
    // 32-wide sub-tile at row 0 and k-step 0.
    template <bool TR>
    __device__ static __forceinline__ int lane_foff(int lane) {
        if constexpr (!KM) {
            return ((lane & 31) * COLS + 8 * (lane >> 5)) * 2;
        } else if constexpr (TR) {
            // 16-lane group q: columns 16*(q&1) .. +15, k = 8*(q>>1) .. +7. Lane i of
            // the group addresses row k + i/4 (+4 for the second read), columns
            // 4*(i%4)..+3; the read hands lane j the 4 k-values of column j.
            const int q = lane >> 4, i = lane & 15;
            return ((8 * (q >> 1) + (i >> 2)) * COLS + 16 * (q & 1) + 4 * (i & 3)) * 2;
        } else {
            return (8 * (lane >> 5) * COLS + (lane & 31)) * 2;
        }
    }
    // Fragment of the sub-tile at row r0 (multiple of 32), k-step kk (16 k each);
    // r0 and kk are compile-time so the whole offset folds into the instruction.
    template <bool TR>
    __device__ static __forceinline__ bf16x8 frag(lds_u8* base, int r0, int kk) {
        if constexpr (!KM) {
            return *(lds_bf16x8*)(base + (r0 * COLS + kk * 16) * 2);
        } else if constexpr (TR) {
            lds_u8* p = base + (kk * 16 * COLS + r0) * 2;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * COLS * 2));
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, both);
        } else {
            bf16x8 out;
            lds_u8* p = base + (kk * 16 * COLS + r0) * 2;
#pragma unroll
            for (int j = 0; j < 8; ++j) out[j] = *(lds_bf16*)(p + j * COLS * 2);
            return out;
        }
    }
};

template <int BM, int BN, bool A_KM, bool B_KM, bool TR, int WGN = 2>
__global__ __launch_bounds__(128 * WGN) void gemm_mfma_kernel(GemmArgs g) {
    constexpr int NT = 128 * WGN;                 // waves are arranged 2 x WGN over the tile
    constexpr int WM = BM / 2, WN = BN / WGN;     // per-wave tile
    constexpr int TM = WM / 32, TN = WN / 32;     // 32x32 MFMA tiles per wave
    using TA = OperandTile<BM, A_KM, NT>;
    using TB = OperandTile<BN, B_KM, NT>;
    constexpr int STAGE = TA::BYTES + TB::BYTES;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    lds_u8* lds = (lds_u8*)smem_raw;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;

    // tile id -> (pm, pn): contiguous chunk of tiles per XCD (workgroups are
    // dealt round-robin to the 8 XCDs, each with its own L2), then groups of 8
    // row-tiles walked column by column so neighbours share operand tiles.
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

    if (g.causal == 1 && n0 > m0 + BM - 1) return;
    int k_lo = 0, k_hi = g.K;
    if (g.causal == 2) k_hi = min(g.K, m0 + BM);
    if (g.causal == 3) k_lo = min(m0, g.K);

    const int z = blockIdx.z;
    const long zo = z / g.batch_inner, zi = z % g.batch_inner;
    const long c_off = zo * g.c_bo + zi * g.c_bi;

    // global source pointers of this thread's first vector, advanced per k-tile
    const char* pa = (const char*)((const bf16*)g.A + zo * g.a_bo + zi * g.a_bi + (long)m0 * g.a_rs + (long)k_lo * g.a_cs) +
                     TA::thread_goff(tid, g.a_rs, g.a_cs);
    const char* pb = (const char*)((const bf16*)g.B + zo * g.b_bo + zi * g.b_bi + (long)n0 * g.b_cs + (long)k_lo * g.b_rs) +
                     TB::thread_goff(tid, g.b_cs, g.b_rs);
    const long a_pass = TA::pass_gstride(g.a_rs, g.a_cs), b_pass = TB::pass_gstride(g.b_cs, g.b_rs);
    const long a_step = TA::ktile_gstride(g.a_cs), b_step = TB::ktile_gstride(g.b_rs);

    // LDS addresses: where this thread stores, where this lane reads fragments
    lds_u8* sa = lds + TA::thread_loff(tid);
    lds_u8* sb = lds + TA::BYTES + TB::thread_loff(tid);
    lds_u8* fa = lds + TA::template lane_foff<TR>(lane) + (wm * WM) * (A_KM ? 2 : TA::COLS * 2);
    lds_u8* fb = lds + TA::BYTES + TB::template lane_foff<TR>(lane) + (wn * WN) * (B_KM ? 2 : TB::COLS * 2);

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    u32x4 ra[TA::NV], rb[TB::NV];
    const int nk = (k_hi - k_lo) / MF_BK;

    constexpr int KSTEPS = MF_BK / 16;
    static_assert(KSTEPS == 4, "the pipeline below is written for four k-steps per tile");
    constexpr int NDS = TM * (A_KM && TR ? 2 : 1) + TN * (B_KM && TR ? 2 : 1);   // LDS reads per k-step
    constexpr int NMF = TM * TN;                                                 // MFMAs per k-step
    constexpr int NVM = TA::NV + TB::NV;                                         // global loads / LDS writes per tile

  if constexpr (BM * BN <= 128 * 128 || WGN == 4) {
    // Fragments are double buffered in registers: buffer kk&1 feeds k-step kk.
    bf16x8 va[2][TM], vb[2][TN];
    auto load_frags = [&](int buf, int stage, int kk) {
#pragma unroll
        for (int i = 0; i < TM; ++i) va[buf][i] = TA::template frag<TR>(fa + stage, i * 32, kk);
#pragma unroll
        for (int j = 0; j < TN; ++j) vb[buf][j] = TB::template frag<TR>(fb + stage, j * 32, kk);
    };
    auto mfma_step = [&](int buf) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[buf][i], vb[buf][j], acc[i][j], 0, 0, 0);
    };
    // scheduling directive: NMF MFMAs, each followed by one LDS read while any remain
    auto interleave_reads = [&]() {
#pragma unroll
        for (int t = 0; t < NMF; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (t < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (NDS > NMF) __builtin_amdgcn_sched_group_barrier(0x100, NDS - NMF, 0);
    };

    // Pipeline. Tile kt is multiplied out of LDS stage kt&1 in four k-steps.
    //   k-steps 0,1 : MFMAs, LDS reads of the next k-step's fragments
    //   k-step 2    : MFMAs, LDS reads for k-step 3, LDS WRITES of tile kt+1 (its
    //                 global loads were issued a whole tile earlier), then the
    //                 global loads of tile kt+2 into the freed registers
    //   barrier     : tile kt+1 complete in LDS; k-step 3's fragments are already
    //                 in registers, so the matrix cores keep working across it
    //   k-step 3    : MFMAs, LDS reads of tile kt+1's first fragments
    if (nk > 0) {
        TA::load(ra, pa, a_pass);
        TB::load(rb, pb, b_pass);
        TA::store(ra, sa);
        TB::store(rb, sb);
        if (nk > 1) {
            pa += a_step;
            pb += b_step;
            TA::load(ra, pa, a_pass);
            TB::load(rb, pb, b_pass);
        }
    }
    __syncthreads();
    if (nk > 0) load_frags(0, 0, 0);

    int kt = 0;
    for (; kt + 2 < nk; ++kt) {     // steady state: tiles kt+1 and kt+2 exist
        const int cur = (kt & 1) * STAGE, nxt = STAGE - cur;
        load_frags(1, cur, 1);
        mfma_step(0);
        interleave_reads();
        load_frags(0, cur, 2);
        mfma_step(1);
        interleave_reads();
        load_frags(1, cur, 3);
        mfma_step(0);
        TA::store(ra, sa + nxt);
        TB::store(rb, sb + nxt);
        pa += a_step;
        pb += b_step;
        TA::load(ra, pa, a_pass);
        TB::load(rb, pb, b_pass);
        __builtin_amdgcn_sched_group_barrier(0x100, NDS, 0);
#pragma unroll
        for (int t = 0; t < NMF; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (t < NVM) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
        if (NVM > NMF) __builtin_amdgcn_sched_group_barrier(0x200, NVM - NMF, 0);
        __builtin_amdgcn_sched_group_barrier(0x020, NVM, 0);
        __syncthreads();
        load_frags(0, nxt, 0);
        mfma_step(1);
        interleave_reads();
    }
    for (; kt < nk; ++kt) {         // last two tiles: nothing left to load
        const int cur = (kt & 1) * STAGE, nxt = STAGE - cur;
        const bool more = kt + 1 < nk;
        load_frags(1, cur, 1);
        mfma_step(0);
        load_frags(0, cur, 2);
        mfma_step(1);
        load_frags(1, cur, 3);
        mfma_step(0);
        if (more) {
            TA::store(ra, sa + nxt);
            TB::store(rb, sb + nxt);
        }
        __syncthreads();
        if (more) load_frags(0, nxt, 0);
        mfma_step(1);
    }
    __syncthreads();

  } else {
    if (nk > 0) {
        TA::load(ra, pa, a_pass);
        TB::load(rb, pb, b_pass);
        TA::store(ra, sa);
        TB::store(rb, sb);
    }
    __syncthreads();

    // One k-tile of matrix work out of the LDS stage at byte offset `cur`.
    // Fragments are double buffered in registers: the LDS reads of k-step kk+1
    // are in flight while the matrix cores work on k-step kk.
    auto compute_tile = [&](int cur) {
        bf16x8 va[2][TM], vb[2][TN];
#pragma unroll
        for (int i = 0; i < TM; ++i) va[0][i] = TA::template frag<TR>(fa + cur, i * 32, 0);
#pragma unroll
        for (int j = 0; j < TN; ++j) vb[0][j] = TB::template frag<TR>(fb + cur, j * 32, 0);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            const int c = kk & 1, n = c ^ 1;
            if (kk + 1 < KSTEPS) {
#pragma unroll
                for (int i = 0; i < TM; ++i) va[n][i] = TA::template frag<TR>(fa + cur, i * 32, kk + 1);
#pragma unroll
                for (int j = 0; j < TN; ++j) vb[n][j] = TB::template frag<TR>(fb + cur, j * 32, kk + 1);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[c][i], vb[c][j], acc[i][j], 0, 0, 0);
        }
    };

    // Steady state: while tile kt is multiplied, tile kt+1 travels global ->
    // registers -> the other LDS stage. The loop body is one basic block; the
    // scheduling directives at its end spread the memory instructions between
    // the matrix instructions instead of letting them bunch up:
    //   k-step 0: global loads of the next tile and LDS reads of k-step 1
    //   k-steps 1..: LDS reads of the following k-step
    //   last k-step: LDS writes of the next tile (its global loads are ~3 k-steps old)
    for (int kt = 0; kt + 1 < nk; ++kt) {
        const int cur = (kt & 1) * STAGE, nxt = STAGE - cur;
        pa += a_step;
        pb += b_step;
        TA::load(ra, pa, a_pass);
        TB::load(rb, pb, b_pass);
        compute_tile(cur);
        TA::store(ra, sa + nxt);
        TB::store(rb, sb + nxt);
        __builtin_amdgcn_sched_group_barrier(0x100, NDS, 0);
        constexpr int NVM = TA::NV + TB::NV;
#pragma unroll
        for (int t = 0; t < NMF; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (t < NVM) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            if (t < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        if (NVM > NMF) __builtin_amdgcn_sched_group_barrier(0x020, NVM - NMF, 0);
#pragma unroll
        for (int kk = 1; kk + 1 < KSTEPS; ++kk)
#pragma unroll
            for (int t = 0; t < NMF; ++t) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                if (t < NDS) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
#pragma unroll
        for (int t = 0; t < NMF; ++t) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            if (t < NVM) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);
        }
        if (NVM > NMF) __builtin_amdgcn_sched_group_barrier(0x200, NVM - NMF, 0);
        __syncthreads();
    }
    if (nk > 0) {
        compute_tile(((nk - 1) & 1) * STAGE);
        __syncthreads();
    }

  }

    // Epilogue through LDS: each wave parks one 32-row strip of its tile in LDS
    // as fp32, then reads it back row-wise so that every lane handles 8
    // consecutive columns and the wave writes whole row segments.
    void* C = g.epi.out_f32 ? (void*)((float*)g.C + c_off) : (void*)((bf16*)g.C + c_off);
    constexpr int SW = WN + 4;                     // strip row stride in floats
    lds_f32* strip = (lds_f32*)lds + wave * (32 * SW);
    // The strip is private to its wave and a wave's LDS operations complete in
    // issue order, so after this barrier (every wave is done with the operand
    // tiles) the passes below need no workgroup barrier between them.
    __syncthreads();
    const bool plain_f32 = epilogue_is_plain_f32(g.epi);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        __builtin_amdgcn_wave_barrier();
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
                epilogue_store4_f32(g.epi, C, g.ldc, m0 + wm * WM + i * 32 + row, n0 + wn * WN + cq * 4, v4);
            }
            continue;
        }
        constexpr int CPR = WN / 8;                // 8-column chunks per strip row
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

template <int BM, int BN, bool A_KM, bool B_KM>
constexpr size_t mfma_lds_bytes() {
    return 2 * (size_t)(OperandTile<BM, A_KM>::BYTES + OperandTile<BN, B_KM>::BYTES);
}

// True when the problem satisfies every assumption of gemm_mfma_kernel<BM,BN,...>.
template <int BM, int BN>
inline bool mfma_shape_ok(const GemmArgs& g, bool a_km, bool b_km) {
    auto al8 = [](long v) { return v % 8 == 0; };
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return false;
    if (g.M % BM || g.N % BN || g.K % MF_BK) return false;
    if (((uintptr_t)g.A | (uintptr_t)g.B) & 15) return false;
    if (!al8(g.a_bo) || !al8(g.a_bi) || !al8(g.b_bo) || !al8(g.b_bi)) return false;
    // the epilogue moves 8-column vectors
    if (!al8(g.c_bo) || !al8(g.c_bi) || !al8(g.ldc) || !al8(g.epi.ldr) || !al8(g.epi.ldu)) return false;
    if (((uintptr_t)g.C | (uintptr_t)g.epi.bias | (uintptr_t)g.epi.res | (uintptr_t)g.epi.gelu_u |
         (uintptr_t)g.epi.aux_out) & 15)
        return false;
    if (a_km ? !(g.a_rs == 1 && al8(g.a_cs)) : !(g.a_cs == 1 && al8(g.a_rs))) return false;
    if (b_km ? !(g.b_cs == 1 && al8(g.b_rs)) : !(g.b_rs == 1 && al8(g.b_cs))) return false;
    if (g.causal && (g.M % 64 || BM % 64)) return false;
    return true;
}

template <int BM, int BN, bool A_KM, bool B_KM, bool TR, int WGN = 2>
inline hipError_t launch_gemm_mfma_inst(const GemmArgs& g, hipStream_t st) {
    constexpr size_t lds = mfma_lds_bytes<BM, BN, A_KM, B_KM>();
    static_assert(lds <= 160 * 1024, "tile does not fit the 160 KB LDS of a CDNA4 compute unit");
    constexpr auto kern = gemm_mfma_kernel<BM, BN, A_KM, B_KM, TR, WGN>;
    if (hipError_t e = allow_dynamic_lds<kern>((int)lds); e != hipSuccess) return e;
    dim3 grid((g.M / BM) * (g.N / BN), 1, g.batch);
    hipLaunchKernelGGL(kern, grid, dim3(128 * WGN), lds, st, g);
    return hipGetLastError();
}

}  // namespace amdp
