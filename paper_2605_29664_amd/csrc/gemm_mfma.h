// bf16 GEMM on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16), fp32
// accumulation. Tiles are staged through LDS; one workgroup = 4 wavefronts of
// 64 lanes arranged 2x2 over the BM x BN output tile.
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
#pragma once
#include "common.h"

namespace amdp {

constexpr int MF_BK = 64;
constexpr int MF_PAD = 8;   // bf16 elements of padding per LDS row

template <int R, bool KM>
struct OperandTile {
    // LDS footprint in elements
    static constexpr int ROWS = KM ? MF_BK : R;
    static constexpr int COLS = (KM ? R : MF_BK) + MF_PAD;
    static constexpr int ELEMS = ROWS * COLS;
    static constexpr int VEC_PER_THREAD = R / 32;   // 16-byte vectors each thread moves per tile

    // global -> registers. `p` points at element (row r0, k = 0) of the operand.
    // rs: stride between consecutive rows (m or n), ks: stride between consecutive k.
    __device__ static __forceinline__ void load(u32x4 (&reg)[VEC_PER_THREAD], const bf16* p, long rs,
                                                long ks, int k0, int tid) {
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) {
            const int v = tid + i * 256;
            if constexpr (!KM) {
                const int row = v / 8, kc = v % 8;
                reg[i] = *(const u32x4*)(p + (long)row * rs + (k0 + kc * 8));
            } else {
                const int krow = v / (R / 8), c = v % (R / 8);
                reg[i] = *(const u32x4*)(p + (long)(k0 + krow) * ks + c * 8);
            }
        }
    }
    __device__ static __forceinline__ void store(const u32x4 (&reg)[VEC_PER_THREAD], bf16* lds, int tid) {
#pragma unroll
        for (int i = 0; i < VEC_PER_THREAD; ++i) {
            const int v = tid + i * 256;
            if constexpr (!KM) {
                const int row = v / 8, kc = v % 8;
                *(u32x4*)(lds + row * COLS + kc * 8) = reg[i];
            } else {
                const int krow = v / (R / 8), c = v % (R / 8);
                *(u32x4*)(lds + krow * COLS + c * 8) = reg[i];
            }
        }
    }
    // fragment for the 32-wide sub-tile starting at row `r`, k-step kk (16 k each)
    template <bool TR>
    __device__ static __forceinline__ bf16x8 frag(const bf16* lds, int r, int kk, int lane) {
        if constexpr (!KM) {
            return *(const bf16x8*)(lds + (r + (lane & 31)) * COLS + kk * 16 + 8 * (lane >> 5));
        } else if constexpr (TR) {
            // 16-lane group q: columns r + 16*(q&1) .. +15, k = kk*16 + 8*(q>>1) .. +7.
            // Lane i of the group addresses row k + i/4 (+4 for the second read),
            // columns 4*(i%4)..+3; the read hands lane j the 4 k-values of column j.
            const int q = lane >> 4, i = lane & 15;
            const bf16* p = lds + (kk * 16 + 8 * (q >> 1) + (i >> 2)) * COLS + r + 16 * (q & 1) + 4 * (i & 3);
            typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
            s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
            s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * COLS));
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, both);
        } else {
            bf16x8 out;
            const bf16* p = lds + (kk * 16 + 8 * (lane >> 5)) * COLS + r + (lane & 31);
#pragma unroll
            for (int j = 0; j < 8; ++j) out[j] = p[j * COLS];
            return out;
        }
    }
};

template <int BM, int BN, bool A_KM, bool B_KM, bool TR>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs g) {
    constexpr int WM = BM / 2, WN = BN / 2;       // per-wave tile
    constexpr int TM = WM / 32, TN = WN / 32;     // 32x32 MFMA tiles per wave
    using TA = OperandTile<BM, A_KM>;
    using TB = OperandTile<BN, B_KM>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* smem = (bf16*)smem_raw;
    bf16* ldsA[2] = {smem, smem + TA::ELEMS + TB::ELEMS};
    bf16* ldsB[2] = {smem + TA::ELEMS, smem + 2 * TA::ELEMS + TB::ELEMS};

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

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
    const bf16* A = (const bf16*)g.A + zo * g.a_bo + zi * g.a_bi + (long)m0 * g.a_rs;
    const bf16* B = (const bf16*)g.B + zo * g.b_bo + zi * g.b_bi + (long)n0 * g.b_cs;
    const long c_off = zo * g.c_bo + zi * g.c_bi;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    u32x4 ra[TA::VEC_PER_THREAD], rb[TB::VEC_PER_THREAD];
    const int nk = (k_hi - k_lo) / MF_BK;
    if (nk > 0) {
        TA::load(ra, A, g.a_rs, g.a_cs, k_lo, tid);
        TB::load(rb, B, g.b_cs, g.b_rs, k_lo, tid);
        TA::store(ra, ldsA[0], tid);
        TB::store(rb, ldsB[0], tid);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const bool more = kt + 1 < nk;
        if (more) {
            TA::load(ra, A, g.a_rs, g.a_cs, k_lo + (kt + 1) * MF_BK, tid);
            TB::load(rb, B, g.b_cs, g.b_rs, k_lo + (kt + 1) * MF_BK, tid);
        }
#pragma unroll
        for (int kk = 0; kk < MF_BK / 16; ++kk) {
            bf16x8 fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = TA::template frag<TR>(ldsA[cur], wm * WM + i * 32, kk, lane);
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = TB::template frag<TR>(ldsB[cur], wn * WN + j * 32, kk, lane);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        if (more) {
            TA::store(ra, ldsA[cur ^ 1], tid);
            TB::store(rb, ldsB[cur ^ 1], tid);
        }
        __syncthreads();
    }

    // Epilogue through LDS: each wave parks one 32-row strip of its tile in LDS
    // as fp32, then reads it back row-wise so that every lane handles 8
    // consecutive columns and the wave writes whole row segments.
    void* C = g.epi.out_f32 ? (void*)((float*)g.C + c_off) : (void*)((bf16*)g.C + c_off);
    constexpr int SW = WN + 4;                     // strip row stride in floats
    float* strip = (float*)smem_raw + wave * (32 * SW);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        __syncthreads();                           // previous strip fully read (first pass: main loop done)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v)
                strip[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * SW + j * 32 + (lane & 31)] = acc[i][j][v];
        __syncthreads();
        constexpr int CPR = WN / 8;                // 8-column chunks per strip row
        for (int it = 0; it < WN / 16; ++it) {
            const int c = lane + 64 * it;
            const int row = c / CPR, cc = c % CPR;
            float v8[8];
            const f32x4 lo = *(const f32x4*)(strip + row * SW + cc * 8);
            const f32x4 hi = *(const f32x4*)(strip + row * SW + cc * 8 + 4);
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
    return 2 * (size_t)(OperandTile<BM, A_KM>::ELEMS + OperandTile<BN, B_KM>::ELEMS) * sizeof(bf16);
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

template <int BM, int BN, bool A_KM, bool B_KM, bool TR>
inline hipError_t launch_gemm_mfma_inst(const GemmArgs& g, hipStream_t st) {
    constexpr size_t lds = mfma_lds_bytes<BM, BN, A_KM, B_KM>();
    auto kern = gemm_mfma_kernel<BM, BN, A_KM, B_KM, TR>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid((g.M / BM) * (g.N / BN), 1, g.batch);
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, g);
    return hipGetLastError();
}

}  // namespace amdp
