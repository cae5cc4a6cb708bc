// Fused attention for bf16 stages (head_dim 64 or 128, sequence length a
// multiple of 128): scores, mask, softmax and the value product in one kernel,
// so the s x s score / probability matrices never touch HBM. Forward saves one
// fp32 number per (sequence, head, query): the log-sum-exp of its scores.
//
// Layout trick (all three kernels): every matrix product is set up so that the
// index a row-wise quantity belongs to (the query for max / sum / LSE / delta)
// is the MFMA *column* index n = lane % 32. Then each lane owns one query, its
// 16 accumulator registers per 32x32 tile hold 16 different keys, and the
// probabilities can be fed straight back into the next MFMA as its B operand
// without leaving registers: in a 32-key tile, lane half h = lane / 32 holds
// keys {4h..4h+3, 8+4h.., 16+4h.., 24+4h..}; taking registers 0..7 as the first
// 16-wide k-step and 8..15 as the second fixes a permutation of the keys, and
// the A operand (V^T, read from the [key][dh] LDS tile with the transposing
// read, 4 consecutive keys per read) is fetched in the same permuted order.
#pragma once
#include "common.h"
#include "gemm_mfma.h"
#include <type_traits>

namespace amdp {

// LDS placement of a [rows][DH] bf16 tile that is read both ways: by 128-bit
// row reads (a 16-lane group reads 16 consecutive rows, 16 bytes each) and by
// transposing reads (half a wave reads 4 consecutive rows, 64 bytes each).
// With 64 banks of 4 bytes the first wants the 16 rows 4 banks apart, the
// second wants the 4 rows 16 banks apart. Both hold when the row stride is
// DH*2 + 16 bytes (4 banks past a multiple of 32 banks) and, inside every
// group of 16 rows, row 4a + i is stored at position 4i + a.
template <int DH> struct AttnTile { static constexpr int STRIDE = DH * 2 + 16; };
__device__ __forceinline__ int tile_pos(int row) { return (row & ~15) | ((row & 3) << 2) | ((row >> 2) & 3); }

constexpr float LOG2E = 1.4426950408889634f;

// 2^x as the bare hardware instruction. The library exp2f wraps it in a range
// test and a rescale for results below the normal range (four more vector
// instructions per call); here x <= 0 always and a result that small is a
// probability that rounds to zero in bf16 anyway.
__device__ __forceinline__ float exp2_raw(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 pack8(const f32x16& p, int first) {
    bf16x8 out;
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = (bf16)p[first + j];
    return out;
}

// A-operand fragment (rows = 32 consecutive columns c0.. of the tile, k = the
// permuted 16 keys of k-step `ks` inside the 32-row group starting at row r0).
template <int STRIDE>
__device__ __forceinline__ bf16x8 frag_tr(lds_u8* tile, int r0, int ks, int c0, int lane) {
    // rows 16ks + 4h + j (h = lane / 32, j = 0..3) sit at positions 16ks + 4j + h,
    // the rows 8 further on at positions 2 further on
    const int q = lane >> 4, i = lane & 15;
    lds_u8* p = tile + (r0 + 16 * ks + 4 * (i >> 2) + (q >> 1)) * STRIDE + (c0 + 16 * (q & 1) + 4 * (i & 3)) * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 2 * STRIDE));
    typedef __attribute__((ext_vector_type(8))) short s16x8;
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// A-operand fragment with rows = 32 consecutive tile rows r0.., k = 16 consecutive columns at 16*kk.
template <int STRIDE>
__device__ __forceinline__ bf16x8 frag_row(lds_u8* tile, int r0, int kk, int lane) {
    return *(lds_bf16x8*)(tile + (r0 + tile_pos(lane & 31)) * STRIDE + (kk * 16 + 8 * (lane >> 5)) * 2);
}
// Cooperative copy of ROWS x DH bf16 (row stride ld elements in memory) into an
// LDS tile, split in two so the global loads of the next tile can be in flight
// while the current one is being multiplied.
template <int DH, int ROWS, int NT>
struct TileCopy {
    static constexpr int VPR = DH / 8, NV = ROWS * VPR / NT, STRIDE = AttnTile<DH>::STRIDE;
    u32x4 r[NV];
    __device__ __forceinline__ void fetch(const bf16* src, long ld, int tid) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = tid + i * NT, row = v / VPR, c = v % VPR;
            r[i] = *(const u32x4*)(src + (long)row * ld + c * 8);
        }
    }
    __device__ __forceinline__ void store(lds_u8* tile, int tid) const {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int v = tid + i * NT, row = v / VPR, c = v % VPR;
            *(lds_u32x4*)(tile + tile_pos(row) * STRIDE + c * 16) = r[i];
        }
    }
};

// Work order. The grid is one-dimensional over (128-row block, sequence*head).
// Under a causal mask a block's work grows with its position, so blocks are
// numbered heaviest first (rank 0 = most work; the dispatcher hands them out
// in order as slots free up). When the whole grid is resident at once
// (total <= resident) that does nothing; there the compute unit that takes
// block i also takes block i + total/2, so the second half is numbered lightest
// first and every unit gets a heavy and a light block.
__device__ __forceinline__ void attn_block(int i, int nq, int nz, int resident, bool causal, int& rank, int& z) {
    if (!causal) { rank = i % nq; z = i / nq; return; }
    const int total = nq * nz;
    int j = i;
    if (total <= resident && i >= total / 2) j = total - 1 - (i - total / 2);
    rank = j / nz;
    z = j % nz;
}

// ---------------------------------------------------------------- forward
// grid (s/128) * (b*H) blocks, see attn_block; 4 waves, each owns 32 queries; keys in blocks of 64.
// qkv: [b*s, 3D] (Q | K | V column blocks, heads of DH); O: [b*s, D];
// lse2: [b*H, s] = log2-domain log-sum-exp of scale*scores.
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void flash_fwd_kernel(const bf16* __restrict__ qkv, bf16* __restrict__ O,
                                                        float* __restrict__ lse2,
                                                        const int32_t* __restrict__ valid_len, int s, int H,
                                                        int D, float scale_log2e, int nz, int resident) {
    constexpr int STRIDE = AttnTile<DH>::STRIDE, BKV = 64, KQ = DH / 16, DT = DH / 32;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * BKV * STRIDE];
    lds_u8* tK = (lds_u8*)smem;
    lds_u8* tV = tK + BKV * STRIDE;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int rank, z;
    attn_block(blockIdx.x, s / 128, nz, resident, CAUSAL, rank, z);
    const int qb = CAUSAL ? s / 128 - 1 - rank : rank;      // late queries see the most keys
    const int b = z / H, h = z % H;
    const long ld = 3L * D;
    const bf16* base = qkv + (long)b * s * ld + (long)h * DH;
    const int q_blk = qb * 128, q_wave = q_blk + wave * 32, q = q_wave + (lane & 31);
    const int half = lane >> 5;

    bf16x8 bq[KQ];   // B operand: n = query, k = head dimension
#pragma unroll
    for (int kk = 0; kk < KQ; ++kk) bq[kk] = *(const bf16x8*)(base + (long)q * ld + kk * 16 + 8 * half);

    f32x16 acc[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    int kend = s;
    if (CAUSAL) kend = q_blk + 128;
    if (valid_len) kend = min(kend, (max(valid_len[b], 1) + BKV - 1) / BKV * BKV);
    const int klimit = valid_len ? valid_len[b] : s;

    TileCopy<DH, BKV, 256> cK, cV;
    if (kend > 0) {
        cK.fetch(base + D, ld, tid);
        cV.fetch(base + 2 * D, ld, tid);
    }
    for (int k0 = 0; k0 < kend; k0 += BKV) {
        __syncthreads();                              // everyone is done with the previous tiles
        cK.store(tK, tid);
        cV.store(tV, tid);
        __syncthreads();
        if (k0 + BKV < kend) {                        // next tiles travel while this one is used
            cK.fetch(base + D + (long)(k0 + BKV) * ld, ld, tid);
            cV.fetch(base + 2 * D + (long)(k0 + BKV) * ld, ld, tid);
        }
        if (CAUSAL && k0 > q_wave + 31) continue;     // every key of the block is hidden from this wave

        f32x16 st[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int v = 0; v < 16; ++v) st[kt][v] = 0.f;
#pragma unroll
            for (int kk = 0; kk < KQ; ++kk)
                st[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_row<STRIDE>(tK, kt * 32, kk, lane), bq[kk],
                                                                st[kt], 0, 0, 0);
        }
        // Softmax in the log2 domain on the raw scores: x = c*s, p = exp2(c*s - m).
        // Masks only where a block touches the diagonal or the padding edge
        // (wave-uniform test); everything else is one max, one fma, one exp2 and
        // one add per score.
        const bool edge = (CAUSAL && k0 + BKV - 1 > q_wave) || k0 + BKV > klimit;
        if (edge) {
#pragma unroll
            for (int kt = 0; kt < 2; ++kt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = k0 + kt * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                    if ((CAUSAL && key > q) || key >= klimit) st[kt][v] = -INFINITY;
                }
        }
        float mloc = -INFINITY;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) mloc = fmaxf(mloc, st[kt][v]);
        mloc = fmaxf(mloc, __shfl_xor(mloc, 32, 64)) * scale_log2e;      // scale > 0 commutes with max
        const float m_new = fmaxf(m_run, mloc);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        float lsum = 0.f;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const float p = exp2_raw(fmaf(st[kt][v], scale_log2e, -m_use));
                st[kt][v] = p;
                lsum += p;
            }
        if (m_new != m_run) {          // most blocks leave the running maximum alone
            const float alpha = exp2_raw(m_run - m_use);
            l_run *= alpha;
#pragma unroll
            for (int t = 0; t < DT; ++t)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[t][v] *= alpha;
            m_run = m_new;
        }
        l_run += lsum;
        // O^T += V^T P^T
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const bf16x8 pb = pack8(st[kt], 8 * ks);
#pragma unroll
                for (int t = 0; t < DT; ++t)
                    acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<STRIDE>(tV, kt * 32, ks, t * 32, lane),
                                                                     pb, acc[t], 0, 0, 0);
            }
    }

    const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    bf16* orow = O + ((long)b * s + q) * D + (long)h * DH;
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)(acc[t][4 * gq + e] * inv);
            *(bf16x4*)(orow + t * 32 + 8 * gq + 4 * half) = o;
        }
    if (half == 0) lse2[(long)z * s + q] = m_run + log2f(l_tot);
}


// Head-wise repacking between widths (32-bit pairs of bf16): output pair i of
// `pairs` belongs to chunk i / wd2 and column pair i % wd2; columns past the
// source width read as zero.
__global__ __launch_bounds__(256) void repack_heads_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst,
                                                           long pairs, int ws2, int wd2) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= pairs) return;
    const long chunk = i / wd2;
    const int c = (int)(i % wd2);
    dst[i] = c < ws2 ? src[chunk * ws2 + c] : 0u;
}

// ---------------------------------------------------------------- backward
// delta[z][q] = sum_d dO[q, h*DH + d] * O[q, h*DH + d]   (z = sequence*H + head)
// One wave per token row; a head's DH/8 vectors sit in DH/8 adjacent lanes.
template <int DH>
__global__ __launch_bounds__(256) void attn_delta_kernel(const bf16* __restrict__ dO, const bf16* __restrict__ O,
                                                         float* __restrict__ delta, int rows, int s, int H, int D) {
    constexpr int LPH = DH / 8;    // lanes per head
    const int lane = threadIdx.x & 63;
    const long row = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const long b = row / s, pos = row % s;
    for (int c = lane; c < D / 8; c += 64) {
        const bf16x8 a = *(const bf16x8*)(dO + row * D + c * 8);
        const bf16x8 o = *(const bf16x8*)(O + row * D + c * 8);
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) t += (float)a[i] * (float)o[i];
#pragma unroll
        for (int m = 1; m < LPH; m <<= 1) t += __shfl_xor(t, m, 64);
        if ((lane & (LPH - 1)) == 0) delta[(b * H + c / LPH) * s + pos] = t;
    }
}

template <int NTILES>
__device__ __forceinline__ void store_headrow(bf16* row, const f32x16 (&acc)[4], int half, float mul) {
#pragma unroll
    for (int t = 0; t < NTILES; ++t)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)(acc[t][4 * gq + e] * mul);
            *(bf16x4*)(row + t * 32 + 8 * gq + 4 * half) = o;
        }
}

// dK, dV. Same grid; each wave owns 32 keys (lane % 32) and walks the
// query tiles of 64 that can see them. dqkv: [b*s, 3D], K block at +D, V at +2D.
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(DH == 64 ? 2 : 1))) void flash_bwd_dkv_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                            const float* __restrict__ lse2,
                                                            const float* __restrict__ delta, bf16* __restrict__ dqkv,
                                                            const int32_t* __restrict__ valid_len, int s, int H,
                                                            int D, float scale, int nz, int resident) {
    constexpr int STRIDE = AttnTile<DH>::STRIDE, BQ = 64, KQ = DH / 16, DT = DH / 32;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * BQ * STRIDE];
    __shared__ __attribute__((aligned(16))) float sstat[2][BQ];
    lds_u8* tQ = (lds_u8*)smem;
    lds_u8* tdO = tQ + BQ * STRIDE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    int rank, z;
    attn_block(blockIdx.x, s / 128, nz, resident, CAUSAL, rank, z);     // early keys are seen by the most queries
    const int b = z / H, h = z % H;
    const long ld = 3L * D;
    const bf16* base = qkv + (long)b * s * ld + (long)h * DH;
    const bf16* dObase = dO + (long)b * s * D + (long)h * DH;
    const int k_blk = rank * 128, k_wave = k_blk + wave * 32, key = k_wave + (lane & 31);
    const int klimit = valid_len ? valid_len[b] : s;
    const float sl2 = scale * LOG2E;
    const bool key_dead = key >= klimit;     // padding: this lane's key is visible to nobody

    bf16x8 bk[KQ], bv[KQ];      // B operands: n = key, k = head dimension
#pragma unroll
    for (int kk = 0; kk < KQ; ++kk) {
        bk[kk] = *(const bf16x8*)(base + D + (long)key * ld + kk * 16 + 8 * half);
        bv[kk] = *(const bf16x8*)(base + 2 * D + (long)key * ld + kk * 16 + 8 * half);
    }
    f32x16 dk[4], dv[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) { dk[t][v] = 0.f; dv[t][v] = 0.f; }

    const int q_begin = CAUSAL ? k_blk : 0;
    const bool block_live = k_blk < klimit;
    TileCopy<DH, BQ, 256> cQ, cdO;
    float stat_next = 0.f;      // threads 0..63: lse of query tid; 64..127: delta of query tid-64
    const float* stat_src = tid < BQ ? lse2 + (long)z * s + tid : delta + (long)z * s + (tid - BQ);
    if (block_live && q_begin < s) {
        cQ.fetch(base + (long)q_begin * ld, ld, tid);
        cdO.fetch(dObase + (long)q_begin * D, D, tid);
        if (tid < 2 * BQ) stat_next = stat_src[q_begin];
    }
    for (int q0 = q_begin; q0 < s && block_live; q0 += BQ) {
        __syncthreads();
        cQ.store(tQ, tid);
        cdO.store(tdO, tid);
        if (tid < 2 * BQ) sstat[tid / BQ][tid % BQ] = stat_next;
        __syncthreads();
        if (q0 + BQ < s) {
            cQ.fetch(base + (long)(q0 + BQ) * ld, ld, tid);
            cdO.fetch(dObase + (long)(q0 + BQ) * D, D, tid);
            if (tid < 2 * BQ) stat_next = stat_src[q0 + BQ];
        }
        if (CAUSAL && q0 + BQ - 1 < k_wave) continue;      // none of these queries sees this wave's keys
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            f32x16 sc, dp;
#pragma unroll
            for (int v = 0; v < 16; ++v) { sc[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
            for (int kk = 0; kk < KQ; ++kk) {
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_row<STRIDE>(tQ, qt * 32, kk, lane), bk[kk], sc, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_row<STRIDE>(tdO, qt * 32, kk, lane), bv[kk], dp, 0, 0, 0);
            }
            // masks only where this wave's keys meet the diagonal or the padding edge
            // (wave-uniform test): elsewhere one fma, one exp2, one sub, one mul per score
            const bool edge = CAUSAL ? (q0 + qt * 32 < k_wave + 31) : (k_wave + 31 >= klimit);
            auto probabilities = [&](auto masked) {
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const f32x4 l4 = *(const f32x4*)&sstat[0][qt * 32 + 8 * gq + 4 * half];
                    const f32x4 d4 = *(const f32x4*)&sstat[1][qt * 32 + 8 * gq + 4 * half];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int v = 4 * gq + e;
                        float p = exp2_raw(fmaf(sc[v], sl2, -l4[e]));
                        if constexpr (decltype(masked)::value) {
                            const int q = q0 + qt * 32 + 8 * gq + 4 * half + e;
                            if ((CAUSAL && key > q) || key_dead) p = 0.f;
                        }
                        sc[v] = p;
                        dp[v] = p * (dp[v] - d4[e]);     // the factor `scale` of dS is applied to dK at the end
                    }
                }
            };
            if (edge) probabilities(std::true_type{}); else probabilities(std::false_type{});
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const bf16x8 pb = pack8(sc, 8 * ks), dsb = pack8(dp, 8 * ks);
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    dv[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<STRIDE>(tdO, qt * 32, ks, t * 32, lane), pb, dv[t], 0, 0, 0);
                    dk[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<STRIDE>(tQ, qt * 32, ks, t * 32, lane), dsb, dk[t], 0, 0, 0);
                }
            }
        }
    }
    bf16* out = dqkv + ((long)b * s + key) * ld + (long)h * DH;
    store_headrow<DT>(out + D, dk, half, scale);
    store_headrow<DT>(out + 2 * D, dv, half, 1.0f);
}

// dQ. Same grid; each wave owns 32 queries and walks the key blocks of 64 it can see.
template <int DH, bool CAUSAL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void flash_bwd_dq_kernel(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                           const float* __restrict__ lse2,
                                                           const float* __restrict__ delta, bf16* __restrict__ dqkv,
                                                           const int32_t* __restrict__ valid_len, int s, int H,
                                                           int D, float scale, int nz, int resident) {
    constexpr int STRIDE = AttnTile<DH>::STRIDE, BKV = 64, KQ = DH / 16, DT = DH / 32;
    __shared__ __attribute__((aligned(16))) unsigned char smem[2 * BKV * STRIDE];
    lds_u8* tK = (lds_u8*)smem;
    lds_u8* tV = tK + BKV * STRIDE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5;
    int rank, z;
    attn_block(blockIdx.x, s / 128, nz, resident, CAUSAL, rank, z);
    const int qb = CAUSAL ? s / 128 - 1 - rank : rank;
    const int b = z / H, h = z % H;
    const long ld = 3L * D;
    const bf16* base = qkv + (long)b * s * ld + (long)h * DH;
    const int q_blk = qb * 128, q_wave = q_blk + wave * 32, q = q_wave + (lane & 31);
    const int klimit = valid_len ? valid_len[b] : s;
    const float sl2 = scale * LOG2E;

    bf16x8 bq[KQ], bdo[KQ];     // B operands: n = query, k = head dimension
#pragma unroll
    for (int kk = 0; kk < KQ; ++kk) {
        bq[kk] = *(const bf16x8*)(base + (long)q * ld + kk * 16 + 8 * half);
        bdo[kk] = *(const bf16x8*)(dO + ((long)b * s + q) * D + (long)h * DH + kk * 16 + 8 * half);
    }
    const float lse_q = lse2[(long)z * s + q], delta_q = delta[(long)z * s + q];
    f32x16 dq[4];
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) dq[t][v] = 0.f;

    int kend = s;
    if (CAUSAL) kend = q_blk + 128;
    if (valid_len) kend = min(kend, (max(klimit, 1) + BKV - 1) / BKV * BKV);
    TileCopy<DH, BKV, 256> cK, cV;
    if (kend > 0) {
        cK.fetch(base + D, ld, tid);
        cV.fetch(base + 2 * D, ld, tid);
    }
    for (int k0 = 0; k0 < kend; k0 += BKV) {
        __syncthreads();
        cK.store(tK, tid);
        cV.store(tV, tid);
        __syncthreads();
        if (k0 + BKV < kend) {
            cK.fetch(base + D + (long)(k0 + BKV) * ld, ld, tid);
            cV.fetch(base + 2 * D + (long)(k0 + BKV) * ld, ld, tid);
        }
        if (CAUSAL && k0 > q_wave + 31) continue;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            f32x16 sc, dp;
#pragma unroll
            for (int v = 0; v < 16; ++v) { sc[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
            for (int kk = 0; kk < KQ; ++kk) {
                sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_row<STRIDE>(tK, kt * 32, kk, lane), bq[kk], sc, 0, 0, 0);
                dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_row<STRIDE>(tV, kt * 32, kk, lane), bdo[kk], dp, 0, 0, 0);
            }
            // masks only where the key tile meets this wave's diagonal or the padding edge (wave-uniform)
            const bool edge = CAUSAL ? (k0 + kt * 32 + 31 > q_wave) : (k0 + kt * 32 + 31 >= klimit);
            auto dscores = [&](auto masked) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float p = exp2_raw(fmaf(sc[v], sl2, -lse_q));
                    if constexpr (decltype(masked)::value) {
                        const int key = k0 + kt * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                        if ((CAUSAL && key > q) || (!CAUSAL && key >= klimit)) p = 0.f;   // causal stages carry no padding mask
                    }
                    dp[v] = p * (dp[v] - delta_q);       // the factor `scale` of dS is applied to dQ at the end
                }
            };
            // (at head dimension 128 the second copy of the loop body costs 14 spilled registers
            // and 13 % of the kernel's time: there every tile takes the masked form)
            if (DH == 128 || edge) dscores(std::true_type{}); else dscores(std::false_type{});
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const bf16x8 dsb = pack8(dp, 8 * ks);
#pragma unroll
                for (int t = 0; t < DT; ++t)
                    dq[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr<STRIDE>(tK, kt * 32, ks, t * 32, lane), dsb, dq[t], 0, 0, 0);
            }
        }
    }
    store_headrow<DT>(dqkv + ((long)b * s + q) * ld + (long)h * DH, dq, half, scale);
}

}  // namespace amdp
