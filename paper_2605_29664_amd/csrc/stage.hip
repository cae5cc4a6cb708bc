// Stage executor: owns the layout of the caller's workspace (master
// parameters, Adam moments, gradient sum and staging, weight-version slots,
// activation slots, scratch), the residency rules for versions and in-flight
// minibatches, and the order of kernel launches for forward, backward,
// accumulate and update. Everything is enqueued on one HIP stream.
#include "amdp.h"
#include "attention.h"
#include "embedding.h"
#include "common.h"
#include "gemm_mfma.h"
#include "gemm_mfma_dl.h"
#include "gemm_simple.h"
#include "rowwise.h"
#include "streaming.h"

#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

using namespace amdp;

namespace {

constexpr size_t ALIGN = 256;
constexpr int MAX_VSLOTS = 16;
constexpr int MAX_ASLOTS = 64;
constexpr int LM_PAD_ROWS = 256;   // vocabulary rows are padded to a multiple of this

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

enum Field { LN1_G, LN1_B, W_QKV, B_QKV, W_O, B_O, LN2_G, LN2_B, W_1, B_1, W_2, B_2, N_FIELDS };
const char* const FIELD_NAMES[N_FIELDS] = {"ln1_gamma", "ln1_beta", "w_qkv", "b_qkv", "w_o", "b_o",
                                           "ln2_gamma", "ln2_beta", "w_1",   "b_1",   "w_2", "b_2"};

struct Dims {
    int L, D, H, dh, F, s, b, N, V;
    long Vld;
    bool lm, bf, causal;
    bool emb = false;      // first stage: token + position embedding in front of the blocks
    size_t esz;
    long field_size(int f) const {
        switch (f) {
            case LN1_G: case LN1_B: case LN2_G: case LN2_B: case B_O: case B_2: return D;
            case W_QKV: return 3L * D * D;
            case B_QKV: return 3L * D;
            case W_O: return (long)D * D;
            case W_1: case W_2: return (long)D * F;
            case B_1: return F;
        }
        return 0;
    }
    long layer_params() const {
        long t = 0;
        for (int f = 0; f < N_FIELDS; ++f) t += field_size(f);
        return t;
    }
    long emb_params() const { return emb ? ((long)V + s) * D : 0; }
    long off_tok() const { return 0; }
    long off_pos() const { return (long)V * D; }
    long off(int layer, int f) const {
        long t = emb_params() + layer * layer_params();
        for (int k = 0; k < f; ++k) t += field_size(k);
        return t;
    }
    long off_lnf() const { return emb_params() + L * layer_params(); }
    long off_embed() const { return off_lnf() + 2L * D; }
    long n_params() const { return lm ? off_embed() + (long)V * D : emb_params() + L * layer_params(); }
    long n_alloc() const {
        long n = n_params() + (lm ? (long)LM_PAD_ROWS * D : 0);
        return (long)round_up((size_t)n, 1024);
    }
};

bool make_dims(const amdp_stage_config_t* c, Dims* d) {
    if (!c || c->struct_size != sizeof(amdp_stage_config_t)) return false;
    if (c->block_kind != AMDP_BLOCK_GPT_PRELN_CAUSAL && c->block_kind != AMDP_BLOCK_BERT_POSTLN_BIDIR)
        return false;
    if (c->dtype != AMDP_FP32 && c->dtype != AMDP_BF16) return false;
    if (c->attention != AMDP_ATTN_AUTO && c->attention != AMDP_ATTN_UNFUSED) return false;
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->d_ffn < 1 || c->seq_len < 1 ||
        c->microbatch < 1)
        return false;
    if (c->d_model % c->n_heads) return false;
    if ((c->has_lm_head || c->has_embedding) && c->vocab < 1) return false;
    if (c->has_lm_head && c->has_embedding) return false;   // input layer or output head, not both
    if (c->has_embedding && c->d_model > 8192) return false; // width of the token-gradient kernel
    if (c->act_slots < 1 || c->act_slots > MAX_ASLOTS) return false;
    if (c->stash_slots < 1 || c->stash_slots + 1 > MAX_VSLOTS) return false;
    if (!(c->ln_eps > 0.f)) return false;
    const int vec = c->dtype == AMDP_BF16 ? 8 : 4;   // row kernels move 16-byte vectors
    if (c->d_model % vec || c->d_ffn % vec || c->seq_len % vec) return false;
    if ((long)c->seq_len * c->microbatch > (1L << 24)) return false;
    d->L = c->n_layers; d->D = c->d_model; d->H = c->n_heads; d->dh = c->d_model / c->n_heads;
    d->F = c->d_ffn; d->s = c->seq_len; d->b = c->microbatch; d->N = c->seq_len * c->microbatch;
    d->lm = c->has_lm_head != 0; d->emb = c->has_embedding != 0; d->V = (d->lm || d->emb) ? c->vocab : 0;
    d->Vld = d->lm ? (long)round_up((size_t)d->V, LM_PAD_ROWS) : 0;
    d->bf = c->dtype == AMDP_BF16; d->esz = d->bf ? 2 : 4;
    d->causal = c->block_kind == AMDP_BLOCK_GPT_PRELN_CAUSAL;
    return true;
}

// ---- workspace carving ------------------------------------------------------
struct LayerAct {   // byte offsets inside an activation slot
    size_t xin, a, qkv, P, o, y1, c, u, h, st1, st2;   // P: probabilities, or the fused kernels' log-sum-exp
};
struct SlotLayout {
    std::vector<LayerAct> layers;
    size_t yL = 0, z = 0, stf = 0, dlogits = 0;
    size_t valid = 0;   // copy of the padding mask (valid_len[b]) for backward
    size_t tokens = 0;  // copy of the token ids [N] of a first stage, for backward
    size_t bytes = 0;
};
struct Carve {
    size_t theta, m, v, G, g, versions, version_bytes, act, slot_bytes;
    // backward scratch: one set per layer so that gradient leaves running on the
    // side stream never see their inputs overwritten by the main chain
    struct BwdScratch { size_t t_a, t_b, t_c, dffn, dqkv, dxout; };
    std::vector<BwdScratch> bw;
    size_t lm_dz, lm_dy, dO, dP, partial, row_loss, total;
    size_t pk_qkv = 0, pk_dqkv = 0, pk_o = 0, pk_do = 0;   // head-padded copies for the fused attention
    size_t splitk = 0, splitk_bytes = 0;                   // parts of a weight-gradient product split over its tokens
    size_t splitm = 0, splitm_bytes = 0;                   // parts of a main-chain product with a split contraction
    int partial_chunks;
    SlotLayout slot;
};

// Fused attention is used whenever the shape allows it (the configuration's
// `attention` field can ask for the three-kernel form instead). With it, only
// the fp32 log-sum-exp per (sequence, head, query) is kept instead of the
// s x s probabilities.
// The fused attention kernels exist for head dimensions 64 and 128. Other even
// head dimensions up to 128 run through them zero-padded: Q, K, V (and dO, O in
// backward) are repacked head by head into scratch with the padded width, which
// changes no result (the padding contributes exact zeros to every product).
inline int flash_head_dim(const Dims& d) { return d.dh <= 64 ? 64 : 128; }
inline bool flash_shape_ok(const Dims& d) { return d.bf && d.dh <= 128 && d.dh % 2 == 0 && d.s % 128 == 0; }
inline bool flash_packed(const Dims& d) { return d.dh != flash_head_dim(d); }

void carve(const Dims& d, const amdp_stage_config_t& c, Carve* w) {
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = round_up(off + bytes, ALIGN); return o; };
    const size_t na = (size_t)d.n_alloc();
    w->theta = take(na * 4); w->m = take(na * 4); w->v = take(na * 4); w->G = take(na * 4);
    w->g = take(na * 4);
    w->version_bytes = round_up(na * d.esz, ALIGN);
    w->versions = take(w->version_bytes * (size_t)(c.stash_slots + 1));

    const size_t ND = (size_t)d.N * d.D * d.esz, NF = (size_t)d.N * d.F * d.esz;
    const bool fused = c.attention == AMDP_ATTN_AUTO && flash_shape_ok(d);
    const size_t PP = fused ? (size_t)d.b * d.H * d.s * 4 : (size_t)d.b * d.H * d.s * d.s * d.esz;
    {
        size_t so = 0;
        auto st = [&](size_t bytes) { size_t o = so; so = round_up(so + bytes, ALIGN); return o; };
        w->slot.layers.resize(d.L);
        for (int l = 0; l < d.L; ++l) {
            LayerAct& a = w->slot.layers[l];
            a.xin = st(ND); a.a = st(ND); a.qkv = st(3 * ND); a.P = st(PP); a.o = st(ND);
            a.y1 = st(ND); a.c = st(ND); a.u = st(NF); a.h = st(NF);
            a.st1 = st((size_t)d.N * 8); a.st2 = st((size_t)d.N * 8);
        }
        if (d.lm) {
            w->slot.yL = st(ND); w->slot.z = st(ND); w->slot.stf = st((size_t)d.N * 8);
            w->slot.dlogits = st((size_t)d.N * d.Vld * d.esz);
        }
        w->slot.valid = st((size_t)d.b * 4);
        w->slot.tokens = st(d.emb ? (size_t)d.N * 4 : 0);
        w->slot.bytes = so;
    }
    w->slot_bytes = w->slot.bytes;
    w->act = take(w->slot_bytes * (size_t)c.act_slots);
    w->bw.resize(d.L);
    for (int l = 0; l < d.L; ++l) {
        Carve::BwdScratch& b = w->bw[l];
        b.t_a = take(ND); b.t_b = take(ND); b.t_c = take(ND);
        b.dffn = take(NF); b.dqkv = take(3 * ND); b.dxout = take(ND);
    }
    w->lm_dz = take(d.lm ? ND : 0);
    w->lm_dy = take(d.lm ? ND : 0);
    w->dO = take(ND);
    w->dP = take(PP);
    {
        const bool pk = fused && flash_packed(d);
        const size_t NDp = pk ? (size_t)d.N * d.H * flash_head_dim(d) * d.esz : 0;
        w->pk_qkv = take(3 * NDp); w->pk_dqkv = take(3 * NDp); w->pk_o = take(NDp); w->pk_do = take(NDp);
    }
    // Only the D x D product of a narrow layer is ever split (the others have three to
    // sixteen times as many tiles); room for eight parts while its 128x128 tiles would
    // leave half of a 256-unit GPU idle.
    w->splitk_bytes = (d.bf && d.D % 128 == 0 && (long)(d.D / 128) * (d.D / 128) * 2 <= 256) ? (size_t)8 * d.D * d.D * 4 : 0;
    w->splitk = take(w->splitk_bytes);
    // [tokens, d_model] outputs whose 256x256 tiles cover at most half of a 256-unit GPU may run with
    // their contraction split in two (main_split): two fp32 copies of the output
    w->splitm_bytes = (d.bf && d.N % 256 == 0 && d.D % 256 == 0 && (long)(d.N / 256) * (d.D / 256) * 2 <= 256)
                          ? (size_t)2 * d.N * d.D * 4 : 0;
    w->splitm = take(w->splitm_bytes);
    w->partial_chunks = 256;
    // one row of partial sums per row chunk for all six column reductions of a layer's backward
    const size_t maxw = (size_t)9 * d.D + d.F;
    w->partial = take((size_t)w->partial_chunks * maxw * 4);
    w->row_loss = take((size_t)d.N * 4);
    w->total = off;
}

// Optional per-launch timing with HIP events on the stage's stream.
struct ProfRecord { int name_id; hipEvent_t start, stop; double flops, bytes; };
struct Profiler {
    bool on = false;
    std::vector<std::string> names;
    std::vector<ProfRecord> recs;
    int id_of(const char* name) {
        for (size_t i = 0; i < names.size(); ++i) if (names[i] == name) return (int)i;
        names.emplace_back(name);
        return (int)names.size() - 1;
    }
};

struct VSlot { bool valid = false; uint32_t version = 0; int pins = 0; };
struct ASlot { bool used = false; int32_t mb = 0; int vslot = -1; bool backwarded = false; };

}  // namespace

struct amdp_stage {
    amdp_stage_config_t cfg;
    Dims d;
    Carve w;
    char* base;
    hipStream_t stream;
    VSlot vs[MAX_VSLOTS];
    ASlot as[MAX_ASLOTS];
    int n_vslots;
    int cur_slot = -1;
    uint32_t cur_version = 0;
    uint64_t step = 0;
    int staged_slot = -1;   // activation slot whose gradient sits in the staging buffer
    bool use_tr = true;
    int force_tile = 0;
    int use_direct = 1;           // plain products load tiles straight into LDS where measured faster
                                  // (AMDP_OPT_GEMM_DIRECT_TO_LDS; 0: never, always through registers; 2: wherever the shape allows)
    Profiler prof;
    // Launch target of the helper functions: the caller's stream, or the side
    // stream while a gradient leaf (dW GEMM, bias / LayerNorm column sums) is
    // being enqueued. Leaves are off the dX critical path and fill the compute
    // units the chain's small GEMMs leave idle.
    hipStream_t launch = nullptr;
    hipStream_t side = nullptr;
    int n_cu = 256;                // compute units of the device
    hipEvent_t events[16] = {};
    int ev_next = 0;
    // A backward leaves its gradient leaves running on the side stream. What must wait
    // for them: the next backward (it reuses the per-layer scratch they read) and the
    // forward that reuses the activation slot they read; both wait for the event
    // recorded behind the leaves, nothing else does. free_seq orders free slots so
    // that a forward takes the one whose leaves are oldest.
    bool lazy_join = true;           // AMDP_OPT_LAZY_JOIN; false: backward ends with a full join (measurement)
    hipEvent_t input_ev = nullptr;   // behind the leaves that read the caller's dY
    hipEvent_t leaves_ev[MAX_ASLOTS] = {};
    bool leaves_pending[MAX_ASLOTS] = {};
    int last_leaves = -1;
    uint64_t free_seq[MAX_ASLOTS] = {};
    uint64_t free_counter = 0;
    bool overlap = true;
    int leaf_forks = 0;            // side-stream forks per layer of a backward: 0 = one per leaf, 1, 2 (set at creation)
    bool fused_acc = false;        // backward adds parameter gradients into G directly
    int splitk_min_k = 512;        // fewest tokens a part of a split weight-gradient product contracts
    int split_main_min_k = 3072;   // shortest half of a main-chain contraction that is worth splitting
    bool flash = true;      // fused attention kernels (shape permitting); false: scores, softmax, probabilities in HBM
    hipEvent_t next_event() { ev_next = (ev_next + 1) % 16; return events[ev_next]; }

    template <class P = void> P* at(size_t off) const { return (P*)(base + off); }
    char* version_ptr(int slot) const { return base + w.versions + (size_t)slot * w.version_bytes; }
    char* act_ptr(int slot) const { return base + w.act + (size_t)slot * w.slot_bytes; }
    int find_version(uint32_t v) const {
        for (int i = 0; i < n_vslots; ++i) if (vs[i].valid && vs[i].version == v) return i;
        return -1;
    }
    int find_mb(int32_t mb) const {
        for (int i = 0; i < cfg.act_slots; ++i) if (as[i].used && as[i].mb == mb) return i;
        return -1;
    }
    // a slot can be reused when it holds no version, or an old one no in-flight
    // minibatch's forward has read
    int free_vslot() const {
        for (int i = 0; i < n_vslots; ++i) if (!vs[i].valid) return i;
        for (int i = 0; i < n_vslots; ++i) if (i != cur_slot && vs[i].pins == 0) return i;
        return -1;
    }
    void drop_unpinned() {
        for (int i = 0; i < n_vslots; ++i)
            if (vs[i].valid && i != cur_slot && vs[i].pins == 0) vs[i].valid = false;
    }
};

namespace {

thread_local char g_hip_detail[160] = "";
inline bool hip_ok(hipError_t e, const char* what) {
    if (e == hipSuccess) return true;
    snprintf(g_hip_detail, sizeof(g_hip_detail), "%s: %s", what, hipGetErrorString(e));
    return false;
}
#define HIP_TRY(expr) do { if (!hip_ok((expr), #expr)) return AMDP_E_HIP; } while (0)
#define TRY(expr) do { int rc_ = (expr); if (rc_ != AMDP_OK) return rc_; } while (0)

inline int after_launch() { return hip_ok(hipGetLastError(), "kernel launch") ? AMDP_OK : AMDP_E_HIP; }

// bytes is a multiple of 4; 16-byte path when both pointers allow it
int device_copy(hipStream_t stream, void* dst, const void* src, size_t bytes) {
    if (!bytes) return AMDP_OK;
    if ((((uintptr_t)dst | (uintptr_t)src) & 15) == 0 && bytes % 16 == 0) {
        const long n16 = (long)(bytes / 16);
        hipLaunchKernelGGL(copy16_kernel, dim3(direct_grid(n16, ACC_BLOCK)), dim3(ACC_BLOCK), 0, stream, (u32x4*)dst,
                           (const u32x4*)src, n16);
    } else {
        if ((((uintptr_t)dst | (uintptr_t)src) & 3) || bytes % 4) return AMDP_E_INVAL;
        const long n = (long)(bytes / 4);
        hipLaunchKernelGGL(copy4_kernel, dim3(stream_grid(n)), dim3(STREAM_BLOCK), 0, stream, (uint32_t*)dst,
                           (const uint32_t*)src, n);
    }
    return after_launch();
}
// dst 16-byte aligned, bytes a multiple of 16 (all workspace regions are)
int device_zero(hipStream_t stream, void* dst, size_t bytes) {
    if (!bytes) return AMDP_OK;
    const long n16 = (long)(bytes / 16);
    hipLaunchKernelGGL(zero16_kernel, dim3(direct_grid(n16, ACC_BLOCK)), dim3(ACC_BLOCK), 0, stream, (u32x4*)dst, n16);
    return after_launch();
}

// Brackets the launches made during its lifetime with two events when the
// stage's profiler is on; costs one branch otherwise.
struct ProfScope {
    amdp_stage* st;
    int idx = -1;
    ProfScope(amdp_stage* s, const char* name, double flops, double bytes) : st(s) {
        if (!st->prof.on) return;
        ProfRecord r{st->prof.id_of(name), nullptr, nullptr, flops, bytes};
        if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) return;
        hipEventRecord(r.start, st->launch);
        st->prof.recs.push_back(r);
        idx = (int)st->prof.recs.size() - 1;
    }
    ~ProfScope() {
        if (idx >= 0) hipEventRecord(st->prof.recs[idx].stop, st->launch);
    }
};

inline double gemm_flops(const GemmArgs& g) {
    double f = 2.0 * g.M * (double)g.N * g.K * g.batch;
    if (g.causal) f *= (g.M + 1.0) / (2.0 * g.M);   // only query/key pairs with key <= query
    return f;
}

// ---- GEMM dispatch ----------------------------------------------------------
template <int BM, int BN, bool A_KM, bool B_KM, int WGN = 2>
hipError_t launch_tile(amdp_stage* st, const GemmArgs& g) {
    return st->use_tr ? launch_gemm_mfma_inst<BM, BN, A_KM, B_KM, true, WGN>(g, st->launch)
                      : launch_gemm_mfma_inst<BM, BN, A_KM, B_KM, false, WGN>(g, st->launch);
}

// Tile choice, from measurement on MI355X: the largest tile that still fills
// the GPU wins (the 256x256 tile needs a workgroup for every compute unit and
// at least 70 % of its last round of workgroups, the smaller ones three
// quarters of the units); when no tile gets there, the one with the most
// workgroups does. Plain products (no batch, no causal band) whose M or N is a
// multiple of 64 but not of the tile run the 128x128 and 256x256 tiles with a
// ragged last tile on the direct-to-LDS kernel.
template <bool A_KM, bool B_KM>
int gemm_bf16_layout(amdp_stage* st, const GemmArgs& g) {
    const bool direct = st->use_direct && g.batch == 1 && g.causal == 0, always = st->use_direct == 2;
    const bool ragged_ok = direct && mfma_dl_edge_shape_ok(g, A_KM, B_KM);
    struct Cand { int bm, bn; bool exact, ok; };
    Cand cand[5] = {{256, 256, mfma_shape_ok<256, 256>(g, A_KM, B_KM), false}, {128, 128, mfma_shape_ok<128, 128>(g, A_KM, B_KM), false},
                    {128, 64, mfma_shape_ok<128, 64>(g, A_KM, B_KM), false},   {64, 128, mfma_shape_ok<64, 128>(g, A_KM, B_KM), false},
                    {64, 64, mfma_shape_ok<64, 64>(g, A_KM, B_KM), false}};
    for (int i = 0; i < 5; ++i) cand[i].ok = cand[i].exact || (i < 2 && ragged_ok);
    auto tiles = [&](const Cand& c) { return (long)((g.M + c.bm - 1) / c.bm) * ((g.N + c.bn - 1) / c.bn) * g.batch; };
    auto fills = [&](int i) {
        const long t = tiles(cand[i]);
        if (i > 0) return t >= st->n_cu * 3 / 4;
        const long rounds = (t + st->n_cu - 1) / st->n_cu;
        return t >= st->n_cu && 10 * t >= 7 * rounds * st->n_cu;
    };
    int pick = -1;
    for (int i = 0; i < 5 && pick < 0; ++i)
        if (cand[i].ok && fills(i)) pick = i;
    if (pick < 0)
        for (int i = 0; i < 5; ++i)
            if (cand[i].ok && (pick < 0 || tiles(cand[i]) > tiles(cand[pick]))) pick = i;
    if (st->force_tile > 0)
        for (int i = 0; i < 5; ++i)
            if (cand[i].ok && (cand[i].bm * 1000 + cand[i].bn == st->force_tile ||
                               (cand[i].bm == cand[i].bn && cand[i].bm == st->force_tile))) pick = i;
    if (st->force_tile < 0) pick = -1;
    char name[48];
    if (pick >= 0)
        snprintf(name, sizeof(name), "gemm_mfma%dx%d_%s%s", cand[pick].bm, cand[pick].bn,
                 A_KM ? "TN" : (B_KM ? "NN" : "NT"), g.batch > 1 ? "_batched" : "");
    else
        snprintf(name, sizeof(name), "gemm_generic_%s%s", A_KM ? "TN" : (B_KM ? "NN" : "NT"), g.batch > 1 ? "_batched" : "");
    ProfScope ps(st, name, gemm_flops(g), 0.0);
    hipError_t e;
    if (pick >= 0 && pick < 2 && !cand[pick].exact) {
        e = pick == 0 ? launch_gemm_mfma_dl<256, 256, A_KM, B_KM, 4, true>(g, st->launch)
                      : launch_gemm_mfma_dl<128, 128, A_KM, B_KM, 2, true>(g, st->launch);
        return hip_ok(e, name) ? AMDP_OK : AMDP_E_HIP;
    }
    // Plain products load their tiles straight into LDS where that measured faster: the
    // 128x128 tile in every layout once more than one workgroup per compute unit is
    // resident (7-18 %; with fewer the eight-wave kernel below stays ahead), the
    // 256x256 tile for NT and TN (1-5 %; NN measured up to 18 % slower there).
    constexpr bool NN_LAYOUT = !A_KM && B_KM;
    if (direct && pick == 0 && (!NN_LAYOUT || always)) {
        e = launch_gemm_mfma_dl<256, 256, A_KM, B_KM, 4>(g, st->launch);
        return hip_ok(e, name) ? AMDP_OK : AMDP_E_HIP;
    }
    if (direct && pick == 1 && (tiles(cand[1]) > st->n_cu || always)) {
        e = launch_gemm_mfma_dl<128, 128, A_KM, B_KM, 2>(g, st->launch);
        return hip_ok(e, name) ? AMDP_OK : AMDP_E_HIP;
    }
    switch (pick) {
        case 0: e = launch_tile<256, 256, A_KM, B_KM, 4>(st, g); break;   // eight waves (two per SIMD), each 128x64 of the tile
        case 1:
            // up to three workgroups per compute unit: eight waves (two per SIMD, each
            // 64x32 of the tile) hide the latency that further resident workgroups
            // would otherwise hide; measured 3-14 % faster there, 2-5 % slower beyond
            e = tiles(cand[1]) <= 3 * st->n_cu ? launch_tile<128, 128, A_KM, B_KM, 4>(st, g)
                                           : launch_tile<128, 128, A_KM, B_KM>(st, g);
            break;
        case 2: e = launch_tile<128, 64, A_KM, B_KM>(st, g); break;
        case 3: e = launch_tile<64, 128, A_KM, B_KM>(st, g); break;
        case 4: e = launch_tile<64, 64, A_KM, B_KM>(st, g); break;
        default: e = launch_gemm_simple<bf16>(g, st->launch);
    }
    return hip_ok(e, name) ? AMDP_OK : AMDP_E_HIP;
}

enum GemmLayout { G_NN, G_NT, G_TN };

// A bf16-output product on the main chain whose 256x256 tiles would cover at most
// half of the compute units, with a long contraction: the contraction is split
// in two so that every unit gets a 256x256 tile (one batched launch into fp32
// scratch), and a second kernel adds the parts in order and applies bias and
// residual. Measured on configuration 5's 2048 x 4096 outputs with operands that
// are not cache-resident, against the 128x128 tile at two workgroups per unit:
// +15 to +19 % at contractions of 12288 and 16384, -6 to -10 % at 4096; on
// configuration 4's 4096 x 2048 outputs +0.5 to +13 % at 8192, +6 to +7 % at 6144,
// -22 to -25 % at 2048. Hence: a half must be at least 3072 long.
int main_split(const amdp_stage* st, const GemmArgs& g, bool a_km, bool b_km) {
    if (!st->d.bf || st->force_tile != 0 || g.batch != 1 || g.causal || g.epi.out_f32 || g.epi.gelu_u || g.epi.aux_out)
        return 1;
    if (g.M % 256 || g.N % 256 || g.ldc != g.N || (g.epi.res && g.epi.ldr != g.N) || g.epi.alpha != 1.0f) return 1;
    const long tiles = (long)(g.M / 256) * (g.N / 256);
    if (tiles * 2 > st->n_cu || g.K % (2 * MF_BK) || g.K / 2 < st->split_main_min_k) return 1;
    if ((size_t)g.M * g.N * 4 * 2 > st->w.splitm_bytes) return 1;
    GemmArgs part = g;
    part.K = g.K / 2;
    return mfma_shape_ok<256, 256>(part, a_km, b_km) ? 2 : 1;
}
template <bool A_KM, bool B_KM>
int gemm_main_split(amdp_stage* st, GemmArgs g, int ways) {
    const Epilogue epi = g.epi;
    void* out = g.C;
    float* partial = st->at<float>(st->w.splitm);
    const int Kz = g.K / ways;
    char name[48];
    snprintf(name, sizeof(name), "gemm_mfma256x256_%s_splitk", A_KM ? "TN" : (B_KM ? "NN" : "NT"));
    {
        ProfScope ps(st, name, 2.0 * g.M * (double)g.N * g.K, 0.0);
        g.C = partial; g.K = Kz; g.epi = Epilogue(); g.epi.out_f32 = 1;
        g.batch = ways; g.batch_inner = 1;
        g.a_bo = (long)Kz * g.a_cs; g.b_bo = (long)Kz * g.b_rs; g.c_bo = (long)g.M * g.N;
        if (!hip_ok(launch_tile<256, 256, A_KM, B_KM, 4>(st, g), name)) return AMDP_E_HIP;
    }
    const long n8 = (long)g.M * g.N / 8;
    ProfScope ps(st, "splitk_reduce", 0.0, (double)g.M * g.N * (4.0 * ways + 2.0 + (epi.res ? 2.0 : 0.0)));
    hipLaunchKernelGGL(splitk_epilogue_kernel, dim3(direct_grid(n8, ACC_BLOCK)), dim3(ACC_BLOCK), 0, st->launch,
                       (bf16*)out, partial, (const bf16*)epi.bias, (const bf16*)epi.res, n8, g.N, ways);
    return after_launch();
}

// lda/ldb are the leading dimensions of the operands AS STORED:
//   NN: A [M,K] lda, B [K,N] ldb      NT: A [M,K], B [N,K]      TN: A [K,M], B [K,N]
int gemm(amdp_stage* st, GemmLayout lay, GemmArgs g, long lda, long ldb) {
    switch (lay) {
        case G_NN: g.a_rs = lda; g.a_cs = 1; g.b_rs = ldb; g.b_cs = 1; break;
        case G_NT: g.a_rs = lda; g.a_cs = 1; g.b_rs = 1; g.b_cs = ldb; break;
        case G_TN: g.a_rs = 1; g.a_cs = lda; g.b_rs = ldb; g.b_cs = 1; break;
    }
    if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return AMDP_OK;
    if (!st->d.bf) {
        ProfScope ps(st, "gemm_generic_fp32", gemm_flops(g), 0.0);
        return hip_ok(launch_gemm_simple<float>(g, st->launch), "gemm_generic_fp32") ? AMDP_OK : AMDP_E_HIP;
    }
    switch (lay) {
        case G_NN:
            if (const int ways = main_split(st, g, false, true); ways > 1) return gemm_main_split<false, true>(st, g, ways);
            return gemm_bf16_layout<false, true>(st, g);
        case G_NT:
            if (const int ways = main_split(st, g, false, false); ways > 1) return gemm_main_split<false, false>(st, g, ways);
            return gemm_bf16_layout<false, false>(st, g);
        default: return gemm_bf16_layout<true, true>(st, g);
    }
}

// ---- typed launch helpers ---------------------------------------------------
// 16-byte vectors per lane of the LayerNorm kernels that keep a row in registers
// (1, 2, 4, 8 or 16: rows up to 64 * 16 vectors), 0 when the row is longer.
template <class T>
inline int ln_reg_vectors(int D) {
    constexpr int V = Vec<T>::N;
    if (D % V) return 0;
    const int need = (D / V + 63) / 64;
    for (int nv : {1, 2, 4, 8, 16})
        if (need <= nv) return nv;
    return 0;
}
template <class T>
int launch_ln_fwd(hipStream_t s, const void* x, const void* gamma, const void* beta, void* y, float* stats, int N,
                  int D, float eps) {
    const dim3 grid((N + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK);
#define LN_FWD(KERN) hipLaunchKernelGGL(KERN, grid, dim3(256), 0, s, (const T*)x, (const T*)gamma, (const T*)beta, (T*)y, stats, N, D, eps)
    switch (ln_reg_vectors<T>(D)) {
        case 1: LN_FWD((ln_fwd_reg_kernel<T, 1>)); break;
        case 2: LN_FWD((ln_fwd_reg_kernel<T, 2>)); break;
        case 4: LN_FWD((ln_fwd_reg_kernel<T, 4>)); break;
        case 8: LN_FWD((ln_fwd_reg_kernel<T, 8>)); break;
        case 16: LN_FWD((ln_fwd_reg_kernel<T, 16>)); break;
        default: LN_FWD(ln_fwd_kernel<T>);
    }
#undef LN_FWD
    return after_launch();
}

template <class T>
int launch_ln_bwd(hipStream_t s, const void* dy, const void* x, const float* stats, const void* gamma,
                  const void* res, void* dx, int N, int D) {
    const dim3 grid((N + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK);
#define LN_BWD(KERN) hipLaunchKernelGGL(KERN, grid, dim3(256), 0, s, (const T*)dy, (const T*)x, stats, (const T*)gamma, \
                                        (const T*)res, (T*)dx, N, D)
    switch (ln_reg_vectors<T>(D)) {
        case 1: LN_BWD((ln_bwd_reg_kernel<T, 1>)); break;
        case 2: LN_BWD((ln_bwd_reg_kernel<T, 2>)); break;
        case 4: LN_BWD((ln_bwd_reg_kernel<T, 4>)); break;
        case 8: LN_BWD((ln_bwd_reg_kernel<T, 8>)); break;
        case 16: LN_BWD((ln_bwd_reg_kernel<T, 16>)); break;
        default: LN_BWD(ln_bwd_kernel<T>);
    }
#undef LN_BWD
    return after_launch();
}
template <class T>
int ln_fwd(amdp_stage* st, const void* x, const void* gamma, const void* beta, void* y, float* stats) {
    const Dims& d = st->d;
    ProfScope ps(st, "layernorm_fwd", 0.0, (double)d.N * d.D * sizeof(T) * 2);
    return launch_ln_fwd<T>(st->launch, x, gamma, beta, y, stats, d.N, d.D, st->cfg.ln_eps);
}

// Column sums in two deterministic stages through `partial` (fp32 [chunks][width]).
// The split of the rows: enough chunks to put ~8 blocks on every compute unit, at
// least 16 rows each (a wave then has four rows' loads in flight), at most
// max_chunks (what `partial` has room for).
struct ColSumPlan { int col_blocks, chunks, rows_per_chunk; };
inline ColSumPlan plan_column_sums(int N, int C, int vec, int n_cu, int max_chunks) {
    ColSumPlan p;
    p.col_blocks = (C + 64 * vec - 1) / (64 * vec);
    int chunks = std::min(max_chunks, std::max(1, 8 * n_cu / p.col_blocks));
    p.rows_per_chunk = std::max(16, (N + chunks - 1) / chunks);
    p.chunks = (N + p.rows_per_chunk - 1) / p.rows_per_chunk;
    return p;
}
// out[0..C) = column sums of dy [N, C]; with LN: out[0..C) = sum dy*xhat, out[C..2C) = sum dy
template <class T, bool LN>
int launch_column_sums(hipStream_t s, const void* dy, const void* x, const float* stats, float* partial, float* out,
                       int N, int C, const ColSumPlan& p, int accumulate) {
    if (p.chunks > 0) {      // no rows: the second stage alone writes zeros
        hipLaunchKernelGGL((colreduce_partial_kernel<T, LN>), dim3(p.col_blocks, p.chunks), dim3(256), 0, s,
                           (const T*)dy, (const T*)x, stats, partial, N, C, p.rows_per_chunk);
        TRY(after_launch());
    }
    const int width = LN ? 2 * C : C;
    hipLaunchKernelGGL(colreduce_final_kernel, dim3((width + 15) / 16), dim3(256), 0, s, partial, out, width,
                       p.chunks, accumulate);
    return after_launch();
}
// The bias and LayerNorm-parameter gradients of one layer's backward, collected while the
// chain runs and reduced together in one pair of launches at the end of the layer (their
// inputs live in the layer's own scratch and in the activation slot until then).
struct ColSumList {
    ColSumBatch b;
    int blocks = 0;
    double bytes = 0.0;
    explicit ColSumList(int N) { b.n = 0; b.N = N; b.width = 0; b.rows_per_chunk = 0; }
};
// out[0..C) = column sums of dy [N, C]; with x: out[0..C) = sum dy*xhat, out[C..2C) = sum dy
template <class T>
void colsum_add(ColSumList& L, const void* dy, const void* x, const float* stats, float* out, int C) {
    ColSumSeg& sg = L.b.seg[L.b.n++];
    sg.dy = dy; sg.x = x; sg.stats = stats; sg.out = out; sg.C = C;
    sg.first_block = L.blocks; sg.woff = L.b.width; sg.width = x ? 2 * C : C;
    L.blocks += (C + 64 * Vec<T>::N - 1) / (64 * Vec<T>::N);
    L.b.width += sg.width;
    L.bytes += (double)L.b.N * C * sizeof(T) * (x ? 2 : 1);
}
template <class T>
int colsum_flush(amdp_stage* st, ColSumList& L) {
    if (L.b.n == 0) return AMDP_OK;
    // ~8 blocks per compute unit, at least 16 rows per chunk (four rows' loads in flight per wave)
    int chunks = std::min(st->w.partial_chunks, std::max(1, 8 * st->n_cu / L.blocks));
    L.b.rows_per_chunk = std::max(16, (L.b.N + chunks - 1) / chunks);
    chunks = (L.b.N + L.b.rows_per_chunk - 1) / L.b.rows_per_chunk;
    float* partial = st->at<float>(st->w.partial);
    ProfScope ps(st, "column_sums", 0.0, L.bytes);
    hipLaunchKernelGGL(colsum_batch_partial_kernel<T>, dim3(L.blocks, chunks), dim3(256), 0, st->launch, L.b, partial);
    TRY(after_launch());
    hipLaunchKernelGGL(colsum_batch_final_kernel, dim3((L.b.width + 15) / 16), dim3(256), 0, st->launch, L.b, partial,
                       chunks, st->fused_acc ? 1 : 0);
    return after_launch();
}

GemmArgs attn_batch(const Dims& d) {
    GemmArgs g{};
    g.batch = d.b * d.H;
    g.batch_inner = d.H;
    return g;
}

inline bool flash_ok(const Dims& d) { return flash_shape_ok(d); }

// Workgroups of 256 lanes of kernel Kern that the whole GPU holds at once.
template <auto Kern>
int resident_blocks(int n_cu) {
    static std::atomic<int> per_cu{0};     // a property of the kernel's code: the same on every gfx950
    int v = per_cu.load(std::memory_order_relaxed);
    if (!v) {
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&v, Kern, 256, 0) != hipSuccess || v < 1) v = 1;
        per_cu.store(v, std::memory_order_relaxed);
    }
    return v * n_cu;
}

// dst[r][j][0..w_dst) = src[r][j][0..w_src) cut or zero-padded to w_dst, for
// `chunks` head-sized column blocks per row (both widths even).
int repack_heads(amdp_stage* st, const void* src, void* dst, long rows, int chunks, int w_src, int w_dst) {
    const long pairs = rows * chunks * (w_dst / 2);
    ProfScope ps(st, "attention_repack_heads", 0.0, 2.0 * rows * chunks * (double)(w_src < w_dst ? w_src + w_dst : 2 * w_dst));
    hipLaunchKernelGGL(repack_heads_kernel, dim3((unsigned)((pairs + 255) / 256)), dim3(256), 0, st->launch,
                       (const uint32_t*)src, (uint32_t*)dst, pairs, w_src / 2, w_dst / 2);
    return after_launch();
}

// qkv [N, 3*Dk], o [N, Dk] with heads of DHK = 64 or 128 columns (Dk = H*DHK)
int flash_fwd_launch(amdp_stage* st, const void* qkv, void* o, float* lse2, const int32_t* valid, int dhk) {
    const Dims& d = st->d;
    const float sc = LOG2E / sqrtf((float)d.dh);
    const int Dk = d.H * dhk;
    if (d.causal && valid) return AMDP_E_INVAL;      // the causal kernels carry no padding mask
    dim3 grid((d.s / 128) * d.b * d.H);
    ProfScope ps(st, "flash_attention_fwd", 4.0 * d.b * d.H * (double)d.s * d.s * d.dh * (d.causal ? (d.s + 1.0) / (2.0 * d.s) : 1.0), 0.0);
#define FLASH_FWD(DH, C) hipLaunchKernelGGL((flash_fwd_kernel<DH, C>), grid, dim3(256), 0, st->launch, (const bf16*)qkv, \
                                            (bf16*)o, lse2, valid, d.s, d.H, Dk, sc, d.b * d.H,                     \
                                            resident_blocks<flash_fwd_kernel<DH, C>>(st->n_cu))
    if (dhk == 128) { if (d.causal) FLASH_FWD(128, true); else FLASH_FWD(128, false); }
    else { if (d.causal) FLASH_FWD(64, true); else FLASH_FWD(64, false); }
#undef FLASH_FWD
    return after_launch();
}

int flash_fwd(amdp_stage* st, const void* qkv, void* o, float* lse2, const int32_t* valid) {
    const Dims& d = st->d;
    const int dhk = flash_head_dim(d);
    if (!flash_packed(d)) return flash_fwd_launch(st, qkv, o, lse2, valid, dhk);
    void* pq = st->at<>(st->w.pk_qkv);
    void* po = st->at<>(st->w.pk_o);
    TRY(repack_heads(st, qkv, pq, d.N, 3 * d.H, d.dh, dhk));
    TRY(flash_fwd_launch(st, pq, po, lse2, valid, dhk));
    return repack_heads(st, po, o, d.N, d.H, dhk, d.dh);
}

// delta, dK/dV and dQ kernels; lse2 is what flash_fwd saved, delta is scratch [b*H*s] fp32
int flash_bwd_launch(amdp_stage* st, const void* dO, const void* qkv, const void* o, const float* lse2, float* delta,
                     void* dqkv, const int32_t* valid, int dhk) {
    const Dims& d = st->d;
    const float scale = 1.0f / sqrtf((float)d.dh);
    const int Dk = d.H * dhk;
    if (d.causal && valid) return AMDP_E_INVAL;      // the causal kernels carry no padding mask
    const double unit = 2.0 * d.b * d.H * (double)d.s * d.s * d.dh * (d.causal ? (d.s + 1.0) / (2.0 * d.s) : 1.0);
    dim3 grid((d.s / 128) * d.b * d.H);
    {
        ProfScope ps(st, "attention_delta", 0.0, 2.0 * d.N * d.D * 2.0);
        if (dhk == 128)
            hipLaunchKernelGGL(attn_delta_kernel<128>, dim3((d.N + 3) / 4), dim3(256), 0, st->launch, (const bf16*)dO,
                               (const bf16*)o, delta, d.N, d.s, d.H, Dk);
        else
            hipLaunchKernelGGL(attn_delta_kernel<64>, dim3((d.N + 3) / 4), dim3(256), 0, st->launch, (const bf16*)dO,
                               (const bf16*)o, delta, d.N, d.s, d.H, Dk);
        TRY(after_launch());
    }
#define FLASH_BWD(KERN, DH, C) hipLaunchKernelGGL((KERN<DH, C>), grid, dim3(256), 0, st->launch, (const bf16*)qkv, \
                                                  (const bf16*)dO, lse2, (const float*)delta, (bf16*)dqkv, valid, d.s, d.H, Dk, scale, \
                                                  d.b * d.H, resident_blocks<KERN<DH, C>>(st->n_cu))
    {
        ProfScope ps(st, "flash_attention_bwd_dkdv", 3.0 * unit, 0.0);   // dP, dV, dK (the recomputed S is not counted)
        if (dhk == 128) { if (d.causal) FLASH_BWD(flash_bwd_dkv_kernel, 128, true); else FLASH_BWD(flash_bwd_dkv_kernel, 128, false); }
        else { if (d.causal) FLASH_BWD(flash_bwd_dkv_kernel, 64, true); else FLASH_BWD(flash_bwd_dkv_kernel, 64, false); }
        TRY(after_launch());
    }
    {
        ProfScope ps(st, "flash_attention_bwd_dq", 1.0 * unit, 0.0);     // dQ (S and dP are recomputed, not counted)
        if (dhk == 128) { if (d.causal) FLASH_BWD(flash_bwd_dq_kernel, 128, true); else FLASH_BWD(flash_bwd_dq_kernel, 128, false); }
        else { if (d.causal) FLASH_BWD(flash_bwd_dq_kernel, 64, true); else FLASH_BWD(flash_bwd_dq_kernel, 64, false); }
        TRY(after_launch());
    }
#undef FLASH_BWD
    return AMDP_OK;
}

int flash_bwd(amdp_stage* st, const void* dO, const void* qkv, const void* o, const float* lse2, float* delta,
              void* dqkv, const int32_t* valid) {
    const Dims& d = st->d;
    const int dhk = flash_head_dim(d);
    if (!flash_packed(d)) return flash_bwd_launch(st, dO, qkv, o, lse2, delta, dqkv, valid, dhk);
    void* pq = st->at<>(st->w.pk_qkv);
    void* po = st->at<>(st->w.pk_o);
    void* pdo = st->at<>(st->w.pk_do);
    void* pdq = st->at<>(st->w.pk_dqkv);
    TRY(repack_heads(st, qkv, pq, d.N, 3 * d.H, d.dh, dhk));
    TRY(repack_heads(st, o, po, d.N, d.H, d.dh, dhk));
    TRY(repack_heads(st, dO, pdo, d.N, d.H, d.dh, dhk));
    TRY(flash_bwd_launch(st, pdo, pq, po, lse2, delta, pdq, valid, dhk));
    return repack_heads(st, pdq, dqkv, d.N, 3 * d.H, dhk, d.dh);
}

template <class T>
int attention_fwd(amdp_stage* st, const void* qkv_, void* P_, void* o_, const int32_t* valid) {
    const Dims& d = st->d;
    if (st->flash && flash_ok(d)) return flash_fwd(st, qkv_, o_, (float*)P_, valid);
    const T* qkv = (const T*)qkv_;
    const long ld3 = 3L * d.D;
    {   // S = Q K^T
        GemmArgs g = attn_batch(d);
        g.A = qkv; g.B = qkv + d.D; g.C = P_;
        g.M = d.s; g.N = d.s; g.K = d.dh; g.ldc = d.s;
        g.a_bo = (long)d.s * ld3; g.a_bi = d.dh; g.b_bo = g.a_bo; g.b_bi = d.dh;
        g.c_bo = (long)d.H * d.s * d.s; g.c_bi = (long)d.s * d.s;
        g.causal = d.causal ? 1 : 0;
        TRY(gemm(st, G_NT, g, ld3, ld3));
    }
    const long rows = (long)d.b * d.H * d.s;
    {
    ProfScope ps(st, "softmax_fwd", 0.0, (double)rows * d.s * sizeof(T) * (d.causal ? 1.5 : 2.0));
    hipLaunchKernelGGL(softmax_fwd_kernel<T>, dim3((unsigned)((rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK)),
                       dim3(256), 0, st->launch, (T*)P_, rows, d.s, 1.0f / sqrtf((float)d.dh),
                       d.causal ? 1 : 0, valid, d.H);
    }
    TRY(after_launch());
    {   // O = P V
        GemmArgs g = attn_batch(d);
        g.A = P_; g.B = qkv + 2 * d.D; g.C = o_;
        g.M = d.s; g.N = d.dh; g.K = d.s; g.ldc = d.D;
        g.a_bo = (long)d.H * d.s * d.s; g.a_bi = (long)d.s * d.s;
        g.b_bo = (long)d.s * ld3; g.b_bi = d.dh;
        g.c_bo = (long)d.s * d.D; g.c_bi = d.dh;
        g.causal = d.causal ? 2 : 0;
        TRY(gemm(st, G_NN, g, d.s, ld3));
    }
    return AMDP_OK;
}

// dqkv from d_out, the saved qkv and probabilities; dP is scratch [b*H, s, s]
template <class T>
int attention_bwd(amdp_stage* st, const void* dO_, const void* qkv_, const void* P_, const void* o_, void* dP_,
                  void* dqkv_, const int32_t* valid) {
    const Dims& d = st->d;
    if (st->flash && flash_ok(d))
        return flash_bwd(st, dO_, qkv_, o_, (const float*)P_, (float*)dP_, dqkv_, valid);
    const T* qkv = (const T*)qkv_;
    T* dqkv = (T*)dqkv_;
    const long ld3 = 3L * d.D;
    const long sP_o = (long)d.H * d.s * d.s, sP_i = (long)d.s * d.s;
    const long sQ_o = (long)d.s * ld3, sQ_i = d.dh;
    const long sO_o = (long)d.s * d.D, sO_i = d.dh;
    {   // dV = P^T dO
        GemmArgs g = attn_batch(d);
        g.A = P_; g.B = dO_; g.C = dqkv + 2 * d.D;
        g.M = d.s; g.N = d.dh; g.K = d.s; g.ldc = ld3;
        g.a_bo = sP_o; g.a_bi = sP_i; g.b_bo = sO_o; g.b_bi = sO_i; g.c_bo = sQ_o; g.c_bi = sQ_i;
        g.causal = d.causal ? 3 : 0;
        TRY(gemm(st, G_TN, g, d.s, d.D));
    }
    {   // dP = dO V^T
        GemmArgs g = attn_batch(d);
        g.A = dO_; g.B = qkv + 2 * d.D; g.C = dP_;
        g.M = d.s; g.N = d.s; g.K = d.dh; g.ldc = d.s;
        g.a_bo = sO_o; g.a_bi = sO_i; g.b_bo = sQ_o; g.b_bi = sQ_i; g.c_bo = sP_o; g.c_bi = sP_i;
        g.causal = d.causal ? 1 : 0;
        TRY(gemm(st, G_NT, g, d.D, ld3));
    }
    const long rows = (long)d.b * d.H * d.s;
    {
    ProfScope ps(st, "softmax_bwd", 0.0, (double)rows * d.s * sizeof(T) * (d.causal ? 2.0 : 3.0));
    hipLaunchKernelGGL(softmax_bwd_kernel<T>, dim3((unsigned)((rows + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK)),
                       dim3(256), 0, st->launch, (const T*)P_, (T*)dP_, rows, d.s, 1.0f / sqrtf((float)d.dh),
                       d.causal ? 1 : 0, valid, d.H);
    }
    TRY(after_launch());
    {   // dQ = dS K
        GemmArgs g = attn_batch(d);
        g.A = dP_; g.B = qkv + d.D; g.C = dqkv;
        g.M = d.s; g.N = d.dh; g.K = d.s; g.ldc = ld3;
        g.a_bo = sP_o; g.a_bi = sP_i; g.b_bo = sQ_o; g.b_bi = sQ_i; g.c_bo = sQ_o; g.c_bi = sQ_i;
        g.causal = d.causal ? 2 : 0;
        TRY(gemm(st, G_NN, g, d.s, ld3));
    }
    {   // dK = dS^T Q
        GemmArgs g = attn_batch(d);
        g.A = dP_; g.B = qkv; g.C = dqkv + d.D;
        g.M = d.s; g.N = d.dh; g.K = d.s; g.ldc = ld3;
        g.a_bo = sP_o; g.a_bi = sP_i; g.b_bo = sQ_o; g.b_bi = sQ_i; g.c_bo = sQ_o; g.c_bi = sQ_i;
        g.causal = d.causal ? 3 : 0;
        TRY(gemm(st, G_TN, g, d.s, ld3));
    }
    return AMDP_OK;
}

// Y[M,N] = X[M,K] W[K,N] (+bias) (+res) ; optional second output gelu(Y)
int linear_fwd(amdp_stage* st, const void* X, const void* W, const void* bias, const void* res, void* Y,
               void* gelu_out, int M, int N, int K) {
    GemmArgs g{};
    g.A = X; g.B = W; g.C = Y; g.M = M; g.N = N; g.K = K; g.ldc = N;
    g.epi.bias = bias; g.epi.res = res; g.epi.ldr = N; g.epi.aux_out = gelu_out;
    return gemm(st, G_NN, g, K, N);
}
// dX[M,K] = dY[M,N] W[K,N]^T (* gelu'(u)) (+res)
int linear_dx(amdp_stage* st, const void* dY, const void* W, const void* gelu_u, const void* res, void* dX,
              int M, int N, int K) {
    GemmArgs g{};
    g.A = dY; g.B = W; g.C = dX; g.M = M; g.N = K; g.K = N; g.ldc = K;
    g.epi.gelu_u = gelu_u; g.epi.ldu = K; g.epi.res = res; g.epi.ldr = K;
    return gemm(st, G_NT, g, N, N);
}
// How many ways the token dimension of a weight-gradient product [rows x cols] is
// split over workgroups (1 = not at all). A product whose 128x128 tiles cover at
// most half of the compute units gets one workgroup per unit instead: the parts
// go to scratch and are added in fixed order afterwards (no float atomics).
int dw_split(const amdp_stage* st, int rows, int cols, int tokens) {
    if (!st->d.bf || st->force_tile != 0 || rows % 128 || cols % 128 || !st->w.splitk_bytes) return 1;
    const long tiles = (long)(rows / 128) * (cols / 128);
    int ways = 1;
    while (ways < 8 && tiles * ways * 2 <= st->n_cu && tokens % (ways * 2 * MF_BK) == 0 &&
           tokens / (ways * 2) >= st->splitk_min_k &&
           (size_t)rows * cols * 4 * (size_t)(ways * 2) <= st->w.splitk_bytes)
        ways *= 2;
    return ways;
}
// dW[K,N] (fp32) = X[M,K]^T dY[M,N]
int linear_dw(amdp_stage* st, const void* X, const void* dY, float* dW, int M, int N, int K) {
    GemmArgs g{};
    g.A = X; g.B = dY; g.C = dW; g.M = K; g.N = N; g.K = M; g.ldc = N;
    g.epi.out_f32 = 1;
    g.epi.accumulate = st->fused_acc ? 1 : 0;
    const int ways = dw_split(st, K, N, M);
    if (ways == 1) return gemm(st, G_TN, g, K, N);
    // one batched launch: part z contracts tokens [z * M/ways, (z+1) * M/ways) into partial[z]
    float* partial = st->at<float>(st->w.splitk);
    const int Mz = M / ways;
    g.C = partial; g.K = Mz; g.epi.accumulate = 0;
    g.batch = ways; g.batch_inner = 1;
    g.a_rs = 1; g.a_cs = K; g.b_rs = N; g.b_cs = 1;
    g.a_bo = (long)Mz * K; g.b_bo = (long)Mz * N; g.c_bo = (long)K * N;
    if (!mfma_shape_ok<128, 128>(g, true, true)) {      // alignment the tile kernel needs: fall back to one launch
        GemmArgs one{};
        one.A = X; one.B = dY; one.C = dW; one.M = K; one.N = N; one.K = M; one.ldc = N;
        one.epi.out_f32 = 1; one.epi.accumulate = st->fused_acc ? 1 : 0;
        return gemm(st, G_TN, one, K, N);
    }
    {
        ProfScope ps(st, "gemm_mfma128x128_TN_splitk", 2.0 * K * (double)N * M, 0.0);
        hipError_t e = st->use_tr ? launch_gemm_mfma_inst<128, 128, true, true, true, 4>(g, st->launch)
                                  : launch_gemm_mfma_inst<128, 128, true, true, false, 4>(g, st->launch);
        if (!hip_ok(e, "gemm_mfma128x128_TN_splitk")) return AMDP_E_HIP;
    }
    const long n4 = (long)K * N / 4;
    ProfScope ps(st, "splitk_reduce", 0.0, (double)K * N * 4 * (ways + 1 + (st->fused_acc ? 1 : 0)));
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3(direct_grid(n4, ACC_BLOCK)), dim3(ACC_BLOCK), 0, st->launch, dW,
                       partial, n4, ways, st->fused_acc ? 1 : 0);
    return after_launch();
}

template <class T>
int forward_impl(amdp_stage* st, int aslot, int vslot, const void* X, const int32_t* aux, void* out) {
    const Dims& d = st->d;
    const T* W = (const T*)st->version_ptr(vslot);
    char* S = st->act_ptr(aslot);
    const size_t ND = (size_t)d.N * d.D * sizeof(T);
    // aux is the padding mask for bidirectional blocks, the targets on an LM-head
    // stage, and on a first stage the token ids followed by the padding mask
    const int32_t* valid = (!d.causal && !d.lm) ? (d.emb ? aux + d.N : aux) : nullptr;
    if (valid) TRY(device_copy(st->launch, S + st->w.slot.valid, valid, (size_t)d.b * 4));
    if (d.emb) {
        TRY(device_copy(st->launch, S + st->w.slot.tokens, aux, (size_t)d.N * 4));
        ProfScope ps(st, "embedding_fwd", 0.0, 3.0 * (double)ND);
        hipLaunchKernelGGL(embed_fwd_kernel<T>, dim3((d.N + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK), dim3(256), 0,
                           st->launch, W + d.off_tok(), W + d.off_pos(), aux, (T*)(S + st->w.slot.layers[0].xin),
                           d.N, d.s, d.D, d.V);
        TRY(after_launch());
    } else {
        ProfScope ps(st, "copy_input", 0.0, 2.0 * (double)ND);
        TRY(device_copy(st->launch, S + st->w.slot.layers[0].xin, X, ND));
    }
    for (int l = 0; l < d.L; ++l) {
        const LayerAct& a = st->w.slot.layers[l];
        void* xin = S + a.xin;
        void* yout = (l + 1 < d.L) ? (void*)(S + st->w.slot.layers[l + 1].xin)
                                   : (d.lm ? (void*)(S + st->w.slot.yL) : out);
        auto P = [&](int f) { return (const void*)(W + d.off(l, f)); };
        if (d.causal) {
            TRY(ln_fwd<T>(st, xin, P(LN1_G), P(LN1_B), S + a.a, (float*)(S + a.st1)));
            TRY(linear_fwd(st, S + a.a, P(W_QKV), P(B_QKV), nullptr, S + a.qkv, nullptr, d.N, 3 * d.D, d.D));
            TRY(attention_fwd<T>(st, S + a.qkv, S + a.P, S + a.o, valid));
            TRY(linear_fwd(st, S + a.o, P(W_O), P(B_O), xin, S + a.y1, nullptr, d.N, d.D, d.D));
            TRY(ln_fwd<T>(st, S + a.y1, P(LN2_G), P(LN2_B), S + a.c, (float*)(S + a.st2)));
            TRY(linear_fwd(st, S + a.c, P(W_1), P(B_1), nullptr, S + a.u, S + a.h, d.N, d.F, d.D));
            TRY(linear_fwd(st, S + a.h, P(W_2), P(B_2), S + a.y1, yout, nullptr, d.N, d.D, d.F));
        } else {
            // post-LN: field `a` holds the pre-norm sum after attention, `c` the one after the MLP
            TRY(linear_fwd(st, xin, P(W_QKV), P(B_QKV), nullptr, S + a.qkv, nullptr, d.N, 3 * d.D, d.D));
            TRY(attention_fwd<T>(st, S + a.qkv, S + a.P, S + a.o, valid));
            TRY(linear_fwd(st, S + a.o, P(W_O), P(B_O), xin, S + a.a, nullptr, d.N, d.D, d.D));
            TRY(ln_fwd<T>(st, S + a.a, P(LN1_G), P(LN1_B), S + a.y1, (float*)(S + a.st1)));
            TRY(linear_fwd(st, S + a.y1, P(W_1), P(B_1), nullptr, S + a.u, S + a.h, d.N, d.F, d.D));
            TRY(linear_fwd(st, S + a.h, P(W_2), P(B_2), S + a.y1, S + a.c, nullptr, d.N, d.D, d.F));
            TRY(ln_fwd<T>(st, S + a.c, P(LN2_G), P(LN2_B), yout, (float*)(S + a.st2)));
        }
    }
    if (d.lm) {
        const SlotLayout& sl = st->w.slot;
        TRY(ln_fwd<T>(st, S + sl.yL, W + d.off_lnf(), W + d.off_lnf() + d.D, S + sl.z, (float*)(S + sl.stf)));
        GemmArgs g{};   // logits = z E^T ; pad rows of E are zero in every version slot
        g.A = S + sl.z; g.B = W + d.off_embed(); g.C = S + sl.dlogits;
        g.M = d.N; g.N = (int)d.Vld; g.K = d.D; g.ldc = d.Vld;
        TRY(gemm(st, G_NT, g, d.D, d.D));
        float* row_loss = st->at<float>(st->w.row_loss);
        ProfScope ps(st, "cross_entropy", 0.0, (double)d.N * d.V * sizeof(T) * 2);
        hipLaunchKernelGGL(ce_fwd_kernel<T>, dim3((d.N + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK), dim3(256), 0,
                           st->launch, (T*)(S + sl.dlogits), aux, row_loss, d.N, d.V, d.Vld);
        TRY(after_launch());
        hipLaunchKernelGGL(mean_kernel, dim3(1), dim3(256), 0, st->launch, row_loss, (float*)out, d.N);
        TRY(after_launch());
    }
    return AMDP_OK;
}

// While a Leaf is alive, launches go to the side stream, ordered after
// everything enqueued on the main stream so far.
struct Leaf {
    amdp_stage* st;
    bool ok = true;
    explicit Leaf(amdp_stage* s) : st(s) {
        if (!st->overlap) return;
        hipEvent_t ev = st->next_event();
        ok = hip_ok(hipEventRecord(ev, st->stream), "hipEventRecord(fork)") &&
             hip_ok(hipStreamWaitEvent(st->side, ev, 0), "hipStreamWaitEvent(fork)");
        if (ok) st->launch = st->side;
    }
    ~Leaf() { st->launch = st->stream; }
};
// The main stream waits for every leaf enqueued so far.
int join_leaves(amdp_stage* st) {
    if (!st->overlap) return AMDP_OK;
    hipEvent_t ev = st->next_event();
    HIP_TRY(hipEventRecord(ev, st->side));
    HIP_TRY(hipStreamWaitEvent(st->stream, ev, 0));
    for (int i = 0; i < st->cfg.act_slots; ++i) st->leaves_pending[i] = false;
    st->last_leaves = -1;
    return AMDP_OK;
}
// End of a backward: remember where its leaves end instead of waiting for them.
int mark_leaves(amdp_stage* st, int aslot) {
    if (!st->overlap) return AMDP_OK;
    if (!st->lazy_join) return join_leaves(st);
    HIP_TRY(hipEventRecord(st->leaves_ev[aslot], st->side));
    st->leaves_pending[aslot] = true;
    st->last_leaves = aslot;
    return AMDP_OK;
}
// The main stream waits for the leaves of the backward that used `aslot`, if they may still run.
int wait_leaves_of(amdp_stage* st, int aslot) {
    if (aslot < 0 || !st->leaves_pending[aslot]) return AMDP_OK;
    HIP_TRY(hipStreamWaitEvent(st->stream, st->leaves_ev[aslot], 0));
    st->leaves_pending[aslot] = false;
    if (st->last_leaves == aslot) st->last_leaves = -1;
    return AMDP_OK;
}
#define LEAF(stmts) do { Leaf leaf_(st); if (!leaf_.ok) return AMDP_E_HIP; stmts } while (0)

// LayerNorm backward: dx on the main chain; the parameter gradients (gain at
// grad_out[0..D), bias at grad_out[D..2D)) join the layer's column reductions.
template <class T>
int ln_bwd_pg(amdp_stage* st, ColSumList& cs, const void* dy, const void* x, const float* stats, const void* gamma,
              const void* res, void* dx, float* grad_out) {
    const Dims& d = st->d;
    colsum_add<T>(cs, dy, x, stats, grad_out, d.D);
    ProfScope ps(st, "layernorm_bwd", 0.0, (double)d.N * d.D * sizeof(T) * (res ? 4 : 3));
    return launch_ln_bwd<T>(st->launch, dy, x, stats, gamma, res, dx, d.N, d.D);
}

template <class T>
int backward_impl(amdp_stage* st, int aslot, int vslot, const int32_t* valid, const void* dY, void* dX) {
    const Dims& d = st->d;
    const T* W = (const T*)st->version_ptr(vslot);
    char* S = st->act_ptr(aslot);
    // parameter gradients go to the staging buffer, or straight into the sum
    float* g = st->at<float>(st->fused_acc ? st->w.G : st->w.g);
    void* dO = st->at<>(st->w.dO);      // main chain only
    void* dP = st->at<>(st->w.dP);      // main chain only

    const void* dcur = dY;
    bool dy_leaves = false;
    if (d.lm) {
        const SlotLayout& sl = st->w.slot;
        void* dz = st->at<>(st->w.lm_dz);
        void* dyL = st->at<>(st->w.lm_dy);
        LEAF({   // dE = dlogits^T z   (rows >= V are zero and land in the padding)
            GemmArgs a{};
            a.A = S + sl.dlogits; a.B = S + sl.z; a.C = g + d.off_embed();
            a.M = (int)d.Vld; a.N = d.D; a.K = d.N; a.ldc = d.D; a.epi.out_f32 = 1;
            a.epi.accumulate = st->fused_acc ? 1 : 0;
            TRY(gemm(st, G_TN, a, d.Vld, d.D));
        });
        {   // dz = dlogits E
            GemmArgs a{};
            a.A = S + sl.dlogits; a.B = W + d.off_embed(); a.C = dz;
            a.M = d.N; a.N = d.D; a.K = (int)d.Vld; a.ldc = d.D;
            TRY(gemm(st, G_NN, a, d.Vld, d.D));
        }
        ColSumList cs(d.N);
        TRY(ln_bwd_pg<T>(st, cs, dz, S + sl.yL, (const float*)(S + sl.stf), W + d.off_lnf(), nullptr, dyL, g + d.off_lnf()));
        LEAF({ TRY(colsum_flush<T>(st, cs)); });
        dcur = dyL;
    }

    for (int l = d.L - 1; l >= 0; --l) {
        const LayerAct& a = st->w.slot.layers[l];
        const Carve::BwdScratch& bw = st->w.bw[l];
        auto P = [&](int f) { return (const void*)(W + d.off(l, f)); };
        auto G = [&](int f) { return g + d.off(l, f); };
        void* ta = st->at<>(bw.t_a);
        void* tb = st->at<>(bw.t_b);
        void* tc = st->at<>(bw.t_c);
        void* dffn = st->at<>(bw.dffn);
        void* dqkv = st->at<>(bw.dqkv);
        void* dnext = (l == 0 && dX) ? dX : st->at<>(bw.dxout);
        const float* st1 = (const float*)(S + a.st1);
        const float* st2 = (const float*)(S + a.st2);
        ColSumList cs(d.N);
        // Weight-gradient products wait in `jobs` until the next fork: switching the
        // stream the host enqueues on costs more than ten launches, so a layer's leaves
        // go to the side stream in one or two groups. Nothing a leaf reads is
        // rewritten before the layer ends (the scratch is per layer).
        struct DwJob { const void* x; const void* dy; float* dw; int n, out, in; };
        DwJob jobs[4];
        int n_jobs = 0;
        auto flush_dw = [&](bool with_colsums) -> int {
            if (n_jobs == 0 && !with_colsums) return AMDP_OK;
            LEAF({
                for (int j = 0; j < n_jobs; ++j)
                    TRY(linear_dw(st, jobs[j].x, jobs[j].dy, jobs[j].dw, jobs[j].n, jobs[j].out, jobs[j].in));
                if (with_colsums) TRY(colsum_flush<T>(st, cs));
            });
            n_jobs = 0;
            return AMDP_OK;
        };
        auto leaf_dw = [&](const void* x, const void* dy, float* dw, int n, int out, int in, bool mid_layer) -> int {
            jobs[n_jobs++] = DwJob{x, dy, dw, n, out, in};
            if (!st->overlap || st->leaf_forks == 0 || (mid_layer && st->leaf_forks == 2)) return flush_dw(false);
            return AMDP_OK;
        };

        if (d.causal) {
            // y = y1 + MLP(LN2(y1))
            colsum_add<T>(cs, dcur, nullptr, nullptr, G(B_2), d.D);
            TRY(leaf_dw(S + a.h, dcur, G(W_2), d.N, d.D, d.F, false));
            TRY(linear_dx(st, dcur, P(W_2), S + a.u, nullptr, dffn, d.N, d.D, d.F));
            colsum_add<T>(cs, dffn, nullptr, nullptr, G(B_1), d.F);
            TRY(leaf_dw(S + a.c, dffn, G(W_1), d.N, d.F, d.D, true));
            TRY(linear_dx(st, dffn, P(W_1), nullptr, nullptr, ta, d.N, d.F, d.D));          // ta = dc
            TRY(ln_bwd_pg<T>(st, cs, ta, S + a.y1, st2, P(LN2_G), dcur, tb, G(LN2_G)));   // tb = dy1
            // y1 = x + Attn(LN1(x))
            colsum_add<T>(cs, tb, nullptr, nullptr, G(B_O), d.D);
            TRY(leaf_dw(S + a.o, tb, G(W_O), d.N, d.D, d.D, false));
            TRY(linear_dx(st, tb, P(W_O), nullptr, nullptr, dO, d.N, d.D, d.D));
            TRY(attention_bwd<T>(st, dO, S + a.qkv, S + a.P, S + a.o, dP, dqkv, valid));
            colsum_add<T>(cs, dqkv, nullptr, nullptr, G(B_QKV), 3 * d.D);
            TRY(leaf_dw(S + a.a, dqkv, G(W_QKV), d.N, 3 * d.D, d.D, false));
            TRY(linear_dx(st, dqkv, P(W_QKV), nullptr, nullptr, tc, d.N, 3 * d.D, d.D));     // tc = da
            TRY(ln_bwd_pg<T>(st, cs, tc, S + a.xin, st1, P(LN1_G), tb, dnext, G(LN1_G)));
        } else {
            // y = LN2(r2), r2 = y1 + MLP(y1); y1 = LN1(r1), r1 = x + Attn(x)
            TRY(ln_bwd_pg<T>(st, cs, dcur, S + a.c, st2, P(LN2_G), nullptr, ta, G(LN2_G)));   // ta = dr2
            colsum_add<T>(cs, ta, nullptr, nullptr, G(B_2), d.D);
            TRY(leaf_dw(S + a.h, ta, G(W_2), d.N, d.D, d.F, false));
            TRY(linear_dx(st, ta, P(W_2), S + a.u, nullptr, dffn, d.N, d.D, d.F));
            colsum_add<T>(cs, dffn, nullptr, nullptr, G(B_1), d.F);
            TRY(leaf_dw(S + a.y1, dffn, G(W_1), d.N, d.F, d.D, true));
            TRY(linear_dx(st, dffn, P(W_1), nullptr, ta, tb, d.N, d.F, d.D));               // tb = dy1
            TRY(ln_bwd_pg<T>(st, cs, tb, S + a.a, st1, P(LN1_G), nullptr, tc, G(LN1_G)));     // tc = dr1
            colsum_add<T>(cs, tc, nullptr, nullptr, G(B_O), d.D);
            TRY(leaf_dw(S + a.o, tc, G(W_O), d.N, d.D, d.D, false));
            TRY(linear_dx(st, tc, P(W_O), nullptr, nullptr, dO, d.N, d.D, d.D));
            TRY(attention_bwd<T>(st, dO, S + a.qkv, S + a.P, S + a.o, dP, dqkv, valid));
            colsum_add<T>(cs, dqkv, nullptr, nullptr, G(B_QKV), 3 * d.D);
            TRY(leaf_dw(S + a.xin, dqkv, G(W_QKV), d.N, 3 * d.D, d.D, false));
            TRY(linear_dx(st, dqkv, P(W_QKV), nullptr, tc, dnext, d.N, 3 * d.D, d.D));
        }
        TRY(flush_dw(true));
        // the leaves of this layer read the caller's dY: remember where they end
        if (dcur == dY && dY && st->overlap) {
            HIP_TRY(hipEventRecord(st->input_ev, st->side));
            dy_leaves = true;
        }
        dcur = dnext;
    }
    // The caller may reuse its buffers as soon as its stream gets past this call: the
    // main stream waits for the few leaves that read dY (they were enqueued first and
    // are long done), and for all of them when the input layer's leaves read the
    // caller's dX; every other leaf reads the stage's own memory and keeps running.
    if (dy_leaves) HIP_TRY(hipStreamWaitEvent(st->stream, st->input_ev, 0));
    if (d.emb) {
        // gradient of the input layer from dcur = d loss / d (block input)
        const int32_t* tokens = (const int32_t*)(S + st->w.slot.tokens);
        const int acc = st->fused_acc ? 1 : 0;
        LEAF({
            ProfScope ps(st, "embedding_bwd", 0.0, 2.0 * (double)d.N * d.D * sizeof(T));
            const long pv = (long)d.s * (d.D / Vec<T>::N);
            hipLaunchKernelGGL(pos_embed_bwd_kernel<T>, dim3((unsigned)((pv + 255) / 256)), dim3(256), 0, st->launch,
                               (const T*)dcur, g + d.off_pos(), d.b, d.s, d.D, acc);
            TRY(after_launch());
            // rows of absent tokens are zero in a minibatch's own gradient
            if (!acc) TRY(device_zero(st->launch, g + d.off_tok(), (size_t)d.V * d.D * 4));
            hipLaunchKernelGGL((tok_embed_bwd_kernel<T, 32 / Vec<T>::N>), dim3(d.N), dim3(256), 0, st->launch,
                               (const T*)dcur, tokens, g + d.off_tok(), d.N, d.D, d.V, acc);
            TRY(after_launch());
        });
        if (dcur == dX && dX) return join_leaves(st);
    }
    return mark_leaves(st, aslot);
}

template <class T>
int publish(amdp_stage* st, int vslot) {
    const long n4 = st->d.n_alloc() / 4;
    hipLaunchKernelGGL(publish_kernel<T>, dim3(stream_grid(n4)), dim3(STREAM_BLOCK), 0, st->launch,
                       st->at<float>(st->w.theta), (T*)st->version_ptr(vslot), n4);
    return after_launch();
}

}  // namespace

// ================================================================== C ABI ====

extern "C" size_t amdp_stage_n_params(const amdp_stage_config_t* cfg) {
    Dims d;
    return make_dims(cfg, &d) ? (size_t)d.n_params() : 0;
}

extern "C" size_t amdp_stage_workspace_bytes(const amdp_stage_config_t* cfg) {
    Dims d;
    if (!make_dims(cfg, &d)) return 0;
    Carve w;
    carve(d, *cfg, &w);
    return w.total;
}

extern "C" int amdp_stage_param_layout(const amdp_stage_config_t* cfg, amdp_param_desc_t* descs, int32_t cap,
                                       int32_t* n) {
    Dims d;
    if (!make_dims(cfg, &d) || !n) return AMDP_E_INVAL;
    const int total = d.L * N_FIELDS + (d.lm ? 3 : 0) + (d.emb ? 2 : 0);
    *n = total;
    if (cap < total || !descs) return AMDP_E_CAPACITY;
    int k = 0;
    auto put = [&](const char* name, long off, long rows, long cols) {
        memset(&descs[k], 0, sizeof(descs[k]));
        snprintf(descs[k].name, sizeof(descs[k].name), "%s", name);
        descs[k].offset = (uint64_t)off; descs[k].rows = (uint32_t)rows; descs[k].cols = (uint32_t)cols;
        ++k;
    };
    if (d.emb) {
        put("tok_embed", d.off_tok(), d.V, d.D);
        put("pos_embed", d.off_pos(), d.s, d.D);
    }
    for (int l = 0; l < d.L; ++l)
        for (int f = 0; f < N_FIELDS; ++f) {
            char name[24];
            snprintf(name, sizeof(name), "l%d.%s", l, FIELD_NAMES[f]);
            long rows = 1, cols = d.field_size(f);
            if (f == W_QKV) { rows = d.D; cols = 3L * d.D; }
            if (f == W_O) { rows = d.D; cols = d.D; }
            if (f == W_1) { rows = d.D; cols = d.F; }
            if (f == W_2) { rows = d.F; cols = d.D; }
            put(name, d.off(l, f), rows, cols);
        }
    if (d.lm) {
        put("lnf_gamma", d.off_lnf(), 1, d.D);
        put("lnf_beta", d.off_lnf() + d.D, 1, d.D);
        put("embed", d.off_embed(), d.V, d.D);
    }
    return AMDP_OK;
}

extern "C" int amdp_stage_create(const amdp_stage_config_t* cfg, void* workspace, size_t workspace_bytes,
                                 void* hip_stream, amdp_stage_t** out) {
    Dims d;
    if (!out || !workspace || !make_dims(cfg, &d)) return AMDP_E_INVAL;
    if ((uintptr_t)workspace % ALIGN) return AMDP_E_INVAL;
    amdp_stage* st = new (std::nothrow) amdp_stage();
    if (!st) return AMDP_E_INVAL;
    st->cfg = *cfg;
    st->d = d;
    carve(d, *cfg, &st->w);
    if (workspace_bytes < st->w.total) { delete st; return AMDP_E_INVAL; }
    st->base = (char*)workspace;
    st->stream = (hipStream_t)hip_stream;
    {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
            st->n_cu = cus;
    }
    st->launch = st->stream;
    st->n_vslots = cfg->stash_slots + 1;
    {
        bool ok = hip_ok(hipStreamCreateWithFlags(&st->side, hipStreamNonBlocking), "hipStreamCreateWithFlags");
        for (int i = 0; ok && i < 16; ++i)
            ok = hip_ok(hipEventCreateWithFlags(&st->events[i], hipEventDisableTiming), "hipEventCreateWithFlags");
        for (int i = 0; ok && i < cfg->act_slots; ++i)
            ok = hip_ok(hipEventCreateWithFlags(&st->leaves_ev[i], hipEventDisableTiming), "hipEventCreateWithFlags");
        ok = ok && hip_ok(hipEventCreateWithFlags(&st->input_ev, hipEventDisableTiming), "hipEventCreateWithFlags");
        if (!ok) { amdp_stage_destroy(st); return AMDP_E_HIP; }
    }
    // The side stream pays while the backward's products leave compute units idle. Once
    // even the smallest weight-gradient product of a layer (D x D) fills every compute
    // unit with a 256x256 tile, concurrent kernels only share the units (measured: no
    // gain at D = 4096, 3 % at 2048, 11 % at 1024), so it is off by default there.
    st->overlap = (long)(st->d.D / 256) * (st->d.D / 256) < st->n_cu;
    // Handing work to the side stream costs the host about 20 us each time (two event calls and
    // a change of the stream it enqueues on). One hand-over per product starts every leaf as
    // early as possible; two per layer cost the host half as much per backward. Measured per
    // step, GPU / host: D = 1024 causal 18.6 / 7.0 ms against 18.7 / 4.7, D = 1024
    // bidirectional 26.9 / 10 against 28.1 / 6.9, D = 2048 with LM head 77.0 / 6.8 against
    // 76.0 / 5.2: grouped from D = 2048 on.
    st->leaf_forks = st->d.D >= 2048 ? 2 : 0;
    st->flash = cfg->attention == AMDP_ATTN_AUTO;
    // parameter buffers, version slots and the padding behind them start at zero
    if (device_zero(st->launch, st->base, st->w.act) != AMDP_OK) {
        amdp_stage_destroy(st);
        return AMDP_E_HIP;
    }
    *out = st;
    return AMDP_OK;
}

extern "C" int amdp_stage_destroy(amdp_stage_t* st) {
    if (!st) return AMDP_E_INVAL;
    if (st->side) {
        hipStreamSynchronize(st->side);     // leaves still running read the workspace
        hipStreamDestroy(st->side);
    }
    for (hipEvent_t e : st->events) if (e) hipEventDestroy(e);
    for (hipEvent_t e : st->leaves_ev) if (e) hipEventDestroy(e);
    if (st->input_ev) hipEventDestroy(st->input_ev);
    delete st;
    return AMDP_OK;
}

extern "C" int amdp_stage_set_state(amdp_stage_t* st, const float* theta, const float* m, const float* v,
                                    uint64_t step, uint32_t version) {
    if (!st || !theta) return AMDP_E_INVAL;
    const size_t nb = (size_t)st->d.n_params() * 4, na = (size_t)st->d.n_alloc() * 4;
    if ((uintptr_t)theta % 4 || (uintptr_t)m % 4 || (uintptr_t)v % 4) return AMDP_E_INVAL;
    TRY(join_leaves(st));
    TRY(device_zero(st->launch, st->base + st->w.theta, na));
    TRY(device_zero(st->launch, st->base + st->w.m, na));
    TRY(device_zero(st->launch, st->base + st->w.v, na));
    TRY(device_zero(st->launch, st->base + st->w.G, na));
    TRY(device_zero(st->launch, st->base + st->w.g, na));
    TRY(device_copy(st->launch, st->base + st->w.theta, theta, nb));
    if (m) TRY(device_copy(st->launch, st->base + st->w.m, m, nb));
    if (v) TRY(device_copy(st->launch, st->base + st->w.v, v, nb));
    for (int i = 0; i < MAX_VSLOTS; ++i) st->vs[i] = VSlot();
    for (int i = 0; i < MAX_ASLOTS; ++i) st->as[i] = ASlot();
    st->staged_slot = -1;
    st->step = step;
    st->cur_version = version;
    st->cur_slot = 0;
    st->vs[0].valid = true;
    st->vs[0].version = version;
    return st->d.bf ? publish<bf16>(st, 0) : publish<float>(st, 0);
}

extern "C" int amdp_stage_get_state(amdp_stage_t* st, float* theta, float* m, float* v, float* G,
                                    uint64_t* step, uint32_t* version) {
    if (!st) return AMDP_E_INVAL;
    const size_t nb = (size_t)st->d.n_params() * 4;
    if (((uintptr_t)theta | (uintptr_t)m | (uintptr_t)v | (uintptr_t)G) % 4) return AMDP_E_INVAL;
    TRY(join_leaves(st));
    if (theta) TRY(device_copy(st->launch, theta, st->base + st->w.theta, nb));
    if (m) TRY(device_copy(st->launch, m, st->base + st->w.m, nb));
    if (v) TRY(device_copy(st->launch, v, st->base + st->w.v, nb));
    if (G) TRY(device_copy(st->launch, G, st->base + st->w.G, nb));
    if (step) *step = st->step;
    if (version) *version = st->cur_version;
    return AMDP_OK;
}

extern "C" int amdp_stage_get_staged_grad(amdp_stage_t* st, float* g) {
    if (!st || !g) return AMDP_E_INVAL;
    if (st->staged_slot < 0) return AMDP_E_MB_STATE;
    if ((uintptr_t)g % 4) return AMDP_E_INVAL;
    if (st->fused_acc) return AMDP_E_MB_STATE;           // the gradient went straight into the sum
    TRY(join_leaves(st));
    return device_copy(st->launch, g, st->base + st->w.g, (size_t)st->d.n_params() * 4);
}

extern "C" int amdp_stage_resident_versions(amdp_stage_t* st, uint32_t* versions, int32_t cap, int32_t* n) {
    if (!st || !n) return AMDP_E_INVAL;
    int k = 0;
    for (int i = 0; i < st->n_vslots; ++i)
        if (st->vs[i].valid) {
            if (versions && k < cap) versions[k] = st->vs[i].version;
            ++k;
        }
    *n = k;
    return (versions && k > cap) ? AMDP_E_CAPACITY : AMDP_OK;
}

extern "C" int amdp_stage_forward(amdp_stage_t* st, int32_t mb, uint32_t version, const void* X,
                                  const int32_t* aux, void* out) {
    if (!st || !out || st->cur_slot < 0) return AMDP_E_INVAL;
    const Dims& d = st->d;
    if (!X && !d.emb) return AMDP_E_INVAL;
    if ((d.lm || d.emb || !d.causal) && !aux) return AMDP_E_INVAL;
    if (st->find_mb(mb) >= 0) return AMDP_E_MB_STATE;
    const int vslot = st->find_version(version);
    if (vslot < 0) return AMDP_E_VERSION;
    int aslot = -1;                     // the free slot that has been free longest
    for (int i = 0; i < st->cfg.act_slots; ++i)
        if (!st->as[i].used && (aslot < 0 || st->free_seq[i] < st->free_seq[aslot])) aslot = i;
    if (aslot < 0) return AMDP_E_NO_SLOT;
    TRY(wait_leaves_of(st, aslot));     // gradient leaves of its previous minibatch may still read it
    int rc = d.bf ? forward_impl<bf16>(st, aslot, vslot, X, aux, out)
                  : forward_impl<float>(st, aslot, vslot, X, aux, out);
    if (rc != AMDP_OK) return rc;
    ASlot& a = st->as[aslot];
    a.used = true; a.mb = mb; a.vslot = vslot; a.backwarded = false;
    st->vs[vslot].pins++;
    return AMDP_OK;
}

extern "C" int amdp_stage_backward(amdp_stage_t* st, int32_t mb, uint32_t version, const void* dY, void* dX) {
    if (!st || st->cur_slot < 0) return AMDP_E_INVAL;
    const Dims& d = st->d;
    if (!d.lm && !dY) return AMDP_E_INVAL;
    const int aslot = st->find_mb(mb);
    if (aslot < 0 || st->as[aslot].backwarded) return AMDP_E_MB_STATE;
    if (st->staged_slot >= 0) return AMDP_E_MB_STATE;
    const int vslot = st->find_version(version);
    if (vslot < 0) return AMDP_E_VERSION;
    // the padding mask was saved with the activations (the fused attention
    // backward recomputes the probabilities and needs it again)
    const int32_t* valid = (!d.causal && !d.lm) ? (const int32_t*)(st->act_ptr(aslot) + st->w.slot.valid) : nullptr;
    TRY(wait_leaves_of(st, st->last_leaves));   // the previous backward's leaves read the scratch this one rewrites
    int rc = d.bf ? backward_impl<bf16>(st, aslot, vslot, valid, dY, dX)
                  : backward_impl<float>(st, aslot, vslot, valid, dY, dX);
    if (rc != AMDP_OK) return rc;
    ASlot& a = st->as[aslot];
    a.backwarded = true;
    st->staged_slot = aslot;
    st->vs[a.vslot].pins--;
    st->drop_unpinned();
    return AMDP_OK;
}

extern "C" int amdp_grad_accumulate(amdp_stage_t* st, int32_t mb) {
    if (!st) return AMDP_E_INVAL;
    const int aslot = st->find_mb(mb);
    if (aslot < 0 || !st->as[aslot].backwarded || st->staged_slot != aslot) return AMDP_E_MB_STATE;
    const long n4 = st->d.n_alloc() / 4;
    if (!st->fused_acc) {
        // HBM-bound and needed by nothing before the next update: it runs on the
        // side stream under whatever the main stream does next (usually the
        // matrix-core-bound forward of another minibatch). The next backward's
        // gradient leaves use the same stream, so they cannot overwrite the
        // staged gradient early; everything else that touches G or g joins first.
        Leaf leaf(st);
        if (!leaf.ok) return AMDP_E_HIP;
        ProfScope ps(st, "grad_accumulate", 0.0, 12.0 * (double)st->d.n_params());
        hipLaunchKernelGGL(accumulate_kernel, dim3(direct_grid(n4, ACC_BLOCK)), dim3(ACC_BLOCK), 0, st->launch,
                           st->at<float>(st->w.G), st->at<float>(st->w.g), n4);
        TRY(after_launch());
    }
    st->as[aslot] = ASlot();
    st->free_seq[aslot] = ++st->free_counter;
    st->staged_slot = -1;
    return AMDP_OK;
}

extern "C" int amdp_apply_update(amdp_stage_t* st, const amdp_adam_t* hp, uint32_t* new_version) {
    if (!st || !hp || hp->struct_size != sizeof(amdp_adam_t) || st->cur_slot < 0) return AMDP_E_INVAL;
    if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0 && hp->beta2 >= 0.0 && hp->beta2 < 1.0)) return AMDP_E_INVAL;
    if (st->staged_slot >= 0) return AMDP_E_MB_STATE;   // a gradient is waiting to be accumulated
    const int slot = st->free_vslot();
    if (slot < 0) return AMDP_E_STASH_FULL;
    TRY(join_leaves(st));                               // accumulations still on the side stream
    AdamScalars sc;
    sc.lr = (float)hp->lr; sc.beta1 = (float)hp->beta1; sc.beta2 = (float)hp->beta2; sc.eps = (float)hp->eps;
    sc.weight_decay = (float)hp->weight_decay; sc.grad_scale = (float)hp->grad_scale;
    sc.omb1 = (float)(1.0 - hp->beta1); sc.omb2 = (float)(1.0 - hp->beta2);
    const uint64_t t = st->step + 1;
    if (hp->bias_correction) {
        sc.inv_bc1 = (float)(1.0 / (1.0 - std::pow(hp->beta1, (double)t)));
        sc.inv_bc2 = (float)(1.0 / (1.0 - std::pow(hp->beta2, (double)t)));
    } else {
        sc.inv_bc1 = sc.inv_bc2 = 1.0f;
    }
    const long n4 = st->d.n_alloc() / 4;
    float* th = st->at<float>(st->w.theta);
    float* m = st->at<float>(st->w.m);
    float* v = st->at<float>(st->w.v);
    float* G = st->at<float>(st->w.G);
    // read theta, m, v, G; write theta, m, v, the new version, and G = 0
    ProfScope ps(st, "adam_update", 0.0, (32.0 + (double)st->d.esz) * (double)st->d.n_params());
    if (st->d.bf)
        hipLaunchKernelGGL(adam_kernel<bf16>, dim3(direct_grid(n4, ACC_BLOCK)), dim3(ACC_BLOCK), 0, st->launch, th, m,
                           v, G, (bf16*)st->version_ptr(slot), n4, sc);
    else
        hipLaunchKernelGGL(adam_kernel<float>, dim3(direct_grid(n4, ACC_BLOCK)), dim3(ACC_BLOCK), 0, st->launch, th,
                           m, v, G, (float*)st->version_ptr(slot), n4, sc);
    TRY(after_launch());
    st->step = t;
    st->cur_version += 1;
    st->vs[slot].valid = true;
    st->vs[slot].version = st->cur_version;
    st->vs[slot].pins = 0;
    st->cur_slot = slot;
    st->drop_unpinned();
    if (new_version) *new_version = st->cur_version;
    return AMDP_OK;
}

extern "C" int amdp_stage_profile_begin(amdp_stage_t* st) {
    if (!st || st->prof.on) return AMDP_E_INVAL;
    st->prof.names.clear();
    st->prof.recs.clear();
    st->prof.on = true;
    return AMDP_OK;
}

extern "C" int amdp_stage_profile_end(amdp_stage_t* st, amdp_profile_entry_t* out, int32_t cap, int32_t* n) {
    if (!st || !n || !st->prof.on) return AMDP_E_INVAL;
    st->prof.on = false;
    // gradient leaves and accumulations carry their events on the side stream:
    // order it before the caller's stream, then wait for both
    int rc = join_leaves(st);
    if (rc == AMDP_OK && !hip_ok(hipStreamSynchronize(st->stream), "hipStreamSynchronize")) rc = AMDP_E_HIP;
    if (rc == AMDP_OK && st->side && !hip_ok(hipStreamSynchronize(st->side), "hipStreamSynchronize(side)")) rc = AMDP_E_HIP;
    std::vector<amdp_profile_entry_t> agg(st->prof.names.size());
    for (size_t i = 0; i < agg.size(); ++i) {
        memset(&agg[i], 0, sizeof(agg[i]));
        snprintf(agg[i].name, sizeof(agg[i].name), "%s", st->prof.names[i].c_str());
    }
    for (ProfRecord& r : st->prof.recs) {
        float ms = 0.f;
        if (rc == AMDP_OK) {
            if (hip_ok(hipEventElapsedTime(&ms, r.start, r.stop), "hipEventElapsedTime")) {
                amdp_profile_entry_t& e = agg[r.name_id];
                e.launches += 1; e.ms += ms; e.flops += r.flops; e.bytes += r.bytes;
            } else {
                rc = AMDP_E_HIP;      // an event that is not complete after both waits: report, do not undercount
            }
        }
        hipEventDestroy(r.start);
        hipEventDestroy(r.stop);
    }
    st->prof.recs.clear();
    *n = (int32_t)agg.size();
    if (rc != AMDP_OK) return rc;
    if (!out || cap < (int32_t)agg.size()) return AMDP_E_CAPACITY;
    for (size_t i = 0; i < agg.size(); ++i) out[i] = agg[i];
    return AMDP_OK;
}

extern "C" const char* amdp_last_hip_error(void) { return g_hip_detail; }

extern "C" int amdp_tie_embedding_grads(amdp_stage_t* first, amdp_stage_t* last) {
    if (!first || !last || !first->d.emb || !last->d.lm || first->d.V != last->d.V || first->d.D != last->d.D)
        return AMDP_E_INVAL;
    if (first->staged_slot >= 0 || last->staged_slot >= 0) return AMDP_E_MB_STATE;
    TRY(join_leaves(first));
    TRY(join_leaves(last));
    const long n4 = (long)first->d.V * first->d.D / 4;
    hipLaunchKernelGGL(tie_sum_kernel, dim3(direct_grid(n4, 64)), dim3(64), 0, first->stream,
                       first->at<float>(first->w.G) + first->d.off_tok(),
                       last->at<float>(last->w.G) + last->d.off_embed(), n4);
    return after_launch();
}

// ---- row operators of the block, callable on their own ---------------------------
namespace {
int device_cu_count() {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        cus = 256;
    return cus;
}
// rows x cols of `dtype`, 16-byte vectors along a row
bool row_op_shape_ok(int32_t rows, int32_t cols, int32_t dtype) {
    if (dtype != AMDP_FP32 && dtype != AMDP_BF16) return false;
    if (rows < 0 || cols < 1) return false;
    return cols % (dtype == AMDP_BF16 ? 8 : 4) == 0;
}
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
constexpr int COLSUM_MAX_CHUNKS = 256;

int column_sums_impl(const void* dy, const void* x, const float* stats, float* out, int32_t rows, int32_t cols,
                     int32_t dtype, float* partial, int max_chunks, hipStream_t s) {
    const bool ln = x != nullptr;
    const ColSumPlan p = plan_column_sums(rows, cols, dtype == AMDP_BF16 ? 8 : 4, device_cu_count(), max_chunks);
    if (dtype == AMDP_BF16)
        return ln ? launch_column_sums<bf16, true>(s, dy, x, stats, partial, out, rows, cols, p, 0)
                  : launch_column_sums<bf16, false>(s, dy, nullptr, nullptr, partial, out, rows, cols, p, 0);
    return ln ? launch_column_sums<float, true>(s, dy, x, stats, partial, out, rows, cols, p, 0)
              : launch_column_sums<float, false>(s, dy, nullptr, nullptr, partial, out, rows, cols, p, 0);
}
}  // namespace

extern "C" int amdp_layernorm_forward(const void* x, const void* gamma, const void* beta, void* y, float* stats,
                                      int32_t rows, int32_t cols, int32_t dtype, float eps, void* hip_stream) {
    if (!row_op_shape_ok(rows, cols, dtype) || !(eps > 0.f)) return AMDP_E_INVAL;
    if (rows == 0) return AMDP_OK;
    if (!x || !gamma || !beta || !y || !stats) return AMDP_E_INVAL;
    if (!aligned16(x) || !aligned16(gamma) || !aligned16(beta) || !aligned16(y) || ((uintptr_t)stats & 3)) return AMDP_E_INVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    return dtype == AMDP_BF16 ? launch_ln_fwd<bf16>(s, x, gamma, beta, y, stats, rows, cols, eps)
                              : launch_ln_fwd<float>(s, x, gamma, beta, y, stats, rows, cols, eps);
}

extern "C" int amdp_layernorm_backward(const void* dy, const void* x, const float* stats, const void* gamma,
                                       const void* res, void* dx, int32_t rows, int32_t cols, int32_t dtype,
                                       void* hip_stream) {
    if (!row_op_shape_ok(rows, cols, dtype)) return AMDP_E_INVAL;
    if (rows == 0) return AMDP_OK;
    if (!dy || !x || !stats || !gamma || !dx) return AMDP_E_INVAL;
    if (!aligned16(dy) || !aligned16(x) || !aligned16(gamma) || !aligned16(res) || !aligned16(dx) || ((uintptr_t)stats & 3))
        return AMDP_E_INVAL;
    hipStream_t s = (hipStream_t)hip_stream;
    return dtype == AMDP_BF16 ? launch_ln_bwd<bf16>(s, dy, x, stats, gamma, res, dx, rows, cols)
                              : launch_ln_bwd<float>(s, dy, x, stats, gamma, res, dx, rows, cols);
}

extern "C" size_t amdp_column_sums_workspace_bytes(int32_t rows, int32_t cols, int32_t dtype, int32_t with_layernorm) {
    if (!row_op_shape_ok(rows, cols, dtype)) return 0;
    // room for the most row chunks any device's plan uses
    return (size_t)COLSUM_MAX_CHUNKS * (size_t)cols * (with_layernorm ? 2 : 1) * sizeof(float);
}

extern "C" int amdp_column_sums(const void* dy, const void* x, const float* stats, float* out, int32_t rows,
                                int32_t cols, int32_t dtype, void* workspace, size_t workspace_bytes,
                                void* hip_stream) {
    if (!row_op_shape_ok(rows, cols, dtype) || !out || !workspace) return AMDP_E_INVAL;
    if (rows > 0 && (!dy || (x && !stats))) return AMDP_E_INVAL;
    if (!aligned16(dy) || !aligned16(x) || ((uintptr_t)stats & 3) || ((uintptr_t)out & 3) || !aligned16(workspace))
        return AMDP_E_INVAL;
    if (workspace_bytes < amdp_column_sums_workspace_bytes(rows, cols, dtype, x != nullptr)) return AMDP_E_INVAL;
    return column_sums_impl(dy, x, stats, out, rows, cols, dtype, (float*)workspace, COLSUM_MAX_CHUNKS,
                            (hipStream_t)hip_stream);
}

// ---- amdp_column_sums for callers that cannot allocate ----------------------------
// The partial sums live in a fixed array in device memory that is part of the
// library's code object: every GPU the library runs on holds its own copy at its
// own address until the process ends. Host code never uses the array's name as an
// address: the per-device address comes from hipGetSymbolAddress, once per device.
namespace {
constexpr size_t COLSUM_STATIC_BYTES = 8u << 20;
constexpr int COLSUM_STATIC_MAX_DEVICES = 64;
}  // namespace
static __device__ __align__(256) unsigned char scratch[COLSUM_STATIC_BYTES];
namespace {
std::atomic<float*> g_scratch_ptr[COLSUM_STATIC_MAX_DEVICES];

// Device address of this device's copy of `scratch` (the current device's).
int static_scratch(float** out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= COLSUM_STATIC_MAX_DEVICES) return AMDP_E_INVAL;
    float* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        void* sym = nullptr;
        HIP_TRY(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
        if (!sym) return AMDP_E_HIP;
        p = (float*)sym;
        g_scratch_ptr[dev].store(p, std::memory_order_release);   // threads that race store the same address
    }
    *out = p;
    return AMDP_OK;
}
}  // namespace

extern "C" size_t amdp_column_sums_static_max_cols(int32_t with_layernorm) {
    // at least one row chunk must fit: width * 4 bytes <= the array
    return COLSUM_STATIC_BYTES / sizeof(float) / (with_layernorm ? 2 : 1);
}

extern "C" int amdp_column_sums_static(const void* dy, const void* x, const float* stats, float* out, int32_t rows,
                                       int32_t cols, int32_t dtype, void* hip_stream) {
    if (!row_op_shape_ok(rows, cols, dtype) || !out) return AMDP_E_INVAL;
    if (rows > 0 && (!dy || (x && !stats))) return AMDP_E_INVAL;
    if (!aligned16(dy) || !aligned16(x) || ((uintptr_t)stats & 3) || ((uintptr_t)out & 3)) return AMDP_E_INVAL;
    const size_t width = (size_t)cols * (x ? 2 : 1);
    if (width * sizeof(float) > COLSUM_STATIC_BYTES) return AMDP_E_TOO_LARGE;
    // as many row chunks as the array has room for (the caller-workspace form takes up to 256)
    const int max_chunks = (int)std::min<size_t>(COLSUM_MAX_CHUNKS, COLSUM_STATIC_BYTES / (width * sizeof(float)));
    float* partial = nullptr;
    TRY(static_scratch(&partial));
    // Nothing in the array has to start at zero: the first stage writes every partial
    // sum the second stage reads (chunks x width floats from the array's start).
    return column_sums_impl(dy, x, stats, out, rows, cols, dtype, partial, max_chunks, (hipStream_t)hip_stream);
}

extern "C" int amdp_device_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
    if (bytes && (!dst || !src)) return AMDP_E_INVAL;
    return device_copy((hipStream_t)hip_stream, dst, src, bytes);
}

extern "C" int amdp_stage_set_option(amdp_stage_t* st, int32_t option, int32_t value) {
    if (!st) return AMDP_E_INVAL;
    switch (option) {
        case AMDP_OPT_GEMM_TILE:
            st->force_tile = value;
            return AMDP_OK;
        case AMDP_OPT_GEMM_TRANSPOSING_READS:
            st->use_tr = value != 0;
            return AMDP_OK;
        case AMDP_OPT_GEMM_DIRECT_TO_LDS:
            if (value < 0 || value > 2) return AMDP_E_INVAL;
            st->use_direct = value;
            return AMDP_OK;
        case AMDP_OPT_LAZY_JOIN:
            TRY(join_leaves(st));
            st->lazy_join = value != 0;
            return AMDP_OK;
        case AMDP_OPT_SPLIT_K_MIN_TOKENS:
            if (value < 64) return AMDP_E_INVAL;
            st->splitk_min_k = value;
            return AMDP_OK;
        case AMDP_OPT_SPLIT_MAIN_MIN_K:
            if (value < 64) return AMDP_E_INVAL;
            st->split_main_min_k = value;
            return AMDP_OK;
        case AMDP_OPT_LEAF_FORKS:
            if (value < 0 || value > 2) return AMDP_E_INVAL;
            st->leaf_forks = value;
            return AMDP_OK;
    }
    return AMDP_E_INVAL;
}

extern "C" int amdp_stage_read_version(amdp_stage_t* st, uint32_t version, void* out) {
    if (!st || !out) return AMDP_E_INVAL;
    const int slot = st->find_version(version);
    if (slot < 0) return AMDP_E_VERSION;
    if ((uintptr_t)out % 4) return AMDP_E_INVAL;
    return device_copy(st->launch, out, st->version_ptr(slot), round_up((size_t)st->d.n_params() * st->d.esz, 4));
}

extern "C" int amdp_stage_set_fused_accumulate(amdp_stage_t* st, int32_t on) {
    if (!st) return AMDP_E_INVAL;
    if (st->staged_slot >= 0) return AMDP_E_MB_STATE;    // between a backward and its accumulate
    st->fused_acc = on != 0;
    return AMDP_OK;
}

extern "C" int amdp_stage_join(amdp_stage_t* st) {
    if (!st) return AMDP_E_INVAL;
    return join_leaves(st);
}

extern "C" int amdp_stage_get_overlap(const amdp_stage_t* st, int32_t* on) {
    if (!st || !on) return AMDP_E_INVAL;
    *on = st->overlap ? 1 : 0;
    return AMDP_OK;
}

extern "C" int amdp_stage_set_overlap(amdp_stage_t* st, int32_t on) {
    if (!st) return AMDP_E_INVAL;
    if (on && !st->side) return AMDP_E_INVAL;   // the stage was created without a side stream
    TRY(join_leaves(st));                       // work still on the side stream stays ordered
    st->overlap = on != 0;
    return AMDP_OK;
}
