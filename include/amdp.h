/*
 * amdp.h -- C ABI of the AMDP pipeline-stage library for AMD MI355X (gfx950).
 *
 * The library implements the work ONE pipeline stage performs on its own GPU
 * under AMDP (Asynchronous Multi-Directional Pipeline parallelism): forward and
 * backward of a contiguous slice of GPT- or BERT-style transformer blocks, each
 * with the weight version the schedule assigns it; accumulation of gradients
 * over a window of minibatches; one fused Adam update per window; and the
 * host-side generator of the stage's event order (paper Sections 3.1-3.3,
 * Lemma 1, Appendix B.1, B.4).
 *
 * Conventions
 *   - Every function returns int: AMDP_OK (0) or a negative AMDP_E_* code. No
 *     exceptions, no aborts, nothing printed. amdp_strerror() names a code.
 *   - "host" pointers are ordinary process memory. "device" pointers are HIP
 *     device memory on the GPU that was current when the stage was created.
 *     All device pointers are owned by the caller and only borrowed for the
 *     duration of the enqueued work.
 *   - The library never allocates device memory. The caller asks
 *     amdp_stage_workspace_bytes(), allocates that many bytes (256-byte
 *     aligned) and hands them to amdp_stage_create(); the workspace must stay
 *     alive and untouched until amdp_stage_destroy().
 *   - All GPU work is enqueued on the HIP stream given at create time and is
 *     ordered by that stream. The library never synchronises; outputs are
 *     valid once the stream reaches them.
 *   - State checks happen before anything is enqueued: a call that returns a
 *     state-machine or argument error (every code but AMDP_E_HIP) has changed
 *     nothing. AMDP_E_HIP means a HIP call or a launch failed part-way: work
 *     enqueued before it stays enqueued and the stage should be reloaded with
 *     amdp_stage_set_state.
 *   - The library reads no environment variables.
 *   - Structs start with `struct_size` = sizeof(the struct) as compiled by the
 *     caller; a mismatch is AMDP_E_INVAL.
 */
#ifndef AMDP_H
#define AMDP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AMDP_OK            0
#define AMDP_E_INVAL      -1  /* bad argument or configuration, null pointer, workspace too small */
#define AMDP_E_MB_STATE   -2  /* minibatch in the wrong state: backward/accumulate without forward,
                                 second forward of a live minibatch, staging buffer still occupied */
#define AMDP_E_NO_SLOT    -3  /* more minibatches in flight than act_slots: the in-flight bound of
                                 the schedule was broken */
#define AMDP_E_VERSION    -4  /* requested weight version is neither current nor stashed */
#define AMDP_E_STASH_FULL -5  /* an update needs a free version slot and every slot is still read
                                 by an in-flight minibatch */
#define AMDP_E_HIP        -6  /* a HIP call or kernel launch failed */
#define AMDP_E_CAPACITY   -7  /* caller's output array is too small; *n_out holds the need */
#define AMDP_E_TOO_LARGE  -8  /* the problem exceeds the fixed capacity of an entry point that allocates
                                 nothing; use the form that takes a caller workspace */

const char* amdp_strerror(int code);
/* Text of the HIP error behind the calling thread's most recent AMDP_E_HIP
 * ("" if none): which call failed and hipGetErrorString of its status. */
const char* amdp_last_hip_error(void);

/* ------------------------------------------------------------------------
 * Schedule generator (host only, integers only, no GPU needed)
 *
 * Emits the ordered events of one logical stage i of a depth-d pipeline whose
 * P concurrent pipelines (Section 3.2) are merged onto it round by round:
 *   - stage i warms up with w = min(n, d-i) forwards per pipeline, n being the
 *     number of minibatches stage 0 may inject before its first backward
 *     (Section 3.1; AMDP fixes n = 2), then alternates backward / forward;
 *   - minibatch m belongs to pipeline m mod P and accumulation window m div T;
 *   - each backward is followed at once by the accumulation of its gradient;
 *   - one update closes each window of T minibatches (Section 3.3). With
 *     AMDP_U_NEXT_BUBBLE it is applied immediately before the first backward of
 *     the next window ("during the next bubble"); with AMDP_U_EAGER right after
 *     the window's last accumulation (the setting of Lemma 1). AMDP_U_FLUSH is
 *     the synchronous comparison schedule of Table 1: each window is a 1F1B
 *     schedule of its own, drained and updated before the next window's first
 *     forward (no mismatch, one live version).
 * Version tags: a forward reads version = number of updates applied before
 * it. A backward reads its forward's version (AMDP_BWD_STASHED) or the
 * version current when it runs (AMDP_BWD_CURRENT; current - forward's tag is
 * the parameter mismatch of Section 3.1). An update event carries the version
 * it produces. Event count is 3*M + ceil(M/T).
 * ------------------------------------------------------------------------ */

enum { AMDP_EV_F = 0, AMDP_EV_B = 1, AMDP_EV_A = 2, AMDP_EV_U = 3 };
enum { AMDP_U_NEXT_BUBBLE = 0, AMDP_U_EAGER = 1, AMDP_U_FLUSH = 2 };
enum { AMDP_BWD_STASHED = 0, AMDP_BWD_CURRENT = 1 };

#define AMDP_FLAG_LAST_USE       1u  /* F/B: no later event reads this version */
#define AMDP_FLAG_PARTIAL_WINDOW 2u  /* U: the window it closes holds fewer than T minibatches */

typedef struct amdp_event_t {
    uint8_t  kind;      /* AMDP_EV_* */
    uint8_t  pipeline;  /* m mod P for F/B/A, 0 for U */
    uint16_t flags;     /* AMDP_FLAG_* */
    int32_t  mb;        /* F/B/A: global minibatch id; U: window index */
    uint32_t version;   /* F/B: version read; A: 0; U: version produced */
} amdp_event_t;

typedef struct amdp_sched_params_t {
    uint32_t struct_size;
    int32_t depth;            /* d >= 1 */
    int32_t pipelines;        /* P >= 1 (at most 256) */
    int32_t stage;            /* i in [0, d) */
    int32_t inject_limit;     /* n >= 1; AMDP uses 2 */
    int32_t threshold;        /* T >= 1, minibatches per update */
    int32_t n_minibatches;    /* M >= 0 */
    int32_t update_placement; /* AMDP_U_* */
    int32_t bwd_version;      /* AMDP_BWD_* */
} amdp_sched_params_t;

/* Writes up to `cap` events to `out` (host). *n_out (host) receives the number
 * of events the schedule has; if it exceeds cap nothing is written and
 * AMDP_E_CAPACITY is returned (call with out = NULL, cap = 0 to size). */
int amdp_schedule_generate(const amdp_sched_params_t* params, amdp_event_t* out, size_t cap,
                           size_t* n_out);

/* Generator settings of the schedules Table 1 compares, for one stage of one
 * pipeline (AMDP: of d/2 merged pipelines), so that the same stage library and
 * amdp_schedule_stats can show their mismatch and weight-version counts:
 *   AMDP           n = 2, P = d/2, update in the next bubble, current weights in
 *                  backward (mismatch <= 1, one version, Lemma 1)
 *   PIPEDREAM      n = d, an update after every minibatch, stashed weights
 *                  (d - i versions live at stage i, no mismatch in backward)
 *   PIPEDREAM_2BW  n = d, gradients coalesced over >= d minibatches, stashed
 *                  weights (two versions live)
 *   SYNC_1F1B      minibatches of `microbatches` microbatches, flushed
 * `microbatches`: window length T (0 = the preset's default: 2d for AMDP, d for
 * 2BW; required for SYNC_1F1B). Fills *out; host only. */
enum { AMDP_PRESET_AMDP = 0, AMDP_PRESET_PIPEDREAM = 1, AMDP_PRESET_PIPEDREAM_2BW = 2, AMDP_PRESET_SYNC_1F1B = 3 };
int amdp_schedule_preset(int32_t preset, int32_t depth, int32_t stage, int32_t n_minibatches,
                         int32_t microbatches, amdp_sched_params_t* out);

typedef struct amdp_sched_stats_t {
    uint32_t struct_size;
    int32_t max_inflight;               /* forwards not yet backwarded, all pipelines */
    int32_t max_inflight_per_pipeline;
    int32_t max_mismatch;               /* updates between F(m) and B(m), Section 3.1 */
    int32_t max_affected_per_window;    /* minibatches of one window with mismatch > 0 */
    int32_t max_live_versions;          /* current + older versions still to be read */
} amdp_sched_stats_t;

/* Bounds of an event list (host arrays). `threshold` groups minibatches into
 * windows for max_affected_per_window. AMDP_E_INVAL on a malformed list
 * (backward before forward, unknown kind). */
int amdp_schedule_stats(const amdp_event_t* events, size_t n, int32_t threshold,
                        amdp_sched_stats_t* out);

/* Chimera-style placement of Section 3.2: stage i of pipeline j runs on GPU
 * (2j+i) mod d for even j and (2j-i+d+1) mod d for odd j. Host only. */
int amdp_stage_map(int32_t depth, int32_t pipeline, int32_t stage, int32_t* gpu_out);

/* ------------------------------------------------------------------------
 * Timed simulation of the whole multi-directional system (Section 3.2): d GPUs,
 * P <= d/2 pipelines placed by amdp_stage_map, each running `minibatches`
 * minibatches; stage 0 of a pipeline keeps at most inject_limit + preload
 * minibatches in flight; forward(i,m) precedes forward(i+1,m) and
 * backward(i,m), backward(i,m) precedes backward(i-1,m) (Appendix B.4). A GPU
 * runs one operation at a time without preemption and, when free, starts the
 * ready operation that became ready first (the FIFO rule of Section 3.2); ties
 * go to a backward before a forward, then the lower pipeline, then the lower
 * minibatch. Time is in integer units: every forward takes t_forward, every
 * backward t_backward, transfers take none. Host only, integer only.
 * The paper's statements this reproduces: one pipeline keeps a GPU busy n/d of
 * the time; with P = d/2 and preload = floor(t_backward / t_forward) the
 * bubbles all but vanish.
 * ------------------------------------------------------------------------ */
typedef struct amdp_sim_params_t {
    uint32_t struct_size;
    int32_t depth;          /* d >= 1: stages per pipeline = number of GPUs */
    int32_t pipelines;      /* 1 <= P <= max(1, d/2) */
    int32_t inject_limit;   /* n >= 1 */
    int32_t preload;        /* extra minibatches stage 0 may have in flight, >= 0 */
    int32_t minibatches;    /* per pipeline, >= 0 */
    int32_t t_forward;      /* >= 1 */
    int32_t t_backward;     /* >= 1 */
} amdp_sim_params_t;

typedef struct amdp_sim_op_t {
    uint8_t  kind;       /* AMDP_EV_F or AMDP_EV_B */
    uint8_t  pipeline;
    uint16_t stage;
    int32_t  mb;         /* minibatch index inside its pipeline */
    int32_t  gpu;
    int64_t  start, end;
} amdp_sim_op_t;

typedef struct amdp_sim_result_t {
    uint32_t struct_size;
    int32_t  max_inflight;   /* most minibatches one pipeline had in flight at stage 0 */
    int64_t  makespan;       /* end of the last operation */
    int64_t  busy_total;     /* sum over GPUs of the time spent in operations */
    int64_t  busy_min, busy_max;   /* over GPUs */
} amdp_sim_result_t;

/* Writes the 2*d*P*minibatches operations in order of start time (ties: lower
 * GPU first) to `ops` (host; may be NULL with cap = 0 to size: *n_ops is always
 * set, AMDP_E_CAPACITY if cap is too small, in which case only `result` is
 * filled). gpu_busy (host, [depth], may be NULL) receives each GPU's busy time. */
int amdp_system_simulate(const amdp_sim_params_t* params, amdp_sim_op_t* ops, size_t cap, size_t* n_ops,
                         int64_t* gpu_busy, amdp_sim_result_t* result);

/* ------------------------------------------------------------------------
 * Stage
 * ------------------------------------------------------------------------ */

enum { AMDP_BLOCK_GPT_PRELN_CAUSAL = 0, AMDP_BLOCK_BERT_POSTLN_BIDIR = 1 };
enum { AMDP_FP32 = 0, AMDP_BF16 = 1 };
/* AMDP_ATTN_AUTO: the fused attention kernels (scores never reach HBM, one fp32
 * log-sum-exp per query kept for backward) wherever the shape allows: bf16,
 * seq_len a multiple of 128, even head dimension <= 128; the three-kernel form
 * elsewhere. AMDP_ATTN_UNFUSED: always scores GEMM, masked softmax, P V GEMM with
 * the probabilities [b*H, s, s] kept in the activation slot. */
enum { AMDP_ATTN_AUTO = 0, AMDP_ATTN_UNFUSED = 1 };

typedef struct amdp_stage_config_t {
    uint32_t struct_size;
    int32_t block_kind;   /* AMDP_BLOCK_* */
    int32_t n_layers;     /* L >= 1 */
    int32_t d_model;      /* D, multiple of n_heads */
    int32_t n_heads;      /* H */
    int32_t d_ffn;        /* F */
    int32_t seq_len;      /* s */
    int32_t microbatch;   /* b sequences per minibatch; tokens N = b*s */
    int32_t dtype;        /* AMDP_FP32: activations and weight versions in fp32;
                             AMDP_BF16: both in bfloat16, fp32 accumulation, statistics, master */
    int32_t has_lm_head;  /* final LayerNorm + tied vocabulary projection + cross-entropy */
    int32_t vocab;        /* V when has_lm_head */
    float   ln_eps;
    int32_t act_slots;    /* minibatches that may be in flight (>= w*P) */
    int32_t stash_slots;  /* weight versions kept besides the current one (>= 1) */
    int32_t has_embedding; /* first stage: the block input is E[token] + P[position] (token and learned
                              position embedding, V = vocab rows and s rows of D); excludes has_lm_head;
                              d_model <= 8192 */
    int32_t attention;     /* AMDP_ATTN_*; fixes the workspace layout together with the other fields */
} amdp_stage_config_t;

typedef struct amdp_stage amdp_stage_t;

/* Parameters live in one flat vector. Per layer, in order: ln1 gamma, beta [D];
 * W_qkv [D,3D] (columns Q|K|V, each split into H heads of D/H), b_qkv [3D];
 * W_o [D,D], b_o [D]; ln2 gamma, beta [D]; W_1 [D,F], b_1 [F]; W_2 [F,D], b_2 [D]
 * -- 12D^2+13D per layer when F = 4D, the count behind Table 2. With an LM head:
 * then final gamma, beta [D] and the tied embedding E [V,D]. With an input
 * embedding: in front of the layers, the token embedding [V,D] and the position
 * embedding [s,D]. Matrices are
 * row-major [in, out]; y = x W + b. */
typedef struct amdp_param_desc_t {
    char     name[24];   /* e.g. "l0.w_qkv", "lnf_gamma", "embed" */
    uint64_t offset;     /* elements from the start of the flat vector */
    uint32_t rows, cols; /* vectors have rows = 1 */
} amdp_param_desc_t;

/* 0 if the configuration is invalid. Host only. */
size_t amdp_stage_n_params(const amdp_stage_config_t* cfg);
size_t amdp_stage_workspace_bytes(const amdp_stage_config_t* cfg);

/* Describes the flat layout (host). AMDP_E_CAPACITY if cap is too small, with
 * *n holding the number of entries. */
int amdp_stage_param_layout(const amdp_stage_config_t* cfg, amdp_param_desc_t* descs, int32_t cap,
                            int32_t* n);

/* workspace: device, >= amdp_stage_workspace_bytes(cfg), 256-byte aligned.
 * hip_stream: a hipStream_t (NULL = the null stream). The stage starts with
 * all state zero and no published version: call amdp_stage_set_state next. */
int amdp_stage_create(const amdp_stage_config_t* cfg, void* workspace, size_t workspace_bytes,
                      void* hip_stream, amdp_stage_t** out);
int amdp_stage_destroy(amdp_stage_t* stage);

/* Loads master parameters and Adam moments (device, fp32, n_params each; m and
 * v may be NULL = zeros), sets the step counter and the current version number,
 * publishes that version in the stage's number type (round to nearest even for
 * bf16), clears the gradient sum, the stash and all in-flight minibatches. */
int amdp_stage_set_state(amdp_stage_t* stage, const float* theta, const float* m, const float* v,
                         uint64_t step, uint32_t version);

/* Copies state out. theta, m, v, G: device fp32 [n_params], each may be NULL.
 * step, version: host, may be NULL. Copies are enqueued on the stage's stream. */
int amdp_stage_get_state(amdp_stage_t* stage, float* theta, float* m, float* v, float* G,
                         uint64_t* step, uint32_t* version);

/* Copies the staged gradient of the last backward (device fp32 [n_params]);
 * AMDP_E_MB_STATE when nothing is staged. */
int amdp_stage_get_staged_grad(amdp_stage_t* stage, float* g);

/* Number of resident versions and their numbers (host; versions may be NULL). */
int amdp_stage_resident_versions(amdp_stage_t* stage, uint32_t* versions, int32_t cap, int32_t* n);

/* Forward of minibatch `mb` with weight version `version` (Section 3.1: the
 * version is whatever the schedule assigns; it must be resident).
 *   X    device [N, D] token-major (row = sequence*s + position), stage dtype;
 *        ignored (may be NULL) on a stage with an input embedding
 *   aux  device int32: on a stage with an input embedding the token ids [N]
 *        (ids outside [0, V) are clamped), followed by valid_len[b] for the BERT
 *        block; otherwise valid_len[b] for the BERT block (keys at positions >=
 *        valid_len are masked; each entry in [1, s] -- a sequence with no
 *        visible key has no softmax and the library does not check device
 *        data), targets[N] in [0, V) on an LM-head stage, else NULL
 *   out  device: Y [N, D] in the stage dtype, or one fp32 (the mean
 *        cross-entropy) on an LM-head stage
 * Saves the activations backward needs in a free activation slot and pins
 * `version` until the minibatch's backward. */
int amdp_stage_forward(amdp_stage_t* stage, int32_t mb, uint32_t version, const void* X,
                       const int32_t* aux, void* out);

/* Backward of minibatch `mb`. Activations are the ones its forward saved; every
 * parameter value that enters (transposed weights, LayerNorm gains, the tied
 * embedding) is read from `version`, which may differ from the forward's.
 *   dY  device [N, D] stage dtype; NULL on an LM-head stage (seed d loss = 1)
 *   dX  device [N, D] stage dtype; may be NULL (not written)
 * Writes the minibatch's parameter gradient (fp32, flat layout) to the staging
 * buffer; it stays there until amdp_grad_accumulate(mb). Unpins the forward's
 * version. */
int amdp_stage_backward(amdp_stage_t* stage, int32_t mb, uint32_t version, const void* dY, void* dX);

/* G <- G + g_mb over the flat buffer (Section 3.3); frees the staging buffer
 * and the minibatch's activation slot. With the side stream on (see
 * amdp_stage_set_overlap) the addition runs there, under whatever the caller's
 * stream does next; every later call that reads or writes G or the staging
 * buffer (backward, apply_update, get_state, get_staged_grad, set_state) is
 * ordered after it by the library. */
int amdp_grad_accumulate(amdp_stage_t* stage, int32_t mb);

typedef struct amdp_adam_t {
    uint32_t struct_size;
    int32_t bias_correction; /* 1: divide moments by (1 - beta^t); 0: the form printed in Appendix B.1 */
    /* Hyper-parameters are doubles so that derived constants (1 - beta, the
     * bias corrections) are formed exactly on the host and rounded to fp32
     * once; the kernel's arithmetic is fp32. */
    double lr, beta1, beta2, eps;
    double weight_decay;     /* decoupled (AdamW); 0 in all benchmark configurations */
    double grad_scale;       /* the update consumes grad_scale * G, e.g. 1/T */
} amdp_adam_t;

/* One Adam step over the flat fp32 master parameters with the accumulated
 * gradient (Section 3.3, Appendix B.1): m, v, theta updated in place, the new
 * version (current + 1) published into a free version slot in the stage dtype,
 * G cleared. *new_version (host, may be NULL) receives its number. Older
 * versions stay resident while an in-flight minibatch's forward has read them. */
int amdp_apply_update(amdp_stage_t* stage, const amdp_adam_t* hp, uint32_t* new_version);

/* Backward enqueues the parameter-gradient work (dW GEMMs, bias and LayerNorm
 * column sums), which is off the dX critical path, on a side stream the stage
 * owns; amdp_grad_accumulate uses the same side stream. The caller still sees
 * one stream: dX is complete in stream order when backward returns, dY (and a
 * dX the input layer's gradient reads) may be overwritten in stream order at
 * once, and every call that reads or changes what the side stream writes
 * (amdp_stage_get_staged_grad, amdp_stage_get_state, amdp_stage_set_state,
 * amdp_apply_update, amdp_tie_embedding_grads, amdp_stage_join) first makes the
 * caller's stream wait for it. What keeps running beside the caller's next
 * calls reads only the stage's workspace: the next backward waits for it
 * before reusing the scratch it reads, and so does the forward that reuses
 * its activation slot.
 * on = 0 keeps everything on the caller's stream (used to time kernels in
 * isolation). Default: on while (d_model / 256)^2 is below the number of compute
 * units, off beyond (every product of the backward then fills the GPU on its
 * own and concurrency measured no gain). Results are bit-identical either way. */
int amdp_stage_set_overlap(amdp_stage_t* stage, int32_t on);
/* *on (host) <- 1 when the side stream is in use, else 0. */
int amdp_stage_get_overlap(const amdp_stage_t* stage, int32_t* on);

/* Copies the published weights of resident version `version` (Section 3.1: the
 * version a forward or backward is assigned; Section 3.4: what the owner of a
 * stage's parameters sends to its replicas after an update) to `out`: device,
 * n_params elements of the stage dtype in the flat layout, room rounded up to a
 * multiple of 4 bytes. AMDP_E_VERSION if it is not resident. Enqueued on the
 * stage's stream. */
int amdp_stage_read_version(amdp_stage_t* stage, uint32_t version, void* out);

/* ------------------------------------------------------------------------
 * Row operators of the transformer block (Section 4.1, Table 2: GPT- and
 * BERT-style layers, each with two LayerNorms and a bias on every linear map),
 * callable on their own on caller-owned device buffers. They are the kernels the
 * stage itself launches; they exist as entry points so that each can be checked
 * and timed in isolation. Matrices are row-major [rows, cols] in `dtype`
 * (AMDP_FP32 / AMDP_BF16), 16-byte aligned, cols a multiple of 4 (fp32) or 8
 * (bf16); rows may be 0. All work is enqueued on `hip_stream`; nothing
 * synchronises. AMDP_E_INVAL on a bad shape, type, alignment or null pointer.
 * ------------------------------------------------------------------------ */

/* y = (x - mean) * rstd * gamma + beta per row, biased variance, rstd =
 * 1/sqrt(var + eps), statistics in fp32; stats[2r] = mean, stats[2r+1] = rstd
 * (device fp32 [rows, 2]) are what the backward operators take. gamma, beta:
 * device [cols] in `dtype`. */
int amdp_layernorm_forward(const void* x, const void* gamma, const void* beta, void* y, float* stats,
                           int32_t rows, int32_t cols, int32_t dtype, float eps, void* hip_stream);

/* dx = (res +) rstd * (g - mean_row(g) - xhat * mean_row(g * xhat)) with g = dy *
 * gamma and xhat = (x - mean) * rstd from `stats`; res (may be NULL) is a
 * residual-branch gradient added in the same pass. dx may alias dy or res. */
int amdp_layernorm_backward(const void* dy, const void* x, const float* stats, const void* gamma,
                            const void* res, void* dx, int32_t rows, int32_t cols, int32_t dtype,
                            void* hip_stream);

/* Parameter gradients that are column sums over the tokens, in fp32, in two
 * deterministic stages (no float atomics: bit-identical run to run):
 *   x == NULL: out[c] = sum_r dy[r][c], c < cols             (bias gradient)
 *   x != NULL: out[c] = sum_r dy[r][c] * xhat[r][c]          (LayerNorm gain)
 *              out[cols + c] = sum_r dy[r][c]                (LayerNorm bias)
 *              with xhat from x and `stats` as above
 * out: device fp32 [cols] or [2*cols]. workspace: device, 16-byte aligned, at
 * least amdp_column_sums_workspace_bytes(...) bytes (0 = invalid arguments); it
 * holds the first stage's partial sums and needs no initialisation. */
size_t amdp_column_sums_workspace_bytes(int32_t rows, int32_t cols, int32_t dtype, int32_t with_layernorm);
int amdp_column_sums(const void* dy, const void* x, const float* stats, float* out, int32_t rows,
                     int32_t cols, int32_t dtype, void* workspace, size_t workspace_bytes, void* hip_stream);

/* amdp_column_sums for callers that cannot allocate device memory or hand over
 * a workspace: code under HIP-graph capture, tight serving loops, harnesses that
 * forbid hipMalloc. Same arguments, results bit-identical to amdp_column_sums
 * whenever both use the same number of row chunks (width <= 8192 floats, see
 * below) and equal to the exact sums within fp32 summation error always. The
 * partial sums go to a fixed 8 MiB array in device memory that belongs to the
 * library's code object (each GPU the library runs on holds its own copy until
 * the process ends); the call makes no hipMalloc / hipFree and calls no
 * allocating routine. Limit: width = cols (2*cols with x) must satisfy width * 4
 * bytes <= 8 MiB, i.e. cols <= amdp_column_sums_static_max_cols(with_layernorm)
 * (2097152, or 1048576 with x); beyond it AMDP_E_TOO_LARGE and nothing is
 * enqueued. Up to min(256, 8 MiB / (4 * width)) row chunks are used, so wide
 * problems run with fewer chunks than the workspace form would take.
 * Every call on a GPU shares that GPU's array: calls that may overlap on one GPU
 * (different streams, different threads) race on it and must be serialised by
 * the caller; calls on one stream are ordered by the stream. Nothing in the
 * array needs clearing between calls (the first stage writes everything the
 * second reads). The first call on each device looks up the array's address
 * (hipGetSymbolAddress) and must therefore happen outside a graph capture. */
size_t amdp_column_sums_static_max_cols(int32_t with_layernorm);
int amdp_column_sums_static(const void* dy, const void* x, const float* stats, float* out, int32_t rows,
                            int32_t cols, int32_t dtype, void* hip_stream);

/* dst <- src, `bytes` bytes of device memory (both 4-byte aligned, bytes a
 * multiple of 4; AMDP_E_INVAL otherwise), by the library's own streaming copy
 * kernel on `hip_stream`. It is what the stage uses for every copy it makes
 * (inputs into activation slots, state in and out), offered to callers that
 * record their work in a HIP graph and want no memcpy nodes in it, and to
 * measurements as the plain copy whose rate is the achievable HBM ceiling. */
int amdp_device_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* Kernel-selection switches for tests and measurements; none changes what is
 * computed beyond rounding order inside a product. Takes effect from the next
 * call on.
 *   AMDP_OPT_GEMM_TILE               0 = the library's choice (default); 256, 128, 64 or
 *                                    BM*1000+BN (128064, 64128) force that matrix-core tile
 *                                    where it divides the product's shape; -1 = generic kernel
 *   AMDP_OPT_GEMM_TRANSPOSING_READS  1 (default) m/n-contiguous operands are read from LDS with
 *                                    the transposing read; 0 element by element
 *   AMDP_OPT_GEMM_DIRECT_TO_LDS      tiles loaded from global memory straight into LDS: 1 (default)
 *                                    where measured faster, 0 never, 2 wherever the shape allows
 *   AMDP_OPT_LAZY_JOIN               1 (default) a backward leaves its gradient leaves running on the
 *                                    side stream; 0 it ends by joining them
 *   AMDP_OPT_SPLIT_K_MIN_TOKENS      a weight-gradient product too small to give every compute unit a
 *                                    128x128 tile is split over its tokens into up to eight parts that
 *                                    are added in fixed order; a part contracts at least this many
 *                                    tokens (default 512, at least 64; a large value switches it off)
 *   AMDP_OPT_SPLIT_MAIN_MIN_K        a [tokens, d_model] product of the forward / dX chain whose 256x256
 *                                    tiles cover at most half of the compute units runs with its
 *                                    contraction split in two halves, added in order by a second
 *                                    kernel together with bias and residual, when a half is at least
 *                                    this long (default 3072, at least 64; a large value switches it off)
 *   AMDP_OPT_LEAF_FORKS              with the side stream on, how often per layer a backward hands its
 *                                    parameter-gradient work to the side stream: 0 once per product
 *                                    (default below d_model 2048: every product starts as early as it
 *                                    can), 2 after the MLP half and at the end of the layer (default
 *                                    from d_model 2048 on), 1 at the end of the layer only. Each
 *                                    hand-over costs the host two event calls and a change of the
 *                                    stream it enqueues on, about 20 us; results are bit-identical */
enum { AMDP_OPT_GEMM_TILE = 0, AMDP_OPT_GEMM_TRANSPOSING_READS = 1, AMDP_OPT_GEMM_DIRECT_TO_LDS = 2,
       AMDP_OPT_LAZY_JOIN = 3, AMDP_OPT_SPLIT_K_MIN_TOKENS = 4, AMDP_OPT_SPLIT_MAIN_MIN_K = 5,
       AMDP_OPT_LEAF_FORKS = 6 };
int amdp_stage_set_option(amdp_stage_t* stage, int32_t option, int32_t value);

/* The input embedding of the first stage and the output projection of the last
 * are one tied parameter held twice; before the update their gradient sums must
 * be added. first: a stage with has_embedding, last: a stage with has_lm_head,
 * same vocab and d_model. Afterwards both hold the sum in their G (token
 * embedding rows resp. tied embedding rows), so both updates move their copy
 * alike. On one GPU this is a local two-buffer sum; across GPUs it would be the
 * one transfer the tie costs per update. Both stages' pending work is joined;
 * the sum runs on `first`'s stream, which the caller must have ordered after
 * `last`'s stream (the same stream is the simple case). */
int amdp_tie_embedding_grads(amdp_stage_t* first, amdp_stage_t* last);

/* on = 1: backward adds the minibatch's parameter gradients straight into the
 * sum G (the dW products and the column sums end in G += instead of g =), and
 * amdp_grad_accumulate only does its bookkeeping. The sum is bit-identical to
 * the two-step form (same fp32 additions in the same order) and 12 bytes per
 * parameter per minibatch of HBM traffic disappear; the price is that the
 * minibatch's own gradient is never materialised (amdp_stage_get_staged_grad
 * returns AMDP_E_MB_STATE). Default 0: the accumulation is its own kernel, as
 * the schedule's A event has it. AMDP_E_MB_STATE between a backward and its
 * accumulate. */
int amdp_stage_set_fused_accumulate(amdp_stage_t* stage, int32_t on);

/* Orders everything the stage has enqueued on its own side stream (gradient
 * leaves of the last backward, accumulations) before whatever the caller enqueues next
 * on its stream. Needed only by a caller that wants a point where the stage's
 * stream alone carries all of its work: before ending a HIP-graph capture that
 * contains amdp_stage_backward or amdp_grad_accumulate, or before reusing the workspace for something
 * else. Enqueues an event wait; does not block the host. */
int amdp_stage_join(amdp_stage_t* stage);

/* ------------------------------------------------------------------------
 * Measurement aid: per-kernel-class device time from HIP events recorded on
 * the stage's stream around every launch between begin and end. `flops` and
 * `bytes` are the ALGORITHMIC work of the launches (2MNK per GEMM; fused
 * attention forward 2 products, backward 4 (dV, dP, dK in one kernel, dQ in the
 * other), recomputed scores not counted, only visible query/key pairs under the
 * causal mask; 12 bytes per parameter for the accumulation, 32 + sizeof(stage
 * dtype) per parameter for the update).
 * Profiling inserts events into the streams: do not time throughput while on.
 * amdp_stage_profile_end joins the stage's side stream and synchronises both
 * streams; an event that still cannot be read is AMDP_E_HIP, never a silently
 * shorter record.
 * ------------------------------------------------------------------------ */
typedef struct amdp_profile_entry_t {
    char     name[48];
    uint64_t launches;
    double   ms;      /* summed event-to-event time of those launches */
    double   flops;
    double   bytes;
} amdp_profile_entry_t;

int amdp_stage_profile_begin(amdp_stage_t* stage);
/* out: host array; AMDP_E_CAPACITY (with *n set) if cap is too small -- the
 * recorded data is discarded either way. */
int amdp_stage_profile_end(amdp_stage_t* stage, amdp_profile_entry_t* out, int32_t cap, int32_t* n);

#ifdef __cplusplus
}
#endif
#endif /* AMDP_H */
