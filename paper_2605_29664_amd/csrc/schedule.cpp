// Host-side AMDP schedule generator: the ordered forward / backward /
// accumulate / update events of one logical pipeline stage and the weight
// version each one reads (paper Sections 3.1-3.3; Lemma 1; Appendix B.4).
// Integer work only; no GPU involved.
#include "amdp.h"

#include <algorithm>
#include <cstring>
#include <map>
#include <queue>
#include <vector>

namespace {

inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace

extern "C" int amdp_schedule_generate(const amdp_sched_params_t* p, amdp_event_t* out, size_t cap,
                                      size_t* n_out) {
    if (!p || !n_out || p->struct_size != sizeof(amdp_sched_params_t)) return AMDP_E_INVAL;
    const int d = p->depth, P = p->pipelines, i = p->stage, n = p->inject_limit;
    const int T = p->threshold, M = p->n_minibatches;
    if (d < 1 || P < 1 || P > 256 || i < 0 || i >= d || n < 1 || T < 1 || M < 0) return AMDP_E_INVAL;
    if (p->update_placement != AMDP_U_NEXT_BUBBLE && p->update_placement != AMDP_U_EAGER &&
        p->update_placement != AMDP_U_FLUSH)
        return AMDP_E_INVAL;
    if (p->bwd_version != AMDP_BWD_STASHED && p->bwd_version != AMDP_BWD_CURRENT) return AMDP_E_INVAL;

    const int n_updates = M ? ceil_div(M, T) : 0;
    const size_t total = 3 * (size_t)M + (size_t)n_updates;
    *n_out = total;
    if (total > cap || (!out && total)) return AMDP_E_CAPACITY;
    if (!total) return AMDP_OK;

    const int w = std::min(n, d - i);          // warm-up forwards per pipeline (Section 3.1)
    const bool flush = p->update_placement == AMDP_U_FLUSH;
    const bool eager = p->update_placement == AMDP_U_EAGER || flush;
    const bool stashed = p->bwd_version == AMDP_BWD_STASHED;

    std::vector<uint32_t> fwd_tag((size_t)M, 0);
    uint32_t applied = 0;   // updates emitted so far = current version
    size_t k = 0;

    auto emit = [&](uint8_t kind, int pipe, uint16_t flags, int32_t mb, uint32_t ver) {
        out[k].kind = kind;
        out[k].pipeline = (uint8_t)pipe;
        out[k].flags = flags;
        out[k].mb = mb;
        out[k].version = ver;
        ++k;
    };
    auto emit_update = [&](int window) {
        ++applied;
        const bool partial = (long long)(window + 1) * T > M;
        emit(AMDP_EV_U, 0, partial ? AMDP_FLAG_PARTIAL_WINDOW : 0, window, applied);
    };
    // 1F1B per replica over minibatches [first, last): w forward rounds, then
    // backward round g / forward round g + w.
    auto one_f_one_b = [&](int first, int last) {
        const int rounds = ceil_div(last - first, P);
        auto forward_round = [&](int g) {
            for (int m = first + g * P; m < std::min(first + (g + 1) * P, last); ++m) {
                fwd_tag[m] = applied;
                emit(AMDP_EV_F, m % P, 0, m, applied);
            }
        };
        auto backward_round = [&](int g) {
            for (int m = first + g * P; m < std::min(first + (g + 1) * P, last); ++m) {
                // "next bubble": the update of the window that just closed goes in
                // front of the first backward of the following window
                if (!eager && m > 0 && m % T == 0) emit_update(m / T - 1);
                emit(AMDP_EV_B, m % P, 0, m, stashed ? fwd_tag[m] : applied);
                emit(AMDP_EV_A, m % P, 0, m, 0);
                if (eager && ((m + 1) % T == 0 || (flush && m == M - 1))) emit_update(m / T);
            }
        };
        for (int g = 0; g < std::min(w, rounds); ++g) forward_round(g);
        for (int g = 0; g < rounds; ++g) {
            backward_round(g);
            if (g + w < rounds) forward_round(g + w);
        }
    };
    if (flush) {
        // synchronous schedule: drain a window and apply its update before the
        // next window's first forward
        for (int first = 0; first < M; first += T) one_f_one_b(first, std::min(first + T, M));
    } else {
        one_f_one_b(0, M);
    }
    while ((int)applied < n_updates) emit_update((int)applied);   // closes the last window

    // last reader of each version
    std::vector<char> seen((size_t)applied + 1, 0);
    for (size_t j = k; j-- > 0;) {
        amdp_event_t& e = out[j];
        if ((e.kind == AMDP_EV_F || e.kind == AMDP_EV_B) && !seen[e.version]) {
            seen[e.version] = 1;
            e.flags |= AMDP_FLAG_LAST_USE;
        }
    }
    return k == total ? AMDP_OK : AMDP_E_INVAL;
}

extern "C" int amdp_schedule_stats(const amdp_event_t* ev, size_t n, int32_t threshold,
                                   amdp_sched_stats_t* out) {
    if ((!ev && n) || !out || out->struct_size != sizeof(amdp_sched_stats_t)) return AMDP_E_INVAL;
    int inflight = 0, max_inflight = 0, max_pp = 0, max_mismatch = 0;
    int per_pipe[256] = {0};
    std::map<int32_t, uint32_t> updates_at_forward;   // in-flight minibatch -> updates seen at F
    std::map<int32_t, int> affected;                   // window -> mismatched minibatches
    uint32_t applied = 0;

    // readers still to come, per version, for the residency count
    std::map<uint32_t, size_t> readers;
    for (size_t j = 0; j < n; ++j)
        if (ev[j].kind == AMDP_EV_F || ev[j].kind == AMDP_EV_B) ++readers[ev[j].version];
    int max_live = 1;

    for (size_t j = 0; j < n; ++j) {
        const amdp_event_t& e = ev[j];
        switch (e.kind) {
            case AMDP_EV_F:
                if (updates_at_forward.count(e.mb)) return AMDP_E_INVAL;
                updates_at_forward[e.mb] = applied;
                ++inflight;
                max_pp = std::max(max_pp, ++per_pipe[e.pipeline]);
                break;
            case AMDP_EV_B: {
                auto it = updates_at_forward.find(e.mb);
                if (it == updates_at_forward.end()) return AMDP_E_INVAL;
                const int mm = (int)(applied - it->second);
                max_mismatch = std::max(max_mismatch, mm);
                if (mm > 0 && threshold > 0) ++affected[e.mb / threshold];
                updates_at_forward.erase(it);
                --inflight;
                --per_pipe[e.pipeline];
                break;
            }
            case AMDP_EV_A:
                break;
            case AMDP_EV_U:
                ++applied;
                break;
            default:
                return AMDP_E_INVAL;
        }
        max_inflight = std::max(max_inflight, inflight);
        // versions resident while this event runs: the current one and every
        // already-published one with a reader at or after this event
        int live = 1;
        for (auto& r : readers)
            if (r.second > 0 && r.first < applied) ++live;
        max_live = std::max(max_live, live);
        if (e.kind == AMDP_EV_F || e.kind == AMDP_EV_B) --readers[e.version];
    }
    int max_aff = 0;
    for (auto& a : affected) max_aff = std::max(max_aff, a.second);
    out->max_inflight = max_inflight;
    out->max_inflight_per_pipeline = max_pp;
    out->max_mismatch = max_mismatch;
    out->max_affected_per_window = max_aff;
    out->max_live_versions = max_live;
    return AMDP_OK;
}

extern "C" int amdp_stage_map(int32_t depth, int32_t pipeline, int32_t stage, int32_t* gpu_out) {
    if (!gpu_out || depth < 1 || stage < 0 || stage >= depth || pipeline < 0 ||
        pipeline >= std::max(1, depth / 2))
        return AMDP_E_INVAL;
    const int d = depth, j = pipeline, i = stage;
    int g = (j % 2 == 0) ? (2 * j + i) % d : (2 * j - i + d + 1) % d;
    *gpu_out = ((g % d) + d) % d;
    return AMDP_OK;
}

extern "C" int amdp_schedule_preset(int32_t preset, int32_t depth, int32_t stage, int32_t n_minibatches,
                                    int32_t microbatches, amdp_sched_params_t* out) {
    if (!out || depth < 1 || stage < 0 || stage >= depth || n_minibatches < 0) return AMDP_E_INVAL;
    std::memset(out, 0, sizeof(*out));
    out->struct_size = sizeof(*out);
    out->depth = depth;
    out->stage = stage;
    out->n_minibatches = n_minibatches;
    out->pipelines = 1;
    switch (preset) {
        case AMDP_PRESET_AMDP:             // n = 2, d/2 pipelines, window >= d, update in the next bubble
            out->pipelines = std::max(1, depth / 2);
            out->inject_limit = 2;
            out->threshold = microbatches > 0 ? microbatches : 2 * depth;
            out->update_placement = AMDP_U_NEXT_BUBBLE;
            out->bwd_version = AMDP_BWD_CURRENT;
            return AMDP_OK;
        case AMDP_PRESET_PIPEDREAM:        // d minibatches in flight, update after every backward, weight stashing
            out->inject_limit = depth;
            out->threshold = 1;
            out->update_placement = AMDP_U_EAGER;
            out->bwd_version = AMDP_BWD_STASHED;
            return AMDP_OK;
        case AMDP_PRESET_PIPEDREAM_2BW:    // d in flight, gradients coalesced over d minibatches, double-buffered weights
            out->inject_limit = depth;
            out->threshold = microbatches > 0 ? microbatches : depth;
            if (out->threshold < depth) return AMDP_E_INVAL;
            out->update_placement = AMDP_U_EAGER;
            out->bwd_version = AMDP_BWD_STASHED;
            return AMDP_OK;
        case AMDP_PRESET_SYNC_1F1B:        // one minibatch of `microbatches` microbatches, flushed
            if (microbatches < 1) return AMDP_E_INVAL;
            out->inject_limit = depth;
            out->threshold = microbatches;
            out->update_placement = AMDP_U_FLUSH;
            out->bwd_version = AMDP_BWD_STASHED;
            return AMDP_OK;
    }
    return AMDP_E_INVAL;
}

namespace {

inline int map_gpu(int d, int j, int i) {
    const int g = (j % 2 == 0) ? (2 * j + i) % d : (2 * j - i + d + 1) % d;
    return ((g % d) + d) % d;
}

// A ready operation; ordering = the FIFO rule with its tie-breaks.
struct ReadyOp {
    int64_t ready;
    int kind, pipeline, mb, stage;
    bool operator>(const ReadyOp& o) const {
        if (ready != o.ready) return ready > o.ready;
        if (kind != o.kind) return kind < o.kind;            // backward (1) before forward (0)
        if (pipeline != o.pipeline) return pipeline > o.pipeline;
        if (mb != o.mb) return mb > o.mb;
        return stage > o.stage;
    }
};

}  // namespace

extern "C" int amdp_system_simulate(const amdp_sim_params_t* p, amdp_sim_op_t* ops, size_t cap, size_t* n_ops,
                                    int64_t* gpu_busy, amdp_sim_result_t* res) {
    if (!p || !n_ops || !res || p->struct_size != sizeof(amdp_sim_params_t) ||
        res->struct_size != sizeof(amdp_sim_result_t))
        return AMDP_E_INVAL;
    const int d = p->depth, P = p->pipelines, M = p->minibatches, tF = p->t_forward, tB = p->t_backward;
    if (d < 1 || d > 65535 || P < 1 || P > std::max(1, d / 2) || P > 255 || M < 0 || tF < 1 || tB < 1 ||
        p->inject_limit < 1 || p->preload < 0)
        return AMDP_E_INVAL;
    const long long limit = (long long)p->inject_limit + p->preload;
    const size_t total = 2 * (size_t)d * P * M;
    *n_ops = total;
    const bool record = ops && total <= cap;

    typedef std::priority_queue<ReadyOp, std::vector<ReadyOp>, std::greater<ReadyOp>> Queue;
    std::vector<Queue> ready((size_t)d);
    struct Running { bool on = false; int kind, pipeline, stage, mb; int64_t start, end; };
    std::vector<Running> running((size_t)d);
    std::vector<int64_t> busy((size_t)d, 0);
    std::vector<int> inflight((size_t)P, 0), next_inject((size_t)P, 0);
    std::priority_queue<int64_t, std::vector<int64_t>, std::greater<int64_t>> ends;
    std::vector<amdp_sim_op_t> done;
    if (record) done.reserve(total);
    int max_inflight = 0;
    int64_t makespan = 0;

    auto make_ready = [&](int64_t t, int kind, int j, int m, int i) {
        ready[(size_t)map_gpu(d, j, i)].push(ReadyOp{t, kind, j, m, i});
    };
    for (int j = 0; j < P; ++j) {
        const int first = (int)std::min<long long>(limit, M);
        for (int m = 0; m < first; ++m) make_ready(0, AMDP_EV_F, j, m, 0);
        inflight[j] = next_inject[j] = first;
        max_inflight = std::max(max_inflight, first);
    }
    int64_t t = 0;
    for (;;) {
        for (int g = 0; g < d; ++g) {          // start what can start now
            if (running[g].on || ready[g].empty() || ready[g].top().ready > t) continue;
            const ReadyOp r = ready[g].top();
            ready[g].pop();
            const int dur = r.kind == AMDP_EV_F ? tF : tB;
            running[g] = Running{true, r.kind, r.pipeline, r.stage, r.mb, t, t + dur};
            busy[g] += dur;
            ends.push(t + dur);
        }
        if (ends.empty()) break;
        t = ends.top();
        while (!ends.empty() && ends.top() == t) ends.pop();
        for (int g = 0; g < d; ++g) {          // finish what ends now
            Running& r = running[g];
            if (!r.on || r.end != t) continue;
            r.on = false;
            makespan = std::max(makespan, r.end);
            if (record) {
                amdp_sim_op_t o;
                std::memset(&o, 0, sizeof(o));
                o.kind = (uint8_t)r.kind; o.pipeline = (uint8_t)r.pipeline; o.stage = (uint16_t)r.stage;
                o.mb = r.mb; o.gpu = g; o.start = r.start; o.end = r.end;
                done.push_back(o);
            }
            const int j = r.pipeline, i = r.stage, m = r.mb;
            if (r.kind == AMDP_EV_F) {
                if (i + 1 < d) make_ready(t, AMDP_EV_F, j, m, i + 1);
                else make_ready(t, AMDP_EV_B, j, m, i);
            } else if (i > 0) {
                make_ready(t, AMDP_EV_B, j, m, i - 1);
            } else {
                --inflight[j];
                if (next_inject[j] < M) {
                    make_ready(t, AMDP_EV_F, j, next_inject[j]++, 0);
                    max_inflight = std::max(max_inflight, ++inflight[j]);
                }
            }
        }
    }
    res->max_inflight = max_inflight;
    res->makespan = makespan;
    res->busy_total = 0;
    res->busy_min = d ? busy[0] : 0;
    res->busy_max = 0;
    for (int g = 0; g < d; ++g) {
        res->busy_total += busy[g];
        res->busy_min = std::min(res->busy_min, busy[g]);
        res->busy_max = std::max(res->busy_max, busy[g]);
        if (gpu_busy) gpu_busy[g] = busy[g];
    }
    if (ops && total > cap) return AMDP_E_CAPACITY;
    if (!ops && total) return AMDP_E_CAPACITY;
    if (record) {
        std::stable_sort(done.begin(), done.end(), [](const amdp_sim_op_t& a, const amdp_sim_op_t& b) {
            return a.start != b.start ? a.start < b.start : a.gpu < b.gpu;
        });
        std::copy(done.begin(), done.end(), ops);
    }
    return AMDP_OK;
}

extern "C" const char* amdp_strerror(int code) {
    switch (code) {
        case AMDP_OK: return "ok";
        case AMDP_E_INVAL: return "invalid argument or configuration";
        case AMDP_E_MB_STATE: return "minibatch is in the wrong state for this call";
        case AMDP_E_NO_SLOT: return "no free activation slot: too many minibatches in flight";
        case AMDP_E_VERSION: return "weight version is not resident";
        case AMDP_E_STASH_FULL: return "no free weight-version slot for the update";
        case AMDP_E_HIP: return "HIP call or kernel launch failed";
        case AMDP_E_CAPACITY: return "output array too small";
        case AMDP_E_TOO_LARGE: return "problem exceeds the fixed capacity of the entry point that allocates nothing";
        default: return "unknown error";
    }
}
