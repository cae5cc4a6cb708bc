// Host-side AMDP schedule generator: the ordered forward / backward /
// accumulate / update events of one logical pipeline stage and the weight
// version each one reads (paper Sections 3.1-3.3; Lemma 1; Appendix B.4).
// Integer work only; no GPU involved.
#include "amdp.h"

#include <algorithm>
#include <cstring>
#include <map>
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
    if (p->update_placement != AMDP_U_NEXT_BUBBLE && p->update_placement != AMDP_U_EAGER)
        return AMDP_E_INVAL;
    if (p->bwd_version != AMDP_BWD_STASHED && p->bwd_version != AMDP_BWD_CURRENT) return AMDP_E_INVAL;

    const int n_updates = M ? ceil_div(M, T) : 0;
    const size_t total = 3 * (size_t)M + (size_t)n_updates;
    *n_out = total;
    if (total > cap || (!out && total)) return AMDP_E_CAPACITY;
    if (!total) return AMDP_OK;

    const int w = std::min(n, d - i);          // warm-up forwards per pipeline (Section 3.1)
    const int rounds = ceil_div(M, P);
    const bool eager = p->update_placement == AMDP_U_EAGER;
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
    auto forward_round = [&](int g) {
        for (int m = g * P; m < std::min((g + 1) * P, M); ++m) {
            fwd_tag[m] = applied;
            emit(AMDP_EV_F, m % P, 0, m, applied);
        }
    };
    auto backward_round = [&](int g) {
        for (int m = g * P; m < std::min((g + 1) * P, M); ++m) {
            // "next bubble": the update of the window that just closed goes in
            // front of the first backward of the following window
            if (!eager && m > 0 && m % T == 0) emit_update(m / T - 1);
            emit(AMDP_EV_B, m % P, 0, m, stashed ? fwd_tag[m] : applied);
            emit(AMDP_EV_A, m % P, 0, m, 0);
            if (eager && (m + 1) % T == 0) emit_update(m / T);
        }
    };

    for (int g = 0; g < std::min(w, rounds); ++g) forward_round(g);
    for (int g = 0; g < rounds; ++g) {
        backward_round(g);
        if (g + w < rounds) forward_round(g + w);
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
        default: return "unknown error";
    }
}
