#!/usr/bin/env python3
"""Benchmark of the AMDP stage hot path on one MI355X.

A step is one accumulation window of the stage's AMDP schedule in steady
state: T minibatches' forward, backward and gradient accumulation in schedule
order (forwards of later minibatches interleaved, each with its assigned
weight version) plus the window's fused Adam update. Inputs are synthetic,
seeded, and already resident in HBM when the timed region starts.

Prints ONE JSON line: stage tokens/s, plus `roofline` (dominant kernel against
the MFMA peak, timed with HIP events recorded on the launch stream inside the
library) and `cpu_baseline` (the CPU oracle timed on the host cores on a
bounded sample of the same workload).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0    # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3     # fp32 vector
PEAK_HBM_GBS = 8000.0


def algorithmic_flops_per_minibatch(w):
    """Linear layers 2*N*(in*out) forward per matrix, attention 4*N*s_eff*D
    forward (s_eff = (s+1)/2 causal; for padded bidirectional blocks the mean
    number of visible keys, valid lengths being uniform on s/4..s), LM head
    2*N*D*V forward; backward = 2 x forward."""
    N, D, F, s = w.tokens, w.d_model, w.d_ffn, w.seq_len
    lin = 2.0 * N * (3 * D * D + D * D + 2 * D * F)
    s_eff = (s + 1) / 2.0 if w.block_kind == 0 else (s // 4 + s) / 2.0
    att = 4.0 * N * s_eff * D
    fwd = w.n_layers * (lin + att)
    if w.has_lm_head:
        fwd += 2.0 * N * D * w.vocab
    return 3.0 * fwd


def recorded_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` on `workload` from the committed
    rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries under profiles/ (lines
    `traffic: <workload> <kernel> <bytes>`), or None."""
    import glob
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*hbm_traffic.md"))):
        for line in open(path):
            parts = line.split()
            if len(parts) == 4 and parts[0] == "traffic:" and parts[1] == workload and parts[2] == kernel:
                return float(parts[3])
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=str, default="5",
                    help="benchmark configuration 1..5 or a test shape name; default 5, the largest "
                         "single-GPU configuration, on which the matrix-core and HBM targets are stated")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--fused-accumulate", action="store_true",
                    help="backward adds parameter gradients straight into the sum (amdp_stage_set_fused_accumulate); "
                         "default is the schedule's own order with the accumulation as its own kernel")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs one pipeline stage on ONE GPU; --gpus must be 1 "
              "(there is no multi-GPU path: stages would be joined by one transfer per event and replicas of a "
              "stage by one gradient reduction per update)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2605_29664_amd as amdp
    import workloads as W

    w = W.get(args.config)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    T, P = w.threshold, w.pipelines
    K, Wu = args.steps, args.warmup
    inflight = w.act_slots
    # warm-up, timed, 2 profiled, a few steps on one stream, a few with fused accumulation
    M = (Wu + K + 3 + 2 * min(K, 3)) * T + inflight

    cfg = amdp.make_config(**W.stage_config_args(w))
    stage = amdp.Stage(cfg, device="cuda:0")
    layout = amdp.amdp_stage_param_layout(cfg)
    theta0 = torch.from_numpy(W.make_theta(w, layout)).to(dev)
    stage.amdp_stage_set_state(theta0)
    del theta0
    if args.fused_accumulate:
        stage.amdp_stage_set_fused_accumulate(True)

    ring = max(2, 2 * inflight)
    dt = stage.act_dtype
    X = [torch.from_numpy(W.make_x(w, k)).to(dev).to(dt) for k in range(ring)]
    dY = [None if w.has_lm_head else torch.from_numpy(W.make_dy(w, k)).to(dev).to(dt) for k in range(ring)]
    if w.has_lm_head:
        aux = [torch.from_numpy(W.make_targets(w, k)).to(dev) for k in range(ring)]
        outs = [torch.empty(1, dtype=torch.float32, device=dev) for _ in range(ring)]
    else:
        # token ids (+ padding mask) on a first stage, padding mask for BERT
        aux = [None if W.make_aux(w, k) is None else torch.from_numpy(np.asarray(W.make_aux(w, k), dtype=np.int32)).to(dev)
               for k in range(ring)]
        outs = [torch.empty((w.tokens, w.d_model), dtype=dt, device=dev) for _ in range(ring)]
    dX = torch.empty((w.tokens, w.d_model), dtype=dt, device=dev)

    events = amdp.amdp_schedule_generate(w.depth, P, w.stage, T, M, w.inject_limit,
                                         amdp.U_NEXT_BUBBLE, amdp.BWD_STASHED)
    # split into steps: a step ends with its update
    steps, cur = [], []
    for e in events:
        cur.append((e.kind, e.mb, e.version))
        if e.kind == amdp.EV_U:
            steps.append(cur)
            cur = []
    assert len(steps) >= Wu + K + 1

    def run_step(evs):
        for kind, mb, ver in evs:
            r = mb % ring
            if kind == amdp.EV_F:
                stage.amdp_stage_forward(mb, ver, X[r], aux[r], outs[r])
            elif kind == amdp.EV_B:
                stage.amdp_stage_backward(mb, ver, dY[r], dX)
            elif kind == amdp.EV_A:
                stage.amdp_grad_accumulate(mb)
            else:
                stage.amdp_apply_update(w.lr, w.beta1, w.beta2, w.eps, w.weight_decay, 1.0 / T, True)

    # step 0 holds the pipeline fill (extra forwards); it is always part of the warm-up
    n_warm = max(1, Wu)
    for i in range(n_warm):
        run_step(steps[i])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n_warm, n_warm + K):
        run_step(steps[i])
    enqueue = time.perf_counter() - t0      # host time to issue the work (the GPU runs behind it)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    cursor = n_warm + K          # next step of the schedule (steps must be run in order)
    tokens = K * T * w.tokens
    value = tokens / elapsed
    flops_step = T * algorithmic_flops_per_minibatch(w)
    peak = PEAK_BF16_TFLOPS if w.dtype == 1 else PEAK_FP32_TFLOPS

    result = {
        "metric": "stage tokens/sec (fwd+bwd+accumulate+update in AMDP schedule order)",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": n_warm,
        "ms_per_step": 1e3 * elapsed / K, "host_enqueue_ms_per_step": 1e3 * enqueue / K, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if w.dtype == 1 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "block": "gpt_preln_causal" if w.block_kind == 0 else "bert_postln_bidir",
                   "layers": w.n_layers, "d_model": w.d_model, "heads": w.n_heads, "d_ffn": w.d_ffn,
                   "seq_len": w.seq_len, "microbatch": w.microbatch,
                   "vocab": w.vocab if (w.has_lm_head or w.has_embedding) else 0,
                   "input_embedding": bool(w.has_embedding),
                   "depth": w.depth, "pipelines": P, "stage": w.stage, "minibatches_per_update": T,
                   "tokens_per_step": T * w.tokens, "parallelism": "1 stage on 1 GPU",
                   "accumulation": "fused into backward" if args.fused_accumulate else "own kernel per minibatch"},
        "end_to_end_mfu": flops_step * K / elapsed / (peak * 1e12),
        "algorithmic_tflop_per_step": flops_step / 1e12,
    }

    # ---- per-kernel device time from HIP events on the launch stream (a second,
    # identical pass over one step so the events do not perturb `value`) --------
    if not args.no_profile:
        def profile_step(step_events):
            stage.amdp_stage_profile_begin()
            run_step(step_events)
            return stage.amdp_stage_profile_end()

        def dominant_gemm(prof):
            gemms = {n: r for n, r in prof.items() if n.startswith("gemm_") and "batched" not in n and r["ms"] > 0}
            dom = max(gemms, key=lambda n: gemms[n]["ms"])
            r = gemms[dom]
            ach = r["flops"] / r["ms"] / 1e9
            return {"kernel": dom, "bound": "mfma" if w.dtype == 1 else "alu", "achieved": ach, "peak": peak,
                    "unit": "TFLOP/s", "frac": ach / peak, "traffic": recorded_traffic(w.name, dom),
                    "launches": r["launches"],
                    "avg_launch_ms": r["ms"] / r["launches"], "flops_per_launch": r["flops"] / r["launches"]}

        # (a) as timed: gradient leaves overlap with the dX chain on the side stream
        prof = profile_step(steps[cursor])
        cursor += 1
        table = {}
        for name, r in sorted(prof.items(), key=lambda kv: -kv[1]["ms"]):
            row = {"launches": r["launches"], "ms": round(r["ms"], 4)}
            if r["flops"] > 0 and r["ms"] > 0:
                row["tflops"] = round(r["flops"] / r["ms"] / 1e9, 2)
            if r["bytes"] > 0 and r["ms"] > 0:
                row["gbs"] = round(r["bytes"] / r["ms"] / 1e6, 1)
            table[name] = row
        result["kernels"] = table
        result["roofline"] = dominant_gemm(prof)
        result["side_stream"] = stage.amdp_stage_get_overlap()
        result["roofline"]["note"] = (("as timed: kernels of the side stream run concurrently, so a launch shares "
                                       "the compute units with others; see roofline_isolated") if result["side_stream"]
                                      else "as timed: the side stream is off at this width, every kernel has the GPU to itself")
        def streaming(pr):
            out = {}
            for nm in ("grad_accumulate", "adam_update"):
                if nm in pr and pr[nm]["ms"] > 0:
                    gbs = pr[nm]["bytes"] / pr[nm]["ms"] / 1e6
                    out[nm] = {"gbs": gbs, "frac_of_hbm_peak": gbs / PEAK_HBM_GBS,
                               "avg_launch_ms": pr[nm]["ms"] / pr[nm]["launches"]}
            return out
        # as timed the accumulation runs on the side stream under the next minibatch's
        # kernels and shares HBM with them; "streaming" below is replaced by the
        # isolated figures (each kernel alone on the GPU) when that pass runs
        result["streaming_as_timed"] = streaming(prof)
        result["streaming"] = result["streaming_as_timed"]
        # (b) every kernel alone on the GPU (side stream off), same launches
        iso = None
        if len(steps) > cursor:
            overlap_default = stage.amdp_stage_get_overlap()
            stage.amdp_stage_set_overlap(False)
            iso = profile_step(steps[cursor])
            cursor += 1
            stage.amdp_stage_set_overlap(overlap_default)
            result["roofline_isolated"] = dominant_gemm(iso)
            result["streaming"] = streaming(iso)
            gem = {n: r for n, r in iso.items() if n.startswith("gemm_") and r["ms"] > 0}
            lin = {n: r for n, r in gem.items() if "batched" not in n}
            for key, grp in (("all_gemm_kernels", gem), ("linear_gemm_kernels", lin)):
                tf, tm = sum(x["flops"] for x in grp.values()), sum(x["ms"] for x in grp.values())
                result[key + "_isolated"] = {"tflops": tf / tm / 1e9, "frac_of_peak": tf / tm / 1e9 / peak, "ms_per_step": tm}
            result["kernels_isolated"] = {n: {"launches": r["launches"], "ms": round(r["ms"], 4),
                                              **({"tflops": round(r["flops"] / r["ms"] / 1e9, 2)} if r["flops"] > 0 else {}),
                                              **({"gbs": round(r["bytes"] / r["ms"] / 1e6, 1)} if r["bytes"] > 0 else {})}
                                          for n, r in sorted(iso.items(), key=lambda kv: -kv[1]["ms"]) if r["ms"] > 0}

        # kernel-level matrix-core figure: every GEMM and fused-attention launch of the step
        # (algorithmic flops / summed durations, each kernel alone on the GPU when that pass ran)
        src = iso if iso is not None else prof
        mat = {n: r for n, r in src.items() if (n.startswith("gemm_") or n.startswith("flash_attention")) and r["ms"] > 0}
        if mat:
            # the library books padded bidirectional attention at all s keys per query (it cannot see
            # the valid lengths on the host); the algorithmic figure uses the mean number of visible keys
            vis = 1.0 if w.block_kind == 0 else ((w.seq_len // 4 + w.seq_len) / 2.0) / w.seq_len
            tf = sum(x["flops"] * (vis if n.startswith("flash_attention") else 1.0) for n, x in mat.items())
            tm = sum(x["ms"] for x in mat.values())
            result["matrix_kernels"] = {"tflops": tf / tm / 1e9, "frac_of_peak": tf / tm / 1e9 / peak, "ms_per_step": tm,
                                        "kernels": "gemm_* and flash_attention_*", "pass": "isolated" if src is iso else "as timed"}

        # achievable HBM ceiling beside the published peak: the library's own plain copy
        # kernel on 2 GiB (far beyond the 256 MB last-level cache), read + write counted
        nb = 2 << 30
        src = torch.empty(nb, dtype=torch.uint8, device=dev).random_()
        dst = torch.empty(nb, dtype=torch.uint8, device=dev)
        best = None
        for _ in range(4):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            amdp.amdp_device_copy(dst, src)
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        del src, dst
        copy_gbs = 2.0 * nb / best / 1e6
        result["hbm_copy_ceiling"] = {"gbs": copy_gbs, "frac_of_hbm_peak": copy_gbs / PEAK_HBM_GBS,
                                      "bytes": 2 * nb, "kernel": "copy16_kernel (amdp_device_copy), 2 GiB"}
        for nm, row in result["streaming"].items():
            row["frac_of_copy_ceiling"] = row["gbs"] / copy_gbs

    # ---- the row kernels on their own (entry points amdp_layernorm_* / amdp_column_sums) at the
    # stage's own size, where a launch moves a few tens of MB and is bound by launch and memory
    # latency, and at 16 times the rows, where it is bound by HBM ------------------------------
    if not args.no_profile and w.dtype == 1:
        result["row_kernels"] = row_kernel_rates(torch, amdp, w, dev)

    # padded sequences (bidirectional blocks): tokens that are not padding, per second
    if w.block_kind != 0 and not w.has_lm_head:
        valid = 0
        for i in range(n_warm, n_warm + K):
            for kind, mb, ver in steps[i]:
                if kind == amdp.EV_F:
                    a = W.make_aux(w, mb % ring)
                    valid += int(np.asarray(a[-w.microbatch:]).sum())
        result["valid_tokens_per_s"] = valid / elapsed

    # ---- the same steps with the accumulation fused into backward (an option of
    # the library; `value` above is the schedule's own order) --------------------
    # (three steps at most: under a kernel trace of this command the launches of this leg, whose
    # weight-gradient products read and write the sum, would otherwise shift every average)
    Kf = min(K, 3)
    # ---- the same steps with everything on the caller's stream (same box, same process):
    # what the side stream is worth on this workload ---------------------------------------
    if stage.amdp_stage_get_overlap() and len(steps) >= cursor + 2 * Kf:
        form = stage.amdp_stage_get_overlap()
        stage.amdp_stage_set_overlap(0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(cursor, cursor + Kf):
            run_step(steps[i])
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        cursor += Kf
        stage.amdp_stage_set_overlap(form)
        result["single_stream"] = {"value": Kf * T * w.tokens / el, "unit": "tokens/s", "ms_per_step": 1e3 * el / Kf,
                                   "steps": Kf, "note": "amdp_stage_set_overlap(0): every kernel on the caller's stream"}
    if not args.fused_accumulate and len(steps) >= cursor + Kf:
        stage.amdp_stage_set_fused_accumulate(True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(cursor, cursor + Kf):
            run_step(steps[i])
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        result["fused_accumulate"] = {"value": Kf * T * w.tokens / el, "unit": "tokens/s", "ms_per_step": 1e3 * el / Kf, "steps": Kf,
                                      "note": "amdp_stage_set_fused_accumulate(1): dW products and column sums add "
                                              "into the gradient sum directly; bit-identical state, no per-minibatch gradient"}

    stage.close()
    del stage
    torch.cuda.empty_cache()

    # ---- the CPU oracle on the host cores, bounded sample ---------------------
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w)

    print(json.dumps(result))


def row_kernel_rates(torch, amdp, w, dev):
    """GB/s of algorithmic traffic (each input read once, each output written once) of the
    LayerNorm and column-sum kernels through their own entry points, HIP-event timed."""
    out = {}
    D = w.d_model
    for label, rows in (("stage_rows", w.tokens), ("rows_x16", 16 * w.tokens)):
        x = torch.randn((rows, D), device=dev, dtype=torch.float32).to(torch.bfloat16)
        dy = (1e-3 * torch.randn((rows, D), device=dev, dtype=torch.float32)).to(torch.bfloat16)
        res = dy.clone()
        g = torch.ones(D, device=dev, dtype=torch.bfloat16)
        y, dx = torch.empty_like(x), torch.empty_like(x)
        stats = torch.empty((rows, 2), device=dev, dtype=torch.float32)
        ws = torch.empty(amdp.amdp_column_sums_workspace_bytes(rows, D, amdp.BF16, True), dtype=torch.uint8, device=dev)
        sums = torch.empty(2 * D, device=dev, dtype=torch.float32)
        nb = rows * D * 2
        cases = {
            "layernorm_fwd": (lambda: amdp.amdp_layernorm_forward(x, g, g, y, stats, 1e-5), 2 * nb),
            "layernorm_bwd": (lambda: amdp.amdp_layernorm_backward(dy, x, stats, g, res, dx), 4 * nb),
            "column_sums_bias": (lambda: amdp.amdp_column_sums(dy, None, None, sums, ws), nb),
            "column_sums_layernorm": (lambda: amdp.amdp_column_sums(dy, x, stats, sums, ws), 2 * nb),
        }
        row = {}
        for name, (fn, nbytes) in cases.items():
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            n_it = 20
            e0.record()
            for _ in range(n_it):
                fn()
            e1.record()
            e1.synchronize()
            ms = e0.elapsed_time(e1) / n_it
            row[name] = {"us": round(1e3 * ms, 2), "gbs": round(nbytes / ms / 1e6, 1),
                         "frac_of_hbm_peak": round(nbytes / ms / 1e6 / PEAK_HBM_GBS, 3)}
        out[label] = {"rows": rows, "cols": D, **row}
        del x, dy, res, y, dx, stats, ws, sums
    return out


def cpu_baseline(w):
    """Times the oracle as it stands: forward + backward + accumulate of a few
    whole minibatches plus one Adam step over the stage's parameters (charged 1/T per
    minibatch), in fp64, on the host's cores."""
    import numpy as np
    import workloads as W
    from oracle import optim
    from oracle.stage import Stage as OStage
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count()
    ost = OStage.from_workload(w)
    theta = W.make_theta(w, ost.layout).astype(np.float64)
    # whole minibatches until about 12 s of CPU time are spent (at least one, at most four)
    G = np.zeros_like(theta)
    n_mb, t0 = 0, time.perf_counter()
    while n_mb < 4 and (n_mb == 0 or time.perf_counter() - t0 < 12.0):
        x = W.make_x(w, n_mb)
        aux = W.make_aux(w, n_mb)
        dy = None if w.has_lm_head else W.make_dy(w, n_mb)
        _, saved = ost.forward(theta, x, aux)
        _, g = ost.backward(theta, saved, dy)
        optim.accumulate(G, g)
        n_mb += 1
    t1 = time.perf_counter()
    optim.adam_step(theta, np.zeros_like(theta), np.zeros_like(theta), G, 1, w.lr, w.beta1, w.beta2, w.eps)
    t2 = time.perf_counter()
    per_mb = (t1 - t0) / n_mb + (t2 - t1) / w.threshold
    scalar = scalar_loop_tier()
    return {"scalar_loop_tier": scalar, "value": w.tokens / per_mb, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n_mb} minibatch(es) of {w.tokens} tokens forward+backward+accumulate in fp64 numpy "
                      f"({t1 - t0:.1f} s) + 1/{w.threshold} of one Adam step ({t2 - t1:.2f} s)",
            "host_cpus": os.cpu_count()}


def scalar_loop_tier():
    """The oracle's second tier (plain C loops over scalars, fp64, one thread) on
    configuration 1, the only benchmark configuration it finishes in seconds:
    forward + backward of whole minibatches for about two seconds."""
    import numpy as np
    import workloads as W
    from oracle.slow import SlowStage
    w = W.get("1")
    sl = SlowStage.from_workload(w)
    from oracle.stage import param_layout
    theta = W.make_theta(w, param_layout(w.n_layers, w.d_model, w.d_ffn)).astype(np.float64)
    n_mb, t0 = 0, time.perf_counter()
    while n_mb == 0 or (n_mb < 64 and time.perf_counter() - t0 < 2.0):
        x, dy = W.make_x(w, n_mb).astype(np.float64), W.make_dy(w, n_mb).astype(np.float64)
        _, saved = sl.forward(theta, x)
        sl.backward(theta, saved, dy)
        n_mb += 1
    dt = time.perf_counter() - t0
    return {"value": n_mb * w.tokens / dt, "unit": "tokens/s", "cores": 1, "workload": w.name,
            "sample": f"{n_mb} minibatch(es) of {w.tokens} tokens forward+backward in fp64 C loops ({dt:.2f} s)"}


if __name__ == "__main__":
    main()
