"""ctypes binding of include/amdp.h. Function names and argument order follow
the header; the only additions are error-code-to-exception translation and the
`Stage` convenience wrapper that owns the workspace tensor."""
import ctypes as C
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
_LIB_NAME = "libamdp.so"

EV_F, EV_B, EV_A, EV_U = 0, 1, 2, 3
U_NEXT_BUBBLE, U_EAGER = 0, 1
BWD_STASHED, BWD_CURRENT = 0, 1
FLAG_LAST_USE, FLAG_PARTIAL_WINDOW = 1, 2
BLOCK_GPT, BLOCK_BERT = 0, 1
FP32, BF16 = 0, 1
ATTN_AUTO, ATTN_UNFUSED = 0, 1
OPT_GEMM_TILE, OPT_GEMM_TRANSPOSING_READS, OPT_GEMM_DIRECT_TO_LDS, OPT_LAZY_JOIN, OPT_SPLIT_K_MIN_TOKENS, OPT_SPLIT_MAIN_MIN_K, OPT_LEAF_FORKS = 0, 1, 2, 3, 4, 5, 6
E_INVAL, E_MB_STATE, E_NO_SLOT, E_VERSION, E_STASH_FULL, E_HIP, E_CAPACITY = -1, -2, -3, -4, -5, -6, -7
E_TOO_LARGE = -8


class AmdpError(RuntimeError):
    def __init__(self, code, what=""):
        self.code = code
        detail = ""
        if code == E_HIP:
            detail = " [" + lib().amdp_last_hip_error().decode() + "]"
        super().__init__(f"{what}: {amdp_strerror(code)} ({code}){detail}")


class amdp_event_t(C.Structure):
    _fields_ = [("kind", C.c_uint8), ("pipeline", C.c_uint8), ("flags", C.c_uint16),
                ("mb", C.c_int32), ("version", C.c_uint32)]


class amdp_sched_params_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("depth", C.c_int32), ("pipelines", C.c_int32),
                ("stage", C.c_int32), ("inject_limit", C.c_int32), ("threshold", C.c_int32),
                ("n_minibatches", C.c_int32), ("update_placement", C.c_int32),
                ("bwd_version", C.c_int32)]


class amdp_sched_stats_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("max_inflight", C.c_int32),
                ("max_inflight_per_pipeline", C.c_int32), ("max_mismatch", C.c_int32),
                ("max_affected_per_window", C.c_int32), ("max_live_versions", C.c_int32)]


class amdp_sim_params_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("depth", C.c_int32), ("pipelines", C.c_int32),
                ("inject_limit", C.c_int32), ("preload", C.c_int32), ("minibatches", C.c_int32),
                ("t_forward", C.c_int32), ("t_backward", C.c_int32)]


class amdp_sim_op_t(C.Structure):
    _fields_ = [("kind", C.c_uint8), ("pipeline", C.c_uint8), ("stage", C.c_uint16), ("mb", C.c_int32),
                ("gpu", C.c_int32), ("start", C.c_int64), ("end", C.c_int64)]


class amdp_sim_result_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("max_inflight", C.c_int32), ("makespan", C.c_int64),
                ("busy_total", C.c_int64), ("busy_min", C.c_int64), ("busy_max", C.c_int64)]


class amdp_stage_config_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("block_kind", C.c_int32), ("n_layers", C.c_int32),
                ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ffn", C.c_int32),
                ("seq_len", C.c_int32), ("microbatch", C.c_int32), ("dtype", C.c_int32),
                ("has_lm_head", C.c_int32), ("vocab", C.c_int32), ("ln_eps", C.c_float),
                ("act_slots", C.c_int32), ("stash_slots", C.c_int32), ("has_embedding", C.c_int32),
                ("attention", C.c_int32)]


class amdp_param_desc_t(C.Structure):
    _fields_ = [("name", C.c_char * 24), ("offset", C.c_uint64), ("rows", C.c_uint32),
                ("cols", C.c_uint32)]


class amdp_profile_entry_t(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_uint64), ("ms", C.c_double),
                ("flops", C.c_double), ("bytes", C.c_double)]


class amdp_adam_t(C.Structure):
    _fields_ = [("struct_size", C.c_uint32), ("bias_correction", C.c_int32), ("lr", C.c_double),
                ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("grad_scale", C.c_double)]


def lib_path():
    return os.path.join(HERE, _LIB_NAME)


def build(verbose=False):
    """Compile libamdp.so for gfx950 with hipcc (cross-compiles without a GPU)."""
    src = [os.path.join(HERE, "csrc", "stage.hip"), os.path.join(HERE, "csrc", "schedule.cpp")]
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-pass-failed", "-I" + os.path.join(ROOT, "include"), "-o", lib_path()] + src
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode:
        print(" ".join(cmd))
        print(res.stdout, res.stderr)
    if res.returncode:
        raise RuntimeError("hipcc failed building libamdp.so")
    global _lib
    _lib = None
    return lib_path()


_lib = None


def lib():
    """The loaded library. Fails loudly when it has not been built: there is no
    fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime under the same soname as the system's.
    # Import it first so that this library binds to the runtime instance that
    # owns the process's device context and streams; loading in the other
    # order leaves two half-initialised runtimes ("no ROCm-capable device").
    import torch  # noqa: F401
    path = lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
    L = C.CDLL(path)
    vp, sz, i32, u32, u64 = C.c_void_p, C.c_size_t, C.c_int32, C.c_uint32, C.c_uint64
    P = C.POINTER
    sigs = {
        "amdp_strerror": (C.c_char_p, [C.c_int]),
        "amdp_last_hip_error": (C.c_char_p, []),
        "amdp_schedule_generate": (C.c_int, [P(amdp_sched_params_t), P(amdp_event_t), sz, P(sz)]),
        "amdp_schedule_stats": (C.c_int, [P(amdp_event_t), sz, i32, P(amdp_sched_stats_t)]),
        "amdp_stage_map": (C.c_int, [i32, i32, i32, P(i32)]),
        "amdp_schedule_preset": (C.c_int, [i32, i32, i32, i32, i32, P(amdp_sched_params_t)]),
        "amdp_system_simulate": (C.c_int, [P(amdp_sim_params_t), P(amdp_sim_op_t), sz, P(sz), P(C.c_int64),
                                           P(amdp_sim_result_t)]),
        "amdp_stage_n_params": (sz, [P(amdp_stage_config_t)]),
        "amdp_stage_workspace_bytes": (sz, [P(amdp_stage_config_t)]),
        "amdp_stage_param_layout": (C.c_int, [P(amdp_stage_config_t), P(amdp_param_desc_t), i32, P(i32)]),
        "amdp_stage_create": (C.c_int, [P(amdp_stage_config_t), vp, sz, vp, P(vp)]),
        "amdp_stage_destroy": (C.c_int, [vp]),
        "amdp_stage_set_state": (C.c_int, [vp, vp, vp, vp, u64, u32]),
        "amdp_stage_get_state": (C.c_int, [vp, vp, vp, vp, vp, P(u64), P(u32)]),
        "amdp_stage_get_staged_grad": (C.c_int, [vp, vp]),
        "amdp_stage_resident_versions": (C.c_int, [vp, P(u32), i32, P(i32)]),
        "amdp_stage_forward": (C.c_int, [vp, i32, u32, vp, vp, vp]),
        "amdp_stage_backward": (C.c_int, [vp, i32, u32, vp, vp]),
        "amdp_grad_accumulate": (C.c_int, [vp, i32]),
        "amdp_apply_update": (C.c_int, [vp, P(amdp_adam_t), P(u32)]),
        "amdp_stage_set_overlap": (C.c_int, [vp, i32]),
        "amdp_stage_get_overlap": (C.c_int, [vp, P(i32)]),
        "amdp_stage_join": (C.c_int, [vp]),
        "amdp_stage_set_option": (C.c_int, [vp, i32, i32]),
        "amdp_device_copy": (C.c_int, [vp, vp, sz, vp]),
        "amdp_layernorm_forward": (C.c_int, [vp, vp, vp, vp, vp, i32, i32, i32, C.c_float, vp]),
        "amdp_layernorm_backward": (C.c_int, [vp, vp, vp, vp, vp, vp, i32, i32, i32, vp]),
        "amdp_column_sums_workspace_bytes": (sz, [i32, i32, i32, i32]),
        "amdp_column_sums": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, vp, sz, vp]),
        "amdp_column_sums_static_max_cols": (sz, [i32]),
        "amdp_column_sums_static": (C.c_int, [vp, vp, vp, vp, i32, i32, i32, vp]),
        "amdp_stage_read_version": (C.c_int, [vp, u32, vp]),
        "amdp_stage_set_fused_accumulate": (C.c_int, [vp, i32]),
        "amdp_tie_embedding_grads": (C.c_int, [vp, vp]),
        "amdp_stage_profile_begin": (C.c_int, [vp]),
        "amdp_stage_profile_end": (C.c_int, [vp, P(amdp_profile_entry_t), i32, P(i32)]),
    }
    for name, (res, args) in sigs.items():
        fn = getattr(L, name)
        fn.restype = res
        fn.argtypes = args
    _lib = L
    return L


EXPORTED = ["amdp_strerror", "amdp_last_hip_error", "amdp_schedule_generate", "amdp_schedule_stats", "amdp_stage_map", "amdp_schedule_preset",
            "amdp_system_simulate",
            "amdp_stage_n_params", "amdp_stage_workspace_bytes", "amdp_stage_param_layout",
            "amdp_stage_create", "amdp_stage_destroy", "amdp_stage_set_state", "amdp_stage_get_state",
            "amdp_stage_get_staged_grad", "amdp_stage_resident_versions", "amdp_stage_forward",
            "amdp_stage_backward", "amdp_grad_accumulate", "amdp_apply_update",
            "amdp_stage_set_overlap", "amdp_stage_get_overlap", "amdp_stage_join", "amdp_stage_set_option", "amdp_device_copy", "amdp_layernorm_forward", "amdp_layernorm_backward",
            "amdp_column_sums_workspace_bytes", "amdp_column_sums", "amdp_column_sums_static_max_cols",
            "amdp_column_sums_static", "amdp_stage_read_version", "amdp_stage_set_fused_accumulate", "amdp_tie_embedding_grads",
            "amdp_stage_profile_begin", "amdp_stage_profile_end"]


def _check(rc, what):
    if rc != 0:
        raise AmdpError(rc, what)


def amdp_strerror(code):
    return lib().amdp_strerror(code).decode()


def amdp_schedule_generate(depth, pipelines, stage, threshold, n_minibatches, inject_limit=2,
                           update_placement=U_NEXT_BUBBLE, bwd_version=BWD_STASHED):
    """Returns a ctypes array of amdp_event_t."""
    p = amdp_sched_params_t(C.sizeof(amdp_sched_params_t), depth, pipelines, stage, inject_limit,
                            threshold, n_minibatches, update_placement, bwd_version)
    n = C.c_size_t(0)
    rc = lib().amdp_schedule_generate(C.byref(p), None, 0, C.byref(n))
    if rc not in (0, E_CAPACITY):
        raise AmdpError(rc, "amdp_schedule_generate")
    arr = (amdp_event_t * max(1, n.value))()
    _check(lib().amdp_schedule_generate(C.byref(p), arr, n.value, C.byref(n)), "amdp_schedule_generate")
    return (amdp_event_t * n.value).from_buffer(arr) if n.value else (amdp_event_t * 0)()


PRESET_AMDP, PRESET_PIPEDREAM, PRESET_PIPEDREAM_2BW, PRESET_SYNC_1F1B = 0, 1, 2, 3
U_FLUSH = 2


def amdp_schedule_preset(preset, depth, stage, n_minibatches, microbatches=0):
    """Events of one of Table 1's schedules for one stage, and the window length used."""
    p = amdp_sched_params_t()
    _check(lib().amdp_schedule_preset(preset, depth, stage, n_minibatches, microbatches, C.byref(p)),
           "amdp_schedule_preset")
    ev = amdp_schedule_generate(p.depth, p.pipelines, p.stage, p.threshold, p.n_minibatches, p.inject_limit,
                                p.update_placement, p.bwd_version)
    return ev, p


def amdp_schedule_stats(events, threshold):
    out = amdp_sched_stats_t(C.sizeof(amdp_sched_stats_t))
    _check(lib().amdp_schedule_stats(events, len(events), threshold, C.byref(out)), "amdp_schedule_stats")
    return {k: getattr(out, k) for k, _ in amdp_sched_stats_t._fields_[1:]}


def amdp_stage_map(depth, pipeline, stage):
    g = C.c_int32(-1)
    _check(lib().amdp_stage_map(depth, pipeline, stage, C.byref(g)), "amdp_stage_map")
    return g.value


def amdp_system_simulate(depth, pipelines, minibatches, t_forward=1, t_backward=2, inject_limit=2, preload=0):
    """Returns (ops, info): ops = list of (kind, pipeline, stage, mb, gpu, start, end) in start order."""
    p = amdp_sim_params_t(C.sizeof(amdp_sim_params_t), depth, pipelines, inject_limit, preload, minibatches,
                          t_forward, t_backward)
    res = amdp_sim_result_t(C.sizeof(amdp_sim_result_t))
    n = C.c_size_t(0)
    rc = lib().amdp_system_simulate(C.byref(p), None, 0, C.byref(n), None, C.byref(res))
    if rc not in (0, E_CAPACITY):
        raise AmdpError(rc, "amdp_system_simulate")
    arr = (amdp_sim_op_t * max(1, n.value))()
    busy = (C.c_int64 * depth)()
    _check(lib().amdp_system_simulate(C.byref(p), arr, n.value, C.byref(n), busy, C.byref(res)),
           "amdp_system_simulate")
    ops = [(o.kind, o.pipeline, o.stage, o.mb, o.gpu, o.start, o.end) for o in arr[:n.value]]
    return ops, dict(makespan=res.makespan, busy=list(busy), max_inflight=res.max_inflight,
                     busy_total=res.busy_total, busy_min=res.busy_min, busy_max=res.busy_max)


def amdp_tie_embedding_grads(first, last):
    """first, last: Stage objects (input-embedding stage, LM-head stage)."""
    _check(lib().amdp_tie_embedding_grads(first.handle, last.handle), "amdp_tie_embedding_grads")


def amdp_device_copy(dst, src, nbytes=None, stream=None):
    """dst, src: contiguous tensors on one device; copies nbytes (default: all of src)."""
    import torch
    n = src.numel() * src.element_size() if nbytes is None else nbytes
    if n > dst.numel() * dst.element_size() or n > src.numel() * src.element_size():
        raise ValueError("amdp_device_copy: buffer too small")
    st = stream if stream is not None else torch.cuda.current_stream(src.device)
    _check(lib().amdp_device_copy(_ptr(dst, device=src.device), _ptr(src), n, C.c_void_p(st.cuda_stream)),
           "amdp_device_copy")


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return FP32
    raise TypeError(f"unsupported element type {t.dtype}")


def _stream_ptr(t, stream):
    import torch
    st = stream if stream is not None else torch.cuda.current_stream(t.device)
    return C.c_void_p(st.cuda_stream)


def amdp_layernorm_forward(x, gamma, beta, y, stats, eps, stream=None):
    """x, y: [rows, cols]; gamma, beta: [cols]; stats: float32 [rows, 2]."""
    import torch
    rows, cols = x.shape
    dev, dt = x.device, x.dtype
    _check(lib().amdp_layernorm_forward(_ptr(x), _ptr(gamma, dt, cols, dev), _ptr(beta, dt, cols, dev),
                                        _ptr(y, dt, rows * cols, dev), _ptr(stats, torch.float32, 2 * rows, dev),
                                        rows, cols, _dtype_code(x), eps, _stream_ptr(x, stream)),
           "amdp_layernorm_forward")


def amdp_layernorm_backward(dy, x, stats, gamma, res, dx, stream=None):
    import torch
    rows, cols = x.shape
    dev, dt = x.device, x.dtype
    _check(lib().amdp_layernorm_backward(_ptr(dy, dt, rows * cols, dev), _ptr(x), _ptr(stats, torch.float32, 2 * rows, dev),
                                         _ptr(gamma, dt, cols, dev), _ptr(res, dt, rows * cols, dev),
                                         _ptr(dx, dt, rows * cols, dev), rows, cols, _dtype_code(x),
                                         _stream_ptr(x, stream)), "amdp_layernorm_backward")


def amdp_column_sums_workspace_bytes(rows, cols, dtype, with_layernorm):
    return lib().amdp_column_sums_workspace_bytes(rows, cols, dtype, int(bool(with_layernorm)))


def amdp_column_sums(dy, x, stats, out, workspace, stream=None):
    """dy: [rows, cols]; x, stats: None for plain column sums (out float32 [cols]),
    else the LayerNorm input and statistics (out float32 [2*cols]); workspace: uint8 tensor."""
    import torch
    rows, cols = dy.shape
    dev = dy.device
    ln = x is not None
    _check(lib().amdp_column_sums(_ptr(dy), _ptr(x, dy.dtype, rows * cols, dev),
                                  _ptr(stats, torch.float32, 2 * rows, dev) if ln else None,
                                  _ptr(out, torch.float32, (2 if ln else 1) * cols, dev), rows, cols, _dtype_code(dy),
                                  _ptr(workspace, torch.uint8, None, dev), workspace.numel(), _stream_ptr(dy, stream)),
           "amdp_column_sums")


def amdp_column_sums_static_max_cols(with_layernorm):
    return lib().amdp_column_sums_static_max_cols(int(bool(with_layernorm)))


def amdp_column_sums_static(dy, x, stats, out, stream=None):
    """amdp_column_sums without a workspace argument (and without any allocation)."""
    import torch
    rows, cols = dy.shape
    dev = dy.device
    ln = x is not None
    _check(lib().amdp_column_sums_static(_ptr(dy), _ptr(x, dy.dtype, rows * cols, dev),
                                         _ptr(stats, torch.float32, 2 * rows, dev) if ln else None,
                                         _ptr(out, torch.float32, (2 if ln else 1) * cols, dev), rows, cols,
                                         _dtype_code(dy), _stream_ptr(dy, stream)), "amdp_column_sums_static")


def make_config(block_kind, n_layers, d_model, n_heads, d_ffn, seq_len, microbatch, dtype,
                has_lm_head=False, vocab=0, ln_eps=1e-5, act_slots=4, stash_slots=1, has_embedding=False,
                attention=ATTN_AUTO):
    return amdp_stage_config_t(C.sizeof(amdp_stage_config_t), block_kind, n_layers, d_model, n_heads,
                               d_ffn, seq_len, microbatch, dtype, int(bool(has_lm_head)), vocab, ln_eps,
                               act_slots, stash_slots, int(bool(has_embedding)), attention)


def amdp_stage_n_params(cfg):
    return lib().amdp_stage_n_params(C.byref(cfg))


def amdp_stage_workspace_bytes(cfg):
    return lib().amdp_stage_workspace_bytes(C.byref(cfg))


def amdp_stage_param_layout(cfg):
    """List of (name, offset, rows, cols)."""
    n = C.c_int32(0)
    rc = lib().amdp_stage_param_layout(C.byref(cfg), None, 0, C.byref(n))
    if rc not in (0, E_CAPACITY):
        raise AmdpError(rc, "amdp_stage_param_layout")
    arr = (amdp_param_desc_t * n.value)()
    _check(lib().amdp_stage_param_layout(C.byref(cfg), arr, n.value, C.byref(n)), "amdp_stage_param_layout")
    return [(d.name.decode(), int(d.offset), int(d.rows), int(d.cols)) for d in arr]


def _ptr(t, dtype=None, numel=None, device=None):
    """Device address of a tensor after checking that it is what the C ABI
    expects: right element type, contiguous, on the stage's GPU, big enough."""
    if t is None:
        return None
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"expected a {dtype} tensor, got {t.dtype}")
    if not t.is_contiguous():
        raise TypeError("tensor must be contiguous")
    if device is not None and t.device != device:
        raise TypeError(f"tensor is on {t.device}, the stage on {device}")
    if numel is not None and t.numel() < numel:
        raise ValueError(f"tensor has {t.numel()} elements, {numel} needed")
    return C.c_void_p(t.data_ptr())


class Stage:
    """Owns the workspace tensor and the amdp_stage_t handle. Methods carry the
    names of the C entry points they call. Tensors must live on the stage's
    device; nothing here synchronises."""

    def __init__(self, cfg, device="cuda:0", stream=None, poison=False):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        self.n_params = amdp_stage_n_params(cfg)
        nbytes = amdp_stage_workspace_bytes(cfg)
        if self.n_params == 0 or nbytes == 0:
            raise AmdpError(E_INVAL, "amdp_stage_workspace_bytes")
        self.workspace_bytes = nbytes
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
            if poison:   # test aid: every byte 0xFF reads as NaN in fp32 and bf16
                self.workspace.fill_(255)
            base = self.workspace.data_ptr()
            self._ws_ptr = (base + 255) // 256 * 256
            h = C.c_void_p()
            _check(lib().amdp_stage_create(C.byref(cfg), C.c_void_p(self._ws_ptr), nbytes,
                                           C.c_void_p(self.stream.cuda_stream), C.byref(h)),
                   "amdp_stage_create")
        self.handle = h
        self.act_dtype = torch.bfloat16 if cfg.dtype == BF16 else torch.float32
        self.tokens = cfg.seq_len * cfg.microbatch
        self.device = self.workspace.device

    def _p32(self, t):
        return _ptr(t, self.torch.float32, self.n_params, self.device)

    def _act(self, t):
        return _ptr(t, self.act_dtype, self.tokens * self.cfg.d_model, self.device)

    def close(self):
        if getattr(self, "handle", None):
            lib().amdp_stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def amdp_stage_set_state(self, theta, m=None, v=None, step=0, version=0):
        _check(lib().amdp_stage_set_state(self.handle, self._p32(theta), self._p32(m), self._p32(v), step,
                                          version), "amdp_stage_set_state")

    def amdp_stage_get_state(self, theta=None, m=None, v=None, G=None):
        step, ver = C.c_uint64(0), C.c_uint32(0)
        _check(lib().amdp_stage_get_state(self.handle, self._p32(theta), self._p32(m), self._p32(v),
                                          self._p32(G), C.byref(step), C.byref(ver)), "amdp_stage_get_state")
        return step.value, ver.value

    def amdp_stage_get_staged_grad(self, g):
        _check(lib().amdp_stage_get_staged_grad(self.handle, self._p32(g)), "amdp_stage_get_staged_grad")

    def amdp_stage_resident_versions(self):
        arr = (C.c_uint32 * 32)()
        n = C.c_int32(0)
        _check(lib().amdp_stage_resident_versions(self.handle, arr, 32, C.byref(n)),
               "amdp_stage_resident_versions")
        return sorted(arr[i] for i in range(n.value))

    def amdp_stage_forward(self, mb, version, X, aux, out):
        torch = self.torch
        if self.cfg.has_lm_head:
            a = _ptr(aux, torch.int32, self.tokens, self.device)
            o = _ptr(out, torch.float32, 1, self.device)
        elif self.cfg.has_embedding:
            n_aux = self.tokens + (self.cfg.microbatch if self.cfg.block_kind == BLOCK_BERT else 0)
            a = _ptr(aux, torch.int32, n_aux, self.device)
            o = self._act(out)
        else:
            a = _ptr(aux, torch.int32, self.cfg.microbatch, self.device)
            o = self._act(out)
        _check(lib().amdp_stage_forward(self.handle, mb, version, self._act(X), a, o), "amdp_stage_forward")

    def amdp_stage_backward(self, mb, version, dY, dX):
        _check(lib().amdp_stage_backward(self.handle, mb, version, self._act(dY), self._act(dX)),
               "amdp_stage_backward")

    def amdp_grad_accumulate(self, mb):
        _check(lib().amdp_grad_accumulate(self.handle, mb), "amdp_grad_accumulate")

    def amdp_apply_update(self, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, grad_scale=1.0,
                          bias_correction=True):
        hp = amdp_adam_t(C.sizeof(amdp_adam_t), int(bool(bias_correction)), lr, beta1, beta2, eps,
                         weight_decay, grad_scale)
        nv = C.c_uint32(0)
        _check(lib().amdp_apply_update(self.handle, C.byref(hp), C.byref(nv)), "amdp_apply_update")
        return nv.value

    def amdp_stage_set_fused_accumulate(self, on):
        _check(lib().amdp_stage_set_fused_accumulate(self.handle, int(bool(on))), "amdp_stage_set_fused_accumulate")

    def amdp_stage_set_option(self, option, value):
        _check(lib().amdp_stage_set_option(self.handle, option, value), "amdp_stage_set_option")

    def amdp_stage_read_version(self, version, out):
        """out: tensor of the stage dtype with at least n_params (+1 if odd) elements."""
        need = self.n_params + (self.n_params & 1 if self.act_dtype == self.torch.bfloat16 else 0)
        _check(lib().amdp_stage_read_version(self.handle, version, _ptr(out, self.act_dtype, need, self.device)),
               "amdp_stage_read_version")

    def amdp_stage_join(self):
        _check(lib().amdp_stage_join(self.handle), "amdp_stage_join")

    def amdp_stage_set_overlap(self, on):
        _check(lib().amdp_stage_set_overlap(self.handle, int(bool(on))), "amdp_stage_set_overlap")

    def amdp_stage_get_overlap(self):
        on = C.c_int32(0)
        _check(lib().amdp_stage_get_overlap(self.handle, C.byref(on)), "amdp_stage_get_overlap")
        return bool(on.value)

    def amdp_stage_profile_begin(self):
        _check(lib().amdp_stage_profile_begin(self.handle), "amdp_stage_profile_begin")

    def amdp_stage_profile_end(self):
        """{name: dict(launches, ms, flops, bytes)}"""
        arr = (amdp_profile_entry_t * 64)()
        n = C.c_int32(0)
        _check(lib().amdp_stage_profile_end(self.handle, arr, 64, C.byref(n)), "amdp_stage_profile_end")
        return {arr[i].name.decode(): dict(launches=int(arr[i].launches), ms=arr[i].ms, flops=arr[i].flops,
                                           bytes=arr[i].bytes) for i in range(n.value)}
