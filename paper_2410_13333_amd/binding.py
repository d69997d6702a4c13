"""ctypes binding of the C ABI in include/mls.h: argument marshalling only.

PyTorch appears here for device memory and the stream handle; every step of the path runs in the HIP
kernels of libmls.so.  There is no fallback: a missing library raises."""
from __future__ import annotations

import ctypes as C
import os

MLS_BF16, MLS_FP32 = 0, 1
P_NAMES = {"gamma1": 0, "w_qkv": 1, "w_o": 2, "gamma2": 3, "w_gu": 4, "w_d": 5}
T_IDS = {"x": 0, "a": 1, "qkv": 2, "o": 3, "h": 4, "b": 5, "gu": 6, "z": 7, "lse": 8,
         "dy": 16, "dgu": 17, "dh": 18, "dqkv": 19}


class MlsError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"mls error {code}: {msg}")
        self.code = code


class MlsConfig(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("ffn", C.c_int32), ("seq", C.c_int32), ("micro_batch", C.c_int32), ("max_layers", C.c_int32),
                ("max_inflight", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32),
                ("recompute", C.c_int32)]


class MlsMemory(C.Structure):
    _fields_ = [("total_bytes", C.c_size_t), ("param_bytes", C.c_size_t), ("stash_bytes", C.c_size_t),
                ("workspace_bytes", C.c_size_t), ("param_bytes_per_layer", C.c_size_t),
                ("grad_bytes_per_layer", C.c_size_t), ("stash_bytes_per_layer_microbatch", C.c_size_t)]


class MlsEndsConfig(C.Structure):
    _fields_ = [("hidden", C.c_int32), ("vocab", C.c_int32), ("seq", C.c_int32), ("micro_batch", C.c_int32),
                ("max_inflight", C.c_int32), ("rms_eps", C.c_float), ("dtype", C.c_int32)]


class MlsAdamW(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float)]


PE_NAMES = {"embed": 0, "gamma_f": 1, "w_lm": 2}


def lib_path():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmls.so")


_lib = None


def lib():
    """Load libmls.so (built in-tree by `python -m paper_2410_13333_amd.build`)."""
    global _lib
    if _lib is None:
        p = lib_path()
        if not os.path.exists(p):
            raise ImportError(f"{p} is missing: build it with `python -m paper_2410_13333_amd.build`")
        L = C.CDLL(p)
        vp, i32, i64, u64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_size_t
        L.mls_stage_init.argtypes = [C.POINTER(MlsConfig), u64, vp, C.POINTER(vp)]
        L.mls_stage_forward.argtypes = [vp, vp, i32, vp]
        L.mls_stage_backward_ex.argtypes = [vp, vp, vp, i32, vp, i32]
        L.mls_stage_backward.argtypes = [vp, vp, vp, i32, vp]
        L.mls_stage_free.argtypes = [vp]
        L.mls_stage_free.restype = None
        L.mls_stage_grad_elems.argtypes = [vp]
        L.mls_stage_grad_elems.restype = sz
        L.mls_stage_param_layout.argtypes = [vp, i32, i32, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
        L.mls_stage_get_params.argtypes = [vp, vp]
        L.mls_stage_set_params.argtypes = [vp, vp]
        L.mls_stage_inflight.argtypes = [vp]
        L.mls_stage_reset.argtypes = [vp]
        L.mls_stage_debug_read.argtypes = [vp, i32, i32, i32, vp]
        L.mls_stage_timing.argtypes = [vp, i32]
        L.mls_stage_timing_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
        L.mls_stage_memory.argtypes = [C.POINTER(MlsConfig), C.POINTER(MlsMemory)]
        L.mls_gemm.argtypes = [i32, i32, vp, i64, vp, i64, vp, i64, vp, i64, i64, i64, vp]
        L.mls_last_error.restype = C.c_char_p
        L.mls_ends_init.argtypes = [C.POINTER(MlsEndsConfig), u64, vp, C.POINTER(vp)]
        L.mls_ends_free.argtypes = [vp]
        L.mls_ends_free.restype = None
        L.mls_embed_forward.argtypes = [vp, vp, vp]
        L.mls_embed_backward.argtypes = [vp, vp, vp, i32]
        L.mls_head_forward.argtypes = [vp, vp, vp, C.c_float, vp]
        L.mls_head_forward_static.argtypes = [vp, vp, vp, C.c_float, vp]
        L.mls_head_backward.argtypes = [vp, vp, i32, vp]
        L.mls_ends_grad_elems.argtypes = [vp]
        L.mls_ends_grad_elems.restype = sz
        L.mls_ends_param_layout.argtypes = [vp, i32, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
        L.mls_ends_get_params.argtypes = [vp, vp]
        L.mls_ends_set_params.argtypes = [vp, vp]
        L.mls_ends_inflight.argtypes = [vp, C.POINTER(i32), C.POINTER(i32)]
        L.mls_ends_debug_dlogits.argtypes = [vp, i32, vp]
        dp_, ip_ = C.POINTER(C.c_double), C.POINTER(i64)
        L.mls_optim_init.argtypes = [sz, vp, i32, vp, C.POINTER(vp)]
        L.mls_optim_free.argtypes = [vp]
        L.mls_optim_free.restype = None
        L.mls_optim_step.argtypes = [vp, vp, C.POINTER(MlsAdamW), C.c_float, vp]
        L.mls_optim_steps.argtypes = [vp]
        L.mls_optim_steps.restype = i64
        L.mls_optim_read.argtypes = [vp, i32, vp]
        L.mls_probe_init.argtypes = [C.c_double, C.c_double, vp, C.POINTER(vp)]
        L.mls_probe_free.argtypes = [vp]
        L.mls_probe_free.restype = None
        L.mls_probe_begin.argtypes = [vp]
        L.mls_probe_end.argtypes = [vp, i32, i32]
        L.mls_probe_read.argtypes = [vp, dp_, dp_, C.POINTER(i32)]
        L.mls_probe_feed.argtypes = [vp, C.c_double, i32, i32, dp_, C.POINTER(i32)]
        L.mls_plan_layers.argtypes = [dp_, ip_, i32, i64, ip_, dp_]
        L.mls_plan_microbatches.argtypes = [dp_, i32, i64, ip_, dp_]
        L.mls_plan_lower_level.argtypes = [dp_, ip_, C.POINTER(i32), i32, i64, i64, C.c_double, ip_, ip_, dp_]
        L.mls_plan_split_groups.argtypes = [dp_, i32, C.POINTER(i32), dp_, i32, C.POINTER(i32), dp_]
        L.mls_plan_layer_cap.argtypes = [C.c_double] * 4 + [i32, i32, C.c_double, C.c_double]
        L.mls_plan_layer_cap.restype = i64
        L.mls_grouping_time_ratio.argtypes = [dp_, i32, dp_, i32]
        L.mls_grouping_time_ratio.restype = C.c_double
        L.mls_theoretic_slowdown.argtypes = [i64, dp_, i32]
        L.mls_theoretic_slowdown.restype = C.c_double
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise MlsError(rc, lib().mls_last_error().decode())


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


def _torch_dtype(dtype):
    import torch
    return torch.bfloat16 if dtype == MLS_BF16 else torch.float32


class Stage:
    """One GPU's pipeline stage.  Tensors are torch CUDA tensors used as plain device buffers."""

    def __init__(self, hidden, n_q_heads, n_kv_heads, head_dim, ffn, seq, micro_batch, max_layers, max_inflight,
                 rms_eps=1e-5, rope_base=10000.0, dtype="bf16", seed=0, stream=None, recompute=False):
        import torch
        self.cfg = MlsConfig(hidden, n_q_heads, n_kv_heads, head_dim, ffn, seq, micro_batch, max_layers, max_inflight,
                             rms_eps, rope_base, MLS_BF16 if dtype == "bf16" else MLS_FP32, int(recompute))
        self.dtype = self.cfg.dtype
        self.tdtype = _torch_dtype(self.dtype)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = C.c_void_p(0)
        _check(lib().mls_stage_init(C.byref(self.cfg), seed, C.c_void_p(self.stream.cuda_stream), C.byref(self._h)))

    @classmethod
    def from_shape(cls, sh, seed=0, max_layers=None, max_inflight=None, stream=None, recompute=False):
        """sh: any object with the StageShape fields (hidden, n_q_heads, ..., layers, microbatches, dtype)."""
        return cls(sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.ffn, sh.seq, sh.micro_batch,
                   sh.layers if max_layers is None else max_layers,
                   sh.microbatches if max_inflight is None else max_inflight,
                   sh.rms_eps, sh.rope_base, sh.dtype, seed, stream, recompute)

    @staticmethod
    def memory(sh, max_layers=None, max_inflight=None, recompute=False):
        """Device bytes a stage of this shape allocates (mls_stage_memory); no GPU needed."""
        cfg = MlsConfig(sh.hidden, sh.n_q_heads, sh.n_kv_heads, sh.head_dim, sh.ffn, sh.seq, sh.micro_batch,
                        sh.layers if max_layers is None else max_layers,
                        sh.microbatches if max_inflight is None else max_inflight, sh.rms_eps, sh.rope_base,
                        MLS_BF16 if sh.dtype == "bf16" else MLS_FP32, int(recompute))
        m = MlsMemory()
        _check(lib().mls_stage_memory(C.byref(cfg), C.byref(m)))
        return {k: getattr(m, k) for k, _ in MlsMemory._fields_}

    # ---- hot path
    def forward(self, x, k_layers, y):
        _check(lib().mls_stage_forward(self._h, _ptr(x), k_layers, _ptr(y)))

    def backward(self, dy, grads, n_microbatches, dx, overwrite=False):
        """overwrite=True: grads is written instead of added to (MLS_BWD_OVERWRITE)."""
        if overwrite:
            _check(lib().mls_stage_backward_ex(self._h, _ptr(dy), _ptr(grads), n_microbatches, _ptr(dx), 1))
        else:
            _check(lib().mls_stage_backward(self._h, _ptr(dy), _ptr(grads), n_microbatches, _ptr(dx)))

    # ---- support
    @property
    def grad_elems(self):
        return lib().mls_stage_grad_elems(self._h)

    @property
    def inflight(self):
        return lib().mls_stage_inflight(self._h)

    def reset(self):
        _check(lib().mls_stage_reset(self._h))

    def param_layout(self, layer, which):
        off, r, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
        which = P_NAMES[which] if isinstance(which, str) else which
        _check(lib().mls_stage_param_layout(self._h, layer, which, C.byref(off), C.byref(r), C.byref(c)))
        return off.value, r.value, c.value

    def get_params(self):
        import torch
        out = torch.empty(self.grad_elems, dtype=self.tdtype, device="cuda")
        _check(lib().mls_stage_get_params(self._h, _ptr(out)))
        return out

    def set_params(self, src):
        assert src.is_cuda and src.dtype == self.tdtype and src.numel() == self.grad_elems and src.is_contiguous()
        _check(lib().mls_stage_set_params(self._h, _ptr(src)))

    def debug_read(self, name, layer=0, slot=0):
        import torch
        c = self.cfg
        T, qd, kvd = c.seq * c.micro_batch, c.n_q_heads * c.head_dim, c.n_kv_heads * c.head_dim
        shapes = {"x": (T, c.hidden), "a": (T, c.hidden), "qkv": (T, qd + 2 * kvd), "o": (T, qd), "h": (T, c.hidden),
                  "b": (T, c.hidden), "gu": (T, 2 * c.ffn), "z": (T, c.ffn), "lse": (c.micro_batch, c.n_q_heads, c.seq),
                  "dy": (T, c.hidden), "dgu": (T, 2 * c.ffn), "dh": (T, c.hidden), "dqkv": (T, qd + 2 * kvd)}
        out = torch.empty(shapes[name], dtype=torch.float32 if name == "lse" else self.tdtype, device="cuda")
        _check(lib().mls_stage_debug_read(self._h, T_IDS[name], layer, slot, _ptr(out)))
        return out

    TIMING_CLASSES = ("gemm_fwd", "gemm_dgrad", "gemm_wgrad", "attn_fwd", "attn_bwd", "rmsnorm", "rope", "swiglu")

    def timing(self, enable):
        _check(lib().mls_stage_timing(self._h, 1 if enable else 0))

    def timing_read(self):
        """{class: (milliseconds, launches)} accumulated since the last read."""
        n = len(self.TIMING_CLASSES)
        ms, cnt = (C.c_double * n)(), (C.c_int64 * n)()
        _check(lib().mls_stage_timing_read(self._h, ms, cnt))
        return {k: (ms[i], cnt[i]) for i, k in enumerate(self.TIMING_CLASSES)}

    def close(self):
        if self._h:
            lib().mls_stage_free(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gemm(mode, a, b, c, r=None, stream=None):
    """Stand-alone call of the stage's contraction kernel; shapes as documented at mls_gemm.  Operands may be
    column slices of wider row-major buffers (row stride = stride(0))."""
    import torch
    dtype = MLS_BF16 if a.dtype == torch.bfloat16 else MLS_FP32
    if mode == 0:
        (M, K), N = a.shape, b.shape[1]
    elif mode == 1:
        (M, K), N = a.shape, b.shape[0]
    else:
        (K, M), N = a.shape, b.shape[1]
    for t in (a, b, c) + ((r,) if r is not None else ()):
        assert t.stride(1) == 1
    assert r is None or r.stride(0) == c.stride(0)
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(lib().mls_gemm(dtype, mode, _ptr(a), a.stride(0), _ptr(b), b.stride(0), _ptr(c), c.stride(0), _ptr(r),
                          M, N, K, C.c_void_p(st.cuda_stream)))


# ---- include/mls_ends.h: the non-uniform layers of the first and the last pipeline stage
class Ends:
    """Token embedding (first stage) and final norm + LM head + loss (last stage); tensors are torch CUDA tensors."""

    def __init__(self, hidden, vocab, seq, micro_batch, max_inflight, rms_eps=1e-5, dtype="bf16", seed=0, stream=None):
        import torch
        self.cfg = MlsEndsConfig(hidden, vocab, seq, micro_batch, max_inflight, rms_eps,
                                 MLS_BF16 if dtype == "bf16" else MLS_FP32)
        self.dtype = self.cfg.dtype
        self.tdtype = _torch_dtype(self.dtype)
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = C.c_void_p(0)
        _check(lib().mls_ends_init(C.byref(self.cfg), seed, C.c_void_p(self.stream.cuda_stream), C.byref(self._h)))

    @classmethod
    def from_shape(cls, sh, seed=0, max_inflight=None, stream=None):
        return cls(sh.hidden, sh.vocab, sh.seq, sh.micro_batch, sh.microbatches if max_inflight is None else max_inflight,
                   sh.rms_eps, sh.dtype, seed, stream)

    def embed_forward(self, tokens, x):
        _check(lib().mls_embed_forward(self._h, _ptr(tokens), _ptr(x)))

    def embed_backward(self, dx, grads, n):
        _check(lib().mls_embed_backward(self._h, _ptr(dx), _ptr(grads), n))

    def head_forward(self, y, targets, loss_weight, loss):
        _check(lib().mls_head_forward(self._h, _ptr(y), _ptr(targets), loss_weight, _ptr(loss)))

    def head_forward_static(self, y, targets, loss_weight, loss):
        _check(lib().mls_head_forward_static(self._h, _ptr(y), _ptr(targets), loss_weight, _ptr(loss)))

    def head_backward(self, grads, n, dy):
        _check(lib().mls_head_backward(self._h, _ptr(grads), n, _ptr(dy)))

    @property
    def grad_elems(self):
        return lib().mls_ends_grad_elems(self._h)

    @property
    def inflight(self):
        a, b = C.c_int32(), C.c_int32()
        _check(lib().mls_ends_inflight(self._h, C.byref(a), C.byref(b)))
        return a.value, b.value

    def param_layout(self, which):
        off, r, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
        _check(lib().mls_ends_param_layout(self._h, PE_NAMES[which] if isinstance(which, str) else which, C.byref(off),
                                           C.byref(r), C.byref(c)))
        return off.value, r.value, c.value

    def get_params(self):
        import torch
        out = torch.empty(self.grad_elems, dtype=self.tdtype, device="cuda")
        _check(lib().mls_ends_get_params(self._h, _ptr(out)))
        return out

    def set_params(self, src):
        assert src.is_cuda and src.dtype == self.tdtype and src.numel() == self.grad_elems and src.is_contiguous()
        _check(lib().mls_ends_set_params(self._h, _ptr(src)))

    def debug_dlogits(self, slot=0):
        import torch
        out = torch.empty((self.cfg.seq * self.cfg.micro_batch, self.cfg.vocab), dtype=self.tdtype, device="cuda")
        _check(lib().mls_ends_debug_dlogits(self._h, slot, _ptr(out)))
        return out

    def close(self):
        if self._h:
            lib().mls_ends_free(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- include/mls_optim.h: optimizer step and straggling-rate probe
class Optim:
    """AdamW on fp32 master weights for a flat parameter vector (a stage's or the first/last-stage layers')."""

    def __init__(self, params, stream=None):
        import torch
        self.n = params.numel()
        self.tdtype = params.dtype
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        self._h = C.c_void_p(0)
        _check(lib().mls_optim_init(self.n, _ptr(params), MLS_BF16 if params.dtype == torch.bfloat16 else MLS_FP32,
                                    C.c_void_p(self.stream.cuda_stream), C.byref(self._h)))

    def step(self, grads, params_out, lr, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, grad_scale=1.0):
        hp = MlsAdamW(lr, beta1, beta2, eps, weight_decay)
        _check(lib().mls_optim_step(self._h, _ptr(grads), C.byref(hp), grad_scale, _ptr(params_out)))

    @property
    def steps(self):
        return lib().mls_optim_steps(self._h)

    def read(self, which):
        import torch
        out = torch.empty(self.n, dtype=torch.float32, device="cuda")
        _check(lib().mls_optim_read(self._h, {"w": 0, "m": 1, "v": 2}[which], _ptr(out)))
        return out

    def close(self):
        if self._h:
            lib().mls_optim_free(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Probe:
    """Straggling-rate probe: brackets steps with HIP events (begin/end/read) or replays elapsed times (feed)."""

    def __init__(self, tau_ref_ms, threshold=0.05, stream_handle=0):
        self._h = C.c_void_p(0)
        _check(lib().mls_probe_init(tau_ref_ms, threshold, C.c_void_p(stream_handle), C.byref(self._h)))

    def begin(self):
        _check(lib().mls_probe_begin(self._h))

    def end(self, layers, microbatches):
        _check(lib().mls_probe_end(self._h, layers, microbatches))

    def read(self):
        r, t, s = C.c_double(), C.c_double(), C.c_int32()
        _check(lib().mls_probe_read(self._h, C.byref(r), C.byref(t), C.byref(s)))
        return r.value, t.value, bool(s.value)

    def feed(self, elapsed_ms, layers, microbatches):
        r, s = C.c_double(), C.c_int32()
        _check(lib().mls_probe_feed(self._h, elapsed_ms, layers, microbatches, C.byref(r), C.byref(s)))
        return r.value, bool(s.value)

    def close(self):
        if self._h:
            lib().mls_probe_free(self._h)
            self._h = C.c_void_p(0)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- include/mls_plan.h: the planner's lower level (host arrays in, host arrays out)
def _darr(v):
    return (C.c_double * len(v))(*[float(x) for x in v])


def _caps(cap, n):
    if cap is None:
        return None
    assert len(cap) == n
    return (C.c_int64 * n)(*[-1 if c is None else int(c) for c in cap])


def plan_layers(y, L, cap=None):
    """Eq. 2: returns (layers per stage, optimal bottleneck max_j y_j l_j)."""
    n = len(y)
    out, o = (C.c_int64 * n)(), C.c_double()
    _check(lib().mls_plan_layers(_darr(y), _caps(cap, n), n, int(L), out, C.byref(o)))
    return list(out), o.value


def plan_microbatches(o, n_mb):
    """Eq. 3: returns (micro-batches per pipeline, optimal max_i o_i m_i)."""
    n = len(o)
    out, t = (C.c_int64 * n)(), C.c_double()
    _check(lib().mls_plan_microbatches(_darr(o), n, int(n_mb), out, C.byref(t)))
    return list(out), t.value


def plan_lower_level(pipelines, L, n_mb, tau, caps=None):
    """Eq. 1 for fixed pipelines (list of lists of stage rates): returns (layers per pipeline per stage,
    micro-batches per pipeline, estimated step time)."""
    pp = [len(p) for p in pipelines]
    flat = [y for p in pipelines for y in p]
    fcap = None if caps is None else [c for p in caps for c in p]
    l, m, t = (C.c_int64 * len(flat))(), (C.c_int64 * len(pp))(), C.c_double()
    _check(lib().mls_plan_lower_level(_darr(flat), _caps(fcap, len(flat)), (C.c_int32 * len(pp))(*pp), len(pp), int(L),
                                      int(n_mb), float(tau), l, m, C.byref(t)))
    ls, at = [], 0
    for k in pp:
        ls.append(list(l[at:at + k]))
        at += k
    return ls, list(m), t.value


def plan_layer_cap(a_f, a_fb, s, nu, pp, j, capacity, reserve=0.0):
    """Appendix B.4: most layers stage j of pp can hold under the linear memory model."""
    return lib().mls_plan_layer_cap(a_f, a_fb, s, nu, pp, j, capacity, reserve)


def plan_split_groups(x, sizes, rho):
    """Appendix B.7: best consecutive-run grouping of GPUs with rates x into groups of the given sizes; returns
    (group index per GPU, sum of 1/y)."""
    n, k = len(x), len(sizes)
    out, s = (C.c_int32 * n)(), C.c_double()
    _check(lib().mls_plan_split_groups(_darr(x), n, (C.c_int32 * k)(*sizes), _darr(rho), k, out, C.byref(s)))
    return list(out), s.value


def grouping_time_ratio(y1, y2):
    """Theorem 2: T'/T'' of two groupings under the relaxed problem."""
    return lib().mls_grouping_time_ratio(_darr(y1), len(y1), _darr(y2), len(y2))


def theoretic_slowdown(n_gpus, x):
    """Sec. 7.2: best possible step-time ratio with stragglers of rates x among n_gpus GPUs."""
    return lib().mls_theoretic_slowdown(int(n_gpus), _darr(x) if len(x) else None, len(x))
