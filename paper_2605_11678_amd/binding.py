"""ctypes binding of include/demand_layering.h: same names, argument marshalling only.

Every step of the path runs inside the native library; nothing here computes.  The
library must be built (``python -m paper_2605_11678_amd.build``); loading fails loudly
otherwise.  torch is imported first so that the library binds to the same HIP runtime
that owns the caller's streams and device memory.
"""
import ctypes as C
import os

try:  # the HIP runtime bundled with torch must be the one in the process
    import torch  # noqa: F401
except Exception:  # pragma: no cover - host-only use without torch
    torch = None

from . import build as _build

DL_OK, DL_ERR_INVALID_ARG, DL_ERR_BUDGET_EXCEEDED, DL_ERR_HOST_ALLOC, DL_ERR_DEVICE, DL_ERR_BAD_STATE = 0, -1, -2, -3, -4, -5
DL_NORM_RMS, DL_NORM_LN = 0, 1
DL_ACT_SWIGLU, DL_ACT_GELU = 0, 1
DL_MODE_PIPELINED, DL_MODE_SEQUENTIAL = 0, 1
DL_OP_WAIT, DL_OP_RECORD, DL_OP_COPY, DL_OP_EXEC = 0, 1, 2, 3
DL_EV_DMA_DONE, DL_EV_COMPUTE_DONE, DL_EV_PASS_DONE = 0, 1, 2
DL_OPF_NEXT_PASS = 1
DL_T_COUNT, DL_R_COUNT = 27, 4
DL_R_EMBED, DL_R_HEAD, DL_R_FINAL_NORM_G, DL_R_FINAL_NORM_B = 0, 1, 2, 3


class dl_module_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_layers", "d_model", "n_q_heads", "n_kv_heads", "d_head", "d_ff", "norm", "act", "has_bias", "causal",
        "d_ctx", "max_seq", "max_tokens", "max_ctx", "vocab")] + [("rope_theta", C.c_float), ("norm_eps", C.c_float)]


class dl_layer_profile(C.Structure):
    _fields_ = [("c_dma_ms", C.c_double), ("c_dma_cont_ms", C.c_double), ("c_exe_ms", C.c_double), ("c_exe_hot_ms", C.c_double), ("c_exe_loaded_ms", C.c_double),
                ("c_fence_ms", C.c_double), ("c_fence_hot_ms", C.c_double), ("bytes", C.c_uint64)]


class dl_run_stats(C.Structure):
    _fields_ = [("total_ms", C.c_double), ("dma_ms", C.c_double), ("exe_ms", C.c_double), ("exposed_ms", C.c_double),
                ("hidden_frac", C.c_double), ("h2d_gbps", C.c_double), ("bytes_streamed", C.c_uint64),
                ("arena_peak", C.c_uint64), ("n_layer_records", C.c_int32)]


class dl_layer_record(C.Structure):
    _fields_ = [("module", C.c_int32), ("layer", C.c_int32), ("streamed", C.c_int32), ("slot", C.c_int32),
                ("dma_start_ms", C.c_float), ("dma_end_ms", C.c_float), ("exe_start_ms", C.c_float),
                ("exe_end_ms", C.c_float)]


class dl_kernel_time(C.Structure):
    _fields_ = [("kind", C.c_int32), ("launches", C.c_int32), ("total_ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


DL_K_NAMES = ["norm", "gemm_qkv", "qkv_post", "attn", "gemm_o", "gemm_up", "gemm_down", "cross"]


class dl_trace_op(C.Structure):
    _fields_ = [("queue", C.c_int32), ("op", C.c_int32), ("event_kind", C.c_int32), ("slot", C.c_int32),
                ("module", C.c_int32), ("layer", C.c_int32), ("flags", C.c_int32)]


class dl_vla_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "m_vit", "m_dec", "m_act", "mlp_proj", "mlp_out", "n_patches", "pool", "n_text", "n_actions", "n_decode",
        "n_euler", "out_dim")]


class dl_vla_buffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in (
        "patches", "vit_out", "proj_out", "seq", "hidden", "hidden_ctx", "x1", "y1", "tokens", "actions", "act_in",
        "velocity", "trajectory")]


_p = C.c_void_p
_i32, _u64, _f64 = C.c_int32, C.c_uint64, C.c_double
_PI32, _PU64, _PF64 = C.POINTER(C.c_int32), C.POINTER(C.c_uint64), C.POINTER(C.c_double)

# name -> (restype, argtypes): one entry per declaration of the header
SIGNATURES = {
    "dl_create": (_i32, [C.POINTER(_p), _i32]),
    "dl_destroy": (_i32, [_p]),
    "dl_last_error": (C.c_char_p, [_p]),
    "dl_set_arena": (_i32, [_p, _p, _u64]),
    "dl_arena_alloc": (_i32, [_p, _u64, C.POINTER(_p)]),
    "dl_arena_free": (_i32, [_p, _p]),
    "dl_arena_stats": (_i32, [_p, _PU64, _PU64, _PU64]),
    "dl_residency_budget": (_i32, [_p, _PU64]),
    "dl_greedy_step_static": (_i32, [_i32, _p, _p, _p, _p, _p, _p, _i32, C.c_float, _i32, _i32, _p, _p]),
    "dl_set_streams": (_i32, [_p, _p, _p]),
    "dl_module_create": (_i32, [_p, C.POINTER(dl_module_desc), _PI32]),
    "dl_layer_set_tensor": (_i32, [_p, _i32, _i32, _i32, _p, _u64]),
    "dl_set_resident_tensor": (_i32, [_p, _i32, _i32, _p, _u64]),
    "dl_module_finalize": (_i32, [_p, _i32]),
    "dl_module_layer_bytes": (_i32, [_p, _i32, _PU64, _PU64]),
    "dl_set_residency": (_i32, [_p, _i32, _PI32, _i32]),
    "dl_get_residency": (_i32, [_p, _i32, _PI32, _PI32]),
    "dl_set_mode": (_i32, [_p, _i32, _i32]),
    "dl_forward": (_i32, [_p, _i32, _p, _p, _i32, _i32, _p, _i32]),
    "dl_embed_token": (_i32, [_p, _i32, _i32, _p]),
    "dl_final_norm": (_i32, [_p, _i32, _p, _p, _i32]),
    "dl_logits_argmax": (_i32, [_p, _i32, _p, _PI32, C.POINTER(C.c_float)]),
    "dl_greedy_step": (_i32, [_p, _i32, _p, _p, _p]),
    "dl_sync": (_i32, [_p]),
    "dl_vla_infer": (_i32, [_p, C.POINTER(dl_vla_desc), C.POINTER(dl_vla_buffers)]),
    "dl_mlp_create": (_i32, [_p, _i32, _i32, _i32, _p, _p, _p, _p, _i32, _PI32]),
    "dl_mlp_forward": (_i32, [_p, _i32, _p, _p, _i32]),
    "dl_mean_pool": (_i32, [_p, _p, _p, _i32, _i32, _i32]),
    "dl_axpy": (_i32, [_p, _p, C.c_float, _p, _u64]),
    "dl_add_time_embedding": (_i32, [_p, _p, _p, C.c_float, _i32, _i32]),
    "dl_profile": (_i32, [_p, _i32, _i32, _i32, _p, _p, _i32, _i32, C.POINTER(dl_layer_profile)]),
    "dl_set_timing": (_i32, [_p, _i32]),
    "dl_collect_stats": (_i32, [_p, C.POINTER(dl_run_stats), C.POINTER(dl_layer_record), _i32]),
    "dl_set_kernel_timing": (_i32, [_p, _i32]),
    "dl_set_run_ahead": (_i32, [_p, _i32]),
    "dl_probe_mfma_rate": (_i32, [_p, _i32, _i32, C.POINTER(C.c_double)]),
    "dl_collect_kernel_times": (_i32, [_p, C.POINTER(dl_kernel_time)]),
    "dl_trace_enable": (_i32, [_p, _i32]),
    "dl_trace_read": (_i32, [_p, C.POINTER(dl_trace_op), _i32, _PI32]),
    "dl_place_interleaved": (_i32, [_i32, _i32, _PI32]),
    "dl_benefit": (_i32, [_f64, _f64, _i32, _PF64, _PI32, _PF64]),
    "dl_consecutive_limit": (_i32, [_f64, _f64, _PI32]),
    "dl_predict_linear": (_i32, [_f64, _f64, _i32, _PF64]),
    "dl_timeline": (_i32, [_PF64, _PF64, _PF64, _PF64, _PF64, _PF64, _PF64, C.POINTER(C.c_uint8), C.POINTER(C.c_uint8), _PI32, _i32, _i32, _i32,
                           _i32, _f64, _PF64, _PF64, _PF64]),
    "dl_set_slot_count": (_i32, [_p, _i32]),
    "dl_module_set_max_tokens": (_i32, [_p, _i32, _i32]),
    "dl_plan": (_i32, [_i32, _PI32, _PU64, _PF64, _u64, _PI32]),
    "dl_plan_shared_slots": (_i32, [_i32, _PI32, _PU64, _PF64, _u64, _i32, _PI32]),
}

_LIB = None


def lib():
    """The loaded C-ABI library (raises if it has not been built)."""
    global _LIB
    if _LIB is None:
        path = _build.LIB_PATH
        if not os.path.exists(path):
            raise RuntimeError(
                "native library missing: %s — build it with `python -m paper_2605_11678_amd.build`" % path)
        L = C.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _LIB = L
    return _LIB


class DLError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("demand_layering error %d: %s" % (code, msg))
        self.code = code


def _arr(ctype, values):
    values = list(values)
    return (ctype * max(len(values), 1))(*values)


class Context:
    """Owns one dl_ctx; methods carry the C function names without the dl_ prefix."""

    def __init__(self, device=0):
        self._h = _p()
        rc = lib().dl_create(C.byref(self._h), device)
        if rc != DL_OK:
            raise DLError(rc, "dl_create failed (device %d)" % device)
        self.device = device
        self._keep = []     # tensors whose memory the library uses (arena, streams)

    def _ck(self, rc):
        if rc != DL_OK:
            raise DLError(rc, lib().dl_last_error(self._h).decode())

    def destroy(self):
        if self._h:
            lib().dl_destroy(self._h)
            self._h = _p()
            self._keep = []

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # ---- setup ----
    def set_arena(self, dev_ptr, nbytes, keep=None):
        self._ck(lib().dl_set_arena(self._h, _p(dev_ptr), nbytes))
        if keep is not None:
            self._keep.append(keep)

    def arena_alloc(self, nbytes):
        out = _p()
        self._ck(lib().dl_arena_alloc(self._h, nbytes, C.byref(out)))
        return out.value

    def arena_free(self, ptr):
        self._ck(lib().dl_arena_free(self._h, _p(ptr)))

    def arena_stats(self):
        u, pk, cp = _u64(), _u64(), _u64()
        self._ck(lib().dl_arena_stats(self._h, C.byref(u), C.byref(pk), C.byref(cp)))
        return dict(used=u.value, peak=pk.value, capacity=cp.value)

    def residency_budget(self):
        b = _u64()
        self._ck(lib().dl_residency_budget(self._h, C.byref(b)))
        return b.value

    def set_streams(self, compute_stream, copy_stream, keep=None):
        self._ck(lib().dl_set_streams(self._h, _p(compute_stream), _p(copy_stream)))
        if keep is not None:
            self._keep.append(keep)

    def module_create(self, **fields):
        d = dl_module_desc()
        known = {n for n, _ in dl_module_desc._fields_}
        for k, v in fields.items():
            if k in known:
                setattr(d, k, v)
        mid = _i32()
        self._ck(lib().dl_module_create(self._h, C.byref(d), C.byref(mid)))
        return mid.value

    def layer_set_tensor(self, module, layer, tensor_id, host_u16):
        assert host_u16.dtype.name == "uint16" and host_u16.flags.c_contiguous
        self._ck(lib().dl_layer_set_tensor(self._h, module, layer, tensor_id, _p(host_u16.ctypes.data), host_u16.size))

    def set_resident_tensor(self, module, which, host_u16):
        assert host_u16.dtype.name == "uint16" and host_u16.flags.c_contiguous
        self._ck(lib().dl_set_resident_tensor(self._h, module, which, _p(host_u16.ctypes.data), host_u16.size))

    def module_finalize(self, module):
        self._ck(lib().dl_module_finalize(self._h, module))

    def module_layer_bytes(self, module):
        a, b = _u64(), _u64()
        self._ck(lib().dl_module_layer_bytes(self._h, module, C.byref(a), C.byref(b)))
        return a.value, b.value

    def set_residency(self, module, layer_idx):
        idx = _arr(_i32, layer_idx)
        self._ck(lib().dl_set_residency(self._h, module, idx, len(list(layer_idx))))

    def get_residency(self, module, n_layers):
        idx = (_i32 * max(n_layers, 1))()
        n = _i32()
        self._ck(lib().dl_get_residency(self._h, module, idx, C.byref(n)))
        return list(idx[:n.value])

    def set_mode(self, mode, wrap_prefetch):
        self._ck(lib().dl_set_mode(self._h, mode, int(wrap_prefetch)))

    # ---- hot path ----
    def forward(self, module, x_ptr, y_ptr, n_tokens, pos0=0, ctx_ptr=None, n_ctx=0):
        self._ck(lib().dl_forward(self._h, module, _p(x_ptr), _p(y_ptr), n_tokens, pos0, _p(ctx_ptr), n_ctx))

    def embed_token(self, module, token, x_ptr):
        self._ck(lib().dl_embed_token(self._h, module, token, _p(x_ptr)))

    def final_norm(self, module, h_ptr, out_ptr, n_tokens):
        self._ck(lib().dl_final_norm(self._h, module, _p(h_ptr), _p(out_ptr), n_tokens))

    def logits_argmax(self, module, h_ptr, logits_out=None):
        tok = _i32()
        lp = None
        if logits_out is not None:
            assert logits_out.dtype.name == "float32" and logits_out.flags.c_contiguous
            lp = logits_out.ctypes.data_as(C.POINTER(C.c_float))
        self._ck(lib().dl_logits_argmax(self._h, module, _p(h_ptr), C.byref(tok), lp))
        return tok.value

    def greedy_step(self, module, h_ptr, token_dev_ptr, x_ptr):
        self._ck(lib().dl_greedy_step(self._h, module, _p(h_ptr), _p(token_dev_ptr), _p(x_ptr)))

    def sync(self):
        self._ck(lib().dl_sync(self._h))

    def vla_infer(self, desc: dict, buffers: dict):
        """desc / buffers: the fields of dl_vla_desc / dl_vla_buffers by name (buffers as device addresses)."""
        d = dl_vla_desc(**{k: int(v) for k, v in desc.items()})
        b = dl_vla_buffers(**{k: (int(v) if v else None) for k, v in buffers.items()})
        self._ck(lib().dl_vla_infer(self._h, C.byref(d), C.byref(b)))

    def mlp_create(self, d_in, d_hidden, d_out, w1, b1, w2, b2, max_tokens):
        def ptr(a):
            if a is None:
                return None
            assert a.dtype.name == "uint16" and a.flags.c_contiguous
            return _p(a.ctypes.data)
        out = _i32()
        self._ck(lib().dl_mlp_create(self._h, d_in, d_hidden, d_out, ptr(w1), ptr(b1), ptr(w2), ptr(b2), max_tokens,
                                     C.byref(out)))
        return out.value

    def mlp_forward(self, mlp, x_ptr, y_ptr, n_tokens):
        self._ck(lib().dl_mlp_forward(self._h, mlp, _p(x_ptr), _p(y_ptr), n_tokens))

    def mean_pool(self, x_ptr, y_ptr, n_out, group, d):
        self._ck(lib().dl_mean_pool(self._h, _p(x_ptr), _p(y_ptr), n_out, group, d))

    def axpy(self, y_ptr, alpha, x_ptr, n):
        self._ck(lib().dl_axpy(self._h, _p(y_ptr), alpha, _p(x_ptr), n))

    def add_time_embedding(self, x_ptr, y_ptr, t_value, n_tokens, d):
        self._ck(lib().dl_add_time_embedding(self._h, _p(x_ptr), _p(y_ptr), t_value, n_tokens, d))

    # ---- measurement ----
    def profile(self, module, n_layers, n_tokens, pos0, x_ptr, iters=4, ctx_ptr=None, n_ctx=0):
        out = (dl_layer_profile * n_layers)()
        self._ck(lib().dl_profile(self._h, module, n_tokens, pos0, _p(x_ptr), _p(ctx_ptr), n_ctx, iters, out))
        return [dict(c_dma_ms=o.c_dma_ms, c_dma_cont_ms=o.c_dma_cont_ms, c_exe_ms=o.c_exe_ms, c_exe_hot_ms=o.c_exe_hot_ms, c_exe_loaded_ms=o.c_exe_loaded_ms, c_fence_ms=o.c_fence_ms, c_fence_hot_ms=o.c_fence_hot_ms,
                     bytes=o.bytes) for o in out]

    def set_timing(self, on):
        self._ck(lib().dl_set_timing(self._h, int(on)))

    def collect_stats(self, max_records=0):
        st = dl_run_stats()
        recs = (dl_layer_record * max(max_records, 1))()
        self._ck(lib().dl_collect_stats(self._h, C.byref(st), recs if max_records else None, max_records))
        d = {n: getattr(st, n) for n, _ in dl_run_stats._fields_}
        n = min(st.n_layer_records, max_records)
        d["records"] = [{f: getattr(recs[i], f) for f, _ in dl_layer_record._fields_} for i in range(n)]
        return d

    def set_kernel_timing(self, on, kinds=None):
        """on False: off.  on True: every kernel class, or only the DL_K_* ids listed in `kinds`."""
        mask = 0
        if on:
            mask = -1 if kinds is None else sum(1 << int(k) for k in kinds)
        self._ck(lib().dl_set_kernel_timing(self._h, mask))

    def set_run_ahead(self, passes):
        self._ck(lib().dl_set_run_ahead(self._h, int(passes)))

    def set_slot_count(self, n_slots):
        """1 or 2 device slots for the streamed layers (re-sizes them)."""
        self._ck(lib().dl_set_slot_count(self._h, int(n_slots)))

    def module_set_max_tokens(self, module, max_tokens):
        """Re-size a module's activation workspace for passes of at most max_tokens tokens (contents discarded)."""
        self._ck(lib().dl_module_set_max_tokens(self._h, int(module), int(max_tokens)))

    def probe_mfma_rate(self, pattern=1, iters=20000):
        """Register-only BF16 MFMA rate of the device in TFLOP/s (diagnostic)."""
        out = C.c_double(0.0)
        self._ck(lib().dl_probe_mfma_rate(self._h, int(pattern), int(iters), C.byref(out)))
        return out.value

    def collect_kernel_times(self):
        out = (dl_kernel_time * len(DL_K_NAMES))()
        self._ck(lib().dl_collect_kernel_times(self._h, out))
        return {DL_K_NAMES[o.kind]: dict(launches=o.launches, total_ms=o.total_ms, flops=o.flops, bytes=o.bytes)
                for o in out}

    def trace_enable(self, on):
        self._ck(lib().dl_trace_enable(self._h, int(on)))

    def trace_read(self, cap=1 << 16):
        ops = (dl_trace_op * cap)()
        n = _i32()
        self._ck(lib().dl_trace_read(self._h, ops, cap, C.byref(n)))
        if n.value > cap:
            raise DLError(DL_ERR_INVALID_ARG, "trace longer than the read buffer")
        return [{f: getattr(ops[i], f) for f, _ in dl_trace_op._fields_} for i in range(n.value)]


# ---- pure host functions (no context) ----
def greedy_step_static(device, stream, h_ptr, head_ptr, embed_ptr, norm_g_ptr, norm_b_ptr, norm, norm_eps, d_model, vocab,
                       token_dev_ptr, x_ptr):
    """dl_greedy_step_static: the greedy head on plain device pointers; allocates nothing."""
    rc = lib().dl_greedy_step_static(int(device), _p(stream), _p(h_ptr), _p(head_ptr), _p(embed_ptr), _p(norm_g_ptr),
                                     _p(norm_b_ptr), int(norm), float(norm_eps), int(d_model), int(vocab),
                                     _p(token_dev_ptr), _p(x_ptr))
    if rc != DL_OK:
        raise DLError(rc, lib().dl_last_error(None).decode())


def place_interleaved(n_layers, k):
    out = (_i32 * max(k, 1))()
    rc = lib().dl_place_interleaved(n_layers, k, out)
    if rc != DL_OK:
        raise DLError(rc, "dl_place_interleaved: invalid argument")
    return list(out[:k])


def benefit(c_dma_ms, m_mib, c_exe_ms, reps):
    n = len(c_exe_ms)
    out = (_f64 * 3)()
    rc = lib().dl_benefit(c_dma_ms, m_mib, n, _arr(_f64, c_exe_ms), _arr(_i32, reps), out)
    if rc != DL_OK:
        raise DLError(rc, "dl_benefit: invalid argument")
    return tuple(out)


def consecutive_limit(c_dma_ms, c_exe_ms):
    out = _i32()
    rc = lib().dl_consecutive_limit(c_dma_ms, c_exe_ms, C.byref(out))
    if rc != DL_OK:
        raise DLError(rc, "dl_consecutive_limit: invalid argument")
    return out.value


def predict_linear(c_total0_ms, slope_ms_per_layer, k):
    out = _f64()
    rc = lib().dl_predict_linear(c_total0_ms, slope_ms_per_layer, k, C.byref(out))
    if rc != DL_OK:
        raise DLError(rc, "dl_predict_linear: invalid argument")
    return out.value


def timeline(c_dma_ms, c_exe_ms, streamed, pass_start, module_id=None, mode=DL_MODE_PIPELINED, wrap_prefetch=0,
             overhead_ms=0.0, c_exe_idle_ms=None, c_fence_ms=None, n_slots=2, c_dma_cont_ms=None, c_fence_hot_ms=None, c_exe_loaded_ms=None):
    n = len(c_dma_ms)
    tot, hid, exp_ = _f64(), _f64(), _f64()
    rc = lib().dl_timeline(_arr(_f64, c_dma_ms), None if c_dma_cont_ms is None else _arr(_f64, c_dma_cont_ms),
                           _arr(_f64, c_exe_ms),
                           None if c_exe_idle_ms is None else _arr(_f64, c_exe_idle_ms),
                           None if c_exe_loaded_ms is None else _arr(_f64, c_exe_loaded_ms),
                           None if c_fence_ms is None else _arr(_f64, c_fence_ms),
                           None if c_fence_hot_ms is None else _arr(_f64, c_fence_hot_ms),
                           _arr(C.c_uint8, [1 if s else 0 for s in streamed]),
                           _arr(C.c_uint8, [1 if s else 0 for s in pass_start]),
                           None if module_id is None else _arr(_i32, module_id), n, mode, int(wrap_prefetch),
                           int(n_slots), overhead_ms, C.byref(tot), C.byref(hid), C.byref(exp_))
    if rc != DL_OK:
        raise DLError(rc, "dl_timeline: invalid argument")
    return dict(total=tot.value, hidden=hid.value, exposed=exp_.value)


def plan_shared_slots(n_layers, layer_bytes, b3, budget_bytes, n_slots=2):
    """dl_plan_shared_slots: budget_bytes covers resident layers AND the slots, which are sized by the modules that
    still stream a layer."""
    m = len(n_layers)
    flat = [v for row in b3 for v in row]
    out = (_i32 * m)()
    rc = lib().dl_plan_shared_slots(m, _arr(_i32, n_layers), _arr(_u64, layer_bytes), _arr(_f64, flat), int(budget_bytes),
                                    int(n_slots), out)
    if rc != DL_OK:
        raise DLError(rc, "dl_plan_shared_slots: " + ("budget cannot hold the slots" if rc == DL_ERR_BUDGET_EXCEEDED else "invalid argument"))
    return list(out)


def plan(n_layers, layer_bytes, b3, budget_bytes):
    m = len(n_layers)
    flat = [v for row in b3 for v in row]
    out = (_i32 * m)()
    rc = lib().dl_plan(m, _arr(_i32, n_layers), _arr(_u64, layer_bytes), _arr(_f64, flat), budget_bytes, out)
    if rc != DL_OK:
        raise DLError(rc, "dl_plan: invalid argument")
    return list(out)
