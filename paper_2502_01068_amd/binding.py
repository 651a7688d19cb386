"""ctypes binding of libfastkv_select (argument marshalling only; every step runs in the HIP kernels).

Functions carry the names of the C ABI in ``include/fastkv_select.h``.  torch is used for
device memory and the current stream; tensors must live on the context's GPU.  A missing
library is an error: there is no fallback path.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfastkv_select.so")

FKV_MAX_SEQS = 64
FKV_OK, FKV_EINVAL, FKV_ENULL, FKV_EALIGN, FKV_EUNSUPPORTED, FKV_EWORKSPACE, FKV_EHIP = 0, -1, -2, -3, -4, -5, -6
FKV_POOL_AVG, FKV_POOL_MAX = 0, 1
_POOL = {"avg": FKV_POOL_AVG, "max": FKV_POOL_MAX, FKV_POOL_AVG: FKV_POOL_AVG, FKV_POOL_MAX: FKV_POOL_MAX}

EXPORTS = [
    "fkv_version", "fkv_strerror", "fkv_last_hip_error", "fkv_check_shape", "fkv_check_counts",
    "fkv_workspace_bytes", "fkv_create", "fkv_destroy", "fkv_score_window", "fkv_select_topk",
    "fkv_gather_rows", "fkv_gather_kv", "fkv_compress_kv", "fkv_profile_kernels",
    "fkv_profile_kernel_name", "fkv_profile_enable", "fkv_profile_read", "fkv_set_score_path", "fkv_query_error",
    "fkv_score_heads", "fkv_gather_kv_per_head", "fkv_count_from_rate", "fkv_decode_attention",
    "fkv_index_overlap", "fkv_mass_recall", "fkv_gather_kv_paged", "fkv_decode_attention_paged", "fkv_probe_read", "fkv_plan_layer", "fkv_set_wait_limit", "fkv_clear_error", "fkv_compress_kv_paged", "fkv_probe_logits", "fkv_window_output",
    "fkv_score_window_static", "fkv_score_plan", "fkv_score_window_output", "fkv_set_select_path",
]


class FkvShape(ctypes.Structure):
    _fields_ = [("n_seq", ctypes.c_int32), ("cu_seqlens", ctypes.POINTER(ctypes.c_int32)), ("L", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("window", ctypes.c_int32), ("pool_kernel", ctypes.c_int32), ("pool_mode", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("causal", ctypes.c_int32)]


class FkvLayerPlan(ctypes.Structure):
    _fields_ = [("tokens_in", ctypes.c_int32), ("k_tsp", ctypes.c_int32), ("kv_budget", ctypes.c_int32)]


class FkvError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = load().fkv_strerror(status).decode()
        if status == FKV_EHIP:
            msg += " [hipError %d]" % load().fkv_last_hip_error()
        super().__init__("%s: %s (%d)" % (where, msg, status))


_lib = None


def load():
    """Open libfastkv_select.so (built in-tree by build.py) and declare its signatures."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError("libfastkv_select.so is not built: run `python -m paper_2502_01068_amd.build` "
                                "(or __graft_entry__.build()); there is no fallback path")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    shp, pi32 = ctypes.POINTER(FkvShape), ctypes.POINTER(ctypes.c_int32)
    lib.fkv_version.restype = ctypes.c_int
    lib.fkv_strerror.restype = ctypes.c_char_p
    lib.fkv_strerror.argtypes = [ctypes.c_int]
    lib.fkv_last_hip_error.restype = ctypes.c_int
    lib.fkv_check_shape.argtypes = [shp]
    lib.fkv_check_counts.argtypes = [shp, pi32]
    lib.fkv_workspace_bytes.restype = sz
    lib.fkv_workspace_bytes.argtypes = [i64, i32]
    lib.fkv_create.argtypes = [ctypes.POINTER(vp), ctypes.c_int, i64, i32]
    lib.fkv_destroy.argtypes = [vp]
    lib.fkv_score_window.argtypes = [vp, shp, vp, vp, vp, vp, vp]
    lib.fkv_score_window_static.argtypes = [shp, vp, vp, vp, vp, vp]
    lib.fkv_score_plan.argtypes = [shp, i32, pi32, pi32, pi32]
    lib.fkv_select_topk.argtypes = [vp, shp, vp, i32, pi32, vp, vp]
    lib.fkv_gather_rows.argtypes = [vp, shp, vp, sz, vp, pi32, vp, vp]
    lib.fkv_gather_kv.argtypes = [vp, shp, vp, vp, vp, pi32, vp, vp, vp]
    lib.fkv_compress_kv.argtypes = [vp, shp, vp, vp, vp, pi32, vp, vp, vp, vp, sz, pi32, vp, vp, vp]
    lib.fkv_score_heads.argtypes = [vp, shp, vp, vp, vp, vp]
    lib.fkv_gather_kv_per_head.argtypes = [vp, shp, vp, vp, vp, pi32, vp, vp, vp]
    lib.fkv_decode_attention.argtypes = [vp, shp, vp, vp, vp, i32, pi32, vp, vp]
    lib.fkv_window_output.argtypes = [vp, shp, vp, vp, vp, vp, vp]
    lib.fkv_score_window_output.argtypes = [vp, shp, vp, vp, vp, vp, vp, vp, vp]
    lib.fkv_gather_kv_paged.argtypes = [vp, shp, vp, vp, vp, pi32, vp, i32, i32, i64, vp, vp, vp]
    lib.fkv_compress_kv_paged.argtypes = [vp, shp, vp, vp, vp, pi32, vp, i32, i32, i64, vp, vp, vp, vp]
    lib.fkv_decode_attention_paged.argtypes = [vp, shp, vp, vp, vp, vp, i32, i32, i64, pi32, vp, vp]
    lib.fkv_plan_layer.argtypes = [i32, i32, i32, i32, ctypes.c_double, ctypes.c_double, i32, ctypes.POINTER(FkvLayerPlan)]
    lib.fkv_probe_logits.argtypes = [vp, shp, vp, vp, i32, vp, vp]
    lib.fkv_probe_read.argtypes = [vp, vp, i64, i32, vp]
    lib.fkv_index_overlap.argtypes = [vp, vp, i64, i32, vp, i64, i32, i32, vp, vp]
    lib.fkv_mass_recall.argtypes = [vp, vp, i64, i32, vp, i64, i32, i32, vp, vp]
    lib.fkv_count_from_rate.restype = i32
    lib.fkv_count_from_rate.argtypes = [i32, ctypes.c_double]
    lib.fkv_set_score_path.argtypes = [vp, ctypes.c_int]
    lib.fkv_set_select_path.argtypes = [vp, ctypes.c_int]
    lib.fkv_query_error.argtypes = [vp, pi32]
    lib.fkv_set_wait_limit.argtypes = [vp, i64]
    lib.fkv_clear_error.argtypes = [vp]
    lib.fkv_profile_kernels.restype = ctypes.c_int
    lib.fkv_profile_kernel_name.restype = ctypes.c_char_p
    lib.fkv_profile_kernel_name.argtypes = [ctypes.c_int]
    lib.fkv_profile_enable.argtypes = [vp, ctypes.c_int]
    lib.fkv_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), pi32, i32]
    for name in EXPORTS:
        getattr(lib, name)  # raises AttributeError if a declared symbol is missing
    _lib = lib
    return lib


def _i32_array(values):
    vals = [int(v) for v in values]
    return (ctypes.c_int32 * len(vals))(*vals)


def make_shape(lengths, n_q_heads=32, n_kv_heads=8, head_dim=128, window=8, pool_kernel=7, pool_mode="max",
               softmax_scale=0.0, causal=True):
    """Build the host descriptor.  `lengths` is an int (single sequence) or a list of
    per-sequence token counts.  Returns (FkvShape, keepalive) - keep both alive for the call."""
    s = FkvShape()
    if isinstance(lengths, int):
        lengths = [lengths]
    cu = [0]
    for n in lengths:
        cu.append(cu[-1] + int(n))
    arr = _i32_array(cu)
    s.n_seq = len(lengths)
    s.cu_seqlens = ctypes.cast(arr, ctypes.POINTER(ctypes.c_int32))
    s.L = int(lengths[0])
    s.n_q_heads, s.n_kv_heads, s.head_dim = int(n_q_heads), int(n_kv_heads), int(head_dim)
    s.window, s.pool_kernel, s.pool_mode = int(window), int(pool_kernel), _POOL[pool_mode]
    s.softmax_scale, s.causal = float(softmax_scale), int(bool(causal))
    s._keep = arr
    s._lengths = [int(n) for n in lengths]
    return s


def fkv_count_from_rate(n_tokens, rate):
    """Round-half-up keep count for a rate (host only)."""
    return int(load().fkv_count_from_rate(int(n_tokens), float(rate)))


def fkv_score_plan(shape, max_blocks=256):
    """Block layout of the single-pass score kernel -> (first_block [B+1], own [B], n_sub_max), or None if
    the batch does not fit max_blocks resident blocks (host only)."""
    first = (ctypes.c_int32 * (shape.n_seq + 1))()
    own = (ctypes.c_int32 * shape.n_seq)()
    n_sub = ctypes.c_int32(0)
    rc = load().fkv_score_plan(ctypes.byref(shape), int(max_blocks), first, own, ctypes.byref(n_sub))
    if rc == FKV_EUNSUPPORTED:
        return None
    _check(rc, "fkv_score_plan")
    return list(first), list(own), int(n_sub.value)


def fkv_plan_layer(layer, n_layers, tsp_layer, n_tokens, tsp_rate, kv_rate, window=8):
    """Algorithm 1's schedule for one layer -> (tokens_in, k_tsp, kv_budget)."""
    plan = FkvLayerPlan()
    _check(load().fkv_plan_layer(layer, n_layers, tsp_layer, n_tokens, tsp_rate, kv_rate, window, ctypes.byref(plan)),
           "fkv_plan_layer")
    return plan.tokens_in, plan.k_tsp, plan.kv_budget


def _check(status, where):
    if status != FKV_OK:
        raise FkvError(status, where)


def _dev_ptr(t, name, dtypes=None, allow_none=False, numel=None, nbytes=None, device=None):
    """Device pointer of a tensor after the checks the C ABI cannot make (it sees no sizes): the
    tensor is on the GPU (`device`: on that one), contiguous, of an accepted dtype and holds at
    least `numel` elements / `nbytes` bytes."""
    if t is None:
        if allow_none:
            return None
        raise ValueError("%s is required" % name)
    if not getattr(t, "is_cuda", False):
        raise ValueError("%s must be a GPU tensor" % name)
    if device is not None and t.device.index != device:
        raise ValueError("%s is on cuda:%s, the context is on cuda:%d" % (name, t.device.index, device))
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtypes is not None and t.dtype not in dtypes:
        raise ValueError("%s has dtype %s, expected one of %s" % (name, t.dtype, dtypes))
    if numel is not None and t.numel() < numel:
        raise ValueError("%s holds %d elements, the shape needs %d" % (name, t.numel(), numel))
    if nbytes is not None and t.numel() * t.element_size() < nbytes:
        raise ValueError("%s holds %d bytes, the shape needs %d" % (name, t.numel() * t.element_size(), nbytes))
    return ctypes.c_void_p(t.data_ptr())


class _Sizes:
    """Element counts of every tensor of a call, from the host descriptor."""

    def __init__(self, shape):
        self.total = sum(shape._lengths)
        self.sum_p = self.total - shape.n_seq * shape.window
        self.q_win = shape.n_seq * shape.window * shape.n_q_heads * shape.head_dim
        self.kv = self.total * shape.n_kv_heads * shape.head_dim
        self.q_dec = shape.n_seq * shape.n_q_heads * shape.head_dim


_BF16 = (torch.bfloat16, torch.int16, torch.uint16)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _counts(shape, counts):
    if isinstance(counts, int):
        counts = [counts] * shape.n_seq
    counts = [int(c) for c in counts]
    if len(counts) != shape.n_seq:
        raise ValueError("need one count per sequence")
    return counts, _i32_array(counts)


def fkv_score_window_static(shape, q_win, k, scores_group=None, scores_tsp=None, want_tsp=True):
    """The score call that needs no context and allocates nothing in the library (at most 131072 tokens in
    16 sequences) -> (scores_group [Hkv, sum P] fp32, scores_tsp [sum P] fp32 or None).  Runs on the
    tensors' device, which must be the current one."""
    n = _Sizes(shape)
    dev = k.device
    if dev.index != torch.cuda.current_device():
        raise ValueError("k is on cuda:%s, the current device is cuda:%d" % (dev.index, torch.cuda.current_device()))
    if scores_group is None:
        scores_group = torch.empty((shape.n_kv_heads, n.sum_p), dtype=torch.float32, device=dev)
    if scores_tsp is None and want_tsp:
        scores_tsp = torch.empty((n.sum_p,), dtype=torch.float32, device=dev)
    _check(load().fkv_score_window_static(
        ctypes.byref(shape), _dev_ptr(q_win, "q_win", _BF16, numel=n.q_win, device=dev.index),
        _dev_ptr(k, "k", _BF16, numel=n.kv, device=dev.index),
        _dev_ptr(scores_group, "scores_group", (torch.float32,), numel=shape.n_kv_heads * n.sum_p, device=dev.index),
        _dev_ptr(scores_tsp, "scores_tsp", (torch.float32,), True, numel=n.sum_p, device=dev.index), _stream()),
        "fkv_score_window_static")
    return scores_group, scores_tsp


class Context:
    """Owns an fkv_ctx (device workspace sized for max_total_tokens / max_seqs)."""

    def __init__(self, max_total_tokens, max_seqs=1, device=None):
        lib = load()
        if not torch.cuda.is_available():
            raise RuntimeError("libfastkv_select needs a GPU; no CPU path exists")
        self.device = torch.cuda.current_device() if device is None else int(device)
        h = ctypes.c_void_p()
        _check(lib.fkv_create(ctypes.byref(h), self.device, int(max_total_tokens), int(max_seqs)), "fkv_create")
        self.handle = h
        self.max_total_tokens = int(max_total_tokens)

    def close(self):
        if getattr(self, "handle", None):
            torch.cuda.synchronize(self.device)
            load().fkv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- the C ABI, same names -----------------------------------------------------------
    # Every wrapper checks tensor sizes against the host descriptor and the tensors' device against
    # the context's before the call: the C ABI takes bare pointers and cannot.
    def _p(self, t, name, dtypes=None, allow_none=False, numel=None, nbytes=None):
        return _dev_ptr(t, name, dtypes, allow_none, numel, nbytes, self.device)

    def fkv_score_window(self, shape, q_win, k, scores_group=None, scores_tsp=None, want_tsp=True):
        """-> (scores_group [Hkv, sum P] fp32, scores_tsp [sum P] fp32 or None)"""
        n = _Sizes(shape)
        dev = k.device
        if scores_group is None:
            scores_group = torch.empty((shape.n_kv_heads, n.sum_p), dtype=torch.float32, device=dev)
        if scores_tsp is None and want_tsp:
            scores_tsp = torch.empty((n.sum_p,), dtype=torch.float32, device=dev)
        _check(load().fkv_score_window(self.handle, ctypes.byref(shape), self._p(q_win, "q_win", _BF16, numel=n.q_win),
                                       self._p(k, "k", _BF16, numel=n.kv),
                                       self._p(scores_group, "scores_group", (torch.float32,), numel=shape.n_kv_heads * n.sum_p),
                                       self._p(scores_tsp, "scores_tsp", (torch.float32,), True, numel=n.sum_p), _stream()),
               "fkv_score_window")
        return scores_group, scores_tsp

    def fkv_select_topk(self, shape, scores, k_per_seq, idx_out=None):
        """scores [n_rows, sum P] (or [sum P]) -> idx [n_rows, sum k] int32"""
        counts, arr = _counts(shape, k_per_seq)
        n = _Sizes(shape)
        n_rows = 1 if scores.dim() == 1 else scores.shape[0]
        if scores.shape[-1] != n.sum_p:
            raise ValueError("scores rows hold %d entries, the shape has %d prefix tokens" % (scores.shape[-1], n.sum_p))
        if idx_out is None:
            idx_out = torch.empty((n_rows, sum(counts)), dtype=torch.int32, device=scores.device)
        _check(load().fkv_select_topk(self.handle, ctypes.byref(shape), self._p(scores, "scores", (torch.float32,)),
                                      n_rows, arr, self._p(idx_out, "idx_out", (torch.int32,), numel=n_rows * sum(counts)),
                                      _stream()), "fkv_select_topk")
        return idx_out

    def fkv_gather_rows(self, shape, x, idx, k_per_seq, out=None):
        """x [sum L, ...] -> out [sum k, ...] (rows copied bit for bit)"""
        counts, arr = _counts(shape, k_per_seq)
        n = _Sizes(shape)
        row_bytes = x.stride(0) * x.element_size()
        if x.shape[0] != n.total:
            raise ValueError("x has %d rows, the shape has %d tokens" % (x.shape[0], n.total))
        if out is None:
            out = torch.empty((sum(counts),) + tuple(x.shape[1:]), dtype=x.dtype, device=x.device)
        _check(load().fkv_gather_rows(self.handle, ctypes.byref(shape), self._p(x, "x"), row_bytes,
                                      self._p(idx, "idx", (torch.int32,), numel=sum(counts)), arr,
                                      self._p(out, "out", nbytes=sum(counts) * row_bytes), _stream()),
               "fkv_gather_rows")
        return out

    def fkv_gather_kv(self, shape, k, v, idx_kv, budget_per_seq, k_out=None, v_out=None):
        counts, arr = _counts(shape, budget_per_seq)
        n = _Sizes(shape)
        tot = sum(counts)
        n_out = shape.n_kv_heads * tot * shape.head_dim
        if k_out is None:
            k_out = torch.empty((shape.n_kv_heads, tot, shape.head_dim), dtype=k.dtype, device=k.device)
        if v is not None and v_out is None:
            v_out = torch.empty((shape.n_kv_heads, tot, shape.head_dim), dtype=v.dtype, device=v.device)
        _check(load().fkv_gather_kv(self.handle, ctypes.byref(shape), self._p(k, "k", _BF16, numel=n.kv),
                                    self._p(v, "v", _BF16, True, numel=n.kv),
                                    self._p(idx_kv, "idx_kv", (torch.int32,), numel=shape.n_kv_heads * tot), arr,
                                    self._p(k_out, "k_out", _BF16, numel=n_out), self._p(v_out, "v_out", _BF16, True, numel=n_out),
                                    _stream()), "fkv_gather_kv")
        return k_out, v_out

    def _compress_outputs(self, shape, k, v, x, b_counts, t_counts, out):
        dev = k.device
        tsp = x is not None
        if out is None:
            out = {"k_out": torch.empty((shape.n_kv_heads, sum(b_counts), shape.head_dim), dtype=k.dtype, device=dev),
                   "v_out": torch.empty((shape.n_kv_heads, sum(b_counts), shape.head_dim), dtype=v.dtype, device=dev),
                   "idx_kv": torch.empty((shape.n_kv_heads, sum(b_counts)), dtype=torch.int32, device=dev)}
            if tsp:
                out["x_out"] = torch.empty((sum(t_counts),) + tuple(x.shape[1:]), dtype=x.dtype, device=dev)
                out["idx_tsp"] = torch.empty((sum(t_counts),), dtype=torch.int32, device=dev)
        return out

    def fkv_compress_kv(self, shape, q_win, k, v, budget_per_seq, x=None, k_tsp_per_seq=None, out=None):
        """One layer of Algorithm 1.  Returns dict(k_out, v_out, idx_kv[, x_out, idx_tsp]).
        Pass `out` (a dict from a previous call of the same shape and counts) to reuse the output buffers."""
        b_counts, b_arr = _counts(shape, budget_per_seq)
        n = _Sizes(shape)
        tsp = x is not None
        t_counts, t_arr = _counts(shape, k_tsp_per_seq) if tsp else ([], None)
        if tsp and x.shape[0] != n.total:
            raise ValueError("x has %d rows, the shape has %d tokens" % (x.shape[0], n.total))
        out = self._compress_outputs(shape, k, v, x, b_counts, t_counts, out)
        row_bytes = x.stride(0) * x.element_size() if tsp else 0
        n_kv_out = shape.n_kv_heads * sum(b_counts) * shape.head_dim
        _check(load().fkv_compress_kv(
            self.handle, ctypes.byref(shape), self._p(q_win, "q_win", _BF16, numel=n.q_win),
            self._p(k, "k", _BF16, numel=n.kv), self._p(v, "v", _BF16, numel=n.kv), b_arr,
            self._p(out["k_out"], "k_out", _BF16, numel=n_kv_out), self._p(out["v_out"], "v_out", _BF16, numel=n_kv_out),
            self._p(out["idx_kv"], "idx_kv", (torch.int32,), numel=shape.n_kv_heads * sum(b_counts)),
            self._p(x, "x", None, True), row_bytes, t_arr,
            self._p(out.get("x_out"), "x_out", None, not tsp, nbytes=sum(t_counts) * row_bytes),
            self._p(out.get("idx_tsp"), "idx_tsp", (torch.int32,), not tsp, numel=sum(t_counts)), _stream()),
            "fkv_compress_kv")
        return out

    def fkv_score_heads(self, shape, q_win, k, scores_head=None):
        """-> scores_head [Hq, sum P] fp32: pooled per-head scores (Eq. 1), no head averaging"""
        n = _Sizes(shape)
        if scores_head is None:
            scores_head = torch.empty((shape.n_q_heads, n.sum_p), dtype=torch.float32, device=k.device)
        _check(load().fkv_score_heads(self.handle, ctypes.byref(shape), self._p(q_win, "q_win", _BF16, numel=n.q_win),
                                      self._p(k, "k", _BF16, numel=n.kv),
                                      self._p(scores_head, "scores_head", (torch.float32,), numel=shape.n_q_heads * n.sum_p),
                                      _stream()), "fkv_score_heads")
        return scores_head

    def fkv_gather_kv_per_head(self, shape, k, v, idx_head, budget_per_seq, k_out=None, v_out=None):
        counts, arr = _counts(shape, budget_per_seq)
        n = _Sizes(shape)
        tot = sum(counts)
        n_out = shape.n_q_heads * tot * shape.head_dim
        if k_out is None:
            k_out = torch.empty((shape.n_q_heads, tot, shape.head_dim), dtype=k.dtype, device=k.device)
        if v is not None and v_out is None:
            v_out = torch.empty((shape.n_q_heads, tot, shape.head_dim), dtype=v.dtype, device=v.device)
        _check(load().fkv_gather_kv_per_head(self.handle, ctypes.byref(shape), self._p(k, "k", _BF16, numel=n.kv),
                                             self._p(v, "v", _BF16, True, numel=n.kv),
                                             self._p(idx_head, "idx_head", (torch.int32,), numel=shape.n_q_heads * tot),
                                             arr, self._p(k_out, "k_out", _BF16, numel=n_out),
                                             self._p(v_out, "v_out", _BF16, True, numel=n_out),
                                             _stream()), "fkv_gather_kv_per_head")
        return k_out, v_out

    def fkv_decode_attention(self, shape, q, k, v, n_per_seq, layout="compact", out=None):
        """q [B,Hq,d] bf16; k, v [Hkv,sum n,d] ("compact") or [sum n,Hkv,d] ("token_major") -> out [B,Hq,d] fp32"""
        counts = [int(c) for c in ([n_per_seq] * shape.n_seq if isinstance(n_per_seq, int) else n_per_seq)]
        if len(counts) != shape.n_seq:
            raise ValueError("need one token count per sequence")
        arr = _i32_array(counts)
        n = _Sizes(shape)
        n_cache = sum(counts) * shape.n_kv_heads * shape.head_dim
        if out is None:
            out = torch.empty((shape.n_seq, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device=q.device)
        lay = {"compact": 0, "token_major": 1}[layout]
        _check(load().fkv_decode_attention(self.handle, ctypes.byref(shape), self._p(q, "q", _BF16, numel=n.q_dec),
                                           self._p(k, "k", _BF16, numel=n_cache), self._p(v, "v", _BF16, numel=n_cache), lay, arr,
                                           self._p(out, "out", (torch.float32,), numel=n.q_dec), _stream()), "fkv_decode_attention")
        return out

    def fkv_window_output(self, shape, q_win, k, v, out=None):
        """q_win [B,W,Hq,d], k, v [sum L,Hkv,d] bf16 -> attention output of the window rows [B,W,Hq,d] fp32"""
        n = _Sizes(shape)
        if out is None:
            out = torch.empty((shape.n_seq, shape.window, shape.n_q_heads, shape.head_dim), dtype=torch.float32,
                              device=k.device)
        _check(load().fkv_window_output(self.handle, ctypes.byref(shape), self._p(q_win, "q_win", _BF16, numel=n.q_win),
                                        self._p(k, "k", _BF16, numel=n.kv), self._p(v, "v", _BF16, numel=n.kv),
                                        self._p(out, "out", (torch.float32,), numel=n.q_win), _stream()), "fkv_window_output")
        return out

    def fkv_score_window_output(self, shape, q_win, k, v, scores_group=None, scores_tsp=None, out=None, want_tsp=True):
        """Scores and the window rows' attention output in one call (V read once, K twice, no grid exchange)
        -> (scores_group [Hkv, sum P], scores_tsp [sum P] or None, out [B,W,Hq,d] fp32)"""
        n = _Sizes(shape)
        dev = k.device
        if scores_group is None:
            scores_group = torch.empty((shape.n_kv_heads, n.sum_p), dtype=torch.float32, device=dev)
        if scores_tsp is None and want_tsp:
            scores_tsp = torch.empty((n.sum_p,), dtype=torch.float32, device=dev)
        if out is None:
            out = torch.empty((shape.n_seq, shape.window, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device=dev)
        _check(load().fkv_score_window_output(
            self.handle, ctypes.byref(shape), self._p(q_win, "q_win", _BF16, numel=n.q_win), self._p(k, "k", _BF16, numel=n.kv),
            self._p(v, "v", _BF16, numel=n.kv), self._p(scores_group, "scores_group", (torch.float32,), numel=shape.n_kv_heads * n.sum_p),
            self._p(scores_tsp, "scores_tsp", (torch.float32,), True, numel=n.sum_p),
            self._p(out, "out", (torch.float32,), numel=n.q_win), _stream()), "fkv_score_window_output")
        return scores_group, scores_tsp, out

    def _paging(self, shape, block_table, k_pages, v_pages, v_required):
        if block_table.dim() != 2 or block_table.shape[0] != shape.n_seq:
            raise ValueError("block_table must be [n_seq, max_pages], got %s" % (tuple(block_table.shape),))
        if k_pages.dim() != 4 or tuple(k_pages.shape[2:]) != (shape.n_kv_heads, shape.head_dim):
            raise ValueError("k_pages must be [n_pages, page_size, Hkv, d], got %s" % (tuple(k_pages.shape),))
        if v_pages is not None and tuple(v_pages.shape) != tuple(k_pages.shape):
            raise ValueError("v_pages must have the shape of k_pages")
        return (self._p(block_table, "block_table", (torch.int32,)), int(block_table.shape[1]), int(k_pages.shape[1]),
                int(k_pages.shape[0]), self._p(k_pages, "k_pages", _BF16), self._p(v_pages, "v_pages", _BF16, not v_required))

    def fkv_gather_kv_paged(self, shape, k, v, idx_kv, budget_per_seq, block_table, k_pages, v_pages=None):
        """k, v [sum L,Hkv,d]; idx_kv [Hkv,sum budget]; block_table [B,max_pages] int32 (GPU);
        k_pages, v_pages [n_pages,page_size,Hkv,d] are updated in place"""
        counts, arr = _counts(shape, budget_per_seq)
        n = _Sizes(shape)
        if (v is None) != (v_pages is None):
            raise ValueError("v and v_pages go together")
        bt, max_pages, page_size, n_pages, kp, vp = self._paging(shape, block_table, k_pages, v_pages, False)
        _check(load().fkv_gather_kv_paged(self.handle, ctypes.byref(shape), self._p(k, "k", _BF16, numel=n.kv),
                                          self._p(v, "v", _BF16, True, numel=n.kv),
                                          self._p(idx_kv, "idx_kv", (torch.int32,), numel=shape.n_kv_heads * sum(counts)), arr,
                                          bt, max_pages, page_size, n_pages, kp, vp, _stream()), "fkv_gather_kv_paged")
        return k_pages, v_pages

    def fkv_compress_kv_paged(self, shape, q_win, k, v, budget_per_seq, block_table, k_pages, v_pages, idx_kv=None):
        """score -> per-KV-head select -> kept K/V rows into the pages; returns idx_kv [Hkv, sum budget]"""
        counts, arr = _counts(shape, budget_per_seq)
        n = _Sizes(shape)
        if idx_kv is None:
            idx_kv = torch.empty((shape.n_kv_heads, sum(counts)), dtype=torch.int32, device=k.device)
        bt, max_pages, page_size, n_pages, kp, vp = self._paging(shape, block_table, k_pages, v_pages, True)
        _check(load().fkv_compress_kv_paged(self.handle, ctypes.byref(shape), self._p(q_win, "q_win", _BF16, numel=n.q_win),
                                            self._p(k, "k", _BF16, numel=n.kv), self._p(v, "v", _BF16, numel=n.kv), arr,
                                            bt, max_pages, page_size, n_pages, kp, vp,
                                            self._p(idx_kv, "idx_kv", (torch.int32,), numel=shape.n_kv_heads * sum(counts)),
                                            _stream()), "fkv_compress_kv_paged")
        return idx_kv

    def fkv_decode_attention_paged(self, shape, q, k_pages, v_pages, block_table, n_per_seq, out=None):
        """q [B,Hq,d] bf16; k_pages, v_pages [n_pages,page_size,Hkv,d]; block_table [B,max_pages] -> out [B,Hq,d] fp32"""
        counts = [int(c) for c in ([n_per_seq] * shape.n_seq if isinstance(n_per_seq, int) else n_per_seq)]
        if len(counts) != shape.n_seq:
            raise ValueError("need one token count per sequence")
        arr = _i32_array(counts)
        n = _Sizes(shape)
        if out is None:
            out = torch.empty((shape.n_seq, shape.n_q_heads, shape.head_dim), dtype=torch.float32, device=q.device)
        bt, max_pages, page_size, n_pages, kp, vp = self._paging(shape, block_table, k_pages, v_pages, True)
        _check(load().fkv_decode_attention_paged(self.handle, ctypes.byref(shape), self._p(q, "q", _BF16, numel=n.q_dec),
                                                 kp, vp, bt, max_pages, page_size, n_pages, arr,
                                                 self._p(out, "out", (torch.float32,), numel=n.q_dec), _stream()),
               "fkv_decode_attention_paged")
        return out

    def fkv_probe_read(self, src, streaming=False):
        """Read-only launch over the tensor's bytes (size must be a multiple of 64 KiB)."""
        _check(load().fkv_probe_read(self.handle, self._p(src, "src"), src.numel() * src.element_size(),
                                     1 if streaming else 0, _stream()), "fkv_probe_read")

    def fkv_probe_logits(self, shape, q_win, k, use_mfma=True, row_keys=None):
        """Largest raw logit of every (head, window row) over all tokens -> fp32 [Hq, W] (G <= 4, one sequence)."""
        if row_keys is None:
            row_keys = torch.empty((shape.n_kv_heads * 32,), dtype=torch.int32, device=k.device)
        n = _Sizes(shape)
        _check(load().fkv_probe_logits(self.handle, ctypes.byref(shape), self._p(q_win, "q_win", _BF16, numel=n.q_win),
                                       self._p(k, "k", _BF16, numel=n.kv), 1 if use_mfma else 0,
                                       self._p(row_keys, "row_keys", (torch.int32,), numel=shape.n_kv_heads * 32), _stream()),
               "fkv_probe_logits")
        return row_keys

    @staticmethod
    def decode_row_keys(row_keys, shape):
        """Order-preserving keys of fkv_probe_logits -> fp32 [Hq, W]."""
        import numpy as np
        key = row_keys.cpu().numpy().view(np.uint32)
        bits = np.where(key & 0x80000000, key ^ np.uint32(0x80000000), ~key).astype(np.uint32)
        g_size = shape.n_q_heads // shape.n_kv_heads
        vals = bits.view(np.float32).reshape(shape.n_kv_heads, 4, 8)[:, :g_size, :shape.window]
        return vals.reshape(shape.n_q_heads, shape.window)

    def fkv_index_overlap(self, a, b, count_out=None):
        """a [R,n_a], b [R,n_b] (or [n_b]: one list for every row) ascending int32 -> shared-index counts [R] int32"""
        a2 = a if a.dim() == 2 else a.unsqueeze(0)
        rows = a2.shape[0]
        b_stride = 0 if b.dim() == 1 else b.stride(0)
        n_b = b.shape[-1]
        if b.dim() == 2 and b.shape[0] != rows:
            raise ValueError("a and b need the same number of rows")
        if (a2.shape[1] > 0 and a2.stride(1) != 1) or (n_b > 0 and b.stride(-1) != 1):
            raise ValueError("index rows must be contiguous")
        if count_out is None:
            count_out = torch.empty((rows,), dtype=torch.int32, device=a.device)
        _check(load().fkv_index_overlap(self.handle, self._p(a2, "a", (torch.int32,), True), a2.stride(0) if rows > 1 else 0,
                                        a2.shape[1], self._p(b, "b", (torch.int32,), True), b_stride, n_b, rows,
                                        self._p(count_out, "count_out", (torch.int32,), numel=rows), _stream()), "fkv_index_overlap")
        return count_out

    def fkv_mass_recall(self, scores, idx, recall_out=None):
        """scores [R,P] fp32, idx [R,n] int32 -> share of each row's mass the kept indices cover, [R] fp32"""
        s2 = scores if scores.dim() == 2 else scores.unsqueeze(0)
        i2 = idx if idx.dim() == 2 else idx.unsqueeze(0)
        rows = s2.shape[0]
        if i2.shape[0] != rows:
            raise ValueError("scores and idx need the same number of rows")
        if (s2.shape[1] > 0 and s2.stride(1) != 1) or (i2.shape[1] > 0 and i2.stride(1) != 1):
            raise ValueError("rows must be contiguous")
        if recall_out is None:
            recall_out = torch.empty((rows,), dtype=torch.float32, device=scores.device)
        _check(load().fkv_mass_recall(self.handle, self._p(s2, "scores", (torch.float32,), True),
                                      s2.stride(0) if rows > 1 else 0, s2.shape[1],
                                      self._p(i2, "idx", (torch.int32,), True), i2.stride(0) if rows > 1 else 0,
                                      i2.shape[1], rows, self._p(recall_out, "recall_out", (torch.float32,), numel=rows),
                                      _stream()), "fkv_mass_recall")
        return recall_out

    def fkv_set_score_path(self, mode):
        """0 auto, 1 two-pass kernels, 2 single-pass resident-grid kernel."""
        _check(load().fkv_set_score_path(self.handle, int(mode)), "fkv_set_score_path")

    def fkv_set_select_path(self, mode):
        """0 auto, 1 never several blocks per row in one launch, 2 several blocks per row whenever the call fits."""
        _check(load().fkv_set_select_path(self.handle, int(mode)), "fkv_set_select_path")

    def fkv_set_wait_limit(self, microseconds):
        _check(load().fkv_set_wait_limit(self.handle, int(microseconds)), "fkv_set_wait_limit")

    def fkv_clear_error(self):
        _check(load().fkv_clear_error(self.handle), "fkv_clear_error")

    def fkv_query_error(self):
        flag = ctypes.c_int32(0)
        _check(load().fkv_query_error(self.handle, ctypes.byref(flag)), "fkv_query_error")
        return int(flag.value)

    # ---- timing facility -----------------------------------------------------------------
    def fkv_profile_enable(self, on=True):
        _check(load().fkv_profile_enable(self.handle, int(bool(on))), "fkv_profile_enable")

    def fkv_profile_read(self):
        """-> {kernel name: (total ms, launches)} since the last read (synchronises)."""
        lib = load()
        n = lib.fkv_profile_kernels()
        ms = (ctypes.c_float * n)()
        cnt = (ctypes.c_int32 * n)()
        _check(lib.fkv_profile_read(self.handle, ms, cnt, n), "fkv_profile_read")
        return {lib.fkv_profile_kernel_name(i).decode(): (float(ms[i]), int(cnt[i])) for i in range(n)}
