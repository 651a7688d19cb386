"""FastKV selection-path oracle (TEST INFRASTRUCTURE ONLY).

numpy front end of ``fastkv_oracle.c``: plain CPU loops for the window-attention
saliency score (Sec. 4.2, Eq. 1), per-head pooling, group / all-head means (Eq. 2,
App. B.1), top-k with the window merged in (Sec. 4.2) and the row gathers of
HiddenCompress / KVCompress (App. B.1, Algorithm 1), the attention output of the window rows,
the decoding step over a cache and the two diagnostics of Sec. 3 (set overlap, mass recall).  Only tests, the smoke check and
the benchmark's CPU-baseline leg may import this package; it shares nothing with the
GPU library.

bf16 tensors are carried as ``uint16`` bit patterns.  ``precision`` picks the fp32
build (``"f32"``, accumulates like the GPU path's arithmetic type) or the fp64 build
(``"f64"``, used to bound rounding).
"""
import ctypes
import math

import numpy as np

from . import build as _build

POOL_AVG = 0
POOL_MAX = 1
_POOL = {"avg": POOL_AVG, "max": POOL_MAX, POOL_AVG: POOL_AVG, POOL_MAX: POOL_MAX}

_libs = {}


def _lib(precision: str):
    if precision not in ("f32", "f64"):
        raise ValueError("precision must be 'f32' or 'f64'")
    if precision not in _libs:
        paths = _build.build()
        lib = ctypes.CDLL(paths[precision])
        assert lib.orc_real_bytes() == (4 if precision == "f32" else 8)
        _libs[precision] = lib
    return _libs[precision]


def max_threads():
    """Threads the head loop of window_attention will use (OpenMP over heads only)."""
    return int(_lib("f32").orc_max_threads())


def _real(precision):
    return np.float32 if precision == "f32" else np.float64


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u16(a, shape_len):
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16 or a.ndim != shape_len:
        raise ValueError("bf16 tensors are passed as uint16 bit patterns with %d dims" % shape_len)
    return a


def window_attention(q_win, k, scale=None, causal=True, precision="f32", threads=None):
    """s[h, j] = sum over the W window queries of the softmax attention row at key j (Eq. 1
    before pooling), j in the prefix [0, L-W).  q_win [W,Hq,d], k [L,Hkv,d] (uint16 bf16)."""
    q_win, k = _u16(q_win, 3), _u16(k, 3)
    W, Hq, d = q_win.shape
    L, Hkv, d2 = k.shape
    if d2 != d:
        raise ValueError("head_dim mismatch")
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    P = L - W
    out = np.empty((Hq, P), dtype=_real(precision))
    lib = _lib(precision)
    if threads is not None:
        lib.orc_set_threads(int(threads))
    rc = lib.orc_window_attention(_ptr(q_win), _ptr(k), L, Hq, Hkv, d, W, ctypes.c_double(scale),
                                  int(bool(causal)), _ptr(out))
    if rc != 0:
        raise ValueError("orc_window_attention failed: %d" % rc)
    return out


def window_output(q_win, k, v, scale=None, causal=True, precision="f64", threads=None):
    """The layer's attention output at the W window positions: out[w, h] = sum over the keys j
    visible to position L-W+w of Att[h, L-W+w, j] * v[j, g(h)], with the same probabilities Eq. 1
    sums.  q_win [W,Hq,d], k, v [L,Hkv,d] (uint16 bf16).  Returns [W,Hq,d]."""
    q_win, k, v = _u16(q_win, 3), _u16(k, 3), _u16(v, 3)
    W, Hq, d = q_win.shape
    L, Hkv, d2 = k.shape
    if d2 != d or v.shape != k.shape:
        raise ValueError("shape mismatch")
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty((W, Hq, d), dtype=_real(precision))
    lib = _lib(precision)
    if threads is not None:
        lib.orc_set_threads(int(threads))
    rc = lib.orc_window_output(_ptr(q_win), _ptr(k), _ptr(v), L, Hq, Hkv, d, W, ctypes.c_double(scale),
                               int(bool(causal)), _ptr(out))
    if rc != 0:
        raise ValueError("orc_window_output failed: %d" % rc)
    return out


def pool_rows(s, kernel=7, mode="max", precision="f32"):
    """Same-length 1-D pooling along the last axis of s [rows, P] (Eq. 1 'Pooling')."""
    s = np.ascontiguousarray(s, dtype=_real(precision))
    rows, P = s.shape
    out = np.empty_like(s)
    lib = _lib(precision)
    for r in range(rows):
        rc = lib.orc_pool_row(_ptr(s[r]), P, int(kernel), _POOL[mode], _ptr(out[r]))
        if rc != 0:
            raise ValueError("orc_pool_row failed: %d" % rc)
    return out


def head_means(p_head, n_kv_heads, precision="f32"):
    """(S_group [Hkv,P], S_tsp [P]) from pooled per-head scores [Hq,P] (App. B.1, Eq. 2)."""
    p_head = np.ascontiguousarray(p_head, dtype=_real(precision))
    Hq, P = p_head.shape
    sg = np.empty((n_kv_heads, P), dtype=p_head.dtype)
    st = np.empty((P,), dtype=p_head.dtype)
    rc = _lib(precision).orc_head_means(_ptr(p_head), Hq, int(n_kv_heads), P, _ptr(sg), _ptr(st))
    if rc != 0:
        raise ValueError("orc_head_means failed: %d" % rc)
    return sg, st


def score_window(q_win, k, pool_kernel=7, pool_mode="max", scale=None, causal=True,
                 precision="f32", threads=None):
    """Full scoring of one sequence.  Returns dict with s_head, p_head [Hq,P],
    scores_group [Hkv,P], scores_tsp [P] in the chosen precision."""
    s_head = window_attention(q_win, k, scale, causal, precision, threads)
    p_head = pool_rows(s_head, pool_kernel, pool_mode, precision)
    sg, st = head_means(p_head, k.shape[1], precision)
    return {"s_head": s_head, "p_head": p_head, "scores_group": sg, "scores_tsp": st}


def select_topk(scores, window, k):
    """Ascending kept indices of one row: the k-W best prefix tokens (ties to the lower
    index) plus the W window tokens P..P+W-1 (Sec. 4.2).  scores are ranked as fp32."""
    scores = np.ascontiguousarray(scores, dtype=np.float32)
    if scores.ndim != 1:
        raise ValueError("one row at a time")
    P = scores.shape[0]
    out = np.empty((int(k),), dtype=np.int32)
    rc = _lib("f32").orc_select_topk(_ptr(scores), P, int(window), int(k), _ptr(out))
    if rc != 0:
        raise ValueError("orc_select_topk failed: %d (need W <= k <= P+W)" % rc)
    return out


def gather_rows(x, idx):
    """out[t] = x[idx[t]] copied bit for bit; x is any C-contiguous array, rows on axis 0."""
    x = np.ascontiguousarray(x)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    if idx.size and (idx.min() < 0 or idx.max() >= x.shape[0]):
        raise IndexError("gather index out of range")
    row_bytes = x.strides[0] if x.ndim > 1 else x.itemsize
    out = np.empty((idx.shape[0],) + x.shape[1:], dtype=x.dtype)
    _lib("f32").orc_gather_rows(_ptr(x), ctypes.c_size_t(row_bytes), ctypes.c_size_t(row_bytes),
                                _ptr(idx), int(idx.shape[0]), _ptr(out))
    return out


def gather_kv(kv, idx_kv):
    """KVCompress gather: kv [L,Hkv,d], idx_kv [Hkv,b] -> [Hkv,b,d] with
    out[g,t] = kv[idx_kv[g,t], g]."""
    kv = np.ascontiguousarray(kv)
    L, Hkv, d = kv.shape
    idx_kv = np.ascontiguousarray(idx_kv, dtype=np.int32)
    if idx_kv.size and (idx_kv.min() < 0 or idx_kv.max() >= L):
        raise IndexError("gather index out of range")
    b = idx_kv.shape[1]
    out = np.empty((Hkv, b, d), dtype=kv.dtype)
    lib = _lib("f32")
    for g in range(Hkv):
        src = kv[:, g, :]
        base = ctypes.c_void_p(kv.ctypes.data + g * d * kv.itemsize)
        lib.orc_gather_rows(base, ctypes.c_size_t(kv.strides[0]), ctypes.c_size_t(d * kv.itemsize),
                            _ptr(idx_kv[g]), b, _ptr(out[g]))
        del src
    return out


def gather_kv_per_head(kv, idx_head):
    """Head-wise KV retention (the layout Sec. 5.3 contrasts with group-wise storage):
    kv [L,Hkv,d], idx_head [Hq,b] -> [Hq,b,d] with out[h,t] = kv[idx_head[h,t], h // G]."""
    kv = np.ascontiguousarray(kv)
    L, Hkv, d = kv.shape
    idx_head = np.ascontiguousarray(idx_head, dtype=np.int32)
    Hq, b = idx_head.shape
    if Hq % Hkv != 0:
        raise ValueError("Hq must be a multiple of Hkv")
    if idx_head.size and (idx_head.min() < 0 or idx_head.max() >= L):
        raise IndexError("gather index out of range")
    G = Hq // Hkv
    out = np.empty((Hq, b, d), dtype=kv.dtype)
    lib = _lib("f32")
    for h in range(Hq):
        base = ctypes.c_void_p(kv.ctypes.data + (h // G) * d * kv.itemsize)
        lib.orc_gather_rows(base, ctypes.c_size_t(kv.strides[0]), ctypes.c_size_t(d * kv.itemsize),
                            _ptr(idx_head[h]), b, _ptr(out[h]))
    return out


def gather_kv_paged(kv, idx_kv, block_table, pages):
    """KVCompress into a paged cache (the paper's Limitations section names paged attention as the
    serving layout the method has to fit): kv [L,Hkv,d], idx_kv [Hkv,b]; pages
    [n_pages,page_size,Hkv,d]; block_table[p] = physical page of logical page p of this sequence.
    The t-th kept row of KV head g lands in page block_table[t // page_size], slot t % page_size.
    Returns the updated copy of `pages`; every other slot keeps its content."""
    kv = np.ascontiguousarray(kv)
    out = np.array(pages, copy=True)
    n_pages, page_size, Hkv, d = out.shape
    if kv.shape[1:] != (Hkv, d):
        raise ValueError("shape mismatch")
    for g in range(Hkv):
        for t in range(idx_kv.shape[1]):
            page = int(block_table[t // page_size])
            if not 0 <= page < n_pages:
                raise IndexError("block table entry out of range")
            out[page, t % page_size, g] = kv[int(idx_kv[g, t]), g]
    return out


def paged_view(pages, block_table, n):
    """The first n logical tokens of a sequence in a paged cache, token-major [n,Hkv,d]."""
    page_size = pages.shape[1]
    out = np.empty((n,) + pages.shape[2:], dtype=pages.dtype)
    for t in range(n):
        out[t] = pages[int(block_table[t // page_size]), t % page_size]
    return out


def decode_attention(q, k, v, layout="compact", scale=None, precision="f32"):
    """Attention output of one new query token over a KV cache (the decoding step that reads the
    compressed cache, Algorithm 1 / Sec. 5.3).  q [Hq,d]; layout "compact": k, v [Hkv,n,d] (what
    KVCompress produced), "token_major": k, v [n,Hkv,d].  Returns [Hq,d] in the chosen precision."""
    q, k, v = _u16(q, 2), _u16(k, 3), _u16(v, 3)
    Hq, d = q.shape
    if layout == "compact":
        Hkv, n, d2 = k.shape
        tok_stride, head_stride = d2, n * d2
    elif layout == "token_major":
        n, Hkv, d2 = k.shape
        tok_stride, head_stride = Hkv * d2, d2
    else:
        raise ValueError("layout must be 'compact' or 'token_major'")
    if d2 != d or v.shape != k.shape:
        raise ValueError("shape mismatch")
    if scale is None:
        scale = 1.0 / math.sqrt(d)
    out = np.empty((Hq, d), dtype=_real(precision))
    rc = _lib(precision).orc_decode_attention(_ptr(q), _ptr(k), _ptr(v), int(n), Hq, Hkv, d,
                                              ctypes.c_long(tok_stride), ctypes.c_long(head_stride),
                                              ctypes.c_double(scale), _ptr(out))
    if rc != 0:
        raise ValueError("orc_decode_attention failed: %d" % rc)
    return out


def index_overlap(a, b):
    """Number of indices two kept sets share (Sec. 3.1: the overlap of the critical-token sets of two
    layers; the overlap ratio is this count over the set size).  a, b: ascending duplicate-free
    index lists.  Walks both lists once."""
    a = np.asarray(a).reshape(-1)
    b = np.asarray(b).reshape(-1)
    i = j = n = 0
    while i < a.size and j < b.size:
        if a[i] == b[j]:
            n += 1
            i += 1
            j += 1
        elif a[i] < b[j]:
            i += 1
        else:
            j += 1
    return n


def mass_recall(scores, idx):
    """Share of a score row's total mass that an index set covers (Sec. 3.2: attention recall of
    a token subset).  scores [P] (non-negative mass per prefix token); idx: kept indices, those
    outside [0, P) (the window tokens of a kept set) carry no score and are skipped.  fp64 sums;
    0 when the row has no mass."""
    scores = np.asarray(scores).reshape(-1)
    total = 0.0
    for x in scores:
        total += float(x)
    kept = 0.0
    for j in np.asarray(idx).reshape(-1):
        if 0 <= j < scores.size:
            kept += float(scores[j])
    return kept / total if total > 0.0 else 0.0


def compress_kv(q_win, k, v, budget, pool_kernel=7, pool_mode="max", scale=None, causal=True,
                x=None, k_tsp=None, precision="f32", threads=None):
    """One layer of Algorithm 1 for one sequence: KVCompress with `budget` kept tokens per
    KV head and, when x and k_tsp are given, HiddenCompress keeping k_tsp rows."""
    W = q_win.shape[0]
    sc = score_window(q_win, k, pool_kernel, pool_mode, scale, causal, precision, threads)
    sg32 = sc["scores_group"].astype(np.float32)
    idx_kv = np.stack([select_topk(sg32[g], W, budget) for g in range(k.shape[1])])
    out = dict(sc)
    out["idx_kv"] = idx_kv
    out["k_out"] = gather_kv(k, idx_kv)
    out["v_out"] = gather_kv(v, idx_kv)
    if x is not None and k_tsp is not None:
        idx_tsp = select_topk(sc["scores_tsp"].astype(np.float32), W, k_tsp)
        out["idx_tsp"] = idx_tsp
        out["x_out"] = gather_rows(x, idx_tsp)
    return out
