"""Seeded synthetic inputs shaped like the paper's workloads (numpy only, no method arithmetic).

The paper evaluates on LLaMA-3.1-8B-Instruct attention (32 query heads, 8 KV heads,
head_dim 128, hidden 4096, 32 layers, Sec. 5.1 / App. C) over long prompts; neither the
weights nor the prompts are available here, so every tensor is drawn i.i.d. N(0,1) from a
counter-based generator (numpy's Philox keyed by (seed, stream)), rounded to bf16 with
round-to-nearest-even and carried as uint16 bit patterns.  A fraction of "heavy" prefix
positions get keys aligned with their KV group's mean window query so the score
distribution has the long tail sparse attention shows (Sec. 3).

The same arrays feed the CPU oracle and the GPU library; this module is imported by tests
and the benchmark only.
"""
import numpy as np

# tensor ids -> Philox stream
_STREAM = {"q_win": 1, "k": 2, "v": 3, "x": 4, "heavy": 5, "lengths": 6, "scores": 7}

LLAMA3_8B = dict(n_q_heads=32, n_kv_heads=8, head_dim=128, hidden=4096, n_layers=32, tsp_layer=15)


def f32_to_bf16_bits(a):
    """Round-to-nearest-even fp32 -> bf16 bit patterns (uint16).  Inputs must be finite."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed, layer, name, seq=0):
    return np.random.Generator(np.random.Philox(key=[int(seed) * 1_000_003 + int(layer) * 4099 + int(seq),
                                                     _STREAM[name]]))


def normal_bf16(seed, layer, name, shape, seq=0, chunk_rows=1 << 14):
    """N(0,1) -> bf16 bits, generated in row chunks to bound host memory."""
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.uint16)
    rng = _rng(seed, layer, name, seq)
    flat = out.reshape(shape[0], -1) if len(shape) > 1 else out.reshape(-1, 1)
    for r0 in range(0, flat.shape[0], chunk_rows):
        r1 = min(flat.shape[0], r0 + chunk_rows)
        flat[r0:r1] = f32_to_bf16_bits(rng.standard_normal((r1 - r0, flat.shape[1]), dtype=np.float32))
    return out


def round_half_up(x):
    """Rate -> count conversion used for k = rate * L (20% of 32768 -> 6554)."""
    return int(np.floor(float(x) + 0.5))


def make_sequence(seed, L, window=8, n_q_heads=32, n_kv_heads=8, head_dim=128, hidden=4096,
                  n_heavy=None, heavy_gain=3.0, layer=0, seq=0, with_v=True, with_x=True):
    """One sequence of one layer.  Returns dict of uint16 arrays:
    q_win [W,Hq,d], k [L,Hkv,d], v [L,Hkv,d] (optional), x [L,hidden] (optional),
    plus heavy (sorted int32 positions in the prefix)."""
    L, W = int(L), int(window)
    P = L - W
    G = n_q_heads // n_kv_heads
    if n_heavy is None:
        n_heavy = round_half_up(0.01 * L)
    n_heavy = min(int(n_heavy), max(P, 0))
    out = {"q_win": normal_bf16(seed, layer, "q_win", (W, n_q_heads, head_dim), seq),
           "k": normal_bf16(seed, layer, "k", (L, n_kv_heads, head_dim), seq)}
    heavy = np.sort(_rng(seed, layer, "heavy", seq).choice(P, size=n_heavy, replace=False)).astype(np.int32) \
        if n_heavy > 0 else np.zeros((0,), np.int32)
    if n_heavy > 0:
        qf = bf16_bits_to_f32(out["q_win"])  # [W,Hq,d]
        for g in range(n_kv_heads):
            mean_q = qf[:, g * G:(g + 1) * G, :].reshape(-1, head_dim).mean(axis=0, dtype=np.float32)
            out["k"][heavy, g, :] = f32_to_bf16_bits(np.float32(heavy_gain) * mean_q)[None, :]
    out["heavy"] = heavy
    if with_v:
        out["v"] = normal_bf16(seed, layer, "v", (L, n_kv_heads, head_dim), seq)
    if with_x:
        out["x"] = normal_bf16(seed, layer, "x", (L, hidden), seq)
    return out


def ragged_lengths(seed, n_seq=8, lo=8192, hi=16384):
    """Sequence lengths uniform in [lo, hi] from the seed."""
    return _rng(seed, 0, "lengths").integers(lo, hi + 1, size=n_seq).astype(np.int64).tolist()


def make_batch(seed, lengths, layer=0, **kw):
    """Packed varlen batch: tensors concatenated along tokens, q_win stacked [B,W,Hq,d],
    cu_seqlens int32 [B+1]."""
    seqs = [make_sequence(seed, L, layer=layer, seq=i + 1, **kw) for i, L in enumerate(lengths)]
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(lengths)
    out = {"cu_seqlens": cu, "q_win": np.stack([s["q_win"] for s in seqs]), "seqs": seqs}
    for name in ("k", "v", "x"):
        if name in seqs[0]:
            out[name] = np.concatenate([s[name] for s in seqs], axis=0)
    return out


def random_scores(seed, rows, P, ties=0.0):
    """Positive fp32 score rows with a log-normal tail; `ties` is the fraction of entries
    overwritten with copies of other entries to exercise the tie rule."""
    rng = _rng(seed, 0, "scores")
    s = np.exp(rng.standard_normal((rows, P), dtype=np.float32)).astype(np.float32) / np.float32(max(P, 1))
    if ties > 0 and P > 1:
        n = int(ties * P)
        for r in range(rows):
            dst = rng.integers(0, P, size=n)
            src = rng.integers(0, P, size=n)
            s[r, dst] = s[r, src]
    return s


def algorithmic_bytes(L, k_tsp, budget, n_q_heads=32, n_kv_heads=8, head_dim=128, hidden=4096, window=8):
    """Bytes one layer's selection must move: K once, Q, scores written+read once, indices
    written+read once, hidden rows read+written, K/V rows read+written (all bf16/fp32/int32)."""
    P = L - window
    b = L * n_kv_heads * head_dim * 2 + window * n_q_heads * head_dim * 2
    rows = n_kv_heads + (1 if k_tsp else 0)
    b += 2 * 4 * rows * P
    b += 2 * 4 * ((k_tsp or 0) + n_kv_heads * budget)
    b += 2 * (k_tsp or 0) * hidden * 2
    b += 2 * 2 * n_kv_heads * budget * head_dim * 2
    return int(b)
