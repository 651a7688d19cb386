"""Seeded random draws over what the boundary accepts, for the parts that are exact: top-k on
arbitrary fp32 rows, row gathers of any 16-byte-multiple width, the fused call against its
separate steps, decode over compact / paged caches.  Complements the fixed cases of the other files."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_01068_amd import binding as fk
from paper_2502_01068_amd import workloads as wl
from parity import dev_bf16, host_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    c = fk.Context(max_total_tokens=300000, max_seqs=8)
    yield c
    assert c.fkv_query_error() == 0
    c.close()


def _score_row(rng, P, kind):
    if kind == 0:      # log-normal, the shape attention mass has
        return np.exp(3 * rng.standard_normal(P)).astype(np.float32)
    if kind == 1:      # signed, with exact zeros of both signs
        x = rng.standard_normal(P).astype(np.float32)
        x[rng.random(P) < 0.2] = 0.0
        x[rng.random(P) < 0.1] = -0.0
        return x
    if kind == 2:      # a handful of distinct values: long runs of ties
        return rng.choice(np.array([0.0, 1e-30, 0.5, 0.5000001, 3.0], np.float32), P)
    if kind == 3:      # plateaus, as max pooling leaves them
        x = np.exp(rng.standard_normal(P)).astype(np.float32)
        return np.maximum.reduce([np.roll(x, s) for s in range(-3, 4)])
    if kind == 4:      # the full fp32 range including infinities and denormals
        x = rng.integers(0, 2 ** 32, size=P, dtype=np.uint64).astype(np.uint32).view(np.float32).copy()
        x[np.isnan(x)] = np.float32(1.0)
        return x
    return np.full(P, np.float32(rng.standard_normal()), np.float32)   # constant row


@pytest.mark.parametrize("case", range(120))
def test_random_select(ctx, case):
    rng = np.random.default_rng(3000 + case)
    W = int(rng.integers(1, 9))
    B = int(rng.integers(1, 4))
    edges = [1, 63, 64, 1023, 1024, 1025, 8191, 8192, 8193, 16383, 16385, 32765, 32766, 32767, 40000, 70000]
    top = 50000 if case < 40 else int(rng.choice([20000, 90000, 260000])) // B   # later cases: rows up to 8 slices of 32768 keys
    Ps = [int(rng.choice(edges)) if rng.random() < 0.5 else int(rng.integers(0, top)) for _ in range(B)]
    rows = int(rng.integers(1, 5))
    ks = [int(rng.integers(W, P + W + 1)) for P in Ps]
    path = (0, 2, 1)[case % 3]   # default / several blocks per row wherever they fit / never
    ctx.fkv_set_select_path(path)
    print("case %d: W=%d P=%s rows=%d ks=%s select path %d" % (case, W, Ps, rows, ks, path), flush=True)
    scores = np.concatenate([np.stack([_score_row(rng, P, int(rng.integers(0, 6))) for _ in range(rows)]) for P in Ps],
                            axis=1) if sum(Ps) else np.zeros((rows, 0), np.float32)
    lengths = [P + W for P in Ps]
    shape = fk.make_shape(lengths if B > 1 else lengths[0], window=W)
    idx = ctx.fkv_select_topk(shape, torch.from_numpy(np.ascontiguousarray(scores)).cuda(), ks).cpu().numpy()
    ctx.fkv_set_select_path(0)
    col = o = 0
    for P, k in zip(Ps, ks):
        for r in range(rows):
            np.testing.assert_array_equal(idx[r, o:o + k], oracle.select_topk(scores[r, col:col + P], W, k),
                                          err_msg="P %d row %d k %d" % (P, r, k))
        col += P
        o += k


@pytest.mark.parametrize("case", range(16))
def test_random_gather_rows(ctx, case):
    rng = np.random.default_rng(4000 + case)
    B = int(rng.integers(1, 6))
    lengths = [int(rng.integers(8, 3000)) for _ in range(B)]
    ks = [int(rng.integers(8, L + 1)) for L in lengths]
    row_bytes = 16 * int(rng.choice([1, 2, 3, 5, 16, 17, 64, 100, 512, 640]))
    print("case %d: lengths=%s ks=%s row_bytes=%d" % (case, lengths, ks, row_bytes), flush=True)
    x = rng.integers(0, 65536, size=(sum(lengths), row_bytes // 2), dtype=np.uint16)
    idx = np.concatenate([np.sort(rng.choice(L, k, replace=False)) for L, k in zip(lengths, ks)]).astype(np.int32)
    shape = fk.make_shape(lengths if B > 1 else lengths[0])
    out = host_bits(ctx.fkv_gather_rows(shape, dev_bf16(x), torch.from_numpy(idx).cuda(), ks))
    cu, oo = np.cumsum([0] + lengths), np.cumsum([0] + ks)
    for b in range(B):
        np.testing.assert_array_equal(out[oo[b]:oo[b + 1]], oracle.gather_rows(x[cu[b]:cu[b + 1]], idx[oo[b]:oo[b + 1]]))


@pytest.mark.parametrize("case", range(10))
def test_random_fused_call_equals_its_steps(ctx, case):
    rng = np.random.default_rng(5000 + case)
    B = int(rng.integers(1, 5))
    lengths = [int(rng.integers(8, 6000)) for _ in range(B)]
    budgets = [int(rng.integers(8, L + 1)) for L in lengths]
    ktsps = [int(rng.integers(8, L + 1)) for L in lengths]
    hidden = 16 * int(rng.integers(1, 20))
    pool_mode = ("max", "avg")[case % 2]
    ctx.fkv_set_score_path(case % 3 if case % 3 != 2 else 0)
    ctx.fkv_set_select_path(2 if case % 4 >= 2 else 0)   # half the cases: several select blocks per row wherever they fit
    print("case %d: lengths=%s budgets=%s ktsps=%s hidden=%d %s" % (case, lengths, budgets, ktsps, hidden, pool_mode), flush=True)
    batch = wl.make_batch(5000 + case, lengths, n_heavy=5, hidden=hidden)
    shape = fk.make_shape(lengths if B > 1 else lengths[0], pool_mode=pool_mode)
    q, k, v, x = (dev_bf16(batch[n]) for n in ("q_win", "k", "v", "x"))
    out = ctx.fkv_compress_kv(shape, q, k, v, budgets, x=x, k_tsp_per_seq=ktsps)
    sg, st = ctx.fkv_score_window(shape, q, k)
    idx_kv = ctx.fkv_select_topk(shape, sg, budgets)
    idx_tsp = ctx.fkv_select_topk(shape, st.unsqueeze(0), ktsps)[0]
    ko, vo = ctx.fkv_gather_kv(shape, k, v, idx_kv, budgets)
    xo = ctx.fkv_gather_rows(shape, x, idx_tsp, ktsps)
    ctx.fkv_set_score_path(0)
    ctx.fkv_set_select_path(0)
    assert torch.equal(out["idx_kv"], idx_kv) and torch.equal(out["idx_tsp"], idx_tsp)
    for a, b in ((out["k_out"], ko), (out["v_out"], vo), (out["x_out"], xo)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


@pytest.mark.parametrize("case", range(12))
def test_random_decode(ctx, case):
    rng = np.random.default_rng(6000 + case)
    Hkv, G = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    Hq, d = Hkv * G, 128
    B = int(rng.integers(1, 5))
    ns = [int(rng.integers(1, 5000)) for _ in range(B)]
    scale = float(rng.choice([0.0, 0.05, 0.12]))
    ps = int(rng.choice([1, 2, 16, 64, 256]))
    print("case %d: Hq=%d Hkv=%d ns=%s scale=%g page=%d" % (case, Hq, Hkv, ns, scale, ps), flush=True)
    tot = sum(ns)
    q = wl.normal_bf16(6000 + case, 0, "q_win", (B, Hq, d))
    k = wl.normal_bf16(6000 + case, 0, "k", (tot, Hkv, d))
    v = wl.normal_bf16(6000 + case, 0, "v", (tot, Hkv, d))
    shape = fk.make_shape([8] * B if B > 1 else 8, n_q_heads=Hq, n_kv_heads=Hkv, softmax_scale=scale)
    out_tm = ctx.fkv_decode_attention(shape, dev_bf16(q), dev_bf16(k), dev_bf16(v), ns, "token_major").cpu().numpy()
    kc, vc = (np.ascontiguousarray(a.transpose(1, 0, 2)) for a in (k, v))
    out_c = ctx.fkv_decode_attention(shape, dev_bf16(q), dev_bf16(kc), dev_bf16(vc), ns, "compact").cpu().numpy()
    np.testing.assert_array_equal(out_tm, out_c)
    # the same tokens scattered over pages
    need = [(n + ps - 1) // ps for n in ns]
    n_pages = sum(need) + 3
    perm = rng.permutation(n_pages)
    table = np.zeros((B, max(need)), np.int32)
    kp = np.zeros((n_pages, ps, Hkv, d), np.uint16)
    vp = np.zeros((n_pages, ps, Hkv, d), np.uint16)
    at = off = 0
    for b, n in enumerate(ns):
        table[b, :need[b]] = perm[at:at + need[b]]
        at += need[b]
        for t in range(n):
            kp[table[b, t // ps], t % ps] = k[off + t]
            vp[table[b, t // ps], t % ps] = v[off + t]
        off += n
    out_p = ctx.fkv_decode_attention_paged(shape, dev_bf16(q), dev_bf16(kp), dev_bf16(vp),
                                           torch.from_numpy(table).cuda(), ns).cpu().numpy()
    np.testing.assert_array_equal(out_p, out_tm)
    off = 0
    for b, n in enumerate(ns):
        ref = oracle.decode_attention(q[b], k[off:off + n], v[off:off + n], "token_major", scale or None, "f64")
        err = np.abs(out_tm[b] - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
        assert err.max() <= 1e-3, (b, err.max())
        off += n


@pytest.mark.parametrize("case", range(12))
def test_random_medium_batches_scores(ctx, case):
    """Ragged batches of a few thousand to tens of thousands of tokens: many blocks and clusters per
    sequence on both variants of the single-pass kernel (totals under their limits) and on the two-pass
    path (totals above)."""
    from parity import assert_scores_close
    rng = np.random.default_rng(7000 + case)
    B = int(rng.integers(1, 8))
    budget = (36000, 90000, 60000)[case % 3]   # 5-sub-tile single pass, two-pass, 8-sub-tile single pass
    cuts = np.sort(rng.integers(0, budget, size=B - 1)) if B > 1 else np.array([], np.int64)
    lengths = [max(8, int(x)) for x in np.diff(np.concatenate([[0], cuts, [budget]]))]
    pool_mode = ("avg", "max")[case % 2]
    pk = int(rng.choice([1, 7, 7, 15]))
    print("case %d: lengths=%s pool=%s %d" % (case, lengths, pool_mode, pk), flush=True)
    batch = wl.make_batch(7000 + case, lengths, with_v=False, with_x=False)
    shape = fk.make_shape(lengths if B > 1 else lengths[0], pool_mode=pool_mode, pool_kernel=pk)
    sg, st = ctx.fkv_score_window(shape, dev_bf16(batch["q_win"]), dev_bf16(batch["k"]))
    sg, st = sg.cpu().numpy(), st.cpu().numpy()
    col = 0
    for b, s_ in enumerate(batch["seqs"]):
        P = lengths[b] - 8
        ref = oracle.score_window(s_["q_win"], s_["k"], pk, pool_mode, precision="f32")
        assert_scores_close(sg[:, col:col + P], ref["scores_group"], "scores_group seq %d" % b)
        assert_scores_close(st[col:col + P], ref["scores_tsp"], "scores_tsp seq %d" % b)
        col += P


def test_gather_clamps_or_skips_indices_outside_the_sequence(ctx):
    print("case: gather with out-of-range indices", flush=True)
    lengths, ks = [100, 60], [8, 8]
    x = np.arange(160 * 8, dtype=np.uint16).reshape(160, 8)
    idx = np.array([0, 5, 99, 100, 2 ** 30, -1, -2 ** 31, 50, 0, 59, 60, 61, 10 ** 9, -5, 1, 2], np.int32)
    # an index beyond the sequence is clamped into it; a negative index (the mark of an invalid selection)
    # copies nothing, so those output rows keep what they held
    buf = torch.full((16, 8), 0x7777, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    out = host_bits(ctx.fkv_gather_rows(fk.make_shape(lengths), dev_bf16(x), torch.from_numpy(idx).cuda(), ks, out=buf))
    want = np.concatenate([x[np.clip(idx[:8], 0, 99)], x[100 + np.clip(idx[8:], 0, 59)]])
    want[idx < 0] = 0x7777
    np.testing.assert_array_equal(out, want)
