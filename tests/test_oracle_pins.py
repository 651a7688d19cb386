"""Pins for the CPU oracle: closed forms, library routines, brute force and invariants.

None of these re-type the oracle's own loops: each compares it with something fixed by the
mathematics (a closed form), by a library routine it must reduce to (torch CPU softmax,
pooling, sort, index_select), or by exhaustive enumeration on tiny inputs.
"""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle
from paper_2502_01068_amd import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_identities.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        name, val, _ = [t.strip() for t in line.split("|", 2)]
        out[name] = val
    return out


def _rand_bf16(rng, shape, scale=1.0):
    return wl.f32_to_bf16_bits((scale * rng.standard_normal(shape)).astype(np.float32))


def _torch_scores(q_win, k, pool_kernel, pool_mode, causal=True, scale=None):
    """The whole scoring chain built from torch CPU library ops in fp64."""
    q = torch.from_numpy(wl.bf16_bits_to_f32(q_win)).double()  # [W,Hq,d]
    kk = torch.from_numpy(wl.bf16_bits_to_f32(k)).double()     # [L,Hkv,d]
    W, Hq, d = q.shape
    L, Hkv, _ = kk.shape
    G, P = Hq // Hkv, L - W
    scale = 1.0 / math.sqrt(d) if scale is None else scale
    kh = kk.repeat_interleave(G, dim=1)                        # head h uses KV head h // G
    logits = torch.einsum("whc,lhc->hwl", q, kh) * scale       # [Hq,W,L]
    if causal:
        pos_q = torch.arange(P, L).view(1, W, 1)
        pos_k = torch.arange(L).view(1, 1, L)
        logits = logits.masked_fill(pos_k > pos_q, float("-inf"))
    att = torch.softmax(logits, dim=-1)
    s = att.sum(dim=1)[:, :P]                                  # [Hq,P]
    r = pool_kernel // 2
    if pool_mode == "max":
        p = torch.nn.functional.max_pool1d(s.unsqueeze(0), pool_kernel, stride=1, padding=r).squeeze(0)
    else:
        p = torch.nn.functional.avg_pool1d(s.unsqueeze(0), pool_kernel, stride=1, padding=r,
                                           count_include_pad=True).squeeze(0)
    sg = p.view(Hkv, G, P).mean(dim=1)
    st = p.mean(dim=0)
    return s.numpy(), p.numpy(), sg.numpy(), st.numpy()


# ----------------------------------------------------------------------------- scoring

@pytest.mark.parametrize("prec,tol", [("f32", 2e-5), ("f64", 1e-12)])
def test_single_row_is_textbook_softmax(prec, tol):
    # Hq=Hkv=1, W=1, kernel 1: the score of prefix token j is softmax(q.K^T/sqrt(d))[j] over all L keys.
    rng = np.random.default_rng(1)
    L, d = 97, 32
    q = _rand_bf16(rng, (1, 1, d))
    k = _rand_bf16(rng, (L, 1, d))
    sc = oracle.score_window(q, k, pool_kernel=1, pool_mode="max", precision=prec)
    logits = torch.from_numpy(wl.bf16_bits_to_f32(k)[:, 0, :]).double() @ \
        torch.from_numpy(wl.bf16_bits_to_f32(q)[0, 0]).double() / math.sqrt(d)
    ref = torch.softmax(logits, dim=0)[: L - 1].numpy()
    for name in ("s_head", "p_head", "scores_group"):
        np.testing.assert_allclose(sc[name][0], ref, rtol=tol, atol=0)
    np.testing.assert_allclose(sc["scores_tsp"], ref, rtol=tol, atol=0)


@pytest.mark.parametrize("causal", [True, False])
def test_equal_keys_closed_form(causal):
    # All keys equal => every visible key gets 1/(number visible): causal row w sees P+w+1 keys.
    W, Hq, Hkv, d, L = 8, 4, 2, 16, 40
    rng = np.random.default_rng(2)
    q = _rand_bf16(rng, (W, Hq, d))
    k = np.zeros((L, Hkv, d), np.uint16)
    P = L - W
    s = oracle.window_attention(q, k, causal=causal, precision="f64")
    expect = sum(1.0 / (P + w + 1) for w in range(W)) if causal else W / L
    np.testing.assert_allclose(s, expect, rtol=1e-13)
    s32 = oracle.window_attention(q, k, causal=causal, precision="f32")
    np.testing.assert_allclose(s32, expect, rtol=1e-6)


def test_causal_corner_by_hand():
    # L = W+1: one prefix token; window row w sees exactly w+2 keys.
    W, d = 8, 8
    q = _rand_bf16(np.random.default_rng(3), (W, 1, d))
    k = np.zeros((W + 1, 1, d), np.uint16)
    s = oracle.window_attention(q, k, precision="f64")
    assert s.shape == (1, 1)
    np.testing.assert_allclose(s[0, 0], sum(1.0 / (w + 2) for w in range(W)), rtol=1e-14)


@pytest.mark.parametrize("pool_mode", ["max", "avg"])
@pytest.mark.parametrize("causal", [True, False])
def test_scoring_chain_matches_library_ops(pool_mode, causal):
    rng = np.random.default_rng(4)
    W, Hq, Hkv, d, L = 8, 8, 2, 32, 150
    q = _rand_bf16(rng, (W, Hq, d), 1.5)
    k = _rand_bf16(rng, (L, Hkv, d), 1.5)
    s, p, sg, st = _torch_scores(q, k, 7, pool_mode, causal)
    o64 = oracle.score_window(q, k, 7, pool_mode, causal=causal, precision="f64")
    np.testing.assert_allclose(o64["s_head"], s, rtol=1e-11)
    np.testing.assert_allclose(o64["p_head"], p, rtol=1e-11)
    np.testing.assert_allclose(o64["scores_group"], sg, rtol=1e-11)
    np.testing.assert_allclose(o64["scores_tsp"], st, rtol=1e-11)
    o32 = oracle.score_window(q, k, 7, pool_mode, causal=causal, precision="f32")
    np.testing.assert_allclose(o32["scores_group"], sg, rtol=3e-5)
    np.testing.assert_allclose(o32["scores_tsp"], st, rtol=3e-5)


def test_group_map_is_contiguous_and_scale_is_used():
    # A key aligned with one head's queries must raise that head's group only; a custom
    # softmax scale must change the result the way the library chain says.
    rng = np.random.default_rng(5)
    W, Hq, Hkv, d, L = 4, 6, 3, 16, 60
    q = _rand_bf16(rng, (W, Hq, d))
    k = _rand_bf16(rng, (L, Hkv, d))
    for scale in (None, 0.05, 1.0):
        _, _, sg, st = _torch_scores(q, k, 3, "max", True, scale)
        o = oracle.score_window(q, k, 3, "max", scale=scale, precision="f64")
        np.testing.assert_allclose(o["scores_group"], sg, rtol=1e-11)
        np.testing.assert_allclose(o["scores_tsp"], st, rtol=1e-11)


def test_attention_mass_invariant():
    # Each window row is a probability vector over the keys it sees, so prefix mass plus
    # window-column mass equals W for every head.  Window-column mass comes from torch.
    rng = np.random.default_rng(6)
    W, Hq, Hkv, d, L = 8, 4, 1, 16, 64
    q = _rand_bf16(rng, (W, Hq, d))
    k = _rand_bf16(rng, (L, Hkv, d))
    s = oracle.window_attention(q, k, precision="f64")
    qf = torch.from_numpy(wl.bf16_bits_to_f32(q)).double()
    kf = torch.from_numpy(wl.bf16_bits_to_f32(k)).double()[:, 0]
    P = L - W
    for h in range(Hq):
        mass_win = 0.0
        for w in range(W):
            lg = kf[: P + w + 1] @ qf[w, h] / math.sqrt(d)
            mass_win += torch.softmax(lg, 0)[P:].sum().item()
        assert abs(s[h].sum() + mass_win - W) < 1e-12


def test_fp32_oracle_rounding_is_far_below_tolerance():
    s = wl.make_sequence(11, 1024, n_heavy=16, with_v=False, with_x=False)
    for mode in ("max", "avg"):
        a = oracle.score_window(s["q_win"], s["k"], 7, mode, precision="f32")
        b = oracle.score_window(s["q_win"], s["k"], 7, mode, precision="f64")
        for name in ("scores_group", "scores_tsp"):
            rel = np.abs(a[name] - b[name]) / b[name]
            assert rel.max() < 2e-5


# ----------------------------------------------------------------------------- pooling / means

@pytest.mark.parametrize("kernel", [1, 3, 7, 9])
@pytest.mark.parametrize("P", [1, 2, 5, 64])
def test_pooling_matches_library(kernel, P):
    rng = np.random.default_rng(7)
    s = rng.random((3, P))
    t = torch.from_numpy(s).unsqueeze(0)
    r = kernel // 2
    mx = torch.nn.functional.max_pool1d(t, kernel, stride=1, padding=r).squeeze(0).numpy()
    av = torch.nn.functional.avg_pool1d(t, kernel, stride=1, padding=r, count_include_pad=True).squeeze(0).numpy()
    np.testing.assert_allclose(oracle.pool_rows(s, kernel, "max", "f64"), mx, rtol=0, atol=0)
    np.testing.assert_allclose(oracle.pool_rows(s, kernel, "avg", "f64"), av, rtol=1e-14)
    if kernel == 1:
        np.testing.assert_array_equal(oracle.pool_rows(s, 1, "avg", "f64"), s)


def test_pooling_invariants():
    rng = np.random.default_rng(8)
    s = rng.random((2, 200)).astype(np.float32)
    mx = oracle.pool_rows(s, 7, "max")
    assert (mx >= s).all()
    # a single spike is replicated to exactly the 7 neighbours (exact ties)
    z = np.zeros((1, 50), np.float32)
    z[0, 20] = 1.0
    m = oracle.pool_rows(z, 7, "max")[0]
    assert (m[17:24] == 1.0).all() and m[:17].sum() == 0 and m[24:].sum() == 0
    a = oracle.pool_rows(z, 7, "avg", "f64")[0]
    np.testing.assert_allclose(a[17:24], 1 / 7, rtol=1e-15)
    # avg pooling keeps interior mass: every input is counted 7 times / 7
    inner = np.zeros((1, 100))
    inner[0, 10:90] = rng.random(80)
    np.testing.assert_allclose(oracle.pool_rows(inner, 7, "avg", "f64").sum(), inner.sum(), rtol=1e-13)


def test_head_means_library_and_consistency():
    rng = np.random.default_rng(9)
    p = rng.random((12, 33))
    sg, st = oracle.head_means(p, 3, "f64")
    np.testing.assert_allclose(sg, p.reshape(3, 4, 33).mean(1), rtol=1e-14)
    np.testing.assert_allclose(st, p.mean(0), rtol=1e-14)
    np.testing.assert_allclose(st, sg.mean(0), rtol=1e-14)  # Eq. 2 == mean of the group means
    perm = np.concatenate([np.array([1, 0, 3, 2]) + 4 * g for g in range(3)])
    sg2, _ = oracle.head_means(p[perm], 3, "f64")
    np.testing.assert_allclose(sg2, sg, rtol=1e-14)


# ----------------------------------------------------------------------------- top-k

def _brute_force(scores, kp):
    """Lexicographically smallest subset of size kp in which every kept score >= every
    dropped score, found by enumerating all subsets."""
    P = len(scores)
    for sub in itertools.combinations(range(P), kp):  # lexicographic order
        kept = set(sub)
        lo = min((scores[i] for i in sub), default=math.inf)
        hi = max((scores[i] for i in range(P) if i not in kept), default=-math.inf)
        if lo >= hi:
            return list(sub)
    raise AssertionError("no admissible subset")


@pytest.mark.parametrize("seed", range(6))
def test_topk_brute_force_tiny(seed):
    rng = np.random.default_rng(100 + seed)
    W = 3
    for P in (1, 2, 5, 9, 12):
        # few distinct values => many exact ties
        scores = rng.integers(0, 4, size=P).astype(np.float32) / 8
        for kp in range(0, P + 1):
            got = oracle.select_topk(scores, W, kp + W)
            want = _brute_force(scores.tolist(), kp) + list(range(P, P + W))
            assert got.tolist() == want, (P, kp, scores)


def test_topk_brute_force_L64():
    rng = np.random.default_rng(42)
    P, W = 56, 8  # L = 64
    scores = (rng.integers(0, 30, size=P) / 64).astype(np.float32)
    for kp in (0, 1, 2, 3, 53, 54, 55, 56):  # C(56, kp) small enough to enumerate
        got = oracle.select_topk(scores, W, kp + W)
        want = _brute_force(scores.tolist(), kp) + list(range(P, P + W))
        assert got.tolist() == want


def test_topk_invariants_and_library_sort():
    P, W = 5000, 8
    scores = wl.random_scores(3, 1, P, ties=0.3)[0]
    prev = None
    for k in (8, 9, 100, 1000, 2500, 5008):
        idx = oracle.select_topk(scores, W, k)
        assert len(idx) == k and (np.diff(idx) > 0).all()
        assert idx[-W:].tolist() == list(range(P, P + W))
        kept = np.zeros(P, bool)
        kept[idx[:-W]] = True
        if kept.any() and (~kept).any():
            assert scores[kept].min() >= scores[~kept].max()
            tau = scores[kept].min()
            # among ties at the threshold the kept ones come first
            eq = np.nonzero(scores == tau)[0]
            flags = kept[eq]
            assert not (np.diff(flags.astype(int)) > 0).any()
        if prev is not None:
            assert set(prev[:-W].tolist()) <= set(idx[:-W].tolist())  # nested
        prev = idx
    # stable library sort on (-score) breaks ties to the lower index too
    order = torch.sort(torch.from_numpy(-scores), stable=True).indices.numpy()
    for k in (50, 2500):
        want = np.sort(order[: k - W])
        np.testing.assert_array_equal(oracle.select_topk(scores, W, k)[:-W], want)


def test_topk_degenerate():
    W = 8
    flat = np.full(100, 0.25, np.float32)
    assert oracle.select_topk(flat, W, 30).tolist() == list(range(22)) + list(range(100, 108))
    assert oracle.select_topk(flat, W, 108).tolist() == list(range(108))  # k = L is the identity
    assert oracle.select_topk(flat, W, 8).tolist() == list(range(100, 108))
    assert oracle.select_topk(np.zeros(0, np.float32), W, 8).tolist() == list(range(8))
    with pytest.raises(ValueError):
        oracle.select_topk(flat, W, 7)
    with pytest.raises(ValueError):
        oracle.select_topk(flat, W, 109)


# ----------------------------------------------------------------------------- gathers / chain

def test_gather_matches_library_and_composes():
    rng = np.random.default_rng(12)
    x = rng.integers(0, 65536, size=(300, 24), dtype=np.uint16)
    i1 = np.sort(rng.choice(300, 120, replace=False)).astype(np.int32)
    i2 = np.sort(rng.choice(120, 40, replace=False)).astype(np.int32)
    g1 = oracle.gather_rows(x, i1)
    ref = torch.index_select(torch.from_numpy(x.astype(np.int32)), 0, torch.from_numpy(i1).long()).numpy()
    np.testing.assert_array_equal(g1, ref.astype(np.uint16))
    np.testing.assert_array_equal(oracle.gather_rows(x, np.arange(300)), x)
    np.testing.assert_array_equal(oracle.gather_rows(g1, i2), oracle.gather_rows(x, i1[i2]))
    kv = rng.integers(0, 65536, size=(50, 3, 8), dtype=np.uint16)
    idx = np.stack([np.sort(rng.choice(50, 7, replace=False)) for _ in range(3)]).astype(np.int32)
    out = oracle.gather_kv(kv, idx)
    for g in range(3):
        np.testing.assert_array_equal(out[g], kv[idx[g], g, :])
    with pytest.raises(IndexError):
        oracle.gather_rows(x, np.array([300], np.int32))


def test_gather_kv_per_head_matches_library():
    rng = np.random.default_rng(13)
    kv = rng.integers(0, 65536, size=(40, 2, 8), dtype=np.uint16)
    idx = np.stack([np.sort(rng.choice(40, 5, replace=False)) for _ in range(6)]).astype(np.int32)
    out = oracle.gather_kv_per_head(kv, idx)
    for h in range(6):
        ref = torch.index_select(torch.from_numpy(kv[:, h // 3].astype(np.int32)), 0, torch.from_numpy(idx[h]).long())
        np.testing.assert_array_equal(out[h], ref.numpy().astype(np.uint16))


def test_compress_kv_composition_and_heavy_recall():
    s = wl.make_sequence(5, 1024, n_heavy=32)
    out = oracle.compress_kv(s["q_win"], s["k"], s["v"], 128, 7, "max", x=s["x"], k_tsp=256)
    assert out["idx_kv"].shape == (8, 128) and out["idx_tsp"].shape == (256,)
    for g in range(8):
        np.testing.assert_array_equal(out["k_out"][g], s["k"][out["idx_kv"][g], g])
        np.testing.assert_array_equal(out["v_out"][g], s["v"][out["idx_kv"][g], g])
    np.testing.assert_array_equal(out["x_out"], s["x"][out["idx_tsp"]])
    # planted heavy positions are far more likely to be kept than chance (sanity, not a gate)
    recall = np.isin(s["heavy"], out["idx_tsp"]).mean()
    assert recall > 0.8


# ----------------------------------------------------------------------------- paged cache layout

def test_paged_gather_round_trip_and_decode_equivalence():
    rng = np.random.default_rng(41)
    L, Hkv, d, b, ps, n_pages = 90, 2, 16, 37, 8, 11
    kv = _rand_bf16(rng, (L, Hkv, d))
    vv = _rand_bf16(rng, (L, Hkv, d))
    idx = np.stack([np.sort(rng.choice(L, b, replace=False)) for _ in range(Hkv)]).astype(np.int32)
    table = rng.permutation(n_pages)[:(b + ps - 1) // ps].astype(np.int32)      # 5 scattered pages
    before = _rand_bf16(rng, (n_pages, ps, Hkv, d))
    pages = oracle.gather_kv_paged(kv, idx, table, before)
    # reading the pages back in logical order gives the compact gather (library index ops)
    view = oracle.paged_view(pages, table, b)
    compact = oracle.gather_kv(kv, idx)
    np.testing.assert_array_equal(view.transpose(1, 0, 2), compact)
    for g in range(Hkv):
        np.testing.assert_array_equal(view[:, g], kv[idx[g], g])
    # nothing else is touched: unused pages and the unused tail of the last page keep their content
    touched = np.zeros((n_pages, ps), bool)
    for t in range(b):
        touched[table[t // ps], t % ps] = True
    assert touched.sum() == b
    np.testing.assert_array_equal(pages[~touched], before[~touched])
    # an identity block table over a fresh pool is the token-major compact cache itself
    ident = oracle.gather_kv_paged(kv, idx, np.arange(5), np.zeros((5, ps, Hkv, d), np.uint16))
    np.testing.assert_array_equal(ident.reshape(5 * ps, Hkv, d)[:b].transpose(1, 0, 2), compact)
    # decoding over the paged view equals decoding over the compact cache, bit for bit
    vpages = oracle.gather_kv_paged(vv, idx, table, before)
    q = _rand_bf16(rng, (4, d))
    a = oracle.decode_attention(q, view, oracle.paged_view(vpages, table, b), "token_major")
    c = oracle.decode_attention(q, compact, oracle.gather_kv(vv, idx), "compact")
    np.testing.assert_array_equal(a, c)
    with pytest.raises(IndexError):
        oracle.gather_kv_paged(kv, idx, np.full(5, n_pages), before)


# ----------------------------------------------------------------------------- diagnostics (Sec. 3)

def test_index_overlap_matches_library_and_sets():
    rng = np.random.default_rng(31)
    for n_a, n_b, hi in ((0, 5, 20), (7, 0, 20), (12, 9, 20), (300, 512, 2000), (512, 512, 600)):
        a = np.sort(rng.choice(hi, n_a, replace=False)).astype(np.int32)
        b = np.sort(rng.choice(hi, n_b, replace=False)).astype(np.int32)
        want = len(set(a.tolist()) & set(b.tolist()))
        assert oracle.index_overlap(a, b) == want == np.intersect1d(a, b).size
        assert oracle.index_overlap(b, a) == want          # symmetric
        assert oracle.index_overlap(a, a) == n_a            # a set overlaps itself completely
    assert oracle.index_overlap(np.arange(0, 40, 2), np.arange(1, 40, 2)) == 0   # interleaved, disjoint
    # nested kept sets (a smaller budget's set is inside a larger budget's): the overlap is the smaller size
    sc = wl.random_scores(3, 1, 500)[0]
    small, large = oracle.select_topk(sc, 8, 60), oracle.select_topk(sc, 8, 200)
    assert oracle.index_overlap(small, large) == 60


def test_mass_recall_closed_forms_and_exact_sums():
    from fractions import Fraction
    rng = np.random.default_rng(32)
    P = 257
    sc = rng.random(P).astype(np.float32) ** 4
    every = np.arange(P + 8)                                # prefix and the 8 window positions behind it
    assert oracle.mass_recall(sc, every) == 1.0             # everything kept: all of the mass
    assert oracle.mass_recall(sc, np.arange(P, P + 8)) == 0.0   # window positions carry no score
    assert oracle.mass_recall(np.zeros(9, np.float32), np.arange(4)) == 0.0
    # uniform mass: the recall is the kept share of the prefix
    assert abs(oracle.mass_recall(np.full(P, 0.25, np.float32), np.arange(0, 100)) - 100 / P) < 1e-15
    # all mass on one token: 1 if it is kept, else 0
    one = np.zeros(P, np.float32)
    one[41] = 3.0
    assert oracle.mass_recall(one, [3, 41, 200]) == 1.0 and oracle.mass_recall(one, [3, 40, 200]) == 0.0
    # a set and its complement split the mass; exact rational arithmetic bounds the fp64 rounding
    idx = np.sort(rng.choice(P, 60, replace=False))
    rest = np.setdiff1d(np.arange(P), idx)
    assert abs(oracle.mass_recall(sc, idx) + oracle.mass_recall(sc, rest) - 1.0) < 1e-14
    exact = sum(Fraction(float(sc[j])) for j in idx) / sum(Fraction(float(x)) for x in sc)
    assert abs(oracle.mass_recall(sc, idx) - float(exact)) < 1e-14
    # the top-k set of a row has the largest recall of any set of its size (brute force, tiny row)
    tiny = rng.random(9).astype(np.float32)
    best = oracle.mass_recall(tiny, oracle.select_topk(tiny, 0, 4))
    for comb in itertools.combinations(range(9), 4):
        assert oracle.mass_recall(tiny, comb) <= best + 1e-15


# ----------------------------------------------------------------------------- decode over the cache

@pytest.mark.parametrize("layout", ["compact", "token_major"])
def test_decode_attention_matches_library(layout):
    rng = np.random.default_rng(21)
    Hq, Hkv, d, n = 6, 2, 16, 37
    q = _rand_bf16(rng, (Hq, d), 1.5)
    k = _rand_bf16(rng, (Hkv, n, d), 1.5)
    v = _rand_bf16(rng, (Hkv, n, d))
    qf, kf, vf = (torch.from_numpy(wl.bf16_bits_to_f32(a)).double() for a in (q, k, v))
    for scale in (None, 0.3):
        sc = 1 / math.sqrt(d) if scale is None else scale
        att = torch.softmax(torch.einsum("hc,htc->ht", qf, kf.repeat_interleave(3, 0)) * sc, dim=-1)
        ref = torch.einsum("ht,htc->hc", att, vf.repeat_interleave(3, 0)).numpy()
        kk, vv = (k, v) if layout == "compact" else (np.ascontiguousarray(k.transpose(1, 0, 2)),
                                                      np.ascontiguousarray(v.transpose(1, 0, 2)))
        np.testing.assert_allclose(oracle.decode_attention(q, kk, vv, layout, scale, "f64"), ref, rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(oracle.decode_attention(q, kk, vv, layout, scale, "f32"), ref, rtol=2e-4, atol=2e-5)


def test_decode_attention_closed_forms():
    rng = np.random.default_rng(22)
    Hq, Hkv, d, n = 4, 2, 8, 9
    q = _rand_bf16(rng, (Hq, d))
    v = _rand_bf16(rng, (Hkv, n, d))
    vf = wl.bf16_bits_to_f32(v).astype(np.float64)
    # equal keys: uniform weights, the output is the mean of the group's value rows
    out = oracle.decode_attention(q, np.zeros((Hkv, n, d), np.uint16), v, precision="f64")
    for h in range(Hq):
        np.testing.assert_allclose(out[h], vf[h // 2].mean(0), rtol=1e-13, atol=1e-15)
    # a single cached token: the output is its value row exactly
    out = oracle.decode_attention(q, _rand_bf16(rng, (Hkv, 1, d)), v[:, :1], precision="f32")
    for h in range(Hq):
        np.testing.assert_array_equal(out[h], wl.bf16_bits_to_f32(v[h // 2, 0]))
    # one key far more aligned with the query than the others: the output approaches its value row
    k = np.zeros((Hkv, n, d), np.float32)
    qf = wl.bf16_bits_to_f32(q)
    k[0, 4] = 40 * qf[0]
    out = oracle.decode_attention(q, wl.f32_to_bf16_bits(k), v, scale=1.0, precision="f64")
    np.testing.assert_allclose(out[0], vf[0, 4], atol=1e-6)


@pytest.mark.parametrize("causal", [True, False])
def test_window_output_matches_library_attention(causal):
    """The last W rows of a full causal attention (library softmax / matrix products, fp64)."""
    rng = np.random.default_rng(31)
    L, W, Hq, Hkv, d = 45, 8, 6, 2, 16
    q_all = _rand_bf16(rng, (L, Hq, d), 1.5)
    k = _rand_bf16(rng, (L, Hkv, d), 1.5)
    v = _rand_bf16(rng, (L, Hkv, d))
    qf, kf, vf = (torch.from_numpy(wl.bf16_bits_to_f32(a)).double() for a in (q_all, k, v))
    kf, vf = kf.repeat_interleave(3, 1), vf.repeat_interleave(3, 1)
    for scale in (None, 0.4):
        sc = 1 / math.sqrt(d) if scale is None else scale
        z = torch.einsum("ihc,jhc->hij", qf, kf) * sc
        if causal:
            z = z.masked_fill(torch.triu(torch.ones(L, L, dtype=torch.bool), 1), -math.inf)
        ref = torch.einsum("hij,jhc->ihc", torch.softmax(z, dim=-1), vf)[L - W:].numpy()
        got = oracle.window_output(q_all[L - W:], k, v, scale, causal, "f64")
        np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-13)
        got32 = oracle.window_output(q_all[L - W:], k, v, scale, causal, "f32")
        np.testing.assert_allclose(got32, ref, rtol=2e-4, atol=2e-5)


def test_window_output_closed_forms_and_structure():
    rng = np.random.default_rng(32)
    L, W, Hq, Hkv, d = 29, 8, 4, 2, 8
    P = L - W
    q = _rand_bf16(rng, (W, Hq, d))
    k = _rand_bf16(rng, (L, Hkv, d))
    v = _rand_bf16(rng, (L, Hkv, d))
    vf = wl.bf16_bits_to_f32(v).astype(np.float64)
    # equal keys: row w is the mean of the value rows it can see (P + w + 1 of them when causal)
    out = oracle.window_output(q, np.zeros_like(k), v, precision="f64")
    for w in range(W):
        for h in range(Hq):
            np.testing.assert_allclose(out[w, h], vf[: P + w + 1, h // 2].mean(0), rtol=1e-13, atol=1e-15)
    out = oracle.window_output(q, np.zeros_like(k), v, causal=False, precision="f64")
    np.testing.assert_allclose(out[3, 1], vf[:, 0].mean(0), rtol=1e-13, atol=1e-15)
    # each window row is the decoding step of its own query over the keys it can see
    out = oracle.window_output(q, k, v, precision="f64")
    for w in range(W):
        n = P + w + 1
        ref = oracle.decode_attention(q[w], k[:n], v[:n], "token_major", precision="f64")
        np.testing.assert_allclose(out[w], ref, rtol=1e-12, atol=1e-14)
    # a key after position P + w must not reach row w: change the last token, rows 0..W-2 keep their bits
    k2, v2 = k.copy(), v.copy()
    k2[L - 1], v2[L - 1] = _rand_bf16(rng, (Hkv, d), 3.0), _rand_bf16(rng, (Hkv, d), 3.0)
    out2 = oracle.window_output(q, k2, v2, precision="f64")
    np.testing.assert_array_equal(out2[: W - 1], out[: W - 1])
    assert np.abs(out2[W - 1] - out[W - 1]).max() > 1e-3
    # the output is linear in V and its weights are the probabilities Eq. 1 sums: with v[j] = e_c * [j == j0]
    # the window rows add up to the un-pooled window-summed score of token j0
    j0 = 5
    onehot = np.zeros((L, Hkv, d), np.float32)
    onehot[j0, :, 2] = 1.0
    o = oracle.window_output(q, k, wl.f32_to_bf16_bits(onehot), precision="f64")
    s = oracle.window_attention(q, k, precision="f64")
    np.testing.assert_allclose(o[:, :, 2].sum(0), s[:, j0], rtol=1e-12)
    assert np.abs(o[:, :, :2]).max() == 0.0
    # constant value rows come back unchanged (the weights of a row add up to one)
    const = np.broadcast_to(wl.bf16_bits_to_f32(_rand_bf16(rng, (1, Hkv, d))), (L, Hkv, d))
    o = oracle.window_output(q, k, wl.f32_to_bf16_bits(np.ascontiguousarray(const)), precision="f64")
    for h in range(Hq):
        np.testing.assert_allclose(o[:, h], np.broadcast_to(const[0, h // 2], (W, d)), rtol=1e-13)


def test_paper_identities():
    g = _gold()
    n_layers, tsp_layer, rate = int(g["n_layers_llama"]), int(g["tsp_layer_llama"]), float(g["tsp_rate"])
    # Algorithm 1: layers 0..L_TSP see the full context, later layers the kept fraction.
    full = tsp_layer + 1
    compute_rate = (full * 1.0 + (n_layers - full) * rate) / n_layers
    assert abs(compute_rate - float(g["prefill_compute_rate"])) < 1e-12
    L = 32768
    k = wl.round_half_up(rate * L)
    assert k == 6554 and wl.round_half_up(0.2 * 131072) == 26214 and wl.round_half_up(0.1 * 131072) == 13107
    assert full * L + (n_layers - full) * k == 16 * 32768 + 16 * 6554
    # printed as 0.38 %; 512 / 131072 is 0.39 %: arithmetic sanity only
    assert abs(100 * 512 / 131072 - float(g["topk_fraction_512_of_128k_percent"])) < 0.015
    assert int(g["window_size"]) == 8 and int(g["pool_kernel"]) == 7 and g["pool_type"] == "max"


def test_workload_recipe():
    a = wl.make_sequence(0, 512, n_heavy=8)
    b = wl.make_sequence(0, 512, n_heavy=8)
    for name in ("q_win", "k", "v", "x", "heavy"):
        np.testing.assert_array_equal(a[name], b[name])
    assert a["heavy"].max() < 512 - 8 and len(np.unique(a["heavy"])) == 8
    kf = wl.bf16_bits_to_f32(a["k"])
    assert abs(kf.std() - 1.0) < 0.05
    # bf16 rounding is round-to-nearest-even and matches torch's
    f = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    ref = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(wl.f32_to_bf16_bits(f), ref)
    assert wl.algorithmic_bytes(32768, 6554, 2048) == 193874576
    # the per-config totals of the byte model: K once, scores and indices written + read once, rows read + written
    assert round(wl.algorithmic_bytes(2048, 512, 256) / 1e6, 1) == 14.9
    assert round(wl.algorithmic_bytes(131072, 26214, 13107) / 1e6, 1) == 815.8
    L, k, b = 32768, 6554, 2048
    by_hand = (L * 8 * 128 * 2 + 8 * 32 * 128 * 2 + 2 * 4 * 9 * (L - 8) + 2 * 4 * (k + 8 * b)
               + 2 * k * 4096 * 2 + 2 * 2 * 8 * b * 128 * 2)
    assert wl.algorithmic_bytes(L, k, b) == by_hand
