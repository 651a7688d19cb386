"""GPU parity: the HIP path through the C ABI against the CPU oracle on identical seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_01068_amd import binding as fk
from paper_2502_01068_amd import workloads as wl
from parity import assert_index_set, assert_scores_close, dev_bf16, host_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", params=["auto", "two_pass", "coop_select"])
def ctx(request):
    """Every case runs three times: with the default paths (the single-pass resident-grid score kernel
    whenever the batch fits, which all cases of this file do; one select block per row up to 16384
    keys, several above), with the two-pass score kernels, and with the several-blocks-per-row select forced for every
    call whose blocks fit the device (rows of any length, down to one slice)."""
    c = fk.Context(max_total_tokens=140000, max_seqs=16)
    c.fkv_set_score_path(1 if request.param == "two_pass" else 0)
    c.fkv_set_select_path(2 if request.param == "coop_select" else 0)
    print("paths:", request.param, flush=True)
    yield c
    assert c.fkv_query_error() == 0
    c.close()


def _oracle_batch(batch_seqs, pool_kernel, pool_mode, causal=True, scale=None, precision="f32"):
    """Oracle scores of each sequence, concatenated like the library's packed layout."""
    sg, st = [], []
    for s in batch_seqs:
        o = oracle.score_window(s["q_win"], s["k"], pool_kernel, pool_mode, scale=scale, causal=causal,
                                precision=precision)
        sg.append(o["scores_group"])
        st.append(o["scores_tsp"])
    return np.concatenate(sg, axis=1), np.concatenate(st)


# ------------------------------------------------------------------------------------ scores

@pytest.mark.parametrize("pool_mode", ["max", "avg"])
def test_scores_config1(ctx, pool_mode):
    print("case: config1 L=2048 pool=%s" % pool_mode, flush=True)
    s = wl.make_sequence(0, 2048, n_heavy=64, with_v=False, with_x=False)
    shape = fk.make_shape(2048, pool_mode=pool_mode)
    sg, st = ctx.fkv_score_window(shape, dev_bf16(s["q_win"]), dev_bf16(s["k"]))
    for prec in ("f32", "f64"):
        rg, rt = _oracle_batch([s], 7, pool_mode, precision=prec)
        e1 = assert_scores_close(sg.cpu().numpy(), rg, "scores_group/" + prec)
        e2 = assert_scores_close(st.cpu().numpy(), rt, "scores_tsp/" + prec)
        print("  max rel err vs %s oracle: group %.2e tsp %.2e" % (prec, e1, e2), flush=True)


@pytest.mark.parametrize("L,Hq,Hkv,W,pk,causal,scale", [
    (9, 32, 8, 8, 7, True, 0.0),        # one prefix token
    (40, 32, 8, 8, 7, True, 0.0),       # less than one MFMA tile
    (135, 32, 8, 8, 7, True, 0.0),      # ragged tail just past one stats chunk
    (8 + 122, 32, 8, 8, 7, True, 0.0),  # exactly one score tile
    (8 + 123, 32, 8, 8, 7, False, 0.0), # one token into the second tile, non-causal
    (1000, 8, 2, 4, 3, True, 0.0),      # W=4, G=4, Hkv=2
    (777, 8, 8, 8, 5, True, 0.0),       # G=1
    (300, 3, 3, 1, 1, True, 0.0),       # W=1, kernel 1: plain softmax row
    (500, 12, 4, 7, 9, True, 0.05),     # odd W, G=3, custom scale
    (513, 16, 8, 8, 31, True, 0.0),     # widest supported pooling kernel
    (1267, 3, 3, 4, 27, True, 0.0),     # pooling radius beyond the window: the halo of the last tokens runs past L
    (200, 4, 4, 1, 31, True, 0.0),      # ... with a one-token window
    (900, 64, 8, 8, 7, True, 0.0),      # G = 8: two row tiles per KV head, 16 virtual groups (two-pass kernels only)
    (700, 32, 4, 8, 7, True, 0.0),      # G = 8 with 4 KV heads: fits the single-pass kernel
    (650, 28, 4, 8, 7, True, 0.0),      # G = 7: the second row tile has 3 heads
    (400, 5, 1, 3, 5, False, 0.0),      # G = 5, one KV head
    (1300, 48, 8, 8, 7, True, 0.0),     # G = 6
])
@pytest.mark.parametrize("pool_mode", ["max", "avg"])
def test_scores_shapes(ctx, L, Hq, Hkv, W, pk, causal, scale, pool_mode):
    print("case: L=%d Hq=%d Hkv=%d W=%d pk=%d causal=%s scale=%g %s" % (L, Hq, Hkv, W, pk, causal, scale, pool_mode),
          flush=True)
    s = wl.make_sequence(3, L, window=W, n_q_heads=Hq, n_kv_heads=Hkv, n_heavy=min(5, L - W), with_v=False,
                         with_x=False)
    shape = fk.make_shape(L, n_q_heads=Hq, n_kv_heads=Hkv, window=W, pool_kernel=pk, pool_mode=pool_mode,
                          causal=causal, softmax_scale=scale)
    sg, st = ctx.fkv_score_window(shape, dev_bf16(s["q_win"]), dev_bf16(s["k"]))
    rg, rt = _oracle_batch([s], pk, pool_mode, causal=causal, scale=(scale or None), precision="f64")
    assert_scores_close(sg.cpu().numpy(), rg, "scores_group")
    assert_scores_close(st.cpu().numpy(), rt, "scores_tsp")


def test_scores_empty_prefix_and_no_tsp(ctx):
    print("case: L == W and scores_tsp=NULL", flush=True)
    s = wl.make_sequence(1, 8, n_heavy=0, with_v=False, with_x=False)
    shape = fk.make_shape(8)
    sg, st = ctx.fkv_score_window(shape, dev_bf16(s["q_win"]), dev_bf16(s["k"]))
    torch.cuda.synchronize()
    assert sg.shape == (8, 0) and st.shape == (0,)
    s = wl.make_sequence(1, 600, n_heavy=4, with_v=False, with_x=False)
    shape = fk.make_shape(600)
    sg, st = ctx.fkv_score_window(shape, dev_bf16(s["q_win"]), dev_bf16(s["k"]), want_tsp=False)
    assert st is None
    rg, _ = _oracle_batch([s], 7, "max", precision="f64")
    assert_scores_close(sg.cpu().numpy(), rg, "scores_group")


def test_scores_large_logits_are_stable(ctx):
    # keys 8x larger: logits of order +-30, far outside what a fixed softmax reference survives
    print("case: large logits", flush=True)
    s = wl.make_sequence(9, 700, n_heavy=6, heavy_gain=20.0, with_v=False, with_x=False)
    shape = fk.make_shape(700, softmax_scale=0.7)
    sg, st = ctx.fkv_score_window(shape, dev_bf16(s["q_win"]), dev_bf16(s["k"]))
    rg, rt = _oracle_batch([s], 7, "max", scale=0.7, precision="f64")
    assert_scores_close(sg.cpu().numpy(), rg, "scores_group")
    assert_scores_close(st.cpu().numpy(), rt, "scores_tsp")


@pytest.mark.parametrize("pool_mode", ["max", "avg"])
def test_scores_below_fp32_normal_range(ctx, pool_mode):
    """A softmax scale that pushes some scores below 2^-126: every score is still compared, with the one
    absolute floor of tests/parity.py (the kernels' exp2 returns 0 where exact arithmetic gives a sub-normal),
    and a selection that reaches down into those scores stays inside the tolerance band."""
    from parity import FLT_MIN
    print("case: scores below fp32's normal range, pool %s" % pool_mode, flush=True)
    L, W = 700, 8
    s = wl.make_sequence(9, L, n_heavy=6, heavy_gain=20.0, with_v=False, with_x=False)
    shape = fk.make_shape(L, softmax_scale=3.0, pool_mode=pool_mode)
    sg, st = ctx.fkv_score_window(shape, dev_bf16(s["q_win"]), dev_bf16(s["k"]))
    rg, rt = _oracle_batch([s], 7, pool_mode, scale=3.0, precision="f64")
    assert (rg < FLT_MIN).any() and (rg < 1e-30).mean() > 0.01, "the case is meant to reach below the normal range"
    assert_scores_close(sg.cpu().numpy(), rg, "scores_group")
    assert_scores_close(st.cpu().numpy(), rt, "scores_tsp")
    k = L - 2                      # keeps all but two prefix tokens: the threshold is one of the smallest scores
    idx = ctx.fkv_select_topk(shape, sg, k).cpu().numpy()
    for g in range(8):
        np.testing.assert_array_equal(idx[g], oracle.select_topk(sg[g].cpu().numpy(), W, k))
        assert_index_set(idx[g], oracle.select_topk(rg[g].astype(np.float32), W, k), rg[g], W, "g%d" % g)


def test_scores_huge_masked_window_logit(ctx):
    """The keys of the later window positions are masked for the earlier window rows (causal corner).  A
    masked key whose logit lies far above everything a row may see must not move that row's softmax
    reference: the last window key is made 40x a window query here, hundreds of log2 units above the
    visible logits of rows 0 .. W-2, on both score paths."""
    print("case: huge masked window-key logit", flush=True)
    L, W = 600, 8
    s = wl.make_sequence(12, L, n_heavy=4, with_v=False, with_x=False)
    qf = wl.bf16_bits_to_f32(s["q_win"])                         # [W, Hq, d]
    for g in range(8):
        s["k"][L - 1, g, :] = wl.f32_to_bf16_bits(40.0 * qf[2, 4 * g + 1, :])   # aligned with window row 2 of one head
    shape = fk.make_shape(L, pool_mode="max")
    sg, st = ctx.fkv_score_window(shape, dev_bf16(s["q_win"]), dev_bf16(s["k"]))
    rg, rt = _oracle_batch([s], 7, "max", precision="f64")
    assert np.isfinite(sg.cpu().numpy()).all()
    assert_scores_close(sg.cpu().numpy(), rg, "scores_group")
    assert_scores_close(st.cpu().numpy(), rt, "scores_tsp")


def test_scores_ragged_batch(ctx):
    lengths = [300, 1000, 57, 8, 2049, 131]
    print("case: ragged batch", lengths, flush=True)
    batch = wl.make_batch(5, lengths, n_heavy=3, with_v=False, with_x=False)
    for pool_mode in ("max", "avg"):
        shape = fk.make_shape(lengths, pool_mode=pool_mode)
        sg, st = ctx.fkv_score_window(shape, dev_bf16(batch["q_win"]), dev_bf16(batch["k"]))
        rg, rt = _oracle_batch(batch["seqs"], 7, pool_mode, precision="f64")
        assert_scores_close(sg.cpu().numpy(), rg, "scores_group")
        assert_scores_close(st.cpu().numpy(), rt, "scores_tsp")


# ------------------------------------------------------------------------------------ select

@pytest.mark.parametrize("P,ks", [
    (0, [8]), (1, [8, 9]), (5, [8, 10, 13]), (64, [8, 9, 40, 72]), (1023, [100, 1031]), (1024, [520]),
    (1025, [8, 9, 1033]), (5000, [1000, 2500, 5008]), (32760, [2048, 6554]), (131064, [13107, 26214]),
])
@pytest.mark.parametrize("ties", [0.0, 0.5])
def test_select_bit_exact(ctx, P, ks, ties):
    W, rows = 8, 3
    print("case: select P=%d ks=%s ties=%g" % (P, ks, ties), flush=True)
    scores = wl.random_scores(P + 1, rows, P, ties=ties)
    if P > 10:
        scores[1, :] = np.float32(0.125)          # a fully tied row
        scores[2, P // 3: P // 3 + 7] = scores[2].max()  # a max-pool style plateau at the top
    d = torch.from_numpy(scores).cuda()
    shape = fk.make_shape(P + W)
    for k in ks:
        idx = ctx.fkv_select_topk(shape, d, k).cpu().numpy()
        for r in range(rows):
            np.testing.assert_array_equal(idx[r], oracle.select_topk(scores[r], W, k), err_msg="row %d k %d" % (r, k))


@pytest.mark.parametrize("P,rows,ks", [
    (1000003, 2, [8, 4096, 200001]),     # 123 slices of the multi-block chain
    (40000, 66, [8008]),                 # many rows on the multi-block chain
    (33000, 260, [3000]),                # more row instances than the chain's state holds: one-block chunked kernel
    (32766, 1, [6554]), (32767, 2, [6554]),  # either side of the register-resident limit
])
def test_select_long_rows(P, rows, ks):
    W = 8
    print("case: select long rows P=%d rows=%d ks=%s" % (P, rows, ks), flush=True)
    scores = wl.random_scores(P % 1000, rows, P, ties=0.25)
    scores[rows - 1, : P // 2] = np.float32(0.5)   # half the last row tied above most of the rest
    c = fk.Context(max_total_tokens=P + W, max_seqs=1)
    try:
        d = torch.from_numpy(scores).cuda()
        shape = fk.make_shape(P + W)
        for k in ks:
            idx = c.fkv_select_topk(shape, d, k).cpu().numpy()
            for r in sorted({0, rows // 2, rows - 1}):
                np.testing.assert_array_equal(idx[r], oracle.select_topk(scores[r], W, k), err_msg="row %d k %d" % (r, k))
            for r in range(rows):  # structure of every row: ascending, unique, window at the end
                assert (np.diff(idx[r]) > 0).all() and idx[r, -W:].tolist() == list(range(P, P + W))
    finally:
        c.close()


def test_select_negative_and_zero_scores(ctx):
    # the API takes any non-NaN fp32: order must hold across sign; -0.0 and +0.0 tie (lower index wins)
    print("case: select signed scores", flush=True)
    rng = np.random.default_rng(0)
    P, W = 3000, 8
    scores = rng.standard_normal((2, P)).astype(np.float32)
    scores[0, ::7] = 0.0
    scores[0, 3::7] = -0.0
    d = torch.from_numpy(scores).cuda()
    shape = fk.make_shape(P + W)
    for k in (8, 500, 1500, 2999, 3008):
        idx = ctx.fkv_select_topk(shape, d, k).cpu().numpy()
        for r in range(2):
            np.testing.assert_array_equal(idx[r], oracle.select_topk(scores[r], W, k))


@pytest.mark.parametrize("P", [3000, 20000, 32760, 50000])
def test_select_rows_with_mass_ties_at_the_minimum(ctx, P):
    """Most of a row at its smallest value (probabilities that underflowed to zero): those keys are not
    histogrammed one by one, their count is recovered from the histogram's total."""
    print("case: select with mass ties at the minimum, P=%d" % P, flush=True)
    W = 8
    rng = np.random.default_rng(P)
    rows = []
    for frac, floor in ((0.5, 0.0), (0.9, 0.0), (0.99, 0.0), (0.9, 1e-20), (0.7, -3.5)):
        x = np.exp(3 * rng.standard_normal(P)).astype(np.float32)
        x[rng.random(P) < frac] = np.float32(floor)
        rows.append(x)
    scores = np.stack(rows)
    d = torch.from_numpy(scores).cuda()
    shape = fk.make_shape(P + W)
    for k in (W, W + 1, P // 50 + W, P // 5, P // 2, P, P + W):   # thresholds above, at and inside the tied mass
        idx = ctx.fkv_select_topk(shape, d, k).cpu().numpy()
        for r in range(len(rows)):
            np.testing.assert_array_equal(idx[r], oracle.select_topk(scores[r], W, k), err_msg="row %d k %d" % (r, k))


def test_select_ragged(ctx):
    lengths = [300, 1000, 57, 8, 2049]
    ks = [100, 8, 57, 8, 1024]
    print("case: select ragged", lengths, ks, flush=True)
    W = 8
    rows = 4
    sum_p = sum(lengths) - W * len(lengths)
    scores = wl.random_scores(77, rows, sum_p, ties=0.3)
    shape = fk.make_shape(lengths)
    idx = ctx.fkv_select_topk(shape, torch.from_numpy(scores).cuda(), ks).cpu().numpy()
    assert idx.shape == (rows, sum(ks))
    col, o = 0, 0
    for L, k in zip(lengths, ks):
        P = L - W
        for r in range(rows):
            np.testing.assert_array_equal(idx[r, o:o + k], oracle.select_topk(scores[r, col:col + P], W, k))
        col += P
        o += k


@pytest.mark.parametrize("P,rows,ks", [
    (8189, 3, [8, 9, 1000, 8197]), (8190, 2, [4000]), (16384, 9, [2048]), (16385, 9, [16393]),
    (24573, 5, [5000]), (32760, 9, [8, 2048, 6554, 32768]), (49152, 9, [9838]), (131064, 9, [13107, 26214]),
    (262136, 7, [8, 50000]),   # 8 slices of 32768 keys per row
])
def test_select_several_blocks_per_row(P, rows, ks):
    """Rows cut into slices, one block each, that agree on the threshold inside one launch: bit-exact
    against the oracle with score-like values (spread over many powers of two), heavy ties, a constant
    row, a two-valued row, a row that is mostly zeros, and a row of both signs whose range spans all of
    fp32 (four histogram exchanges)."""
    W = 8
    print("case: select, several blocks per row, P=%d rows=%d ks=%s" % (P, rows, ks), flush=True)
    rng = np.random.default_rng(P + rows)
    scores = np.exp(4.0 * rng.standard_normal((rows, P))).astype(np.float32) * np.float32(8.0 / P)
    scores[0] = wl.random_scores(P % 977, 1, P, ties=0.5)[0]
    if rows > 1:
        scores[1, :] = np.float32(0.125)
    if rows > 2:
        scores[2] = np.where(rng.random(P) < 0.3, np.float32(0.75), np.float32(0.25))
    if rows > 3:
        scores[3, rng.random(P) < 0.97] = 0.0
    if rows > 4:
        scores[4] = rng.standard_normal(P).astype(np.float32) * np.float32(1000.0)
        scores[4, ::5] = np.float32(1e-30) * rng.random(len(scores[4, ::5])).astype(np.float32)
    c = fk.Context(max_total_tokens=P + W, max_seqs=1)
    try:
        d = torch.from_numpy(scores).cuda()
        shape = fk.make_shape(P + W)
        for path in (2, 1):
            c.fkv_set_select_path(path)
            for k in ks:
                idx = c.fkv_select_topk(shape, d, k).cpu().numpy()
                for r in range(rows):
                    np.testing.assert_array_equal(idx[r], oracle.select_topk(scores[r], W, k),
                                                  err_msg="path %d row %d k %d" % (path, r, k))
        assert c.fkv_query_error() == 0
    finally:
        c.close()


def test_select_several_blocks_ragged_batch():
    """Several sequences of different lengths in one resident launch (slice counts differ per sequence)."""
    lengths = [20000, 9000, 33000, 8, 50]
    ks = [4000, 8, 33000, 8, 20]
    print("case: select, several blocks per row, ragged", lengths, ks, flush=True)
    W, rows = 8, 5
    sum_p = sum(lengths) - W * len(lengths)
    scores = wl.random_scores(78, rows, sum_p, ties=0.3)
    shape = fk.make_shape(lengths)
    c = fk.Context(max_total_tokens=sum(lengths), max_seqs=len(lengths))
    try:
        c.fkv_set_select_path(2)
        for _ in range(3):   # back-to-back launches: the epoch moves on, stale mailbox words are ignored
            idx = c.fkv_select_topk(shape, torch.from_numpy(scores).cuda(), ks).cpu().numpy()
            col, o = 0, 0
            for L, k in zip(lengths, ks):
                P = L - W
                for r in range(rows):
                    np.testing.assert_array_equal(idx[r, o:o + k], oracle.select_topk(scores[r, col:col + P], W, k))
                col += P
                o += k
        assert c.fkv_query_error() == 0
    finally:
        c.close()


def test_select_exchange_gives_up_cleanly_and_recovers():
    """Failure path of the several-blocks-per-row select, forced from the host with a wait limit of
    1 us: blocks that have to wait give up, the flag is raised, the launch ends normally with -1 in
    every index; after fkv_clear_error with the limit restored the next call is correct."""
    print("case: select exchange wait limit", flush=True)
    P, W, rows, k = 65536 - 8, 8, 9, 5000
    scores = wl.random_scores(5, rows, P, ties=0.1)
    c = fk.Context(max_total_tokens=P + W, max_seqs=1)
    try:
        d = torch.from_numpy(scores).cuda()
        shape = fk.make_shape(P + W)
        c.fkv_set_select_path(2)
        want = c.fkv_select_topk(shape, d, k).clone()
        assert c.fkv_query_error() == 0
        c.fkv_set_wait_limit(1)
        failed = 0
        for _ in range(5):
            bad = c.fkv_select_topk(shape, d, k)
            if c.fkv_query_error() == 1:
                failed += 1
                assert (bad == -1).all()   # the failure is visible in the output
                c.fkv_clear_error()
            else:                          # every wait happened to be over in time: then the result is right
                assert torch.equal(bad, want)
        print("  launches that gave up: %d of 5" % failed, flush=True)
        assert failed >= 1
        c.fkv_set_wait_limit(0)
        for _ in range(2):
            assert torch.equal(c.fkv_select_topk(shape, d, k), want)
        assert c.fkv_query_error() == 0
    finally:
        c.close()


# ------------------------------------------------------------------------------------ gathers

def test_gather_rows_and_kv_bit_exact(ctx):
    print("case: gathers", flush=True)
    rng = np.random.default_rng(4)
    lengths = [700, 64, 1500]
    ks = [200, 64, 8]
    shape = fk.make_shape(lengths)
    total = sum(lengths)
    for hidden in (4096, 40, 8):  # 8 KiB rows, 80-byte rows, one 16-byte chunk
        x = rng.integers(0, 65536, size=(total, hidden), dtype=np.uint16)
        idx = np.concatenate([np.sort(rng.choice(L, k, replace=False)) for L, k in zip(lengths, ks)]).astype(np.int32)
        out = ctx.fkv_gather_rows(shape, dev_bf16(x), torch.from_numpy(idx).cuda(), ks)
        ref = np.concatenate([oracle.gather_rows(x[c:c + L], idx[o:o + k])
                              for c, L, o, k in zip(np.cumsum([0] + lengths[:-1]), lengths,
                                                    np.cumsum([0] + ks[:-1]), ks)])
        np.testing.assert_array_equal(host_bits(out), ref)
    kk = rng.integers(0, 65536, size=(total, 8, 128), dtype=np.uint16)
    vv = rng.integers(0, 65536, size=(total, 8, 128), dtype=np.uint16)
    idx_kv = np.stack([np.concatenate([np.sort(rng.choice(L, k, replace=False)) for L, k in zip(lengths, ks)])
                       for _ in range(8)]).astype(np.int32)
    ko, vo = ctx.fkv_gather_kv(shape, dev_bf16(kk), dev_bf16(vv), torch.from_numpy(idx_kv).cuda(), ks)
    cu = np.cumsum([0] + lengths)
    oo = np.cumsum([0] + ks)
    for b in range(3):
        sl = slice(oo[b], oo[b + 1])
        np.testing.assert_array_equal(host_bits(ko)[:, sl], oracle.gather_kv(kk[cu[b]:cu[b + 1]], idx_kv[:, sl]))
        np.testing.assert_array_equal(host_bits(vo)[:, sl], oracle.gather_kv(vv[cu[b]:cu[b + 1]], idx_kv[:, sl]))
    ko2, none = ctx.fkv_gather_kv(shape, dev_bf16(kk), None, torch.from_numpy(idx_kv).cuda(), ks)
    assert none is None
    np.testing.assert_array_equal(host_bits(ko2), host_bits(ko))


# ------------------------------------------------------------------------------------ fused layer

def _check_layer(ctx, seqs, lengths, budget, k_tsp, pool_mode, what):
    """compress_kv on the GPU vs the oracle, sequence by sequence."""
    B = len(lengths)
    W = 8
    shape = fk.make_shape(lengths, pool_mode=pool_mode)
    cat = lambda n: np.concatenate([s[n] for s in seqs], axis=0)
    q = dev_bf16(np.stack([s["q_win"] for s in seqs]))
    k, v = dev_bf16(cat("k")), dev_bf16(cat("v"))
    x = dev_bf16(cat("x")) if k_tsp is not None else None
    budgets = budget if isinstance(budget, list) else [budget] * B
    ktsps = (k_tsp if isinstance(k_tsp, list) else [k_tsp] * B) if k_tsp is not None else None
    out = ctx.fkv_compress_kv(shape, q, k, v, budgets, x=x, k_tsp_per_seq=ktsps)
    sg, st = ctx.fkv_score_window(shape, q, k)   # the scores the fused call ranked (same kernels)
    torch.cuda.synchronize()
    sg, st = sg.cpu().numpy(), st.cpu().numpy()
    idx_kv = out["idx_kv"].cpu().numpy()
    k_out, v_out = host_bits(out["k_out"]), host_bits(out["v_out"])
    n_flip = 0
    col = ob = ot = 0
    for b, (s, L) in enumerate(zip(seqs, lengths)):
        P = L - W
        ref = oracle.compress_kv(s["q_win"], s["k"], s["v"], budgets[b], 7, pool_mode,
                                 x=s.get("x") if k_tsp is not None else None,
                                 k_tsp=ktsps[b] if k_tsp is not None else None)
        assert_scores_close(sg[:, col:col + P], ref["scores_group"], what + " scores_group seq %d" % b)
        for g in range(8):
            mine = idx_kv[g, ob:ob + budgets[b]]
            n_flip += assert_index_set(mine, ref["idx_kv"][g], ref["scores_group"][g], W, what + " kv g%d" % g)
            # exact with respect to the scores the GPU itself produced
            np.testing.assert_array_equal(mine, oracle.select_topk(sg[g, col:col + P], W, budgets[b]))
            # gathered rows are the rows of the GPU's own indices, bit for bit
            np.testing.assert_array_equal(k_out[g, ob:ob + budgets[b]], s["k"][mine, g])
            np.testing.assert_array_equal(v_out[g, ob:ob + budgets[b]], s["v"][mine, g])
        if k_tsp is not None:
            assert_scores_close(st[col:col + P], ref["scores_tsp"], what + " scores_tsp seq %d" % b)
            mine = out["idx_tsp"].cpu().numpy()[ot:ot + ktsps[b]]
            n_flip += assert_index_set(mine, ref["idx_tsp"], ref["scores_tsp"], W, what + " tsp")
            np.testing.assert_array_equal(mine, oracle.select_topk(st[col:col + P], W, ktsps[b]))
            np.testing.assert_array_equal(host_bits(out["x_out"])[ot:ot + ktsps[b]], s["x"][mine])
            ot += ktsps[b]
        col += P
        ob += budgets[b]
    print("  %s: index flips inside the tolerance band: %d" % (what, n_flip), flush=True)
    return out


@pytest.mark.parametrize("pool_mode", ["avg", "max"])
def test_compress_kv_config1(ctx, pool_mode):
    print("case: compress_kv config1 %s" % pool_mode, flush=True)
    s = wl.make_sequence(0, 2048, n_heavy=64)
    _check_layer(ctx, [s], [2048], 256, 512, pool_mode, "config1/" + pool_mode)


def test_compress_kv_without_tsp_and_edges(ctx):
    print("case: compress_kv edges", flush=True)
    s = wl.make_sequence(2, 700, n_heavy=8)
    _check_layer(ctx, [s], [700], 64, None, "max", "no-tsp")
    _check_layer(ctx, [s], [700], 8, 8, "max", "window only")        # k == W
    _check_layer(ctx, [s], [700], 700, 700, "avg", "identity")       # k == L
    s = wl.make_sequence(2, 8, n_heavy=0)
    _check_layer(ctx, [s], [8], 8, 8, "max", "L == W")


def test_compress_kv_ragged_batch(ctx):
    lengths = [300, 1000, 57, 2049, 131]
    print("case: compress_kv ragged", lengths, flush=True)
    batch = wl.make_batch(8, lengths, n_heavy=3)
    _check_layer(ctx, batch["seqs"], lengths, [64, 100, 57, 512, 8],
                 [wl.round_half_up(0.2 * L) for L in lengths], "max", "ragged")


@pytest.mark.parametrize("score_path", [0, 1])
def test_compress_kv_largest_batch(score_path):
    """FKV_MAX_SEQS sequences in one call, lengths from the window alone up to a few tiles."""
    rng = np.random.default_rng(5)
    lengths = [8, 9, 40, 41] + [int(x) for x in rng.integers(8, 400, size=60)]
    assert len(lengths) == 64
    print("case: compress_kv 64 sequences, score path %d" % score_path, flush=True)
    batch = wl.make_batch(9, lengths, n_heavy=2)
    budgets = [max(8, L // 3) for L in lengths]
    ktsps = [max(8, wl.round_half_up(0.2 * L)) for L in lengths]
    c = fk.Context(max_total_tokens=sum(lengths), max_seqs=64)
    try:
        c.fkv_set_score_path(score_path)
        _check_layer(c, batch["seqs"], lengths, budgets, ktsps, "max", "64 sequences")
        assert c.fkv_query_error() == 0
    finally:
        c.close()


@pytest.mark.parametrize("pool_mode", ["max", "avg"])
def test_per_head_retention(ctx, pool_mode):
    # head-wise variant: pooled per-head scores (Eq. 1), one index set per query head, per-head K/V copies
    lengths, W, budget = [900, 2100], 8, [64, 300]
    print("case: per-head retention", lengths, pool_mode, flush=True)
    batch = wl.make_batch(12, lengths, n_heavy=6, with_x=False)
    shape = fk.make_shape(lengths, pool_mode=pool_mode)
    q, k, v = dev_bf16(batch["q_win"]), dev_bf16(np.concatenate([s["k"] for s in batch["seqs"]])), \
        dev_bf16(np.concatenate([s["v"] for s in batch["seqs"]]))
    sh = ctx.fkv_score_heads(shape, q, k)
    idx = ctx.fkv_select_topk(shape, sh, budget)
    ko, vo = ctx.fkv_gather_kv_per_head(shape, k, v, idx, budget)
    sh, idx, ko, vo = sh.cpu().numpy(), idx.cpu().numpy(), host_bits(ko), host_bits(vo)
    col = o = 0
    for b, s in enumerate(batch["seqs"]):
        P = lengths[b] - W
        ref = oracle.score_window(s["q_win"], s["k"], 7, pool_mode, precision="f64")["p_head"]
        assert_scores_close(sh[:, col:col + P], ref, "scores_head seq %d" % b)
        mine = idx[:, o:o + budget[b]]
        for h in range(32):
            assert_index_set(mine[h], oracle.select_topk(ref[h].astype(np.float32), W, budget[b]), ref[h], W, "head %d" % h)
            np.testing.assert_array_equal(mine[h], oracle.select_topk(sh[h, col:col + P], W, budget[b]))
        np.testing.assert_array_equal(ko[:, o:o + budget[b]], oracle.gather_kv_per_head(s["k"], mine))
        np.testing.assert_array_equal(vo[:, o:o + budget[b]], oracle.gather_kv_per_head(s["v"], mine))
        col += P
        o += budget[b]


@pytest.mark.parametrize("Hq,Hkv", [(64, 8), (28, 4), (40, 8)])
def test_wide_groups_pipeline(ctx, Hq, Hkv):
    """Groups of more than 4 query heads (two MFMA row tiles per KV head): fused call, head-wise scores and
    head-wise gather against the oracle."""
    L, W, budget, k_tsp = 1800, 8, 200, 360
    G = Hq // Hkv
    print("case: wide groups Hq=%d Hkv=%d" % (Hq, Hkv), flush=True)
    s = wl.make_sequence(17, L, n_q_heads=Hq, n_kv_heads=Hkv, n_heavy=10, hidden=256)
    shape = fk.make_shape(L, n_q_heads=Hq, n_kv_heads=Hkv, pool_mode="max")
    q, k, v, x = (dev_bf16(s[n]) for n in ("q_win", "k", "v", "x"))
    out = ctx.fkv_compress_kv(shape, q[None], k, v, budget, x=x, k_tsp_per_seq=k_tsp)
    sg, st = ctx.fkv_score_window(shape, q[None], k)
    sh = ctx.fkv_score_heads(shape, q[None], k)
    ref = oracle.compress_kv(s["q_win"], s["k"], s["v"], budget, 7, "max", x=s["x"], k_tsp=k_tsp)
    sc = oracle.score_window(s["q_win"], s["k"], 7, "max", precision="f64")
    assert_scores_close(sg.cpu().numpy(), sc["scores_group"], "scores_group")
    assert_scores_close(st.cpu().numpy(), sc["scores_tsp"], "scores_tsp")
    assert_scores_close(sh.cpu().numpy(), sc["p_head"], "scores_head")
    idx_kv, idx_tsp = out["idx_kv"].cpu().numpy(), out["idx_tsp"].cpu().numpy()
    for g in range(Hkv):
        assert_index_set(idx_kv[g], ref["idx_kv"][g], ref["scores_group"][g], W, "kv g%d" % g)
        np.testing.assert_array_equal(host_bits(out["k_out"][g]), s["k"][idx_kv[g], g])
        np.testing.assert_array_equal(host_bits(out["v_out"][g]), s["v"][idx_kv[g], g])
    assert_index_set(idx_tsp, ref["idx_tsp"], ref["scores_tsp"], W, "tsp")
    np.testing.assert_array_equal(host_bits(out["x_out"]), s["x"][idx_tsp])
    idx_h = ctx.fkv_select_topk(shape, sh, budget)
    ko, vo = ctx.fkv_gather_kv_per_head(shape, k, v, idx_h, budget)
    idx_hh = idx_h.cpu().numpy()
    np.testing.assert_array_equal(host_bits(ko), oracle.gather_kv_per_head(s["k"], idx_hh))
    np.testing.assert_array_equal(host_bits(vo), oracle.gather_kv_per_head(s["v"], idx_hh))
    for h in (0, G - 1, G, Hq - 1):
        np.testing.assert_array_equal(idx_hh[h], oracle.select_topk(sh[h].cpu().numpy(), W, budget))


def test_deterministic(ctx):
    print("case: determinism", flush=True)
    s = wl.make_sequence(4, 3000, n_heavy=30)
    shape = fk.make_shape(3000)
    q, k, v, x = dev_bf16(s["q_win"]), dev_bf16(s["k"]), dev_bf16(s["v"]), dev_bf16(s["x"])
    a = ctx.fkv_compress_kv(shape, q, k, v, 300, x=x, k_tsp_per_seq=600)
    a = {n: t.clone() for n, t in a.items()}
    for _ in range(3):
        b = ctx.fkv_compress_kv(shape, q, k, v, 300, x=x, k_tsp_per_seq=600)
        for n in a:
            assert torch.equal(a[n].view(torch.int16) if a[n].dtype == torch.bfloat16 else a[n],
                               b[n].view(torch.int16) if b[n].dtype == torch.bfloat16 else b[n]), n


def test_single_pass_path_is_taken_and_rejects_oversize(ctx):
    print("case: forced single-pass path", flush=True)
    c2 = fk.Context(max_total_tokens=140000, max_seqs=4)
    c2.fkv_set_score_path(2)
    s = wl.make_sequence(6, 5000, n_heavy=20, with_v=False, with_x=False)
    shape = fk.make_shape(5000)
    sg, st = c2.fkv_score_window(shape, dev_bf16(s["q_win"]), dev_bf16(s["k"]))
    rg, rt = _oracle_batch([s], 7, "max", precision="f64")
    assert_scores_close(sg.cpu().numpy(), rg, "scores_group")
    assert_scores_close(st.cpu().numpy(), rt, "scores_tsp")
    big = fk.make_shape(131072)
    k = torch.zeros((131072, 8, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fk.FkvError) as ei:
        c2.fkv_score_window(big, dev_bf16(s["q_win"]), k)
    assert ei.value.status == fk.FKV_EUNSUPPORTED
    with pytest.raises(fk.FkvError):
        c2.fkv_set_score_path(3)
    assert c2.fkv_query_error() == 0
    c2.close()


def test_grid_wait_gives_up_cleanly_and_recovers():
    """Failure path of the single-pass kernel, forced from the host with a wait limit of 1 us: waves
    that have to wait give up, raise the sticky flag, write NaN scores and leave the kernel normally;
    while the flag is set a fused call marks every index -1; after fkv_clear_error with the limit
    restored the very next call is correct again."""
    print("case: single-pass grid wait limit", flush=True)
    L = 8192
    s = wl.make_sequence(21, L, with_x=False)
    c = fk.Context(max_total_tokens=L, max_seqs=1)
    try:
        shape = fk.make_shape(L, pool_mode="max")
        q, k = dev_bf16(s["q_win"]), dev_bf16(s["k"])
        c.fkv_set_score_path(1)
        want_g, want_t = (t.clone() for t in c.fkv_score_window(shape, q, k))
        c.fkv_set_score_path(2)
        assert c.fkv_query_error() == 0
        c.fkv_set_wait_limit(1)   # 1 us: far below the exchange's round trips
        for _ in range(3):
            bad_g, bad_t = c.fkv_score_window(shape, q, k)
        assert c.fkv_query_error() == 1     # also proves the launches drained: the query synchronises
        assert torch.isnan(bad_g).all() and torch.isnan(bad_t).all()   # a launch under a set flag writes nothing else
        out = c.fkv_compress_kv(shape, q, k, dev_bf16(s["v"]), 256)
        torch.cuda.synchronize()
        assert (out["idx_kv"] == -1).all()  # the failure is visible in the outputs, without a query
        c.fkv_clear_error()
        c.fkv_set_wait_limit(0)
        for _ in range(2):
            got_g, got_t = c.fkv_score_window(shape, q, k)
            assert_scores_close(got_g.cpu().numpy(), want_g.cpu().numpy(), "scores_group after recovery")
            assert_scores_close(got_t.cpu().numpy(), want_t.cpu().numpy(), "scores_tsp after recovery")
        assert c.fkv_query_error() == 0
    finally:
        c.close()


@pytest.mark.parametrize("select_path", [0, 2])
def test_two_contexts_on_two_streams(select_path):
    """Two calls in flight: two contexts, two streams, resident-grid launches chained on the GPU (the
    single-pass score kernel; with select path 2 also the several-blocks-per-row select, which the
    default path leaves alone while two contexts exist).  Every interleaved call must reproduce the
    result of the same call run alone, bit for bit."""
    print("case: two contexts on two streams, select path %d" % select_path, flush=True)
    L, budget, k_tsp = 20000, 512, 4000
    seqs = [wl.make_sequence(31 + i, L) for i in range(2)]
    ctxs = [fk.Context(max_total_tokens=L, max_seqs=1) for _ in range(2)]
    for c in ctxs:
        c.fkv_set_select_path(select_path)
    streams = [torch.cuda.Stream() for _ in range(2)]
    try:
        shape = fk.make_shape(L, pool_mode="avg")
        dev = [{n: dev_bf16(s[n]) for n in ("q_win", "k", "v", "x")} for s in seqs]
        alone = []
        for c, d in zip(ctxs, dev):
            out = c.fkv_compress_kv(shape, d["q_win"], d["k"], d["v"], budget, x=d["x"], k_tsp_per_seq=k_tsp)
            alone.append({n: t.clone() for n, t in out.items()})
        torch.cuda.synchronize()
        outs = [None, None]
        for st in streams:
            st.wait_stream(torch.cuda.current_stream())
        for it in range(6):
            for i in (0, 1):
                with torch.cuda.stream(streams[i]):
                    outs[i] = ctxs[i].fkv_compress_kv(shape, dev[i]["q_win"], dev[i]["k"], dev[i]["v"], budget,
                                                      x=dev[i]["x"], k_tsp_per_seq=k_tsp, out=outs[i])
        torch.cuda.synchronize()
        for i in (0, 1):
            for n, t in alone[i].items():
                a, b = (u.view(torch.int16) if u.dtype == torch.bfloat16 else u for u in (t, outs[i][n]))
                assert torch.equal(a, b), (i, n)
            assert ctxs[i].fkv_query_error() == 0
    finally:
        for c in ctxs:
            c.close()


@pytest.mark.parametrize("case", range(64))
def test_random_valid_shapes(ctx, case):
    """Seeded random draws over everything the boundary accepts: head counts, window, pooling kernel and
    mode, mask, scale, ragged batches, keep counts; score -> select -> K/V gather against the oracle."""
    rng = np.random.default_rng(1000 + case)
    Hkv, G, W = int(rng.integers(1, 9)), int(rng.integers(1, 9)), int(rng.integers(1, 9))
    Hq = Hkv * G
    pk = int(rng.integers(0, 16)) * 2 + 1
    causal, pool_mode = bool(rng.integers(0, 2)), ("max", "avg")[int(rng.integers(0, 2))]
    scale = float(rng.choice([0.0, 0.03, 0.1, 0.3, 1.0]))   # the larger scales push many scores below fp32's normal range
    B = int(rng.integers(1, 6))
    lengths = [int(rng.integers(W, 1500)) for _ in range(B)]
    if case % 5 == 0:
        lengths[0] = W                      # a sequence that is only its window
    ks = [int(rng.integers(W, L + 1)) for L in lengths]
    print("case %d: Hq=%d Hkv=%d W=%d pk=%d %s causal=%s scale=%g lengths=%s ks=%s" % (
        case, Hq, Hkv, W, pk, pool_mode, causal, scale, lengths, ks), flush=True)
    seqs = [wl.make_sequence(2000 + case, L, window=W, n_q_heads=Hq, n_kv_heads=Hkv, n_heavy=min(4, L - W),
                             seq=b, with_x=False) for b, L in enumerate(lengths)]
    shape = fk.make_shape(lengths if B > 1 else lengths[0], n_q_heads=Hq, n_kv_heads=Hkv, window=W,
                          pool_kernel=pk, pool_mode=pool_mode, causal=causal, softmax_scale=scale)
    q = dev_bf16(np.stack([s_["q_win"] for s_ in seqs]))
    k = dev_bf16(np.concatenate([s_["k"] for s_ in seqs]))
    v = dev_bf16(np.concatenate([s_["v"] for s_ in seqs]))
    sg, st = ctx.fkv_score_window(shape, q, k)
    idx = ctx.fkv_select_topk(shape, sg, ks)
    ko, vo = ctx.fkv_gather_kv(shape, k, v, idx, ks)
    sg_h, st_h, idx_h, ko_h, vo_h = sg.cpu().numpy(), st.cpu().numpy(), idx.cpu().numpy(), host_bits(ko), host_bits(vo)
    col = o = 0
    for b, (s_, L) in enumerate(zip(seqs, lengths)):
        P = L - W
        ref = oracle.score_window(s_["q_win"], s_["k"], pk, pool_mode, scale=(scale or None), causal=causal,
                                  precision="f64")
        assert_scores_close(sg_h[:, col:col + P], ref["scores_group"], "scores_group seq %d" % b)
        assert_scores_close(st_h[col:col + P], ref["scores_tsp"], "scores_tsp seq %d" % b)
        for g in range(Hkv):
            mine = idx_h[g, o:o + ks[b]]
            np.testing.assert_array_equal(mine, oracle.select_topk(sg_h[g, col:col + P], W, ks[b]))
            assert_index_set(mine, oracle.select_topk(ref["scores_group"][g].astype(np.float32), W, ks[b]),
                             ref["scores_group"][g], W, "seq %d g %d" % (b, g))
            np.testing.assert_array_equal(ko_h[g, o:o + ks[b]], s_["k"][mine, g])
            np.testing.assert_array_equal(vo_h[g, o:o + ks[b]], s_["v"][mine, g])
        col += P
        o += ks[b]


def test_chain_small(ctx):
    # Algorithm 1 at reduced size: 6 layers, TSP layer 2; layers after it run on the kept tokens.
    print("case: chain small", flush=True)
    L, k_tsp, budget, n_layers, tsp_layer = 1500, wl.round_half_up(0.2 * 1500), 128, 6, 2
    tokens = 0
    for layer in range(n_layers):
        Lc = L if layer <= tsp_layer else k_tsp
        tokens += Lc
        s = wl.make_sequence(21, Lc, n_heavy=10, layer=layer)
        _check_layer(ctx, [s], [Lc], min(budget, Lc), k_tsp if layer == tsp_layer else None, "max",
                     "chain layer %d" % layer)
    assert tokens == (tsp_layer + 1) * L + (n_layers - tsp_layer - 1) * k_tsp
