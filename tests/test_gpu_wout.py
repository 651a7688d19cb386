"""GPU parity of the window rows' attention output (fkv_window_output) against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_01068_amd import binding as fk
from paper_2502_01068_amd import workloads as wl
from parity import dev_bf16

pytestmark = pytest.mark.gpu
# Relative to the largest magnitude of the output row (outputs are signed sums that may cancel).  The
# kernel keeps 16 bits of every probability and accumulates in fp32: 2^-17 per term, far below this.
TOL = 1e-4


def _close(gpu, ref, what):
    gpu, ref = np.asarray(gpu, np.float64), np.asarray(ref, np.float64)
    assert gpu.shape == ref.shape, what
    assert np.isfinite(gpu).all(), what
    scale = np.abs(ref).max(axis=-1, keepdims=True)
    err = np.abs(gpu - ref) / scale
    assert err.max() <= TOL, "%s: max error %.3g of the row scale" % (what, err.max())
    return float(err.max())


@pytest.fixture(scope="module")
def ctx():
    c = fk.Context(max_total_tokens=40000, max_seqs=8)
    yield c
    c.close()


def _run(ctx, lens, Hq, Hkv, W=8, scale=0.0, causal=True, seed=70, q_scale=1.0):
    B, d, tot = len(lens), 128, sum(lens)
    q = wl.normal_bf16(seed, 0, "q_win", (B, W, Hq, d))
    if q_scale != 1.0:
        q = wl.f32_to_bf16_bits(wl.bf16_bits_to_f32(q) * q_scale)
    k = wl.normal_bf16(seed, 0, "k", (tot, Hkv, d))
    v = wl.normal_bf16(seed, 0, "v", (tot, Hkv, d))
    shape = fk.make_shape(lens, n_q_heads=Hq, n_kv_heads=Hkv, window=W, softmax_scale=scale, causal=causal)
    out = ctx.fkv_window_output(shape, dev_bf16(q), dev_bf16(k), dev_bf16(v))
    torch.cuda.synchronize()
    assert ctx.fkv_query_error() == 0
    out = out.cpu().numpy()
    worst, o = 0.0, 0
    for b, n in enumerate(lens):
        ref = oracle.window_output(q[b], k[o:o + n], v[o:o + n], scale or None, causal, "f64")
        worst = max(worst, _close(out[b], ref, "seq %d" % b))
        o += n
    return worst


@pytest.mark.parametrize("L", [8, 9, 31, 32, 33, 40, 255, 256, 257, 2048, 5000, 8200])
def test_window_output_lengths(ctx, L):
    print("case: window output L=%d" % L, flush=True)
    print("  worst %.2e" % _run(ctx, [L], 32, 8), flush=True)


@pytest.mark.parametrize("Hq,Hkv,W,scale,causal", [
    (32, 8, 8, 0.0, False), (8, 8, 8, 0.25, True), (12, 4, 8, 0.0, True), (64, 8, 8, 0.0, True),
    (28, 4, 8, 0.0, True), (32, 8, 4, 0.0, True), (32, 8, 1, 0.0, True), (16, 2, 5, 0.05, False),
])
def test_window_output_shapes(ctx, Hq, Hkv, W, scale, causal):
    print("case: window output Hq=%d Hkv=%d W=%d scale=%g causal=%d" % (Hq, Hkv, W, scale, causal), flush=True)
    print("  worst %.2e" % _run(ctx, [1333], Hq, Hkv, W, scale, causal), flush=True)


def test_window_output_ragged_batch(ctx):
    print("case: window output ragged batch", flush=True)
    print("  worst %.2e" % _run(ctx, [300, 8, 2049, 64, 4097, 33], 32, 8), flush=True)
    print("  worst %.2e" % _run(ctx, [777, 1500], 64, 8, seed=71), flush=True)


def test_window_output_peaked_rows(ctx):
    """Large query norms make every row put almost all of its weight on a few keys: the case where
    rounding the probabilities to 8 bits would show (the kernel keeps 16)."""
    print("case: window output peaked rows", flush=True)
    print("  worst %.2e" % _run(ctx, [3000], 32, 8, q_scale=6.0, seed=72), flush=True)
    print("  worst %.2e" % _run(ctx, [3000], 32, 8, scale=1.0, seed=73), flush=True)


def test_window_output_equal_keys_and_repeatability(ctx):
    print("case: window output equal keys / repeatability", flush=True)
    L, Hq, Hkv, d, W = 1000, 32, 8, 128, 8
    q = wl.normal_bf16(74, 0, "q_win", (1, W, Hq, d))
    v = wl.normal_bf16(74, 0, "v", (L, Hkv, d))
    shape = fk.make_shape(L)
    k0 = torch.zeros((L, Hkv, d), dtype=torch.bfloat16, device="cuda")
    out = ctx.fkv_window_output(shape, dev_bf16(q), k0, dev_bf16(v)).cpu().numpy()[0]
    vf = wl.bf16_bits_to_f32(v).astype(np.float64)
    for w in range(W):
        mean = vf[: L - W + w + 1].mean(0)   # [Hkv, d]
        _close(out[w], np.repeat(mean, Hq // Hkv, axis=0), "row %d" % w)
    k = dev_bf16(wl.normal_bf16(74, 0, "k", (L, Hkv, d)))
    a = ctx.fkv_window_output(shape, dev_bf16(q), k, dev_bf16(v)).clone()
    b = ctx.fkv_window_output(shape, dev_bf16(q), k, dev_bf16(v))
    assert torch.equal(a, b)


def test_window_output_rejects_bad_arguments(ctx):
    shape = fk.make_shape(64)
    q = torch.zeros((1, 8, 32, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((64, 8, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fk.FkvError) as e:
        ctx.fkv_window_output(shape, q, k, k, out=torch.zeros((8 * 32 * 128 + 1,), dtype=torch.float32, device="cuda")[1:])
    assert e.value.status == fk.FKV_EALIGN
    big = fk.make_shape(50000)
    with pytest.raises(ValueError):           # the binding stops a tensor shorter than the descriptor says
        ctx.fkv_window_output(big, q, k, k)
    kbig = torch.zeros((50000, 8, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fk.FkvError) as e:
        ctx.fkv_window_output(big, q, kbig, kbig)
    assert e.value.status == fk.FKV_EWORKSPACE


def test_window_output_full_size_32k():
    """Config 2's layer (workload recipe with planted heavy keys), every output row against the oracle."""
    print("case: window output at L=32768, all rows", flush=True)
    L = 32768
    s = wl.make_sequence(0, L, with_x=False)
    c = fk.Context(max_total_tokens=L, max_seqs=1)
    out = c.fkv_window_output(fk.make_shape(L), dev_bf16(s["q_win"]), dev_bf16(s["k"]), dev_bf16(s["v"])).cpu().numpy()[0]
    print("  gpu done", flush=True)
    ref = oracle.window_output(s["q_win"], s["k"], s["v"], precision="f64")
    print("  worst %.2e" % _close(out, ref, "L=32768"), flush=True)
    c.close()


def test_window_output_full_size_128k_sampled():
    """131072 tokens: the heads of two KV groups against the oracle run on those groups alone."""
    print("case: window output at L=131072, sampled groups", flush=True)
    L = 131072
    s = wl.make_sequence(1, L, with_x=False)
    c = fk.Context(max_total_tokens=L, max_seqs=1)
    out = c.fkv_window_output(fk.make_shape(L), dev_bf16(s["q_win"]), dev_bf16(s["k"]), dev_bf16(s["v"])).cpu().numpy()[0]
    print("  gpu done", flush=True)
    for g in (2, 7):
        ref = oracle.window_output(np.ascontiguousarray(s["q_win"][:, 4 * g:4 * g + 4]), np.ascontiguousarray(s["k"][:, g:g + 1]),
                                   np.ascontiguousarray(s["v"][:, g:g + 1]), precision="f64")
        print("  group %d worst %.2e" % (g, _close(out[:, 4 * g:4 * g + 4], ref, "group %d" % g)), flush=True)
    c.close()


def test_window_output_many_sequences_and_many_splits():
    """40 short sequences (one block per sequence and group) and one KV head over 70000 tokens (256 splits)."""
    print("case: window output, 40 sequences", flush=True)
    c = fk.Context(max_total_tokens=80000, max_seqs=40)
    rng = np.random.default_rng(5)
    lens = [int(n) for n in rng.integers(8, 700, size=40)]
    print("  worst %.2e" % _run(c, lens, 32, 8, seed=75), flush=True)
    print("case: window output, one KV head, 70000 tokens", flush=True)
    print("  worst %.2e" % _run(c, [70000], 4, 1, seed=76), flush=True)
    print("  worst %.2e" % _run(c, [70001], 2, 2, W=3, seed=77), flush=True)
    c.close()


# ---- scores and window output in one call (fkv_score_window_output) ----------------------------------

@pytest.mark.parametrize("lens,Hq,Hkv,W,pk,pool_mode,scale,causal", [
    ([2048], 32, 8, 8, 7, "avg", 0.0, True),
    ([2048], 32, 8, 8, 7, "max", 0.0, True),
    ([9], 32, 8, 8, 7, "max", 0.0, True),
    ([8], 32, 8, 8, 7, "max", 0.0, True),              # no prefix token: only the output exists
    ([300, 8, 2049, 64, 4097, 33], 32, 8, 8, 7, "avg", 0.0, True),
    ([1333], 12, 4, 7, 9, "max", 0.05, True),
    ([1333], 16, 2, 5, 3, "avg", 0.0, False),
    ([900], 64, 8, 8, 7, "max", 0.0, True),            # G = 8: two row tiles per KV head
    ([1267], 3, 3, 4, 27, "avg", 0.0, True),           # pooling radius beyond the window
])
def test_score_window_output_against_oracle(ctx, lens, Hq, Hkv, W, pk, pool_mode, scale, causal):
    from parity import assert_scores_close
    print("case: scores + window output lens=%s Hq=%d Hkv=%d W=%d pk=%d %s" % (lens, Hq, Hkv, W, pk, pool_mode), flush=True)
    B, d, tot = len(lens), 128, sum(lens)
    q = wl.normal_bf16(80, 0, "q_win", (B, W, Hq, d))
    k = wl.normal_bf16(80, 0, "k", (tot, Hkv, d))
    v = wl.normal_bf16(80, 0, "v", (tot, Hkv, d))
    shape = fk.make_shape(lens, n_q_heads=Hq, n_kv_heads=Hkv, window=W, pool_kernel=pk, pool_mode=pool_mode,
                          softmax_scale=scale, causal=causal)
    dq, dk, dv = dev_bf16(q), dev_bf16(k), dev_bf16(v)
    sg, st, out = ctx.fkv_score_window_output(shape, dq, dk, dv)
    alone = ctx.fkv_window_output(shape, dq, dk, dv)
    torch.cuda.synchronize()
    assert torch.equal(out, alone)            # the same kernels formed it: bit-identical
    sg, st, out = sg.cpu().numpy(), st.cpu().numpy(), out.cpu().numpy()
    o = col = 0
    for b, n in enumerate(lens):
        P = n - W
        ref_o = oracle.window_output(q[b], k[o:o + n], v[o:o + n], scale or None, causal, "f64")
        _close(out[b], ref_o, "out seq %d" % b)
        ref = oracle.score_window(q[b], k[o:o + n], pk, pool_mode, scale=(scale or None), causal=causal, precision="f64")
        assert_scores_close(sg[:, col:col + P], ref["scores_group"], "scores_group seq %d" % b)
        assert_scores_close(st[col:col + P], ref["scores_tsp"], "scores_tsp seq %d" % b)
        o += n
        col += P
    assert ctx.fkv_query_error() == 0


def test_score_window_output_full_size_32k():
    """Config 2's layer: scores element by element against the oracle, output against the stand-alone call."""
    from parity import assert_scores_close
    print("case: scores + window output at L=32768", flush=True)
    L = 32768
    s = wl.make_sequence(0, L, with_x=False)
    c = fk.Context(max_total_tokens=L, max_seqs=1)
    try:
        shape = fk.make_shape(L, pool_mode="avg")
        q, k, v = dev_bf16(s["q_win"]), dev_bf16(s["k"]), dev_bf16(s["v"])
        sg, st, out = c.fkv_score_window_output(shape, q, k, v)
        alone = c.fkv_window_output(shape, q, k, v)
        torch.cuda.synchronize()
        assert torch.equal(out, alone)
        ref = oracle.score_window(s["q_win"], s["k"], 7, "avg", precision="f32")
        print("  scores: group %.2e tsp %.2e" % (assert_scores_close(sg.cpu().numpy(), ref["scores_group"], "scores_group"),
                                                 assert_scores_close(st.cpu().numpy(), ref["scores_tsp"], "scores_tsp")), flush=True)
        assert c.fkv_query_error() == 0
    finally:
        c.close()
