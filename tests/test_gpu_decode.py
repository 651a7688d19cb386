"""GPU parity of the decode-step attention over a (compacted) KV cache against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_01068_amd import binding as fk
from paper_2502_01068_amd import workloads as wl
from parity import dev_bf16, host_bits

pytestmark = pytest.mark.gpu
TOL = 1e-3  # relative to the largest magnitude of the output row (outputs are sums that may cancel)


def _close(gpu, ref, what):
    gpu, ref = np.asarray(gpu, np.float64), np.asarray(ref, np.float64)
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


@pytest.mark.parametrize("ns,Hq,Hkv,scale", [
    ([1], 32, 8, 0.0), ([17], 32, 8, 0.0), ([128], 32, 8, 0.0), ([129], 32, 8, 0.0), ([2048], 32, 8, 0.0),
    ([5000], 32, 8, 0.0), ([300, 1, 2049, 64], 32, 8, 0.0), ([777], 8, 8, 0.25), ([513, 90], 12, 4, 0.0), ([1500], 64, 8, 0.0), ([333, 70], 28, 4, 0.0),
])
@pytest.mark.parametrize("layout", ["compact", "token_major"])
def test_decode_attention_parity(ctx, ns, Hq, Hkv, scale, layout):
    print("case: decode n=%s Hq=%d Hkv=%d scale=%g %s" % (ns, Hq, Hkv, scale, layout), flush=True)
    B, d, tot = len(ns), 128, sum(ns)
    q = wl.normal_bf16(40, 0, "q_win", (B, Hq, d))
    k = wl.normal_bf16(40, 0, "k", (tot, Hkv, d))       # token-major master copy
    v = wl.normal_bf16(40, 0, "v", (tot, Hkv, d))
    shape = fk.make_shape([max(n, 8) for n in ns], n_q_heads=Hq, n_kv_heads=Hkv, softmax_scale=scale)
    if layout == "compact":
        kd, vd = np.ascontiguousarray(k.transpose(1, 0, 2)), np.ascontiguousarray(v.transpose(1, 0, 2))
    else:
        kd, vd = k, v
    out = ctx.fkv_decode_attention(shape, dev_bf16(q), dev_bf16(kd), dev_bf16(vd), ns, layout).cpu().numpy()
    o = 0
    for b, n in enumerate(ns):
        ref = oracle.decode_attention(q[b], k[o:o + n], v[o:o + n], "token_major", scale or None, "f64")
        _close(out[b], ref, "seq %d" % b)
        o += n


def test_decode_after_compress(ctx):
    # end to end: compress a 2048-token layer, then decode over the compacted cache it produced
    print("case: decode over compress_kv output", flush=True)
    L, budget = 2048, 256
    s = wl.make_sequence(0, L, n_heavy=64)
    shape = fk.make_shape(L, pool_mode="max")
    k, v = dev_bf16(s["k"]), dev_bf16(s["v"])
    comp = ctx.fkv_compress_kv(shape, dev_bf16(s["q_win"]), k, v, budget)
    qn = wl.normal_bf16(41, 0, "q_win", (1, 32, 128))
    out_c = ctx.fkv_decode_attention(shape, dev_bf16(qn), comp["k_out"], comp["v_out"], budget, "compact").cpu().numpy()
    ref = oracle.decode_attention(qn[0], host_bits(comp["k_out"]), host_bits(comp["v_out"]), "compact", None, "f64")
    _close(out_c[0], ref, "compacted cache")
    out_f = ctx.fkv_decode_attention(shape, dev_bf16(qn), k, v, L, "token_major").cpu().numpy()
    ref_f = oracle.decode_attention(qn[0], s["k"], s["v"], "token_major", None, "f64")
    _close(out_f[0], ref_f, "full cache")


def test_decode_rejects_bad_arguments(ctx):
    shape = fk.make_shape(64)
    q = torch.zeros((1, 32, 128), dtype=torch.bfloat16, device="cuda")
    kv = torch.zeros((8, 16, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fk.FkvError) as ei:
        ctx.fkv_decode_attention(shape, q, kv, kv, 0)
    assert ei.value.status == fk.FKV_EINVAL
