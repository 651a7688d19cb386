"""GPU parity of KVCompress into a paged cache and of decoding over it, against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_01068_amd import binding as fk
from paper_2502_01068_amd import workloads as wl
from parity import dev_bf16, host_bits

pytestmark = pytest.mark.gpu
TOL = 1e-3  # decode outputs, relative to the largest magnitude of the output row


@pytest.fixture(scope="module")
def ctx():
    c = fk.Context(max_total_tokens=40000, max_seqs=8)
    yield c
    c.close()


def _tables(rng, budgets, page_size, n_pages):
    """One row of scattered, distinct physical pages per sequence; unused entries hold -1."""
    need = [(b + page_size - 1) // page_size for b in budgets]
    perm = rng.permutation(n_pages)
    table = np.full((len(budgets), max(need) + 1), -1, np.int32)
    at = 0
    for b, n in enumerate(need):
        table[b, :n] = perm[at:at + n]
        at += n
    return table


@pytest.mark.parametrize("lengths,budgets,page_size", [
    ([2048], [256], 16), ([2048], [250], 64), ([2048], [2048], 256), ([1000], [9], 1),
    ([700, 2048, 90], [100, 513, 90], 32), ([3000, 3000], [128, 129], 128),
])
def test_paged_gather_and_decode(ctx, lengths, budgets, page_size):
    print("case: paged lengths=%s budgets=%s page=%d" % (lengths, budgets, page_size), flush=True)
    Hq, Hkv, d, B = 32, 8, 128, len(lengths)
    rng = np.random.default_rng(sum(lengths) + page_size)
    seqs = [wl.make_sequence(60 + b, L) for b, L in enumerate(lengths)]
    k = np.concatenate([s["k"] for s in seqs])
    v = np.concatenate([s["v"] for s in seqs])
    idx = [np.stack([np.sort(rng.choice(L, n, replace=False)) for _ in range(Hkv)]).astype(np.int32)
           for L, n in zip(lengths, budgets)]
    idx_packed = np.concatenate(idx, axis=1)
    n_pages = sum((n + page_size - 1) // page_size for n in budgets) + 5
    table = _tables(rng, budgets, page_size, n_pages)
    before_k = wl.normal_bf16(61, 0, "k", (n_pages, page_size, Hkv, d))
    before_v = wl.normal_bf16(61, 0, "v", (n_pages, page_size, Hkv, d))
    shape = fk.make_shape(lengths if B > 1 else lengths[0])
    kp, vp = dev_bf16(before_k), dev_bf16(before_v)
    ctx.fkv_gather_kv_paged(shape, dev_bf16(k), dev_bf16(v), torch.from_numpy(idx_packed).cuda(), budgets,
                            torch.from_numpy(table).cuda(), kp, vp)
    want_k, want_v = before_k, before_v
    for b in range(B):
        want_k = oracle.gather_kv_paged(seqs[b]["k"], idx[b], table[b], want_k)
        want_v = oracle.gather_kv_paged(seqs[b]["v"], idx[b], table[b], want_v)
    np.testing.assert_array_equal(host_bits(kp), want_k)   # kept rows in place, every other slot untouched
    np.testing.assert_array_equal(host_bits(vp), want_v)

    q = wl.normal_bf16(62, 0, "q_win", (B, Hq, d))
    out = ctx.fkv_decode_attention_paged(shape, dev_bf16(q), kp, vp, torch.from_numpy(table).cuda(), budgets).cpu().numpy()
    for b in range(B):
        ref = oracle.decode_attention(q[b], oracle.paged_view(want_k, table[b], budgets[b]),
                                      oracle.paged_view(want_v, table[b], budgets[b]), "token_major")
        err = np.abs(out[b] - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
        assert err.max() <= TOL, "sequence %d: %.3g" % (b, err.max())
    # same tokens, same split boundaries: the paged and the compact decode agree bit for bit
    kc, vc = ctx.fkv_gather_kv(shape, dev_bf16(k), dev_bf16(v), torch.from_numpy(idx_packed).cuda(), budgets)
    out_c = ctx.fkv_decode_attention(shape, dev_bf16(q), kc, vc, budgets, "compact").cpu().numpy()
    np.testing.assert_array_equal(out, out_c)


def test_out_of_pool_table_entries_write_nothing(ctx):
    print("case: paged gather with table entries outside the pool", flush=True)
    L, Hkv, d, n, ps, n_pages = 512, 8, 128, 64, 16, 6
    s = wl.make_sequence(63, L)
    idx = np.tile(np.arange(n, dtype=np.int32), (Hkv, 1))
    table = np.array([[2, -1, 6, 4]], np.int32)   # logical pages 1 and 2 point outside the pool
    before = wl.normal_bf16(64, 0, "k", (n_pages, ps, Hkv, d))
    kp = dev_bf16(before)
    ctx.fkv_gather_kv_paged(fk.make_shape(L), dev_bf16(s["k"]), None, torch.from_numpy(idx).cuda(), n,
                            torch.from_numpy(table).cuda(), kp)
    want = before.copy()
    want[2] = s["k"][0:16]
    want[4] = s["k"][48:64]
    np.testing.assert_array_equal(host_bits(kp), want)


def test_paged_full_size_pipeline(ctx):
    """Config-2 shape end to end: score, select, KVCompress into 16-token pages, decode over the
    pages; checked against the compact path of the same call sequence and, on sampled slots,
    against the source rows."""
    print("case: paged pipeline L=32768 budget=2048 page=16", flush=True)
    L, budget, ps, Hkv = 32768, 2048, 16, 8
    s = wl.make_sequence(70, L, with_x=False)
    shape = fk.make_shape(L, pool_mode="avg")
    q, k, v = dev_bf16(s["q_win"]), dev_bf16(s["k"]), dev_bf16(s["v"])
    sg, _ = ctx.fkv_score_window(shape, q, k, want_tsp=False)
    idx = ctx.fkv_select_topk(shape, sg, budget)
    n_pages = budget // ps + 37
    rng = np.random.default_rng(70)
    table = rng.permutation(n_pages)[: budget // ps].astype(np.int32)[None, :]
    kp = torch.zeros((n_pages, ps, Hkv, 128), dtype=torch.bfloat16, device="cuda")
    vp = torch.zeros_like(kp)
    ctx.fkv_gather_kv_paged(shape, k, v, idx, budget, torch.from_numpy(table).cuda(), kp, vp)
    kc, vc = ctx.fkv_gather_kv(shape, k, v, idx, budget)
    # logical view of the pages == compact cache, bit for bit
    order = torch.from_numpy(table[0]).long().cuda()
    view_k = kp[order].reshape(budget, Hkv, 128).permute(1, 0, 2)
    view_v = vp[order].reshape(budget, Hkv, 128).permute(1, 0, 2)
    assert torch.equal(view_k.view(torch.int16), kc.view(torch.int16))
    assert torch.equal(view_v.view(torch.int16), vc.view(torch.int16))
    # sampled slots against the source rows through the oracle's addressing
    idx_h, kp_h = idx.cpu().numpy(), host_bits(kp)
    for g, t in [(0, 0), (3, 17), (7, 2047), (5, 1024), (2, 999)]:
        np.testing.assert_array_equal(kp_h[table[0, t // ps], t % ps, g], s["k"][idx_h[g, t], g])
    untouched = np.setdiff1d(np.arange(n_pages), table[0])
    assert not kp_h[untouched].any()
    # the one-call variant fills a fresh pool identically and returns the same indices
    kp2, vp2 = torch.zeros_like(kp), torch.zeros_like(vp)
    idx2 = ctx.fkv_compress_kv_paged(shape, q, k, v, budget, torch.from_numpy(table).cuda(), kp2, vp2)
    assert torch.equal(idx2, idx)
    assert torch.equal(kp2.view(torch.int16), kp.view(torch.int16)) and torch.equal(vp2.view(torch.int16), vp.view(torch.int16))
    qd = dev_bf16(wl.normal_bf16(71, 0, "q_win", (1, 32, 128)))
    a = ctx.fkv_decode_attention_paged(shape, qd, kp, vp, torch.from_numpy(table).cuda(), budget)
    b = ctx.fkv_decode_attention(shape, qd, kc, vc, budget, "compact")
    assert torch.equal(a, b)
