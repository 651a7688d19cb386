"""The whole selection call can be recorded into a HIP graph (it never allocates, synchronises or
memsets): replays must reproduce the eager result bit for bit, with eager work in between."""
import numpy as np
import pytest
import torch

from paper_2502_01068_amd import binding as fk
from paper_2502_01068_amd import workloads as wl
from parity import dev_bf16

pytestmark = pytest.mark.gpu


def _eq(a, b):
    for n in a:
        x, y = a[n], b[n]
        if x.dtype == torch.bfloat16:
            x, y = x.view(torch.int16), y.view(torch.int16)
        assert torch.equal(x, y), n


@pytest.mark.parametrize("score_path", [0, 1])
def test_compress_kv_graph_replays_match_eager(score_path):
    print("case: graph capture, score path %d" % score_path, flush=True)
    L, k_tsp, budget = 5000, 1000, 300
    ctx = fk.Context(max_total_tokens=L, max_seqs=1)
    ctx.fkv_set_score_path(score_path)
    shape = fk.make_shape(L, pool_mode="max")
    seqs = [wl.make_sequence(30 + i, L, n_heavy=40) for i in range(2)]
    dev = [{n: dev_bf16(s[n]) for n in ("q_win", "k", "v", "x")} for s in seqs]
    # static input buffers the graph reads; refilled between replays
    buf = {n: dev[0][n].clone() for n in dev[0]}
    eager = []
    for d in dev:
        out = ctx.fkv_compress_kv(shape, d["q_win"], d["k"], d["v"], budget, x=d["x"], k_tsp_per_seq=k_tsp)
        eager.append({n: t.clone() for n, t in out.items()})
    torch.cuda.synchronize()

    out = ctx.fkv_compress_kv(shape, buf["q_win"], buf["k"], buf["v"], budget, x=buf["x"], k_tsp_per_seq=k_tsp)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        for _ in range(2):  # warm-up on the capture stream
            ctx.fkv_compress_kv(shape, buf["q_win"], buf["k"], buf["v"], budget, x=buf["x"], k_tsp_per_seq=k_tsp, out=out)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            ctx.fkv_compress_kv(shape, buf["q_win"], buf["k"], buf["v"], budget, x=buf["x"], k_tsp_per_seq=k_tsp, out=out)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        which = rep % 2
        for n in buf:
            buf[n].copy_(dev[which][n])
        for t in out.values():
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        _eq(eager[which], out)
        # eager work between replays (same context, same workspace)
        e2 = ctx.fkv_compress_kv(shape, dev[1 - which]["q_win"], dev[1 - which]["k"], dev[1 - which]["v"], budget,
                                 x=dev[1 - which]["x"], k_tsp_per_seq=k_tsp)
        torch.cuda.synchronize()
        _eq(eager[1 - which], e2)
    assert ctx.fkv_query_error() == 0
    ctx.close()


@pytest.mark.parametrize("select_path", [0, 1])
def test_serving_step_graph_replays_match_eager(select_path):
    """A serving-style step recorded as one graph: the window rows' attention output, KVCompress into a
    paged cache, decode over the pages, and a long-row select (several blocks per row inside one launch,
    whose mailbox epoch lives in device memory and so moves on with every replay; or the multi-launch
    chain); replays with changed inputs must match eager runs."""
    print("case: graph capture of paged compress + paged decode + long select, select path %d" % select_path, flush=True)
    L, budget, ps, Hkv = 6000, 512, 16, 8
    n_pages = budget // ps + 9
    ctx = fk.Context(max_total_tokens=40008, max_seqs=1)
    ctx.fkv_set_select_path(select_path)
    shape = fk.make_shape(L, pool_mode="avg")
    long_shape = fk.make_shape(40008)
    rng = np.random.default_rng(3)
    table = torch.from_numpy(rng.permutation(n_pages)[: budget // ps].astype(np.int32)[None, :]).cuda()
    seqs = [wl.make_sequence(40 + i, L, n_heavy=30, with_x=False) for i in range(2)]
    dev = [{n: dev_bf16(s[n]) for n in ("q_win", "k", "v")} for s in seqs]
    qd = [dev_bf16(wl.normal_bf16(50 + i, 0, "q_win", (1, 32, 128))) for i in range(2)]
    rows = [torch.from_numpy(wl.random_scores(60 + i, 2, 40000, ties=0.2)).cuda() for i in range(2)]
    buf = {n: dev[0][n].clone() for n in dev[0]}
    buf["qd"], buf["rows"] = qd[0].clone(), rows[0].clone()
    kp = torch.zeros((n_pages, ps, Hkv, 128), dtype=torch.bfloat16, device="cuda")
    vp = torch.zeros_like(kp)
    idx = torch.empty((Hkv, budget), dtype=torch.int32, device="cuda")
    dec = torch.empty((1, 32, 128), dtype=torch.float32, device="cuda")
    sel = torch.empty((2, 9000), dtype=torch.int32, device="cuda")
    wo = torch.empty((1, 8, 32, 128), dtype=torch.float32, device="cuda")

    def step(b):
        ctx.fkv_window_output(shape, b["q_win"], b["k"], b["v"], out=wo)
        ctx.fkv_compress_kv_paged(shape, b["q_win"], b["k"], b["v"], budget, table, kp, vp, idx)
        ctx.fkv_decode_attention_paged(shape, b["qd"], kp, vp, table, budget, out=dec)
        ctx.fkv_select_topk(long_shape, b["rows"], 9000, idx_out=sel)

    eager = []
    for i in range(2):
        step({**dev[i], "qd": qd[i], "rows": rows[i]})
        torch.cuda.synchronize()
        eager.append([t.clone() for t in (kp, vp, idx, dec, sel, wo)])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(buf)
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(buf)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        which = rep % 2
        for n in dev[which]:
            buf[n].copy_(dev[which][n])
        buf["qd"].copy_(qd[which])
        buf["rows"].copy_(rows[which])
        for t in (kp, vp, idx, dec, sel, wo):
            t.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for got, want in zip((kp, vp, idx, dec, sel, wo), eager[which]):
            a, b = (t.view(torch.int16) if t.dtype == torch.bfloat16 else t for t in (got, want))
            assert torch.equal(a, b)
        step({**dev[1 - which], "qd": qd[1 - which], "rows": rows[1 - which]})   # eager work between replays
        torch.cuda.synchronize()
    assert ctx.fkv_query_error() == 0
    ctx.close()
