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
