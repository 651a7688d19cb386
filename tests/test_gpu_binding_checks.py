"""The binding stops tensors that do not match the host descriptor before any launch (GPU machine:
real tensors, real context; nothing is enqueued by a rejected call)."""
import pytest
import torch

from paper_2502_01068_amd import binding as fk

pytestmark = pytest.mark.gpu


def test_wrappers_reject_mismatched_tensors():
    print("case: binding size checks", flush=True)
    L, budget, k_tsp = 512, 64, 100
    ctx = fk.Context(max_total_tokens=L, max_seqs=1)
    shape = fk.make_shape(L)
    bf = dict(dtype=torch.bfloat16, device="cuda")
    q = torch.zeros((8, 32, 128), **bf)
    k = torch.zeros((L, 8, 128), **bf)
    v = torch.zeros((L, 8, 128), **bf)
    x = torch.zeros((L, 256), **bf)
    try:
        good = ctx.fkv_compress_kv(shape, q, k, v, budget, x=x, k_tsp_per_seq=k_tsp)
        with pytest.raises(ValueError, match="k holds"):
            ctx.fkv_score_window(shape, q, k[: L - 1])
        with pytest.raises(ValueError, match="q_win holds"):
            ctx.fkv_score_window(shape, q[:7], k)
        with pytest.raises(ValueError, match="v holds"):
            ctx.fkv_compress_kv(shape, q, k, v[: L // 2], budget)
        with pytest.raises(ValueError, match="x has"):
            ctx.fkv_compress_kv(shape, q, k, v, budget, x=x[:-1], k_tsp_per_seq=k_tsp)
        with pytest.raises(ValueError, match="k_out holds"):          # an `out` dict of a smaller budget
            ctx.fkv_compress_kv(shape, q, k, v, budget * 2, x=x, k_tsp_per_seq=k_tsp, out=good)
        with pytest.raises(ValueError, match="x_out holds|idx_tsp holds"):
            ctx.fkv_compress_kv(shape, q, k, v, budget, x=x, k_tsp_per_seq=k_tsp + 1, out=good)
        sg, _ = ctx.fkv_score_window(shape, q, k)
        with pytest.raises(ValueError, match="scores rows"):
            ctx.fkv_select_topk(shape, sg[:, :-1].contiguous(), budget)
        idx = ctx.fkv_select_topk(shape, sg, budget)
        with pytest.raises(ValueError, match="idx_kv holds"):
            ctx.fkv_gather_kv(shape, k, v, idx[:7], budget)
        with pytest.raises(ValueError, match="GPU tensor"):
            ctx.fkv_score_window(shape, q.cpu(), k)
        pages = torch.zeros((8, 16, 8, 128), **bf)
        with pytest.raises(ValueError, match="block_table"):
            ctx.fkv_gather_kv_paged(shape, k, v, idx, budget, torch.zeros((2, 4), dtype=torch.int32, device="cuda"), pages, pages.clone())
        torch.cuda.synchronize()
        assert ctx.fkv_query_error() == 0
    finally:
        ctx.close()
