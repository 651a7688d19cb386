"""The score entry point that allocates nothing (static scratch array in the library's device image)
against the context-based entry point it is a variant of: two calls in a row, the second on a
smaller input, both through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2502_01068_amd import binding as fk
from paper_2502_01068_amd import workloads as wl
from parity import assert_scores_close, dev_bf16

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_matches_context_entry():
    print("case: fkv_score_window_static, 2 calls (9000 tokens in 3 sequences, then 700 tokens)", flush=True)
    ctx = fk.Context(max_total_tokens=9000, max_seqs=4)
    ctx.fkv_set_score_path(1)  # the static entry point runs the two-pass kernels: compare like with like
    try:
        for seed, lengths, pool_mode in ((41, [5000, 8, 3992], "avg"), (42, [700], "max")):
            batch = wl.make_batch(seed, lengths, n_heavy=6, with_v=False, with_x=False)
            shape = fk.make_shape(lengths, pool_mode=pool_mode)
            q, k = dev_bf16(batch["q_win"]), dev_bf16(batch["k"])
            want_g, want_t = ctx.fkv_score_window(shape, q, k)
            got_g, got_t = fk.fkv_score_window_static(shape, q, k)
            torch.cuda.synchronize()
            # same kernels, same launch plan: the two must agree to the last bit, and with the oracle to the score bar
            assert torch.equal(got_g, want_g) and torch.equal(got_t, want_t), "static and context entry points differ"
            col = 0
            for s in batch["seqs"]:
                P = s["k"].shape[0] - 8
                ref = oracle.score_window(s["q_win"], s["k"], 7, pool_mode, precision="f64")
                assert_scores_close(got_g[:, col:col + P].cpu().numpy(), ref["scores_group"], "scores_group")
                assert_scores_close(got_t[col:col + P].cpu().numpy(), ref["scores_tsp"], "scores_tsp")
                col += P
        assert ctx.fkv_query_error() == 0
    finally:
        ctx.close()


def test_static_scratch_entry_rejects_oversize():
    print("case: fkv_score_window_static limits", flush=True)
    shape = fk.make_shape(131073)
    q = torch.zeros((1, 8, 32, 128), dtype=torch.bfloat16, device="cuda")
    k = torch.zeros((131073, 8, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fk.FkvError) as ei:
        fk.fkv_score_window_static(shape, q, k)
    assert ei.value.status == fk.FKV_EWORKSPACE
    lengths = [16] * 17
    shape = fk.make_shape(lengths)
    with pytest.raises(fk.FkvError) as ei:
        fk.fkv_score_window_static(shape, torch.zeros((17, 8, 32, 128), dtype=torch.bfloat16, device="cuda"),
                                   torch.zeros((17 * 16, 8, 128), dtype=torch.bfloat16, device="cuda"))
    assert ei.value.status == fk.FKV_EWORKSPACE
