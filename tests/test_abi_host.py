"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects invalid problems before any launch."""
import ctypes
import os
import re

import pytest

from paper_2502_01068_amd import binding as fk

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fastkv_select.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fk.LIB_PATH):
        from paper_2502_01068_amd import build
        build.build()
    return fk.load()


def test_every_declared_symbol_is_exported(lib):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = sorted(set(re.findall(r"\b(fkv_[a-z_]+)\s*\(", text)))
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(fk.EXPORTS) == declared
    assert lib.fkv_version() >= 100
    assert lib.fkv_profile_kernels() == 10
    assert lib.fkv_strerror(fk.FKV_EALIGN).decode().startswith("device pointer")


def test_shape_struct_matches_header_layout():
    # int32, pointer (8-aligned), then 8 x 4-byte fields
    assert ctypes.sizeof(fk.FkvShape) == 4 + 4 + 8 + 4 * 9 + 4
    assert fk.FkvShape.cu_seqlens.offset == 8 and fk.FkvShape.L.offset == 16
    assert fk.FkvShape.causal.offset == 16 + 4 * 8


def _shape(**kw):
    lengths = kw.pop("lengths", 2048)
    return fk.make_shape(lengths, **kw)


def test_check_shape_accepts_paper_configs(lib):
    assert lib.fkv_check_shape(ctypes.byref(_shape())) == fk.FKV_OK
    assert lib.fkv_check_shape(ctypes.byref(_shape(lengths=[8192, 16384, 9000], pool_mode="avg"))) == fk.FKV_OK
    assert lib.fkv_check_shape(ctypes.byref(_shape(lengths=8))) == fk.FKV_OK  # L == W: empty prefix
    assert lib.fkv_check_shape(ctypes.byref(_shape(n_q_heads=8, n_kv_heads=8, window=4, pool_kernel=1))) == fk.FKV_OK
    assert lib.fkv_check_shape(ctypes.byref(_shape(n_q_heads=64, n_kv_heads=8))) == fk.FKV_OK   # G = 8
    assert lib.fkv_check_shape(ctypes.byref(_shape(n_q_heads=28, n_kv_heads=4))) == fk.FKV_OK   # G = 7


@pytest.mark.parametrize("kw,code", [
    (dict(lengths=7), fk.FKV_EINVAL),                       # shorter than the window
    (dict(lengths=[100, 5]), fk.FKV_EINVAL),
    (dict(pool_kernel=6), fk.FKV_EINVAL),                   # even kernel
    (dict(pool_kernel=0), fk.FKV_EINVAL),
    (dict(window=0), fk.FKV_EINVAL),
    (dict(n_q_heads=30), fk.FKV_EINVAL),                    # not a multiple of Hkv
    (dict(softmax_scale=-1.0), fk.FKV_EINVAL),
    (dict(softmax_scale=float("nan")), fk.FKV_EINVAL),
    (dict(head_dim=64), fk.FKV_EUNSUPPORTED),
    (dict(window=16), fk.FKV_EUNSUPPORTED),
    (dict(n_q_heads=72), fk.FKV_EUNSUPPORTED),              # G = 9
    (dict(n_q_heads=32, n_kv_heads=16), fk.FKV_EUNSUPPORTED),
    (dict(pool_kernel=33), fk.FKV_EUNSUPPORTED),
    (dict(lengths=[64] * 65), fk.FKV_EUNSUPPORTED),
])
def test_check_shape_rejects(lib, kw, code):
    assert lib.fkv_check_shape(ctypes.byref(_shape(**kw))) == code


def test_check_shape_null_and_flags(lib):
    assert lib.fkv_check_shape(None) == fk.FKV_ENULL
    s = _shape(lengths=[100, 200])
    s.cu_seqlens = None
    assert lib.fkv_check_shape(ctypes.byref(s)) == fk.FKV_ENULL   # B > 1 needs cu_seqlens
    s = _shape()
    s.cu_seqlens = None                                            # B == 1: L is used
    assert lib.fkv_check_shape(ctypes.byref(s)) == fk.FKV_OK
    s.L = 3
    assert lib.fkv_check_shape(ctypes.byref(s)) == fk.FKV_EINVAL
    s = _shape()
    s.pool_mode = 2
    assert lib.fkv_check_shape(ctypes.byref(s)) == fk.FKV_EINVAL
    s = _shape()
    s.causal = 5
    assert lib.fkv_check_shape(ctypes.byref(s)) == fk.FKV_EINVAL
    bad = fk.make_shape([100, 200])
    bad._keep[0] = 1                                               # cu[0] != 0
    assert lib.fkv_check_shape(ctypes.byref(bad)) == fk.FKV_EINVAL
    bad = fk.make_shape([100, 200])
    bad._keep[2] = 50                                              # not increasing
    assert lib.fkv_check_shape(ctypes.byref(bad)) == fk.FKV_EINVAL


def test_check_counts(lib):
    s = _shape(lengths=[100, 200])
    ok = (ctypes.c_int32 * 2)(8, 200)
    assert lib.fkv_check_counts(ctypes.byref(s), ok) == fk.FKV_OK
    assert lib.fkv_check_counts(ctypes.byref(s), (ctypes.c_int32 * 2)(7, 50)) == fk.FKV_EINVAL    # k < W
    assert lib.fkv_check_counts(ctypes.byref(s), (ctypes.c_int32 * 2)(101, 50)) == fk.FKV_EINVAL  # k > L
    assert lib.fkv_check_counts(ctypes.byref(s), None) == fk.FKV_ENULL


def test_entry_points_validate_before_touching_the_context(lib):
    # With a NULL context every call must still report the *argument* problem first, and a
    # valid call must stop at the context check: nothing is launched without a context.
    s = _shape(lengths=7)
    assert lib.fkv_score_window(None, ctypes.byref(s), None, None, None, None, None) == fk.FKV_EINVAL
    s = _shape()
    assert lib.fkv_score_window(None, ctypes.byref(s), None, None, None, None, None) == fk.FKV_ENULL
    p16, p8 = ctypes.c_void_p(4096), ctypes.c_void_p(4104)
    assert lib.fkv_score_window(None, ctypes.byref(s), p8, p16, p16, None, None) == fk.FKV_EALIGN
    assert lib.fkv_score_window(None, ctypes.byref(s), p16, p16, p16, None, None) == fk.FKV_ENULL  # ctx
    k = (ctypes.c_int32 * 1)(512)
    assert lib.fkv_select_topk(None, ctypes.byref(s), p16, 0, k, p16, None) == fk.FKV_EINVAL      # n_rows
    assert lib.fkv_select_topk(None, ctypes.byref(s), p16, 1, (ctypes.c_int32 * 1)(4), p16, None) == fk.FKV_EINVAL
    assert lib.fkv_gather_rows(None, ctypes.byref(s), p16, 24, p16, k, p16, None) == fk.FKV_EALIGN  # row bytes
    assert lib.fkv_gather_rows(None, ctypes.byref(s), p16, 0, p16, k, p16, None) == fk.FKV_EINVAL
    assert lib.fkv_gather_kv(None, ctypes.byref(s), p16, p16, p16, k, p16, None, None) == fk.FKV_ENULL  # v without v_out
    assert lib.fkv_compress_kv(None, ctypes.byref(s), p16, p16, p16, k, p16, p16, p16,
                               p16, 8192, None, p16, p16, None) == fk.FKV_ENULL                   # half a TSP leg
    assert lib.fkv_compress_kv(None, ctypes.byref(s), p16, p16, p16, k, p16, p16, p16,
                               None, 0, None, None, None, None) == fk.FKV_ENULL                   # ctx
    assert lib.fkv_index_overlap(None, p16, 4, -1, p16, 4, 4, 1, p16, None) == fk.FKV_EINVAL      # n_a < 0
    assert lib.fkv_index_overlap(None, p16, 4, 4, p16, 4, 4, 1, p16, None) == fk.FKV_ENULL        # ctx
    assert lib.fkv_mass_recall(None, p16, -8, 8, p16, 4, 4, 1, p16, None) == fk.FKV_EINVAL        # stride < 0
    assert lib.fkv_mass_recall(None, p16, 8, 8, p16, 4, 4, 1, p16, None) == fk.FKV_ENULL          # ctx
    n1 = (ctypes.c_int32 * 1)(300)
    assert lib.fkv_gather_kv_paged(None, ctypes.byref(s), p16, p16, p16, k, p16, 8, 48, 100, p16, p16, None) == fk.FKV_EINVAL  # page size
    assert lib.fkv_gather_kv_paged(None, ctypes.byref(s), p16, p16, p16, k, p16, 8, 32, 100, p16, p16, None) == fk.FKV_EINVAL  # 8*32 < 512
    assert lib.fkv_gather_kv_paged(None, ctypes.byref(s), p16, p16, p16, k, None, 8, 64, 100, p16, p16, None) == fk.FKV_ENULL  # table
    assert lib.fkv_gather_kv_paged(None, ctypes.byref(s), p16, p16, p16, k, p16, 8, 64, 100, p16, p16, None) == fk.FKV_ENULL   # ctx
    assert lib.fkv_compress_kv_paged(None, ctypes.byref(s), p16, p16, p16, k, p16, 8, 32, 100, p16, p16, p16, None) == fk.FKV_EINVAL  # 8*32 < 512
    assert lib.fkv_compress_kv_paged(None, ctypes.byref(s), p16, p16, p16, k, p16, 8, 64, 100, p16, p16, p16, None) == fk.FKV_ENULL   # ctx
    assert lib.fkv_decode_attention_paged(None, ctypes.byref(s), p16, p16, p16, p16, 4, 64, 100, n1, p16, None) == fk.FKV_EINVAL  # 4*64 < 300
    assert lib.fkv_decode_attention_paged(None, ctypes.byref(s), p16, p16, p16, p16, 8, 64, 0, n1, p16, None) == fk.FKV_EINVAL   # no pages
    assert lib.fkv_decode_attention_paged(None, ctypes.byref(s), p16, p16, p16, p16, 8, 64, 100, n1, p16, None) == fk.FKV_ENULL  # ctx
    assert lib.fkv_probe_logits(None, ctypes.byref(s), p16, p16, 1, p16, None) == fk.FKV_ENULL   # ctx
    assert lib.fkv_window_output(None, ctypes.byref(_shape(lengths=7)), p16, p16, p16, p16, None) == fk.FKV_EINVAL  # L < W
    assert lib.fkv_window_output(None, ctypes.byref(s), p16, p16, None, p16, None) == fk.FKV_ENULL    # v
    assert lib.fkv_window_output(None, ctypes.byref(s), p16, p16, p16, p8, None) == fk.FKV_EALIGN     # out
    assert lib.fkv_window_output(None, ctypes.byref(s), p16, p16, p16, p16, None) == fk.FKV_ENULL     # ctx
    assert lib.fkv_probe_read(None, p16, 1000, 0, None) == fk.FKV_EINVAL and lib.fkv_probe_read(None, p16, 65536, 0, None) == fk.FKV_ENULL
    assert lib.fkv_set_wait_limit(None, 5) == fk.FKV_ENULL and lib.fkv_clear_error(None) == fk.FKV_ENULL
    assert lib.fkv_destroy(None) == fk.FKV_ENULL
    assert lib.fkv_set_select_path(None, 0) == fk.FKV_ENULL
    assert lib.fkv_set_score_path(None, 0) == fk.FKV_ENULL and lib.fkv_query_error(None, None) == fk.FKV_ENULL


def test_workspace_bytes(lib):
    small, big = lib.fkv_workspace_bytes(2048, 1), lib.fkv_workspace_bytes(131072, 1)
    assert 0 < small < big < 64 << 20
    assert big >= 131072 * 9 * 4
    assert lib.fkv_workspace_bytes(0, 1) == 0 and lib.fkv_workspace_bytes(100, 65) == 0


def test_count_from_rate_matches_the_stated_counts(lib):
    # 20 % of 32768 -> 6554 kept, 20 % / 10 % of 131072 -> 26214 / 13107 (round half up, not ceil)
    assert lib.fkv_count_from_rate(32768, 0.2) == 6554
    assert lib.fkv_count_from_rate(131072, 0.2) == 26214
    assert lib.fkv_count_from_rate(131072, 0.1) == 13107
    assert lib.fkv_count_from_rate(10, 0.25) == 3 and lib.fkv_count_from_rate(10, 0.24) == 2
    assert lib.fkv_count_from_rate(100, 1.5) == 100 and lib.fkv_count_from_rate(0, 0.2) == 0
    assert lib.fkv_count_from_rate(-1, 0.2) == -1 and lib.fkv_count_from_rate(10, -0.1) == -1
    assert lib.fkv_count_from_rate(10, float("nan")) == -1
    assert lib.fkv_score_heads(None, None, None, None, None, None) == fk.FKV_ENULL


def test_plan_layer_follows_algorithm_1(lib):
    # the three evaluated models (Sec. 5.1, App. C.1): layers, TSP layer; TSP rate 20 % gives the
    # stated 60 % prefill compute rate for each of them
    for n_layers, tsp in ((32, 15), (36, 17), (40, 19)):
        plans = [fk.fkv_plan_layer(l, n_layers, tsp, 32768, 0.2, 0.0625) for l in range(n_layers)]
        assert [p[0] for p in plans] == [32768] * (tsp + 1) + [6554] * (n_layers - tsp - 1)
        assert [p[1] for p in plans] == [0] * tsp + [6554] + [0] * (n_layers - tsp - 1)
        assert all(p[2] == 2048 for p in plans)
        assert abs(sum(p[0] for p in plans) / (n_layers * 32768) - 0.6) < 1e-4
    assert fk.fkv_plan_layer(15, 32, 15, 131072, 0.2, 0.1) == (131072, 26214, 13107)
    assert fk.fkv_plan_layer(20, 32, 15, 131072, 0.2, 0.5) == (26214, 0, 26214)      # budget capped by what the layer sees
    assert fk.fkv_plan_layer(3, 4, 1, 16, 0.01, 0.01) == (8, 0, 8)                   # never below the window
    p = fk.FkvLayerPlan()
    assert lib.fkv_plan_layer(32, 32, 15, 100, 0.2, 0.1, 8, ctypes.byref(p)) == fk.FKV_EINVAL
    assert lib.fkv_plan_layer(0, 32, 15, 100, 0.0, 0.1, 8, ctypes.byref(p)) == fk.FKV_EINVAL
    assert lib.fkv_plan_layer(0, 32, 15, 4, 0.2, 0.1, 8, ctypes.byref(p)) == fk.FKV_EINVAL
    assert lib.fkv_plan_layer(0, 32, 15, 100, 0.2, 0.1, 8, None) == fk.FKV_ENULL


def test_score_plan_covers_every_prefix_token():
    """Host logic of the single-pass kernel's block layout: every prefix token is owned by exactly one
    block, no block is empty, no block computes more than its sub-tiles hold, the block budget is kept,
    and a smaller budget never gives a smaller share."""
    import numpy as np
    rng = np.random.default_rng(5)
    cases = [([32768], 8, 7, 256), ([6554], 8, 7, 256), ([2048], 8, 7, 256), ([9], 8, 7, 256), ([8], 8, 7, 256),
             ([61440], 8, 7, 256), ([70000], 8, 7, 256), ([300, 1000, 57, 8, 2049, 131], 8, 7, 256), ([40], 8, 31, 4)]
    for _ in range(300):
        B = int(rng.integers(1, 9))
        W = int(rng.integers(1, 9))
        cases.append(([int(rng.integers(W, 9000)) for _ in range(B)], W, int(rng.integers(0, 16)) * 2 + 1,
                      int(rng.choice([1, 7, 64, 213, 256]))))
    for lengths, W, pk, max_blocks in cases:
        shape = fk.make_shape(lengths, window=W, pool_kernel=pk)
        plan = fk.fkv_score_plan(shape, max_blocks)
        r = pk // 2
        total_prefix = sum(L - W for L in lengths)
        if plan is None:
            # only when even 8 sub-tiles per block are not enough for the block budget (or nothing is to be scored)
            cap = 256 - 2 * r
            assert total_prefix == 0 or cap <= max(0, W - r) or \
                sum(-(-(L - W) // cap) for L in lengths if L > W) >= max_blocks, (lengths, W, pk, max_blocks)
            continue
        first, own, n_sub = plan
        assert first[0] == 0 and first[-1] <= max_blocks and 1 <= n_sub <= 8
        for b, L in enumerate(lengths):
            P, nb = L - W, first[b + 1] - first[b]
            assert nb == (0 if P <= 0 else -(-P // own[b])), (lengths, W, pk, max_blocks, plan)
            for i in range(nb):
                o0, o1 = i * own[b], min(P, (i + 1) * own[b])
                assert o1 > o0
                c1 = max(L, o1 + r) if i == nb - 1 else o1 + r
                assert c1 - (o0 - r) <= n_sub * 32, (lengths, W, pk, max_blocks, plan, i)
    # config 2: 5 full sub-tiles per block on 213 blocks; the 6554 propagated tokens: 2 sub-tiles on 113 blocks
    assert fk.fkv_score_plan(fk.make_shape(32768), 256) == ([0, 213], [154], 5)
    assert fk.fkv_score_plan(fk.make_shape(6554), 256) == ([0, 113], [58], 2)
