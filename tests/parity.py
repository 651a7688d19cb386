"""Shared helpers of the GPU parity tests: device upload of bf16 bit patterns and the
comparison rules (scores within 1e-3 relative plus the fp32 underflow floor; index sets exact
except inside the tolerance band around the k-th score; gathered rows bit-exact)."""
import numpy as np
import torch

SCORE_RTOL = 1e-3  # fp32 accumulate from bf16 inputs: bound stated for the selection path
# Absolute floor at the bottom of fp32's normal range.  A score is a sum over the W <= 8 window rows
# of probabilities 2^(z - lse); the kernels form each with the hardware exp2, which returns 0 for a
# result below FLT_MIN = 2^-126 instead of a sub-normal.  Pooling and the head means never enlarge
# that loss, so a score may miss up to 8 * FLT_MIN of what exact arithmetic (or the fp64 oracle)
# gives.  No selection can depend on it: such scores are 30 orders of magnitude below 1/L.
FLT_MIN = 1.1754943508222875e-38
SCORE_ATOL = 8 * FLT_MIN


def dev_bf16(a):
    """uint16 bf16 bit patterns -> bfloat16 tensor on cuda:0 (same bits)."""
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)


def host_bits(t):
    """bfloat16 / 16-bit tensor -> uint16 numpy (same bits)."""
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def assert_scores_close(gpu, ref, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (what, gpu.shape, ref.shape)
    assert np.isfinite(gpu).all(), what
    err = np.abs(gpu - ref)
    bad = err > SCORE_RTOL * np.abs(ref) + SCORE_ATOL
    if bad.any():
        i = np.unravel_index(np.argmax(np.where(bad, err / np.maximum(np.abs(ref), SCORE_ATOL), 0)), ref.shape)
        raise AssertionError("%s: %d scores off by more than %g relative + %g; worst at %s gpu=%r ref=%r"
                             % (what, bad.sum(), SCORE_RTOL, SCORE_ATOL, i, gpu[i], ref[i]))
    return float((np.maximum(err - SCORE_ATOL, 0) / np.maximum(np.abs(ref), SCORE_ATOL)).max()) if ref.size else 0.0


def assert_index_set(gpu_idx, ref_idx, ref_scores, window, what=""):
    """gpu_idx / ref_idx: ascending kept positions of one row (length k).  They must agree
    except for prefix positions whose reference score lies within the score tolerance
    (SCORE_RTOL relative + SCORE_ATOL) of the k-th largest reference score (either choice is then
    a correct selection)."""
    gpu_idx = np.asarray(gpu_idx)
    ref_idx = np.asarray(ref_idx)
    k, P = len(ref_idx), len(ref_scores)
    assert gpu_idx.shape == ref_idx.shape, what
    assert (np.diff(gpu_idx) > 0).all(), what + ": not ascending/unique"
    assert gpu_idx[k - window:].tolist() == list(range(P, P + window)), what + ": window not kept"
    if k > window:
        assert gpu_idx[0] >= 0 and gpu_idx[k - window - 1] < P, what
    diff = np.setxor1d(gpu_idx, ref_idx)
    if diff.size == 0:
        return 0
    tau = float(np.asarray(ref_scores, dtype=np.float64)[ref_idx[: k - window]].min())
    sc = np.asarray(ref_scores, dtype=np.float64)[diff]
    off = np.abs(sc - tau) > SCORE_RTOL * abs(tau) + SCORE_ATOL
    assert not off.any(), "%s: %d index differences outside the tolerance band (tau=%g, scores %s)" % (
        what, off.sum(), tau, sc[off][:5])
    return int(diff.size)
