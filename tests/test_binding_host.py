"""Host-only checks of the binding's argument validation: the C ABI takes bare device pointers, so a
tensor that is too short, on another GPU, strided or of the wrong dtype has to be stopped here."""
import pytest
import torch

from paper_2502_01068_amd import binding as fk


class FakeGpuTensor:
    """Stands in for a CUDA tensor where no GPU exists: only the attributes the checks read."""

    def __init__(self, numel, dtype=torch.bfloat16, index=0, contiguous=True):
        self._numel, self.dtype, self._contig = numel, dtype, contiguous
        self.is_cuda = True
        self.device = torch.device("cuda", index)

    def numel(self):
        return self._numel

    def element_size(self):
        return torch.empty((), dtype=self.dtype).element_size()

    def is_contiguous(self):
        return self._contig

    def data_ptr(self):
        return 0x1000


def test_sizes_follow_the_descriptor():
    shape = fk.make_shape([100, 50, 8], n_q_heads=12, n_kv_heads=4, window=8)
    n = fk._Sizes(shape)
    assert n.total == 158 and n.sum_p == 158 - 3 * 8
    assert n.q_win == 3 * 8 * 12 * 128 and n.kv == 158 * 4 * 128 and n.q_dec == 3 * 12 * 128


def test_accepts_exact_and_larger_buffers():
    assert fk._dev_ptr(FakeGpuTensor(64), "k", fk._BF16, numel=64, device=0).value == 0x1000
    assert fk._dev_ptr(FakeGpuTensor(65), "k", fk._BF16, numel=64, device=0).value == 0x1000
    assert fk._dev_ptr(None, "v", fk._BF16, allow_none=True) is None
    assert fk._dev_ptr(FakeGpuTensor(8, torch.float32), "x_out", nbytes=32).value == 0x1000


@pytest.mark.parametrize("kwargs,tensor,match", [
    (dict(numel=64), FakeGpuTensor(63), "holds 63 elements"),
    (dict(nbytes=130), FakeGpuTensor(64), "holds 128 bytes"),
    (dict(device=0), FakeGpuTensor(64, index=1), "context is on cuda:0"),
    (dict(), FakeGpuTensor(64, contiguous=False), "contiguous"),
    (dict(), FakeGpuTensor(64, dtype=torch.float32), "dtype"),
    (dict(), torch.zeros(64, dtype=torch.bfloat16), "GPU tensor"),
    (dict(), None, "required"),
])
def test_rejects(kwargs, tensor, match):
    with pytest.raises(ValueError, match=match):
        fk._dev_ptr(tensor, "k", fk._BF16, **kwargs)


def test_counts_need_one_entry_per_sequence():
    shape = fk.make_shape([100, 50])
    assert fk._counts(shape, 16)[0] == [16, 16]
    with pytest.raises(ValueError):
        fk._counts(shape, [16])
