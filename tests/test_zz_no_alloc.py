"""The allocation-free entry point ``arrow_spmm_static`` (scratch memory in a device array that
is part of the library) against ``arrow_spmm`` (scratch memory in the caller's workspace): the
same kernels in the same order, so the results must agree bit for bit, and both stay within the
oracle's bound.  Two calls in a row, the second on a smaller operand: the array keeps the first
call's contents, which must not matter."""
import os

import numpy as np
import pytest

import oracle
from paper_2307_05740_amd import binding, synth

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def torch():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: this test needs a real MI355X")
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libarrow.so is not built")
    return torch


def _both_ways(torch, w, b, X):
    op = binding.ArrowSpMM(w.rowptr, w.colidx, w.vals, b)
    k = X.shape[1]
    Xd = torch.from_numpy(X).cuda()
    Yws = op.spmm(Xd)                                    # caller's workspace
    Yst = torch.full_like(Xd, float("nan"))              # every element must be written
    stream = torch.cuda.current_stream().cuda_stream
    binding.arrow_spmm_static(op.h, Xd.data_ptr(), Yst.data_ptr(), k, stream)
    torch.cuda.synchronize()
    a, s = Yws.cpu().numpy(), Yst.cpu().numpy()
    levels = op.levels()
    op.close()
    return a, s, levels


def test_static_scratch_matches_workspace_on_two_calls_in_a_row(torch):
    # first call: several levels, split head rows (partial vectors) and a staged head
    w1 = synth.make_config(3, shrink=8)                  # R-MAT scale 15, k = 128, b = 1024
    X1 = w1.make_x()
    a1, s1, lv1 = _both_ways(torch, w1, w1.b, X1)
    assert sum(l["partials"] for l in lv1) > 0           # the scratch array really is used
    assert np.array_equal(a1.view(np.uint32), s1.view(np.uint32))
    Yref, B = oracle.spmm(w1.rowptr, w1.colidx, w1.vals, X1)
    assert np.all(np.abs(s1.astype(np.float64) - Yref) <= TOL * B)
    # second call, smaller operand and other k: the array still holds the first call's partials
    w2 = synth.make_config(0)                            # R-MAT scale 12, b = 512
    X2 = synth.normal_matrix(w2.n, 36, seed=4242)
    a2, s2, lv2 = _both_ways(torch, w2, w2.b, X2)
    assert np.array_equal(a2.view(np.uint32), s2.view(np.uint32))
    Yref, B = oracle.spmm(w2.rowptr, w2.colidx, w2.vals, X2)
    assert np.all(np.abs(s2.astype(np.float64) - Yref) <= TOL * B)
    assert np.all(s2[B == 0] == 0)


def test_static_scratch_rejects_what_does_not_fit(torch):
    # a hub row of 3 M entries cut into 256-entry chunks needs 11,719 partial vectors; at k = 2048
    # that is 96 MB, above the 64 MiB array
    n = 3_000_000
    rowptr = np.zeros(n + 1, np.int64)
    rowptr[1:] = n
    colidx = np.arange(n, dtype=np.int32)
    vals = np.ones(n, np.float32)
    h = binding.arrow_decompose(rowptr, colidx, vals, 1024)
    try:
        k = 2048
        need = binding.arrow_workspace_bytes(h, k) - n * k * 4
        assert need > binding.ARROW_STATIC_SCRATCH_BYTES
        img = torch.empty(binding.arrow_device_bytes(h), dtype=torch.uint8, device="cuda")
        binding.arrow_upload(h, img.data_ptr(), img.numel(), 0)
        torch.cuda.synchronize()
        X = torch.zeros(16, device="cuda")               # never touched: the call must fail first
        with pytest.raises(binding.ArrowError) as ei:
            binding.arrow_spmm_static(h, X.data_ptr(), X.data_ptr() + 64, k, 0)
        assert ei.value.code == binding.ARROW_ETOOSMALL
    finally:
        binding.arrow_destroy(h)
