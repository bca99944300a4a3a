"""Dense operands of more than 4 GiB: the kernels switch from 32-bit to 64-bit row offsets there.
The fp64 oracle checks sampled rows (the product), sampled entries (the sampled product) and the
whole result (MTTKRP, whose output is small)."""
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
        pytest.fail("no GPU visible")
    return torch


def test_product_and_sampled_product_beyond_4gib(torch):
    w = synth.make_config(3, shrink=2)                  # R-MAT scale 21, 2,097,152 vertices
    k = 516                                             # 2,097,152 x 516 x 4 B = 4.33 GB > 2^32 B
    assert w.n * k * 4 > (1 << 32)
    print(f"n={w.n} nnz={w.nnz} k={k}: generating X ...", flush=True)
    X = synth.normal_matrix(w.n, k, seed=811)
    op = binding.ArrowSpMM(w.rowptr, w.colidx, w.vals, w.b)
    Xd = torch.from_numpy(X).cuda()
    Yd = torch.full_like(Xd, float("nan"))
    print("product ...", flush=True)
    op.spmm(Xd, Yd)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Yd).any())
    deg = np.diff(w.rowptr)
    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([np.argsort(deg)[-16:], rng.integers(0, w.n, 1500),
                                     np.arange(w.n - 64, w.n)])).astype(np.int64)     # hubs, sample, the last rows
    Yref, B = oracle.spmm(w.rowptr, w.colidx, w.vals, X, rows=rows)
    Ys = Yd[torch.from_numpy(rows).cuda()].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(Ys - Yref) <= TOL * B) and np.all(Ys[B == 0] == 0)
    # the sampled product with U = X and V = X shifted by one row (another 4.33 GB operand)
    print("sampled product ...", flush=True)
    Vd = torch.roll(Xd, 1, 0)
    V = np.roll(X, 1, 0)
    Sd = torch.full((w.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    op.sddmm(Xd, Vd, Sd)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Sd).any())
    cnt = np.zeros(w.n, np.int64)
    cnt[rows] = deg[rows]
    rp = np.concatenate([[0], np.cumsum(cnt)])
    first = np.cumsum(deg[rows]) - deg[rows]
    idx = np.repeat(w.rowptr[rows] - first, deg[rows]) + np.arange(int(deg[rows].sum()), dtype=np.int64)
    Sref, Bs = oracle.sddmm(rp, w.colidx[idx], w.vals[idx], X, V)
    Ss = Sd[torch.from_numpy(idx).cuda()].cpu().numpy().astype(np.float64)
    assert np.all(np.abs(Ss - Sref) <= TOL * Bs) and np.all(Ss[Bs == 0] == 0)
    op.close()


def test_mttkrp_factor_matrices_beyond_4gib(torch):
    dims = (2048, (1 << 21) - 8, (1 << 21) - 8)
    R = 516                                             # (2^21 - 8) x 516 x 4 B = 4.33 GB per factor
    assert dims[1] * R * 4 > (1 << 32)
    i, j, k, v = synth.tensor3(dims, 3_000_000, seed=synth.SEED_TENSOR + 9, skew=(2.0, 1.0, 1.0))
    # make sure the last rows of both factor matrices are referenced
    i = np.concatenate([i, [2047, 2047]]).astype(np.int32)
    j = np.concatenate([j, [dims[1] - 1, dims[1] - 2]]).astype(np.int32)
    k = np.concatenate([k, [dims[2] - 1, dims[2] - 1]]).astype(np.int32)
    v = np.concatenate([v, [0.5, -0.25]]).astype(np.float32)
    print(f"nnz={len(v)}: generating factors ...", flush=True)
    B = synth.normal_matrix(dims[1], R, seed=821)
    C = synth.normal_matrix(dims[2], R, seed=822)
    op = binding.Csf3Mttkrp(dims, i, j, k, v)
    Ad = torch.full((dims[0], R), float("nan"), dtype=torch.float32, device="cuda")
    op.mttkrp(torch.from_numpy(B).cuda(), torch.from_numpy(C).cuda(), Ad)
    torch.cuda.synchronize()
    A = Ad.cpu().numpy().astype(np.float64)
    assert not np.isnan(A).any()
    print("oracle ...", flush=True)
    Aref, E = oracle.mttkrp(dims, i, j, k, v, B, C)
    assert np.all(np.abs(A - Aref) <= TOL * E) and np.all(A[E == 0] == 0)
    op.close()
