"""Parity at the full sizes of the named workloads, in the launch configuration ``bench.py``
times (default options).  The products are checked on every row (in slabs where the fp64 result
is too large to hold at once: every output row is an independent sum, so the oracle computes any
set of rows on its own); the sampled dense-dense product at the headline on sampled rows."""
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


def check(Y, Yref, B, scale=1.0):
    err = np.abs(np.asarray(Y, np.float64) - Yref)
    assert np.all(err <= scale * TOL * B), f"max err/bound = {np.max(err / np.maximum(B, 1e-300)):.3e}"
    assert np.all(np.asarray(Y)[B == 0] == 0)


def test_config1_grid_1024_full(torch):
    w = synth.make_config(1)
    X = w.make_x()
    op = binding.ArrowSpMM(w.rowptr, w.colidx, w.vals, w.b)
    assert op.info["levels"] == 1                       # one arrow matrix, as the workload states
    Y = op.spmm(torch.from_numpy(X).cuda()).cpu().numpy()
    Yref, B = oracle.spmm(w.rowptr, w.colidx, w.vals, X)
    check(Y, Yref, B)
    op.close()


def test_config2_rmat_s20_cubed_full(torch):
    w = synth.make_config(2)
    X = w.make_x()
    op = binding.ArrowSpMM(w.rowptr, w.colidx, w.vals, w.b)
    Xd = torch.from_numpy(X).cuda()
    op.spmm_iter(Xd, w.l)
    Xl, El = oracle.spmm_iter(w.rowptr, w.colidx, w.vals, X, w.l)
    check(Xd.cpu().numpy(), Xl, El, scale=w.l)
    op.close()


def test_config3_rmat_s23_k128_all_rows(torch):
    print("generating R-MAT scale 23 ...", flush=True)
    w = synth.make_config(3)
    print(f"decomposing n={w.n} nnz={w.nnz} ...", flush=True)
    op = binding.ArrowSpMM(w.rowptr, w.colidx, w.vals, w.b)
    X = w.make_x()
    print(f"levels={op.info['levels']}; product ...", flush=True)
    Xd = torch.from_numpy(X).cuda()
    Yd = torch.full_like(Xd, float("nan"))
    op.spmm(Xd, Yd)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Yd).any())              # every row of Y was written
    deg = np.diff(w.rowptr)
    rng = np.random.default_rng(23)
    rows = np.unique(np.concatenate([
        np.argsort(deg)[-48:],                          # the heaviest hub rows (split + reduced)
        np.flatnonzero(deg == 0)[:16],                  # empty rows
        rng.integers(0, w.n, 4096),                     # uniform sample
        np.arange(0, w.n, w.n // 512)])).astype(np.int64)
    # every row of the result against the oracle, in slabs of 2^20 rows (fp64 result and bound of
    # a slab: 2 GiB); the heaviest hub rows, which are split and reduced, are part of it
    print("oracle on all rows ...", flush=True)
    worst = 0.0
    for s0 in range(0, w.n, 1 << 20):
        slab = np.arange(s0, min(w.n, s0 + (1 << 20)), dtype=np.int64)
        Yref, B = oracle.spmm(w.rowptr, w.colidx, w.vals, X, rows=slab)
        Ys = Yd[s0:s0 + len(slab)].cpu().numpy()
        check(Ys, Yref, B)
        worst = max(worst, float(np.max(np.abs(Ys - Yref) / np.maximum(B, 1e-300))))
    print(f"max err / bound over all rows = {worst:.2e}", flush=True)
    assert worst < 1e-5
    # properties that hold at any size: column sums  1^T Y = (1^T A) X  in fp64
    colsum = torch.zeros(w.k, dtype=torch.float64, device="cuda")
    for s in range(0, w.n, 1 << 20):
        colsum += Yd[s:s + (1 << 20)].double().sum(0)
    ata = np.zeros(w.n, np.float64)
    np.add.at(ata, w.colidx, w.vals.astype(np.float64))          # 1^T A
    want = ata @ X.astype(np.float64)
    scale = np.abs(ata) @ np.abs(X.astype(np.float64))
    assert np.all(np.abs(colsum.cpu().numpy() - want) <= 1e-5 * scale)

    # the sampled dense-dense product on the same handle: S = A .* (U V^T), U = X
    print("sampled product ...", flush=True)
    V = synth.normal_matrix(w.n, w.k, seed=w.seed_x + 1)
    Vd = torch.from_numpy(V).cuda()
    Sd = torch.full((w.nnz,), float("nan"), dtype=torch.float32, device="cuda")
    op.sddmm(Xd, Vd, Sd)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Sd).any())              # every element of S was written
    # the operand restricted to the sampled rows (all other rows empty), so the oracle's output
    # is the sampled rows' entries in CSR order
    cnt = np.zeros(w.n, np.int64)
    cnt[rows] = deg[rows]
    rp = np.concatenate([[0], np.cumsum(cnt)])
    first = np.cumsum(deg[rows]) - deg[rows]
    idx = np.repeat(w.rowptr[rows] - first, deg[rows]) + np.arange(int(deg[rows].sum()), dtype=np.int64)
    print(f"oracle on {len(idx)} sampled entries ...", flush=True)
    Sref, Bs = oracle.sddmm(rp, w.colidx[idx], w.vals[idx], X, V)
    Ss = Sd[torch.from_numpy(idx).cuda()].cpu().numpy()
    check(Ss, Sref, Bs)
    # a property that holds at any size: sum_p S[p] = sum_i <U[i], (A V)[i]>, scaled by the same
    # product with |U|, |V| (a bound on sum_p |a_p| <|U[i]|, |V[j]|> up to fp32 rounding)
    op.spmm(Vd, Yd)
    lhs = float(Sd.double().sum())
    rhs = float((Xd.double() * Yd.double()).sum())
    Sa = op.sddmm(Xd.abs(), Vd.abs())
    assert abs(lhs - rhs) <= 2e-5 * float(Sa.double().abs().sum())
    op.close()


def test_config4_chung_lu_16m_fifth_power_sampled(torch):
    """Chung-Lu, n = 16,777,216, row-normalised, A^5.X with k = 32: hub-heavy arrow heads and
    many levels.  The fp64 iterate is computed in full by the oracle (17 GB of host memory)."""
    print("generating Chung-Lu n=2^24 ...", flush=True)
    w = synth.make_config(4)
    print(f"decomposing n={w.n} nnz={w.nnz} ...", flush=True)
    op = binding.ArrowSpMM(w.rowptr, w.colidx, w.vals, w.b)
    X = w.make_x()
    Xd = torch.from_numpy(X).cuda()
    print(f"levels={op.info['levels']}; five chained products ...", flush=True)
    op.spmm_iter(Xd, w.l)
    torch.cuda.synchronize()
    print("oracle: five fp64 products ...", flush=True)
    Xl, El = oracle.spmm_iter(w.rowptr, w.colidx, w.vals, X, w.l)
    got = Xd.cpu().numpy()
    # whole result, in slabs to bound temporaries
    for s in range(0, w.n, 1 << 21):
        check(got[s:s + (1 << 21)], Xl[s:s + (1 << 21)], El[s:s + (1 << 21)], scale=w.l)
    op.close()


@pytest.mark.parametrize("idx", [0, 1])
def test_mttkrp_tensor_workloads_full(torch, idx):
    """Order-3 MTTKRP at the sizes ``bench.py --op mttkrp`` times: the uniform 4096^3 tensor at
    density 0.1 % and the skewed 2^20 x 2^17 x 2^17 tensor, R = 64; the whole result is compared."""
    print(f"generating tensor workload {idx} ...", flush=True)
    w = synth.make_tensor_config(idx)
    B, C = w.factors()
    print(f"building nnz={w.nnz} ...", flush=True)
    op = binding.Csf3Mttkrp(w.dims, w.i, w.j, w.k, w.vals)
    Ad = torch.full((w.dims[0], w.R), float("nan"), dtype=torch.float32, device="cuda")
    op.mttkrp(torch.from_numpy(B).cuda(), torch.from_numpy(C).cuda(), Ad)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(Ad).any())
    print("oracle ...", flush=True)
    Aref, E = oracle.mttkrp(w.dims, w.i, w.j, w.k, w.vals, B, C)
    check(Ad.cpu().numpy(), Aref, E)
    op.close()
