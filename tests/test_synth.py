"""Seeded input generators: shapes, structure and determinism (no arithmetic of the method)."""
import numpy as np
import scipy.sparse as sp

from paper_2307_05740_amd import synth


def _check_csr(rp, ci, n):
    assert rp.dtype == np.int64 and ci.dtype == np.int32 and rp.shape == (n + 1,)
    assert rp[0] == 0 and np.all(np.diff(rp) >= 0) and rp[-1] == ci.shape[0]
    assert ci.min() >= 0 and ci.max() < n
    rows = np.repeat(np.arange(n), np.diff(rp))
    key = rows.astype(np.int64) * n + ci
    assert np.all(np.diff(key) > 0), "columns must be sorted and duplicate-free inside every row"


def _is_symmetric(rp, ci, n):
    A = sp.csr_matrix((np.ones(ci.shape[0]), ci, rp), shape=(n, n))
    return (A - A.T).nnz == 0


def test_rmat_pattern_structure_and_determinism():
    rp, ci = synth.rmat_pattern(12, 65536, seed=7)
    _check_csr(rp, ci, 4096)
    assert _is_symmetric(rp, ci, 4096)
    assert 65536 < rp[-1] <= 131072               # merged duplicates, both directions stored
    rp2, ci2 = synth.rmat_pattern(12, 65536, seed=7)
    assert np.array_equal(rp, rp2) and np.array_equal(ci, ci2)
    rp3, _ = synth.rmat_pattern(12, 65536, seed=8)
    assert not np.array_equal(rp, rp3)
    deg = np.diff(rp)
    assert deg[0] == deg.max()                    # a = 0.57 concentrates mass on low ids
    # quadrant convention: b and c are symmetric here, so check a > d via id halves
    assert deg[:2048].sum() > 2 * deg[2048:].sum()


def test_grid_pattern_counts():
    for N in (1, 2, 5, 32):
        rp, ci = synth.grid5_pattern(N)
        _check_csr(rp, ci, N * N)
        assert rp[-1] == 5 * N * N - 4 * N
        assert _is_symmetric(rp, ci, N * N)
        vals = synth.fill_grid5(rp, ci)
        assert vals.sum() == 4 * N * N - (4 * N * N - 4 * N)


def test_chung_lu_is_power_law_like():
    n = 1 << 14
    rp, ci = synth.chung_lu_pattern(n, 2.1, 20.0, n / 4, seed=5)
    _check_csr(rp, ci, n)
    assert _is_symmetric(rp, ci, n)
    deg = np.diff(rp)
    assert 10 < deg.mean() <= 20 and deg.max() > 40 * deg.mean()
    assert deg[:16].min() > np.median(deg) * 10      # weights decrease with the vertex id


def test_value_fills():
    rp, ci = synth.rmat_pattern(10, 8192, seed=1)
    v = synth.fill_uniform(rp, ci, seed=2)
    assert v.dtype == np.float32 and v.min() >= -1 and v.max() < 1
    assert abs(v.mean()) < 0.02 and abs(v.var() - 1 / 3) < 0.02
    assert np.array_equal(v, synth.fill_uniform(rp, ci, seed=2))
    w = synth.fill_row_normalized(rp)
    deg = np.diff(rp)
    rows = np.repeat(np.arange(1024), deg)
    assert np.array_equal(w, (1.0 / deg[rows]).astype(np.float32))


def test_normal_matrix_moments_and_determinism():
    X = synth.normal_matrix(4096, 16, seed=9)
    assert X.dtype == np.float32 and X.shape == (4096, 16)
    assert abs(X.mean()) < 0.02 and abs(X.std() - 1) < 0.02
    assert abs(np.mean(X ** 4) - 3) < 0.2
    assert abs(np.corrcoef(X[:, 0], X[:, 1])[0, 1]) < 0.05
    assert np.array_equal(X, synth.normal_matrix(4096, 16, seed=9))
    Xo = synth.normal_matrix(100, 3, seed=9)           # odd k: last column alone in its pair
    assert np.isfinite(Xo).all()


def test_named_configs_small():
    w = synth.make_config(0)
    assert (w.n, w.k, w.b, w.l) == (4096, 16, 512, 1) and w.nnz <= 131072
    w = synth.make_config(3, shrink=9)
    assert (w.n, w.k, w.b, w.l) == (1 << 14, 128, 512, 1)
    w = synth.make_config(1, shrink=8)
    assert (w.n, w.k, w.b) == (64 * 64, 32, 256)
    w = synth.make_config(2, shrink=8)
    assert (w.n, w.k, w.l) == (4096, 64, 3) and np.allclose(w.vals[:w.rowptr[1]].sum(), 1, atol=1e-6)
    w = synth.make_config(4, shrink=10)
    assert (w.n, w.k, w.l) == (16384, 32, 5)
