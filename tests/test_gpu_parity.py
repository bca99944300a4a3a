"""GPU parity: the HIP path, called through the C-ABI, against the fp64 CPU oracle on the same
seeded inputs.  Bar (elementwise): |Y - Yref| <= 1e-5 * (|A|.|X|), times l for chained products,
and exactly 0 where the bound is 0 (empty rows)."""
import os

import numpy as np
import pytest

import oracle
from oracle import arrow_checks
from paper_2307_05740_amd import binding, synth

pytestmark = pytest.mark.gpu

TOL = 1e-5


@pytest.fixture(scope="module")
def torch():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the parity tests need a real MI355X")
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libarrow.so is not built")
    return torch


def assert_within(Y, Yref, B, scale=1.0):
    Y = np.asarray(Y, dtype=np.float64)
    err = np.abs(Y - Yref)
    lim = scale * TOL * B
    bad = err > lim
    if bad.any():
        i = np.unravel_index(np.argmax(err - lim), err.shape)
        raise AssertionError(f"{bad.sum()} of {bad.size} elements outside the bound; worst at {i}: "
                             f"got {Y[i]!r} want {Yref[i]!r} bound {lim[i]!r}")
    assert np.all(Y[B == 0] == 0)
    # the bound is not vacuous: typical error is far below it
    nz = B > 0
    if nz.any():
        assert np.median(err[nz] / B[nz]) < 1e-6


def run_product(torch, w_or_csr, b, X, **opts):
    rowptr, colidx, vals = w_or_csr
    op = binding.ArrowSpMM(rowptr, colidx, vals, b)
    for name, v in opts.items():
        binding.arrow_set_option(op.h, name, v)
    Xd = torch.from_numpy(X).cuda()
    Yd = torch.full_like(Xd, float("nan"))          # every element must be written
    op.spmm(Xd, Yd)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()
    return op, Xd, Y


def csr_of(w):
    return (w.rowptr, w.colidx, w.vals)


def test_config0_rmat_s12_k16(torch):
    w = synth.make_config(0)
    X = w.make_x()
    op, Xd, Y = run_product(torch, csr_of(w), w.b, X)
    Yref, B = oracle.spmm(*csr_of(w), X)
    assert_within(Y, Yref, B)
    assert op.info["levels"] >= 1
    # run-to-run bitwise reproducibility (no floating-point atomics)
    Y2 = op.spmm(Xd).cpu().numpy()
    assert np.array_equal(Y.view(np.uint32), Y2.view(np.uint32))
    op.close()


@pytest.mark.parametrize("k", [1, 2, 3, 4, 6, 7, 12, 16, 20, 33, 64, 100, 128, 130, 200, 256, 260, 516])
def test_all_column_counts(torch, k):
    w = synth.make_config(0, shrink=1)              # n = 2048, b = 256
    X = synth.normal_matrix(w.n, k, seed=100 + k)
    op, _, Y = run_product(torch, csr_of(w), w.b, X)
    Yref, B = oracle.spmm(*csr_of(w), X)
    assert_within(Y, Yref, B)
    op.close()


@pytest.mark.parametrize("opts", [dict(kc=16), dict(kc=32), dict(kc=64), dict(kc=200),
                                  dict(l2_resident_bytes=1 << 16)])
def test_launch_options(torch, opts):
    w = synth.make_config(3, shrink=9)              # R-MAT scale 14, k = 128, b = 512
    X = w.make_x()
    op, _, Y = run_product(torch, csr_of(w), w.b, X, **opts)
    Yref, B = oracle.spmm(*csr_of(w), X)
    assert_within(Y, Yref, B)
    op.close()


@pytest.mark.parametrize("b", [1, 5, 64, 1000, 2048, 5000])
def test_block_widths(torch, b):
    w = synth.make_config(0, shrink=1)
    X = synth.normal_matrix(w.n, 24, seed=7)
    op, _, Y = run_product(torch, csr_of(w), b, X)
    Yref, B = oracle.spmm(*csr_of(w), X)
    assert_within(Y, Yref, B)
    op.close()


def test_pack_options_short_and_chunk(torch, monkeypatch):
    w = synth.make_config(0)
    X = synth.normal_matrix(w.n, 32, seed=8)
    Yref, B = oracle.spmm(*csr_of(w), X)
    for short_max, chunk in ((0, 7), (4, 64), (64, 100000), (1000000, 512)):
        monkeypatch.setenv("ARROW_SHORT_MAX", str(short_max))
        monkeypatch.setenv("ARROW_CHUNK_NNZ", str(chunk))
        op, _, Y = run_product(torch, csr_of(w), w.b, X)
        assert_within(Y, Yref, B)
        op.close()


@pytest.mark.parametrize("env", [
    dict(ARROW_CLASSES="0", ARROW_STAGE_HEAD="0"),
    dict(ARROW_CLASSES="0", ARROW_STAGE_HEAD="1"),
    dict(ARROW_CLASSES="8", ARROW_CLASS_MIN="2", ARROW_CLASS_GRAN="16"),
    dict(ARROW_CLASSES="16", ARROW_CLASS_MIN="1", ARROW_CLASS_GRAN="1", ARROW_SHORT_MAX="0"),
    dict(ARROW_CLASSES="24", ARROW_CLASS_MIN="4", ARROW_CLASS_GRAN="64", ARROW_STAGE_HEAD="0"),
    dict(ARROW_CLASSES="16", ARROW_CLASS_MIN="8", ARROW_CHUNK_NNZ="16", ARROW_WINDOW_ROWS="128"),
    dict(ARROW_CLASSES="16", ARROW_CLASS_MIN="2", ARROW_PIECE_MAX="0"),
    dict(ARROW_CLASSES="16", ARROW_CLASS_MIN="2", ARROW_PIECE_MAX="1000000", ARROW_CLASS_GRAN="32"),
    dict(ARROW_CLASSES="8", ARROW_CLASS_MIN="3", ARROW_PIECE_MAX="5", ARROW_SHORT_MAX="2"),
    dict(ARROW_STAGE_SHORT="1", ARROW_EMPTY_LAST="1"),
    dict(ARROW_STAGE_SHORT="0", ARROW_EMPTY_LAST="0"),
    dict(ARROW_STAGE_SHORT="1", ARROW_SHORT_MAX="64", ARROW_CLASSES="8", ARROW_CLASS_MIN="2"),
])
@pytest.mark.parametrize("k", [16, 128, 36])
def test_die_queues_and_head_staging(torch, monkeypatch, env, k):
    """Column classes, die queues with padding slots, and the staged head buffer."""
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    w = synth.make_config(0)
    X = synth.normal_matrix(w.n, k, seed=9 + k)
    Yref, B = oracle.spmm(*csr_of(w), X)
    for opts in (dict(), dict(kc=16)):
        op, _, Y = run_product(torch, csr_of(w), w.b, X, **opts)
        assert_within(Y, Yref, B)
        op.close()


@pytest.mark.parametrize("env", [
    dict(ARROW_WINDOW_ROWS="64"),
    dict(ARROW_WINDOW_ROWS="32", ARROW_PANEL_MIN="1", ARROW_SHORT_MAX="0"),
    dict(ARROW_WINDOW_ROWS="128", ARROW_CHUNK_MIN="16"),
    dict(ARROW_WINDOW_ROWS="64", ARROW_HEAD_BY_ID="0"),
])
@pytest.mark.parametrize("k", [1, 3, 6, 16, 36, 64, 128, 130, 260])
def test_head_panels(torch, monkeypatch, env, k):
    """Head rows whose head-block entries run in panels (accumulators in LDS, added to Y last);
    small windows make the head span several of them so that panels are formed."""
    monkeypatch.setenv("ARROW_PANEL", "1")
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    w = synth.make_config(0)
    X = synth.normal_matrix(w.n, k, seed=77 + k)
    op, Xd, Y = run_product(torch, csr_of(w), w.b, X)
    lv = op.levels()
    assert lv[0]["panel_rows"] > 0 and lv[0]["nnz_panel"] > 0
    Yref, B = oracle.spmm(*csr_of(w), X)
    assert_within(Y, Yref, B)
    Y2 = op.spmm(Xd).cpu().numpy()
    assert np.array_equal(Y.view(np.uint32), Y2.view(np.uint32))
    op.close()


def test_head_panels_larger_operand_and_chained(torch, monkeypatch):
    monkeypatch.setenv("ARROW_PANEL", "1")
    monkeypatch.setenv("ARROW_WINDOW_ROWS", "64")
    w = synth.make_config(4, shrink=8)              # Chung-Lu, 65536 vertices, k = 32, A^5
    X = w.make_x()
    op = binding.ArrowSpMM(*csr_of(w), w.b)
    assert op.levels()[0]["panel_rows"] > 256       # several workgroups of panels
    Xd = torch.from_numpy(X).cuda()
    op.spmm_iter(Xd, w.l)
    Xl, El = oracle.spmm_iter(*csr_of(w), X, w.l)
    assert_within(Xd.cpu().numpy(), Xl, El, scale=w.l)
    op.close()


def test_grid_one_level(torch):
    w = synth.make_config(1, shrink=4)              # 256 x 256 grid, k = 32, b = 4096
    X = w.make_x()
    op, _, Y = run_product(torch, csr_of(w), w.b, X)
    assert op.info["levels"] == 1
    Yref, B = oracle.spmm(*csr_of(w), X)
    assert_within(Y, Yref, B)
    # closed form: the operator applied to ones is 4 - (number of neighbours), exactly
    ones = np.ones((w.n, 4), np.float32)
    Y1 = op.spmm(torch.from_numpy(ones).cuda()).cpu().numpy().reshape(256, 256, 4)
    assert np.all(Y1[1:-1, 1:-1] == 0) and np.all(Y1[0, 1:-1] == 1) and Y1[0, 0, 0] == 2
    op.close()


@pytest.mark.parametrize("k", [4, 7, 32, 36, 130])
def test_diagonal_blocks_with_lds_window(torch, monkeypatch, k):
    """Grid operator: the stencil sits in the diagonal blocks, whose X window is staged in LDS
    (the reuse threshold is lowered: by default a five-point stencil is left to the L2)."""
    monkeypatch.setenv("ARROW_WINDOW_REUSE_X10", "20")
    w = synth.make_config(1, shrink=6)              # 128 x 128 grid
    X = synth.normal_matrix(w.n, k, seed=40 + k)
    op, _, Y = run_product(torch, csr_of(w), 2048, X)
    lv = op.levels()
    assert lv[0]["window_tiles"] > 0 and lv[0]["nnz_window"] > 0.5 * w.nnz
    Yref, B = oracle.spmm(*csr_of(w), X)
    assert_within(Y, Yref, B)
    op.close()


def test_dense_diagonal_blocks_use_lds_window_by_default(torch):
    """Block-diagonal operand with 24 entries per row inside blocks of 256: every block's window
    is reused 24 times, which the default rule accepts."""
    rng = np.random.default_rng(21)
    n, b, k = 8192, 256, 36
    rows = np.repeat(np.arange(n), 24)
    cols = (rows // b) * b + rng.integers(0, b, rows.shape[0])
    key = np.unique(rows.astype(np.int64) * n + cols)
    rows, cols = key // n, key % n
    rowptr = np.zeros(n + 1, np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    colidx = cols.astype(np.int32)
    vals = synth.fill_uniform(rowptr, colidx, seed=22)
    X = synth.normal_matrix(n, k, seed=23)
    op, _, Y = run_product(torch, (rowptr, colidx, vals), b, X)
    lv = op.levels()
    assert lv[0]["window_tiles"] >= n // b - 1 and lv[0]["nnz_window"] > 0.9 * len(vals)
    Yref, B = oracle.spmm(rowptr, colidx, vals, X)
    assert_within(Y, Yref, B)
    op.close()


@pytest.mark.parametrize("fuse", ["0", "1"])
def test_lds_window_on_a_later_level_accumulates(torch, monkeypatch, fuse):
    """Banded operator plus scattered far entries and a few hubs: with the separator rule off the
    band is cut at block boundaries, so later levels own banded diagonal blocks and must add
    (levels run one after the other), or their entries join the window rows of level 0 and are
    read from memory there (fused levels)."""
    monkeypatch.setenv("ARROW_FUSE_LEVELS", fuse)
    monkeypatch.setenv("ARROW_SEPARATORS", "0")
    monkeypatch.setenv("ARROW_WINDOW_REUSE_X10", "5")
    monkeypatch.setenv("ARROW_WINDOW_SHARE_X1000", "0")
    rng = np.random.default_rng(12)
    n, b, k = 6000, 500, 20
    rows, cols = [], []
    for d in (-3, -2, -1, 0, 1, 2, 3):
        i = np.arange(max(0, -d), min(n, n - d))
        rows.append(i); cols.append(i + d)
    far = rng.integers(0, n, (3000, 2))
    rows += [far[:, 0], far[:, 1]]; cols += [far[:, 1], far[:, 0]]
    rows = np.concatenate(rows); cols = np.concatenate(cols)
    key = np.unique(rows.astype(np.int64) * n + cols)
    rows, cols = key // n, key % n
    rowptr = np.zeros(n + 1, np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    colidx = cols.astype(np.int32)
    vals = synth.fill_uniform(rowptr, colidx, seed=13)
    X = synth.normal_matrix(n, k, seed=14)
    op, _, Y = run_product(torch, (rowptr, colidx, vals), b, X)
    lv = op.levels()
    assert len(lv) >= 2 and sum(l["window_tiles"] for l in lv) > 0
    Yref, B = oracle.spmm(rowptr, colidx, vals, X)
    assert_within(Y, Yref, B)
    monkeypatch.setenv("ARROW_WINDOW_SPAN", "0")                 # same operand without LDS tiles
    op2, _, Y2 = run_product(torch, (rowptr, colidx, vals), b, X)
    assert sum(l["window_tiles"] for l in op2.levels()) == 0
    assert_within(Y2, Yref, B)
    op.close(); op2.close()


def test_hub_row_is_split_and_reduced(torch):
    # one vertex adjacent to everything: its row has n entries -> many chunks + reduction
    n, k, b = 40000, 20, 1024
    rows = np.concatenate([np.zeros(n, np.int64), np.arange(1, n)])
    cols = np.concatenate([np.arange(n), np.zeros(n - 1, np.int64)])
    order = np.lexsort((cols, rows))
    rows, cols = rows[order], cols[order]
    rowptr = np.zeros(n + 1, np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    colidx = cols.astype(np.int32)
    vals = synth.fill_uniform(rowptr, colidx, seed=5)
    X = synth.normal_matrix(n, k, seed=6)
    op, _, Y = run_product(torch, (rowptr, colidx, vals), b, X)
    assert op.levels()[0]["split_rows"] >= 1
    Yref, B = oracle.spmm(rowptr, colidx, vals, X)
    assert_within(Y, Yref, B)
    op.close()


def _csr(n, rows, cols, seed):
    key = np.unique(np.asarray(rows, np.int64) * n + np.asarray(cols, np.int64))
    rows, cols = key // n, key % n
    rowptr = np.zeros(n + 1, np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    colidx = cols.astype(np.int32)
    return rowptr, colidx, synth.fill_uniform(rowptr, colidx, seed=seed)


@pytest.mark.parametrize("lower", [False, True])
def test_directed_operands(torch, lower):
    """Non-symmetric operands: a pure shift (strictly triangular, every vertex has a row entry or
    a column entry, seldom both), and a strictly triangular random pattern with a few full rows.
    The decomposition takes adjacency from A + A^T; the product must still be A X, not A^T X."""
    n, b, k = 4096, 64, 20
    i = np.arange(n - 300)
    r, c = (i + 100, i) if lower else (i, i + 100)
    csr = _csr(n, r, c, seed=31)
    X = synth.normal_matrix(n, k, seed=32)
    op, _, Y = run_product(torch, csr, b, X)
    assert op.info["levels"] <= 2
    Yref, B = oracle.spmm(*csr, X)
    assert_within(Y, Yref, B)
    op.close()
    rng = np.random.default_rng(33)
    n, b, k = 20000, 256, 36
    m = 16 * n
    r = rng.integers(0, n, m)
    c = rng.integers(0, n, m)
    hubs = rng.integers(0, n, 5)
    r = np.concatenate([r, np.repeat(hubs, n // 2)])
    c = np.concatenate([c, rng.integers(0, n, 5 * (n // 2))])
    keep = (r > c) if lower else (r < c)
    csr = _csr(n, r[keep], c[keep], seed=34)
    X = synth.normal_matrix(n, k, seed=35)
    op, _, Y = run_product(torch, csr, b, X)
    levels = [binding.arrow_export_level(op.h, i) for i in range(op.info["levels"])]
    arrow_checks.check_decomposition(n, *csr, b, levels)
    Yref, B = oracle.spmm(*csr, X)
    assert_within(Y, Yref, B)
    op.close()


@pytest.mark.parametrize("idx,shrink,k", [(3, 8, 128), (4, 8, 32), (2, 6, 36), (0, 0, 7)])
def test_fused_and_separate_levels(torch, monkeypatch, idx, shrink, k):
    """One launch set that sums over all arrow matrices (fused levels, the default) against one
    launch set per level with a read-modify-write of Y in between: both within the bound of the
    oracle, on operands with several levels."""
    w = synth.make_config(idx, shrink=shrink)
    X = synth.normal_matrix(w.n, k, seed=300 + k)
    Yref, B = oracle.spmm(*csr_of(w), X)
    seen = {}
    for fuse in ("1", "0"):
        monkeypatch.setenv("ARROW_FUSE_LEVELS", fuse)
        op, Xd, Y = run_product(torch, csr_of(w), w.b, X)
        lv = op.levels()
        assert len(lv) >= 2
        seen[fuse] = [l["nnz_rows"] + l["nnz_chunks"] + l["nnz_window"] + l["nnz_panel"] + l["nnz_corner"] for l in lv]
        assert_within(Y, Yref, B)
        Z = torch.from_numpy(X).cuda()
        op.spmm_iter(Z, 2)
        X2, E2 = oracle.spmm_iter(*csr_of(w), X, 2)
        assert_within(Z.cpu().numpy(), X2, E2, scale=2)
        op.close()
    assert all(x == 0 for x in seen["1"][1:]) and all(x > 0 for x in seen["0"][1:])
    assert sum(seen["1"]) == sum(seen["0"]) == w.nnz


@pytest.mark.parametrize("env", [
    dict(ARROW_HUBS_FIRST="65536"),
    dict(ARROW_HUBS_FIRST="65536", ARROW_CORNER_MIN_TILE="1"),
    dict(ARROW_HUBS_FIRST="300", ARROW_CORNER_MAX="256", ARROW_FUSE_LEVELS="0"),
    dict(ARROW_HUBS_FIRST="0", ARROW_CORNER_MIN_TILE="200"),
])
@pytest.mark.parametrize("k", [1, 3, 16, 36, 64, 128, 130, 260])
def test_dense_corner_tiles(torch, monkeypatch, env, k):
    """The dense corner of the head block in LDS tiles (staged head rows and accumulators in LDS),
    on and off, against the oracle; bitwise repeatable."""
    w = synth.make_config(3, shrink=8)              # R-MAT scale 15, b = 1024: corners of 256 .. 1024
    X = synth.normal_matrix(w.n, k, seed=500 + k)
    Yref, B = oracle.spmm(*csr_of(w), X)
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    for corner in ("1", "0"):
        monkeypatch.setenv("ARROW_CORNER", corner)
        op, Xd, Y = run_product(torch, csr_of(w), w.b, X)
        lv = op.levels()
        assert (lv[0]["nnz_corner"] > 0) == (corner == "1")
        assert_within(Y, Yref, B)
        Y2 = op.spmm(Xd).cpu().numpy()
        assert np.array_equal(Y.view(np.uint32), Y2.view(np.uint32))
        op.close()


def test_dense_corner_larger_operand_and_chained(torch, monkeypatch):
    monkeypatch.setenv("ARROW_CORNER", "1")
    monkeypatch.setenv("ARROW_HUBS_FIRST", "65536")
    w = synth.make_config(4, shrink=6)              # Chung-Lu, 262144 vertices, k = 32, b = 4096, A^5
    X = w.make_x()
    op = binding.ArrowSpMM(*csr_of(w), w.b)
    lv = op.levels()
    assert lv[0]["corner"] >= 1024 and lv[0]["corner_items"] > lv[0]["corner"] // 256   # panels cut into several items
    Xd = torch.from_numpy(X).cuda()
    op.spmm_iter(Xd, w.l)
    Xl, El = oracle.spmm_iter(*csr_of(w), X, w.l)
    assert_within(Xd.cpu().numpy(), Xl, El, scale=w.l)
    op.close()


def test_special_operands_bitwise(torch):
    rng = np.random.default_rng(3)
    n, k = 3000, 12
    X = rng.standard_normal((n, k)).astype(np.float32)
    rp = np.arange(n + 1, dtype=np.int64)
    perm = rng.permutation(n).astype(np.int32)
    d = rng.uniform(-2, 2, n).astype(np.float32)
    for colidx, vals, want in ((np.arange(n, dtype=np.int32), np.ones(n, np.float32), X),
                               (perm, np.ones(n, np.float32), X[perm]),
                               (np.arange(n, dtype=np.int32), d, d[:, None] * X)):
        op, _, Y = run_product(torch, (rp, colidx, vals), 256, X)
        assert np.array_equal(Y, want.astype(np.float32))     # one term per row: no rounding freedom
        op.close()
    # empty operand: Y is all zeros
    op, _, Y = run_product(torch, (np.zeros(n + 1, np.int64), np.zeros(0, np.int32), np.zeros(0, np.float32)),
                           256, X)
    assert np.all(Y == 0)
    op.close()


def test_gather_kernel_matches_exported_permutation(torch):
    w = synth.make_config(2, shrink=8)
    X = w.make_x()
    op = binding.ArrowSpMM(*csr_of(w), w.b)
    Xd = torch.from_numpy(X).cuda()
    for level in range(op.info["levels"]):
        perm = binding.arrow_export_level(op.h, level)[0]
        Xp = op.gather(level, Xd).cpu().numpy()
        assert np.array_equal(Xp, X[perm])
    op.close()


@pytest.mark.parametrize("idx,shrink", [(2, 6), (4, 8)])
def test_chained_products(torch, idx, shrink):
    w = synth.make_config(idx, shrink=shrink)       # row-normalised operands, A^3 / A^5
    X = w.make_x()
    op = binding.ArrowSpMM(*csr_of(w), w.b)
    for l in (0, 1, 2, w.l):
        Xd = torch.from_numpy(X).cuda()
        op.spmm_iter(Xd, l)
        torch.cuda.synchronize()
        Xl, El = oracle.spmm_iter(*csr_of(w), X, l)
        if l == 0:
            assert np.array_equal(Xd.cpu().numpy(), X)
        else:
            assert_within(Xd.cpu().numpy(), Xl, El, scale=l)
    op.close()


def test_grid_eigenvector_powers(torch):
    N = 64
    rp, ci = synth.grid5_pattern(N)
    vals = synth.fill_grid5(rp, ci)
    xs = np.arange(1, N + 1)
    v = np.outer(np.sin(np.pi * 3 * xs / (N + 1)), np.sin(np.pi * 2 * xs / (N + 1))).reshape(-1, 1)
    lam = 4 - 2 * np.cos(np.pi * 2 / (N + 1)) - 2 * np.cos(np.pi * 3 / (N + 1))
    X = np.repeat(v, 4, axis=1).astype(np.float32)
    op = binding.ArrowSpMM(rp, ci, vals, 1024)
    Xd = torch.from_numpy(X).cuda()
    op.spmm_iter(Xd, 4)
    got = Xd.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(got - lam ** 4 * X) <= 4 * TOL * 8.0 ** 4 * np.abs(X).max())
    op.close()


def test_loaded_handle_gives_the_same_product(torch, tmp_path):
    w = synth.make_config(3, shrink=8)
    X = w.make_x()
    op, Xd, Y = run_product(torch, csr_of(w), w.b, X)
    path = str(tmp_path / "levels.arrow")
    binding.arrow_save(op.h, path)
    op2 = binding.ArrowSpMM(handle=binding.arrow_load(path))
    Y2 = op2.spmm(Xd).cpu().numpy()
    assert np.array_equal(Y.view(np.uint32), Y2.view(np.uint32))   # same image, same order of sums
    op.close(); op2.close()


def test_errors_on_device(torch):
    w = synth.make_config(0, shrink=3)
    op = binding.ArrowSpMM(*csr_of(w), w.b)
    Xd = torch.zeros((w.n, 8), device="cuda")
    op.spmm(Xd)
    with pytest.raises(binding.ArrowError) as ei:                     # in place is refused
        binding.arrow_spmm(op.h, Xd.data_ptr(), Xd.data_ptr(), 8, 0)
    assert ei.value.code == binding.ARROW_EINVAL
    # partial overlap of X and Y, and operands inside the workspace, are refused as well
    big = torch.zeros((2 * w.n, 8), device="cuda")
    half = big.data_ptr() + w.n * 8 * 4 // 2
    half -= half % 16
    for x_ptr, y_ptr in ((big.data_ptr(), half), (half, big.data_ptr()),
                         (Xd.data_ptr(), op._ws.data_ptr()), (op._ws.data_ptr() + 256, big.data_ptr())):
        with pytest.raises(binding.ArrowError) as ei:
            binding.arrow_spmm(op.h, x_ptr, y_ptr, 8, 0)
        assert ei.value.code == binding.ARROW_EINVAL and "overlap" in str(ei.value)
    with pytest.raises(binding.ArrowError) as ei:
        binding.arrow_spmm_static(op.h, big.data_ptr(), half, 8, 0)
    assert ei.value.code == binding.ARROW_EINVAL
    with pytest.raises(binding.ArrowError) as ei:                     # workspace bound for k = 8 only
        binding.arrow_spmm_iter(op.h, Xd.data_ptr(), 64, 2, 0)
    assert ei.value.code == binding.ARROW_ETOOSMALL
    op.close()


def test_exported_levels_match_what_the_gpu_ran(torch):
    """Invariants on the very handle the GPU product used (bit-exact reassembly, arrow shape)."""
    w = synth.make_config(3, shrink=8)              # R-MAT scale 15, b = 1024
    X = w.make_x()
    op, _, Y = run_product(torch, csr_of(w), w.b, X)
    levels = [binding.arrow_export_level(op.h, i) for i in range(op.info["levels"])]
    arrow_checks.check_decomposition(w.n, w.rowptr, w.colidx, w.vals, w.b, levels)
    Yref, B = oracle.spmm(*csr_of(w), X)
    assert_within(Y, Yref, B)
    op.close()


def test_product_under_graph_capture(torch):
    """The product only launches kernels on the caller's stream (no allocation, no memset), so a
    caller can capture it into a HIP graph; every replay is checked against the eager result, with
    eager work and synchronisation between the replays."""
    w = synth.make_config(0)
    op = binding.ArrowSpMM(*csr_of(w), w.b)
    Xs = [synth.normal_matrix(w.n, 24, seed=900 + t) for t in range(3)]
    Xd = torch.from_numpy(Xs[0]).cuda()
    Yd = torch.empty_like(Xd)
    Zd = Xd.clone()
    op.spmm(Xd, Yd)                                     # eager first: sizes the workspace
    op.spmm_iter(Zd, 3)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        op.spmm(Xd, Yd)                                 # Y = A X
        Zd.copy_(Xd)
        op.spmm_iter(Zd, 3)                             # Z = A^3 X (odd count: ends with a device copy)
    for t in range(3):
        Xd.copy_(torch.from_numpy(Xs[t]).cuda())
        g.replay()
        torch.cuda.synchronize()
        Yg, Zg = Yd.cpu().numpy(), Zd.cpu().numpy()
        Xe = torch.from_numpy(Xs[t]).cuda()
        Ye = op.spmm(Xe).cpu().numpy()                  # eager work between the replays
        Ze = Xe.clone()
        op.spmm_iter(Ze, 3)
        torch.cuda.synchronize()
        assert np.array_equal(Yg.view(np.uint32), Ye.view(np.uint32)), t
        assert np.array_equal(Zg.view(np.uint32), Ze.cpu().numpy().view(np.uint32)), t
        Yref, B = oracle.spmm(*csr_of(w), Xs[t])
        assert_within(Yg, Yref, B)
    op.close()


def test_gather_probe_runs_and_validates(torch):
    """The bare row gather that bench.py uses as its yardstick: every mode launches and completes;
    regions that do not fit, unsupported k and short output buffers are refused on the host."""
    n, k = 1 << 16, 128
    X = torch.ones((n, k), device="cuda")
    gathers = 1 << 20
    nbytes = binding.arrow_probe_gather_out_bytes(gathers)
    out = torch.zeros(nbytes // 4, device="cuda")
    for rows, per_die, lds in ((128, True, True), (4096, True, False), (n, False, False)):
        binding.arrow_probe_gather(X.data_ptr(), n, k, rows, per_die, lds, gathers, out.data_ptr(), nbytes)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        # X is all ones: a lane sums 4 columns of the 2048 / 2 rows its lane group reads (16 times
        # as many when the region sits in LDS, with 16 times fewer wavefronts)
        reps = 16 if lds else 1
        assert np.all(got[: (gathers // (2048 * reps)) * 64] == 4 * 1024 * reps)
    for bad in (dict(k=24), dict(rows=n, per_die=True), dict(rows=256, lds=True), dict(nbytes=64)):
        a = dict(k=k, rows=4096, per_die=False, lds=False, nbytes=nbytes)
        a.update(bad)
        with pytest.raises(binding.ArrowError):
            binding.arrow_probe_gather(X.data_ptr(), n, a["k"], a["rows"], a["per_die"], a["lds"], gathers,
                                       out.data_ptr(), a["nbytes"])


def test_explicit_options_and_repack(torch):
    """Options passed as a struct instead of through the environment, and an image rebuilt on the
    same handle with other options: every variant within the oracle's bound."""
    w = synth.make_config(3, shrink=8)
    X = synth.normal_matrix(w.n, 36, seed=77)
    Yref, B = oracle.spmm(*csr_of(w), X)
    Xd = torch.from_numpy(X).cuda()
    op = binding.ArrowSpMM(*csr_of(w), w.b, options=binding.arrow_options_default(hubs_first=65536, chunk_nnz=100))
    assert_within(op.spmm(Xd).cpu().numpy(), Yref, B)
    for kw in (dict(corner=1), dict(fuse_levels=0, short_max=4), dict(panel=1, window_rows=64),
               dict(classes=8, class_min=2, class_gran=16, kc=16), dict()):
        op.repack(binding.arrow_options_default(**kw))
        lv = op.levels()
        assert (lv[0]["nnz_corner"] > 0) == bool(kw.get("corner")) and (lv[0]["nnz_panel"] > 0) == bool(kw.get("panel"))
        Yd = torch.full_like(Xd, float("nan"))
        assert_within(op.spmm(Xd, Yd).cpu().numpy(), Yref, B)
    op.close()
