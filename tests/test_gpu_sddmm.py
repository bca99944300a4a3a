"""GPU parity of the sampled dense-dense product  S[p] = a_p <U[i, :], V[j, :]>  (nonzero p = (i, j)),
called through the C-ABI, against the fp64 CPU oracle on the same seeded inputs.
Bar (per stored entry): |S - Sref| <= 1e-5 * |a_p| <|U[i]|, |V[j]|>, exactly 0 where the bound is 0;
every element of S is written (the output starts as NaN)."""
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
        pytest.fail("no GPU visible: the parity tests need a real MI355X")
    if not os.path.exists(binding.LIB_PATH):
        pytest.fail("libarrow.so is not built")
    return torch


def assert_within(S, Sref, B):
    S = np.asarray(S, dtype=np.float64)
    assert not np.isnan(S).any(), f"{np.isnan(S).sum()} entries were never written"
    err = np.abs(S - Sref)
    lim = TOL * B
    bad = err > lim
    if bad.any():
        i = int(np.argmax(err - lim))
        raise AssertionError(f"{bad.sum()} of {bad.size} entries outside the bound; worst at {i}: "
                             f"got {S[i]!r} want {Sref[i]!r} bound {lim[i]!r}")
    assert np.all(S[B == 0] == 0)
    nz = B > 0
    if nz.any():
        assert np.median(err[nz] / B[nz]) < 1e-6


def run_sampled(torch, csr, b, U, V):
    op = binding.ArrowSpMM(*csr, b)
    Ud = torch.from_numpy(U).cuda()
    Vd = Ud if V is U else torch.from_numpy(V).cuda()
    Sd = torch.full((len(csr[2]),), float("nan"), dtype=torch.float32, device="cuda")
    op.sddmm(Ud, Vd, Sd)
    torch.cuda.synchronize()
    return op, Ud, Vd, Sd.cpu().numpy()


def csr_of(w):
    return (w.rowptr, w.colidx, w.vals)


def test_config0_rmat_s12_k16(torch):
    w = synth.make_config(0)
    U = synth.normal_matrix(w.n, w.k, seed=301)
    V = synth.normal_matrix(w.n, w.k, seed=302)
    op, Ud, Vd, S = run_sampled(torch, csr_of(w), w.b, U, V)
    Sref, B = oracle.sddmm(*csr_of(w), U, V)
    assert_within(S, Sref, B)
    S2 = op.sddmm(Ud, Vd).cpu().numpy()                    # bitwise reproducible run to run
    assert np.array_equal(S.view(np.uint32), S2.view(np.uint32))
    # U and V swapped is another product (the operand is not symmetric in its values)
    S3 = op.sddmm(Vd, Ud).cpu().numpy()
    Sref3, B3 = oracle.sddmm(*csr_of(w), V, U)
    assert_within(S3, Sref3, B3)
    assert not np.allclose(S3, S, atol=1e-3)
    # the product kernels still work on the same handle afterwards
    X = w.make_x()
    Y = op.spmm(torch.from_numpy(X).cuda()).cpu().numpy()
    Yref, By = oracle.spmm(*csr_of(w), X)
    assert np.all(np.abs(Y - Yref) <= TOL * By)
    op.close()


@pytest.mark.parametrize("k", [1, 2, 3, 4, 6, 7, 12, 16, 20, 33, 64, 100, 128, 130, 200, 256, 260, 516, 1030])
def test_all_column_counts(torch, k):
    w = synth.make_config(0, shrink=1)              # n = 2048, b = 256
    U = synth.normal_matrix(w.n, k, seed=400 + k)
    V = synth.normal_matrix(w.n, k, seed=500 + k)
    op, _, _, S = run_sampled(torch, csr_of(w), w.b, U, V)
    Sref, B = oracle.sddmm(*csr_of(w), U, V)
    assert_within(S, Sref, B)
    op.close()


@pytest.mark.parametrize("b", [1, 5, 64, 1000, 2048, 5000])
def test_block_widths(torch, b):
    w = synth.make_config(0, shrink=1)
    U = synth.normal_matrix(w.n, 24, seed=17)
    op, _, _, S = run_sampled(torch, csr_of(w), b, U, U)     # U == V: the same device buffer twice
    Sref, B = oracle.sddmm(*csr_of(w), U, U)
    assert_within(S, Sref, B)
    op.close()


@pytest.mark.parametrize("env", [
    dict(ARROW_SHORT_MAX="0", ARROW_CHUNK_NNZ="7"),
    dict(ARROW_SHORT_MAX="1000000"),
    dict(ARROW_STAGE_HEAD="0"),
    dict(ARROW_WINDOW_ROWS="0"),
    dict(ARROW_CLASSES="8", ARROW_CLASS_MIN="2", ARROW_CLASS_GRAN="16"),
    dict(ARROW_CLASSES="16", ARROW_CLASS_MIN="1", ARROW_CLASS_GRAN="1", ARROW_SHORT_MAX="0"),
    dict(ARROW_CLASSES="8", ARROW_CLASS_MIN="3", ARROW_PIECE_MAX="5", ARROW_SHORT_MAX="2"),
    dict(ARROW_SEPARATORS="0", ARROW_BFS_TAIL="0"),
])
@pytest.mark.parametrize("k", [16, 36, 128])
def test_pack_options(torch, monkeypatch, env, k):
    """Work lists of every kind: split rows, class pieces, die queues with padding, staged head."""
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    w = synth.make_config(0)
    U = synth.normal_matrix(w.n, k, seed=19 + k)
    V = synth.normal_matrix(w.n, k, seed=29 + k)
    op, _, _, S = run_sampled(torch, csr_of(w), w.b, U, V)
    Sref, B = oracle.sddmm(*csr_of(w), U, V)
    assert_within(S, Sref, B)
    op.close()


@pytest.mark.parametrize("k", [4, 7, 36, 130])
def test_window_rows(torch, monkeypatch, k):
    """Grid operator with the diagonal blocks packed as LDS-window tiles: their entries name
    positions inside the tile's window, which the sampled kernel translates through perm."""
    monkeypatch.setenv("ARROW_WINDOW_REUSE_X10", "20")
    w = synth.make_config(1, shrink=6)              # 128 x 128 grid
    U = synth.normal_matrix(w.n, k, seed=60 + k)
    V = synth.normal_matrix(w.n, k, seed=70 + k)
    op, _, _, S = run_sampled(torch, csr_of(w), 2048, U, V)
    lv = op.levels()
    assert lv[0]["window_tiles"] > 0 and lv[0]["nnz_window"] > 0.5 * w.nnz
    Sref, B = oracle.sddmm(*csr_of(w), U, V)
    assert_within(S, Sref, B)
    op.close()


@pytest.mark.parametrize("env", [
    dict(ARROW_WINDOW_ROWS="64"),
    dict(ARROW_WINDOW_ROWS="32", ARROW_PANEL_MIN="1", ARROW_SHORT_MAX="0"),
])
@pytest.mark.parametrize("k", [1, 3, 16, 36, 128, 260, 1030])
def test_head_panels(torch, monkeypatch, env, k):
    """Entries that the product runs in head panels: their row is found through the panel table."""
    monkeypatch.setenv("ARROW_PANEL", "1")
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    w = synth.make_config(0)
    U = synth.normal_matrix(w.n, k, seed=81 + k)
    V = synth.normal_matrix(w.n, k, seed=82 + k)
    op, _, _, S = run_sampled(torch, csr_of(w), w.b, U, V)
    assert op.levels()[0]["nnz_panel"] > 0
    Sref, B = oracle.sddmm(*csr_of(w), U, V)
    assert_within(S, Sref, B)
    op.close()


@pytest.mark.parametrize("env", [
    dict(ARROW_HUBS_FIRST="65536"),
    dict(ARROW_HUBS_FIRST="100", ARROW_CORNER_MAX="256", ARROW_CORNER_MIN_TILE="1", ARROW_FUSE_LEVELS="0"),
])
@pytest.mark.parametrize("k", [1, 3, 16, 36, 128, 260, 1030])
def test_dense_corner(torch, monkeypatch, env, k):
    """Entries that the product runs in the LDS tiles of the dense corner: their row is found
    through the corner row table, their V row is a staged head row of the tile's column range."""
    monkeypatch.setenv("ARROW_CORNER", "1")
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    w = synth.make_config(0)
    U = synth.normal_matrix(w.n, k, seed=91 + k)
    V = synth.normal_matrix(w.n, k, seed=92 + k)
    op, _, _, S = run_sampled(torch, csr_of(w), w.b, U, V)
    assert op.levels()[0]["nnz_corner"] > 0
    Sref, B = oracle.sddmm(*csr_of(w), U, V)
    assert_within(S, Sref, B)
    op.close()


@pytest.mark.parametrize("env", [dict(), dict(ARROW_PANEL="1", ARROW_WINDOW_ROWS="64"),
                                 dict(ARROW_CORNER="1", ARROW_HUBS_FIRST="65536")])
def test_image_order_output(torch, monkeypatch, env):
    """Option "sddmm_image_order": contiguous stores; the exported entry map brings S back to CSR order."""
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    w = synth.make_config(0)
    U = synth.normal_matrix(w.n, 36, seed=11)
    V = synth.normal_matrix(w.n, 36, seed=12)
    op, Ud, Vd, S = run_sampled(torch, csr_of(w), w.b, U, V)
    binding.arrow_set_option(op.h, "sddmm_image_order", 1)
    Simg = op.sddmm(Ud, Vd, torch.full((w.nnz,), float("nan"), device="cuda")).cpu().numpy()
    emap = binding.arrow_export_entry_map(op.h)
    back = np.empty_like(Simg)
    back[emap] = Simg
    assert np.array_equal(back.view(np.uint32), S.view(np.uint32))
    binding.arrow_set_option(op.h, "sddmm_image_order", 0)
    S2 = op.sddmm(Ud, Vd).cpu().numpy()
    assert np.array_equal(S2.view(np.uint32), S.view(np.uint32))
    op.close()


def test_several_levels_and_hub_row(torch):
    # a hub adjacent to everything plus a sparse random remainder: long split row, several levels
    rng = np.random.default_rng(33)
    n, b, k = 5000, 64, 40
    far = rng.integers(0, n, (20000, 2))
    rows = np.concatenate([far[:, 0], far[:, 1], np.zeros(n, np.int64), np.arange(n)])
    cols = np.concatenate([far[:, 1], far[:, 0], np.arange(n), np.zeros(n, np.int64)])
    key = np.unique(rows.astype(np.int64) * n + cols)
    rows, cols = key // n, key % n
    rowptr = np.zeros(n + 1, np.int64)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr)
    colidx = cols.astype(np.int32)
    vals = synth.fill_uniform(rowptr, colidx, seed=34)
    U = synth.normal_matrix(n, k, seed=35)
    V = synth.normal_matrix(n, k, seed=36)
    op, _, _, S = run_sampled(torch, (rowptr, colidx, vals), b, U, V)
    assert op.info["levels"] >= 2
    Sref, B = oracle.sddmm(rowptr, colidx, vals, U, V)
    assert_within(S, Sref, B)
    op.close()


def test_special_operands_bitwise(torch):
    w = synth.make_config(0, shrink=1)
    n, k = w.n, 8
    ones = np.ones((n, k), np.float32)
    op, _, _, S = run_sampled(torch, csr_of(w), w.b, ones, ones)
    assert np.array_equal(S, (k * w.vals.astype(np.float64)).astype(np.float32))   # k * a exactly
    U = synth.normal_matrix(n, k, seed=3)
    E = np.zeros((n, k), np.float32); E[:, 5] = 1
    S2 = op.sddmm(torch.from_numpy(U).cuda(), torch.from_numpy(E).cuda()).cpu().numpy()
    rows = np.repeat(np.arange(n), np.diff(w.rowptr))
    assert np.array_equal(S2, w.vals * U[rows, 5])                                    # one product each
    Z = np.zeros((n, k), np.float32)
    S3 = op.sddmm(torch.from_numpy(U).cuda(), torch.from_numpy(Z).cuda()).cpu().numpy()
    assert np.all(S3 == 0)
    op.close()


def test_row_sums_match_the_product_kernels(torch):
    """sum_j S(i, j) = <U[i], (A V)[i]>: the sampled product against arrow_spmm on the same handle."""
    w = synth.make_config(3, shrink=9)              # R-MAT scale 14, k = 128
    U = synth.normal_matrix(w.n, w.k, seed=91)
    V = synth.normal_matrix(w.n, w.k, seed=92)
    op, Ud, Vd, S = run_sampled(torch, csr_of(w), w.b, U, V)
    Sref, B = oracle.sddmm(*csr_of(w), U, V)
    assert_within(S, Sref, B)
    Y = op.spmm(Vd).cpu().numpy().astype(np.float64)
    lhs = np.zeros(w.n)
    np.add.at(lhs, np.repeat(np.arange(w.n), np.diff(w.rowptr)), S.astype(np.float64))
    rhs = np.sum(U.astype(np.float64) * Y, axis=1)
    scale = np.zeros(w.n)
    np.add.at(scale, np.repeat(np.arange(w.n), np.diff(w.rowptr)), B)
    assert np.all(np.abs(lhs - rhs) <= 2e-5 * scale + 1e-30)
    op.close()


def test_loaded_handle(torch, tmp_path):
    w = synth.make_config(0)
    h = binding.arrow_decompose(*csr_of(w), w.b)
    path = str(tmp_path / "levels.bin")
    binding.arrow_save(h, path)
    binding.arrow_destroy(h)
    op = binding.ArrowSpMM(handle=binding.arrow_load(path))
    U = synth.normal_matrix(w.n, 20, seed=44)
    V = synth.normal_matrix(w.n, 20, seed=45)
    S = op.sddmm(torch.from_numpy(U).cuda(), torch.from_numpy(V).cuda()).cpu().numpy()
    Sref, B = oracle.sddmm(*csr_of(w), U, V)
    assert_within(S, Sref, B)
    op.close()


def test_errors(torch):
    w = synth.make_config(0, shrink=2)
    op = binding.ArrowSpMM(*csr_of(w), w.b)
    U = torch.zeros((w.n, 8), device="cuda")
    S = torch.zeros(w.nnz, device="cuda")
    op._ensure_workspace(8)
    with pytest.raises(binding.ArrowError) as e:        # no entry map yet
        binding.arrow_sddmm(op.h, U.data_ptr(), U.data_ptr(), S.data_ptr(), 8, 0)
    assert e.value.code == binding.ARROW_ENOTREADY
    buf = torch.empty(binding.arrow_sddmm_device_bytes(op.h), dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.ArrowError) as e:
        binding.arrow_sddmm_upload(op.h, buf.data_ptr(), 16, 0)
    assert e.value.code == binding.ARROW_ETOOSMALL
    with pytest.raises(binding.ArrowError):
        binding.arrow_sddmm_upload(op.h, buf.data_ptr() + 4, buf.numel(), 0)
    binding.arrow_sddmm_upload(op.h, buf.data_ptr(), buf.numel(), 0)
    with pytest.raises(binding.ArrowError):
        binding.arrow_sddmm(op.h, 0, U.data_ptr(), S.data_ptr(), 8, 0)
    with pytest.raises(binding.ArrowError):
        binding.arrow_sddmm(op.h, U.data_ptr(), U.data_ptr(), S.data_ptr(), 0, 0)
    with pytest.raises(binding.ArrowError) as e:        # workspace sized for k = 8
        binding.arrow_sddmm(op.h, U.data_ptr(), U.data_ptr(), S.data_ptr(), 4096, 0)
    assert e.value.code == binding.ARROW_ETOOSMALL
    op.close()
