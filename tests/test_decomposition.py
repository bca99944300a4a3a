"""Host-side checks of ``arrow_decompose`` (no GPU): the exported levels must reassemble A bit
for bit, every level must have arrow shape of width b, and the slow fp64 evaluation of
``sum_i P_i^T B_i P_i X`` over the exported levels must equal the CSR product of A."""
import os

import numpy as np
import pytest

import oracle
from oracle import arrow_checks
from paper_2307_05740_amd import _build, binding, synth


@pytest.fixture(scope="module", autouse=True)
def _lib_built():
    if not os.path.exists(_build.ARROW_LIB):
        _build.build_arrow()


def decompose_and_export(rowptr, colidx, vals, b):
    h = binding.arrow_decompose(rowptr, colidx, vals, b)
    try:
        binding.arrow_self_check(h)                      # the packed device image matches the levels
        info = binding.arrow_info(h)
        levels = [binding.arrow_export_level(h, i) for i in range(info["levels"])]
        linfo = [binding.arrow_level_info(h, i) for i in range(info["levels"])]
    finally:
        binding.arrow_destroy(h)
    return info, linfo, levels


def full_check(rowptr, colidx, vals, b, X=None):
    n = rowptr.shape[0] - 1
    info, linfo, levels = decompose_and_export(rowptr, colidx, vals, b)
    assert info["n"] == n and info["nnz"] == rowptr[-1] and info["b"] == b
    arrow_checks.check_decomposition(n, rowptr, colidx, vals, b, levels)
    assert len(levels[0][0]) == n                       # perm_0 is a full permutation
    for (perm, r, c, v), li in zip(levels, linfo):
        assert li["n_i"] == len(perm) and li["nnz"] == len(v)
        assert li["nnz_head_head"] + li["nnz_head_row"] + li["nnz_head_col"] + li["nnz_diag"] == li["nnz"]
        assert li["nnz_head_head"] == np.count_nonzero((r < b) & (c < b))
        assert li["nnz_diag"] == np.count_nonzero((r >= b) & (c >= b))
        key = r.astype(np.int64) * max(len(perm), 1) + c
        assert np.all(np.diff(key) > 0)                 # rows ascending, columns ascending in a row
    assert sum(li["nnz"] for li in linfo) == rowptr[-1]
    if X is not None:
        Y, B = oracle.spmm(rowptr, colidx, vals, X)
        Ya = arrow_checks.arrow_product(n, levels, X)
        assert np.all(np.abs(Ya - Y) <= 1e-12 * B + 1e-300)
    return info, linfo, levels


def csr_from_coo(n, rows, cols, vals):
    order = np.lexsort((cols, rows))
    rows, cols, vals = rows[order], cols[order], vals[order]
    rowptr = np.zeros(n + 1, np.int64)
    np.add.at(rowptr, rows + 1, 1)
    return np.cumsum(rowptr), cols.astype(np.int32), vals.astype(np.float32)


def test_config0_rmat():
    w = synth.make_config(0)
    info, linfo, _ = full_check(w.rowptr, w.colidx, w.vals, w.b, w.make_x())
    assert 1 <= info["levels"] <= 8                      # never more than ceil(n / b) levels
    assert linfo[0]["nnz"] > 0.8 * w.nnz                 # hubs in the head capture most entries
    assert linfo[0]["blocks"] == 8


@pytest.mark.parametrize("b", [1, 3, 64, 100, 4096, 10000])
def test_block_widths_including_degenerate(b):
    w = synth.make_config(0, shrink=2)                   # n = 1024
    info, linfo, levels = full_check(w.rowptr, w.colidx, w.vals, b, w.make_x())
    if b >= w.n:
        assert info["levels"] == 1 and linfo[0]["nnz"] == w.nnz


def test_grid_gives_one_arrow_matrix_with_separators():
    w = synth.make_config(1, shrink=8)                   # 64 x 64 grid; b = 1024 = 16 grid rows,
    info, linfo, _ = full_check(w.rowptr, w.colidx, w.vals, 1024, w.make_x())   # 3 separators fit
    assert info["levels"] == 1 and linfo[0]["separator_rule"] == 1
    assert linfo[0]["nnz_diag"] > 0.5 * w.nnz            # the stencil lives in the diagonal blocks


def test_grid_plain_rule_needs_second_level(monkeypatch):
    monkeypatch.setenv("ARROW_SEPARATORS", "0")
    w = synth.make_config(1, shrink=8)
    info, linfo, _ = full_check(w.rowptr, w.colidx, w.vals, 1024, w.make_x())
    assert info["levels"] >= 2 and linfo[0]["separator_rule"] == 0


def test_row_normalized_rmat_and_chung_lu_small():
    for idx, shrink in ((2, 8), (4, 10)):
        w = synth.make_config(idx, shrink=shrink)
        info, linfo, _ = full_check(w.rowptr, w.colidx, w.vals, w.b, w.make_x()[:, :4].copy())
        assert info["levels"] <= (w.n + w.b - 1) // w.b + 1


def test_star_plus_short_paths_is_one_level():
    # one hub joined to everything, plus disjoint paths shorter than b
    n, b = 257, 16
    rows, cols = [], []
    for v in range(1, n):
        rows += [0, v]; cols += [v, 0]
    for start in range(1, n - 8, 8):
        for v in range(start, start + 7):
            rows += [v, v + 1]; cols += [v + 1, v]
    rng = np.random.default_rng(0)
    rp, ci, va = csr_from_coo(n, np.array(rows), np.array(cols), rng.uniform(-1, 1, len(rows)))
    info, _, _ = full_check(rp, ci, va, b, rng.standard_normal((n, 3)).astype(np.float32))
    assert info["levels"] == 1


def test_block_diagonal_is_one_level_without_arrow_strips():
    n, b = 96, 8
    rng = np.random.default_rng(1)
    rows, cols = [], []
    for blk in range(n // b):
        for i in range(b):
            for j in range(b):
                if rng.random() < 0.5 or i == j:
                    rows.append(blk * b + i); cols.append(blk * b + j)
    rp, ci, va = csr_from_coo(n, np.array(rows), np.array(cols), rng.uniform(-1, 1, len(rows)))
    info, linfo, _ = full_check(rp, ci, va, b, rng.standard_normal((n, 2)).astype(np.float32))
    assert info["levels"] == 1


def test_single_crossing_entry_needs_two_levels_with_plain_rule(monkeypatch):
    monkeypatch.setenv("ARROW_SEPARATORS", "0")
    # a cycle-free chain of equal-degree vertices in two far-apart blocks plus one crossing pair
    n, b = 64, 8
    rows = list(range(n)); cols = list(range(n))          # diagonal only: all degrees 0
    rows += [20, 50]; cols += [50, 20]                    # crossing entries between blocks 2 and 6
    rows += [3, 4]; cols += [4, 3]                        # a pair with the same degree but lower ids
    rp, ci, va = csr_from_coo(n, np.array(rows), np.array(cols), np.arange(1, len(rows) + 1, dtype=np.float64))
    info, linfo, levels = full_check(rp, ci, va, b, np.eye(n, dtype=np.float32)[:, :5].copy())
    assert info["levels"] == 1    # degree-1 vertices sort ahead of degree-0 ones, so they are in the head
    # now make the head too small to take them all: b = 2 and three disjoint far pairs
    rows = list(range(n)); cols = list(range(n))
    for u, v in ((10, 40), (20, 50), (30, 60)):
        rows += [u, v]; cols += [v, u]
    rp, ci, va = csr_from_coo(n, np.array(rows), np.array(cols), np.arange(1, len(rows) + 1, dtype=np.float64))
    info, _, _ = full_check(rp, ci, va, 2, np.eye(n, dtype=np.float32)[:, :5].copy())
    assert info["levels"] == 1    # the traversal arrangement puts the partners next to each other
    monkeypatch.setenv("ARROW_BFS_TAIL", "0")            # id order keeps them in different blocks
    info, _, _ = full_check(rp, ci, va, 2, np.eye(n, dtype=np.float32)[:, :5].copy())
    assert info["levels"] == 2


def test_nonsymmetric_operand():
    rng = np.random.default_rng(4)
    n = 200
    M = rng.random((n, n)) < 0.03
    r, c = np.nonzero(M)
    rp, ci, va = csr_from_coo(n, r, c, rng.uniform(-1, 1, len(r)))
    full_check(rp, ci, va, 16, rng.standard_normal((n, 3)).astype(np.float32))
    full_check(rp, ci, va, 7, rng.standard_normal((n, 3)).astype(np.float32))


def _directed(n, rows, cols, seed=11):
    rng = np.random.default_rng(seed)
    rp, ci, va = csr_from_coo(n, np.asarray(rows), np.asarray(cols), rng.uniform(-1, 1, len(rows)))
    return rp, ci, va, rng.standard_normal((n, 3)).astype(np.float32)


@pytest.mark.parametrize("n,b,off,cnt", [(4096, 64, 2048, 2048 - 64), (64, 4, 32, 28),
                                         (4096, 64, 100, 4096 - 300)])
@pytest.mark.parametrize("lower", [False, True])
def test_directed_shift_operands(n, b, off, cnt, lower):
    """Entries (i, i + off) only -- strictly upper (or, mirrored, strictly lower) triangular, every
    vertex with one entry in its row or one in its column but seldom both.  Adjacency has to be
    taken from the pattern of A + A^T: a rule that follows rows alone finds nothing to do for the
    column ends.  Both orientations must decompose, into the same small number of levels."""
    i = np.arange(cnt)
    r, c = (i + off, i) if lower else (i, i + off)
    rp, ci, va, X = _directed(n, r, c)
    info, linfo, _ = full_check(rp, ci, va, b, X)
    assert info["levels"] <= 2
    assert linfo[0]["nnz"] >= 0.9 * cnt


def test_directed_strictly_triangular_random_and_long_cycle():
    rng = np.random.default_rng(8)
    n = 600
    M = np.triu(rng.random((n, n)) < 0.01, k=1)
    r, c = np.nonzero(M)
    for b in (8, 50):
        rp, ci, va, X = _directed(n, r, c)
        info, _, _ = full_check(rp, ci, va, b, X)
        rp, ci, va, X = _directed(n, c, r)                   # the transposed operand
        info_t, _, _ = full_check(rp, ci, va, b, X)
        assert info["levels"] == info_t["levels"]           # the rules only see A + A^T
    # one directed cycle through all vertices in a scrambled order, much longer than b
    n, b = 1000, 16
    order = rng.permutation(n)
    rp, ci, va, X = _directed(n, order, np.roll(order, -1))
    info, linfo, _ = full_check(rp, ci, va, b, X)
    assert info["levels"] <= 3 and linfo[0]["nnz"] >= 0.9 * n


def test_random_directed_operands_always_decompose():
    rng = np.random.default_rng(2024)
    for trial in range(60):
        n = int(rng.integers(2, 300))
        b = int(rng.integers(1, 40))
        m = int(rng.integers(0, 4 * n))
        r = rng.integers(0, n, m)
        c = rng.integers(0, n, m)
        if trial % 3 == 0:
            r, c = np.minimum(r, c), np.maximum(r, c)         # upper triangular with diagonal
        key = np.unique(r * n + c)
        rp, ci, va, X = _directed(n, key // n, key % n, seed=trial)
        info, _, _ = full_check(rp, ci, va, b, X)
        assert info["levels"] <= 4 * ((n + b - 1) // b) + 64


# --- the invariant checkers themselves: each must reject a violating level -------------------

def _valid_small_level():
    """n = 6, b = 2, one level holding the whole of a small matrix: positions are a rotation of
    the vertex ids; entries sit in the head row, the head column and the diagonal blocks."""
    n, b = 6, 2
    perm = np.array([4, 5, 0, 1, 2, 3], np.int32)
    r = np.array([0, 0, 1, 2, 3, 3, 4, 5, 5], np.int32)     # positions
    c = np.array([0, 5, 3, 3, 2, 0, 5, 4, 1], np.int32)
    v = np.arange(1, 10, dtype=np.float32) / 8
    rows, cols = perm[r], perm[c]
    rp, ci, va = csr_from_coo(n, rows.astype(np.int64), cols.astype(np.int64), v.astype(np.float64))
    return n, b, rp, ci, va, (perm, r, c, v)


def test_checkers_accept_a_valid_hand_made_level():
    n, b, rp, ci, va, lev = _valid_small_level()
    arrow_checks.check_decomposition(n, rp, ci, va, b, [lev])


def test_check_arrow_shape_rejects_an_entry_outside_the_arrow():
    n, b, rp, ci, va, (perm, r, c, v) = _valid_small_level()
    r2, c2 = r.copy(), c.copy()
    r2[3], c2[3] = 2, 4                                      # blocks 1 and 2, neither in the head
    with pytest.raises(AssertionError, match="outside the arrow"):
        arrow_checks.check_arrow_shape(r2, c2, b, len(perm))
    arrow_checks.check_arrow_shape(r2, c2, 3, len(perm))     # 2 // 3 = 0: first block row at b = 3
    c3 = c.copy()
    c3[0] = len(perm)                                        # a position outside the level
    with pytest.raises(AssertionError, match="outside the level"):
        arrow_checks.check_arrow_shape(r, c3, b, len(perm))
    with pytest.raises(AssertionError):                      # ... and through the front door
        arrow_checks.check_decomposition(n, rp, ci, va, b, [(perm, r2, c2, v)])


def test_check_perm_injective_rejects_duplicates_and_out_of_range():
    n, b, rp, ci, va, (perm, r, c, v) = _valid_small_level()
    dup = perm.copy()
    dup[5] = dup[0]
    with pytest.raises(AssertionError, match="injective"):
        arrow_checks.check_perm_injective(dup, n)
    far = perm.copy()
    far[2] = n
    with pytest.raises(AssertionError, match="out of range"):
        arrow_checks.check_perm_injective(far, n)
    neg = perm.copy()
    neg[2] = -1
    with pytest.raises(AssertionError, match="out of range"):
        arrow_checks.check_perm_injective(neg, n)
    with pytest.raises(AssertionError):
        arrow_checks.check_decomposition(n, rp, ci, va, b, [(dup, r, c, v)])


def test_check_reassembly_rejects_flipped_bits_dropped_moved_and_split_entries():
    n, b, rp, ci, va, (perm, r, c, v) = _valid_small_level()
    flipped = v.copy()
    flipped.view(np.uint32)[4] ^= 1                           # one mantissa bit
    with pytest.raises(AssertionError, match="value bits"):
        arrow_checks.check_reassembly(n, rp, ci, va, [(perm, r, c, flipped)])
    negz = v.copy()
    with pytest.raises(AssertionError, match="entry count"):  # a dropped entry
        arrow_checks.check_reassembly(n, rp, ci, va, [(perm, r[:-1], c[:-1], v[:-1])])
    moved = c.copy()
    moved[6] = 4                                              # same count, other coordinate
    with pytest.raises(AssertionError, match="coordinates"):
        arrow_checks.check_reassembly(n, rp, ci, va, [(perm, r, moved, v)])
    # an entry split into two halves in two levels sums to A but is not a reassembly
    half = v.copy()
    half[2] /= 2
    second = (perm, r[2:3], c[2:3], half[2:3])
    with pytest.raises(AssertionError):
        arrow_checks.check_reassembly(n, rp, ci, va, [(perm, r, c, half), second])
    # the same entry in two levels
    with pytest.raises(AssertionError, match="entry count"):
        arrow_checks.check_reassembly(n, rp, ci, va, [(perm, r, c, v), (perm, r[:1], c[:1], v[:1])])
    # signed zero is a different bit pattern
    rp0, ci0, va0 = csr_from_coo(2, np.array([0]), np.array([1]), np.array([0.0]))
    lev = (np.array([0, 1], np.int32), np.array([0], np.int32), np.array([1], np.int32),
           np.array([-0.0], np.float32))
    with pytest.raises(AssertionError, match="value bits"):
        arrow_checks.check_reassembly(2, rp0, ci0, va0, [lev])
    del negz


def test_empty_matrix_and_explicit_zeros():
    n = 10
    rp = np.zeros(n + 1, np.int64)
    info, linfo, levels = full_check(rp, np.zeros(0, np.int32), np.zeros(0, np.float32), 4,
                                     np.ones((n, 2), np.float32))
    assert info["levels"] == 1 and linfo[0]["nnz"] == 0
    rp, ci, va = csr_from_coo(3, np.array([0, 1, 2]), np.array([2, 1, 0]), np.array([0.0, -0.0, 1.0]))
    full_check(rp, ci, va, 1, np.ones((3, 1), np.float32))       # signed zeros survive bit-exactly


def test_error_paths():
    w = synth.make_config(0, shrink=4)
    bad = [
        dict(b=0), dict(n=0), dict(rowptr=w.rowptr[::-1].copy()),
        dict(colidx=np.where(np.arange(w.nnz) == 5, w.n, w.colidx).astype(np.int32)),
        dict(colidx=np.where(np.arange(w.nnz) == 1, w.colidx[0], w.colidx).astype(np.int32)),
    ]
    for kw in bad:
        args = dict(rowptr=w.rowptr, colidx=w.colidx, vals=w.vals, b=8)
        args.update(kw)
        with pytest.raises(binding.ArrowError) as ei:
            binding.arrow_decompose(**args)
        assert ei.value.code == binding.ARROW_EINVAL and binding.arrow_last_error()
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, 8)
    try:
        # compute calls before upload / workspace are refused on the host, no GPU involved
        with pytest.raises(binding.ArrowError) as ei:
            binding.arrow_spmm(h, 4096, 8192, 4)
        assert ei.value.code == binding.ARROW_ENOTREADY
        with pytest.raises(binding.ArrowError) as ei:
            binding.arrow_spmm(h, 4096, 8192, 0)
        assert ei.value.code == binding.ARROW_EINVAL
        with pytest.raises(binding.ArrowError) as ei:
            binding.arrow_spmm_iter(h, 4096, 4, -1)
        assert ei.value.code == binding.ARROW_EINVAL
        with pytest.raises(binding.ArrowError):
            binding.arrow_level_info(h, 99)
        with pytest.raises(binding.ArrowError):
            binding.arrow_set_option(h, "no_such_option", 1)
        with pytest.raises(binding.ArrowError) as ei:
            binding.arrow_upload(h, 4096, 1, 0)
        assert ei.value.code == binding.ARROW_ETOOSMALL
        assert binding.arrow_device_bytes(h) > 0 and binding.arrow_workspace_bytes(h, 4) > 0
    finally:
        binding.arrow_destroy(h)
    binding.arrow_destroy(None)                          # NULL is ignored


@pytest.mark.parametrize("env", [
    dict(ARROW_CLASSES="16", ARROW_CLASS_MIN="2", ARROW_CLASS_GRAN="16"),
    dict(ARROW_CLASSES="8", ARROW_CLASS_MIN="1", ARROW_PIECE_MAX="0", ARROW_SHORT_MAX="0"),
    dict(ARROW_CLASSES="24", ARROW_CLASS_MIN="3", ARROW_PIECE_MAX="1000", ARROW_STAGE_HEAD="0"),
    dict(ARROW_WINDOW_ROWS="0", ARROW_CHUNK_NNZ="7", ARROW_SHORT_MAX="3"),
    dict(ARROW_WINDOW_ROWS="64", ARROW_CHUNK_MIN="5", ARROW_CHUNK_NNZ="40"),
    dict(ARROW_WINDOW_SPAN="0"), dict(ARROW_WINDOW_SPAN="4096", ARROW_WINDOW_REUSE_X10="1"),
    dict(ARROW_WINDOW_REUSE_X10="20", ARROW_WINDOW_SHARE_X1000="0"),
    dict(ARROW_PANEL="1", ARROW_WINDOW_ROWS="32", ARROW_PANEL_MIN="1", ARROW_SHORT_MAX="0"),
    dict(ARROW_PANEL="1", ARROW_WINDOW_ROWS="128", ARROW_CHUNK_MIN="16", ARROW_HEAD_BY_ID="0"),
    dict(ARROW_WINDOW_ROWS="64", ARROW_HEAD_BY_ID="0"),
    dict(ARROW_STAGE_SHORT="1"), dict(ARROW_STAGE_SHORT="0", ARROW_EMPTY_LAST="0"),
    dict(ARROW_STAGE_SHORT="1", ARROW_EMPTY_LAST="1", ARROW_SHORT_MAX="64", ARROW_CLASSES="8", ARROW_CLASS_MIN="2"),
    dict(ARROW_CORNER="1"), dict(ARROW_CORNER="1", ARROW_HUBS_FIRST="65536", ARROW_CORNER_MIN_TILE="1"),
    dict(ARROW_CORNER="1", ARROW_HUBS_FIRST="300", ARROW_CORNER_MAX="256", ARROW_FUSE_LEVELS="0"),
    dict(ARROW_CORNER="1", ARROW_HUBS_FIRST="65536", ARROW_CORNER_MIN_TILE="4000", ARROW_SHORT_MAX="0"),
    dict(ARROW_FUSE_LEVELS="0"), dict(ARROW_FUSE_LEVELS="0", ARROW_WINDOW_ROWS="64", ARROW_CHUNK_NNZ="40"),
    dict(ARROW_FUSE_LEVELS="0", ARROW_PANEL="1", ARROW_WINDOW_ROWS="32", ARROW_PANEL_MIN="1"),
])
def test_packed_image_self_check_under_pack_options(monkeypatch, env):
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    for idx, shrink, b in ((0, 0, 512), (1, 8, 1024), (2, 8, None), (4, 10, None)):
        w = synth.make_config(idx, shrink=shrink)
        h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, b or w.b)
        try:
            binding.arrow_self_check(h)
        finally:
            binding.arrow_destroy(h)


@pytest.mark.parametrize("env", [dict(), dict(ARROW_PANEL="1", ARROW_WINDOW_ROWS="64"),
                                 dict(ARROW_CLASSES="8", ARROW_CLASS_MIN="2", ARROW_CLASS_GRAN="16")])
@pytest.mark.parametrize("fuse", ["0", "1"])
def test_entry_map_is_a_bijection_onto_the_nonzeros(monkeypatch, env, fuse):
    monkeypatch.setenv("ARROW_FUSE_LEVELS", fuse)
    for name, v in env.items():
        monkeypatch.setenv(name, v)
    w = synth.make_config(0)
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    try:
        binding.arrow_self_check(h)
        emap = binding.arrow_export_entry_map(h)
        assert emap.shape == (w.nnz,) and np.array_equal(np.sort(emap), np.arange(w.nnz, dtype=np.uint32))
        n_levels = binding.arrow_info(h)["levels"]
        assert n_levels >= 2
        fused = binding.arrow_level_info(h, 0)["nnz_fused"]
        if fuse == "1":
            # one image level holds every entry: the later levels' entries sit with the level-0 rows
            assert fused == sum(binding.arrow_level_info(h, i)["nnz"] for i in range(1, n_levels))
            return
        assert fused == 0
        # level by level the map's image is that level's set of nonzeros (as (row, column, value))
        at = 0
        csr_row = np.repeat(np.arange(w.n), np.diff(w.rowptr))
        for i in range(n_levels):
            perm, r, c, v = binding.arrow_export_level(h, i)
            src = np.sort(emap[at:at + len(v)])
            at += len(v)
            want = np.lexsort((perm[c], perm[r]))
            got = np.lexsort((w.colidx[src], csr_row[src]))
            assert np.array_equal(csr_row[src][got], perm[r][want])
            assert np.array_equal(w.colidx[src][got], perm[c][want])
            assert np.array_equal(w.vals[src][got].view(np.uint32), v[want].view(np.uint32))
        assert at == w.nnz
    finally:
        binding.arrow_destroy(h)


def _banded_with_far_entries(n=6000, seed=12):
    rng = np.random.default_rng(seed)
    rows, cols = [], []
    for d in (-3, -2, -1, 0, 1, 2, 3):
        i = np.arange(max(0, -d), min(n, n - d))
        rows.append(i); cols.append(i + d)
    far = rng.integers(0, n, (3000, 2))
    rows += [far[:, 0], far[:, 1]]; cols += [far[:, 1], far[:, 0]]
    rows = np.concatenate(rows); cols = np.concatenate(cols)
    key = np.unique(rows.astype(np.int64) * n + cols)
    return csr_from_coo(n, key // n, key % n, rng.uniform(-1, 1, len(key)))


@pytest.mark.parametrize("fuse", ["0", "1"])
def test_fused_levels_keep_the_decomposition_and_cover_every_entry(monkeypatch, fuse):
    """The levels a handle exports do not depend on how the image executes them; with fused levels
    the level-0 work lists hold every entry and the later levels hold none.  The operand (a band
    cut at block boundaries plus far entries, separator rule off) has several levels, and LDS-window
    tiles whose rows also carry entries of other blocks once the levels are fused."""
    monkeypatch.setenv("ARROW_SEPARATORS", "0")
    monkeypatch.setenv("ARROW_WINDOW_REUSE_X10", "5")
    monkeypatch.setenv("ARROW_WINDOW_SHARE_X1000", "0")
    monkeypatch.setenv("ARROW_FUSE_LEVELS", fuse)
    rp, ci, va = _banded_with_far_entries()
    n, b = len(rp) - 1, 500
    X = np.random.default_rng(5).standard_normal((n, 3)).astype(np.float32)
    info, linfo, levels = full_check(rp, ci, va, b, X)          # runs arrow_self_check as well
    assert info["levels"] >= 2
    total = sum(li["nnz"] for li in linfo)
    in_lists = [li["nnz_rows"] + li["nnz_chunks"] + li["nnz_window"] + li["nnz_panel"] + li["nnz_corner"] for li in linfo]
    if fuse == "1":
        assert in_lists[0] == total and all(x == 0 for x in in_lists[1:])
        assert linfo[0]["nnz_fused"] == total - linfo[0]["nnz"]
    else:
        assert in_lists == [li["nnz"] for li in linfo] and linfo[0]["nnz_fused"] == 0
    assert sum(li["window_tiles"] for li in linfo) > 0
    # the exported decomposition is the same either way
    monkeypatch.setenv("ARROW_FUSE_LEVELS", "1" if fuse == "0" else "0")
    _, _, other = decompose_and_export(rp, ci, va, b)
    assert len(other) == len(levels)
    for a, c in zip(levels, other):
        for x, y in zip(a, c):
            assert np.array_equal(x.view(np.uint32) if x.dtype == np.float32 else x,
                                  y.view(np.uint32) if y.dtype == np.float32 else y)


def test_dense_corner_takes_the_leading_entries_of_its_rows(monkeypatch):
    """With the hubs leading the head, rows and columns [0, S) of level 0 form the dense corner:
    S is a multiple of 256, the corner holds exactly the entries (p, q) with p, q < S, and the
    work lists hold the rest."""
    monkeypatch.setenv("ARROW_CORNER", "1")
    monkeypatch.setenv("ARROW_HUBS_FIRST", "65536")
    w = synth.make_config(3, shrink=8)                   # R-MAT scale 15, b = 1024
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    try:
        binding.arrow_self_check(h)
        li = binding.arrow_level_info(h, 0)
        S = li["corner"]
        assert S > 0 and S % 256 == 0 and S <= w.b
        perm, r, c, v = binding.arrow_export_level(h, 0)
        inside = np.count_nonzero((r < S) & (c < S))
        assert li["nnz_corner"] == inside and inside >= 0.02 * li["nnz"]
        assert 1 <= li["corner_items"] <= li["corner_tiles"] <= (S // 256) ** 2
        assert li["nnz_rows"] + li["nnz_chunks"] + li["nnz_window"] + li["nnz_corner"] == li["nnz"] + li["nnz_fused"]
        assert binding.arrow_level_info(h, 1)["corner"] == 0          # later levels stage no head
        with_corner = binding.arrow_workspace_bytes(h, 32)
    finally:
        binding.arrow_destroy(h)
    monkeypatch.setenv("ARROW_CORNER_MIN_TILE", "100000")             # no band of tiles is that dense
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    assert binding.arrow_level_info(h, 0)["corner"] == 0
    assert binding.arrow_workspace_bytes(h, 32) < with_corner         # the items' result rows are gone
    binding.arrow_destroy(h)


def test_long_rows_do_not_become_lds_window_rows():
    """Rows that spread over many blocks (most of their entries belong to later levels and join
    the level-0 row when levels are fused) are not run as LDS-window rows, whose entries outside
    the window are read by one lane group per row; rows that live in their diagonal block are."""
    rng = np.random.default_rng(3)
    n, b, per_row = 2048, 256, 512
    cols = np.sort(np.stack([rng.choice(n, per_row, replace=False) for _ in range(n)]), axis=1)
    rp = np.arange(n + 1, dtype=np.int64) * per_row
    h = binding.arrow_decompose(rp, cols.astype(np.int32).ravel(), rng.uniform(-1, 1, n * per_row).astype(np.float32), b)
    try:
        binding.arrow_self_check(h)
        li = binding.arrow_level_info(h, 0)
        assert li["nnz_window"] == 0 and li["nnz_fused"] > 0
        assert li["nnz_chunks"] + li["nnz_rows"] == n * per_row
    finally:
        binding.arrow_destroy(h)
    # block-diagonal operand with a few far entries per row: the rows still qualify
    rows = np.repeat(np.arange(n), 24)
    c = (rows // b) * b + rng.integers(0, b, rows.shape[0])
    far = rng.integers(0, n, (n, 2))
    key = np.unique(np.concatenate([rows * n + c, np.repeat(np.arange(n), 2) * n + far.ravel()]))
    rp, ci, va = csr_from_coo(n, key // n, key % n, rng.uniform(-1, 1, len(key)))
    h = binding.arrow_decompose(rp, ci, va, b)
    try:
        binding.arrow_self_check(h)
        li = binding.arrow_level_info(h, 0)
        assert li["window_tiles"] > 0 and li["nnz_window"] > 0.5 * len(key)
    finally:
        binding.arrow_destroy(h)


def test_head_order_inside_the_head(monkeypatch):
    """The arrow shape only fixes WHICH vertices are in the head; inside it they sit in id order
    (so that position order follows the caller's column order), or by falling degree on request.
    Both give the same head set and the same level sizes."""
    w = synth.make_config(0)
    deg = np.diff(w.rowptr) + np.bincount(w.colidx, minlength=w.n)
    deg -= 2 * np.array([np.any(w.colidx[w.rowptr[v]:w.rowptr[v + 1]] == v) for v in range(w.n)])
    monkeypatch.setenv("ARROW_HUBS_FIRST", "100")      # 100 hubs by falling degree, then id order
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    mixed = binding.arrow_export_level(h, 0)[0][:w.b]
    binding.arrow_destroy(h)
    assert np.all(np.diff(deg[mixed[:100]]) <= 0) and np.all(np.diff(mixed[100:]) > 0)
    assert deg[mixed[:100]].min() >= deg[mixed[100:]].max()
    monkeypatch.setenv("ARROW_HUBS_FIRST", "0")
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    head_id = binding.arrow_export_level(h, 0)[0][:w.b]
    nnz_id = [binding.arrow_level_info(h, i)["nnz"] for i in range(binding.arrow_info(h)["levels"])]
    binding.arrow_destroy(h)
    assert np.all(np.diff(head_id) > 0) and np.array_equal(np.sort(mixed), head_id)
    monkeypatch.setenv("ARROW_HEAD_BY_ID", "0")
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    head_deg = binding.arrow_export_level(h, 0)[0][:w.b]
    nnz_deg = [binding.arrow_level_info(h, i)["nnz"] for i in range(binding.arrow_info(h)["levels"])]
    binding.arrow_destroy(h)
    assert not np.all(np.diff(head_deg) > 0)
    assert np.array_equal(np.sort(head_deg), head_id) and nnz_id[0] == nnz_deg[0]


def test_head_panels_take_the_sparse_head_rows(monkeypatch):
    """With windows of 64 positions the head of width 512 spans 8 of them: head rows with fewer
    than chunk_min * 8 head-block entries hand those entries to panels, the rest stays in chunks."""
    monkeypatch.setenv("ARROW_WINDOW_ROWS", "64")
    monkeypatch.setenv("ARROW_PANEL", "1")
    w = synth.make_config(0)
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    try:
        binding.arrow_self_check(h)
        li = binding.arrow_level_info(h, 0)
        perm, r, c, v = binding.arrow_export_level(h, 0)
        hh = np.bincount(r[(r < w.b) & (c < w.b)], minlength=w.b)
        want = (hh >= 8) & (hh < 64 * 8)
        cap = 6 * (hh[want].sum() // np.count_nonzero(want)) + 1     # rows far above the mean stay in chunks
        if cap < 64 * 8:
            want = (hh >= 8) & (hh < cap)
        assert li["panel_rows"] == np.count_nonzero(want) and li["nnz_panel"] == hh[want].sum()
        assert li["panel_bins"] % 256 == 0 and li["panel_bins"] >= li["panel_rows"]   # 8 x 32 streams per 256 rows
        assert li["nnz_rows"] + li["nnz_chunks"] + li["nnz_window"] + li["nnz_panel"] + li["nnz_corner"] == li["nnz"] + li["nnz_fused"]
        assert binding.arrow_level_info(h, 1)["panel_rows"] == 0        # later levels stage no head
    finally:
        binding.arrow_destroy(h)
    monkeypatch.setenv("ARROW_PANEL", "0")
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    assert binding.arrow_level_info(h, 0)["panel_rows"] == 0
    binding.arrow_destroy(h)


def test_save_and_load_round_trip(tmp_path, monkeypatch):
    w = synth.make_config(2, shrink=8)
    h = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    path = str(tmp_path / "levels.arrow")
    binding.arrow_save(h, path)
    monkeypatch.setenv("ARROW_CHUNK_NNZ", "32")          # the image is rebuilt with the loader's choices
    g = binding.arrow_load(path)
    try:
        ia, ib = binding.arrow_info(h), binding.arrow_info(g)
        assert (ia["n"], ia["nnz"], ia["b"], ia["levels"]) == (ib["n"], ib["nnz"], ib["b"], ib["levels"])
        for i in range(ia["levels"]):
            for x, y in zip(binding.arrow_export_level(h, i), binding.arrow_export_level(g, i)):
                assert np.array_equal(x.view(np.uint32) if x.dtype == np.float32 else x,
                                      y.view(np.uint32) if y.dtype == np.float32 else y)
        binding.arrow_self_check(g)
        assert binding.arrow_level_info(g, 0)["chunks"] >= binding.arrow_level_info(h, 0)["chunks"]
    finally:
        binding.arrow_destroy(h)
        binding.arrow_destroy(g)
    # damaged files are refused, never half-loaded
    raw = open(path, "rb").read()
    bad = tmp_path / "bad.arrow"
    for blob in (raw[:len(raw) // 2], b"NOTARROW" + raw[8:], raw[:-8] + b"XXXXXXXX", b""):
        bad.write_bytes(blob)
        with pytest.raises(binding.ArrowError) as ei:
            binding.arrow_load(str(bad))
        assert ei.value.code == binding.ARROW_EINVAL
    # a column position outside the level fails the structural check
    levels_off = 8 + 4 + 8 + 8 + 4 + 4
    n_i = int(np.frombuffer(raw, np.int64, 1, levels_off)[0])
    lev_nnz = int(np.frombuffer(raw, np.int64, 1, levels_off + 8)[0])
    col_off = levels_off + 8 + 8 + 32 + 4 + 4 * n_i + 8 * (n_i + 1)
    cols = np.frombuffer(raw, np.int32, lev_nnz, col_off).copy()
    cols[-1] = n_i                                        # a column position outside the level
    blob = bytearray(raw)
    blob[col_off:col_off + 4 * lev_nnz] = cols.tobytes()
    bad.write_bytes(bytes(blob))
    with pytest.raises(binding.ArrowError):
        binding.arrow_load(str(bad))
    # two entries that claim the same nonzero of the caller's CSR
    src_off = col_off + 8 * lev_nnz
    src = np.frombuffer(raw, np.uint32, lev_nnz, src_off).copy()
    assert len(np.unique(src)) == lev_nnz and src.max() < w.nnz
    # the stored source indices name the right nonzeros: same value, same row and column vertex
    perm0 = np.frombuffer(raw, np.int32, n_i, levels_off + 8 + 8 + 32 + 4)
    rp0 = np.frombuffer(raw, np.int64, n_i + 1, levels_off + 8 + 8 + 32 + 4 + 4 * n_i)
    vals0 = np.frombuffer(raw, np.float32, lev_nnz, col_off + 4 * lev_nnz)
    cols0 = np.frombuffer(raw, np.int32, lev_nnz, col_off)
    assert np.array_equal(w.vals[src].view(np.uint32), vals0.view(np.uint32))
    assert np.array_equal(w.colidx[src], perm0[cols0])
    csr_row = np.repeat(np.arange(w.n), np.diff(w.rowptr))
    assert np.array_equal(csr_row[src], perm0[np.repeat(np.arange(n_i), np.diff(rp0))])
    src[0] = src[1]
    blob = bytearray(raw)
    blob[src_off:src_off + 4 * lev_nnz] = src.tobytes()
    bad.write_bytes(bytes(blob))
    with pytest.raises(binding.ArrowError) as ei:
        binding.arrow_load(str(bad))
    assert "bijection" in str(ei.value)
    with pytest.raises(binding.ArrowError):
        binding.arrow_load(str(tmp_path / "does_not_exist"))


def test_explicit_options_replace_the_environment(monkeypatch):
    """Options are an argument: the struct arrow_options_default() returns carries the built-in
    defaults plus ARROW_* overrides, and what a call receives is all that counts."""
    for name in list(os.environ):
        if name.startswith("ARROW_"):
            monkeypatch.delenv(name)
    d = binding.arrow_options_default()
    assert (d.separators, d.bfs_tail, d.head_by_id, d.hubs_first) == (1, 1, 1, 0)
    assert (d.short_max, d.chunk_nnz, d.chunk_min, d.window_rows, d.piece_max) == (16, 256, 64, 4096, 48)
    assert (d.fuse_levels, d.corner, d.panel, d.classes, d.kc) == (1, 0, 0, 0, 0)
    assert d.window_reuse == 8.0 and d.window_level_share == 0.05 and d.l2_resident_bytes == 2 << 20
    monkeypatch.setenv("ARROW_CHUNK_NNZ", "32")
    monkeypatch.setenv("ARROW_WINDOW_REUSE_X10", "25")
    e = binding.arrow_options_default(short_max=3)
    assert e.chunk_nnz == 32 and e.window_reuse == 2.5 and e.short_max == 3
    with pytest.raises(KeyError):
        binding.arrow_options_default(no_such_field=1)
    w = synth.make_config(0)
    # explicit options win over the environment; NULL options take the environment
    h_env = binding.arrow_decompose(w.rowptr, w.colidx, w.vals, w.b)
    h_opt = binding.arrow_decompose_with(w.rowptr, w.colidx, w.vals, w.b, d)
    h_sep = binding.arrow_decompose_with(w.rowptr, w.colidx, w.vals, w.b,
                                         binding.arrow_options_default(fuse_levels=0, chunk_nnz=256))
    try:
        for h in (h_env, h_opt, h_sep):
            binding.arrow_self_check(h)
        c_env, c_opt = (binding.arrow_level_info(h, 0)["chunks"] for h in (h_env, h_opt))
        assert c_env > c_opt                              # chunks of 32 against chunks of 256
        assert binding.arrow_level_info(h_opt, 0)["nnz_fused"] > 0
        assert binding.arrow_level_info(h_sep, 0)["nnz_fused"] == 0
        # repacking changes the image, not the levels
        before = [binding.arrow_export_level(h_opt, i) for i in range(binding.arrow_info(h_opt)["levels"])]
        binding.arrow_repack(h_opt, binding.arrow_options_default(chunk_nnz=64, fuse_levels=0, corner=1,
                                                                  corner_min_tile=1))
        binding.arrow_self_check(h_opt)
        li = binding.arrow_level_info(h_opt, 0)
        assert li["nnz_fused"] == 0 and li["nnz_corner"] > 0 and li["chunks"] != c_opt
        after = [binding.arrow_export_level(h_opt, i) for i in range(binding.arrow_info(h_opt)["levels"])]
        for a, c in zip(before, after):
            for x, y in zip(a, c):
                assert np.array_equal(x.view(np.uint32) if x.dtype == np.float32 else x,
                                      y.view(np.uint32) if y.dtype == np.float32 else y)
        with pytest.raises(binding.ArrowError) as ei:     # the old device image is no longer bound
            binding.arrow_spmm(h_opt, 4096, 1 << 20, 4)
        assert ei.value.code == binding.ARROW_ENOTREADY
    finally:
        for h in (h_env, h_opt, h_sep):
            binding.arrow_destroy(h)


def test_library_exports_every_declared_symbol():
    import glob
    import re
    declared = set()
    for path in glob.glob(os.path.join(_build.REPO_DIR, "include", "*.h")):
        declared |= set(re.findall(r"\b((?:arrow|csf3)_[a-z0-9_]+)\s*\(", open(path).read()))
    L = binding.lib()
    for name in sorted(declared):
        assert hasattr(L, name), f"{name} is declared in include/ but not exported"
    assert declared == set(binding.EXPORTED)
