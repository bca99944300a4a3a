"""Seeded synthetic inputs (ctypes binding of ``synth.c``).

Only input generation lives here: graph patterns, value fills, the dense
operand.  Both the test oracle's callers and the GPU library's callers take
their inputs from this module; it contains none of the method's arithmetic.

The five named workloads are reachable through :func:`make_config`.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsynth.so")
_lib = None

# base seeds: graph pattern, nonzero values, dense operand; the config index is added to each
SEED_GRAPH = 230705740
SEED_VALUES = SEED_GRAPH + 1000
SEED_X = SEED_GRAPH + 2000


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: run `python -m paper_2307_05740_amd._build synth`")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i64, i32, u64, dbl = (ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32,
                              ctypes.c_uint64, ctypes.c_double)
    lib.synth_rmat.restype = vp
    lib.synth_rmat.argtypes = [i32, i64, dbl, dbl, dbl, u64]
    lib.synth_chung_lu.restype = vp
    lib.synth_chung_lu.argtypes = [i64, dbl, dbl, dbl, u64]
    lib.synth_grid5.restype = vp
    lib.synth_grid5.argtypes = [i64]
    lib.synth_graph_free.restype = None
    lib.synth_graph_free.argtypes = [vp]
    lib.synth_graph_n.restype = i64
    lib.synth_graph_n.argtypes = [vp]
    lib.synth_graph_nnz.restype = i64
    lib.synth_graph_nnz.argtypes = [vp]
    lib.synth_graph_export.restype = ctypes.c_int
    lib.synth_graph_export.argtypes = [vp, vp, vp]
    lib.synth_fill_uniform.restype = ctypes.c_int
    lib.synth_fill_uniform.argtypes = [i64, vp, vp, u64, vp]
    lib.synth_fill_row_normalized.restype = ctypes.c_int
    lib.synth_fill_row_normalized.argtypes = [i64, vp, vp]
    lib.synth_fill_grid5.restype = ctypes.c_int
    lib.synth_fill_grid5.argtypes = [i64, vp, vp, vp]
    lib.synth_normal_matrix.restype = ctypes.c_int
    lib.synth_normal_matrix.argtypes = [i64, i32, u64, vp]
    lib.synth_num_threads.restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(a: np.ndarray) -> int:
    return a.ctypes.data


def _take(handle) -> tuple[np.ndarray, np.ndarray]:
    lib = _load()
    if not handle:
        raise RuntimeError("generator failed (bad arguments or out of memory)")
    try:
        n = lib.synth_graph_n(handle)
        nnz = lib.synth_graph_nnz(handle)
        rowptr = np.empty(n + 1, dtype=np.int64)
        colidx = np.empty(max(nnz, 0), dtype=np.int32)
        if lib.synth_graph_export(handle, _ptr(rowptr), _ptr(colidx)) != 0:
            raise RuntimeError("export failed")
    finally:
        lib.synth_graph_free(handle)
    return rowptr, colidx


def rmat_pattern(scale: int, samples: int, a: float = 0.57, b: float = 0.19, c: float = 0.19,
                 seed: int = SEED_GRAPH) -> tuple[np.ndarray, np.ndarray]:
    """Symmetrised R-MAT pattern on 2**scale vertices from ``samples`` directed samples."""
    return _take(_load().synth_rmat(scale, samples, a, b, c, seed))


def chung_lu_pattern(n: int, gamma: float = 2.1, avg_deg: float = 20.0, max_deg: float = 1e6,
                     seed: int = SEED_GRAPH) -> tuple[np.ndarray, np.ndarray]:
    """Symmetrised Chung-Lu pattern with power-law expected degrees."""
    return _take(_load().synth_chung_lu(n, gamma, avg_deg, max_deg, seed))


def grid5_pattern(N: int) -> tuple[np.ndarray, np.ndarray]:
    """Five-point stencil pattern of an N x N grid in natural order, no wrap-around."""
    return _take(_load().synth_grid5(N))


def fill_uniform(rowptr: np.ndarray, colidx: np.ndarray, seed: int = SEED_VALUES) -> np.ndarray:
    vals = np.empty(colidx.shape[0], dtype=np.float32)
    rc = _load().synth_fill_uniform(rowptr.shape[0] - 1, _ptr(rowptr), _ptr(colidx), seed, _ptr(vals))
    assert rc == 0
    return vals


def fill_row_normalized(rowptr: np.ndarray) -> np.ndarray:
    vals = np.empty(int(rowptr[-1]), dtype=np.float32)
    rc = _load().synth_fill_row_normalized(rowptr.shape[0] - 1, _ptr(rowptr), _ptr(vals))
    assert rc == 0
    return vals


def fill_grid5(rowptr: np.ndarray, colidx: np.ndarray) -> np.ndarray:
    vals = np.empty(colidx.shape[0], dtype=np.float32)
    rc = _load().synth_fill_grid5(rowptr.shape[0] - 1, _ptr(rowptr), _ptr(colidx), _ptr(vals))
    assert rc == 0
    return vals


def normal_matrix(n: int, k: int, seed: int = SEED_X, out: np.ndarray | None = None) -> np.ndarray:
    """n x k row-major fp32 matrix of independent standard normals."""
    X = out if out is not None else np.empty((n, k), dtype=np.float32)
    assert X.shape == (n, k) and X.dtype == np.float32 and X.flags.c_contiguous
    rc = _load().synth_normal_matrix(n, k, seed, _ptr(X))
    assert rc == 0
    return X


def num_threads() -> int:
    return int(_load().synth_num_threads())


@dataclass
class Workload:
    """One named configuration: CSR operand, dense-operand shape and product count."""
    name: str
    n: int
    rowptr: np.ndarray   # int64, n + 1
    colidx: np.ndarray   # int32, nnz
    vals: np.ndarray     # float32, nnz
    k: int
    b: int
    l: int               # number of chained products (1 = single product)
    seed_x: int

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])

    def make_x(self) -> np.ndarray:
        return normal_matrix(self.n, self.k, self.seed_x)


def make_config(index: int, shrink: int = 0) -> Workload:
    """Build workload ``index`` (0..4).

    ``shrink`` > 0 divides the vertex count by 2**shrink (R-MAT scale, grid side and
    Chung-Lu n shrink accordingly, the block width b shrinks with n, k is kept) so that
    tests can run the same recipe at a size the CPU checker finishes quickly.
    """
    s = int(shrink)
    if index == 0:
        scale = 12 - s
        rp, ci = rmat_pattern(scale, (1 << scale) * 16, seed=SEED_GRAPH + 0)
        return Workload(f"rmat_s{scale}_k16", 1 << scale, rp, ci,
                        fill_uniform(rp, ci, SEED_VALUES + 0), 16, max(512 >> s, 8), 1, SEED_X + 0)
    if index == 1:
        assert s % 2 == 0, "grid shrink must be even (side halves per two steps)"
        N = 1024 >> (s // 2)
        rp, ci = grid5_pattern(N)
        return Workload(f"grid5_{N}x{N}_k32", N * N, rp, ci, fill_grid5(rp, ci), 32,
                        max(65536 >> s, 8), 1, SEED_X + 1)
    if index == 2:
        scale = 20 - s
        rp, ci = rmat_pattern(scale, (1 << scale) * 8, seed=SEED_GRAPH + 2)
        return Workload(f"rmat_s{scale}_k64_pow3", 1 << scale, rp, ci, fill_row_normalized(rp),
                        64, max(65536 >> s, 8), 3, SEED_X + 2)
    if index == 3:
        scale = 23 - s
        rp, ci = rmat_pattern(scale, (1 << scale) * 16, seed=SEED_GRAPH + 3)
        return Workload(f"rmat_s{scale}_k128", 1 << scale, rp, ci,
                        fill_uniform(rp, ci, SEED_VALUES + 3), 128, max(262144 >> s, 8), 1,
                        SEED_X + 3)
    if index == 4:
        n = 16777216 >> s
        rp, ci = chung_lu_pattern(n, 2.1, 20.0, min(1e6, n / 4), seed=SEED_GRAPH + 4)
        return Workload(f"chunglu_n{n}_k32_pow5", n, rp, ci, fill_row_normalized(rp), 32,
                        max(262144 >> s, 8), 5, SEED_X + 4)
    raise ValueError("config index must be 0..4")


# ---------------------------------------------------------------------------------------------
# order-3 sparse tensors (inputs of the MTTKRP kernel); pure numpy, counter-based
# ---------------------------------------------------------------------------------------------
SEED_TENSOR = SEED_GRAPH + 3000


def _mix64(x: np.ndarray) -> np.ndarray:
    """splitmix64 finaliser on a uint64 array (wrap-around arithmetic)."""
    with np.errstate(over="ignore"):
        x = x + np.uint64(0x9E3779B97F4A7C15)
        x = (x ^ (x >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        x = (x ^ (x >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return x ^ (x >> np.uint64(31))


def _unit(seed: int, counter: np.ndarray, stream: int) -> np.ndarray:
    """Uniform [0, 1) doubles keyed by (seed, counter, stream): 53 random bits each."""
    with np.errstate(over="ignore"):
        h = _mix64(_mix64(counter * np.uint64(4) + np.uint64(stream)) ^ np.uint64(seed))
    return (h >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def tensor3(dims, samples: int, seed: int = SEED_TENSOR, skew=(1.0, 1.0, 1.0), block: int = 1 << 24):
    """Sparse I x J x K tensor from ``samples`` seeded index triples (duplicates merged).

    Index m of a triple is ``floor(dim_m * u ** skew_m)`` with u uniform: skew 1 is the uniform
    tensor of a given density, skew > 1 concentrates entries on low indices (hub slices and
    long fibres, as in real multi-way data).  Values are uniform in [-1, 1), keyed by the triple.
    Returns ``(i, j, k, vals)`` sorted by (i, j, k): int32, int32, int32, float32.
    """
    I, J, K = (int(d) for d in dims)
    assert max(I, J, K) < (1 << 21) and min(I, J, K) >= 1 and samples >= 0
    keys = []
    for t0 in range(0, samples, block):
        t = np.arange(t0, min(samples, t0 + block), dtype=np.uint64)
        idx = []
        for m, (d, a) in enumerate(zip((I, J, K), skew)):
            u = _unit(seed, t, m)
            idx.append(np.minimum((d * (u ** a if a != 1.0 else u)).astype(np.uint64), np.uint64(d - 1)))
        keys.append((idx[0] << np.uint64(42)) | (idx[1] << np.uint64(21)) | idx[2])
    key = np.unique(np.concatenate(keys)) if keys else np.zeros(0, np.uint64)
    i = (key >> np.uint64(42)).astype(np.int32)
    j = ((key >> np.uint64(21)) & np.uint64((1 << 21) - 1)).astype(np.int32)
    k = (key & np.uint64((1 << 21) - 1)).astype(np.int32)
    with np.errstate(over="ignore"):
        h = _mix64(key ^ np.uint64(seed + 77))
    vals = ((h >> np.uint64(40)).astype(np.float64) * (2.0 / (1 << 24)) - 1.0).astype(np.float32)
    return i, j, k, vals


@dataclass
class TensorWorkload:
    """One order-3 MTTKRP configuration: COO tensor sorted by (i, j, k) and the rank R."""
    name: str
    dims: tuple
    i: np.ndarray
    j: np.ndarray
    k: np.ndarray
    vals: np.ndarray
    R: int
    seed_f: int

    @property
    def nnz(self) -> int:
        return int(self.vals.shape[0])

    def factors(self):
        """The two dense factor matrices B (J x R) and C (K x R), standard normal."""
        return (normal_matrix(self.dims[1], self.R, self.seed_f),
                normal_matrix(self.dims[2], self.R, self.seed_f + 1))


def make_tensor_config(index: int, shrink: int = 0) -> TensorWorkload:
    """Order-3 workloads: 0 = uniform, density 0.1 %, side 4096 >> shrink, R = 64 (the shape of
    the paper's synthetic scaling tensors at half their side); 1 = skewed indices (hub slices,
    long fibres), 2^20 x 2^17 x 2^17 >> shrink with 64 M samples, R = 64."""
    s = int(shrink)
    if index == 0:
        d = max(4096 >> s, 8)
        i, j, k, v = tensor3((d, d, d), int(round(1e-3 * d ** 3)), SEED_TENSOR + 0)
        return TensorWorkload(f"tensor3_uniform_{d}_d0.001_R64", (d, d, d), i, j, k, v, 64, SEED_X + 10)
    if index == 1:
        dims = (max((1 << 20) >> s, 8), max((1 << 17) >> s, 8), max((1 << 17) >> s, 8))
        i, j, k, v = tensor3(dims, (64 << 20) >> (2 * s) if s < 13 else 64, SEED_TENSOR + 1, skew=(3.0, 2.0, 1.5))
        return TensorWorkload(f"tensor3_skewed_{dims[0]}x{dims[1]}x{dims[2]}_R64", dims, i, j, k, v, 64, SEED_X + 11)
    raise ValueError("tensor config index must be 0..1")
