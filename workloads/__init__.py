"""Seeded synthetic inputs shared by the HIP path's tests/bench and the CPU oracle's tests.

Only random structure and numbers are drawn here; none of the method's arithmetic
(normalisation, products, loss) lives in this package.  The native generator
(`gen.cpp`, plain C++ with OpenMP) is compiled by `build()` into `libworkloads.so`
next to this file.

Configurations mirror the shapes of the paper's Table 1 workloads (vertex count,
edge count, feature and class widths) with synthetic graphs; the datasets
themselves are not used anywhere.
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libworkloads.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the generator (host code only)."""
    src = os.path.join(_HERE, "gen.cpp")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(
            ["g++", "-O2", "-fopenmp", "-shared", "-fPIC", "-std=c++17", "-o", _SO, src]
        )
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build(force=False)
        lib = C.CDLL(_SO)
        vp, i64, u64, dbl, i32 = C.c_void_p, C.c_int64, C.c_uint64, C.c_double, C.c_int32
        lib.wl_pattern_rows.restype = i64
        lib.wl_pattern_rows.argtypes = [vp]
        lib.wl_pattern_cols.restype = i64
        lib.wl_pattern_cols.argtypes = [vp]
        lib.wl_pattern_nnz.restype = i64
        lib.wl_pattern_nnz.argtypes = [vp]
        lib.wl_pattern_export.restype = C.c_int
        lib.wl_pattern_export.argtypes = [vp, vp, vp]
        lib.wl_pattern_free.restype = None
        lib.wl_pattern_free.argtypes = [vp]
        lib.wl_erdos_renyi.restype = vp
        lib.wl_erdos_renyi.argtypes = [i64, dbl, u64]
        lib.wl_chung_lu.restype = vp
        lib.wl_chung_lu.argtypes = [i64, dbl, dbl, dbl, C.c_int, u64]
        lib.wl_rmat.restype = vp
        lib.wl_rmat.argtypes = [C.c_int, i64, dbl, dbl, dbl, u64]
        lib.wl_row_block.restype = vp
        lib.wl_row_block.argtypes = [i64, i64, dbl, dbl, dbl, dbl, u64]
        lib.wl_normal_f32.restype = None
        lib.wl_normal_f32.argtypes = [u64, u64, i64, i64, vp]
        lib.wl_uniform_f32.restype = None
        lib.wl_uniform_f32.argtypes = [u64, u64, i64, i64, dbl, dbl, vp]
        lib.wl_labels_i32.restype = None
        lib.wl_labels_i32.argtypes = [u64, u64, i64, i32, vp]
        _lib = lib
    return _lib


@dataclass
class Pattern:
    """CSR sparsity pattern: sorted, duplicate-free rows, int32 indices, no values."""

    n_rows: int
    n_cols: int
    rowptr: np.ndarray  # int32 [n_rows+1]
    colidx: np.ndarray  # int32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


def _export(handle) -> Pattern:
    lib = _load()
    try:
        n_rows, n_cols, nnz = (
            lib.wl_pattern_rows(handle),
            lib.wl_pattern_cols(handle),
            lib.wl_pattern_nnz(handle),
        )
        rowptr = np.empty(n_rows + 1, dtype=np.int32)
        colidx = np.empty(nnz, dtype=np.int32)
        rc = lib.wl_pattern_export(handle, rowptr.ctypes.data, colidx.ctypes.data)
        if rc != 0:
            raise OverflowError("pattern has >= 2^31 entries")
        return Pattern(n_rows, n_cols, rowptr, colidx)
    finally:
        lib.wl_pattern_free(handle)


def erdos_renyi(n: int, p: float, seed: int) -> Pattern:
    return _export(_load().wl_erdos_renyi(n, p, seed))


def chung_lu(n: int, target_nnz: float, gamma: float, dmax: float, seed: int, relabel: bool = True) -> Pattern:
    return _export(_load().wl_chung_lu(n, float(target_nnz), gamma, float(dmax), int(relabel), seed))


def rmat(scale: int, n_draws: int, a: float, b: float, c: float, seed: int) -> Pattern:
    return _export(_load().wl_rmat(scale, n_draws, a, b, c, seed))


def row_block(n_rows: int, n_cols: int, target_nnz: float, gamma_r: float, dmax: float, alpha: float, seed: int) -> Pattern:
    return _export(_load().wl_row_block(n_rows, n_cols, float(target_nnz), gamma_r, float(dmax), alpha, seed))


def normal_f32(seed: int, stream: int, shape, first: int = 0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().wl_normal_f32(seed, stream, first, out.size, out.ctypes.data)
    return out


def uniform_f32(seed: int, stream: int, shape, lo: float, hi: float, first: int = 0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().wl_uniform_f32(seed, stream, first, out.size, lo, hi, out.ctypes.data)
    return out


def labels_i32(seed: int, stream: int, n: int, n_classes: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    _load().wl_labels_i32(seed, stream, n, n_classes, out.ctypes.data)
    return out


def glorot_f32(seed: int, stream: int, d_in: int, d_out: int) -> np.ndarray:
    a = math.sqrt(6.0 / (d_in + d_out))
    return uniform_f32(seed, stream, (d_in, d_out), -a, a)


# ---------------------------------------------------------------------------
# Named configurations
# ---------------------------------------------------------------------------

_SEED0 = 0x6D670001


@dataclass
class Config:
    name: str
    index: int
    dims: tuple  # layer widths d_0 .. d_L
    make_graph: object = field(repr=False)

    @property
    def seed(self) -> int:
        return _SEED0 + self.index

    def graph(self) -> Pattern:
        return self.make_graph(self.seed)

    def features(self, n: int, width: int | None = None) -> np.ndarray:
        return normal_f32(self.seed + 0x100, 0, (n, self.dims[0] if width is None else width))

    def weights(self) -> list:
        return [
            glorot_f32(self.seed + 0x200, l, self.dims[l], self.dims[l + 1])
            for l in range(len(self.dims) - 1)
        ]

    def labels(self, n: int) -> np.ndarray:
        return labels_i32(self.seed + 0x300, 0, n, self.dims[-1])


CONFIGS = {
    # 4,096 vertices, average degree 16, 2-layer 64-16-8
    "tiny": Config("tiny", 0, (64, 16, 8), lambda s: erdos_renyi(4096, 16.0 / 4095.0, s)),
    # Reddit-shaped: 232,965 vertices, ~114.6M directed entries, 602-128-41
    "medium": Config("medium", 1, (602, 128, 41), lambda s: chung_lu(232965, 114.6e6, 2.1, 21000.0, s)),
    # Products-shaped: 2,449,029 vertices, ~123.7M entries, 100-256-256-47
    "large": Config("large", 2, (100, 256, 256, 47), lambda s: chung_lu(2449029, 123.7e6, 2.3, 20000.0, s)),
    # one GPU's 1/8 row block of a Papers-shaped graph, single layer 128-256
    "block": Config(
        "block", 3, (128, 256),
        lambda s: row_block(13_900_000, 111_000_000, 200e6 - 13.9e6, 2.5, 20000.0, 0.909, s),
    ),
    # Proteins-shaped (the largest graph the paper trains on one GPU): 8.74M vertices, ~1.3B directed
    # entries (average degree ~150), 128-256-256-256.  Beyond the benchmark's named configurations;
    # needs ~30 GB of host memory to generate
    "proteins": Config("proteins", 5, (128, 256, 256, 256), lambda s: chung_lu(8_740_000, 1.3e9, 2.3, 20000.0, s)),
    # skewed R-MAT graph for the feature-width sweep
    "rmat": Config("rmat", 4, (128, 128), lambda s: rmat(22, 32_000_000, 0.57, 0.19, 0.19, s)),
}
