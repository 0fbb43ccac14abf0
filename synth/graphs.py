"""Seeded synthetic graph STRUCTURE (no edge weights, none of the method's arithmetic).

Every graph comes back as a symmetric CSR with exactly one self-loop per vertex and
ascending columns inside each row: ``row_ptr`` int64 [n+1], ``col`` int32 [nnz].
The graphs stand in for the paper's datasets (Table 2 gives only their shapes); no
dataset content is reproduced.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "librmat_gen.so")
_SRC_PATH = os.path.join(_HERE, "rmat_gen.c")
_lock = threading.Lock()
_lib = None


def build_generator(force: bool = False) -> str:
    """Compile the R-MAT builder with gcc (host-only C)."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC_PATH):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC_PATH, "-o", _LIB_PATH]
        )
    return _LIB_PATH


def _load():
    global _lib
    with _lock:
        if _lib is None:
            lib = ctypes.CDLL(build_generator())
            lib.rmat_build.restype = ctypes.c_void_p
            lib.rmat_build.argtypes = [
                ctypes.c_int64, ctypes.c_int64, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                ctypes.c_uint64, ctypes.c_int, ctypes.POINTER(ctypes.c_int64),
            ]
            lib.rmat_fill.restype = None
            lib.rmat_fill.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
            _lib = lib
    return _lib


def rmat(n: int, n_candidates: int, seed: int, a: float = 0.57, b: float = 0.19, c: float = 0.19,
         relabel: bool = True):
    """R-MAT power-law graph on ``n`` vertices from ``n_candidates`` quadrant draws.

    Self pairs, duplicates and ids >= n are dropped, the graph is symmetrised, one
    self-loop per vertex is added and (by default) vertex ids are randomly permuted so
    that contiguous chunks carry no locality.
    """
    lib = _load()
    nnz = ctypes.c_int64(0)
    h = lib.rmat_build(n, n_candidates, a, b, c, seed, 1 if relabel else 0, ctypes.byref(nnz))
    row_ptr = np.empty(n + 1, dtype=np.int64)
    col = np.empty(nnz.value, dtype=np.int32)
    lib.rmat_fill(h, row_ptr.ctypes.data, col.ctypes.data)
    return row_ptr, col


def erdos_renyi(n: int, avg_degree: float, seed: int):
    """Undirected G(n, p) with p = avg_degree / (n - 1), plus self-loops."""
    rng = np.random.Generator(np.random.PCG64(seed))
    p = avg_degree / (n - 1)
    iu, ju = np.triu_indices(n, k=1)
    keep = rng.random(iu.shape[0]) < p
    iu, ju = iu[keep], ju[keep]
    return from_undirected_pairs(n, iu, ju)


def planted_partition(n: int, n_groups: int, deg_in: float, deg_out: float, seed: int):
    """Planted-partition (stochastic block) graph: vertex v belongs to group ``group[v]`` (drawn uniformly);
    every vertex draws about ``deg_in`` partners inside its group and ``deg_out`` anywhere.  Returns
    ``(row_ptr, col, group)``; a synthetic node-classification task whose labels the structure reveals."""
    rng = np.random.Generator(np.random.PCG64([seed, 77]))
    group = rng.integers(0, n_groups, size=n).astype(np.int32)
    order = np.argsort(group, kind="stable")
    start = np.searchsorted(group[order], np.arange(n_groups + 1))
    size = np.diff(start)
    k_in = rng.poisson(deg_in / 2.0, size=n)
    src_in = np.repeat(np.arange(n), k_in)
    g = group[src_in]
    pick = (rng.random(src_in.shape[0]) * size[g]).astype(np.int64)
    dst_in = order[start[g] + np.minimum(pick, size[g] - 1)]
    k_out = rng.poisson(deg_out / 2.0, size=n)
    src_out = np.repeat(np.arange(n), k_out)
    dst_out = rng.integers(0, n, size=src_out.shape[0])
    iu = np.concatenate([src_in, src_out])
    ju = np.concatenate([dst_in, dst_out])
    keep = iu != ju
    row_ptr, col = from_undirected_pairs(n, iu[keep], ju[keep])
    return row_ptr, col, group


def from_undirected_pairs(n: int, iu, ju):
    """Symmetric CSR with self-loops from a list of distinct undirected pairs."""
    iu = np.asarray(iu, dtype=np.int64)
    ju = np.asarray(ju, dtype=np.int64)
    loops = np.arange(n, dtype=np.int64)
    rows = np.concatenate([iu, ju, loops])
    cols = np.concatenate([ju, iu, loops])
    key = np.unique(rows * n + cols)
    rows, cols = key // n, key % n
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(row_ptr, rows + 1, 1)
    np.cumsum(row_ptr, out=row_ptr)
    return row_ptr, cols.astype(np.int32)


def from_directed_pairs(n: int, dst, src):
    """General (possibly non-symmetric) CSR: row = destination v, column = source u of
    edge u -> v; duplicates removed, no self-loops added."""
    dst = np.asarray(dst, dtype=np.int64)
    src = np.asarray(src, dtype=np.int64)
    key = np.unique(dst * n + src)
    rows, cols = key // n, key % n
    row_ptr = np.zeros(n + 1, dtype=np.int64)
    np.add.at(row_ptr, rows + 1, 1)
    np.cumsum(row_ptr, out=row_ptr)
    return row_ptr, cols.astype(np.int32)


def equal_chunks(n: int, k: int) -> np.ndarray:
    """K contiguous vertex-id ranges of (nearly) equal size: chunk_ptr int64 [K+1]."""
    return (np.arange(k + 1, dtype=np.int64) * n) // k


def ragged_chunks(n: int, k: int, seed: int) -> np.ndarray:
    """K contiguous ranges of unequal (possibly tiny) sizes."""
    rng = np.random.Generator(np.random.PCG64(seed))
    cuts = np.sort(rng.choice(np.arange(1, n), size=k - 1, replace=False)) if k > 1 else np.array([], dtype=np.int64)
    return np.concatenate([[0], cuts, [n]]).astype(np.int64)


def degree_stats(row_ptr: np.ndarray) -> dict:
    deg = np.diff(row_ptr)
    return {
        "n": int(deg.shape[0]),
        "nnz": int(row_ptr[-1]),
        "max_degree": int(deg.max()),
        "median_degree": float(np.median(deg)),
        "mean_degree": float(deg.mean()),
    }
