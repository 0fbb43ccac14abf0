"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may
import this module.  It marshals numpy arrays into ``gnnstage_oracle.c``; every sum of the
method runs in that C file, which follows Algorithm 1 and Sections 2.1 / 3.3 / 3.4 of the
paper step by step.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gnnstage_oracle.c")
_LIBS = {}


def build(force: bool = False) -> None:
    """Compile both oracle builds (fp32 storage, and fp64 storage for finite differences)."""
    for name, flags in (("liboracle.so", []), ("liboracle_f64.so", ["-DORACLE_F64"])):
        out = os.path.join(_HERE, name)
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
            subprocess.check_call(
                ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", *flags, _SRC, "-o", out, "-lm"]
            )


class _CStage(C.Structure):
    _fields_ = [
        ("n", C.c_int64),
        ("row_ptr", C.c_void_p), ("col", C.c_void_p), ("val", C.c_void_p),
        ("t_ptr", C.c_void_p), ("t_row", C.c_void_p), ("t_edge", C.c_void_p),
        ("K", C.c_int32), ("chunk_ptr", C.c_void_p), ("chunk_of", C.c_void_p),
        ("L", C.c_int32), ("dims", C.c_void_p),
        ("variant", C.c_int32), ("a", C.c_double), ("beta", C.c_void_p),
        ("quant", C.c_int32), ("level0_f32", C.c_int32),
        ("W", C.c_void_p), ("b", C.c_void_p), ("cur", C.c_void_p), ("hist", C.c_void_p),
        ("h0", C.c_void_p), ("Z", C.c_void_p), ("dZ", C.c_void_p),
        ("dW", C.c_void_p), ("db", C.c_void_p), ("dH0", C.c_void_p),
        ("grad_in", C.c_void_p),
        ("processed", C.c_void_p), ("bprocessed", C.c_void_p),
        ("g0", C.c_void_p), ("g1", C.c_void_p),
        ("ln_g", C.c_void_p), ("ln_b", C.c_void_p), ("d_ln_g", C.c_void_p), ("d_ln_b", C.c_void_p),
        ("ln_eps", C.c_double), ("fwd_pos", C.c_void_p), ("n_fwd", C.c_int32),
        ("dropout_p", C.c_double), ("dropout_seed", C.c_uint64),
    ]


def _lib(f64: bool):
    key = "f64" if f64 else "f32"
    if key not in _LIBS:
        build()
        lib = C.CDLL(os.path.join(_HERE, "liboracle_f64.so" if f64 else "liboracle.so"))
        lib.oracle_gcn_norm.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.oracle_chunk_of.argtypes = [C.c_int64, C.c_int32, C.c_void_p, C.c_void_p]
        lib.oracle_build_transpose.argtypes = [C.c_int64] + [C.c_void_p] * 5
        lib.oracle_begin_pass.argtypes = [C.c_void_p]
        lib.oracle_select_counts.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        lib.oracle_forward_chunk.argtypes = [C.c_void_p, C.c_int32]
        lib.oracle_backward_chunk.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32]
        lib.oracle_update_history.argtypes = [C.c_void_p]
        lib.oracle_backward_finish.argtypes = [C.c_void_p]
        lib.oracle_backward_finish.restype = None
        lib.oracle_dropout_keep.argtypes = [C.c_uint64, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_double]
        lib.oracle_dropout_keep.restype = C.c_int32
        lib.oracle_splitmix64.argtypes = [C.c_uint64]
        lib.oracle_splitmix64.restype = C.c_uint64
        lib.oracle_set_threads.argtypes = [C.c_int]
        lib.oracle_max_threads.restype = C.c_int
        for f in ("oracle_gcn_norm", "oracle_chunk_of", "oracle_build_transpose", "oracle_begin_pass",
                  "oracle_select_counts", "oracle_forward_chunk", "oracle_backward_chunk",
                  "oracle_update_history", "oracle_set_threads"):
            getattr(lib, f).restype = None
        _LIBS[key] = lib
    return _LIBS[key]


def set_threads(n: int) -> None:
    _lib(False).oracle_set_threads(int(n))
    if "f64" in _LIBS:
        _LIBS["f64"].oracle_set_threads(int(n))


def max_threads() -> int:
    return int(_lib(False).oracle_max_threads())


def splitmix64_c(z: int, f64: bool = False) -> int:
    """Output function of SplitMix64 as the C oracle's dropout draws use it (state in, output out)."""
    return int(_lib(f64).oracle_splitmix64(int(z) & ((1 << 64) - 1)))


def gcn_norm(row_ptr: np.ndarray, col: np.ndarray, f64: bool = False) -> np.ndarray:
    """Section 2.1: weight 1/sqrt(D_v D_u) of every CSR entry, D = row length (self-loop included)."""
    rt = np.float64 if f64 else np.float32
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.empty(col.shape[0], dtype=rt)
    _lib(f64).oracle_gcn_norm(row_ptr.shape[0] - 1, row_ptr.ctypes.data, col.ctypes.data, val.ctypes.data)
    return val


def _ptr_array(arrs: Sequence[Optional[np.ndarray]]):
    out = (C.c_void_p * max(len(arrs), 1))()
    for i, a in enumerate(arrs):
        out[i] = None if a is None else a.ctypes.data
    return out


class OracleStage:
    """One pipeline stage on the CPU.  All buffers are numpy arrays owned by this object
    (``cur``, ``hist``, ``W``, ``b``, ``Z``, ``dZ``, ``dW``, ``db``, ``dH0``, ``grad_in``)."""

    def __init__(self, row_ptr, col, val, chunk_ptr, dims, W, b=None, *, variant="gcn", a=0.0,
                 beta=None, h0=None, quant=False, level0_f32=False, f64=False, ln_gamma=None, ln_beta=None,
                 ln_eps=1e-5, dropout_p=0.0):
        self.f64 = f64
        self.rt = rt = np.float64 if f64 else np.float32
        self.lib = _lib(f64)
        self.row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
        self.col = np.ascontiguousarray(col, dtype=np.int32)
        self.val = np.ascontiguousarray(val, dtype=rt)
        self.n = n = self.row_ptr.shape[0] - 1
        self.nnz = int(self.row_ptr[-1])
        assert self.col.shape[0] == self.nnz == self.val.shape[0]
        self.chunk_ptr = np.ascontiguousarray(chunk_ptr, dtype=np.int64)
        self.K = K = self.chunk_ptr.shape[0] - 1
        assert self.chunk_ptr[0] == 0 and self.chunk_ptr[-1] == n and np.all(np.diff(self.chunk_ptr) >= 0)
        self.dims = np.ascontiguousarray(dims, dtype=np.int32)
        self.L = L = self.dims.shape[0] - 1
        self.variant = {"gcn": 0, "gcnii": 1, "sage": 2, "resgcn": 3}[variant]
        self.a = float(a)
        self.beta = np.ascontiguousarray(beta if beta is not None else np.zeros(L), dtype=np.float64)
        assert self.beta.shape[0] == L
        self.quant = bool(quant)
        self.level0_f32 = bool(level0_f32)
        d = [int(x) for x in self.dims]
        wr = 2 if self.variant == 2 else 1  # GraphSage stacks [W_self ; W_neigh]
        self.W = [np.ascontiguousarray(W[j], dtype=rt).reshape(wr * d[j], d[j + 1]) for j in range(L)]
        self.b = [np.ascontiguousarray(b[j] if b is not None else np.zeros(d[j + 1]), dtype=rt) for j in range(L)]
        self.cur = [np.zeros((n, d[j]), dtype=rt) for j in range(L + 1)]
        self.hist = [np.zeros((n, d[j]), dtype=rt) for j in range(L)]
        self.h0 = None if h0 is None else np.ascontiguousarray(h0, dtype=rt)
        if self.variant == 1:
            assert self.h0 is not None and all(x == d[0] for x in d)
        self.Z = [np.zeros((n, d[j]), dtype=rt) for j in range(L)]
        self.dZ = [np.zeros((n, d[j]), dtype=rt) for j in range(L)]
        self.dW = [np.zeros((wr * d[j], d[j + 1]), dtype=np.float64) for j in range(L)]
        self.db = [np.zeros(d[j + 1], dtype=np.float64) for j in range(L)]
        self.dH0 = np.zeros((n, d[0]), dtype=np.float64) if self.variant == 1 else None
        self.grad_in = np.zeros((n, d[0]), dtype=rt)
        # ResGCN+: LayerNorm parameters of every layer and their gradients
        self.ln_eps = float(ln_eps)
        # ResGCN+: rate of the dropout between ReLU and the convolution; GCN, GraphSage: on the layer's output
        assert dropout_p == 0.0 or self.variant != 1, "no dropout in GCNII layers"
        self.dropout_p = float(dropout_p)
        self.dropout_seed = 0               # per pass, see set_dropout_seed
        self.ln_g = [np.ascontiguousarray(ln_gamma[j] if ln_gamma is not None else np.ones(d[j]), dtype=rt) for j in range(L)]
        self.ln_b = [np.ascontiguousarray(ln_beta[j] if ln_beta is not None else np.zeros(d[j]), dtype=rt) for j in range(L)]
        self.d_ln_g = [np.zeros(d[j], dtype=np.float64) for j in range(L)]
        self.d_ln_b = [np.zeros(d[j], dtype=np.float64) for j in range(L)]
        self.fwd_pos = np.zeros(K, dtype=np.int32)
        if self.variant == 3:
            assert all(x == d[0] for x in d)
        self.processed = np.zeros(K, dtype=np.uint8)
        self.bprocessed = np.zeros(K, dtype=np.uint8)
        mrows = int(np.diff(self.chunk_ptr).max()) if K else 0
        self._g0 = np.zeros(max(mrows * max(d), 1), dtype=rt)
        self._g1 = np.zeros(max(mrows * max(d), 1), dtype=rt)
        self.chunk_of = np.zeros(n, dtype=np.int32)
        self.lib.oracle_chunk_of(n, K, self.chunk_ptr.ctypes.data, self.chunk_of.ctypes.data)
        self.t_ptr = np.zeros(n + 1, dtype=np.int64)
        self.t_row = np.zeros(self.nnz, dtype=np.int32)
        self.t_edge = np.zeros(self.nnz, dtype=np.int64)
        self.lib.oracle_build_transpose(n, self.row_ptr.ctypes.data, self.col.ctypes.data,
                                        self.t_ptr.ctypes.data, self.t_row.ctypes.data, self.t_edge.ctypes.data)
        self._fwd_order: List[int] = []
        self._bwd_done = 0
        self._refresh()

    def _refresh(self):
        """(Re)build the C struct; call after replacing any array object."""
        self._keep = [_ptr_array(x) for x in (self.W, self.b, self.cur, self.hist, self.Z, self.dZ, self.dW, self.db,
                                              self.ln_g, self.ln_b, self.d_ln_g, self.d_ln_b)]
        pw, pb, pc, ph, pz, pdz, pdw, pdb, plg, plb, pdlg, pdlb = self._keep
        cs = _CStage()
        cs.n = self.n
        cs.row_ptr, cs.col, cs.val = self.row_ptr.ctypes.data, self.col.ctypes.data, self.val.ctypes.data
        cs.t_ptr, cs.t_row, cs.t_edge = self.t_ptr.ctypes.data, self.t_row.ctypes.data, self.t_edge.ctypes.data
        cs.K, cs.chunk_ptr, cs.chunk_of = self.K, self.chunk_ptr.ctypes.data, self.chunk_of.ctypes.data
        cs.L, cs.dims = self.L, self.dims.ctypes.data
        cs.variant, cs.a, cs.beta = self.variant, self.a, self.beta.ctypes.data
        cs.quant, cs.level0_f32 = int(self.quant), int(self.level0_f32)
        vp = lambda p: C.cast(p, C.c_void_p)
        cs.W, cs.b, cs.cur, cs.hist = vp(pw), vp(pb), vp(pc), vp(ph)
        cs.h0 = None if self.h0 is None else self.h0.ctypes.data
        cs.Z, cs.dZ, cs.dW, cs.db = vp(pz), vp(pdz), vp(pdw), vp(pdb)
        cs.dH0 = None if self.dH0 is None else self.dH0.ctypes.data
        cs.grad_in = self.grad_in.ctypes.data
        cs.processed, cs.bprocessed = self.processed.ctypes.data, self.bprocessed.ctypes.data
        cs.g0, cs.g1 = self._g0.ctypes.data, self._g1.ctypes.data
        cs.ln_g, cs.ln_b, cs.d_ln_g, cs.d_ln_b = vp(plg), vp(plb), vp(pdlg), vp(pdlb)
        cs.ln_eps, cs.fwd_pos, cs.n_fwd = self.ln_eps, self.fwd_pos.ctypes.data, 0
        cs.dropout_p, cs.dropout_seed = self.dropout_p, self.dropout_seed
        self._cs = cs

    # ---- Algorithm 1 driver pieces -------------------------------------------------
    def rows(self, k: int) -> slice:
        return slice(int(self.chunk_ptr[k]), int(self.chunk_ptr[k + 1]))

    def set_dropout_seed(self, seed: int) -> None:
        """Seed of the dropout masks of the next pass (forward and backward use the same)."""
        self.dropout_seed = int(seed) & ((1 << 64) - 1)
        self._cs.dropout_seed = self.dropout_seed

    def dropout_keep_mask(self, j: int) -> np.ndarray:
        """The 0/1 keep decisions of layer j for the current seed, element by element (for dense references):
        over the layer's input rows for ResGCN+, over its output rows for GCN and GraphSage."""
        d = int(self.dims[j] if self.variant == 3 else self.dims[j + 1])
        out = np.zeros((self.n, d), dtype=np.float64)
        for u in range(self.n):
            for c in range(d):
                out[u, c] = self.lib.oracle_dropout_keep(self.dropout_seed, j, u, d, c, self.dropout_p)
        return out

    def begin_pass(self) -> None:
        self.lib.oracle_begin_pass(C.byref(self._cs))
        self._fwd_order = []
        self._bwd_done = 0

    def select_counts(self, k: int) -> np.ndarray:
        out = np.zeros(int(self.chunk_ptr[k + 1] - self.chunk_ptr[k]), dtype=np.int32)
        self.lib.oracle_select_counts(C.byref(self._cs), int(k), out.ctypes.data)
        return out

    def forward_chunk(self, k: int) -> None:
        assert k not in self._fwd_order
        self._fwd_order.append(int(k))
        self.lib.oracle_forward_chunk(C.byref(self._cs), int(k))

    def backward_chunk(self, k: int, grad_out_rows: np.ndarray, need_input_grad: bool = True) -> None:
        assert len(self._fwd_order) == self.K, "forward pass incomplete"
        expect = self._fwd_order[self.K - 1 - self._bwd_done]
        assert k == expect, "backward must walk the chunks in reverse forward order"
        self._bwd_done += 1
        g = np.ascontiguousarray(grad_out_rows, dtype=self.rt)
        assert g.shape == (int(self.chunk_ptr[k + 1] - self.chunk_ptr[k]), int(self.dims[-1]))
        self.lib.oracle_backward_chunk(C.byref(self._cs), int(k), g.ctypes.data, int(need_input_grad))
        if self._bwd_done == self.K:  # ResGCN+: parameter gradients through the historical rows (no-op otherwise)
            self.lib.oracle_backward_finish(C.byref(self._cs))

    def update_history(self) -> None:
        self.lib.oracle_update_history(C.byref(self._cs))

    # ---- conveniences ----------------------------------------------------------------
    def zero_grads(self) -> None:
        for x in self.dW + self.db + self.d_ln_g + self.d_ln_b:
            x[...] = 0
        if self.dH0 is not None:
            self.dH0[...] = 0
        self.grad_in[...] = 0

    def forward_pass(self, order: Sequence[int]) -> None:
        self.begin_pass()
        for k in order:
            self.forward_chunk(int(k))

    def backward_pass(self, grad_out: np.ndarray, need_input_grad: bool = True) -> None:
        for k in reversed(self._fwd_order[:]):
            self.backward_chunk(k, grad_out[self.rows(k)], need_input_grad)
