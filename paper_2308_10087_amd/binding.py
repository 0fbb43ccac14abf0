"""ctypes binding of libgnnstage.so: same names as the C ABI, argument marshalling only.

PyTorch supplies device memory and the stream handle; no arithmetic of the method happens
in Python.  ``GnnStage`` keeps the tensors a stage points at alive and forwards each call.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgnnstage.so")

GNNSTAGE_GCN, GNNSTAGE_GCNII, GNNSTAGE_SAGE, GNNSTAGE_RESGCN = 0, 1, 2, 3
GNNSTAGE_F32, GNNSTAGE_BF16 = 0, 1
KIND_NAMES = ["spmm_fwd", "gemm_fwd", "spmm_bwd", "gemm_dgrad", "gemm_wgrad", "history_copy", "other", "spmm_reduce"]
_ERRORS = {-1: "EINVAL", -2: "ERANGE", -3: "EORDER", -4: "ENOMEM", -5: "EHIP", -6: "ENOTSUP"}


class GnnStageError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"gnnstage error {_ERRORS.get(code, code)}: {msg}")
        self.code = code


class gnnstage_desc(C.Structure):
    _fields_ = [
        ("n_vertices", C.c_int64), ("nnz", C.c_int64),
        ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("edge_val", C.c_void_p),
        ("n_chunks", C.c_int32), ("chunk_ptr", C.c_void_p),
        ("n_layers", C.c_int32), ("dims", C.c_void_p),
        ("variant", C.c_int32), ("alpha", C.c_float), ("beta", C.c_void_p),
        ("dtype", C.c_int32), ("level0_f32", C.c_int32),
        ("W", C.c_void_p), ("bias", C.c_void_p), ("cur", C.c_void_p), ("hist", C.c_void_p),
        ("h0", C.c_void_p), ("dW", C.c_void_p), ("dbias", C.c_void_p),
        ("grad_in", C.c_void_p), ("grad_h0", C.c_void_p), ("need_input_grad", C.c_int32),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
        ("ln_gamma", C.c_void_p), ("ln_beta", C.c_void_p), ("d_ln_gamma", C.c_void_p), ("d_ln_beta", C.c_void_p),
        ("ln_eps", C.c_float), ("dropout_p", C.c_float),
    ]


class gnntrain_param(C.Structure):
    _fields_ = [("master", C.c_void_p), ("compute", C.c_void_p), ("compute_dtype", C.c_int32),
                ("grad", C.c_void_p), ("count", C.c_int64)]


class gnntrain_desc(C.Structure):
    _fields_ = [
        ("n_stages", C.c_int32), ("stages", C.c_void_p),
        ("n_classes", C.c_int32), ("head_W", C.c_void_p), ("head_b", C.c_void_p),
        ("head_dW", C.c_void_p), ("head_db", C.c_void_p), ("labels", C.c_void_p), ("train_mask", C.c_void_p),
        ("n_params", C.c_int32), ("params", C.c_void_p),
        ("optimizer", C.c_int32), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
        ("weight_decay", C.c_float),
        ("shuffle", C.c_int32), ("seed", C.c_uint64), ("alpha_hist", C.c_int32), ("history_swap", C.c_int32),
        ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
    ]


def _load():
    # The process must hold ONE HIP runtime.  PyTorch ships its own libamdhip64; importing torch
    # first makes the dynamic loader resolve this library's libamdhip64.so.7 dependency to the copy
    # that is already loaded, so both share the device context and the streams.
    import torch  # noqa: F401

    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2308_10087_amd.build` "
            "(there is no CPU fallback for the stage kernels)")
    lib = C.CDLL(_LIB_PATH)
    lib.gnnstage_version.restype = C.c_int
    lib.gnnstage_workspace_size.restype = C.c_size_t
    lib.gnnstage_workspace_size.argtypes = [C.POINTER(gnnstage_desc)]
    lib.gnnstage_create.restype = C.c_int
    lib.gnnstage_create.argtypes = [C.POINTER(gnnstage_desc), C.POINTER(C.c_void_p)]
    lib.stage_forward_chunk.restype = C.c_int
    lib.stage_forward_chunk.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
    lib.stage_backward_chunk.restype = C.c_int
    lib.stage_backward_chunk.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p]
    lib.gnnstage_flush_weight_gradients.restype = C.c_int
    lib.gnnstage_flush_weight_gradients.argtypes = [C.c_void_p, C.c_void_p]
    lib.update_history.restype = C.c_int
    lib.update_history.argtypes = [C.c_void_p, C.c_void_p]
    lib.gnnstage_update_history_swap.restype = C.c_int
    lib.gnnstage_update_history_swap.argtypes = [C.c_void_p, C.c_void_p]
    lib.gnnstage_level_buffers.restype = C.c_int
    lib.gnnstage_level_buffers.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p), C.POINTER(C.c_void_p)]
    lib.gnnstage_destroy.restype = C.c_int
    lib.gnnstage_destroy.argtypes = [C.c_void_p]
    lib.gnnstage_last_error.restype = C.c_char_p
    lib.gnnstage_last_error.argtypes = [C.c_void_p]
    lib.gnnstage_debug_select_counts.restype = C.c_int
    lib.gnnstage_debug_select_counts.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
    lib.gnnstage_plan_transpose.restype = C.c_int
    lib.gnnstage_plan_transpose.argtypes = [C.c_int64] + [C.c_void_p] * 5
    lib.gnnstage_plan_pack.restype = C.c_int
    lib.gnnstage_plan_pack.argtypes = [C.c_int64, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p,
                                       C.POINTER(C.c_int32)]
    lib.gnnstage_plan_tasks.restype = C.c_int64
    lib.gnnstage_plan_tasks.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int32,
                                        C.c_void_p, C.c_int32, C.c_void_p, C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p,
                                        C.POINTER(C.c_int64), C.c_void_p, C.c_void_p]
    lib.gnnstage_dense_plan_create.restype = C.c_int
    lib.gnnstage_dense_plan_create.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32,
                                               C.c_double, C.POINTER(C.c_void_p)]
    lib.gnnstage_dense_plan_create_capped.restype = C.c_int
    lib.gnnstage_dense_plan_create_capped.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_void_p, C.c_int32,
                                                      C.c_double, C.c_int32, C.c_int64, C.c_int32, C.POINTER(C.c_void_p)]
    lib.gnnstage_dense_plan_get.restype = C.c_int64
    lib.gnnstage_dense_plan_get.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p)]
    lib.gnnstage_dense_plan_destroy.restype = C.c_int
    lib.gnnstage_dense_plan_destroy.argtypes = [C.c_void_p]
    lib.gnnstage_dense_entries.restype = C.c_int64
    lib.gnnstage_dense_entries.argtypes = [C.c_void_p, C.c_int32]
    lib.gnnstage_layer_order.restype = C.c_int
    lib.gnnstage_layer_order.argtypes = [C.c_void_p, C.c_int32]
    lib.gnnstage_profile_enable.restype = C.c_int
    lib.gnnstage_profile_enable.argtypes = [C.c_void_p, C.c_int32]
    lib.gnnstage_profile_select.restype = C.c_int
    lib.gnnstage_profile_select.argtypes = [C.c_void_p, C.c_uint32]
    lib.gnnstage_profile_read.restype = C.c_int
    lib.gnnstage_profile_read.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.gnnstage_profile_reset.restype = C.c_int
    lib.gnnstage_profile_reset.argtypes = [C.c_void_p]
    lib.gnnstage_set_dropout_rate.restype = C.c_int
    lib.gnnstage_set_dropout_rate.argtypes = [C.c_void_p, C.c_float]
    lib.gnnstage_set_dropout_seed.restype = C.c_int
    lib.gnnstage_set_dropout_seed.argtypes = [C.c_void_p, C.c_uint64]
    lib.gnnstage_partition_chunks.restype = C.c_int
    lib.gnnstage_partition_chunks.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_double, C.c_double,
                                              C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gnnstage_permute_csr.restype = C.c_int
    lib.gnnstage_permute_csr.argtypes = [C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gnnstage_query.restype = C.c_int64
    lib.gnnstage_query.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    lib.gnnstage_buffer.restype = C.c_void_p
    lib.gnnstage_buffer.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
    # training loop (include/gnntrain.h)
    lib.gnntrain_workspace_size.restype = C.c_size_t
    lib.gnntrain_workspace_size.argtypes = [C.POINTER(gnntrain_desc)]
    lib.gnntrain_create.restype = C.c_int
    lib.gnntrain_create.argtypes = [C.POINTER(gnntrain_desc), C.POINTER(C.c_void_p)]
    lib.gnntrain_epoch.restype = C.c_int
    lib.gnntrain_epoch.argtypes = [C.c_void_p, C.c_int64, C.POINTER(C.c_float), C.c_void_p]
    lib.gnntrain_last_order.restype = C.c_int
    lib.gnntrain_last_order.argtypes = [C.c_void_p, C.c_void_p]
    lib.gnntrain_destroy.restype = C.c_int
    lib.gnntrain_destroy.argtypes = [C.c_void_p]
    lib.gnntrain_last_error.restype = C.c_char_p
    lib.gnntrain_last_error.argtypes = [C.c_void_p]
    lib.gnntrain_chunk_order.restype = C.c_int
    lib.gnntrain_chunk_order.argtypes = [C.c_uint64, C.c_int64, C.c_int32, C.c_int32, C.c_void_p]
    lib.gnntrain_softmax_xent.restype = C.c_int
    lib.gnntrain_softmax_xent.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int32,
                                          C.c_float, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.gnntrain_sum.restype = C.c_int
    lib.gnntrain_sum.argtypes = [C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p, C.c_void_p]
    lib.gnnstage_debug_gather_rate.restype = C.c_int
    lib.gnnstage_debug_gather_rate.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_int64, C.c_int32, C.c_int64, C.c_double,
                                               C.c_int32, C.c_uint32, C.c_void_p, C.c_void_p, C.POINTER(C.c_double)]
    lib.gnntrain_sum_static.restype = C.c_int
    lib.gnntrain_sum_static.argtypes = [C.c_void_p, C.c_int64, C.c_float, C.c_void_p, C.c_void_p]
    lib.gnntrain_adam_step.restype = C.c_int
    lib.gnntrain_adam_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64,
                                       C.c_float, C.c_float, C.c_float, C.c_float, C.c_float, C.c_int64, C.c_void_p]
    lib.gnntrain_sgd_step.restype = C.c_int
    lib.gnntrain_sgd_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int64, C.c_float, C.c_float,
                                      C.c_void_p]
    return lib


lib = _load()


def gnnstage_version() -> int:
    return int(lib.gnnstage_version())


# ---- host-only planning helpers (no GPU needed) -----------------------------------------
def gnnstage_plan_transpose(row_ptr: np.ndarray, col_idx: np.ndarray):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    n, nnz = row_ptr.shape[0] - 1, col_idx.shape[0]
    t_ptr = np.zeros(n + 1, dtype=np.int64)
    t_row = np.zeros(nnz, dtype=np.int32)
    t_edge = np.zeros(nnz, dtype=np.int64)
    rc = lib.gnnstage_plan_transpose(n, row_ptr.ctypes.data, col_idx.ctypes.data, t_ptr.ctypes.data,
                                     t_row.ctypes.data, t_edge.ctypes.data)
    if rc != 0:
        raise GnnStageError(rc, "gnnstage_plan_transpose")
    return t_ptr, t_row, t_edge


def gnnstage_plan_pack(n: int, idx: np.ndarray, chunk_ptr: np.ndarray):
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    chunk_ptr = np.ascontiguousarray(chunk_ptr, dtype=np.int64)
    packed = np.zeros(idx.shape[0], dtype=np.uint32)
    vbits = C.c_int32(0)
    rc = lib.gnnstage_plan_pack(n, idx.shape[0], idx.ctypes.data, chunk_ptr.shape[0] - 1, chunk_ptr.ctypes.data,
                                packed.ctypes.data, C.byref(vbits))
    if rc != 0:
        raise GnnStageError(rc, "gnnstage_plan_pack")
    return packed, int(vbits.value)


def gnnstage_plan_tasks(ptr: np.ndarray, row_begin: int, row_end: int, split_edges: int, idx=None,
                        n_vertices: int = 0, n_classes: int = 1, class_min_row: int = 0, return_classes: bool = False,
                        class_lo=None, force_slot=None):
    ptr = np.ascontiguousarray(ptr, dtype=np.int64)
    if force_slot is not None:
        force_slot = np.ascontiguousarray(force_slot, dtype=np.uint8)
        assert force_slot.shape[0] == ptr.shape[0] - 1
    fs = None if force_slot is None else force_slot.ctypes.data
    if class_lo is not None:
        class_lo = np.ascontiguousarray(class_lo, dtype=np.int64)
        assert class_lo.shape[0] == n_classes + 1
    lo = None if class_lo is None else class_lo.ctypes.data
    if idx is not None:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
    ip = None if idx is None else idx.ctypes.data
    nv = n_vertices if n_vertices > 0 else ptr.shape[0] - 1
    ns = C.c_int64(0)
    n = lib.gnnstage_plan_tasks(ptr.ctypes.data, ip, nv, row_begin, row_end, split_edges, n_classes, lo, class_min_row,
                                fs, 0, None, None, None, None, C.byref(ns), None, None)
    if n < 0:
        raise GnnStageError(int(n), "gnnstage_plan_tasks")
    row, e0 = np.zeros(n, np.int32), np.zeros(n, np.int64)
    ne, slot = np.zeros(n, np.int32), np.zeros(n, np.int32)
    class_off = np.zeros(n_classes + 1, np.int64)
    slot_class = np.zeros(max(int(ns.value), 1), np.uint8)
    got = lib.gnnstage_plan_tasks(ptr.ctypes.data, ip, nv, row_begin, row_end, split_edges, n_classes, lo,
                                  class_min_row, fs, n, row.ctypes.data, e0.ctypes.data, ne.ctypes.data, slot.ctypes.data, C.byref(ns),
                                  class_off.ctypes.data, slot_class.ctypes.data)
    if got != n:
        raise GnnStageError(int(got), "gnnstage_plan_tasks")
    if return_classes:
        return row, e0, ne, slot, int(ns.value), class_off, slot_class[:int(ns.value)]
    return row, e0, ne, slot, int(ns.value)


def gnnstage_debug_gather_rate(table, n_rows: int, row_bytes: int, gathers_per_launch: int, n_launches: int = 3,
                               hot_rows: int = 0, hot_share: float = 0.0, mode: int = 0, seed: int = 1) -> float:
    """Gathered bytes per second of random whole-row reads from ``table`` (a device tensor of at least
    n_rows * row_bytes bytes); see include/gnnstage.h."""
    import torch
    sink = torch.zeros(1, dtype=torch.int32, device=table.device)
    out = C.c_double(0.0)
    rc = lib.gnnstage_debug_gather_rate(table.data_ptr(), int(n_rows), int(row_bytes), int(gathers_per_launch), int(n_launches),
                                        int(hot_rows), float(hot_share), int(mode), int(seed) & 0xffffffff, sink.data_ptr(),
                                        C.c_void_p(torch.cuda.current_stream().cuda_stream), C.byref(out))
    if rc != 0:
        raise GnnStageError(rc, "gnnstage_debug_gather_rate")
    return float(out.value)


def gnnstage_partition_chunks(row_ptr: np.ndarray, col_idx: np.ndarray, n_chunks: int, passes: int = 6, slack: float = 1.1,
                              balance: float = 4.0, by_entries: bool = False):
    """Locality-aware chunks: returns (part, perm with perm[old id] = new id, chunk_ptr)."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    n = row_ptr.shape[0] - 1
    part, perm = np.zeros(n, dtype=np.int32), np.zeros(n, dtype=np.int32)
    chunk_ptr = np.zeros(n_chunks + 1, dtype=np.int64)
    rc = lib.gnnstage_partition_chunks(n, row_ptr.ctypes.data, col_idx.ctypes.data, int(n_chunks), int(passes), float(slack),
                                       float(balance), int(bool(by_entries)), part.ctypes.data, perm.ctypes.data,
                                       chunk_ptr.ctypes.data)
    if rc != 0:
        raise GnnStageError(rc, "gnnstage_partition_chunks")
    return part, perm, chunk_ptr


def gnnstage_permute_csr(row_ptr: np.ndarray, col_idx: np.ndarray, perm: np.ndarray):
    """The same graph with vertex ``old`` renamed ``perm[old]`` (columns ascending inside every row)."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    perm = np.ascontiguousarray(perm, dtype=np.int32)
    n = row_ptr.shape[0] - 1
    out_ptr, out_idx = np.zeros(n + 1, dtype=np.int64), np.zeros(col_idx.shape[0], dtype=np.int32)
    rc = lib.gnnstage_permute_csr(n, row_ptr.ctypes.data, col_idx.ctypes.data, perm.ctypes.data, out_ptr.ctypes.data,
                                  out_idx.ctypes.data)
    if rc != 0:
        raise GnnStageError(rc, "gnnstage_permute_csr")
    return out_ptr, out_idx


_DENSE_FIELDS = [("rem_ptr", np.int64), ("rem_idx", np.int32), ("rem_orig", np.int64), ("row_perm", np.int32),
                 ("cb_off", np.int64), ("colslot_vertex", np.int32), ("chunk_blk_off", np.int64), ("blk_rb", np.int32),
                 ("blk_cb", np.int32), ("blk_e0", np.int64), ("ent_pos", np.uint16), ("ent_orig", np.int64),
                 ("min_nnz_used", np.int32)]


def gnnstage_dense_plan(ptr: np.ndarray, idx: np.ndarray, chunk_ptr: np.ndarray, min_nnz: int, min_share: float,
                        item_blocks: int = 0, max_items: int = 0, min_nnz_many: int = 0) -> dict:
    """Dense-block plan of one aggregation direction as a dict of numpy arrays (copies); every array but
    min_nnz_used is empty when the plan is inactive.  With item_blocks, max_items and min_nnz_many a row chunk
    with more than max_items items at min_nnz takes min_nnz_many instead (gnnstage_dense_plan_create_capped)."""
    ptr = np.ascontiguousarray(ptr, dtype=np.int64)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    chunk_ptr = np.ascontiguousarray(chunk_ptr, dtype=np.int64)
    h = C.c_void_p(None)
    if item_blocks or max_items:
        rc = lib.gnnstage_dense_plan_create_capped(ptr.ctypes.data, idx.ctypes.data, ptr.shape[0] - 1, chunk_ptr.shape[0] - 1,
                                                   chunk_ptr.ctypes.data, int(min_nnz), float(min_share), int(item_blocks),
                                                   int(max_items), int(min_nnz_many), C.byref(h))
    else:
        rc = lib.gnnstage_dense_plan_create(ptr.ctypes.data, idx.ctypes.data, ptr.shape[0] - 1, chunk_ptr.shape[0] - 1,
                                            chunk_ptr.ctypes.data, int(min_nnz), float(min_share), C.byref(h))
    if rc != 0:
        raise GnnStageError(rc, "gnnstage_dense_plan_create")
    out = {}
    try:
        for what, (name, dt) in enumerate(_DENSE_FIELDS):
            data = C.c_void_p(None)
            cnt = lib.gnnstage_dense_plan_get(h, what, C.byref(data))
            if cnt < 0:
                raise GnnStageError(int(cnt), "gnnstage_dense_plan_get")
            if cnt == 0:
                out[name] = np.zeros(0, dt)
            else:
                buf = (C.c_char * (cnt * np.dtype(dt).itemsize)).from_address(data.value)
                out[name] = np.frombuffer(buf, dtype=dt).copy()
    finally:
        lib.gnnstage_dense_plan_destroy(h)
    return out


def _ptrs(tensors: Sequence) -> "C.Array":
    arr = (C.c_void_p * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i] = None if t is None else t.data_ptr()
    return arr


class GnnStage:
    """A stage handle plus the tensors it points at.

    ``cur`` / ``hist`` / ``W`` / ``bias`` / ``dW`` / ``dbias`` are lists of CUDA(HIP) tensors owned by
    the caller; the workspace is allocated here with ``torch.empty`` (device memory only).
    """

    def __init__(self, row_ptr, col_idx, chunk_ptr, dims, *, W, cur, hist, dW, bias=None, dbias=None,
                 edge_val=None, variant=GNNSTAGE_GCN, alpha=0.0, beta=None, h0=None, grad_h0=None,
                 dtype=GNNSTAGE_F32, level0_f32=False, grad_in=None, device="cuda:0", ln_gamma=None, ln_beta=None,
                 d_ln_gamma=None, d_ln_beta=None, ln_eps=1e-5, dropout_p=0.0):
        import torch

        self._torch = torch
        self.row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int64)
        self.col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
        self.chunk_ptr = np.ascontiguousarray(chunk_ptr, dtype=np.int64)
        self.dims = np.ascontiguousarray(dims, dtype=np.int32)
        self.edge_val = None if edge_val is None else np.ascontiguousarray(edge_val, dtype=np.float32)
        self.beta = None if beta is None else np.ascontiguousarray(beta, dtype=np.float32)
        self.n, self.nnz = self.row_ptr.shape[0] - 1, self.col_idx.shape[0]
        self.K, self.L = self.chunk_ptr.shape[0] - 1, self.dims.shape[0] - 1
        self.W, self.cur, self.hist, self.dW = list(W), list(cur), list(hist), list(dW)
        self.bias = None if bias is None else list(bias)
        self.dbias = None if dbias is None else list(dbias)
        self.h0, self.grad_h0, self.grad_in = h0, grad_h0, grad_in
        self._keep = [_ptrs(self.W), _ptrs(self.cur), _ptrs(self.hist), _ptrs(self.dW),
                      None if self.bias is None else _ptrs(self.bias),
                      None if self.dbias is None else _ptrs(self.dbias)]
        self.ln = [None if x is None else list(x) for x in (ln_gamma, ln_beta, d_ln_gamma, d_ln_beta)]
        self._keep_ln = [None if x is None else _ptrs(x) for x in self.ln]
        d = gnnstage_desc()
        d.n_vertices, d.nnz = self.n, self.nnz
        d.row_ptr, d.col_idx = self.row_ptr.ctypes.data, self.col_idx.ctypes.data
        d.edge_val = None if self.edge_val is None else self.edge_val.ctypes.data
        d.n_chunks, d.chunk_ptr = self.K, self.chunk_ptr.ctypes.data
        d.n_layers, d.dims = self.L, self.dims.ctypes.data
        d.variant, d.alpha = int(variant), float(alpha)
        d.beta = None if self.beta is None else self.beta.ctypes.data
        d.dtype, d.level0_f32 = int(dtype), int(bool(level0_f32))
        vp = lambda a: None if a is None else C.cast(a, C.c_void_p)
        d.W, d.cur, d.hist, d.dW = vp(self._keep[0]), vp(self._keep[1]), vp(self._keep[2]), vp(self._keep[3])
        d.bias, d.dbias = vp(self._keep[4]), vp(self._keep[5])
        d.h0 = None if h0 is None else h0.data_ptr()
        d.grad_h0 = None if grad_h0 is None else grad_h0.data_ptr()
        d.grad_in = None if grad_in is None else grad_in.data_ptr()
        d.need_input_grad = int(grad_in is not None)
        d.ln_gamma, d.ln_beta, d.d_ln_gamma, d.d_ln_beta = (vp(x) for x in self._keep_ln)
        d.ln_eps = float(ln_eps)
        d.dropout_p = float(dropout_p)
        size = int(lib.gnnstage_workspace_size(C.byref(d)))
        if size == 0:
            raise GnnStageError(-1, lib.gnnstage_last_error(None).decode())
        self.workspace_bytes = size
        self.workspace = torch.empty(size, dtype=torch.uint8, device=device)
        d.workspace, d.workspace_bytes = self.workspace.data_ptr(), size
        self._desc = d
        h = C.c_void_p(None)
        rc = lib.gnnstage_create(C.byref(d), C.byref(h))
        if rc != 0:
            raise GnnStageError(rc, lib.gnnstage_last_error(None).decode())
        self._h = h

    # -- same names as the C ABI -------------------------------------------------------------
    def _check(self, rc: int):
        if rc != 0:
            raise GnnStageError(rc, lib.gnnstage_last_error(self._h).decode())

    def _stream(self, stream):
        if stream is None:
            stream = self._torch.cuda.current_stream()
        return C.c_void_p(stream.cuda_stream)

    def stage_forward_chunk(self, chunk_id: int, pos_in_pass: int, stream=None) -> None:
        self._check(lib.stage_forward_chunk(self._h, int(chunk_id), int(pos_in_pass), self._stream(stream)))

    def stage_backward_chunk(self, chunk_id: int, grad_out_rows, stream=None) -> None:
        ptr = None if grad_out_rows is None else grad_out_rows.data_ptr()
        self._check(lib.stage_backward_chunk(self._h, int(chunk_id), ptr, self._stream(stream)))

    def gnnstage_set_dropout_seed(self, seed: int) -> None:
        self._check(lib.gnnstage_set_dropout_seed(self._h, int(seed) & ((1 << 64) - 1)))

    def gnnstage_set_dropout_rate(self, dropout_p: float) -> None:
        self._check(lib.gnnstage_set_dropout_rate(self._h, float(dropout_p)))

    def gnnstage_flush_weight_gradients(self, stream=None) -> None:
        self._check(lib.gnnstage_flush_weight_gradients(self._h, self._stream(stream)))

    def update_history(self, stream=None) -> None:
        self._check(lib.update_history(self._h, self._stream(stream)))

    def gnnstage_update_history_swap(self, stream=None) -> None:
        """The refresh without a copy: levels 1 .. L-1 trade their current and historical buffers inside the
        library.  ``self.cur`` / ``self.hist`` are re-ordered to match (same tensors, other places)."""
        self._check(lib.gnnstage_update_history_swap(self._h, self._stream(stream)))
        self.sync_level_lists()

    def sync_level_lists(self) -> None:
        """Re-orders ``self.cur`` / ``self.hist`` after the library's view of which buffer holds which level."""
        by_ptr = {t.data_ptr(): t for t in self.cur + self.hist}
        for j in range(self.L):
            c, h = self.gnnstage_level_buffers(j)
            self.cur[j], self.hist[j] = by_ptr[c], by_ptr[h]

    def gnnstage_level_buffers(self, level: int):
        """(device address of the current level, of the historical level or None for level L)."""
        c, h = C.c_void_p(None), C.c_void_p(None)
        self._check(lib.gnnstage_level_buffers(self._h, int(level), C.byref(c), C.byref(h)))
        return c.value, h.value

    def gnnstage_debug_select_counts(self, chunk_id: int) -> np.ndarray:
        rows = max(int(self.chunk_ptr[chunk_id + 1] - self.chunk_ptr[chunk_id]), 0) if 0 <= chunk_id < self.K else 0
        out = np.zeros(max(rows, 1), dtype=np.int32)
        self._check(lib.gnnstage_debug_select_counts(self._h, int(chunk_id), out.ctypes.data))
        return out[:rows]

    def gnnstage_layer_order(self, layer: int) -> int:
        rc = lib.gnnstage_layer_order(self._h, int(layer))
        if rc < 0:
            raise GnnStageError(rc, "gnnstage_layer_order")
        return rc

    def gnnstage_dense_entries(self, transposed: bool = False) -> int:
        return int(lib.gnnstage_dense_entries(self._h, int(transposed)))

    def gnnstage_profile_enable(self, on: bool) -> None:
        self._check(lib.gnnstage_profile_enable(self._h, int(on)))

    def gnnstage_profile_select(self, kinds) -> None:
        """Time only the given kinds (names from KIND_NAMES)."""
        mask = 0
        for k in kinds:
            mask |= 1 << KIND_NAMES.index(k)
        self._check(lib.gnnstage_profile_select(self._h, mask))

    def gnnstage_profile_reset(self) -> None:
        self._check(lib.gnnstage_profile_reset(self._h))

    def gnnstage_profile_read(self, layer: int = -1) -> dict:
        """{kernel kind: (milliseconds, launches)} for one layer, or summed over layers (layer < 0)."""
        out = {}
        for kind, name in enumerate(KIND_NAMES):
            ms, n = C.c_double(0), C.c_int64(0)
            self._check(lib.gnnstage_profile_read(self._h, kind, int(layer), C.byref(ms), C.byref(n)))
            out[name] = (float(ms.value), int(n.value))
        return out

    def gnnstage_destroy(self) -> None:
        if getattr(self, "_h", None) is not None and self._h.value is not None:
            rc = lib.gnnstage_destroy(self._h)
            self._h = C.c_void_p(None)
            if rc != 0:
                raise GnnStageError(rc, "gnnstage_destroy")

    def __del__(self):
        try:
            self.gnnstage_destroy()
        except Exception:
            pass

    # -- conveniences built only from the calls above ----------------------------------------
    def rows(self, k: int) -> slice:
        return slice(int(self.chunk_ptr[k]), int(self.chunk_ptr[k + 1]))

    def forward_pass(self, order, stream=None) -> None:
        for pos, k in enumerate(order):
            self.stage_forward_chunk(int(k), pos, stream)

    def backward_pass(self, order, grad_out, stream=None) -> None:
        for k in reversed(list(order)):
            self.stage_backward_chunk(int(k), grad_out[self.rows(int(k))], stream)


# ---- training loop (include/gnntrain.h) -------------------------------------------------------
GNNTRAIN_SGD, GNNTRAIN_ADAM = 0, 1


def _cur_stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def gnntrain_chunk_order(seed: int, epoch: int, n_chunks: int, shuffle: bool = True) -> np.ndarray:
    order = np.zeros(max(n_chunks, 1), dtype=np.int32)
    rc = lib.gnntrain_chunk_order(int(seed), int(epoch), int(n_chunks), int(bool(shuffle)), order.ctypes.data)
    if rc != 0:
        raise GnnStageError(rc, "gnntrain_chunk_order")
    return order[:n_chunks]


def gnntrain_softmax_xent(logits, bias, labels, mask, n_classes: int, inv_n_train: float, dlogits, row_loss) -> None:
    """logits: fp32 [rows, ld]; dlogits: fp32 or bf16 [rows, dl_ld]; labels int32 [rows]; mask uint8 [rows] or None."""
    import torch
    rows = logits.shape[0]
    rc = lib.gnntrain_softmax_xent(
        logits.data_ptr(), logits.stride(0) if rows else max(n_classes, 1), None if bias is None else bias.data_ptr(),
        labels.data_ptr(), None if mask is None else mask.data_ptr(), rows, int(n_classes), float(inv_n_train),
        dlogits.data_ptr(), GNNSTAGE_BF16 if dlogits.dtype == torch.bfloat16 else GNNSTAGE_F32,
        dlogits.stride(0) if rows else max(n_classes, 1), row_loss.data_ptr(), _cur_stream())
    if rc != 0:
        raise GnnStageError(rc, "gnntrain_softmax_xent")


def gnntrain_sum(x, scale: float, scratch, out) -> None:
    rc = lib.gnntrain_sum(x.data_ptr(), x.numel(), float(scale), scratch.data_ptr(), out.data_ptr(), _cur_stream())
    if rc != 0:
        raise GnnStageError(rc, "gnntrain_sum")


def gnntrain_sum_static(x, scale: float, out, n: Optional[int] = None) -> None:
    """gnntrain_sum without a scratch argument (the block sums go to an array inside the library)."""
    rc = lib.gnntrain_sum_static(x.data_ptr(), x.numel() if n is None else int(n), float(scale), out.data_ptr(), _cur_stream())
    if rc != 0:
        raise GnnStageError(rc, lib.gnntrain_last_error(None).decode())


def _compute_args(compute):
    import torch
    if compute is None:
        return None, GNNSTAGE_F32
    return compute.data_ptr(), GNNSTAGE_BF16 if compute.dtype == torch.bfloat16 else GNNSTAGE_F32


def gnntrain_adam_step(p, g, m, v, compute, lr, beta1, beta2, eps, weight_decay, t) -> None:
    cp, cdt = _compute_args(compute)
    rc = lib.gnntrain_adam_step(p.data_ptr(), g.data_ptr(), m.data_ptr(), v.data_ptr(), cp, cdt, p.numel(), float(lr),
                                float(beta1), float(beta2), float(eps), float(weight_decay), int(t), _cur_stream())
    if rc != 0:
        raise GnnStageError(rc, "gnntrain_adam_step")


def gnntrain_sgd_step(p, g, compute, lr, weight_decay) -> None:
    cp, cdt = _compute_args(compute)
    rc = lib.gnntrain_sgd_step(p.data_ptr(), g.data_ptr(), cp, cdt, p.numel(), float(lr), float(weight_decay), _cur_stream())
    if rc != 0:
        raise GnnStageError(rc, "gnntrain_sgd_step")


class GnnTrainer:
    """Handle of the epoch loop plus the tensors it points at.  ``params`` is a list of
    ``(master fp32 tensor, compute tensor or None, grad fp32 tensor)``."""

    def __init__(self, stages: Sequence["GnnStage"], *, head_W, head_b, head_dW, head_db, labels, train_mask, params,
                 optimizer=GNNTRAIN_ADAM, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0, shuffle=True,
                 seed=0, alpha_hist=1, history_swap=False, device="cuda:0"):
        import torch

        self._torch = torch
        self.history_swap = bool(history_swap)
        self.stages = list(stages)
        self._tensors = [head_W, head_b, head_dW, head_db, labels, train_mask, params]
        hs = (C.c_void_p * len(self.stages))(*[st._h for st in self.stages])
        ps = (gnntrain_param * max(len(params), 1))()
        for i, (master, compute, grad) in enumerate(params):
            assert master.dtype == torch.float32 and grad.dtype == torch.float32 and master.numel() == grad.numel()
            ps[i].master, ps[i].grad, ps[i].count = master.data_ptr(), grad.data_ptr(), master.numel()
            ps[i].compute, ps[i].compute_dtype = _compute_args(compute)
        self._keep = [hs, ps]
        d = gnntrain_desc()
        d.n_stages, d.stages = len(self.stages), C.cast(hs, C.c_void_p)
        d.n_classes = int(head_b.numel())
        d.head_W, d.head_b = head_W.data_ptr(), head_b.data_ptr()
        d.head_dW, d.head_db = head_dW.data_ptr(), head_db.data_ptr()
        d.labels = labels.data_ptr()
        d.train_mask = None if train_mask is None else train_mask.data_ptr()
        d.n_params, d.params = len(params), C.cast(ps, C.c_void_p)
        d.optimizer, d.lr, d.beta1, d.beta2, d.eps = int(optimizer), float(lr), float(beta1), float(beta2), float(eps)
        d.weight_decay = float(weight_decay)
        d.shuffle, d.seed, d.alpha_hist = int(bool(shuffle)), int(seed), int(alpha_hist)
        d.history_swap = int(bool(history_swap))
        size = int(lib.gnntrain_workspace_size(C.byref(d)))
        if size == 0:
            raise GnnStageError(-1, "gnntrain_workspace_size: invalid descriptor")
        self.workspace_bytes = size
        self.workspace = torch.empty(size, dtype=torch.uint8, device=device)
        d.workspace, d.workspace_bytes = self.workspace.data_ptr(), size
        self._desc = d
        h = C.c_void_p(None)
        rc = lib.gnntrain_create(C.byref(d), C.byref(h))
        if rc != 0:
            raise GnnStageError(rc, lib.gnntrain_last_error(None).decode())
        self._h = h
        self.K = self.stages[0].K

    def gnntrain_epoch(self, epoch: int, want_loss: bool = True):
        loss = C.c_float(0.0)
        rc = lib.gnntrain_epoch(self._h, int(epoch), C.byref(loss) if want_loss else None, _cur_stream())
        if rc != 0:
            raise GnnStageError(rc, lib.gnntrain_last_error(self._h).decode())
        if self.history_swap:  # the stages' level buffers may have traded places
            for st in self.stages:
                st.sync_level_lists()
        return float(loss.value) if want_loss else None

    def gnntrain_last_order(self) -> np.ndarray:
        order = np.zeros(self.K, dtype=np.int32)
        rc = lib.gnntrain_last_order(self._h, order.ctypes.data)
        if rc != 0:
            raise GnnStageError(rc, "gnntrain_last_order")
        return order

    def close(self):
        if getattr(self, "_h", None):
            lib.gnntrain_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
