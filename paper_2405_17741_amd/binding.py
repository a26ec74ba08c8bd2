"""ctypes binding of liblsw.so: same names as include/lsw.h, argument marshalling only.

Every step of the switch runs inside the library's kernels; nothing here computes.
The library must have been built (python -m paper_2405_17741_amd.build); loading fails
loudly otherwise -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

LSW_OK, LSW_ERR_ARG, LSW_ERR_SHAPE, LSW_ERR_STATE, LSW_ERR_NOMEM, LSW_ERR_DEVICE = range(6)
LSW_MAX_K = 8
LSW_OPT_KERNEL, LSW_OPT_STRICT_STATE, LSW_OPT_GRID, LSW_OPT_TILE_COLS, LSW_OPT_XCD_REMAP, LSW_OPT_GEMV_GRID, LSW_OPT_ONE_PASS, LSW_OPT_RESIDENT_Q, LSW_OPT_XCD_POOL, LSW_OPT_PANEL_GROUP = 1, 2, 3, 4, 5, 6, 7, 8, 9, 10
(LSW_Q_N_LINEARS, LSW_Q_N_LAYERS, LSW_Q_LAST_KERNEL, LSW_Q_LAST_ITEMS, LSW_Q_LAST_GRID, LSW_Q_PACKED_BYTES,
 LSW_Q_GEMV_X_ELEMS, LSW_Q_GEMV_Y_ELEMS, LSW_Q_LAST_VARIANT) = range(1, 10)
KERNEL_AUTO, KERNEL_VALU, KERNEL_MFMA = 0, 1, 2
LSW_FACTOR_F32, LSW_FACTOR_BF16 = 0, 1

EXPORTS = (
    "lsw_create_adapters", "lsw_switch", "lsw_merged_gemv", "lsw_route", "lsw_build_terms",
    "lsw_get_state", "lsw_set_option", "lsw_query", "lsw_worklist_size", "lsw_worklist_item", "lsw_worklist_item_grouped", "lsw_walk_share", "lsw_walk_pool_item",
    "lsw_destroy", "lsw_last_error", "lsw_probe_inplace", "lsw_merged_gemv_all",
    "lsw_route_dev", "lsw_switch_dev", "lsw_dev_status", "lsw_gemv_bf16", "lsw_create_adapters_ex",
    "lsw_set_base", "lsw_rebase", "lsw_enable_adapter_path", "lsw_adapter_workspace_bytes", "lsw_route_batch_dev",
    "lsw_adapter_forward", "lsw_drop_subset_tables", "lsw_adapter_forward_static",
    "lsw_adapter_layer_workspace_bytes", "lsw_adapter_forward_layer", "lsw_probe_matrix_loop", "lsw_flat_item",
)

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblsw.so")
_lib = None


class LswError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"lsw status {status}: {message}")
        self.status = status


class lsw_linear(C.Structure):
    _fields_ = [("W", C.c_void_p), ("A", C.c_void_p), ("B", C.c_void_p),
                ("out", C.c_int32), ("in_", C.c_int32), ("layer", C.c_int32), ("kind", C.c_int32), ("ld", C.c_int32)]


_i32p = C.POINTER(C.c_int32)
_f32p = C.POINTER(C.c_float)


def lib() -> C.CDLL:
    """Load liblsw.so once; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2405_17741_amd.build`")
        L = C.CDLL(_LIB_PATH)
        L.lsw_create_adapters.argtypes = [C.POINTER(lsw_linear), C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                          C.POINTER(C.c_void_p)]
        L.lsw_create_adapters_ex.argtypes = [C.POINTER(lsw_linear), C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                             C.c_int32, C.POINTER(C.c_void_p)]
        L.lsw_switch.argtypes = [C.c_void_p, _i32p, C.c_int32, _i32p, _f32p, C.c_int32, _i32p, _f32p, C.c_int32,
                                 C.c_void_p]
        L.lsw_enable_adapter_path.argtypes = [C.c_void_p]
        L.lsw_adapter_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.lsw_adapter_workspace_bytes.restype = C.c_int64
        L.lsw_route_batch_dev.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.lsw_adapter_forward.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                          C.c_void_p, C.c_void_p, C.c_void_p]
        L.lsw_adapter_forward_static.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                                 C.c_void_p, C.c_void_p]
        L.lsw_adapter_layer_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        L.lsw_adapter_layer_workspace_bytes.restype = C.c_int64
        L.lsw_adapter_forward_layer.argtypes = [C.c_void_p, C.c_int32, C.POINTER(C.c_void_p), C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                                C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p]
        L.lsw_set_base.argtypes = [C.c_void_p, C.POINTER(C.c_void_p), C.c_int32]
        L.lsw_rebase.argtypes = [C.c_void_p, _i32p, C.c_int32, _i32p, _f32p, C.c_int32, C.c_void_p]
        L.lsw_merged_gemv.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.lsw_merged_gemv_all.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.lsw_route_dev.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        L.lsw_switch_dev.argtypes = [C.c_void_p, _i32p, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                     C.c_void_p, C.c_void_p, C.c_int32, C.c_void_p]
        L.lsw_dev_status.argtypes = [C.c_void_p, _i32p]
        L.lsw_gemv_bf16.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.lsw_route.argtypes = [_f32p, C.c_int32, C.c_int32, _i32p, _f32p]
        L.lsw_build_terms.argtypes = [_i32p, _f32p, C.c_int32, _i32p, _f32p, C.c_int32, C.c_int32, C.c_float,
                                      _i32p, _f32p, _i32p]
        L.lsw_get_state.argtypes = [C.c_void_p, C.c_int32, _i32p, _f32p, _i32p]
        L.lsw_set_option.argtypes = [C.c_void_p, C.c_int32, C.c_int64]
        L.lsw_query.argtypes = [C.c_void_p, C.c_int32]
        L.lsw_query.restype = C.c_int64
        L.lsw_worklist_size.argtypes = [_i32p, _i32p, C.c_int32, C.c_int32, C.c_int32]
        L.lsw_worklist_size.restype = C.c_int64
        L.lsw_worklist_item.argtypes = [_i32p, _i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                                        _i32p, _i32p, _i32p, _i32p, _i32p]
        L.lsw_worklist_item_grouped.argtypes = [_i32p, _i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int64,
                                                _i32p, _i32p, _i32p, _i32p, _i32p]
        L.lsw_walk_share.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, _i32p]
        L.lsw_walk_pool_item.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32]
        L.lsw_walk_pool_item.restype = C.c_int32
        L.lsw_probe_inplace.argtypes = [C.c_void_p, C.c_int32, C.c_void_p]
        L.lsw_drop_subset_tables.argtypes = [C.c_void_p]
        L.lsw_probe_matrix_loop.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double)]
        L.lsw_destroy.argtypes = [C.c_void_p]
        L.lsw_destroy.restype = None
        L.lsw_last_error.restype = C.c_char_p
        for name in EXPORTS:
            if name not in ("lsw_query", "lsw_worklist_size", "lsw_destroy", "lsw_last_error", "lsw_adapter_workspace_bytes",
                            "lsw_adapter_layer_workspace_bytes"):
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def lsw_last_error() -> str:
    return lib().lsw_last_error().decode()


def _check(status: int):
    if status != LSW_OK:
        raise LswError(status, lsw_last_error())


def _i32(a):
    if a is None:
        return None, None, 0
    arr = np.ascontiguousarray(a, dtype=np.int32).reshape(-1)
    return arr, arr.ctypes.data_as(_i32p), arr.size


def _f32(a):
    if a is None:
        return None, None, 0
    arr = np.ascontiguousarray(a, dtype=np.float32).reshape(-1)
    return arr, arr.ctypes.data_as(_f32p), arr.size


def lsw_create_adapters(linears, E: int, r: int, scale: float = 1.0, factor_dtype=None) -> int:
    """linears: iterable of (W_ptr, A_ptr, B_ptr, out, in, layer, kind[, ld]) with device addresses as ints (ld: the leading
    dimension of W in elements, 0 or absent = dense).

    factor_dtype None calls lsw_create_adapters (fp32 factors); LSW_FACTOR_F32 / LSW_FACTOR_BF16 call
    lsw_create_adapters_ex.  Returns the opaque context handle (an int); release it with lsw_destroy.
    """
    linears = list(linears)
    arr = (lsw_linear * max(len(linears), 1))()
    for i, (w, a, b, o, n, layer, kind, *ld) in enumerate(linears):
        arr[i] = lsw_linear(w, a, b, o, n, layer, kind, ld[0] if ld else 0)
    ctx = C.c_void_p()
    if factor_dtype is None:
        _check(lib().lsw_create_adapters(arr if linears else None, len(linears), E, r, scale, C.byref(ctx)))
    else:
        _check(lib().lsw_create_adapters_ex(arr if linears else None, len(linears), E, r, scale, factor_dtype, C.byref(ctx)))
    return ctx.value


def lsw_switch(ctx: int, old_ids, old_gates, new_ids, new_gates, layers=None, stream: int = 0) -> None:
    _, lp, nl = _i32(layers)
    ko, oi, k_old = _i32(old_ids)
    kg, og, n_og = _f32(old_gates)
    kn, ni, k_new = _i32(new_ids)
    kh, ng, n_ng = _f32(new_gates)
    if n_og != k_old or n_ng != k_new:
        raise LswError(LSW_ERR_ARG, "ids and gates differ in length")
    _check(lib().lsw_switch(ctx, lp, nl, oi, og, k_old, ni, ng, k_new, C.c_void_p(stream)))


def lsw_enable_adapter_path(ctx: int) -> None:
    _check(lib().lsw_enable_adapter_path(ctx))


def lsw_adapter_workspace_bytes(ctx: int, lin_index: int, T: int) -> int:
    n = int(lib().lsw_adapter_workspace_bytes(ctx, lin_index, T))
    if n < 0:
        raise LswError(LSW_ERR_ARG, lsw_last_error())
    return n


def lsw_route_batch_dev(ctx: int, logits_ptr: int, n_tokens: int, k: int, ids_ptr: int, gates_ptr: int, stream: int = 0) -> None:
    _check(lib().lsw_route_batch_dev(ctx, C.c_void_p(logits_ptr), n_tokens, k, C.c_void_p(ids_ptr), C.c_void_p(gates_ptr),
                                     C.c_void_p(stream)))


def lsw_adapter_forward(ctx: int, lin_index: int, X_ptr: int, T: int, ids_ptr: int, gates_ptr: int, k: int, Y_ptr: int,
                        workspace_ptr: int, stream: int = 0) -> None:
    _check(lib().lsw_adapter_forward(ctx, lin_index, C.c_void_p(X_ptr), T, C.c_void_p(ids_ptr), C.c_void_p(gates_ptr), k,
                                     C.c_void_p(Y_ptr), C.c_void_p(workspace_ptr), C.c_void_p(stream)))


def lsw_adapter_forward_static(ctx: int, lin_index: int, X_ptr: int, T: int, ids_ptr: int, gates_ptr: int, k: int, Y_ptr: int,
                               stream: int = 0) -> None:
    _check(lib().lsw_adapter_forward_static(ctx, lin_index, C.c_void_p(X_ptr), T, C.c_void_p(ids_ptr), C.c_void_p(gates_ptr), k,
                                            C.c_void_p(Y_ptr), C.c_void_p(stream)))


def lsw_adapter_layer_workspace_bytes(ctx: int, layer: int, T: int) -> int:
    n = int(lib().lsw_adapter_layer_workspace_bytes(ctx, layer, T))
    if n < 0:
        raise LswError(LSW_ERR_ARG, lsw_last_error())
    return n


def lsw_adapter_forward_layer(ctx: int, layer: int, X_ptrs, T: int, ids_ptr: int, gates_ptr: int, k: int, Y_ptrs,
                              workspace_ptr: int, stream: int = 0) -> None:
    """X_ptrs / Y_ptrs: device addresses (ints), one per linear of `layer` in registration order."""
    X_ptrs, Y_ptrs = list(X_ptrs), list(Y_ptrs)
    xa = (C.c_void_p * max(len(X_ptrs), 1))(*X_ptrs)
    ya = (C.c_void_p * max(len(Y_ptrs), 1))(*Y_ptrs)
    _check(lib().lsw_adapter_forward_layer(ctx, layer, xa, T, C.c_void_p(ids_ptr), C.c_void_p(gates_ptr), k, ya,
                                           C.c_void_p(workspace_ptr), C.c_void_p(stream)))


def lsw_set_base(ctx: int, base_ptrs) -> None:
    """base_ptrs: device addresses (ints) of the base copy of every registered linear, in registration order."""
    base_ptrs = list(base_ptrs)
    arr = (C.c_void_p * max(len(base_ptrs), 1))(*base_ptrs)
    _check(lib().lsw_set_base(ctx, arr if base_ptrs else None, len(base_ptrs)))


def lsw_rebase(ctx: int, ids, gates, layers=None, stream: int = 0) -> None:
    _, lp, nl = _i32(layers)
    ki, ip, k = _i32(ids)
    kg, gp, n_g = _f32(gates)
    if n_g != k:
        raise LswError(LSW_ERR_ARG, "ids and gates differ in length")
    _check(lib().lsw_rebase(ctx, lp, nl, ip, gp, k, C.c_void_p(stream)))


def lsw_merged_gemv(ctx: int, lin_index: int, x_ptr: int, y_ptr: int, stream: int = 0) -> None:
    _check(lib().lsw_merged_gemv(ctx, lin_index, C.c_void_p(x_ptr), C.c_void_p(y_ptr), C.c_void_p(stream)))


def lsw_merged_gemv_all(ctx: int, x_all_ptr: int, y_all_ptr: int, stream: int = 0) -> None:
    _check(lib().lsw_merged_gemv_all(ctx, C.c_void_p(x_all_ptr), C.c_void_p(y_all_ptr), C.c_void_p(stream)))


def lsw_route_dev(ctx: int, logits_ptr: int, k: int, ids_ptr: int, gates_ptr: int, stream: int = 0) -> None:
    _check(lib().lsw_route_dev(ctx, C.c_void_p(logits_ptr), k, C.c_void_p(ids_ptr), C.c_void_p(gates_ptr), C.c_void_p(stream)))


def lsw_switch_dev(ctx: int, old_ids_ptr: int, old_gates_ptr: int, k_old: int, new_ids_ptr: int, new_gates_ptr: int,
                   k_new: int, layers=None, stream: int = 0) -> None:
    _, lp, nl = _i32(layers)
    _check(lib().lsw_switch_dev(ctx, lp, nl, C.c_void_p(old_ids_ptr), C.c_void_p(old_gates_ptr), k_old,
                                C.c_void_p(new_ids_ptr), C.c_void_p(new_gates_ptr), k_new, C.c_void_p(stream)))


def lsw_dev_status(ctx: int) -> int:
    flags = C.c_int32(0)
    _check(lib().lsw_dev_status(ctx, C.byref(flags)))
    return flags.value


def lsw_gemv_bf16(W_ptr: int, x_ptr: int, y_ptr: int, out: int, inn: int, stream: int = 0) -> None:
    _check(lib().lsw_gemv_bf16(C.c_void_p(W_ptr), C.c_void_p(x_ptr), C.c_void_p(y_ptr), out, inn, C.c_void_p(stream)))


def lsw_route(logits, k: int):
    la, lp, E = _f32(logits)
    ids = np.zeros(max(k, 1), dtype=np.int32)
    gates = np.zeros(max(k, 1), dtype=np.float32)
    _check(lib().lsw_route(lp, E, k, ids.ctypes.data_as(_i32p), gates.ctypes.data_as(_f32p)))
    return ids[:k].copy(), gates[:k].copy()


def lsw_build_terms(old_ids, old_gates, new_ids, new_gates, E: int, scale: float = 1.0):
    ko, oi, k_old = _i32(old_ids)
    kg, og, _ = _f32(old_gates)
    kn, ni, k_new = _i32(new_ids)
    kh, ng, _ = _f32(new_gates)
    ids = np.zeros(max(k_old + k_new, 1), dtype=np.int32)
    coeff = np.zeros(max(k_old + k_new, 1), dtype=np.float32)
    n = C.c_int32(0)
    _check(lib().lsw_build_terms(oi, og, k_old, ni, ng, k_new, E, scale,
                                 ids.ctypes.data_as(_i32p), coeff.ctypes.data_as(_f32p), C.byref(n)))
    return ids[: n.value].copy(), coeff[: n.value].copy()


def lsw_get_state(ctx: int, layer: int):
    ids = np.zeros(LSW_MAX_K, dtype=np.int32)
    gates = np.zeros(LSW_MAX_K, dtype=np.float32)
    k = C.c_int32(0)
    _check(lib().lsw_get_state(ctx, layer, ids.ctypes.data_as(_i32p), gates.ctypes.data_as(_f32p), C.byref(k)))
    return ids[: k.value].copy(), gates[: k.value].copy()


def lsw_set_option(ctx: int, option: int, value: int) -> None:
    _check(lib().lsw_set_option(ctx, option, value))


def lsw_query(ctx: int, what: int) -> int:
    return int(lib().lsw_query(ctx, what))


def lsw_worklist_size(out, inn, tile_rows: int, tile_cols: int) -> int:
    oa, op, n = _i32(out)
    ia, ip, _ = _i32(inn)
    return int(lib().lsw_worklist_size(op, ip, n, tile_rows, tile_cols))


def lsw_worklist_item(out, inn, tile_rows: int, tile_cols: int, item: int):
    oa, op, n = _i32(out)
    ia, ip, _ = _i32(inn)
    v = [C.c_int32(0) for _ in range(5)]
    _check(lib().lsw_worklist_item(op, ip, n, tile_rows, tile_cols, item, *[C.byref(x) for x in v]))
    return tuple(x.value for x in v)   # lin, row0, n_rows, col0, n_cols


def lsw_worklist_item_grouped(out, inn, tile_rows: int, tile_cols: int, panel_group: int, item: int):
    oa, op, n = _i32(out)
    ia, ip, _ = _i32(inn)
    v = [C.c_int32(0) for _ in range(5)]
    _check(lib().lsw_worklist_item_grouped(op, ip, n, tile_rows, tile_cols, panel_group, item, *[C.byref(x) for x in v]))
    return tuple(x.value for x in v)   # lin, row0, n_rows, col0, n_cols


def lsw_walk_share(n_items: int, grid: int, block: int, pool_div: int):
    v = (C.c_int32 * 5)()
    _check(lib().lsw_walk_share(n_items, grid, block, pool_div, v))
    return tuple(v)          # first, step, static_end, per, pool_len


def lsw_walk_pool_item(n_items: int, grid: int, pool_div: int, claim: int) -> int:
    return int(lib().lsw_walk_pool_item(n_items, grid, pool_div, claim))


def lsw_flat_item(rows, cols, grid: int, block: int, unit: int = -1):
    """One item of workgroup `block`'s range in the flat order of the prompt path's up-projection:
    (matrix, row0, col0, n_cols, next_unit); matrix = -1 for an empty range, next_unit = -1 at the range's end."""
    n = len(rows)
    r, c = (C.c_int32 * n)(*rows), (C.c_int32 * n)(*cols)
    mat, row0, col0, n_cols, nxt = C.c_int32(), C.c_int32(), C.c_int32(), C.c_int32(), C.c_int64()
    _check(lib().lsw_flat_item(r, c, n, grid, block, C.c_int64(unit), C.byref(mat), C.byref(row0), C.byref(col0), C.byref(n_cols),
                               C.byref(nxt)))
    return mat.value, row0.value, col0.value, n_cols.value, nxt.value


def lsw_probe_inplace(ctx: int, waves_per_cu: int, stream: int = 0) -> None:
    _check(lib().lsw_probe_inplace(ctx, waves_per_cu, C.c_void_p(stream)))


def lsw_probe_matrix_loop(iters: int, launches: int, copies_per_group: int, zero_operands: bool) -> float:
    """Nanoseconds per group of 6 matrix instructions (192 matrix-pipe cycles) in the bare three-pass loop."""
    ns = C.c_double(0.0)
    _check(lib().lsw_probe_matrix_loop(iters, launches, copies_per_group, 1 if zero_operands else 0, C.byref(ns)))
    return ns.value


def lsw_drop_subset_tables(ctx: int) -> None:
    _check(lib().lsw_drop_subset_tables(ctx))


def lsw_destroy(ctx: int) -> None:
    lib().lsw_destroy(ctx)


# ---------------------------------------------------------------------------
# convenience for torch users: tensors -> device addresses (still marshalling only)
# ---------------------------------------------------------------------------
def create_from_tensors(stack, shapes, E: int, r: int, scale: float = 1.0) -> int:
    """stack: [(W bf16 [out,in], A [E,r,in], B [E,out,r])] torch CUDA tensors, A and B all fp32 or all bf16;
    shapes: [(layer, kind, out, in)] as produced by inputs.Workload.linear_shapes()."""
    import torch
    dtypes = {t.dtype for _, A, B in stack for t in (A, B)}
    assert dtypes in ({torch.float32}, {torch.bfloat16}), dtypes
    factor_dtype = None if dtypes == {torch.float32} else LSW_FACTOR_BF16
    lin = []
    for (W, A, B), (layer, kind, o, n) in zip(stack, shapes):
        # W may be a column slice [:, :in] of a wider contiguous tensor: its row stride is the leading dimension
        assert A.is_contiguous() and B.is_contiguous() and W.stride(1) == 1 and W.stride(0) >= n
        assert tuple(W.shape) == (o, n) and tuple(A.shape) == (E, r, n) and tuple(B.shape) == (E, o, r)
        lin.append((W.data_ptr(), A.data_ptr(), B.data_ptr(), o, n, layer, kind, 0 if W.stride(0) == n else W.stride(0)))
    return lsw_create_adapters(lin, E, r, scale, factor_dtype)
