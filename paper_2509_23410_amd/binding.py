"""Thin ctypes binding of the C-ABI library declared in include/patch.h (argument marshalling only).

Every function takes raw device pointers (ints, e.g. ``tensor.data_ptr()``) or torch tensors and a stream
handle (``torch.cuda.current_stream().cuda_stream``); all computation happens inside the library's HIP
kernels.  Loading fails loudly if the library has not been built (``python -m paper_2509_23410_amd.build``).
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpatch_hip.so")

OK, ERR_ARG, ERR_SHAPE, ERR_NOT_24, ERR_ALLOC, ERR_HIP, ERR_SIZE, ERR_NOT_FOUND = range(8)
PATH_AUTO, PATH_DECODE, PATH_PREFILL = 0, 1, 2

EXPORTS = [
    "patch_hard_masks", "patch_apply_mask", "patch_pack", "patch_gemm", "patch_gemm_ex", "patch_gemm_many", "patch_gemm_static", "patch_gemm_workspace_bytes", "patch_tune", "patch_tune_all",
    "patch_tune_bucket", "patch_tune_table_create", "patch_tune_table_destroy", "patch_tune_table_size", "patch_tune_table_put",
    "patch_tune_table_get", "patch_tune_table_export", "patch_tune_table_import", "patch_tune_layer", "patch_unpack",
    "patch_pack4", "patch_pack_from4", "patch_gemm4", "patch_gemm4_many", "patch_unpack4", "patch_packed4_bytes", "patch_packed4_dims", "patch_free4",
    "patch_canonical_sizes", "patch_export_canonical", "patch_packed_bytes", "patch_table_bytes", "patch_packed_dims",
    "patch_packed_tile_map", "patch_packed_row_order", "patch_probe_matrix_rate", "patch_probe_stream_read", "patch_probe_lds_fill", "patch_probe_store_tiles", "patch_probe_lds_read", "patch_gemm4_ex",
    "patch_serialized_bytes", "patch_serialize", "patch_deserialize", "patch_serialized4_bytes", "patch_serialize4", "patch_deserialize4", "patch_free", "patch_strerror", "patch_last_hip_error", "patch_version",
]


class GemmOpts(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int), ("split_k", ctypes.c_int), ("variant", ctypes.c_int),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t), ("y_bf16", ctypes.c_int)]


class TuneResult(ctypes.Structure):
    _fields_ = [("opts", GemmOpts), ("us", ctypes.c_float)]


class TuneEntry(ctypes.Structure):
    _fields_ = [("m_bucket", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64), ("n_sparse_tiles", ctypes.c_int64),
                ("tile", ctypes.c_int), ("path", ctypes.c_int), ("split_k", ctypes.c_int), ("variant", ctypes.c_int),
                ("y_bf16", ctypes.c_int), ("uses_workspace", ctypes.c_int)]


class PatchError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status}")


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2509_23410_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t
        L.patch_apply_mask.argtypes = [vp, vp, vp, i64, i64, ci, vp, vp]
        L.patch_pack.argtypes = [vp, i64, i64, vp, ci, vp, ctypes.POINTER(vp)]
        L.patch_gemm.argtypes = [vp, i64, vp, vp, vp]
        L.patch_gemm_static.argtypes = [vp, i64, vp, vp, vp]
        L.patch_gemm_static.restype = ci
        L.patch_hard_masks.argtypes = [vp, vp, i64, i64, ci, vp, vp, vp]
        L.patch_hard_masks.restype = ci
        L.patch_gemm_ex.argtypes = [vp, i64, vp, vp, vp, ctypes.POINTER(GemmOpts)]
        L.patch_tune.argtypes = [vp, i64, vp, vp, vp, sz, vp, ci, ctypes.POINTER(GemmOpts), ctypes.POINTER(ctypes.c_float)]
        L.patch_tune.restype = ci
        L.patch_tune_all.argtypes = [vp, i64, vp, vp, vp, sz, vp, ci, ctypes.POINTER(TuneResult), sz, ctypes.POINTER(sz)]
        L.patch_tune_all.restype = ci
        L.patch_tune_bucket.argtypes = [i64]
        L.patch_tune_bucket.restype = i64
        L.patch_tune_table_create.argtypes = [ctypes.POINTER(vp)]
        L.patch_tune_table_create.restype = ci
        L.patch_tune_table_destroy.argtypes = [vp]
        L.patch_tune_table_destroy.restype = None
        L.patch_tune_table_size.argtypes = [vp]
        L.patch_tune_table_size.restype = sz
        L.patch_tune_table_put.argtypes = [vp, i64, i64, i64, ci, i64, ctypes.POINTER(GemmOpts)]
        L.patch_tune_table_put.restype = ci
        L.patch_tune_table_get.argtypes = [vp, i64, i64, i64, ci, i64, vp, sz, ctypes.POINTER(GemmOpts)]
        L.patch_tune_table_get.restype = ci
        L.patch_tune_table_export.argtypes = [vp, ctypes.POINTER(TuneEntry), sz, ctypes.POINTER(sz)]
        L.patch_tune_table_export.restype = ci
        L.patch_tune_table_import.argtypes = [vp, ctypes.POINTER(TuneEntry), sz]
        L.patch_tune_table_import.restype = ci
        L.patch_tune_layer.argtypes = [vp, vp, i64, vp, i64, vp, vp, vp, sz, vp, ci]
        L.patch_tune_layer.restype = ci
        L.patch_gemm_workspace_bytes.argtypes = [i64, vp, ctypes.POINTER(GemmOpts)]
        L.patch_gemm_workspace_bytes.restype = sz
        L.patch_gemm_many.argtypes = [vp, i64, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.c_int, vp, ctypes.POINTER(GemmOpts)]
        L.patch_unpack.argtypes = [vp, vp, vp]
        L.patch_canonical_sizes.argtypes = [vp, ctypes.POINTER(sz), ctypes.POINTER(sz)]
        L.patch_export_canonical.argtypes = [vp, vp, sz, vp, sz]
        L.patch_packed_bytes.argtypes = [vp]
        L.patch_packed_bytes.restype = sz
        L.patch_table_bytes.argtypes = [vp]
        L.patch_table_bytes.restype = sz
        L.patch_packed_dims.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(ci), ctypes.POINTER(i64)]
        L.patch_packed_tile_map.argtypes = [vp, vp, sz]
        L.patch_packed_row_order.argtypes = [vp, vp, sz, ctypes.POINTER(sz)]
        L.patch_probe_matrix_rate.argtypes = [ci, vp, sz, ci, ci, vp, sz, vp]
        L.patch_probe_matrix_rate.restype = ci
        L.patch_probe_stream_read.argtypes = [vp, sz, ci, ci, vp, sz, vp]
        L.patch_probe_stream_read.restype = ci
        L.patch_probe_lds_fill.argtypes = [ci, vp, sz, ci, ci, vp, sz, vp]
        L.patch_probe_lds_fill.restype = ci
        L.patch_probe_store_tiles.argtypes = [ci, ci, vp, sz, i64, i64, vp]
        L.patch_probe_store_tiles.restype = ci
        L.patch_probe_lds_read.argtypes = [ci, ci, vp, sz, vp]
        L.patch_probe_lds_read.restype = ci
        L.patch_pack4.argtypes = [vp, i64, i64, vp, ci, vp, ctypes.POINTER(vp)]
        L.patch_pack4.restype = ci
        L.patch_gemm4.argtypes = [vp, i64, vp, vp, vp]
        L.patch_gemm4.restype = ci
        L.patch_gemm4_ex.argtypes = [vp, i64, vp, vp, vp, sz, vp]
        L.patch_gemm4_ex.restype = ci
        L.patch_pack_from4.argtypes = [vp, vp, ctypes.POINTER(vp)]
        L.patch_pack_from4.restype = ci
        L.patch_gemm4_many.argtypes = [vp, i64, ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp]
        L.patch_gemm4_many.restype = ci
        L.patch_unpack4.argtypes = [vp, vp, vp, vp, vp]
        L.patch_unpack4.restype = ci
        L.patch_packed4_bytes.argtypes = [vp]
        L.patch_packed4_bytes.restype = sz
        L.patch_packed4_dims.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(ci), ctypes.POINTER(i64)]
        L.patch_packed4_dims.restype = ci
        L.patch_free4.argtypes = [vp]
        L.patch_free4.restype = None
        for sfx in ("", "4"):
            getattr(L, f"patch_serialized{sfx}_bytes").argtypes = [vp]
            getattr(L, f"patch_serialized{sfx}_bytes").restype = sz
            getattr(L, f"patch_serialize{sfx}").argtypes = [vp, vp, sz, vp]
            getattr(L, f"patch_serialize{sfx}").restype = ci
            getattr(L, f"patch_deserialize{sfx}").argtypes = [vp, sz, vp, ctypes.POINTER(vp)]
            getattr(L, f"patch_deserialize{sfx}").restype = ci
        L.patch_free.argtypes = [vp]
        L.patch_free.restype = None
        L.patch_strerror.argtypes = [ci]
        L.patch_strerror.restype = ctypes.c_char_p
        L.patch_last_hip_error.restype = ci
        L.patch_version.restype = ctypes.c_char_p
        for f in ("patch_apply_mask", "patch_pack", "patch_gemm", "patch_gemm_ex", "patch_gemm_many", "patch_unpack", "patch_canonical_sizes",
                  "patch_export_canonical", "patch_packed_dims", "patch_packed_tile_map", "patch_packed_row_order"):
            getattr(L, f).restype = ci
        _lib = L
    return _lib


def _ptr(x) -> int:
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    raise TypeError(type(x))


def _check(st: int, what: str):
    if st != OK:
        msg = lib().patch_strerror(st).decode()
        if st == ERR_HIP:
            msg += f" (hipError {lib().patch_last_hip_error()})"
        raise PatchError(st, f"{what}: {msg}")


def strerror(st: int) -> str:
    return lib().patch_strerror(st).decode()


def version() -> str:
    return lib().patch_version().decode()


def _map_host(tile_map) -> np.ndarray:
    return np.ascontiguousarray(tile_map, dtype=np.uint8)


def patch_apply_mask(W, mask24, tile_map, N: int, K: int, tile: int, W_hat, stream: int = 0) -> None:
    tm = _map_host(tile_map)
    if N > 0 and K > 0 and tile > 0 and N % tile == 0 and K % tile == 0 and tm.size != (N // tile) * (K // tile):
        raise PatchError(ERR_ARG, "patch_apply_mask: tile_map has the wrong number of entries")
    _check(lib().patch_apply_mask(_ptr(W), _ptr(mask24), tm.ctypes.data, N, K, tile, _ptr(W_hat), stream), "patch_apply_mask")


class Packed:
    """Owner of a ``patch_packed*``; freed on ``close()`` or garbage collection."""

    def __init__(self, handle: int):
        self.handle = handle

    def close(self):
        if self.handle:
            lib().patch_free(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def nbytes(self) -> int:
        return int(lib().patch_packed_bytes(self.handle))

    @property
    def table_bytes(self) -> int:
        return int(lib().patch_table_bytes(self.handle))

    def dims(self):
        N, K, t, ns = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int(), ctypes.c_int64()
        _check(lib().patch_packed_dims(self.handle, ctypes.byref(N), ctypes.byref(K), ctypes.byref(t), ctypes.byref(ns)),
               "patch_packed_dims")
        return int(N.value), int(K.value), int(t.value), int(ns.value)

    def serialize(self, stream: int = 0) -> np.ndarray:
        """The packed weight as host bytes (header, tile map, device payload); patch_deserialize loads it again."""
        buf = np.empty(int(lib().patch_serialized_bytes(self.handle)), np.uint8)
        _check(lib().patch_serialize(self.handle, buf.ctypes.data, buf.size, stream), "patch_serialize")
        return buf

    def tile_map(self) -> np.ndarray:
        N, K, t, _ = self.dims()
        out = np.empty((N // t, K // t), np.uint8)
        _check(lib().patch_packed_tile_map(self.handle, out.ctypes.data, out.size), "patch_packed_tile_map")
        return out

    def row_order(self) -> np.ndarray:
        """(workgroups, 2) tile-row indices in prefill launch order, -1 = no second row; empty for tile 64."""
        N, K, t, _ = self.dims()
        out = np.empty(2 * ((N // t + 1) // 2), np.int32)
        n = ctypes.c_size_t(0)
        _check(lib().patch_packed_row_order(self.handle, out.ctypes.data, out.size, ctypes.byref(n)), "patch_packed_row_order")
        return out[: n.value].reshape(-1, 2)


def patch_pack(W_hat, N: int, K: int, tile_map, tile: int, stream: int = 0) -> Packed:
    tm = _map_host(tile_map)
    if N > 0 and K > 0 and tile > 0 and N % tile == 0 and K % tile == 0 and tm.size != (N // tile) * (K // tile):
        raise PatchError(ERR_ARG, "patch_pack: tile_map has the wrong number of entries")
    out = ctypes.c_void_p(0)
    _check(lib().patch_pack(_ptr(W_hat), N, K, tm.ctypes.data, tile, stream, ctypes.byref(out)), "patch_pack")
    return Packed(out.value)


def _opts(path, split_k, variant, workspace, workspace_bytes, y_bf16=False):
    if workspace is not None and workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return GemmOpts(path, split_k, variant, _ptr(workspace) if workspace is not None else None, workspace_bytes or 0, 1 if y_bf16 else 0)


def patch_gemm(X, M: int, P: Packed, Y, stream: int = 0, path: int = PATH_AUTO, split_k: int = 0, variant: int = 0,
               workspace=None, workspace_bytes=None, y_bf16: bool = False) -> None:
    """workspace: a device tensor (or pointer + workspace_bytes) for split prefill launches; y_bf16: Y is bf16; see patch.h."""
    if path == PATH_AUTO and split_k == 0 and variant == 0 and workspace is None and not y_bf16:
        st = lib().patch_gemm(_ptr(X), M, P.handle, _ptr(Y), stream)
    else:
        o = _opts(path, split_k, variant, workspace, workspace_bytes, y_bf16)
        st = lib().patch_gemm_ex(_ptr(X), M, P.handle, _ptr(Y), stream, ctypes.byref(o))
    _check(st, "patch_gemm")


def patch_gemm_static(X, M: int, P: Packed, Y, stream: int = 0) -> None:
    """patch_gemm with the library's own static scratch array in place of a caller workspace (allocates nothing)."""
    _check(lib().patch_gemm_static(_ptr(X), M, P.handle, _ptr(Y), stream), "patch_gemm_static")


STATIC_SCRATCH_BYTES = 32 << 20


def patch_tune(X, M: int, P: Packed, Y, workspace=None, workspace_bytes=None, stream: int = 0, reps: int = 20):
    """-> (dict(path, split_k, variant, uses_workspace), microseconds per launch) of the fastest schedule.  Run it with
    run_tuned(): the winner is either a schedule timed with the workspace (pass the same one again) or one timed without
    (pass none: with a workspace the library might pick K chunks the tuner never timed)."""
    if workspace is not None and workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    o, us = GemmOpts(), ctypes.c_float(0)
    _check(lib().patch_tune(_ptr(X), M, P.handle, _ptr(Y), _ptr(workspace) if workspace is not None else None,
                            workspace_bytes or 0, stream, reps, ctypes.byref(o), ctypes.byref(us)), "patch_tune")
    return dict(path=o.path, split_k=o.split_k, variant=o.variant, uses_workspace=bool(o.workspace)), float(us.value)


def _sched(o: GemmOpts) -> dict:
    return dict(path=o.path, split_k=o.split_k, variant=o.variant, uses_workspace=bool(o.workspace))


def patch_tune_all(X, M: int, P: Packed, Y, workspace=None, workspace_bytes=None, stream: int = 0, reps: int = 20):
    """-> list of (schedule dict, microseconds per launch) for every candidate the tuner times, in candidate order."""
    if workspace is not None and workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    cap = 64
    res, n = (TuneResult * cap)(), ctypes.c_size_t(0)
    _check(lib().patch_tune_all(_ptr(X), M, P.handle, _ptr(Y), _ptr(workspace) if workspace is not None else None,
                                workspace_bytes or 0, stream, reps, res, cap, ctypes.byref(n)), "patch_tune_all")
    return [(_sched(res[i].opts), float(res[i].us)) for i in range(min(n.value, cap))]


class TuneTable:
    """Owner of a patch_tune_table*: tuned schedules keyed by (M bucket, N, K, tile, 2:4 tile count)."""

    def __init__(self):
        h = ctypes.c_void_p(0)
        _check(lib().patch_tune_table_create(ctypes.byref(h)), "patch_tune_table_create")
        self.handle = h.value

    def close(self):
        if self.handle:
            lib().patch_tune_table_destroy(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __len__(self):
        return int(lib().patch_tune_table_size(self.handle))

    def put(self, M: int, N: int, K: int, tile: int, n_sparse: int, path=PATH_AUTO, split_k=0, variant=0, uses_workspace=False):
        o = GemmOpts(path, split_k, variant, 16 if uses_workspace else None, 0, 0)
        _check(lib().patch_tune_table_put(self.handle, M, N, K, tile, n_sparse, ctypes.byref(o)), "patch_tune_table_put")

    def get(self, M: int, N: int, K: int, tile: int, n_sparse: int, workspace=None, workspace_bytes=None):
        """-> schedule dict, or None when nothing usable is stored for the key."""
        if workspace is not None and workspace_bytes is None:
            workspace_bytes = workspace.numel() * workspace.element_size()
        o = GemmOpts()
        st = lib().patch_tune_table_get(self.handle, M, N, K, tile, n_sparse, _ptr(workspace) if workspace is not None else None,
                                        workspace_bytes or 0, ctypes.byref(o))
        if st == ERR_NOT_FOUND:
            return None
        _check(st, "patch_tune_table_get")
        return _sched(o)

    _FIELDS = ("m_bucket", "N", "K", "n_sparse_tiles", "tile", "path", "split_k", "variant", "y_bf16", "uses_workspace")

    def export(self) -> list:
        """Every entry as a plain dict (JSON-friendly), to keep a tuned table between processes."""
        n = ctypes.c_size_t(0)
        _check(lib().patch_tune_table_export(self.handle, None, 0, ctypes.byref(n)), "patch_tune_table_export")
        arr = (TuneEntry * max(n.value, 1))()
        _check(lib().patch_tune_table_export(self.handle, arr, n.value, ctypes.byref(n)), "patch_tune_table_export")
        return [{f: int(getattr(arr[i], f)) for f in self._FIELDS} for i in range(n.value)]

    def load(self, entries) -> None:
        """Stores / replaces entries given as the dicts export() returns; nothing is stored if one of them is bad."""
        entries = list(entries)
        arr = (TuneEntry * max(len(entries), 1))()
        for i, e in enumerate(entries):
            for f in self._FIELDS:
                setattr(arr[i], f, int(e[f]))
        _check(lib().patch_tune_table_import(self.handle, arr, len(entries)), "patch_tune_table_import")

    def get_for(self, M: int, P: Packed, workspace=None):
        N, K, t, ns = P.dims()
        return self.get(M, N, K, t, ns, workspace)

    def tune_layer(self, X_decode, M_decode: int, X_prefill, M_prefill: int, P: Packed, Y, workspace=None, stream: int = 0, reps: int = 10):
        """Decode input first, then the prefill input; both schedules are stored."""
        wb = workspace.numel() * workspace.element_size() if workspace is not None else 0
        _check(lib().patch_tune_layer(self.handle, _ptr(X_decode), M_decode, _ptr(X_prefill), M_prefill, P.handle, _ptr(Y),
                                      _ptr(workspace) if workspace is not None else None, wb, stream, reps), "patch_tune_layer")


def tune_bucket(M: int) -> int:
    return int(lib().patch_tune_bucket(M))


def run_tuned(X, M: int, P: Packed, Y, tuned: dict, workspace=None, stream: int = 0) -> None:
    """patch_gemm with exactly the schedule patch_tune returned."""
    patch_gemm(X, M, P, Y, stream, path=tuned["path"], split_k=tuned["split_k"], variant=tuned["variant"],
               workspace=workspace if tuned["uses_workspace"] else None)


def patch_gemm_workspace_bytes(M: int, P: Packed, path: int = PATH_AUTO, split_k: int = 0, variant: int = 0) -> int:
    o = GemmOpts(path, split_k, variant, None, 0, 0)
    return int(lib().patch_gemm_workspace_bytes(M, P.handle, ctypes.byref(o)))


def patch_hard_masks(P_tile, P_24, N: int, K: int, tile: int, mask24, stream: int = 0) -> np.ndarray:
    """-> tile_map (N/tile, K/tile) uint8 on the host; mask24 (device, N x K bytes) is written on the stream."""
    pt = np.ascontiguousarray(P_tile, dtype=np.float32)
    if N > 0 and K > 0 and tile > 0 and N % tile == 0 and K % tile == 0 and pt.size != (N // tile) * (K // tile):
        raise PatchError(ERR_ARG, "patch_hard_masks: P_tile has the wrong number of entries")
    tm = np.empty(max(pt.size, 1), np.uint8)
    _check(lib().patch_hard_masks(pt.ctypes.data, _ptr(P_24), N, K, tile, tm.ctypes.data, _ptr(mask24), stream), "patch_hard_masks")
    return tm[: pt.size].reshape(pt.shape)


def patch_gemm_many(X, M: int, Ps, Ys, stream: int = 0, path: int = PATH_AUTO, split_k: int = 0, variant: int = 0,
                    workspace=None, workspace_bytes=None, y_bf16: bool = False) -> None:
    """Y[i] = X * W_hat[i]^T for weights that share X (same K, same tile); one decode launch for all of them."""
    n = len(Ps)
    if n != len(Ys):
        raise PatchError(ERR_ARG, "patch_gemm_many: as many outputs as weights")
    hp = (ctypes.c_void_p * max(n, 1))(*[p.handle for p in Ps])
    yp = (ctypes.c_void_p * max(n, 1))(*[_ptr(y) for y in Ys])
    o = _opts(path, split_k, variant, workspace, workspace_bytes, y_bf16)
    _check(lib().patch_gemm_many(_ptr(X), M, hp, yp, n, stream, ctypes.byref(o)), "patch_gemm_many")


class Packed4:
    """Owner of a ``patch_packed4*`` (4-bit weight-only storage); freed on ``close()`` or garbage collection."""

    def __init__(self, handle: int):
        self.handle = handle

    def close(self):
        if self.handle:
            lib().patch_free4(self.handle)
            self.handle = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def nbytes(self) -> int:
        return int(lib().patch_packed4_bytes(self.handle))

    def serialize(self, stream: int = 0) -> np.ndarray:
        """The 4-bit storage as host bytes (header, tile map, codes and positions, scales); patch_deserialize4 loads it."""
        buf = np.empty(int(lib().patch_serialized4_bytes(self.handle)), np.uint8)
        _check(lib().patch_serialize4(self.handle, buf.ctypes.data, buf.size, stream), "patch_serialize4")
        return buf

    def dims(self):
        N, K, t, ns = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int(), ctypes.c_int64()
        _check(lib().patch_packed4_dims(self.handle, ctypes.byref(N), ctypes.byref(K), ctypes.byref(t), ctypes.byref(ns)), "patch_packed4_dims")
        return int(N.value), int(K.value), int(t.value), int(ns.value)


def _host_bytes(buf) -> np.ndarray:
    a = np.ascontiguousarray(np.frombuffer(buf, np.uint8) if isinstance(buf, (bytes, bytearray, memoryview)) else buf)
    if a.dtype != np.uint8:
        raise PatchError(ERR_ARG, "a saved weight is a uint8 buffer")
    return a


def patch_deserialize(buf, stream: int = 0) -> Packed:
    a = _host_bytes(buf)
    h = ctypes.c_void_p(0)
    _check(lib().patch_deserialize(a.ctypes.data, a.size, stream, ctypes.byref(h)), "patch_deserialize")
    return Packed(h.value)


def patch_deserialize4(buf, stream: int = 0) -> "Packed4":
    a = _host_bytes(buf)
    h = ctypes.c_void_p(0)
    _check(lib().patch_deserialize4(a.ctypes.data, a.size, stream, ctypes.byref(h)), "patch_deserialize4")
    return Packed4(h.value)


def patch_pack4(W_hat, N: int, K: int, tile_map, tile: int, stream: int = 0) -> Packed4:
    tm = _map_host(tile_map)
    if N > 0 and K > 0 and tile > 0 and N % tile == 0 and K % tile == 0 and tm.size != (N // tile) * (K // tile):
        raise PatchError(ERR_ARG, "patch_pack4: tile_map has the wrong number of entries")
    out = ctypes.c_void_p(0)
    _check(lib().patch_pack4(_ptr(W_hat), N, K, tm.ctypes.data, tile, stream, ctypes.byref(out)), "patch_pack4")
    return Packed4(out.value)


def patch_pack_from4(P4: Packed4, stream: int = 0) -> Packed:
    """The dequantized weight of a 4-bit storage packed for ``patch_gemm`` (dequantize once for prefill)."""
    out = ctypes.c_void_p(0)
    _check(lib().patch_pack_from4(P4.handle, stream, ctypes.byref(out)), "patch_pack_from4")
    return Packed(out.value)


def patch_gemm4(X, M: int, P: Packed4, Y, stream: int = 0, workspace=None) -> None:
    """Y = X . bf16(q s)^T from the 4-bit storage; with a workspace tensor: patch_gemm4_ex (K split for prefill shapes)."""
    if workspace is None:
        _check(lib().patch_gemm4(_ptr(X), M, P.handle, _ptr(Y), stream), "patch_gemm4")
    else:
        _check(lib().patch_gemm4_ex(_ptr(X), M, P.handle, _ptr(Y), _ptr(workspace), workspace.numel() * workspace.element_size(), stream),
               "patch_gemm4_ex")


def patch_gemm4_many(X, M: int, Ps, Ys, stream: int = 0) -> None:
    """Several 4-bit weights (same K, same tile) against one X in one launch per 16 rows."""
    n = len(Ps)
    if n != len(Ys):
        raise PatchError(ERR_ARG, "patch_gemm4_many: as many outputs as weights")
    hp = (ctypes.c_void_p * n)(*[p.handle for p in Ps])
    yp = (ctypes.c_void_p * n)(*[_ptr(y) for y in Ys])
    _check(lib().patch_gemm4_many(_ptr(X), M, hp, yp, n, stream), "patch_gemm4_many")


def patch_unpack4(P: Packed4, W_deq=None, codes=None, scales=None, stream: int = 0) -> None:
    _check(lib().patch_unpack4(P.handle, _ptr(W_deq) if W_deq is not None else None, _ptr(codes) if codes is not None else None,
                               _ptr(scales) if scales is not None else None, stream), "patch_unpack4")


PROBE_OPERAND_BYTES = 12 * 256 * 16


def patch_probe_matrix_rate(kind: int, operands, workgroups: int, iters: int, out, stream: int = 0) -> None:
    """Register-resident loop of the dense (kind 0) or 2:4 (kind 1) matrix instruction; see patch.h."""
    _check(lib().patch_probe_matrix_rate(kind, _ptr(operands), operands.numel() * operands.element_size(), workgroups, iters,
                                         _ptr(out), out.numel() * out.element_size(), stream), "patch_probe_matrix_rate")


def patch_probe_stream_read(src, nbytes: int, workgroups: int, threads: int, out, stream: int = 0) -> None:
    """128-bit streaming read of nbytes at src (a tensor or a device address); see patch.h."""
    _check(lib().patch_probe_stream_read(_ptr(src), nbytes, workgroups, threads, _ptr(out), out.numel() * out.element_size(), stream),
           "patch_probe_stream_read")


def patch_probe_lds_fill(kind: int, src, nbytes: int, workgroups: int, rounds: int, out, stream: int = 0) -> None:
    """The 48 KB-per-round fetch pattern of the LDS-staged prefill kernel on its own (see include/patch.h)."""
    _check(lib().patch_probe_lds_fill(kind, _ptr(src), nbytes, workgroups, rounds, _ptr(out), out.numel() * out.element_size(), stream),
           "patch_probe_lds_fill")


def patch_probe_lds_read(workgroups: int, iters: int, out, stream: int = 0) -> None:
    """Conflict-free 128-bit LDS reads by workgroups of 4 wavefronts, iters * 32 KB per workgroup (see include/patch.h)."""
    _check(lib().patch_probe_lds_read(workgroups, iters, _ptr(out), out.numel() * out.element_size(), stream), "patch_probe_lds_read")


def patch_probe_store_tiles(pattern: int, bf16: bool, Y, M: int, N: int, stream: int = 0) -> None:
    """The store instructions of a prefill workgroup's output stage on their own, one workgroup per 256 x 256 tile of Y
    (see include/patch.h)."""
    _check(lib().patch_probe_store_tiles(pattern, 1 if bf16 else 0, _ptr(Y), Y.numel() * Y.element_size(), M, N, stream),
           "patch_probe_store_tiles")


def patch_unpack(P: Packed, W_out, stream: int = 0) -> None:
    _check(lib().patch_unpack(P.handle, _ptr(W_out), stream), "patch_unpack")


def patch_export_canonical(P: Packed):
    """-> (vals uint16[...], meta uint8[...]) in the canonical order described in include/patch.h."""
    vb, mb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib().patch_canonical_sizes(P.handle, ctypes.byref(vb), ctypes.byref(mb)), "patch_canonical_sizes")
    vals = np.empty(vb.value // 2, np.uint16)
    meta = np.zeros(max(mb.value, 1), np.uint8)
    _check(lib().patch_export_canonical(P.handle, vals.ctypes.data, vb.value, meta.ctypes.data, mb.value), "patch_export_canonical")
    return vals, meta[:mb.value]
