"""ctypes front end of the CPU oracle in ``patch_oracle.c``.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline``
leg of ``bench.py``; never by the product package.  It holds no arithmetic of its own: every function
below only marshals numpy arrays (bf16 as uint16 bit patterns) into the C routines.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "patch_oracle.c")
_LIB = os.path.join(_HERE, "libpatch_oracle.so")

OK, ERR_ARG, ERR_SHAPE, ERR_NOT_24, ERR_ALLOC, ERR_META = 0, 1, 2, 3, 4, 5


class OracleError(RuntimeError):
    def __init__(self, code, where=None):
        self.code, self.where = code, where
        super().__init__(f"oracle error code {code}" + (f" at (n, k) = {where}" if where else ""))


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no -march flags, no fast-math, no FP contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i64, ci, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p
        L.patch_oracle_apply_mask.argtypes = [vp, vp, vp, i64, i64, ci, vp]
        L.patch_oracle_hard_masks.argtypes = [vp, vp, i64, i64, ci, vp, vp]
        L.patch_oracle_packed_sizes.argtypes = [i64, i64, ci, vp, vp, vp]
        L.patch_oracle_pack.argtypes = [vp, i64, i64, vp, ci, vp, vp, vp]
        L.patch_oracle_unpack.argtypes = [vp, vp, i64, i64, vp, ci, vp]
        L.patch_oracle_gemm.argtypes = [vp, i64, vp, vp, i64, i64, vp, ci, vp]
        L.patch_oracle_gemm_points.argtypes = [vp, i64, vp, i64, i64, vp, i64, vp]
        L.patch_oracle_quantize4.argtypes = [vp, i64, i64, ci, vp, vp]
        L.patch_oracle_quantize4.restype = ci
        L.patch_oracle_dequantize4.argtypes = [vp, vp, i64, i64, ci, vp]
        L.patch_oracle_dequantize4.restype = ci
        L.patch_oracle_packed4_sizes.argtypes = [i64, i64, ci, vp, vp, vp, vp]
        L.patch_oracle_packed4_sizes.restype = ci
        L.patch_oracle_round_bf16.argtypes = [vp, i64, vp]
        L.patch_oracle_round_bf16.restype = ci
        for f in ("apply_mask", "packed_sizes", "pack", "unpack", "gemm", "gemm_points", "num_threads"):
            getattr(L, "patch_oracle_" + f).restype = ci
        _lib = L
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _u16(a, shape=None):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    if shape is not None:
        assert a.shape == tuple(shape), (a.shape, shape)
    return a


def _map(tile_map, N, K, t):
    tm = np.ascontiguousarray(tile_map, dtype=np.uint8)
    if N % t == 0 and K % t == 0 and t > 0:
        assert tm.size == (N // t) * (K // t), "tile_map size"
    return tm


def num_threads() -> int:
    return int(_load().patch_oracle_num_threads())


def apply_mask(W, tile_map, mask24, t):
    W = _u16(W)
    N, K = W.shape
    tm = _map(tile_map, N, K, t)
    m24 = np.ascontiguousarray(mask24, dtype=np.uint8)
    assert m24.shape == (N, K)
    out = np.empty_like(W)
    rc = _load().patch_oracle_apply_mask(_p(W), _p(tm), _p(m24), N, K, t, _p(out))
    if rc:
        raise OracleError(rc)
    return out


def hard_masks(P_tile, P_24, N, K, t):
    """-> (tile_map (N/t, K/t) uint8, mask24 (N, K) uint8) from the logits (Algorithm 1, hard masks)."""
    pt = np.ascontiguousarray(P_tile, dtype=np.float32)
    p24 = np.ascontiguousarray(P_24, dtype=np.float32)
    assert pt.shape == (N // t, K // t) and p24.shape == (6, N * K // 4)
    tm = np.empty((N // t, K // t), np.uint8)
    m24 = np.empty((N, K), np.uint8)
    rc = _load().patch_oracle_hard_masks(_p(pt), _p(p24), N, K, t, _p(tm), _p(m24))
    if rc:
        raise OracleError(rc)
    return tm, m24


def packed_sizes(N, K, t, tile_map):
    tm = _map(tile_map, N, K, t)
    nv, nm = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = _load().patch_oracle_packed_sizes(N, K, t, _p(tm), ctypes.byref(nv), ctypes.byref(nm))
    if rc:
        raise OracleError(rc)
    return int(nv.value), int(nm.value)


def pack(W_hat, tile_map, t):
    """-> (vals uint16[n_vals], meta uint8[n_meta]) in the canonical order."""
    W_hat = _u16(W_hat)
    N, K = W_hat.shape
    tm = _map(tile_map, N, K, t)
    nv, nm = packed_sizes(N, K, t, tm)
    vals, meta = np.empty(nv, np.uint16), np.zeros(max(nm, 1), np.uint8)
    bad = np.zeros(2, np.int64)
    rc = _load().patch_oracle_pack(_p(W_hat), N, K, _p(tm), t, _p(vals), _p(meta), _p(bad))
    if rc:
        raise OracleError(rc, (int(bad[0]), int(bad[1])) if rc == ERR_NOT_24 else None)
    return vals, meta[:nm]


def unpack(vals, meta, N, K, tile_map, t):
    tm = _map(tile_map, N, K, t)
    nv, nm = packed_sizes(N, K, t, tm)
    vals, meta = _u16(vals, (nv,)), np.ascontiguousarray(meta, dtype=np.uint8)
    assert meta.shape == (nm,)
    meta = meta if nm else np.zeros(1, np.uint8)
    out = np.empty((N, K), np.uint16)
    rc = _load().patch_oracle_unpack(_p(vals), _p(meta), N, K, _p(tm), t, _p(out))
    if rc:
        raise OracleError(rc)
    return out


def gemm(X, vals, meta, N, K, tile_map, t):
    """Y (float64, M x N) = X . W_hat^T from the canonical compressed form."""
    X = _u16(X)
    M = X.shape[0]
    assert X.shape == (M, K)
    tm = _map(tile_map, N, K, t)
    nv, nm = packed_sizes(N, K, t, tm)
    vals, meta = _u16(vals, (nv,)), np.ascontiguousarray(meta, dtype=np.uint8)
    assert meta.shape == (nm,)
    meta = meta if nm else np.zeros(1, np.uint8)
    Y = np.empty((M, N), np.float64)
    rc = _load().patch_oracle_gemm(_p(X), M, _p(vals), _p(meta), N, K, _p(tm), t, _p(Y))
    if rc:
        raise OracleError(rc)
    return Y


def round_bf16(Y):
    """float64 array -> bf16 bit patterns (uint16, same shape): one rounding, to nearest, ties to even."""
    Y = np.ascontiguousarray(Y, dtype=np.float64)
    out = np.empty(Y.shape, np.uint16)
    rc = _load().patch_oracle_round_bf16(_p(Y), Y.size, _p(out))
    if rc:
        raise OracleError(rc)
    return out


def quantize4(W_hat, t):
    """-> (codes int8 (N, K) in [-7, 7], scales uint16 bf16 bits (N, K / t)): symmetric 4-bit codes, one scale per row of a tile."""
    W_hat = _u16(W_hat)
    N, K = W_hat.shape
    codes, scales = np.empty((N, K), np.int8), np.empty((N, K // t), np.uint16)
    rc = _load().patch_oracle_quantize4(_p(W_hat), N, K, t, _p(codes), _p(scales))
    if rc:
        raise OracleError(rc)
    return codes, scales


def dequantize4(codes, scales, t):
    """-> bf16 bit patterns (N, K) of bf16(code * scale)."""
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    N, K = codes.shape
    scales = _u16(scales, (N, K // t))
    out = np.empty((N, K), np.uint16)
    rc = _load().patch_oracle_dequantize4(_p(codes), _p(scales), N, K, t, _p(out))
    if rc:
        raise OracleError(rc)
    return out


def packed4_sizes(N, K, t, tile_map):
    """-> (code bytes, position bytes, scale bytes) of the 4-bit storage."""
    tm = _map(tile_map, N, K, t)
    a, b, c = ctypes.c_int64(0), ctypes.c_int64(0), ctypes.c_int64(0)
    rc = _load().patch_oracle_packed4_sizes(N, K, t, _p(tm), ctypes.byref(a), ctypes.byref(b), ctypes.byref(c))
    if rc:
        raise OracleError(rc)
    return int(a.value), int(b.value), int(c.value)


def gemm_points(X, W_hat_dense, mn):
    """Exact-definition dot products at the listed (m, n) coordinates (int64 array [P, 2])."""
    X, W = _u16(X), _u16(W_hat_dense)
    (M, K), (N, K2) = X.shape, W.shape
    assert K == K2
    mn = np.ascontiguousarray(mn, dtype=np.int64)
    assert mn.ndim == 2 and mn.shape[1] == 2
    out = np.empty(mn.shape[0], np.float64)
    rc = _load().patch_oracle_gemm_points(_p(X), M, _p(W), N, K, _p(mn), mn.shape[0], _p(out))
    if rc:
        raise OracleError(rc)
    return out
