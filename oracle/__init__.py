"""ctypes binding of the CPU oracle (oracle/adaqp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the benchmark's cpu_baseline leg.
The product package never imports this module.  All arrays are host numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "adaqp_oracle.c")
_LIB = os.path.join(_DIR, "libadaqp_oracle.so")
CFLAGS = ["-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra", "-shared", "-fPIC"]

_lib: Optional[ctypes.CDLL] = None


def build(force: bool = True) -> str:
    """Compiles the oracle with gcc.  Building the checker is not using it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_LIB)
        i64, i32, u64, u32 = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_uint32
        vp = ctypes.c_void_p
        L.oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.oracle_philox4x32_10.restype = None
        L.oracle_rand16.argtypes = [u64, u64, u32]
        L.oracle_rand16.restype = u32
        L.oracle_row_stride.argtypes = [i32, i32]
        L.oracle_row_stride.restype = i64
        L.oracle_plan_layout.argtypes = [i64, i32, vp, vp, i32, vp, vp, vp]
        L.oracle_plan_layout.restype = ctypes.c_int
        L.oracle_quantize_pack.argtypes = [vp, i64, i32, vp, vp, vp, i64, u64, i64, vp, vp, vp]
        L.oracle_quantize_pack.restype = ctypes.c_int
        L.oracle_unpack_dequant.argtypes = [vp, vp, vp, vp, vp, i64, i32, vp, i64, vp]
        L.oracle_unpack_dequant.restype = ctypes.c_int
        L.oracle_trace_beta.argtypes = [vp, i64, i32, vp, vp, i64, vp]
        L.oracle_trace_beta.restype = ctypes.c_int
        L.oracle_unpack_dequant_add.argtypes = [vp, vp, vp, vp, vp, i64, i32, vp, i64]
        L.oracle_unpack_dequant_add.restype = ctypes.c_int
        L.oracle_spmm_csr.argtypes = [vp, vp, vp, i64, i64, vp, i64, i32, vp, i64, vp, vp]
        L.oracle_spmm_csr.restype = ctypes.c_int
        _lib = L
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _chk(a: np.ndarray, dtype) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    o = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(_p(c), _p(k), _p(o))
    return o


def rand16(seed: int, slot: int, column: int) -> int:
    return int(lib().oracle_rand16(seed, slot, column))


def row_stride(dim: int, bits: int) -> int:
    return int(lib().oracle_row_stride(dim, bits))


def plan_layout(dim: int, bits: np.ndarray, peer_of_slot: np.ndarray, n_peers: int
                ) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    bits = _chk(bits, np.uint8)
    peer = _chk(peer_of_slot, np.int32)
    n = bits.shape[0]
    perm = np.zeros(n, dtype=np.int64)
    off = np.zeros(n, dtype=np.int64)
    pbp = np.zeros(n_peers + 1, dtype=np.int64)
    rc = lib().oracle_plan_layout(n, dim, _p(bits), _p(peer), n_peers, _p(perm), _p(off), _p(pbp))
    if rc != 0:
        raise ValueError(f"oracle_plan_layout failed: {rc}")
    return perm, off, pbp


def quantize_pack(feat: np.ndarray, dim: int, send_idx: np.ndarray, bits: np.ndarray,
                  row_offset: np.ndarray, seed: int, packed_bytes: int, want_codes: bool = False,
                  slot_base: int = 0):
    """Returns (packed uint8[packed_bytes], params float32[n,2], codes uint8[n,dim] or None).
    slot_base is the slot number of entry 0 (the random stream is keyed by slot number)."""
    assert feat.dtype == np.float32 and feat.ndim == 2 and feat.flags.c_contiguous
    send_idx = _chk(send_idx, np.int32)
    bits = _chk(bits, np.uint8)
    row_offset = _chk(row_offset, np.int64)
    n = send_idx.shape[0]
    packed = np.zeros(packed_bytes, dtype=np.uint8)
    params = np.zeros((n, 2), dtype=np.float32)
    codes = np.zeros((n, dim), dtype=np.uint8) if want_codes else None
    rc = lib().oracle_quantize_pack(_p(feat), feat.shape[1], dim, _p(send_idx), _p(bits), _p(row_offset),
                                    n, seed, slot_base, _p(packed), _p(params), _p(codes))
    if rc != 0:
        raise ValueError(f"oracle_quantize_pack failed: {rc}")
    return packed, params, codes


def unpack_dequant(packed: np.ndarray, params: np.ndarray, bits: np.ndarray, row_offset: np.ndarray,
                   halo_idx: np.ndarray, dim: int, feat: np.ndarray, want_codes: bool = False):
    """Writes the de-quantised rows into feat (in place); returns codes or None."""
    assert feat.dtype == np.float32 and feat.ndim == 2 and feat.flags.c_contiguous
    packed = _chk(packed, np.uint8)
    params = _chk(params, np.float32)
    bits = _chk(bits, np.uint8)
    row_offset = _chk(row_offset, np.int64)
    halo_idx = _chk(halo_idx, np.int32)
    n = halo_idx.shape[0]
    codes = np.zeros((n, dim), dtype=np.uint8) if want_codes else None
    rc = lib().oracle_unpack_dequant(_p(packed), _p(params), _p(bits), _p(row_offset), _p(halo_idx),
                                     n, dim, _p(feat), feat.shape[1], _p(codes))
    if rc != 0:
        raise ValueError(f"oracle_unpack_dequant failed: {rc}")
    return codes


def trace_beta(feat: np.ndarray, dim: int, send_idx: np.ndarray, alpha_sq: np.ndarray) -> np.ndarray:
    """beta[s] = alpha_sq[s] * dim * (max - min)^2 / 6 of row send_idx[s] (Sec. 4.2)."""
    assert feat.dtype == np.float32 and feat.ndim == 2 and feat.flags.c_contiguous
    send_idx = _chk(send_idx, np.int32)
    alpha_sq = _chk(alpha_sq, np.float32)
    beta = np.zeros(send_idx.shape[0], dtype=np.float32)
    rc = lib().oracle_trace_beta(_p(feat), feat.shape[1], dim, _p(send_idx), _p(alpha_sq), send_idx.shape[0], _p(beta))
    if rc != 0:
        raise ValueError(f"oracle_trace_beta failed: {rc}")
    return beta


def unpack_dequant_add(packed: np.ndarray, params: np.ndarray, bits: np.ndarray, row_offset: np.ndarray,
                       dst_idx: np.ndarray, dim: int, grad: np.ndarray) -> None:
    """grad[dst_idx[t]] += de-quantised slot t, slots applied in order (in place)."""
    assert grad.dtype == np.float32 and grad.ndim == 2 and grad.flags.c_contiguous
    packed = _chk(packed, np.uint8)
    params = _chk(params, np.float32)
    bits = _chk(bits, np.uint8)
    row_offset = _chk(row_offset, np.int64)
    dst_idx = _chk(dst_idx, np.int32)
    rc = lib().oracle_unpack_dequant_add(_p(packed), _p(params), _p(bits), _p(row_offset), _p(dst_idx),
                                         dst_idx.shape[0], dim, _p(grad), grad.shape[1])
    if rc != 0:
        raise ValueError(f"oracle_unpack_dequant_add failed: {rc}")


def spmm_csr(rowptr: np.ndarray, col: np.ndarray, val: np.ndarray, row_begin: int, row_end: int,
             H: np.ndarray, dim: int, out: Optional[np.ndarray] = None, want64: bool = True):
    """Aggregates rows [row_begin, row_end).  Returns (out64, abs64) of shape [rows, dim] when want64."""
    assert H.dtype == np.float32 and H.ndim == 2 and H.flags.c_contiguous
    rowptr = _chk(rowptr, np.int64)
    col = _chk(col, np.int32)
    val = _chk(val, np.float32)
    rows = row_end - row_begin
    out64 = np.zeros((rows, dim), dtype=np.float64) if want64 else None
    abs64 = np.zeros((rows, dim), dtype=np.float64) if want64 else None
    ldo = 0
    if out is not None:
        assert out.dtype == np.float32 and out.ndim == 2 and out.flags.c_contiguous
        ldo = out.shape[1]
    rc = lib().oracle_spmm_csr(_p(rowptr), _p(col), _p(val), row_begin, row_end, _p(H), H.shape[1], dim,
                               _p(out), ldo, _p(out64), _p(abs64))
    if rc != 0:
        raise ValueError(f"oracle_spmm_csr failed: {rc}")
    return out64, abs64
