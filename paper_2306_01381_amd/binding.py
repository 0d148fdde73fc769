"""Thin ctypes binding of libadaqp.so (include/adaqp.h).  Argument marshalling only.

Every function has the name of the C entry point it calls.  Tensors are torch tensors that already live
where the C function expects them (device tensors for *_dev arguments, numpy arrays for the host-only
layout call); torch supplies device memory and streams and nothing else.  There is no fallback: if the
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libadaqp.so")

OK, EINVAL, EBITS, ESIZE, EHIP = 0, -1, -2, -3, -4
SERIAL, ISOLATED, FREE = 0, 1, 2
FORWARD, BACKWARD = 0, 1

_i64, _i32, _u64, _vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_void_p


class AdaqpError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        L = lib()
        msg = L.adaqp_strerror(status).decode()
        if status == EHIP:
            msg += ": " + L.adaqp_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({status})")


class SpmmPanels(ctypes.Structure):
    """Mirror of struct adaqp_spmm_panels."""
    _fields_ = [
        ("n_panels", _i32), ("n_per_tile", _i32), ("n_groups", _i64), ("n_panel_pieces", _i64),
        ("panel_rows_dev", _vp), ("pcol_dev", _vp), ("palpha_dev", _vp), ("piece_dev", _vp),
        ("panel_piece_ptr_dev", _vp), ("panel_piece_dev", _vp),
    ]


class LayerDesc(ctypes.Structure):
    """Mirror of struct adaqp_layer_desc."""
    _fields_ = [
        ("direction", _i32), ("schedule", _i32),
        ("rowptr_dev", _vp), ("col_dev", _vp), ("val_dev", _vp), ("nnz", _i64),
        ("overlap_begin", _i64), ("overlap_end", _i64), ("overlap_nnz", _i64),
        ("dependent_begin", _i64), ("dependent_end", _i64), ("dependent_nnz", _i64),
        ("feat_dev", _vp), ("n_feat_rows", _i64), ("ld", _i64), ("dim", _i32),
        ("out_dev", _vp), ("ldo", _i64),
        ("send_idx_dev", _vp), ("bits_dev", _vp), ("row_offset_dev", _vp), ("halo_idx_dev", _vp),
        ("recv_order_dev", _vp),
        ("slot_of_row_dev", _vp),
        ("tile_off_overlap_dev", _vp), ("tile_off_dependent_dev", _vp),
        ("tile_chunk_overlap", _i32), ("tile_chunk_dependent", _i32),
        ("panels_overlap", SpmmPanels), ("panels_dependent", SpmmPanels),
        ("recv_seg_order_dev", _vp), ("recv_seg_ptr_dev", _vp), ("n_recv_seg", _i64),
        ("n_send", _i64), ("seed", _u64),
        ("packed_dev", _vp), ("params_dev", _vp), ("alpha_sq_dev", _vp), ("beta_dev", _vp),
        ("recv_packed_dev", _vp), ("recv_params_dev", _vp),
        ("packed_bytes", _i64),
        ("workspace_overlap_dev", _vp), ("workspace_overlap_bytes", _i64),
        ("workspace_dependent_dev", _vp), ("workspace_dependent_bytes", _i64),
        ("stream_msg", _vp), ("stream_agg", _vp), ("event_fork", _vp), ("event_join", _vp),
    ]


_lib: Optional[ctypes.CDLL] = None

_SIGNATURES = {
    "adaqp_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "adaqp_last_hip_error": (ctypes.c_char_p, []),
    "adaqp_version": (ctypes.c_int, []),
    "adaqp_row_stride": (_i64, [_i32, _i32]),
    "adaqp_plan_layout": (ctypes.c_int, [_i64, _i32, _vp, _vp, _i32, _vp, _vp, _vp]),
    "adaqp_quantize_pack": (ctypes.c_int, [_vp, _i64, _i64, _i32, _vp, _vp, _vp, _i64, _u64, _vp, _i64, _vp, _vp]),
    "adaqp_quantize_pack_trace": (ctypes.c_int, [_vp, _i64, _i64, _i32, _vp, _vp, _vp, _i64, _u64, _vp, _i64, _vp,
                                                 _vp, _vp, _vp]),
    "adaqp_plan_recv_order": (ctypes.c_int, [_i64, _vp, _vp]),
    "adaqp_unpack_dequant": (ctypes.c_int, [_vp, _i64, _vp, _vp, _vp, _vp, _vp, _i64, _i32, _vp, _i64, _i64, _vp]),
    "adaqp_plan_recv_segments": (ctypes.c_int, [_i64, _vp, _vp, _vp, ctypes.POINTER(_i64)]),
    "adaqp_unpack_dequant_add": (ctypes.c_int, [_vp, _i64, _vp, _vp, _vp, _vp, _i64, _vp, _vp, _i64, _i32,
                                                _vp, _i64, _i64, _vp]),
    "adaqp_spmm_workspace_bytes": (ctypes.c_int, [_i64, _i64, _i32, ctypes.POINTER(_i64)]),
    "adaqp_spmm_csr": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _vp, _i64, _i64, _i32,
                                      _vp, _i64, _vp, _i64, _vp]),
    "adaqp_spmm_csr_noalloc": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _vp, _i64, _i64, _i32,
                                              _vp, _i64, _vp]),
    "adaqp_plan_spmm_tiles": (ctypes.c_int, [_vp, _vp, _i64, _i64, _i64, _vp, _vp]),
    "adaqp_spmm_tiled_workspace_bytes": (ctypes.c_int, [_i64, _i32, _vp]),
    "adaqp_spmm_tiled_pays": (_i32, [_i64, _i64]),
    "adaqp_spmm_tiled_chunk_cols": (_i32, [_vp, _i32]),
    "adaqp_spmm_csr_tiled": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _i64, _i64, _i32, _vp, _i64,
                                            _vp, _i32, _vp, _i64, _vp]),
    "adaqp_plan_spmm_panels": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _vp, _i32, _i32, _vp, _vp, _vp, _vp,
                                              _vp, _vp, _vp, _vp]),
    "adaqp_spmm_panels_workspace_bytes": (ctypes.c_int, [_i32, _i32, _vp]),
    "adaqp_spmm_panels_pay": (_i32, [_i64, _i32]),
    "adaqp_spmm_csr_panels": (ctypes.c_int, [ctypes.POINTER(SpmmPanels), _i64, _i64, _vp, _i64, _i64, _i32, _vp,
                                             _i64, _vp, _i64, _vp]),
    "adaqp_assign_bits": (ctypes.c_int, [_i64, _vp, _vp, _i32, _i32, _i32, ctypes.c_double, _vp, _vp, _vp, _vp]),
    "adaqp_plan_slot_of_row": (ctypes.c_int, [_i64, _i64, _vp, _vp]),
    "adaqp_spmm_csr_packed": (ctypes.c_int, [_vp, _vp, _vp, _i64, _i64, _i64, _i64, _vp, _i64, _i64, _i32,
                                             _vp, _i64, _vp, _vp, _i64, _vp, _vp, _vp, _i64, _vp, _i64, _vp]),
    "adaqp_layer_step": (ctypes.c_int, [ctypes.POINTER(LayerDesc)]),
    "adaqp_probe_quantize_pack": (ctypes.c_int, [_vp, _i64, _i64, _i32, _vp, _vp, _vp, _i64, _vp, _i64, _vp, _vp]),
    "adaqp_probe_unpack_dequant_add": (ctypes.c_int, [_vp, _i64, _vp, _vp, _vp, _vp, _i64, _vp, _vp, _i64, _i32,
                                                _vp, _i64, _i64, _vp]),
    "adaqp_probe_stream": (ctypes.c_int, [_vp, _vp, _i64, _i32, _vp]),
    "adaqp_probe_xcd_of_workgroup": (ctypes.c_int, [_vp, _i32, _vp]),
    "adaqp_layer_desc_bytes": (_i64, []),
}
EXPORTS = tuple(_SIGNATURES)


def lib() -> ctypes.CDLL:
    """Loads the in-tree library; raises if it has not been built (python -m paper_2306_01381_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2306_01381_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(L, name)
            fn.restype = res
            fn.argtypes = args
        if int(L.adaqp_layer_desc_bytes()) != ctypes.sizeof(LayerDesc):
            raise ImportError(f"LayerDesc ({ctypes.sizeof(LayerDesc)} bytes) does not mirror adaqp_layer_desc "
                              f"({int(L.adaqp_layer_desc_bytes())} bytes) of {LIB_PATH}: rebuild the library")
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != OK:
        raise AdaqpError(status, where)


def _dev(t: Optional[torch.Tensor], dtype: torch.dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError(f"{name} must be a device tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise TypeError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream(stream: Optional[torch.cuda.Stream]) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _matrix(t: torch.Tensor, name: str) -> Tuple[int, int, int]:
    """(pointer, rows, leading dimension) of a 2-D fp32 device tensor whose rows are contiguous."""
    if not t.is_cuda or t.dtype != torch.float32 or t.dim() != 2 or t.stride(1) != 1:
        raise TypeError(f"{name} must be a 2-D fp32 device tensor with unit column stride")
    return t.data_ptr(), t.shape[0], t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def adaqp_version() -> int:
    return lib().adaqp_version()


def adaqp_row_stride(dim: int, bits: int) -> int:
    return int(lib().adaqp_row_stride(dim, bits))


def adaqp_plan_layout(dim: int, bits_host: np.ndarray, peer_of_slot_host: np.ndarray, n_peers: int):
    """Host-only.  Returns (perm, row_offset, peer_byte_ptr) as int64 numpy arrays."""
    bits = np.ascontiguousarray(bits_host, dtype=np.uint8)
    peer = np.ascontiguousarray(peer_of_slot_host, dtype=np.int32)
    n = bits.shape[0]
    if peer.shape[0] != n:
        raise ValueError("bits and peer_of_slot differ in length")
    perm = np.zeros(n, dtype=np.int64)
    off = np.zeros(n, dtype=np.int64)
    pbp = np.zeros(max(n_peers, 0) + 1, dtype=np.int64)
    _check(lib().adaqp_plan_layout(n, dim, bits.ctypes.data, peer.ctypes.data, n_peers,
                                   perm.ctypes.data, off.ctypes.data, pbp.ctypes.data), "adaqp_plan_layout")
    return perm, off, pbp


def adaqp_quantize_pack(feat: torch.Tensor, dim: int, send_idx: torch.Tensor, bits: torch.Tensor,
                        row_offset: torch.Tensor, seed: int, packed: torch.Tensor, params: torch.Tensor,
                        stream: Optional[torch.cuda.Stream] = None) -> None:
    fp, n_rows, ld = _matrix(feat, "feat")
    n = send_idx.shape[0]
    _check(lib().adaqp_quantize_pack(fp, n_rows, ld, dim, _dev(send_idx, torch.int32, "send_idx"),
                                     _dev(bits, torch.uint8, "bits"), _dev(row_offset, torch.int64, "row_offset"),
                                     n, seed & (2**64 - 1), _dev(packed, torch.uint8, "packed"), packed.numel(),
                                     _dev(params, torch.float32, "params"), _stream(stream)),
           "adaqp_quantize_pack")


def adaqp_quantize_pack_trace(feat: torch.Tensor, dim: int, send_idx: torch.Tensor, bits: torch.Tensor,
                              row_offset: torch.Tensor, seed: int, packed: torch.Tensor, params: torch.Tensor,
                              alpha_sq: torch.Tensor, beta: torch.Tensor,
                              stream: Optional[torch.cuda.Stream] = None) -> None:
    fp, n_rows, ld = _matrix(feat, "feat")
    n = send_idx.shape[0]
    _check(lib().adaqp_quantize_pack_trace(fp, n_rows, ld, dim, _dev(send_idx, torch.int32, "send_idx"),
                                           _dev(bits, torch.uint8, "bits"),
                                           _dev(row_offset, torch.int64, "row_offset"), n, seed & (2**64 - 1),
                                           _dev(packed, torch.uint8, "packed"), packed.numel(),
                                           _dev(params, torch.float32, "params"),
                                           _dev(alpha_sq, torch.float32, "alpha_sq"),
                                           _dev(beta, torch.float32, "beta"), _stream(stream)),
           "adaqp_quantize_pack_trace")


def adaqp_plan_recv_order(halo_idx_host: np.ndarray) -> np.ndarray:
    """Host-only.  Returns the int32 visiting order of the receive slots (ascending destination rows)."""
    halo = np.ascontiguousarray(halo_idx_host, dtype=np.int32)
    order = np.zeros(halo.shape[0], dtype=np.int32)
    _check(lib().adaqp_plan_recv_order(halo.shape[0], halo.ctypes.data, order.ctypes.data), "adaqp_plan_recv_order")
    return order


def adaqp_unpack_dequant(packed: torch.Tensor, params: torch.Tensor, bits: torch.Tensor,
                         row_offset: torch.Tensor, halo_idx: torch.Tensor, dim: int, feat: torch.Tensor,
                         order: Optional[torch.Tensor] = None,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
    fp, n_rows, ld = _matrix(feat, "feat")
    n = halo_idx.shape[0]
    _check(lib().adaqp_unpack_dequant(_dev(packed, torch.uint8, "packed"), packed.numel(),
                                      _dev(params, torch.float32, "params"), _dev(bits, torch.uint8, "bits"),
                                      _dev(row_offset, torch.int64, "row_offset"),
                                      _dev(halo_idx, torch.int32, "halo_idx"), _dev(order, torch.int32, "order"),
                                      n, dim, fp, n_rows, ld,
                                      _stream(stream)),
           "adaqp_unpack_dequant")


def adaqp_plan_recv_segments(dst_idx_host: np.ndarray):
    """Host-only.  Returns (order int32[n], seg_ptr int64[n_seg + 1])."""
    dst = np.ascontiguousarray(dst_idx_host, dtype=np.int32)
    n = dst.shape[0]
    order = np.zeros(n, dtype=np.int32)
    seg_ptr = np.zeros(n + 1, dtype=np.int64)
    n_seg = _i64(0)
    _check(lib().adaqp_plan_recv_segments(n, dst.ctypes.data, order.ctypes.data, seg_ptr.ctypes.data,
                                          ctypes.byref(n_seg)), "adaqp_plan_recv_segments")
    return order, seg_ptr[: n_seg.value + 1].copy()


def adaqp_unpack_dequant_add(packed: torch.Tensor, params: torch.Tensor, bits: torch.Tensor,
                             row_offset: torch.Tensor, dst_idx: torch.Tensor, seg_order: torch.Tensor,
                             seg_ptr: torch.Tensor, dim: int, grad: torch.Tensor,
                             stream: Optional[torch.cuda.Stream] = None) -> None:
    gp, n_rows, ld = _matrix(grad, "grad")
    _check(lib().adaqp_unpack_dequant_add(_dev(packed, torch.uint8, "packed"), packed.numel(),
                                          _dev(params, torch.float32, "params"), _dev(bits, torch.uint8, "bits"),
                                          _dev(row_offset, torch.int64, "row_offset"),
                                          _dev(dst_idx, torch.int32, "dst_idx"), dst_idx.shape[0],
                                          _dev(seg_order, torch.int32, "seg_order"),
                                          _dev(seg_ptr, torch.int64, "seg_ptr"), seg_ptr.shape[0] - 1,
                                          dim, gp, n_rows, ld, _stream(stream)),
           "adaqp_unpack_dequant_add")


def adaqp_spmm_workspace_bytes(n_rows: int, nnz: int, dim: int) -> int:
    out = _i64(0)
    _check(lib().adaqp_spmm_workspace_bytes(n_rows, nnz, dim, ctypes.byref(out)), "adaqp_spmm_workspace_bytes")
    return int(out.value)


def adaqp_spmm_csr(rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor, row_begin: int, row_end: int,
                   H: torch.Tensor, dim: int, out: torch.Tensor, workspace: torch.Tensor,
                   nnz_range: int = -1, stream: Optional[torch.cuda.Stream] = None) -> None:
    hp, n_cols, ldh = _matrix(H, "H")
    op, _, ldo = _matrix(out, "out")
    _check(lib().adaqp_spmm_csr(_dev(rowptr, torch.int64, "rowptr"), _dev(col, torch.int32, "col"),
                                _dev(val, torch.float32, "val"), col.numel(), row_begin, row_end, nnz_range,
                                hp, n_cols, ldh, dim, op, ldo, _dev(workspace, torch.uint8, "workspace"),
                                workspace.numel(), _stream(stream)),
           "adaqp_spmm_csr")


SPMM_NOALLOC_SCRATCH_BYTES = 64 << 20


def adaqp_spmm_csr_noalloc(rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor, row_begin: int, row_end: int,
                           H: torch.Tensor, dim: int, out: torch.Tensor, nnz_range: int = -1,
                           stream: Optional[torch.cuda.Stream] = None) -> None:
    hp, n_cols, ldh = _matrix(H, "H")
    op, _, ldo = _matrix(out, "out")
    _check(lib().adaqp_spmm_csr_noalloc(_dev(rowptr, torch.int64, "rowptr"), _dev(col, torch.int32, "col"),
                                        _dev(val, torch.float32, "val"), col.numel(), row_begin, row_end, nnz_range,
                                        hp, n_cols, ldh, dim, op, ldo, _stream(stream)),
           "adaqp_spmm_csr_noalloc")


SPMM_TILES = 8
SPMM_TILED_SHORT_ROW = 64
SPMM_PANEL_ROWS = 32
SPMM_PANEL_MIN_ROW = 6144
SPMM_PANEL_PIECE_COLS = 1024


def adaqp_plan_spmm_tiles(rowptr_host: np.ndarray, col_host: np.ndarray, row_begin: int, row_end: int,
                          n_cols: int) -> Tuple[np.ndarray, np.ndarray]:
    """Host-only.  Returns (col_bounds int32[9], tile_off int32[rows, 9])."""
    rowptr = np.ascontiguousarray(rowptr_host, dtype=np.int64)
    col = np.ascontiguousarray(col_host, dtype=np.int32)
    bounds = np.zeros(SPMM_TILES + 1, dtype=np.int32)
    off = np.zeros((max(row_end - row_begin, 0), SPMM_TILES + 1), dtype=np.int32)
    _check(lib().adaqp_plan_spmm_tiles(rowptr.ctypes.data, col.ctypes.data, row_begin, row_end, n_cols,
                                       bounds.ctypes.data, off.ctypes.data), "adaqp_plan_spmm_tiles")
    return bounds, off


def adaqp_spmm_tiled_workspace_bytes(n_rows: int, dim: int) -> int:
    out = ctypes.c_int64(0)
    _check(lib().adaqp_spmm_tiled_workspace_bytes(n_rows, dim, ctypes.byref(out)), "adaqp_spmm_tiled_workspace_bytes")
    return int(out.value)


def adaqp_spmm_tiled_pays(n_rows: int, nnz: int) -> bool:
    """Host-only.  True if a row range of this shape is better served by adaqp_spmm_csr_tiled."""
    return bool(lib().adaqp_spmm_tiled_pays(n_rows, nnz))


def adaqp_spmm_tiled_chunk_cols(col_bounds_host: np.ndarray, dim: int) -> int:
    """Host-only.  64 or 128: the feature-chunk width for a plan with these column bounds."""
    b = np.ascontiguousarray(col_bounds_host, dtype=np.int32)
    if b.shape[0] != SPMM_TILES + 1:
        raise ValueError("col_bounds needs SPMM_TILES + 1 entries")
    c = int(lib().adaqp_spmm_tiled_chunk_cols(b.ctypes.data, dim))
    if c == 0:
        raise AdaqpError("adaqp_spmm_tiled_chunk_cols", -1)
    return c


def adaqp_plan_spmm_panels(rowptr_host: np.ndarray, col_host: np.ndarray, val_host: np.ndarray, row_begin: int,
                           row_end: int, n_cols: int, col_bounds_host: np.ndarray,
                           tile_off: Optional[np.ndarray] = None, min_row_len: int = SPMM_PANEL_MIN_ROW,
                           piece_cols: int = SPMM_PANEL_PIECE_COLS, only_if_pays_for_dim: int = 0) -> Optional[dict]:
    """Host-only.  Returns None when no row of the range has min_row_len entries (or, with only_if_pays_for_dim =
    the row width, when adaqp_spmm_panels_pay turns the sized plan down), else a dict of host arrays
    (panel_rows, pcol, palpha, piece, panel_piece_ptr, panel_piece) and sizes (n_rows_taken, n_panels, n_groups,
    n_per_tile, n_panel_pieces).  tile_off (the C-contiguous int32 table of adaqp_plan_spmm_tiles for the same
    range) is changed in place: the rows taken are struck from it."""
    rowptr = np.ascontiguousarray(rowptr_host, dtype=np.int64)
    col = np.ascontiguousarray(col_host, dtype=np.int32)
    val = np.ascontiguousarray(val_host, dtype=np.float32)
    bounds = np.ascontiguousarray(col_bounds_host, dtype=np.int32)
    if bounds.shape[0] != SPMM_TILES + 1:
        raise ValueError("col_bounds needs SPMM_TILES + 1 entries")
    if tile_off is not None:
        if tile_off.dtype != np.int32 or not tile_off.flags.c_contiguous or \
                tile_off.shape != (max(row_end - row_begin, 0), SPMM_TILES + 1):
            raise ValueError("tile_off must be the C-contiguous int32 table of adaqp_plan_spmm_tiles for this range")
    sizes = np.zeros(5, dtype=np.int64)
    args = (rowptr.ctypes.data, col.ctypes.data, val.ctypes.data, row_begin, row_end, n_cols, bounds.ctypes.data,
            min_row_len, piece_cols, sizes.ctypes.data)
    _check(lib().adaqp_plan_spmm_panels(*args, None, None, None, None, None, None, None), "adaqp_plan_spmm_panels")
    taken, n_panels, n_groups, n_per_tile, n_pieces = (int(x) for x in sizes)
    if taken == 0:
        return None
    if only_if_pays_for_dim > 0 and not adaqp_spmm_panels_pay(n_pieces, only_if_pays_for_dim):
        return None
    plan = {
        "n_rows_taken": taken, "n_panels": n_panels, "n_groups": n_groups, "n_per_tile": n_per_tile,
        "n_panel_pieces": n_pieces,
        "panel_rows": np.empty(n_panels * SPMM_PANEL_ROWS, dtype=np.int32),
        "pcol": np.empty((n_groups, 2, 4), dtype=np.int32),
        "palpha": np.empty((n_groups, 64, 4), dtype=np.float32),
        "piece": np.empty((SPMM_TILES, n_per_tile, 2), dtype=np.int32),
        "panel_piece_ptr": np.empty(n_panels + 1, dtype=np.int32),
        "panel_piece": np.empty(n_pieces, dtype=np.int32),
    }
    _check(lib().adaqp_plan_spmm_panels(*args, None if tile_off is None else tile_off.ctypes.data,
                                        plan["panel_rows"].ctypes.data, plan["pcol"].ctypes.data,
                                        plan["palpha"].ctypes.data, plan["piece"].ctypes.data,
                                        plan["panel_piece_ptr"].ctypes.data, plan["panel_piece"].ctypes.data),
           "adaqp_plan_spmm_panels")
    return plan


class DevicePanels:
    """Device copies of a panel plan plus the struct the C calls take.  Keeps the tensors alive."""

    def __init__(self, plan: Optional[dict], device="cuda"):
        self.c = SpmmPanels()
        self.tensors = {}
        self.n_per_tile = 0
        if plan is None:
            return
        for k in ("panel_rows", "pcol", "palpha", "piece", "panel_piece_ptr", "panel_piece"):
            self.tensors[k] = torch.from_numpy(plan[k]).to(device)
        t = self.tensors
        self.n_per_tile = plan["n_per_tile"]
        self.c = SpmmPanels(plan["n_panels"], plan["n_per_tile"], plan["n_groups"], plan["n_panel_pieces"],
                            t["panel_rows"].data_ptr(), t["pcol"].data_ptr(), t["palpha"].data_ptr(),
                            t["piece"].data_ptr(), t["panel_piece_ptr"].data_ptr(), t["panel_piece"].data_ptr())

    def __bool__(self) -> bool:
        return self.c.n_panels > 0


def adaqp_spmm_panels_pay(n_panel_pieces: int, dim: int) -> bool:
    """Host-only.  True if a panel plan of that many pieces is worth launching (it fills enough of the GPU)."""
    return bool(lib().adaqp_spmm_panels_pay(n_panel_pieces, dim))


def adaqp_spmm_panels_workspace_bytes(n_per_tile: int, dim: int) -> int:
    out = ctypes.c_int64(0)
    _check(lib().adaqp_spmm_panels_workspace_bytes(n_per_tile, dim, ctypes.byref(out)),
           "adaqp_spmm_panels_workspace_bytes")
    return int(out.value)


def adaqp_spmm_csr_panels(panels: DevicePanels, row_begin: int, row_end: int, H: torch.Tensor, dim: int,
                          out: torch.Tensor, workspace: torch.Tensor,
                          stream: Optional[torch.cuda.Stream] = None) -> None:
    hp, n_cols, ldh = _matrix(H, "H")
    op, _, ldo = _matrix(out, "out")
    _check(lib().adaqp_spmm_csr_panels(ctypes.byref(panels.c), row_begin, row_end, hp, n_cols, ldh, dim, op, ldo,
                                       _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                       _stream(stream)), "adaqp_spmm_csr_panels")


def adaqp_spmm_csr_tiled(rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor, row_begin: int, row_end: int,
                         H: torch.Tensor, dim: int, out: torch.Tensor, tile_off: torch.Tensor,
                         workspace: torch.Tensor, chunk_cols: int = 0,
                         stream: Optional[torch.cuda.Stream] = None) -> None:
    hp, n_cols, ldh = _matrix(H, "H")
    op, _, ldo = _matrix(out, "out")
    _check(lib().adaqp_spmm_csr_tiled(_dev(rowptr, torch.int64, "rowptr"), _dev(col, torch.int32, "col"),
                                      _dev(val, torch.float32, "val"), col.numel(), row_begin, row_end,
                                      hp, n_cols, ldh, dim, op, ldo, _dev(tile_off, torch.int32, "tile_off"),
                                      chunk_cols, _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                      _stream(stream)), "adaqp_spmm_csr_tiled")


def adaqp_assign_bits(beta_host: np.ndarray, peer_of_slot_host: np.ndarray, n_peers: int, dim: int,
                      group_size: int, lam: float, theta: np.ndarray, gamma: np.ndarray
                      ) -> Tuple[np.ndarray, np.ndarray]:
    """Host-only.  Returns (bits uint8[n], float64[3] = Eq. 9 value, variance, largest pair time)."""
    beta = np.ascontiguousarray(beta_host, dtype=np.float32)
    peer = np.ascontiguousarray(peer_of_slot_host, dtype=np.int32)
    theta = np.ascontiguousarray(theta, dtype=np.float64)
    gamma = np.ascontiguousarray(gamma, dtype=np.float64)
    if theta.shape[0] != n_peers or gamma.shape[0] != n_peers or peer.shape[0] != beta.shape[0]:
        raise ValueError("theta / gamma need n_peers entries, peer_of_slot one per beta")
    bits = np.zeros(beta.shape[0], dtype=np.uint8)
    obj = np.zeros(3, dtype=np.float64)
    _check(lib().adaqp_assign_bits(beta.shape[0], beta.ctypes.data, peer.ctypes.data, n_peers, dim, group_size,
                                   float(lam), theta.ctypes.data, gamma.ctypes.data, bits.ctypes.data,
                                   obj.ctypes.data), "adaqp_assign_bits")
    return bits, obj


def adaqp_plan_slot_of_row(n_rows: int, halo_idx_host: np.ndarray) -> np.ndarray:
    """Host-only.  Returns int32[n_rows]: the slot received into each row, -1 elsewhere."""
    halo = np.ascontiguousarray(halo_idx_host, dtype=np.int32)
    out = np.zeros(n_rows, dtype=np.int32)
    _check(lib().adaqp_plan_slot_of_row(n_rows, halo.shape[0], halo.ctypes.data, out.ctypes.data),
           "adaqp_plan_slot_of_row")
    return out


def adaqp_spmm_csr_packed(rowptr: torch.Tensor, col: torch.Tensor, val: torch.Tensor, row_begin: int, row_end: int,
                          H: torch.Tensor, dim: int, out: torch.Tensor, slot_of_row: torch.Tensor,
                          packed: torch.Tensor, params: torch.Tensor, bits: torch.Tensor, row_offset: torch.Tensor,
                          workspace: torch.Tensor, nnz_range: int = -1,
                          stream: Optional[torch.cuda.Stream] = None) -> None:
    hp, n_cols, ldh = _matrix(H, "H")
    op, _, ldo = _matrix(out, "out")
    _check(lib().adaqp_spmm_csr_packed(_dev(rowptr, torch.int64, "rowptr"), _dev(col, torch.int32, "col"),
                                       _dev(val, torch.float32, "val"), col.numel(), row_begin, row_end, nnz_range,
                                       hp, n_cols, ldh, dim, op, ldo,
                                       _dev(slot_of_row, torch.int32, "slot_of_row"),
                                       _dev(packed, torch.uint8, "packed"), packed.numel(),
                                       _dev(params, torch.float32, "params"), _dev(bits, torch.uint8, "bits"),
                                       _dev(row_offset, torch.int64, "row_offset"), bits.shape[0],
                                       _dev(workspace, torch.uint8, "workspace"), workspace.numel(),
                                       _stream(stream)),
           "adaqp_spmm_csr_packed")


def adaqp_layer_step(desc: LayerDesc) -> None:
    _check(lib().adaqp_layer_step(ctypes.byref(desc)), "adaqp_layer_step")


def adaqp_probe_quantize_pack(feat: torch.Tensor, dim: int, send_idx: torch.Tensor, bits: torch.Tensor,
                              row_offset: torch.Tensor, packed: torch.Tensor, params: torch.Tensor,
                              stream: Optional[torch.cuda.Stream] = None) -> None:
    """Measurement aid (include/adaqp_probe.h): the no-compute twin of adaqp_quantize_pack."""
    fp, n_rows, ld = _matrix(feat, "feat")
    _check(lib().adaqp_probe_quantize_pack(fp, n_rows, ld, dim, _dev(send_idx, torch.int32, "send_idx"),
                                           _dev(bits, torch.uint8, "bits"),
                                           _dev(row_offset, torch.int64, "row_offset"), send_idx.shape[0],
                                           _dev(packed, torch.uint8, "packed"), packed.numel(),
                                           _dev(params, torch.float32, "params"), _stream(stream)),
           "adaqp_probe_quantize_pack")


def adaqp_probe_unpack_dequant_add(packed: torch.Tensor, params: torch.Tensor, bits: torch.Tensor,
                                   row_offset: torch.Tensor, dst_idx: torch.Tensor, seg_order: torch.Tensor,
                                   seg_ptr: torch.Tensor, dim: int, grad: torch.Tensor,
                                   stream: Optional[torch.cuda.Stream] = None) -> None:
    """Measurement aid (include/adaqp_probe.h): the no-compute twin of adaqp_unpack_dequant_add."""
    gp, n_rows, ld = _matrix(grad, "grad")
    _check(lib().adaqp_probe_unpack_dequant_add(_dev(packed, torch.uint8, "packed"), packed.numel(),
                                                _dev(params, torch.float32, "params"),
                                                _dev(bits, torch.uint8, "bits"),
                                                _dev(row_offset, torch.int64, "row_offset"),
                                                _dev(dst_idx, torch.int32, "dst_idx"), dst_idx.shape[0],
                                                _dev(seg_order, torch.int32, "seg_order"),
                                                _dev(seg_ptr, torch.int64, "seg_ptr"), seg_ptr.shape[0] - 1,
                                                dim, gp, n_rows, ld, _stream(stream)),
           "adaqp_probe_unpack_dequant_add")


def adaqp_probe_stream(src: torch.Tensor, dst: torch.Tensor, nbytes: int, write_side: int,
                       stream: Optional[torch.cuda.Stream] = None) -> None:
    """Measurement aid (include/adaqp_probe.h): a plain stream over nbytes bytes of src (write_side 0), of dst
    (1), or of dst read and written back in place (2)."""
    write_side = int(write_side)
    big, small = (dst, src) if write_side else (src, dst)
    if big.numel() * big.element_size() < nbytes or small.numel() * small.element_size() < nbytes // 8 + 4096:
        raise ValueError("adaqp_probe_stream: a buffer is smaller than the stream")
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise TypeError("adaqp_probe_stream needs contiguous device tensors")
    _check(lib().adaqp_probe_stream(src.data_ptr(), dst.data_ptr(), nbytes, write_side, _stream(stream)),
           "adaqp_probe_stream")


def adaqp_probe_xcd_of_workgroup(n_workgroups: int, device="cuda:0",
                                 stream: Optional[torch.cuda.Stream] = None) -> torch.Tensor:
    """Measurement aid (include/adaqp_probe.h): the XCD each workgroup of a 1-D grid runs on (int32 device tensor)."""
    out = torch.full((max(n_workgroups, 1),), -1, dtype=torch.int32, device=device)
    _check(lib().adaqp_probe_xcd_of_workgroup(out.data_ptr(), n_workgroups, _stream(stream)),
           "adaqp_probe_xcd_of_workgroup")
    return out[:n_workgroups]
