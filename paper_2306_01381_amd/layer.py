"""Device-resident state of one partition's layer step: uploads a partition, plans the buffer layout,
allocates buffers / workspaces / streams / events with torch and HIP, and fills an adaqp_layer_desc.

Everything computational happens inside libadaqp; this module only owns memory and handles.
"""
from __future__ import annotations

import ctypes
from typing import Optional

import numpy as np
import torch

from . import binding as B
from .synth import Partition, alpha_sq_stand_in

_hip: Optional[ctypes.CDLL] = None


def _hip_runtime() -> ctypes.CDLL:
    global _hip
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipEventCreateWithFlags.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_uint]
        _hip.hipEventCreateWithFlags.restype = ctypes.c_int
        _hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        _hip.hipEventDestroy.restype = ctypes.c_int
    return _hip


class HipEvent:
    """A raw hipEvent_t (timing disabled) whose handle can be passed through the C ABI."""
    _DISABLE_TIMING = 0x2

    def __init__(self):
        h = ctypes.c_void_p()
        rc = _hip_runtime().hipEventCreateWithFlags(ctypes.byref(h), self._DISABLE_TIMING)
        if rc != 0:
            raise RuntimeError(f"hipEventCreateWithFlags failed: {rc}")
        self.handle = h.value

    def __del__(self):
        try:
            if getattr(self, "handle", None):
                _hip_runtime().hipEventDestroy(self.handle)
        except Exception:
            pass


class SendPlan:
    """Sorted slot order and byte offsets of one direction's messages (host arrays + device copies)."""

    def __init__(self, dim: int, send_idx: np.ndarray, bits: np.ndarray, peer_of_slot: np.ndarray,
                 n_peers: int, halo_idx: Optional[np.ndarray], device, add_segments: bool = False):
        perm, off, pbp = B.adaqp_plan_layout(dim, bits, peer_of_slot, n_peers)
        self.perm, self.row_offset_host, self.peer_byte_ptr = perm, off, pbp
        self.send_idx_host = np.ascontiguousarray(send_idx[perm], dtype=np.int32)
        self.bits_host = np.ascontiguousarray(bits[perm], dtype=np.uint8)
        self.halo_idx_host = None if halo_idx is None or halo_idx.size == 0 else \
            np.ascontiguousarray(halo_idx[perm], dtype=np.int32)
        self.n = int(perm.shape[0])
        self.packed_bytes = int(pbp[-1])
        self.send_idx = torch.from_numpy(self.send_idx_host).to(device)
        self.bits = torch.from_numpy(self.bits_host).to(device)
        self.row_offset = torch.from_numpy(off).to(device)
        self.halo_idx = None if self.halo_idx_host is None else torch.from_numpy(self.halo_idx_host).to(device)
        self.recv_order_host = None if self.halo_idx_host is None else B.adaqp_plan_recv_order(self.halo_idx_host)
        self.recv_order = None if self.recv_order_host is None else torch.from_numpy(self.recv_order_host).to(device)
        # backward receive: slots grouped by destination row
        self.seg_order = self.seg_ptr = None
        if add_segments and self.halo_idx_host is not None:
            order, seg_ptr = B.adaqp_plan_recv_segments(self.halo_idx_host)
            self.seg_order_host, self.seg_ptr_host = order, seg_ptr
            self.seg_order = torch.from_numpy(order).to(device)
            self.seg_ptr = torch.from_numpy(seg_ptr).to(device)


def line_padded(a: np.ndarray, device, pad: bool = True) -> torch.Tensor:
    """Uploads a [n, dim] fp32 matrix into rows whose pitch is a whole number of 128-byte lines (the layout
    the kernels are built for) and returns the [n, dim] view; the padding columns are zero."""
    n, dim = a.shape
    ld = (dim + 31) // 32 * 32 if pad else dim
    buf = torch.zeros((n, ld), dtype=torch.float32, device=device)
    view = buf[:, :dim]
    view.copy_(torch.from_numpy(a))
    return view


class LayerStep:
    def __init__(self, p: Partition, device="cuda:0", seed: int = 0, pad: bool = True, use_recv_order: bool = False,
                 backward_receive: bool = True, trace: bool = True, fused_receive: bool = False,
                 tiled: Optional[bool] = None, panels: Optional[bool] = None, panel_min_row=B.SPMM_PANEL_MIN_ROW,
                 panel_piece_cols: int = B.SPMM_PANEL_PIECE_COLS, streams=None):
        self.p = p
        self.device = torch.device(device)
        dev = self.device
        cfg = p.cfg
        self.dim = cfg.dim
        self.backward = bool(cfg.backward)
        self.seed = seed
        self.use_recv_order = use_recv_order
        self.backward_receive = backward_receive
        self.fused_receive = fused_receive and not self.backward
        self.rowptr = torch.from_numpy(p.rowptr).to(dev)
        self.col = torch.from_numpy(p.col).to(dev)
        self.val = torch.from_numpy(p.val).to(dev)
        self.feat = line_padded(p.feat, dev, pad)
        self.out = line_padded(np.zeros((p.n_rows, cfg.dim), dtype=np.float32), dev, pad)
        self.plan = SendPlan(cfg.dim, p.send_idx, p.bits, p.peer_of_slot, cfg.n_peers, p.halo_idx, dev,
                             add_segments=self.backward)
        n = self.plan.n
        # forward, fused receive: the dependent aggregation reads received rows straight from the receive buffer
        self.slot_of_row = None
        self.set_fused_receive(self.fused_receive)
        nbytes = max(self.plan.packed_bytes, 4)
        self.packed = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        self.params = torch.zeros((max(n, 1), 2), dtype=torch.float32, device=dev)
        # trace for the bit-width assigner: per slot, the sum of squared coefficients the message meets on its
        # target device is an input (the generator supplies a stand-in)
        self.alpha_sq = self.beta = None
        if trace and n > 0:
            self.alpha_sq_host = np.ascontiguousarray(alpha_sq_stand_in(p)[self.plan.perm])
            self.alpha_sq = torch.from_numpy(self.alpha_sq_host).to(dev)
            self.beta = torch.zeros(n, dtype=torch.float32, device=dev)
        self.recv_packed = torch.zeros(nbytes, dtype=torch.uint8, device=dev)
        self.recv_params = torch.zeros((max(n, 1), 2), dtype=torch.float32, device=dev)
        ob, oe = p.overlap_rows
        db, de = p.dependent_rows
        self.overlap_nnz = int(p.rowptr[oe] - p.rowptr[ob])
        self.dependent_nnz = int(p.rowptr[de] - p.rowptr[db])
        # aggregation tiled over the L2 caches: pays when rows are long (every row of feat re-used many times).
        # tiled=None lets the library decide per row range (adaqp_spmm_tiled_pays: mean row length).
        self.tile_off_overlap = self.tile_off_dependent = None
        self.tile_chunk_overlap = self.tile_chunk_dependent = 0
        # within a tiled range, rows with thousands of entries go into dense panels for the matrix cores.
        # panels=None: where the library says the plan fills enough of the GPU (adaqp_spmm_panels_pay); True: always
        self.panels_overlap = self.panels_dependent = B.DevicePanels(None)
        # panel_min_row: one threshold, or one per row range (overlap, dependent)
        min_row_o, min_row_d = panel_min_row if isinstance(panel_min_row, tuple) else (panel_min_row, panel_min_row)
        ws_o = B.adaqp_spmm_workspace_bytes(oe - ob, self.overlap_nnz, cfg.dim)
        ws_d = B.adaqp_spmm_workspace_bytes(de - db, self.dependent_nnz, cfg.dim)
        if pad and tiled is not False:
            if oe > ob and (tiled or B.adaqp_spmm_tiled_pays(oe - ob, self.overlap_nnz)):
                bounds, off = B.adaqp_plan_spmm_tiles(p.rowptr, p.col, ob, oe, p.feat.shape[0])
                if panels is not False:
                    self.panels_overlap = B.DevicePanels(B.adaqp_plan_spmm_panels(
                        p.rowptr, p.col, p.val, ob, oe, p.feat.shape[0], bounds, off, min_row_o, panel_piece_cols,
                        only_if_pays_for_dim=0 if panels else cfg.dim), dev)
                self.tile_off_overlap = torch.from_numpy(off).to(dev)
                self.tile_chunk_overlap = B.adaqp_spmm_tiled_chunk_cols(bounds, cfg.dim)
                # partial sums of the tiled kernel, then the piece sums of the panel kernel (they may run together)
                ws_o = max(ws_o, B.adaqp_spmm_tiled_workspace_bytes(oe - ob, cfg.dim)
                           + B.adaqp_spmm_panels_workspace_bytes(self.panels_overlap.n_per_tile, cfg.dim))
            if de > db and (tiled or B.adaqp_spmm_tiled_pays(de - db, self.dependent_nnz)):
                bounds, off = B.adaqp_plan_spmm_tiles(p.rowptr, p.col, db, de, p.feat.shape[0])
                if panels is not False:
                    self.panels_dependent = B.DevicePanels(B.adaqp_plan_spmm_panels(
                        p.rowptr, p.col, p.val, db, de, p.feat.shape[0], bounds, off, min_row_d, panel_piece_cols,
                        only_if_pays_for_dim=0 if panels else cfg.dim), dev)
                self.tile_off_dependent = torch.from_numpy(off).to(dev)
                self.tile_chunk_dependent = B.adaqp_spmm_tiled_chunk_cols(bounds, cfg.dim)
                ws_d = max(ws_d, B.adaqp_spmm_tiled_workspace_bytes(de - db, cfg.dim)
                           + B.adaqp_spmm_panels_workspace_bytes(self.panels_dependent.n_per_tile, cfg.dim))
        self.ws_overlap = torch.empty(max(ws_o, 256), dtype=torch.uint8, device=dev)
        self.ws_dependent = torch.empty(max(ws_d, 256), dtype=torch.uint8, device=dev)
        # streams=(msg, agg): take over an existing pair.  HIP deals streams to a few hardware queues in turn, so a
        # process that keeps creating streams can end up with a step's two streams on one queue (no overlap)
        self.stream_msg, self.stream_agg = streams if streams is not None else (torch.cuda.Stream(device=dev),
                                                                                  torch.cuda.Stream(device=dev))
        self.event_fork = HipEvent()
        self.event_join = HipEvent()

    def set_fused_receive(self, on: bool) -> None:
        """Forward only.  On: received rows are not de-quantised into feat; the dependent aggregation reads
        them from the receive buffer."""
        self.fused_receive = bool(on) and not self.backward and self.plan.halo_idx_host is not None
        if self.fused_receive and self.slot_of_row is None:
            self.slot_of_row = torch.from_numpy(
                B.adaqp_plan_slot_of_row(self.p.feat.shape[0], self.plan.halo_idx_host)).to(self.device)

    def desc(self, schedule: int) -> B.LayerDesc:
        p, pl = self.p, self.plan
        d = B.LayerDesc()
        d.direction = B.BACKWARD if self.backward else B.FORWARD
        d.schedule = schedule
        d.rowptr_dev, d.col_dev, d.val_dev = self.rowptr.data_ptr(), self.col.data_ptr(), self.val.data_ptr()
        d.nnz = p.nnz
        d.overlap_begin, d.overlap_end = p.overlap_rows
        d.dependent_begin, d.dependent_end = p.dependent_rows
        d.overlap_nnz, d.dependent_nnz = self.overlap_nnz, self.dependent_nnz
        d.feat_dev, d.n_feat_rows, d.ld, d.dim = self.feat.data_ptr(), self.feat.shape[0], self.feat.stride(0), self.dim
        d.out_dev, d.ldo = self.out.data_ptr(), self.out.stride(0)
        d.send_idx_dev, d.bits_dev = pl.send_idx.data_ptr(), pl.bits.data_ptr()
        d.row_offset_dev = pl.row_offset.data_ptr()
        d.halo_idx_dev = None if pl.halo_idx is None else pl.halo_idx.data_ptr()
        d.recv_order_dev = pl.recv_order.data_ptr() if (self.use_recv_order and pl.recv_order is not None
                                                        and not self.backward) else None
        d.slot_of_row_dev = self.slot_of_row.data_ptr() if self.fused_receive else None
        d.tile_off_overlap_dev = None if self.tile_off_overlap is None else self.tile_off_overlap.data_ptr()
        d.tile_chunk_overlap, d.tile_chunk_dependent = self.tile_chunk_overlap, self.tile_chunk_dependent
        d.tile_off_dependent_dev = None if (self.tile_off_dependent is None or self.fused_receive) \
            else self.tile_off_dependent.data_ptr()
        if d.tile_off_overlap_dev:
            d.panels_overlap = self.panels_overlap.c
        if d.tile_off_dependent_dev:
            d.panels_dependent = self.panels_dependent.c
        if self.backward and self.backward_receive and pl.seg_order is not None:
            d.recv_seg_order_dev, d.recv_seg_ptr_dev = pl.seg_order.data_ptr(), pl.seg_ptr.data_ptr()
            d.n_recv_seg = pl.seg_ptr.shape[0] - 1
        d.n_send, d.seed = pl.n, self.seed
        d.packed_dev, d.params_dev = self.packed.data_ptr(), self.params.data_ptr()
        if self.alpha_sq is not None:
            d.alpha_sq_dev, d.beta_dev = self.alpha_sq.data_ptr(), self.beta.data_ptr()
        d.recv_packed_dev, d.recv_params_dev = self.recv_packed.data_ptr(), self.recv_params.data_ptr()
        d.packed_bytes = pl.packed_bytes
        d.workspace_overlap_dev, d.workspace_overlap_bytes = self.ws_overlap.data_ptr(), self.ws_overlap.numel()
        d.workspace_dependent_dev, d.workspace_dependent_bytes = self.ws_dependent.data_ptr(), self.ws_dependent.numel()
        d.stream_msg = self.stream_msg.cuda_stream
        d.stream_agg = self.stream_agg.cuda_stream
        d.event_fork, d.event_join = self.event_fork.handle, self.event_join.handle
        return d

    def run(self, schedule: int = B.ISOLATED) -> None:
        """Enqueues one layer step; synchronise stream_msg to wait for it."""
        B.adaqp_layer_step(self.desc(schedule))

    def synchronize(self) -> None:
        self.stream_msg.synchronize()
        self.stream_agg.synchronize()
