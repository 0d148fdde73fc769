#!/usr/bin/env python3
"""Benchmark of the quantised message path on one MI355X.

A step is one adaqp_layer_step over one synthetic partition: quantise + pack the send rows, loop the buffers
back (the exchange itself is out of scope), unpack + de-quantise into the halo rows, aggregate the central
rows on a second stream and the marginal rows after the de-quantisation (backward: the transposed graph, then
quantise the halo-gradient rows, then add the received gradients).  Inputs are resident in HBM before the timed
region starts.

Prints ONE JSON line.  The headline (`value`, `ms_per_step`, `kernels`, `roofline`, `cpu_baseline`) is workload c1,
the configuration the metric is quoted on; `configs` holds the same measurements, shortened, for c2, c3 and c4.
`value` is whole-step throughput in aggregated edges per second; the codec kernels' GB/s and fractions of the
8 TB/s HBM peak are in `kernels`, next to the floor of their own access pattern (a no-compute twin of the kernel)
and to a plain stream of the same size; `roofline` describes the dominant kernel against the limit that binds it;
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
GATHER_RATE_GBPS = 25000.0      # 16-byte-per-lane gather out of L2, every XCD on its own 4 MB: measured on MI355X
MFMA_FP32_PEAK_TFLOPS = 157.3   # dense fp32 on the matrix cores
FMA_RATE_PER_S = 78.65e12       # fp32 vector FMAs per second (157.3 TFLOP/s)
METRIC = "quantize+pack / unpack+dequant GB/s, halo SpMM edges/s, % HBM peak, 1xMI355X"
OTHER_CONFIGS = ("c2", "c3", "c4")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="c1", help="headline workload, c0..c4 (c1 is the one the metric is quoted on)")
    ap.add_argument("--only-headline", action="store_true",
                    help="skip the `configs` block (c2, c3, c4 after the headline): for profiling one workload")
    ap.add_argument("--schedule", default=None, choices=["serial", "isolated", "free"],
                    help="schedule of the timed steps.  Default: isolated (Fig. 7: the central rows start on the second "
                         "stream once quantisation is done).  On workload c1 that pairs a panel kernel with a tiled "
                         "kernel on the two streams; elsewhere (one aggregation kernel per row range, no transfer to "
                         "hide on one GPU) it is worth 0-4 %.  The figures under `kernels` are always timed one "
                         "launch at a time")
    ap.add_argument("--kernel-reps", type=int, default=20, help="launches per kernel in the breakdown")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-panels", action="store_true",
                    help="keep the longest rows in the L2-tiled kernel instead of dense panels on the matrix cores")
    ap.add_argument("--no-tiled", action="store_true",
                    help="aggregate with the merge-path kernel even where the L2-tiled kernel would be chosen")
    ap.add_argument("--calibrate", action="store_true",
                    help="also launch a plain elementwise kernel of known size (reads and writes 256 MiB): the "
                         "reference dispatch that scales the FETCH_SIZE / WRITE_SIZE counters of a --pmc run")
    ap.add_argument("--cpu-budget-s", type=float, default=15.0, help="oracle time for the headline workload")
    ap.add_argument("--cpu-budget-other-s", type=float, default=5.0, help="oracle time for each of c2, c3, c4")
    return ap.parse_args()


def codec_bytes(dim, bits_sorted, B):
    """Algorithmic bytes of the two codec kernels: the row (4*dim), its packed form, (Z, S), and the per-slot
    index entries (send_idx 4 + bits 1 + row_offset 8; the receive side also reads halo_idx 4)."""
    import numpy as np
    strides = np.array([B.adaqp_row_stride(dim, int(b)) for b in (2, 4, 8)], dtype=np.int64)
    cnt = np.array([(bits_sorted == b).sum() for b in (2, 4, 8)], dtype=np.int64)
    n = int(cnt.sum())
    packed = int((cnt * strides).sum())
    q = n * 4 * dim + packed + n * 8 + n * 13
    d = packed + n * 8 + n * 17 + n * 4 * dim
    return q, d


def spmm_bytes(nnz, n_rows, dim):
    """Algorithmic bytes of the aggregation: per entry (col 4 + alpha 4 + one neighbour row 4*dim), per output
    row 4*dim written."""
    return nnz * (8 + 4 * dim) + n_rows * 4 * dim


def event_time_ms(stream, fn, reps):
    """Average duration of fn() over `reps` back-to-back launches, from HIP events recorded on `stream`."""
    import torch
    start = torch.cuda.Event(enable_timing=True)
    stop = torch.cuda.Event(enable_timing=True)
    fn(0)
    stream.synchronize()
    start.record(stream)
    for i in range(reps):
        fn(i + 1)
    stop.record(stream)
    stop.synchronize()
    return start.elapsed_time(stop) / reps


def per_launch_ms(stream, fn, reps):
    """Duration of each of `reps` launches from its own pair of HIP events.  Returns (median, min) in ms."""
    import torch
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    fn(0)
    stream.synchronize()
    for i, (a, b) in enumerate(pairs):
        a.record(stream)
        fn(i + 1)
        b.record(stream)
    stream.synchronize()
    t = sorted(a.elapsed_time(b) for a, b in pairs)
    return t[len(t) // 2], t[0]


def host_cpu():
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return model, os.cpu_count()


def cpu_baseline(p, plan, budget_s, B):
    """The oracle as it stands, single thread, on a bounded sample: the whole codec (all slots) plus the
    aggregation of a contiguous block of rows sized to the time budget."""
    import numpy as np
    import oracle
    cfg = p.cfg
    dim = cfg.dim
    t0 = time.perf_counter()
    src = p.feat
    idx = plan.send_idx_host
    if cfg.backward:                       # the rows that are quantised are aggregation results: use dY rows as stand-ins
        idx = (idx % p.feat.shape[0]).astype(np.int32)
    packed, params, _ = oracle.quantize_pack(src, dim, idx, plan.bits_host, plan.row_offset_host, 1,
                                             plan.packed_bytes)
    t_q = time.perf_counter() - t0
    t0 = time.perf_counter()
    dst = np.empty((plan.n, dim), dtype=np.float32)
    oracle.unpack_dequant(packed, params, plan.bits_host, plan.row_offset_host,
                          np.arange(plan.n, dtype=np.int32), dim, dst)
    t_d = time.perf_counter() - t0
    # probe the aggregation rate on a few rows, then size the sample
    n_rows = p.n_rows
    probe_rows = min(n_rows, 64)
    t0 = time.perf_counter()
    oracle.spmm_csr(p.rowptr, p.col, p.val, 0, probe_rows, p.feat, dim, want64=True)
    t_probe = time.perf_counter() - t0
    probe_edges = int(p.rowptr[probe_rows] - p.rowptr[0])
    rate = max(probe_edges, 1) / max(t_probe, 1e-6)
    want_edges = int(min(p.nnz, rate * max(budget_s - t_q - t_d, 2.0)))
    row_end = int(np.searchsorted(p.rowptr, p.rowptr[0] + want_edges, side="right") - 1)
    row_end = max(min(row_end, n_rows), min(n_rows, 1))
    t0 = time.perf_counter()
    oracle.spmm_csr(p.rowptr, p.col, p.val, 0, row_end, p.feat, dim, want64=True)
    t_s = time.perf_counter() - t0
    edges = int(p.rowptr[row_end] - p.rowptr[0])
    share = edges / max(p.nnz, 1)
    t_step = t_s + (t_q + t_d) * share
    qb, db = codec_bytes(dim, plan.bits_host, B)
    return {
        "value": edges / t_step, "unit": "edges/s", "cores": 1, "kind": "oracle",
        "sample": f"all {plan.n} slots quantised+packed ({t_q:.2f}s) and unpacked+de-quantised ({t_d:.2f}s), "
                  f"aggregation of rows [0,{row_end}) = {edges} of {p.nnz} edges ({t_s:.2f}s); codec time "
                  f"pro-rated by the edge share",
        "quantize_pack_GBps": qb / t_q / 1e9, "unpack_dequant_GBps": db / t_d / 1e9,
        "spmm_edges_per_s": edges / t_s,
        "host_cpu": host_cpu()[0], "host_logical_cpus": host_cpu()[1],
    }


def codec_entry(t, tw, t_med, t_min, nbytes, extra=None):
    e = {"ms": t, "GBps": nbytes / t / 1e6, "frac_hbm": nbytes / t / 1e6 / HBM_PEAK_GBPS,
         "ms_warm": tw, "GBps_warm": nbytes / tw / 1e6, "frac_hbm_warm": nbytes / tw / 1e6 / HBM_PEAK_GBPS,
         "bytes": nbytes, "ms_median_single_launch": t_med, "ms_min_single_launch": t_min}
    if extra:
        e.update(extra)
    return e


_STREAMS = {}


def measure_config(name, args, headline, B, torch, np):
    """All measurements of one workload.  `headline`: also the graph replay, the fused-receive variant, the merge-path
    comparison and the one-launch aggregation."""
    from paper_2306_01381_amd.layer import LayerStep, line_padded
    from paper_2306_01381_amd.synth import config_by_name, make_partition

    cfg = config_by_name(name)
    t0 = time.perf_counter()
    p = make_partition(cfg)
    t_gen = time.perf_counter() - t0
    dev = "cuda:0"
    t0 = time.perf_counter()
    # every workload of the run on the same pair of streams (a fresh pair per workload could land on one hardware queue)
    L = LayerStep(p, dev, seed=2306, tiled=False if args.no_tiled else None, panels=False if args.no_panels else None,
                  streams=_STREAMS.get("pair"))
    _STREAMS["pair"] = (L.stream_msg, L.stream_agg)
    torch.cuda.synchronize()
    t_plan = time.perf_counter() - t0
    schedule = args.schedule if headline else None
    pairs = (not cfg.backward and L.tile_off_overlap is not None and L.tile_off_dependent is not None
             and bool(L.panels_overlap or L.panels_dependent))
    if schedule is None:
        schedule = "isolated"
    sched = {"serial": B.SERIAL, "isolated": B.ISOLATED, "free": B.FREE}

    def timed_steps(sch, steps, warmup):
        desc = L.desc(sch)
        for _ in range(warmup):
            B.adaqp_layer_step(desc)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            B.adaqp_layer_step(desc)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) * 1e3 / steps

    ms_per_step = timed_steps(sched[schedule], args.steps, args.warmup)
    by_schedule = {}
    for s_name, s in sched.items():
        by_schedule[s_name] = ms_per_step if s_name == schedule else timed_steps(s, max(3, args.steps // 4), 1)
    # a two-stream schedule that does not beat the serial one has lost its overlap (the two streams share a hardware
    # queue): say so instead of printing the serial time under its name.  Only where the step pairs the panel and
    # the tiled kernel (14 % to win); with one aggregation kernel per row range there is no transfer to hide on one
    # GPU and the two-stream schedules stay within +-3 % of the serial one
    overlap_lost = pairs and schedule != "serial" and ms_per_step > 0.97 * by_schedule["serial"]

    fused = None
    ms_graph = None
    if headline:
        if not cfg.backward:
            # variant (not the headline): the dependent aggregation de-quantises received rows in registers, straight
            # from the receive buffer, instead of reading rows that a separate kernel wrote into the feature matrix
            L.set_fused_receive(True)
            ms_fused = timed_steps(sched[schedule], max(3, args.steps // 2), 1)
            L.set_fused_receive(False)
            timed_steps(sched[schedule], 1, 0)          # leaves feat's halo rows as the plain step writes them
            fused = {"ms_per_step": ms_fused, "value": p.nnz / ms_fused * 1e3, "unit": "edges/s",
                     "note": "adaqp_spmm_csr_packed for the marginal rows, no adaqp_unpack_dequant launch; "
                             "output bit-identical to the step with the untiled aggregation"}
        # the same step captured into a HIP graph and replayed (no per-launch host work between the kernels)
        desc_g = L.desc(sched[schedule])
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=L.stream_msg):
            B.adaqp_layer_step(desc_g)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t_g = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms_graph = (time.perf_counter() - t_g) * 1e3 / args.steps
        del graph

    # ---- per-kernel breakdown: the same launches the step makes, each alone on its stream, HIP events ----
    dim = cfg.dim
    pl = L.plan
    reps = args.kernel_reps
    qbytes, dbytes = codec_bytes(dim, pl.bits_host, B)
    st = L.stream_msg
    kernels = {}
    # cold protocol for the codec: rotate over enough copies of the operand that the rows a launch touches
    # (n_send rows, not the whole matrix) cannot survive in the 256 MB last-level cache until their next use
    src = L.out if cfg.backward else L.feat
    touched = max(1, pl.n * dim * 4)
    n_copies = int(min(12, max(2, -(-640_000_000 // touched))))
    srcs = [src] + [line_padded(src.cpu().numpy(), dev) for _ in range(n_copies - 1)]
    packs = [L.packed] + [torch.zeros_like(L.packed) for _ in range(n_copies - 1)]
    pars = [L.params] + [torch.empty_like(L.params) for _ in range(n_copies - 1)]
    torch.cuda.synchronize()
    creps = max(reps, 50)                       # the codec kernels are short: 50 launches cost a millisecond

    def q_cold(i):
        k = i % n_copies
        B.adaqp_quantize_pack(srcs[k], dim, pl.send_idx, pl.bits, pl.row_offset, 2306, packs[k], pars[k], stream=st)

    def q_warm(i):
        B.adaqp_quantize_pack(srcs[0], dim, pl.send_idx, pl.bits, pl.row_offset, 2306, packs[0], pars[0], stream=st)

    def q_floor(i):
        k = i % n_copies
        B.adaqp_probe_quantize_pack(srcs[k], dim, pl.send_idx, pl.bits, pl.row_offset, packs[k], pars[k], stream=st)

    # plain streams of the same size, out of / into the same buffers (the rows of the send / receive block)
    row_bytes = (pl.n * dim * 4) // 16 * 16
    small = [torch.empty(row_bytes // 8 + 4096, dtype=torch.uint8, device=dev) for _ in range(n_copies)]
    flat = [s_._base if s_._base is not None else s_ for s_ in srcs]

    def stream_read(i):
        k = i % n_copies
        B.adaqp_probe_stream(flat[k], small[k], row_bytes, False, stream=st)

    def stream_write(i):
        k = i % n_copies
        B.adaqp_probe_stream(small[k], flat[k], row_bytes, True, stream=st)

    t = event_time_ms(st, q_cold, creps)
    tw = event_time_ms(st, q_warm, creps)
    t_med, t_min = per_launch_ms(st, q_cold, creps)
    t_floor = event_time_ms(st, q_floor, creps)
    t_sr = event_time_ms(st, stream_read, creps)
    kernels["quantize_pack"] = codec_entry(t, tw, t_med, t_min, qbytes, {
        "cold_copies": n_copies, "launches": creps,
        "floor_no_compute_twin": {"ms": t_floor, "frac_hbm": qbytes / t_floor / 1e6 / HBM_PEAK_GBPS,
                                  "kernel_over_floor": t / t_floor,
                                  "note": "adaqp_probe_quantize_pack: same grid, index loads, row loads and stores, "
                                          "no generator / reduction / codes"},
        "stream_of_same_size": {"ms": t_sr, "frac_hbm": row_bytes * 1.125 / t_sr / 1e6 / HBM_PEAK_GBPS,
                                "note": "adaqp_probe_stream: the row bytes read front to back (non-temporal loads, "
                                        "2 KiB per wave), an eighth of them written"}})
    for k in range(n_copies):           # every copy holds valid packed data
        q_cold(k)
    st.synchronize()
    t_sw = event_time_ms(st, stream_write, creps)
    stream_w = {"ms": t_sw, "frac_hbm": row_bytes * 1.125 / t_sw / 1e6 / HBM_PEAK_GBPS,
                "note": "adaqp_probe_stream: the row bytes written front to back (non-temporal stores, 4 KiB per "
                        "wave), an eighth of them read"}
    if not cfg.backward:
        def d_cold(i):
            k = i % n_copies
            B.adaqp_unpack_dequant(packs[k], pars[k], pl.bits, pl.row_offset, pl.halo_idx, dim, srcs[k],
                                   order=(pl.recv_order if L.use_recv_order else None), stream=st)

        def d_warm(i):
            B.adaqp_unpack_dequant(packs[0], pars[0], pl.bits, pl.row_offset, pl.halo_idx, dim, srcs[0],
                                   order=(pl.recv_order if L.use_recv_order else None), stream=st)

        t = event_time_ms(st, d_cold, creps)
        tw = event_time_ms(st, d_warm, creps)
        t_med, t_min = per_launch_ms(st, d_cold, creps)
        kernels["unpack_dequant"] = codec_entry(t, tw, t_med, t_min, dbytes,
                                                {"launches": creps, "stream_of_same_size": stream_w})
    else:
        # backward receive: the received buffer is de-quantised and added to the local rows it targets
        n_seg = pl.seg_ptr.shape[0] - 1
        strides = {b: B.adaqp_row_stride(dim, b) for b in (2, 4, 8)}
        abytes = int(sum(strides[int(b)] for b in pl.bits_host)) + pl.n * (8 + 17) + n_seg * (8 * dim + 8)

        def a_cold(i):
            k = i % n_copies
            B.adaqp_unpack_dequant_add(packs[k], pars[k], pl.bits, pl.row_offset, pl.halo_idx, pl.seg_order,
                                       pl.seg_ptr, dim, srcs[k], stream=st)

        def a_warm(i):
            B.adaqp_unpack_dequant_add(packs[0], pars[0], pl.bits, pl.row_offset, pl.halo_idx, pl.seg_order,
                                       pl.seg_ptr, dim, srcs[0], stream=st)

        def a_floor(i):
            k = i % n_copies
            B.adaqp_probe_unpack_dequant_add(packs[k], pars[k], pl.bits, pl.row_offset, pl.halo_idx, pl.seg_order,
                                             pl.seg_ptr, dim, srcs[k], stream=st)

        upd_bytes = (n_seg * dim * 4) // 16 * 16

        def stream_update(i):
            k = i % n_copies
            B.adaqp_probe_stream(small[k], flat[k], upd_bytes, 2, stream=st)

        t = event_time_ms(st, a_cold, creps)
        tw = event_time_ms(st, a_warm, creps)
        t_med, t_min = per_launch_ms(st, a_cold, creps)
        extra = {"rows": n_seg, "messages": pl.n, "launches": creps}
        if dim % 32 == 0 and dim <= 512:
            t_floor = event_time_ms(st, a_floor, creps)     # leaves meaningless bits in the rows: timed last
            extra["floor_no_compute_twin"] = {
                "ms": t_floor, "frac_hbm": abytes / t_floor / 1e6 / HBM_PEAK_GBPS, "kernel_over_floor": t / t_floor,
                "note": "adaqp_probe_unpack_dequant_add: same grid, index loads, row and packed-word loads and row "
                        "stores, no decoding / adding"}
        t_su = event_time_ms(st, stream_update, creps)
        extra["stream_of_same_size"] = {
            "ms": t_su, "frac_hbm": upd_bytes * 2.125 / t_su / 1e6 / HBM_PEAK_GBPS,
            "note": "adaqp_probe_stream: as many row bytes read front to back and written back in place "
                    "(non-temporal loads and stores, 4 KiB per wave), an eighth of them read beside"}
        kernels["unpack_dequant_add"] = codec_entry(t, tw, t_med, t_min, abytes, extra)
    del srcs, packs, pars, small, flat
    # the stream probes wrote into the step's own operand (copy 0): put the inputs back before the aggregation is timed
    if cfg.backward:
        timed_steps(sched["serial"], 1, 0)
    else:
        L.feat.copy_(torch.from_numpy(p.feat))
        timed_steps(sched["serial"], 1, 0)

    (ob, oe), (db_, de) = p.overlap_rows, p.dependent_rows

    # the same launches the step makes: tiled over the L2 caches where LayerStep planned tiles, else merge-path
    def spmm_overlap(i):
        if L.tile_off_overlap is not None:
            B.adaqp_spmm_csr_tiled(L.rowptr, L.col, L.val, ob, oe, L.feat, dim, L.out, L.tile_off_overlap,
                                   L.ws_overlap, chunk_cols=L.tile_chunk_overlap, stream=st)
            if L.panels_overlap:
                B.adaqp_spmm_csr_panels(L.panels_overlap, ob, oe, L.feat, dim, L.out, L.ws_overlap, stream=st)
        else:
            B.adaqp_spmm_csr(L.rowptr, L.col, L.val, ob, oe, L.feat, dim, L.out, L.ws_overlap,
                             nnz_range=L.overlap_nnz, stream=st)

    def spmm_dependent(i):
        if L.tile_off_dependent is not None:
            B.adaqp_spmm_csr_tiled(L.rowptr, L.col, L.val, db_, de, L.feat, dim, L.out, L.tile_off_dependent,
                                   L.ws_dependent, chunk_cols=L.tile_chunk_dependent, stream=st)
            if L.panels_dependent:
                B.adaqp_spmm_csr_panels(L.panels_dependent, db_, de, L.feat, dim, L.out, L.ws_dependent, stream=st)
        else:
            B.adaqp_spmm_csr(L.rowptr, L.col, L.val, db_, de, L.feat, dim, L.out, L.ws_dependent,
                             nnz_range=L.dependent_nnz, stream=st)

    def spmm_merge_both(i):
        B.adaqp_spmm_csr(L.rowptr, L.col, L.val, ob, oe, L.feat, dim, L.out, L.ws_overlap,
                         nnz_range=L.overlap_nnz, stream=st)
        B.adaqp_spmm_csr(L.rowptr, L.col, L.val, db_, de, L.feat, dim, L.out, L.ws_dependent,
                         nnz_range=L.dependent_nnz, stream=st)

    tiled_both = L.tile_off_overlap is not None and L.tile_off_dependent is not None
    sreps = max(3, min(reps, int(2000 / max(ms_per_step, 0.05))))
    t_o = event_time_ms(st, spmm_overlap, sreps)
    t_d = event_time_ms(st, spmm_dependent, sreps)
    b_o = spmm_bytes(L.overlap_nnz, oe - ob, dim)
    b_d = spmm_bytes(L.dependent_nnz, de - db_, dim)
    names = ("spmm_local_rows", "spmm_halo_rows") if cfg.backward else ("spmm_central", "spmm_marginal")
    kernels[names[0]] = {"ms": t_o, "edges": L.overlap_nnz, "edges_per_s": L.overlap_nnz / t_o * 1e3,
                         "GBps_primary": b_o / t_o / 1e6, "pct_hbm_primary": 100 * b_o / t_o / 1e6 / HBM_PEAK_GBPS}
    kernels[names[1]] = {"ms": t_d, "edges": L.dependent_nnz, "edges_per_s": L.dependent_nnz / t_d * 1e3,
                         "GBps_primary": b_d / t_d / 1e6, "pct_hbm_primary": 100 * b_d / t_d / 1e6 / HBM_PEAK_GBPS}
    # where panels take the longest rows: the two kernels of each range on their own
    deg = np.diff(p.rowptr)
    panel_parts = {}
    panel_table_bytes = 0
    for tag, pan, rb, re, ws, off_dev, chunk in (
            (names[0], L.panels_overlap, ob, oe, L.ws_overlap, L.tile_off_overlap, L.tile_chunk_overlap),
            (names[1], L.panels_dependent, db_, de, L.ws_dependent, L.tile_off_dependent, L.tile_chunk_dependent)):
        if not pan:
            continue
        panel_table_bytes += sum(int(t_.numel() * t_.element_size()) for t_ in pan.tensors.values())
        rows_p = pan.tensors["panel_rows"].cpu().numpy()
        rows_p = rows_p[rows_p >= 0]
        t_p = event_time_ms(st, lambda i: B.adaqp_spmm_csr_panels(pan, rb, re, L.feat, dim, L.out, ws, stream=st), sreps)
        t_t = event_time_ms(st, lambda i: B.adaqp_spmm_csr_tiled(L.rowptr, L.col, L.val, rb, re, L.feat, dim, L.out,
                                                                 off_dev, ws, chunk_cols=chunk, stream=st), sreps)
        wdim = (dim + 31) // 32 * 32            # the kernel multiplies whole tiles of 32 feature columns
        panel_parts[tag] = {"panel_rows": int(rows_p.size), "panel_edges": int(deg[rows_p].sum()),
                            "panels": int(pan.c.n_panels), "panel_columns_padded": int(pan.c.n_groups) * 8,
                            "ms_panels": t_p, "ms_tiled_other_rows": t_t,
                            "mfma_flops_executed": 2.0 * 32 * int(pan.c.n_groups) * 8 * wdim}
        kernels[tag]["panels"] = panel_parts[tag]
    tiled = L.tile_off_overlap is not None or L.tile_off_dependent is not None
    if headline:
        # the whole row range in one launch (what a step without the central / marginal split would run)
        all_rows = p.n_rows
        if tiled_both:
            bounds_all, off_all = B.adaqp_plan_spmm_tiles(p.rowptr, p.col, 0, all_rows, p.feat.shape[0])
            panels_all = B.DevicePanels(None)
            if not args.no_panels:
                panels_all = B.DevicePanels(B.adaqp_plan_spmm_panels(p.rowptr, p.col, p.val, 0, all_rows,
                                                                     p.feat.shape[0], bounds_all, off_all), dev)
            off_all_dev = torch.from_numpy(off_all).to(dev)
            chunk_all = B.adaqp_spmm_tiled_chunk_cols(bounds_all, dim)
            ws_all = torch.empty(max(B.adaqp_spmm_tiled_workspace_bytes(all_rows, dim),
                                     B.adaqp_spmm_panels_workspace_bytes(panels_all.n_per_tile, dim)),
                                 dtype=torch.uint8, device=dev)

            def spmm_all(i):
                B.adaqp_spmm_csr_tiled(L.rowptr, L.col, L.val, 0, all_rows, L.feat, dim, L.out, off_all_dev, ws_all,
                                       chunk_cols=chunk_all, stream=st)
                if panels_all:
                    B.adaqp_spmm_csr_panels(panels_all, 0, all_rows, L.feat, dim, L.out, ws_all, stream=st)
        else:
            ws_all = torch.empty(max(B.adaqp_spmm_workspace_bytes(all_rows, p.nnz, dim), 256), dtype=torch.uint8,
                                 device=dev)

            def spmm_all(i):
                B.adaqp_spmm_csr(L.rowptr, L.col, L.val, 0, all_rows, L.feat, dim, L.out, ws_all, nnz_range=p.nnz,
                                 stream=st)
        t_all = event_time_ms(st, spmm_all, sreps)
        kernels["spmm_all_rows_one_launch"] = {"ms": t_all, "edges": p.nnz, "edges_per_s": p.nnz / t_all * 1e3,
                                               "kernel": ("tiled + panels" if panel_parts else "tiled") if tiled_both
                                               else "merge-path"}
        del ws_all
        if tiled:
            t_m = event_time_ms(st, spmm_merge_both, max(3, sreps // 2))
            kernels["spmm_merge_path_both_launches"] = {"ms": t_m, "edges_per_s": p.nnz / t_m * 1e3,
                                                        "note": "the untiled kernel on the same rows, for comparison"}

    # ---- roofline of the dominant kernel, against the limit that binds it ----
    # Floors of the whole aggregation: what has to cross the HBM interface at least (every entry, every row of H that
    # is referenced and every output row once), the gather of one neighbour row per entry at the rate a gather
    # kernel reaches out of L2 on this part (measured with a scratch kernel: 25 TB/s when each XCD's working set
    # fits its L2), the fp32 FMA rate.
    touched_cols = int(np.count_nonzero(np.bincount(p.col, minlength=p.feat.shape[0])))
    compulsory = p.nnz * 8 + touched_cols * 4 * dim + p.n_rows * 4 * dim
    t_both = t_o + t_d
    t_ceiling = max(compulsory / HBM_PEAK_GBPS / 1e6, p.nnz * 4 * dim / GATHER_RATE_GBPS / 1e6,
                    p.nnz * dim / FMA_RATE_PER_S * 1e3)
    ceilings = {"compulsory_bytes_both_launches": compulsory,
                "frac_hbm_compulsory": compulsory / t_both / 1e6 / HBM_PEAK_GBPS,
                "gather_rate_GBps": GATHER_RATE_GBPS, "fma_rate_per_s": FMA_RATE_PER_S,
                "t_ceiling_ms": t_ceiling, "t_ceiling_over_t": t_ceiling / t_both}
    primary_gbps = (b_o + b_d) / t_both / 1e6
    if panel_parts:
        # most of the step's time is in the panel kernel: a dense product on the fp32 matrix cores
        t_p = sum(v["ms_panels"] for v in panel_parts.values())
        launches = len(panel_parts)
        executed = sum(v["mfma_flops_executed"] for v in panel_parts.values())
        useful = sum(2.0 * v["panel_edges"] * dim for v in panel_parts.values())
        fetched = sum(v["panel_columns_padded"] for v in panel_parts.values()) + \
            p.nnz - sum(v["panel_edges"] for v in panel_parts.values())
        ceilings["with_panels"] = {
            "neighbour_rows_fetched": fetched, "t_gather_ms": fetched * 4 * dim / GATHER_RATE_GBPS / 1e6,
            "t_mfma_executed_ms": executed / MFMA_FP32_PEAK_TFLOPS / 1e9,
            "note": "floors of the panel + tiled pair: its gather at the L2 rate, its matrix-core work at the "
                    "fp32 MFMA peak; the two overlap at best"}
        roofline = {
            "kernel": "spmm_panel_kernel", "bound": "mfma", "dtype": "f32",
            "achieved": useful / t_p / 1e9, "peak": MFMA_FP32_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": useful / t_p / 1e9 / MFMA_FP32_PEAK_TFLOPS, "traffic": None,
            "launches_per_step": launches, "avg_launch_ms": t_p / launches,
            "algorithmic_flops_per_launch": useful / launches,
            "executed": {"TFLOPs": executed / t_p / 1e9, "frac": executed / t_p / 1e9 / MFMA_FP32_PEAK_TFLOPS,
                         "panel_density": sum(v["panel_edges"] for v in panel_parts.values())
                         / (32.0 * sum(v["panel_columns_padded"] for v in panel_parts.values())),
                         "note": "counts the zeros of the dense panels and the padding of dim to whole tiles of 32 columns"},
            "binding_limit": "the fp32 matrix cores and the gather that feeds them: each neighbour row is fetched once "
                             "per 32-row panel (out of the XCD's L2) and multiplied with the panel's dense "
                             "coefficient table; `frac` counts the method's own multiply-adds (2 * entries * dim)"}
    else:
        alg = (b_o + b_d) / 2
        avg_ms = t_both / 2
        frac_hbm = primary_gbps / HBM_PEAK_GBPS
        roofline = {
            "kernel": "spmm_tiled_kernel" if tiled else "spmm_merge_kernel",
            "bound": "hbm" if frac_hbm <= 1.0 else "l2",
            "achieved": primary_gbps, "peak": HBM_PEAK_GBPS if frac_hbm <= 1.0 else GATHER_RATE_GBPS, "unit": "GB/s",
            "frac": frac_hbm if frac_hbm <= 1.0 else primary_gbps / GATHER_RATE_GBPS, "traffic": None,
            "launches_per_step": 2, "avg_launch_ms": avg_ms, "algorithmic_bytes_per_launch": alg,
            "binding_limit": ("the path behind L2 (fabric / Infinity Cache / HBM) for the neighbour rows that miss L2"
                              if frac_hbm <= 1.0 else
                              "the CUs' gather rate out of L2 (25 TB/s measured on this part with a gather kernel, not "
                              "a published peak): most neighbour rows hit in L2 or the Infinity Cache, so the "
                              "algorithmic bytes exceed what HBM alone could deliver")}
    roofline["pct_hbm_primary"] = 100 * primary_gbps / HBM_PEAK_GBPS
    roofline["whole_aggregation"] = {"GBps_primary": primary_gbps, "ms": t_both}
    roofline["ceilings"] = ceilings
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):
        # bytes behind L2 per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this benchmark; not measured
        # in this run: the entry names the commit it was taken at
        tf = json.load(open(traffic_file))
        entry = tf.get(cfg.name, {}).get(roofline["kernel"])
        if entry:
            roofline["traffic"] = entry["fetch"] + entry["write"]
            roofline["traffic_detail"] = dict(entry, measured_at=tf.get("measured_at", "unknown"),
                                              file="profiles/hbm_traffic.json")

    rec = {
        "workload": f"{cfg.name}: {cfg.stands_in_for}", "ms_per_step": ms_per_step,
        "value": p.nnz / ms_per_step * 1e3, "unit": "edges/s",
        "config": {"workload": f"{cfg.name}: {cfg.stands_in_for}", "n_local": cfg.n_local, "n_halo": cfg.n_halo,
                   "nnz": p.nnz, "dim": dim, "n_send": pl.n, "n_peers": cfg.n_peers,
                   "packed_bytes": pl.packed_bytes, "direction": p.meta["direction"],
                   "schedule": schedule, "seed": cfg.seed},
        "ms_per_step_by_schedule": by_schedule, "overlap_lost": bool(overlap_lost),
        "kernels": kernels, "roofline": roofline,
        "setup_s": {"generate": t_gen, "upload_and_plan": t_plan, "panel_table_bytes": panel_table_bytes,
                    "note": "upload_and_plan: device copies, buffer layout, and (long-row graphs) the tile table and "
                            "the dense panels, once per graph"},
    }
    if ms_graph is not None:
        rec["ms_per_step_graph_replay"] = ms_graph
    if fused is not None:
        rec["fused_receive_variant"] = fused
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(p, pl, args.cpu_budget_s if headline else args.cpu_budget_other_s, B)
    del L
    torch.cuda.empty_cache()
    return rec


def degree_law_check(args, B, torch, np):
    """c1's sizes with a milder degree law (log-normal instead of Zipf(1.5)): what the library's rules choose there
    (tiles, panels) and what the other choices would cost.  Not one of the metric's workloads."""
    from paper_2306_01381_amd.layer import LayerStep
    from paper_2306_01381_amd.synth import config_by_name, make_partition
    cfg = config_by_name("c1m")
    p = make_partition(cfg)
    deg = np.diff(p.rowptr)
    out = {"workload": f"{cfg.name}: {cfg.stands_in_for}", "nnz": p.nnz, "max_row": int(deg.max()),
           "rows_at_or_above_panel_threshold": int(np.count_nonzero(deg >= B.SPMM_PANEL_MIN_ROW)), "ms_per_step": {}}
    steps = max(3, args.steps // 2)
    for tag, kw in (("library_rules", {}), ("panels_forced", {"panels": True}), ("tiled_without_panels", {"panels": False}),
                    ("merge_path", {"tiled": False})):
        L = LayerStep(p, "cuda:0", seed=2306, streams=_STREAMS.get("pair"), **kw)
        _STREAMS["pair"] = (L.stream_msg, L.stream_agg)
        paired = L.tile_off_overlap is not None and L.tile_off_dependent is not None and \
            bool(L.panels_overlap or L.panels_dependent)
        desc = L.desc(B.ISOLATED if paired else B.SERIAL)
        for _ in range(2):
            B.adaqp_layer_step(desc)
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(steps):
            B.adaqp_layer_step(desc)
        torch.cuda.synchronize()
        out["ms_per_step"][tag] = (time.perf_counter() - t) * 1e3 / steps
        if tag == "library_rules":
            out["library_rules_chose"] = {"tiled": L.tile_off_overlap is not None,
                                          "panels": int(L.panels_overlap.c.n_panels + L.panels_dependent.c.n_panels)}
        del L
        torch.cuda.empty_cache()
    best = min(out["ms_per_step"].values())
    out["library_rules_over_best"] = out["ms_per_step"]["library_rules"] / best
    return out


def short(rec):
    """The record of a non-headline workload, reduced to what the metric asks for."""
    k = rec["kernels"]
    out = {"workload": rec["workload"], "ms_per_step": rec["ms_per_step"], "value": rec["value"], "unit": rec["unit"],
           "schedule": rec["config"]["schedule"], "nnz": rec["config"]["nnz"], "dim": rec["config"]["dim"],
           "n_send": rec["config"]["n_send"], "ms_per_step_by_schedule": rec["ms_per_step_by_schedule"],
           "overlap_lost": rec["overlap_lost"], "kernels": {}}
    for name, v in k.items():
        if "frac_hbm" in v:
            e = {"ms": v["ms"], "GBps": v["GBps"], "frac_hbm": v["frac_hbm"], "ms_warm": v["ms_warm"],
                 "frac_hbm_warm": v["frac_hbm_warm"], "bytes": v["bytes"]}
            if "floor_no_compute_twin" in v:
                e["floor_ms"] = v["floor_no_compute_twin"]["ms"]
                e["kernel_over_floor"] = v["floor_no_compute_twin"]["kernel_over_floor"]
            if "stream_of_same_size" in v:
                e["stream_of_same_size_ms"] = v["stream_of_same_size"]["ms"]
                e["stream_frac_hbm"] = v["stream_of_same_size"]["frac_hbm"]
            out["kernels"][name] = e
        elif "edges_per_s" in v:
            out["kernels"][name] = {kk: v[kk] for kk in ("ms", "edges", "edges_per_s", "pct_hbm_primary") if kk in v}
    r = rec["roofline"]
    out["roofline"] = {kk: r[kk] for kk in ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic",
                                            "avg_launch_ms", "pct_hbm_primary") if kk in r}
    out["roofline"]["t_ceiling_over_t"] = r["ceilings"]["t_ceiling_over_t"]
    out["roofline"]["frac_hbm_compulsory"] = r["ceilings"]["frac_hbm_compulsory"]
    out["setup_s"] = {kk: rec["setup_s"][kk] for kk in ("generate", "upload_and_plan")}
    if "cpu_baseline" in rec:
        out["cpu_baseline"] = rec["cpu_baseline"]
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2306_01381_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()                                     # fails loudly if the HIP library has not been built
    head = measure_config(args.config, args, True, B, torch, np)
    result = {
        "metric": METRIC, "value": head["value"], "unit": "edges/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": head["config"],
        "ms_per_step_by_schedule": head["ms_per_step_by_schedule"], "overlap_lost": head["overlap_lost"],
    }
    for key in ("ms_per_step_graph_replay", "fused_receive_variant"):
        if key in head:
            result[key] = head[key]
    result["kernels"] = head["kernels"]
    result["roofline"] = head["roofline"]
    result["setup_s"] = head["setup_s"]
    if "cpu_baseline" in head:
        result["cpu_baseline"] = head["cpu_baseline"]
    if not args.only_headline:
        result["configs"] = {}
        for name in OTHER_CONFIGS:
            if name == args.config:
                continue
            print(f"bench.py: {name}", file=sys.stderr, flush=True)
            result["configs"][name] = short(measure_config(name, args, False, B, torch, np))
    if not args.only_headline and args.config == "c1":
        print("bench.py: c1m (degree-law check)", file=sys.stderr, flush=True)
        result["degree_law_check"] = degree_law_check(args, B, torch, np)
    if args.calibrate:
        a_ = torch.zeros(1 << 26, dtype=torch.float32, device="cuda:0")
        b_ = torch.empty_like(a_)
        for _ in range(3):
            torch.add(a_, 1.0, out=b_)
        torch.cuda.synchronize()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
