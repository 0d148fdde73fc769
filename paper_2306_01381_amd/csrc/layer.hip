// Host side of libadaqp: status strings, the buffer layout of Sec. 5 "Implementation" (messages grouped by
// bit-width, groups concatenated per peer) and the layer step that overlaps the message path with the
// aggregation of the rows that do not depend on it (Sec. 3.1, Sec. 3.4 Fig. 7).
#include <stdio.h>
#include <string.h>

#include <algorithm>

#include "common.hpp"

namespace adaqp {

static thread_local char g_hip_error[256] = "";

int note_hip_error(hipError_t err, const char *what)
{
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(err));
    return ADAQP_EHIP;
}

}  // namespace adaqp

using namespace adaqp;

extern "C" const char *adaqp_strerror(int status)
{
    switch (status) {
        case ADAQP_OK: return "ok";
        case ADAQP_EINVAL: return "invalid argument";
        case ADAQP_EBITS: return "bit-width outside {2, 4, 8}";
        case ADAQP_ESIZE: return "buffer or workspace too small, or size beyond a documented limit";
        case ADAQP_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

extern "C" const char *adaqp_last_hip_error(void) { return g_hip_error; }

extern "C" int adaqp_version(void) { return 100; }

extern "C" int64_t adaqp_row_stride(int32_t dim, int32_t bits)
{
    if (dim <= 0 || !valid_bits(bits)) return -1;
    return 4 * (((int64_t)dim * bits + 31) / 32);
}

extern "C" int adaqp_plan_layout(int64_t n, int32_t dim, const uint8_t *bits_host,
                                 const int32_t *peer_of_slot_host, int32_t n_peers, int64_t *perm_out,
                                 int64_t *row_offset_out, int64_t *peer_byte_ptr_out)
{
    if (n < 0 || dim <= 0 || n_peers < 0 || !peer_byte_ptr_out) return ADAQP_EINVAL;
    if (n > 0 && (!bits_host || !peer_of_slot_host || !perm_out || !row_offset_out)) return ADAQP_EINVAL;
    if (n > 0 && n_peers == 0) return ADAQP_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        if (!valid_bits(bits_host[i])) return ADAQP_EBITS;
        const int32_t p = peer_of_slot_host[i];
        if (p < 0 || p >= n_peers) return ADAQP_EINVAL;
        if (i > 0 && p < peer_of_slot_host[i - 1]) return ADAQP_EINVAL;
    }
    // One counting pass per peer segment: slots of width 2 first, then 4, then 8, input order kept.
    const int64_t stride_of[3] = {adaqp_row_stride(dim, 2), adaqp_row_stride(dim, 4), adaqp_row_stride(dim, 8)};
    int64_t seg_begin = 0, bytes = 0;
    for (int32_t p = 0; p < n_peers; ++p) {
        int64_t seg_end = seg_begin;
        int64_t count[3] = {0, 0, 0};
        while (seg_end < n && peer_of_slot_host[seg_end] == p) {
            const int w = bits_host[seg_end] == 2 ? 0 : (bits_host[seg_end] == 4 ? 1 : 2);
            ++count[w];
            ++seg_end;
        }
        peer_byte_ptr_out[p] = bytes;
        int64_t next_slot[3], next_byte[3];
        next_slot[0] = seg_begin;
        next_slot[1] = next_slot[0] + count[0];
        next_slot[2] = next_slot[1] + count[1];
        next_byte[0] = bytes;
        next_byte[1] = next_byte[0] + count[0] * stride_of[0];
        next_byte[2] = next_byte[1] + count[1] * stride_of[1];
        bytes = next_byte[2] + count[2] * stride_of[2];
        for (int64_t i = seg_begin; i < seg_end; ++i) {
            const int w = bits_host[i] == 2 ? 0 : (bits_host[i] == 4 ? 1 : 2);
            const int64_t k = next_slot[w]++;
            perm_out[k] = i;
            row_offset_out[k] = next_byte[w];
            next_byte[w] += stride_of[w];
        }
        seg_begin = seg_end;
    }
    peer_byte_ptr_out[n_peers] = bytes;
    return ADAQP_OK;
}

extern "C" int adaqp_plan_recv_order(int64_t n, const int32_t *halo_idx_host, int32_t *order_out)
{
    if (n < 0) return ADAQP_EINVAL;
    if (n == 0) return ADAQP_OK;
    if (!halo_idx_host || !order_out) return ADAQP_EINVAL;
    if (n > INT32_MAX) return ADAQP_ESIZE;
    for (int64_t i = 0; i < n; ++i) order_out[i] = (int32_t)i;
    std::stable_sort(order_out, order_out + n,
                     [halo_idx_host](int32_t x, int32_t y) { return halo_idx_host[x] < halo_idx_host[y]; });
    return ADAQP_OK;
}

extern "C" int adaqp_plan_slot_of_row(int64_t n_rows, int64_t n, const int32_t *halo_idx_host,
                                      int32_t *slot_of_row_out)
{
    if (n_rows < 0 || n < 0) return ADAQP_EINVAL;
    if (n_rows > 0 && !slot_of_row_out) return ADAQP_EINVAL;
    if (n > 0 && !halo_idx_host) return ADAQP_EINVAL;
    if (n > INT32_MAX) return ADAQP_ESIZE;
    for (int64_t r = 0; r < n_rows; ++r) slot_of_row_out[r] = -1;
    for (int64_t t = 0; t < n; ++t) {
        const int32_t r = halo_idx_host[t];
        if (r < 0 || r >= n_rows || slot_of_row_out[r] != -1) return ADAQP_EINVAL;
        slot_of_row_out[r] = (int32_t)t;
    }
    return ADAQP_OK;
}

extern "C" int adaqp_plan_recv_segments(int64_t n, const int32_t *dst_idx_host, int32_t *order_out,
                                        int64_t *seg_ptr_out, int64_t *n_seg_out)
{
    if (n < 0 || !n_seg_out || !seg_ptr_out) return ADAQP_EINVAL;
    *n_seg_out = 0;
    seg_ptr_out[0] = 0;
    if (n == 0) return ADAQP_OK;
    if (!dst_idx_host || !order_out) return ADAQP_EINVAL;
    if (n > INT32_MAX) return ADAQP_ESIZE;
    for (int64_t i = 0; i < n; ++i) order_out[i] = (int32_t)i;
    std::stable_sort(order_out, order_out + n,
                     [dst_idx_host](int32_t x, int32_t y) { return dst_idx_host[x] < dst_idx_host[y]; });
    int64_t n_seg = 0;
    for (int64_t k = 0; k < n; ++k) {
        if (k == 0 || dst_idx_host[order_out[k]] != dst_idx_host[order_out[k - 1]]) seg_ptr_out[n_seg++] = k;
    }
    seg_ptr_out[n_seg] = n;
    *n_seg_out = n_seg;
    return ADAQP_OK;
}

namespace {

int check_desc(const adaqp_layer_desc *d)
{
    if (!d) return ADAQP_EINVAL;
    if (d->direction != ADAQP_FORWARD && d->direction != ADAQP_BACKWARD) return ADAQP_EINVAL;
    if (d->schedule != ADAQP_SERIAL && d->schedule != ADAQP_ISOLATED && d->schedule != ADAQP_FREE)
        return ADAQP_EINVAL;
    if (d->dim <= 0 || d->ld < d->dim || d->ldo < d->dim || d->n_send < 0 || d->packed_bytes < 0 || d->nnz < 0)
        return ADAQP_EINVAL;
    if (d->overlap_begin < 0 || d->overlap_end < d->overlap_begin || d->dependent_begin < 0 ||
        d->dependent_end < d->dependent_begin)
        return ADAQP_EINVAL;
    // the two row ranges are written concurrently: they must not intersect
    if (d->overlap_begin < d->dependent_end && d->dependent_begin < d->overlap_end &&
        d->overlap_end > d->overlap_begin && d->dependent_end > d->dependent_begin)
        return ADAQP_EINVAL;
    if (!d->feat_dev || !d->out_dev || !d->rowptr_dev) return ADAQP_EINVAL;
    if (d->n_send > 0) {
        if (!d->send_idx_dev || !d->bits_dev || !d->row_offset_dev || !d->packed_dev || !d->params_dev ||
            !d->recv_packed_dev || !d->recv_params_dev)
            return ADAQP_EINVAL;
        if (d->direction == ADAQP_FORWARD && !d->halo_idx_dev) return ADAQP_EINVAL;
    }
    for (int part = 0; part < 2; ++part) {
        const adaqp_spmm_panels *p = part ? &d->panels_overlap : &d->panels_dependent;
        const int32_t *tile_off = part ? d->tile_off_overlap_dev : d->tile_off_dependent_dev;
        if (p->n_panels < 0 || p->n_per_tile < 0 || p->n_groups < 0 || p->n_panel_pieces < 0) return ADAQP_EINVAL;
        if (p->n_panels == 0) continue;
        if (!tile_off) return ADAQP_EINVAL;                 // panels complement a tile table, never the merge path
        if (!p->panel_rows_dev || !p->pcol_dev || !p->palpha_dev || !p->piece_dev || !p->panel_piece_ptr_dev ||
            !p->panel_piece_dev)
            return ADAQP_EINVAL;
    }
    if (d->schedule != ADAQP_SERIAL) {
        if (!d->event_fork || !d->event_join) return ADAQP_EINVAL;
        if (d->stream_msg == d->stream_agg) return ADAQP_EINVAL;
        // the two aggregations run at the same time: they need separate scratch
        if (d->workspace_overlap_dev && d->workspace_overlap_dev == d->workspace_dependent_dev) return ADAQP_EINVAL;
    }
    return ADAQP_OK;
}

bool fused_receive(const adaqp_layer_desc *d)
{
    return d->direction == ADAQP_FORWARD && d->slot_of_row_dev && !d->tile_off_dependent_dev && d->n_send > 0 &&
           d->packed_bytes >= 4;
}

// Workspace of a row range: the tiled kernel's partial sums first, then (if the range has panels) the panel
// kernel's piece sums, so that the two kernels can run at the same time.
int64_t tiled_part_bytes(const adaqp_layer_desc *d, bool overlap_part)
{
    const int64_t rows = overlap_part ? d->overlap_end - d->overlap_begin : d->dependent_end - d->dependent_begin;
    int64_t bytes = 0;
    if (adaqp_spmm_tiled_workspace_bytes(rows, d->dim, &bytes) != ADAQP_OK) return -1;
    return bytes;
}

// The rows of a range that are aggregated entry by entry: all of them, or those outside the panels.
int aggregate_rows(const adaqp_layer_desc *d, bool overlap_part, hipStream_t st)
{
    const int64_t rb = overlap_part ? d->overlap_begin : d->dependent_begin;
    const int64_t re = overlap_part ? d->overlap_end : d->dependent_end;
    const int64_t nz = overlap_part ? d->overlap_nnz : d->dependent_nnz;
    void *ws = overlap_part ? d->workspace_overlap_dev : d->workspace_dependent_dev;
    const int64_t wsb = overlap_part ? d->workspace_overlap_bytes : d->workspace_dependent_bytes;
    const int32_t *tile_off = overlap_part ? d->tile_off_overlap_dev : d->tile_off_dependent_dev;
    if (tile_off)
        return adaqp_spmm_csr_tiled(d->rowptr_dev, d->col_dev, d->val_dev, d->nnz, rb, re, d->feat_dev,
                                    d->n_feat_rows, d->ld, d->dim, d->out_dev, d->ldo, tile_off,
                                    overlap_part ? d->tile_chunk_overlap : d->tile_chunk_dependent, ws, wsb, st);
    if (!overlap_part && fused_receive(d))
        return adaqp_spmm_csr_packed(d->rowptr_dev, d->col_dev, d->val_dev, d->nnz, rb, re, nz, d->feat_dev,
                                     d->n_feat_rows, d->ld, d->dim, d->out_dev, d->ldo, d->slot_of_row_dev,
                                     d->recv_packed_dev, d->packed_bytes, d->recv_params_dev, d->bits_dev,
                                     d->row_offset_dev, d->n_send, ws, wsb, st);
    return adaqp_spmm_csr(d->rowptr_dev, d->col_dev, d->val_dev, d->nnz, rb, re, nz, d->feat_dev,
                          d->n_feat_rows, d->ld, d->dim, d->out_dev, d->ldo, ws, wsb, st);
}

bool has_panels(const adaqp_layer_desc *d, bool overlap_part)
{
    const int32_t *tile_off = overlap_part ? d->tile_off_overlap_dev : d->tile_off_dependent_dev;
    return tile_off && (overlap_part ? d->panels_overlap.n_panels : d->panels_dependent.n_panels) > 0;
}

// The rows of a range that were struck from its tile table.  Own part of the workspace, disjoint output rows:
// independent of aggregate_rows of the same range.
int aggregate_panels(const adaqp_layer_desc *d, bool overlap_part, hipStream_t st)
{
    if (!has_panels(d, overlap_part)) return ADAQP_OK;
    const int64_t rb = overlap_part ? d->overlap_begin : d->dependent_begin;
    const int64_t re = overlap_part ? d->overlap_end : d->dependent_end;
    char *ws = static_cast<char *>(overlap_part ? d->workspace_overlap_dev : d->workspace_dependent_dev);
    const int64_t wsb = overlap_part ? d->workspace_overlap_bytes : d->workspace_dependent_bytes;
    const int64_t skip = tiled_part_bytes(d, overlap_part);
    if (skip < 0 || !ws || wsb < skip) return ADAQP_ESIZE;
    return adaqp_spmm_csr_panels(overlap_part ? &d->panels_overlap : &d->panels_dependent, rb, re, d->feat_dev,
                                 d->n_feat_rows, d->ld, d->dim, d->out_dev, d->ldo, ws + skip, wsb - skip, st);
}

int aggregate(const adaqp_layer_desc *d, bool overlap_part, hipStream_t st)
{
    const int rc = aggregate_rows(d, overlap_part, st);
    return rc != ADAQP_OK ? rc : aggregate_panels(d, overlap_part, st);
}

int loop_back(const adaqp_layer_desc *d, hipStream_t st)
{
    if (d->n_send == 0) return ADAQP_OK;
    if (d->packed_bytes > 0)
        ADAQP_HIP_TRY(hipMemcpyAsync(d->recv_packed_dev, d->packed_dev, (size_t)d->packed_bytes,
                                     hipMemcpyDeviceToDevice, st));
    ADAQP_HIP_TRY(hipMemcpyAsync(d->recv_params_dev, d->params_dev, (size_t)d->n_send * 2 * sizeof(float),
                                 hipMemcpyDeviceToDevice, st));
    return ADAQP_OK;
}

}  // namespace

extern "C" int64_t adaqp_layer_desc_bytes(void) { return (int64_t)sizeof(adaqp_layer_desc); }

extern "C" int adaqp_layer_step(const adaqp_layer_desc *d)
{
    int rc = check_desc(d);
    if (rc != ADAQP_OK) return rc;
    // workspace sizes are checked up front so that a failure cannot leave the two streams half-joined
    for (int part = 0; part < 2; ++part) {
        const int64_t rows = part ? d->overlap_end - d->overlap_begin : d->dependent_end - d->dependent_begin;
        int64_t nz = part ? d->overlap_nnz : d->dependent_nnz;
        if (nz < 0 || nz > d->nnz) nz = d->nnz;
        int64_t need = 0;
        rc = adaqp_spmm_workspace_bytes(rows, nz, d->dim, &need);
        if (rc != ADAQP_OK) return rc;
        if (part ? d->tile_off_overlap_dev != nullptr : d->tile_off_dependent_dev != nullptr) {
            rc = adaqp_spmm_tiled_workspace_bytes(rows, d->dim, &need);         // that range takes the tiled kernel
            if (rc != ADAQP_OK) return rc;
            const adaqp_spmm_panels *panels = part ? &d->panels_overlap : &d->panels_dependent;
            if (panels->n_panels > 0) {
                int64_t need_panels = 0;
                rc = adaqp_spmm_panels_workspace_bytes(panels->n_per_tile, d->dim, &need_panels);
                if (rc != ADAQP_OK) return rc;
                need += need_panels;                        // side by side: the two kernels may run together
            }
        }
        const int64_t have = part ? d->workspace_overlap_bytes : d->workspace_dependent_bytes;
        const void *ws = part ? d->workspace_overlap_dev : d->workspace_dependent_dev;
        if (rows > 0 && need > 0 && (!ws || have < need)) return ADAQP_ESIZE;
    }

    hipStream_t msg = (hipStream_t)d->stream_msg;
    hipStream_t agg = d->schedule == ADAQP_SERIAL ? msg : (hipStream_t)d->stream_agg;
    hipEvent_t fork = (hipEvent_t)d->event_fork, join = (hipEvent_t)d->event_join;
    const bool forward = d->direction == ADAQP_FORWARD;
    const bool both_tiled = d->tile_off_overlap_dev && d->tile_off_dependent_dev;
    const bool paired = forward && both_tiled && d->schedule != ADAQP_SERIAL &&
                        (has_panels(d, true) || has_panels(d, false));
    bool forked = false;
    auto fork_now = [&]() -> int {
        if (d->schedule == ADAQP_SERIAL) return ADAQP_OK;
        ADAQP_HIP_TRY(hipEventRecord(fork, msg));
        ADAQP_HIP_TRY(hipStreamWaitEvent(agg, fork, 0));
        forked = true;
        return ADAQP_OK;
    };
    auto join_now = [&]() -> int {
        if (!forked) return ADAQP_OK;
        ADAQP_HIP_TRY(hipEventRecord(join, agg));
        ADAQP_HIP_TRY(hipStreamWaitEvent(msg, join, 0));
        forked = false;
        return ADAQP_OK;
    };
    auto agg_waits_for_msg = [&]() -> int {
        // the fork event is free again: its first wait has been enqueued, and a wait refers to the record before it
        ADAQP_HIP_TRY(hipEventRecord(fork, msg));
        ADAQP_HIP_TRY(hipStreamWaitEvent(agg, fork, 0));
        return ADAQP_OK;
    };
#define ADAQP_STEP(expr)                    \
    do {                                    \
        rc = (expr);                        \
        if (rc != ADAQP_OK) { join_now(); return rc; } \
    } while (0)

    if (forward) {
        // FREE: the central rows start right away.  ISOLATED: they start once quantisation is done.
        if (d->schedule == ADAQP_FREE) {
            ADAQP_STEP(fork_now());
            ADAQP_STEP(paired ? aggregate_rows(d, true, agg) : aggregate(d, true, agg));
        }
        ADAQP_STEP(adaqp_quantize_pack_trace(d->feat_dev, d->n_feat_rows, d->ld, d->dim, d->send_idx_dev,
                                             d->bits_dev, d->row_offset_dev, d->n_send, d->seed, d->packed_dev,
                                             d->packed_bytes, d->params_dev, d->alpha_sq_dev, d->beta_dev, msg));
        if (d->schedule == ADAQP_ISOLATED) {
            ADAQP_STEP(fork_now());
            ADAQP_STEP(paired ? aggregate_rows(d, true, agg) : aggregate(d, true, agg));
        }
        ADAQP_STEP(loop_back(d, msg));
        if (!fused_receive(d))
            ADAQP_STEP(adaqp_unpack_dequant(d->recv_packed_dev, d->packed_bytes, d->recv_params_dev, d->bits_dev,
                                            d->row_offset_dev, d->halo_idx_dev, d->recv_order_dev, d->n_send, d->dim,
                                            d->feat_dev, d->n_feat_rows, d->ld, msg));
        if (d->schedule == ADAQP_SERIAL) ADAQP_STEP(aggregate(d, true, msg));
        if (paired) {
            // a panel kernel (matrix cores) and a tiled kernel (vector-memory pipeline) fill each other's gaps:
            // both tiled launches on the second stream, one after the other, both panel launches here
            ADAQP_STEP(agg_waits_for_msg());                            // the halo rows are in place
            ADAQP_STEP(aggregate_panels(d, true, msg));
            ADAQP_STEP(aggregate_rows(d, false, agg));
            ADAQP_STEP(aggregate_panels(d, false, msg));
        } else {
            // two tiled aggregations side by side would bring two column ranges to every L2 and lose what the
            // tiling is for: the dependent one waits for the other (which has overlapped the message path by now)
            if (both_tiled) ADAQP_STEP(join_now());
            ADAQP_STEP(aggregate(d, false, msg));
        }
    } else {
        // backward: the rows that are sent are aggregated first, the local rows overlap their quantisation
        // (FREE) or only their transfer (ISOLATED)
        if (d->schedule == ADAQP_FREE) {
            ADAQP_STEP(fork_now());
            ADAQP_STEP(aggregate(d, true, agg));
            if (both_tiled) ADAQP_STEP(join_now());         // as in the forward step: one tiled launch at a time
        }
        ADAQP_STEP(aggregate(d, false, msg));
        ADAQP_STEP(adaqp_quantize_pack_trace(d->out_dev,
                                             d->dependent_end > d->overlap_end ? d->dependent_end : d->overlap_end,
                                             d->ldo, d->dim, d->send_idx_dev, d->bits_dev, d->row_offset_dev,
                                             d->n_send, d->seed, d->packed_dev, d->packed_bytes, d->params_dev,
                                             d->alpha_sq_dev, d->beta_dev, msg));
        if (d->schedule == ADAQP_ISOLATED) {
            ADAQP_STEP(fork_now());
            ADAQP_STEP(aggregate(d, true, agg));
        }
        ADAQP_STEP(loop_back(d, msg));
        if (d->schedule == ADAQP_SERIAL) ADAQP_STEP(aggregate(d, true, msg));
        if (d->n_recv_seg > 0 && d->recv_seg_order_dev && d->recv_seg_ptr_dev && d->halo_idx_dev) {
            // the received gradients are added to rows that the local aggregation also writes: join first
            ADAQP_STEP(join_now());
            ADAQP_STEP(adaqp_unpack_dequant_add(d->recv_packed_dev, d->packed_bytes, d->recv_params_dev, d->bits_dev,
                                                d->row_offset_dev, d->halo_idx_dev, d->n_send,
                                                d->recv_seg_order_dev, d->recv_seg_ptr_dev, d->n_recv_seg, d->dim,
                                                d->out_dev,
                                                d->dependent_end > d->overlap_end ? d->dependent_end : d->overlap_end,
                                                d->ldo, msg));
        }
    }
    ADAQP_STEP(join_now());
#undef ADAQP_STEP
    return ADAQP_OK;
}
