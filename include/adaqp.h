/*
 * adaqp.h - C ABI of the quantised message path of one graph partition (AdaQP, arXiv 2306.01381) for
 * AMD MI355X (gfx950).
 *
 * The library implements, for ONE device's partition, the data-parallel part of a GNN layer's aggregation
 * step under message quantisation (Sec. 3.1 "Overview", Fig. 4):
 *
 *   send side     gather the marginal-node rows to send, per-row min / max, stochastic rounding to the
 *                 assigned width b in {2, 4, 8}, sub-byte merging into per-peer byte buffers   (Sec. 2.3 Eq. 4,
 *                 App. A.1, Sec. 5 "Implementation")
 *   receive side  unpack the received buffers and de-quantise them into the halo rows          (Sec. 2.3 Eq. 5)
 *   aggregation   out_v = sum over u in {v} U N(v) of alpha(u,v) * h_u as a CSR SpMM, central rows on a
 *                 second stream so that they overlap the message path      (Sec. 2.1 Eq. 3, Sec. 3.4 Fig. 7)
 *                 - optionally straight from the packed receive buffer, or tiled over the GPU's eight L2
 *                 caches for graphs with long rows, the longest of them as dense panels on the matrix cores
 *   assignment    the next period's bit-widths from the traced beta values (host code)     (Sec. 4.2 Eq. 7-9)
 *
 * Conventions
 *   - "dev" pointers are device pointers valid on the current HIP device, "host" pointers are host memory.
 *   - Every buffer is owned by the caller.  The library allocates and frees no device memory; scratch memory
 *     is passed in as a workspace.  (The host-only planning calls use temporary host memory.)
 *   - Calls that take a stream only enqueue work on it and return; they never synchronise.
 *     `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Return value: ADAQP_OK (0) or a negative adaqp_status.  Argument errors are detected on the host
 *     before anything is launched.  Nothing throws, nothing aborts.
 *   - Device-side index arrays are trusted to be what adaqp_plan_layout / the caller's partitioner
 *     produced, but the kernels never touch memory outside the stated extents: a slot whose row index,
 *     width or offset is out of range is skipped, an edge whose column is out of range is skipped.
 *   - A count of zero is a successful no-op.
 *   - Inputs must be finite; denormal values and ranges are handled like any other.  A row whose range
 *     max - min is so small that (2^b - 1) / range is not an fp32 number (below about 2^-120) is quantised as a
 *     constant row: S = 0, every code 0, de-quantised to Z.
 *   - Feature matrices are fp32 row-major with a leading dimension (pitch) ld >= dim, counted in elements.
 *   - Preferred layout ("line-padded"): base pointer 128-byte aligned and ld a multiple of 32, so that every
 *     row starts on a 128-byte line and covers whole lines.  Any other layout is accepted and gives the same
 *     values, but partial-line writes are slower.  For a line-padded OUTPUT matrix the calls below write the
 *     rows they produce in whole lines: columns [dim, 32*ceil(dim/32)) of a written row are set to +0.0f
 *     (columns beyond that, and rows that are not written, stay untouched).  For any other output layout
 *     only columns [0, dim) are written.  Padding columns of INPUT matrices may hold anything.
 */
#ifndef ADAQP_H
#define ADAQP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum adaqp_status {
    ADAQP_OK     = 0,
    ADAQP_EINVAL = -1,  /* NULL pointer with a non-zero count, non-positive dim, ld < dim, negative count, ... */
    ADAQP_EBITS  = -2,  /* a host-visible bit-width outside {2, 4, 8} */
    ADAQP_ESIZE  = -3,  /* a declared buffer or workspace is too small, or a size exceeds a documented limit */
    ADAQP_EHIP   = -4   /* the HIP runtime reported an error (adaqp_last_hip_error gives its text) */
} adaqp_status;

const char *adaqp_strerror(int status);
const char *adaqp_last_hip_error(void);     /* text of the last HIP error seen by this thread, "" if none */
int adaqp_version(void);                    /* major * 10000 + minor * 100 + patch */

/* ---------------------------------------------------------------------------------------------------- */
/* Buffer layout (host only).  Sec. 5 "Implementation": messages are grouped by assigned bit-width, each   */
/* group is quantised at one width, the groups are concatenated into one byte array per peer; Sec. 3.3:    */
/* the buffer sizes follow from the assignment.                                                            */
/* ---------------------------------------------------------------------------------------------------- */

/* Bytes one packed row occupies: dim codes of `bits` bits, little-endian, padded with zero bits to a whole
 * number of 32-bit words: 4 * ceil(dim * bits / 32).  Returns -1 for dim <= 0 or bits outside {2,4,8}. */
int64_t adaqp_row_stride(int32_t dim, int32_t bits);

/* Orders n send slots and sizes the buffers.
 *   bits_host[n]          width of each slot, in {2, 4, 8}
 *   peer_of_slot_host[n]  destination peer of each slot, non-decreasing, in [0, n_peers)
 *   perm_out[n]           perm_out[k] = input slot that becomes sorted slot k.  Order: peer ascending, inside a
 *                         peer width ascending (2, 4, 8), inside a width the input order (stable).
 *   row_offset_out[n]     byte offset of sorted slot k in the single concatenated buffer (multiple of 4)
 *   peer_byte_ptr_out[n_peers + 1]  bytes [ptr[p], ptr[p+1]) go to peer p; ptr[n_peers] = total bytes
 * The quantise / de-quantise calls take their per-slot arrays (send_idx, bits, row_offset, halo_idx) in
 * SORTED slot order; the sorted slot index is the "row" that keys the random stream.
 * Errors: EINVAL (NULL, negative n, dim <= 0, peer order), EBITS. */
int adaqp_plan_layout(int64_t n, int32_t dim, const uint8_t *bits_host, const int32_t *peer_of_slot_host,
                      int32_t n_peers, int64_t *perm_out, int64_t *row_offset_out,
                      int64_t *peer_byte_ptr_out);

/* ---------------------------------------------------------------------------------------------------- */
/* Send side: Sec. 2.3 Eq. 4 with the stochastic rounding of App. A.1, then sub-byte merging (Sec. 5).    */
/* ---------------------------------------------------------------------------------------------------- */

/* For each slot s in [0, n_send):  h = feat[send_idx[s], 0:dim],  b = bits[s],  L = 2^b - 1
 *     Z = min(h) + 0.0f,  range = (max(h) + 0.0f) - Z,  S = range / L,  inv = L / range   (S = inv = 0 if range == 0
 *     or inv overflows)
 *     x_j = min((h_j - Z) * inv, L);  t_j = trunc(x_j * 2^16);  code_j = (t_j + r16(seed, s, j)) >> 16
 *     params[s] = {Z, S};  code_j is stored in bits [j*b, j*b+b) of the row at packed + row_offset[s]
 *     (little-endian bit string, zero padded to adaqp_row_stride(dim, b) bytes).
 * r16(seed, s, j): Philox4x32-10 with key (seed low, seed high) and counter (j / 8, s low, s high,
 * 0x41645150); its four output words, low half first, give the 16-bit values of columns 8*(j/8) .. +7.
 * All arithmetic is single fp32 operations in the order written (no fused multiply-add).
 *
 *   feat_dev      [n_feat_rows, ld] fp32, read only
 *   send_idx_dev  [n_send] int32 row of feat per slot;  bits_dev [n_send] uint8;  row_offset_dev [n_send] int64
 *   packed_dev    [packed_bytes] uint8, written (only the rows' own bytes);  params_dev [n_send][2] fp32, written
 * Slots with send_idx outside [0, n_feat_rows), bits outside {2,4,8} or a row that does not fit into
 * packed_bytes are skipped (nothing is written for them).
 * Errors: EINVAL, EHIP. */
int adaqp_quantize_pack(const float *feat_dev, int64_t n_feat_rows, int64_t ld, int32_t dim,
                        const int32_t *send_idx_dev, const uint8_t *bits_dev, const int64_t *row_offset_dev,
                        int64_t n_send, uint64_t seed,
                        uint8_t *packed_dev, int64_t packed_bytes, float *params_dev, void *stream);

/* Same as adaqp_quantize_pack, and additionally emits the trace the bit-width assigner works from (Sec. 4.2):
 *     beta[s] = ((alpha_sq[s] * (float)dim) * (range * range)) / 6.0f        with range = max - min of the row,
 * the numerator of message s in the variance objective (Eq. 8); fp32 in the order written.
 *   alpha_sq_dev [n_send] fp32, read: sum of the squared aggregation coefficients the message meets on its
 *                target device (an input; the sender cannot compute it);  beta_dev [n_send] fp32, written.
 * Both NULL: identical to adaqp_quantize_pack.  Exactly one NULL: EINVAL.  Skipped slots write no beta. */
int adaqp_quantize_pack_trace(const float *feat_dev, int64_t n_feat_rows, int64_t ld, int32_t dim,
                              const int32_t *send_idx_dev, const uint8_t *bits_dev, const int64_t *row_offset_dev,
                              int64_t n_send, uint64_t seed,
                              uint8_t *packed_dev, int64_t packed_bytes, float *params_dev,
                              const float *alpha_sq_dev, float *beta_dev, void *stream);

/* ---------------------------------------------------------------------------------------------------- */
/* Receive side: Sec. 2.3 Eq. 5.  (bits, row_offset, halo_idx) are the receiver's "bit-retrieval index    */
/* set" of Sec. 5.                                                                                         */
/* ---------------------------------------------------------------------------------------------------- */

/* Host only: the order in which the receive side should visit its slots so that consecutive waves write
 * ascending rows (DRAM takes sequential row writes faster than scattered ones).  order_out[k] = the slot
 * visited at position k; slots sorted by halo_idx_host, ties by slot index.  n <= 2^31 - 1.
 * Errors: EINVAL, ESIZE. */
int adaqp_plan_recv_order(int64_t n, const int32_t *halo_idx_host, int32_t *order_out);

/* For each slot t in [0, n_recv):  feat[halo_idx[t], j] = (float)code_j * S + Z   (product rounded, then sum
 * rounded), j in [0, dim), with {Z, S} = params[t] and code_j read from packed + row_offset[t].
 * Rows not listed are left untouched; padding columns as described under "Preferred layout".
 *   order_dev  optional [n_recv] int32 permutation of the slots (adaqp_plan_recv_order); NULL = slot order.
 *              It only changes which wave handles which slot, never a value; entries outside [0, n_recv)
 *              are skipped.  halo_idx must not list a row twice.
 * Out-of-range slots are skipped as above.  Errors: EINVAL, ESIZE, EHIP. */
int adaqp_unpack_dequant(const uint8_t *packed_dev, int64_t packed_bytes, const float *params_dev,
                         const uint8_t *bits_dev, const int64_t *row_offset_dev,
                         const int32_t *halo_idx_dev, const int32_t *order_dev, int64_t n_recv, int32_t dim,
                         float *feat_dev, int64_t n_feat_rows, int64_t ld, void *stream);

/* ---------------------------------------------------------------------------------------------------- */
/* Backward receive: Sec. 3.1 - in the backward pass the gradients of remote neighbours travel back to the */
/* node's owner quantised the same way; the owner de-quantises them (Eq. 5) and adds them to its own rows. */
/* ---------------------------------------------------------------------------------------------------- */

/* Host only: groups n received slots by destination row.  order_out[n] lists the slots sorted by
 * (dst_idx, slot); seg_ptr_out[n + 1] delimits runs of equal destination: segment g is
 * order_out[seg_ptr_out[g] .. seg_ptr_out[g+1]); *n_seg_out = number of segments (distinct rows).
 * Errors: EINVAL, ESIZE (n > 2^31 - 1). */
int adaqp_plan_recv_segments(int64_t n, const int32_t *dst_idx_host, int32_t *order_out, int64_t *seg_ptr_out,
                             int64_t *n_seg_out);

/* For every segment, in slot order:  grad[dst, j] = grad[dst, j] + ((float)code_j * S + Z)  - one fp32
 * addition per slot and element, so a node that hears from several peers accumulates them in slot order and
 * the result does not depend on the launch.  Per-slot arrays (params, bits, row_offset, dst_idx) are in slot
 * order as for adaqp_unpack_dequant; seg_order_dev / seg_ptr_dev come from adaqp_plan_recv_segments.
 * Only columns [0, dim) of the destination rows change (padding columns keep their contents).
 * Out-of-range slots are skipped.  Errors: EINVAL, ESIZE, EHIP. */
int adaqp_unpack_dequant_add(const uint8_t *packed_dev, int64_t packed_bytes, const float *params_dev,
                             const uint8_t *bits_dev, const int64_t *row_offset_dev, const int32_t *dst_idx_dev,
                             int64_t n_recv, const int32_t *seg_order_dev, const int64_t *seg_ptr_dev,
                             int64_t n_seg, int32_t dim, float *grad_dev, int64_t n_grad_rows, int64_t ld,
                             void *stream);

/* ---------------------------------------------------------------------------------------------------- */
/* Aggregation: Sec. 2.1 Eq. 3, inner sum.  The coefficients alpha(u,v) are the CSR values; the self term  */
/* is an explicit entry.                                                                                   */
/* ---------------------------------------------------------------------------------------------------- */

/* Workspace (bytes) adaqp_spmm_csr needs for a launch over `n_rows` rows holding at most `nnz` entries.
 * Writes *bytes_out (a multiple of 256).  Errors: EINVAL. */
int adaqp_spmm_workspace_bytes(int64_t n_rows, int64_t nnz, int32_t dim, int64_t *bytes_out);

/* out[v, 0:dim] = sum_{k = rowptr[v]}^{rowptr[v+1]-1} val[k] * H[col[k], 0:dim]   for v in [row_begin, row_end).
 * fp32 fused multiply-adds; the summation order is fixed by (row range, nnz_range, dim), so repeated calls
 * give bit-identical results.  Rows without entries give zeros.
 *
 *   rowptr_dev [>= row_end + 1] int64 (non-decreasing), col_dev / val_dev [nnz] int32 / fp32
 *   nnz        length of col_dev and val_dev; no entry index >= nnz is ever read
 *   nnz_range  number of entries in rows [row_begin, row_end) if the caller knows it, else -1 (nnz is
 *              used).  It only sizes the launch; the exact count is re-read from rowptr on the device.
 *   H_dev      [n_cols, ldh] fp32; entries with col outside [0, n_cols) are skipped
 *   out_dev    [>= row_end, ldo] fp32; only rows [row_begin, row_end) are written (columns [0, dim), plus
 *              zeroed padding when H and out are both line-padded, see "Preferred layout")
 *   workspace_dev / workspace_bytes   scratch of at least adaqp_spmm_workspace_bytes(row_end - row_begin,
 *              nnz_range or nnz, dim) bytes, 256-byte aligned; contents need not be initialised and are
 *              undefined afterwards.  Two launches that may run concurrently need distinct workspaces.
 * Errors: EINVAL, ESIZE (workspace too small), EHIP. */
int adaqp_spmm_csr(const int64_t *rowptr_dev, const int32_t *col_dev, const float *val_dev, int64_t nnz,
                   int64_t row_begin, int64_t row_end, int64_t nnz_range,
                   const float *H_dev, int64_t n_cols, int64_t ldh, int32_t dim,
                   float *out_dev, int64_t ldo,
                   void *workspace_dev, int64_t workspace_bytes, void *stream);

/* adaqp_spmm_csr for callers that cannot allocate device memory and have no workspace to pass: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same
 * launch geometry and therefore the same bits as adaqp_spmm_csr, but the carry scratch is a buffer of
 * ADAQP_SPMM_NOALLOC_SCRATCH_BYTES that is built into the library (one copy per GPU, held until the process
 * ends).  The call allocates and frees nothing.  The first call on a GPU looks the buffer's address up once (make
 * that call outside a capture).
 *   Limit: adaqp_spmm_workspace_bytes(row_end - row_begin, nnz_range or nnz, dim) must not exceed
 *          ADAQP_SPMM_NOALLOC_SCRATCH_BYTES, else ESIZE and nothing is launched.
 *   Every call on a GPU uses that GPU's one buffer: two calls that may run at the same time on one GPU (two
 *   streams, two threads) race on it - order them, or give one of them adaqp_spmm_csr with its own workspace.
 *   The buffer keeps the last call's contents; nothing in it needs to start at zero (every piece writes its
 *   carry slot's row number before the fix-up kernel reads it).
 * Errors: as adaqp_spmm_csr. */
#define ADAQP_SPMM_NOALLOC_SCRATCH_BYTES (64 << 20)
int adaqp_spmm_csr_noalloc(const int64_t *rowptr_dev, const int32_t *col_dev, const float *val_dev, int64_t nnz,
                           int64_t row_begin, int64_t row_end, int64_t nnz_range,
                           const float *H_dev, int64_t n_cols, int64_t ldh, int32_t dim,
                           float *out_dev, int64_t ldo, void *stream);

/* Host only: bit-widths for the next period from the traced beta values (Sec. 4.2).  Per device pair the
 * messages are sorted by descending beta (ties: ascending slot) and cut into groups of group_size that share a
 * width (the last group of a pair may be shorter).  The widths minimise, over the assignments a greedy search
 * visits, Eq. 9:  lambda * sum_k beta_k / (2^b_k - 1)^2  +  (1 - lambda) * max_i (theta_i * dim * sum_{k in i} b_k
 * + gamma_i), pairs without messages left out of the maximum.  The paper solves the same problem with a MILP
 * solver; the search here starts at 2 bits everywhere, orders a pair's upgrades (2->4, 4->8) by variance
 * removed per extra bit, and for every pair time such a prefix can reach lets each pair take the longest prefix
 * that fits under it (exact for one pair; within one upgrade's gain per pair otherwise).
 *   beta_host [n] float >= 0 (adaqp_quantize_pack_trace's output, copied to the host);  peer_of_slot_host [n];
 *   theta_host, gamma_host [n_peers]: cost model of Eq. 7, seconds per bit (>= 0) and seconds;
 *   bits_out [n]: 2, 4 or 8;  objective_out: NULL or [3] = {Eq. 9 value, Eq. 8 variance, largest pair time} of
 *   the result, evaluated from their definitions.
 * Errors: EINVAL (negative or non-finite beta / theta, peer out of range, lambda outside [0, 1],
 * group_size <= 0), ESIZE. */
int adaqp_assign_bits(int64_t n, const float *beta_host, const int32_t *peer_of_slot_host, int32_t n_peers,
                      int32_t dim, int32_t group_size, double lambda, const double *theta_host,
                      const double *gamma_host, uint8_t *bits_out, double *objective_out);

/* Host only: inverse of halo_idx.  slot_of_row_out[n_rows] = t for the row halo_idx_host[t], -1 for every
 * other row.  Errors: EINVAL (index out of range, a row listed twice), ESIZE (n > 2^31 - 1). */
int adaqp_plan_slot_of_row(int64_t n_rows, int64_t n, const int32_t *halo_idx_host, int32_t *slot_of_row_out);

/* adaqp_spmm_csr with some rows of H still packed: an entry whose column c has slot_of_row[c] = t >= 0 takes
 * the neighbour row from the receive buffer (packed + row_offset[t], bits[t], params[t]) and de-quantises it
 * in registers, (float)code * S + Z with the two roundings of Eq. 5, instead of reading H[c].  The result is
 * bit-identical to adaqp_unpack_dequant into H followed by adaqp_spmm_csr; the rows of H are neither written
 * nor read.  A slot that is out of range falls back to H[c].  slot_of_row_dev NULL: plain adaqp_spmm_csr.
 *   slot_of_row_dev [n_cols] int32;  per-slot arrays [n_slots] as for adaqp_unpack_dequant.
 * Errors: as adaqp_spmm_csr; EINVAL if slot_of_row_dev is given without the per-slot arrays. */
int adaqp_spmm_csr_packed(const int64_t *rowptr_dev, const int32_t *col_dev, const float *val_dev, int64_t nnz,
                          int64_t row_begin, int64_t row_end, int64_t nnz_range,
                          const float *H_dev, int64_t n_cols, int64_t ldh, int32_t dim,
                          float *out_dev, int64_t ldo,
                          const int32_t *slot_of_row_dev, const uint8_t *packed_dev, int64_t packed_bytes,
                          const float *params_dev, const uint8_t *bits_dev, const int64_t *row_offset_dev,
                          int64_t n_slots,
                          void *workspace_dev, int64_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------------- */
/* Aggregation for graphs with long rows (mean degree in the hundreds, as the densest dataset of Sec. 5):
 * the same sum as adaqp_spmm_csr (Sec. 2.1 Eq. 3), scheduled so that each of the GPU's ADAQP_SPMM_TILES L2
 * caches keeps re-using one range of the rows of H.  The graph's columns are cut into ADAQP_SPMM_TILES ranges
 * with equal entry counts, once per graph, on the host.  Line-padded layout only. */
#define ADAQP_SPMM_TILES 8
#define ADAQP_SPMM_TILED_SHORT_ROW 64   /* rows with fewer entries are kept whole in one tile */
#define ADAQP_SPMM_TILED_MIN_MEAN_ROW 128    /* mean entries per row from which adaqp_spmm_tiled_pays says yes */

/* Host only: 1 if a row range with n_rows rows and nnz entries is worth aggregating with adaqp_spmm_csr_tiled
 * rather than adaqp_spmm_csr (long rows: every row of H re-used many times), else 0. */
int32_t adaqp_spmm_tiled_pays(int64_t n_rows, int64_t nnz);

/* Host only.  For rows [row_begin, row_end) of a host CSR whose rows list ascending, distinct, in-range
 * columns: col_bounds_out[ADAQP_SPMM_TILES + 1] (0 = bounds[0] <= ... <= bounds[TILES] = one past the last
 * column these rows reference, at most n_cols) and
 * tile_off_out[(row_end - row_begin) * (ADAQP_SPMM_TILES + 1)]: entry t of a row = number of its entries that
 * belong to tiles before t.  For a row of at least ADAQP_SPMM_TILED_SHORT_ROW entries that is the number of
 * entries with column < bounds[t]; a shorter row is assigned whole to tile (row - row_begin) mod
 * ADAQP_SPMM_TILES (eight segments of one or two entries each would cost more than they save).
 * Errors: EINVAL (unsorted / repeated / out-of-range column, bad rowptr). */
int adaqp_plan_spmm_tiles(const int64_t *rowptr_host, const int32_t *col_host, int64_t row_begin, int64_t row_end,
                          int64_t n_cols, int32_t *col_bounds_out, int32_t *tile_off_out);

/* Host only: the feature-chunk width (64 or 128 columns) to pass to adaqp_spmm_csr_tiled for a plan with these
 * column bounds: 128 unless the widest column range times a 128-column chunk would overflow an L2.  0 on bad
 * arguments. */
int32_t adaqp_spmm_tiled_chunk_cols(const int32_t *col_bounds_host, int32_t dim);

/* Bytes of workspace adaqp_spmm_csr_tiled needs for n_rows rows (one partial row per tile). */
int adaqp_spmm_tiled_workspace_bytes(int64_t n_rows, int32_t dim, int64_t *bytes_out);

/* out[r, 0:dim] = sum_j val[j] * H[col[j], 0:dim] for r in [row_begin, row_end), like adaqp_spmm_csr.
 * tile_off_dev: device copy of adaqp_plan_spmm_tiles' table for the same row range (planning rejects graphs
 * with out-of-range columns; should the device arrays hold one nevertheless, it is read as column 0 with
 * coefficient 0).  A row whose table entries are negative (struck by adaqp_plan_spmm_panels) is skipped: its
 * row of out is not written.  A table that disagrees with rowptr is clamped to the row (wrong sums, no stray
 * access).  The summation order is fixed by the table and the launch geometry: runs are bit-identical.
 * H and out must be line-padded (pitch a multiple of 32 floats, base 128-byte aligned); the padding of the
 * written rows is set to zero.  chunk_cols: 64, 128 or 0 (= 128), see adaqp_spmm_tiled_chunk_cols; the result's
 * bits depend on it.  workspace_dev: 256-byte aligned, >= adaqp_spmm_tiled_workspace_bytes.
 * Errors: EINVAL (layout, alignment, null), ESIZE (workspace too small, too many rows), EHIP. */
int adaqp_spmm_csr_tiled(const int64_t *rowptr_dev, const int32_t *col_dev, const float *val_dev, int64_t nnz,
                         int64_t row_begin, int64_t row_end, const float *H_dev, int64_t n_cols, int64_t ldh,
                         int32_t dim, float *out_dev, int64_t ldo, const int32_t *tile_off_dev, int32_t chunk_cols,
                         void *workspace_dev, int64_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------------- */
/* Dense panels for the longest rows of such a graph.  In a power-law graph (the degree shape of the paper's
 * densest dataset, Sec. 5) a few thousand rows hold most of the entries, and any 32 of them share most of their
 * columns.  The host gathers such rows into panels of ADAQP_SPMM_PANEL_ROWS rows: per panel the sorted list of
 * the distinct columns its rows reference and a dense [columns][32] table of coefficients alpha(u, v) (0 where a
 * row lacks the column).  The same sum of Sec. 2.1 Eq. 3 is then a small dense product per panel: each row of H
 * is fetched once per panel instead of once per entry, and the multiply-adds run on the fp32 matrix cores.
 * The rows taken into panels are struck from the tile table (all entries -1), so adaqp_spmm_csr_tiled covers the
 * remaining rows and adaqp_spmm_csr_panels these.  The two calls write disjoint rows of out: with a workspace
 * each they may run in either order or at the same time on two streams (they suit each other: one keeps the
 * matrix cores busy, the other the vector-memory pipeline).
 * A zero coefficient times a non-finite H entry is NaN: H must be finite (as everywhere in this library), or a
 * non-finite row of H reaches all rows of the panels that list its column. */
#define ADAQP_SPMM_PANEL_ROWS 32
#define ADAQP_SPMM_PANEL_MIN_ROW 6144     /* default: rows with at least this many entries go into panels (about a
                                             tenth of the columns such rows reference in the Reddit-shaped workload:
                                             panels sparser than that lose against the tiled kernel) */
#define ADAQP_SPMM_PANEL_PIECE_COLS 1024  /* default: panel columns per piece of work (a multiple of 8) */

/* Device side of a panel plan for one row range.  All arrays are device copies of what adaqp_plan_spmm_panels
 * wrote; the struct itself lives in host memory and is read during the call only. */
typedef struct adaqp_spmm_panels {
    int32_t n_panels;                   /* 0: no panels, the struct is ignored */
    int32_t n_per_tile;                 /* pieces per tile list */
    int64_t n_groups;                   /* groups of 8 panel columns */
    int64_t n_panel_pieces;             /* pieces in use */
    const int32_t *panel_rows_dev;      /* [n_panels * 32] row of out per panel row, -1 = unused */
    const int32_t *pcol_dev;            /* [n_groups][2][4]: column of H for panel column 8g + 2u + h at [g][h][u] */
    const float   *palpha_dev;          /* [n_groups][64][4]: coefficient of panel column 8g + 2u + h, panel row m
                                           at [g][32h + m][u] */
    const int32_t *piece_dev;           /* [ADAQP_SPMM_TILES][n_per_tile][2]: first and end group; equal = unused */
    const int32_t *panel_piece_ptr_dev; /* [n_panels + 1] into panel_piece */
    const int32_t *panel_piece_dev;     /* [n_panel_pieces] piece numbers tile * n_per_tile + i, ascending per panel */
} adaqp_spmm_panels;

/* Host only.  Plans the panels of rows [row_begin, row_end) of a host CSR (ascending, distinct, in-range columns
 * per row) with at least min_row_len entries; col_bounds_host is adaqp_plan_spmm_tiles' output for the same
 * range (the pieces of a panel follow the same eight column ranges, so that each L2 keeps seeing one range).
 * Rows are taken in order of descending length (ties: ascending row), 32 per panel; the last panel may be
 * partly filled.  Every (panel, tile) column list is padded to a multiple of 8 with coefficient 0 and cut
 * into as few pieces of at most piece_cols columns as that takes, equal in size to within one group of 8; a tile's
 * pieces are listed in order of their first column.
 * Call twice: first with panel_rows_out NULL, which only fills sizes_out[5] = { rows taken, n_panels,
 * n_groups, n_per_tile, n_panel_pieces }; then with arrays of those sizes (layouts as in adaqp_spmm_panels).
 * tile_off_inout (may be NULL): adaqp_plan_spmm_tiles' table for the range; on the filling call all entries of
 * the rows taken become -1, i.e. adaqp_spmm_csr_tiled neither aggregates nor writes them.
 * Errors: EINVAL (bad CSR, min_row_len < 1, piece_cols not a positive multiple of 8), ESIZE (sizes beyond
 * 2^31 - 1). */
int adaqp_plan_spmm_panels(const int64_t *rowptr_host, const int32_t *col_host, const float *val_host,
                           int64_t row_begin, int64_t row_end, int64_t n_cols, const int32_t *col_bounds_host,
                           int32_t min_row_len, int32_t piece_cols, int64_t *sizes_out,
                           int32_t *tile_off_inout, int32_t *panel_rows_out, int32_t *pcol_out, float *palpha_out,
                           int32_t *piece_out, int32_t *panel_piece_ptr_out, int32_t *panel_piece_out);

/* Host only: 1 if a panel plan of n_panel_pieces pieces (sizes_out[4] of adaqp_plan_spmm_panels) is worth launching
 * for rows of dim columns, else 0.  The panel kernel runs one wave per (piece, 128-column chunk); a plan with fewer
 * than ADAQP_SPMM_PANEL_MIN_WAVES of them (a graph with only a handful of very long rows) leaves most of the GPU
 * idle and loses against leaving those rows to adaqp_spmm_csr_tiled (measured on a log-normal degree law: one or
 * two panels cost 0.14 ms where the tiled kernel takes 0.04 ms more for the same rows). */
#define ADAQP_SPMM_PANEL_MIN_WAVES 2048
int32_t adaqp_spmm_panels_pay(int64_t n_panel_pieces, int32_t dim);

/* Bytes of workspace adaqp_spmm_csr_panels needs (one [32][dim padded to lines] partial per piece slot). */
int adaqp_spmm_panels_workspace_bytes(int32_t n_per_tile, int32_t dim, int64_t *bytes_out);

/* out[r, 0:dim] = sum_j val[j] * H[col[j], 0:dim] (Sec. 2.1 Eq. 3) for the rows r listed in the panels; other
 * rows of out are not touched.  Products and sums in fp32 on the matrix cores (v_mfma_f32_32x32x2_f32); the
 * summation order is fixed by the plan: per piece in panel-column order; then the pieces of a panel in four
 * interleaved runs (every fourth piece of the panel's list, ascending) whose sums are added in run order - so
 * runs are bit-identical.  H and out line-padded as for adaqp_spmm_csr_tiled; padding of the
 * written rows is set to zero.  A column number outside [0, n_cols) in pcol_dev is clamped into range and a
 * group number outside [0, n_groups] likewise (wrong sums, no stray access); panel rows outside [row_begin,
 * row_end) are skipped.  workspace_dev: 256-byte aligned, >= adaqp_spmm_panels_workspace_bytes.
 * Errors: EINVAL (layout, alignment, null, negative sizes), ESIZE (workspace too small), EHIP. */
int adaqp_spmm_csr_panels(const adaqp_spmm_panels *panels_host, int64_t row_begin, int64_t row_end,
                          const float *H_dev, int64_t n_cols, int64_t ldh, int32_t dim, float *out_dev, int64_t ldo,
                          void *workspace_dev, int64_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------------------- */
/* One layer's aggregation step with the message path overlapped (Sec. 3.1, Sec. 3.4 Fig. 7).             */
/* ---------------------------------------------------------------------------------------------------- */

typedef enum adaqp_schedule {
    ADAQP_SERIAL   = 0, /* everything on stream_msg in program order */
    ADAQP_ISOLATED = 1, /* Fig. 7: the overlapped SpMM starts only once quantisation has finished, so it
                           overlaps the transfer (here: the loop-back copy) and nothing else by design */
    ADAQP_FREE     = 2  /* the overlapped SpMM starts at once on stream_agg and may overlap quantisation */
} adaqp_schedule;

typedef enum adaqp_direction {
    ADAQP_FORWARD  = 0, /* quantise send rows of `feat`, loop back, de-quantise into halo rows of `feat`,
                           aggregate: overlap_rows (central) on stream_agg, dependent_rows (marginal) after
                           the de-quantisation */
    ADAQP_BACKWARD = 1  /* the CSR is the transposed graph and `feat` holds the output gradients: aggregate
                           dependent_rows (halo rows of A^T dY) first, quantise + pack them from `out`,
                           loop back; overlap_rows (local rows) on stream_agg; then, if receive segments are
                           given, de-quantise the received buffer and add it to rows of `out` (halo_idx_dev =
                           destination rows), after both aggregations have finished */
} adaqp_direction;

typedef struct adaqp_layer_desc {
    int32_t direction;          /* adaqp_direction */
    int32_t schedule;           /* adaqp_schedule */
    /* graph */
    const int64_t *rowptr_dev;
    const int32_t *col_dev;
    const float   *val_dev;
    int64_t nnz;
    int64_t overlap_begin, overlap_end, overlap_nnz;        /* rows that do not depend on received messages */
    int64_t dependent_begin, dependent_end, dependent_nnz;  /* rows that do (forward) / that are sent (backward) */
    /* dense operands */
    float  *feat_dev;           /* forward: [n_feat_rows, ld], halo rows are overwritten; backward: dY, read only */
    int64_t n_feat_rows, ld;
    int32_t dim;
    float  *out_dev;            /* aggregation result, [>= max(overlap_end, dependent_end), ldo] */
    int64_t ldo;
    /* message path, all per-slot arrays in sorted slot order */
    const int32_t *send_idx_dev;    /* forward: rows of feat; backward: rows of out */
    const uint8_t *bits_dev;
    const int64_t *row_offset_dev;
    const int32_t *halo_idx_dev;    /* forward only: destination rows of the received slots */
    const int32_t *recv_order_dev;  /* forward only, optional: adaqp_plan_recv_order of halo_idx */
    const int32_t *slot_of_row_dev; /* forward only, optional: adaqp_plan_slot_of_row of halo_idx.  If given, the
                                       received rows are NOT de-quantised into feat; the dependent aggregation
                                       reads them from the receive buffer (adaqp_spmm_csr_packed) */
    const int32_t *tile_off_overlap_dev;    /* optional: adaqp_plan_spmm_tiles of the overlap / dependent row range. */
    const int32_t *tile_off_dependent_dev;  /* If given, that range is aggregated by adaqp_spmm_csr_tiled (line-padded
                                               layout required; the range's workspace must then hold
                                               adaqp_spmm_tiled_workspace_bytes as well).  With a table for the
                                               dependent range, slot_of_row_dev is ignored: the received rows are
                                               de-quantised into feat.  With tables for both ranges the dependent
                                               aggregation waits for the other one in every schedule (two tiled
                                               launches at once would share each L2 between two column ranges);
                                               the overlap with the message path stays */
    int32_t tile_chunk_overlap, tile_chunk_dependent;   /* chunk_cols of the two tiled launches (0 = 128) */
    adaqp_spmm_panels panels_overlap;       /* optional (n_panels = 0: none): adaqp_plan_spmm_panels of the two row */
    adaqp_spmm_panels panels_dependent;     /* ranges; only with that range's tile table.  The range's workspace must
                                               then hold adaqp_spmm_tiled_workspace_bytes PLUS
                                               adaqp_spmm_panels_workspace_bytes (the panel part starts where the
                                               tiled part ends).  Forward step, both ranges tiled, schedule ISOLATED
                                               or FREE: the panel launches go to stream_msg (after the
                                               de-quantisation) and both tiled launches to stream_agg, so that a
                                               panel kernel and a tiled kernel run side by side; otherwise a
                                               range's panels follow its tiled launch on the same stream */
    const int32_t *recv_seg_order_dev;  /* backward only, optional: adaqp_plan_recv_segments of halo_idx */
    const int64_t *recv_seg_ptr_dev;
    int64_t n_recv_seg;
    int64_t n_send;
    uint64_t seed;
    uint8_t *packed_dev;   float *params_dev;           /* send buffers */
    const float *alpha_sq_dev; float *beta_dev;         /* optional trace (adaqp_quantize_pack_trace); both or none */
    uint8_t *recv_packed_dev; float *recv_params_dev;   /* receive buffers; the loop-back copy stands in for the exchange */
    int64_t packed_bytes;
    /* scratch and streams */
    void *workspace_overlap_dev;   int64_t workspace_overlap_bytes;
    void *workspace_dependent_dev; int64_t workspace_dependent_bytes;
    void *stream_msg;           /* message path and dependent aggregation */
    void *stream_agg;           /* overlapped aggregation; joined back into stream_msg before returning */
    void *event_fork;           /* two hipEvent_t created by the caller (timing may be disabled) */
    void *event_join;
} adaqp_layer_desc;

/* Enqueues one layer step.  On return all work has been enqueued and stream_msg has been made to wait for
 * stream_agg, so synchronising stream_msg completes the step.  The three schedules give bit-identical
 * results.
 * ISOLATED and FREE only overlap anything if stream_msg and stream_agg sit on different hardware queues.  HIP maps
 * the streams of a process onto a few hardware queues (four by default): in a process that has created more
 * streams than that, the two may share a queue, and the step then takes the SERIAL time (same results).  A caller
 * that depends on the overlap creates these two streams first, or times the step against SERIAL once.
 * Errors: EINVAL, ESIZE, EHIP. */
int adaqp_layer_step(const adaqp_layer_desc *desc_host);

/* sizeof(adaqp_layer_desc) as this library was built: lets a binding in another language check its mirror of the
 * struct before the first call. */
int64_t adaqp_layer_desc_bytes(void);

#ifdef __cplusplus
}
#endif
#endif /* ADAQP_H */
