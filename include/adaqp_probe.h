/*
 * adaqp_probe.h - measurement aids of libadaqp.  Nothing here is part of the method: these kernels move the bytes
 * a codec kernel moves and compute nothing, so that a benchmark can put a kernel's time beside the floor of its own
 * access pattern and beside what the GPU delivers for a plain stream of the same size, in the same run.  They
 * answer the question the roofline fraction raises for kernels that run for 15-40 microseconds: how much of
 * the distance to the 8 TB/s peak is the kernel's, how much the access pattern's (a gather of rows in send-list
 * order), how much the part's (launch ramp, DRAM efficiency).
 *
 * Same conventions as adaqp.h: device pointers, caller-owned buffers, work is only enqueued on `stream`.
 */
#ifndef ADAQP_PROBE_H
#define ADAQP_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The no-compute twin of adaqp_quantize_pack (the send side of Sec. 2.3 Eq. 4): the same launch shape, the same
 * index loads, the same row loads and the same stores to packed_dev / params_dev (same instructions and addresses)
 * - but the stored words are the xor of two loaded values, there is no random generator, no reduction, no codes.
 * packed_dev / params_dev receive meaningless bytes.  Only for rows that take 16-byte vectors (base 16-byte
 * aligned, ld a multiple of 4) and fit the register-resident kernel; otherwise EINVAL.
 * Errors: as adaqp_quantize_pack. */
int adaqp_probe_quantize_pack(const float *feat_dev, int64_t n_feat_rows, int64_t ld, int32_t dim,
                              const int32_t *send_idx_dev, const uint8_t *bits_dev, const int64_t *row_offset_dev,
                              int64_t n_send, uint8_t *packed_dev, int64_t packed_bytes, float *params_dev,
                              void *stream);

/* The no-compute twin of adaqp_unpack_dequant_add (backward receive: Eq. 5 applied to every message, messages added
 * to their gradient rows in slot order): the same launch shape, the same loads of segment bounds, slot numbers,
 * index entries, parameters, gradient rows and packed words, the same stores of the rows - but a message's words
 * are xor-ed into its row instead of being decoded and added.  The rows named by dst_idx_dev end up holding
 * meaningless bits; other rows are not touched.  Only for the shape the full-size workloads take (base 128-byte
 * aligned, ld a multiple of 32, dim a multiple of 32 and at most 512); otherwise EINVAL.
 * Errors: as adaqp_unpack_dequant_add. */
int adaqp_probe_unpack_dequant_add(const uint8_t *packed_dev, int64_t packed_bytes, const float *params_dev,
                                   const uint8_t *bits_dev, const int64_t *row_offset_dev,
                                   const int32_t *dst_idx_dev, int64_t n_recv, const int32_t *seg_order_dev,
                                   const int64_t *seg_ptr_dev, int64_t n_seg, int32_t dim, float *grad_dev,
                                   int64_t n_grad_rows, int64_t ld, void *stream);

/* A plain stream over `bytes` bytes (a multiple of 16, both pointers 16-byte aligned):
 *   write_side = 0: reads src_dev[0, bytes) front to back with 16-byte non-temporal loads, 2 KiB per wave, and
 *                   writes bytes / 8 to dst_dev (the traffic mix of the send side: 4-bit codes for fp32 values);
 *   write_side = 1: writes dst_dev[0, bytes) front to back with 16-byte non-temporal stores, 4 KiB per wave, and
 *                   reads bytes / 8 from src_dev (the mix of the receive side);
 *   write_side = 2: reads dst_dev[0, bytes) front to back (non-temporal loads), reads bytes / 8 from src_dev and
 *                   writes dst_dev[0, bytes) back in place (non-temporal stores), 4 KiB per wave: the mix of the
 *                   backward receive, which adds messages to gradient rows.
 * The small side needs bytes / 8 + 4096 bytes.  What is written is derived from what is read.
 * Errors: EINVAL (null, alignment, negative size, another write_side), ESIZE (more than 2^40 bytes), EHIP. */
int adaqp_probe_stream(const void *src_dev, void *dst_dev, int64_t bytes, int32_t write_side, void *stream);

/* Launches a 1-D grid of n_workgroups workgroups (256 threads, as every kernel of the library) and records the XCD
 * each one runs on: xcd_out_dev[i] = XCC_ID of workgroup i.  adaqp_spmm_csr_tiled and adaqp_spmm_csr_panels pin
 * column range i mod ADAQP_SPMM_TILES of the graph to workgroup i, which keeps one range per L2 only if the
 * hardware deals consecutive workgroups of a grid to consecutive XCDs; this call lets a test or a benchmark check
 * that on the GPU at hand (on an idle MI355X: xcd[i] - xcd[0] = i mod 8).  If the mapping were different the two
 * kernels would still be correct, only slower.
 * Errors: EINVAL, EHIP. */
int adaqp_probe_xcd_of_workgroup(int32_t *xcd_out_dev, int32_t n_workgroups, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ADAQP_PROBE_H */
