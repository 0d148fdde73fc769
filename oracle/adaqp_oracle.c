/*
 * CPU oracle for the quantised message path of one graph partition (AdaQP, arXiv 2306.01381).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, single-threaded, obviously-correct statement of what
 * the path computes.  It shares no code, header, table or constant with the HIP library; only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may load it.  Plain C11, built with
 *   gcc -O2 -ffp-contract=off -fno-fast-math
 * so that every fp32 operation below is a single correctly-rounded IEEE operation in the order written.
 *
 * What follows the paper and where:
 *   quantisation       Sec. 2.3 Eq. 4:  code = round_st((h - Z) / S),  Z = min(h),  S = (max(h) - min(h)) / (2^b - 1)
 *   stochastic round   App. A.1:        round up with probability frac(x), down with probability 1 - frac(x)
 *   de-quantisation    Sec. 2.3 Eq. 5:  h^ = code * S + Z
 *   sub-byte merging   Sec. 5 "Implementation": 2- and 4-bit codes are merged into a byte stream; messages are
 *                      grouped by bit-width, each group quantised at one width, groups concatenated per peer
 *   aggregation        Sec. 2.1 Eq. 3 (inner sum):  out_v = sum over u in {v} U N(v) of alpha(u,v) * h_u
 *   backward receive   Sec. 3.1: received gradient messages are de-quantised (Eq. 5) and added to the owner's rows
 *
 * Readings taken where the paper is silent (each one is restated next to the code that uses it):
 *   R1  one fp32 division per row gives inv = (2^b-1)/(max-min); elements are multiplied by inv and clamped
 *       to 2^b-1 (a literal per-element division differs by at most one ulp of the quotient).
 *   R2  round_st is realised in 16.16 fixed point: t = trunc(x * 2^16), code = (t + r) >> 16 with r a uniform
 *       16-bit integer, i.e. P(round up) = floor(frac(x) * 2^16) / 2^16.
 *   R3  r comes from Philox4x32-10 keyed by the seed, counter = (column / 8, slot low, slot high, tag); the
 *       128 output bits serve eight consecutive columns as eight 16-bit slices.
 *   R4  a constant row has S = 0, inv = 0, all codes 0; min and max are passed through "+ 0.0f" so that a
 *       row holding both -0 and +0 has one well-defined zero-point.  A row whose range is so small that
 *       (2^b-1)/(max-min) overflows fp32 (range below about 2^-120) is treated as constant as well: Eq. 4 has
 *       no finite argument for it in fp32, and its de-quantisation error stays below that range.
 *   R5  codes are laid down little-endian: column j occupies bits [j*b, j*b + b) of the row's bit string,
 *       bit k of the string is bit (k mod 8) of byte (k / 8).  A row occupies 4 * ceil(dim*b/32) bytes, unused
 *       bits are zero.
 *   R6  (Z, S) travel as two fp32 values per slot in a separate array.
 *   R7  buffer order: peers in order; inside a peer, widths ascending (2, 4, 8); inside a width, the
 *       original order of the send list.
 *
 * Pins (tests/test_oracle_*.py): closed-form rows and byte patterns, endpoints, code range, two-point
 * support, unbiasedness and variance over 1e5 seeds, the Theorem 1 value D*S^2/6, exhaustive pack/unpack
 * round trips, Philox known-answer vectors, dense brute-force A*H and special matrices for the SpMM.
 * Nothing in this file is "parity unpinned".
 */
#include <float.h>
#include <math.h>
#include <stdint.h>
#include <stddef.h>
#include <string.h>

#define ORACLE_OK      0
#define ORACLE_EINVAL -1
#define ORACLE_EBITS  -2

/* ------------------------------------------------------------------------------------------------------ */
/* Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy as 1, 2, 3",   */
/* SC'11).  One round maps (c0,c1,c2,c3) to (hi(M1*c2)^c1^k0, lo(M1*c2), hi(M0*c0)^c3^k1, lo(M0*c0)); the   */
/* key words are then bumped by the two Weyl constants.                                                    */
/* ------------------------------------------------------------------------------------------------------ */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)M0 * c0;
        uint64_t p1 = (uint64_t)M1 * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += W0; k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* R3: the 16 random bits used for (seed, slot, column). */
uint32_t oracle_rand16(uint64_t seed, uint64_t slot, uint32_t column)
{
    uint32_t ctr[4] = { column >> 3, (uint32_t)slot, (uint32_t)(slot >> 32), 0x41645150u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    uint32_t out[4];
    oracle_philox4x32_10(ctr, key, out);
    uint32_t word = out[(column & 7u) >> 1];
    return (column & 1u) ? (word >> 16) : (word & 0xFFFFu);
}

/* ------------------------------------------------------------------------------------------------------ */
/* Layout (R5, R7)                                                                                          */
/* ------------------------------------------------------------------------------------------------------ */
int64_t oracle_row_stride(int32_t dim, int32_t bits)
{
    return 4 * (((int64_t)dim * bits + 31) / 32);
}

/* Orders the n slots (already sorted by peer) by (peer, width, original position) and sizes the buffers.
 * perm[k] = index of the original slot that becomes sorted slot k; row_offset[k] = byte offset of sorted
 * slot k in the single concatenated buffer; peer_byte_ptr[p] .. peer_byte_ptr[p+1] = bytes sent to peer p. */
int oracle_plan_layout(int64_t n, int32_t dim, const uint8_t *bits, const int32_t *peer_of_slot,
                       int32_t n_peers, int64_t *perm, int64_t *row_offset, int64_t *peer_byte_ptr)
{
    static const int widths[3] = { 2, 4, 8 };
    if (n < 0 || dim <= 0 || n_peers < 0) return ORACLE_EINVAL;
    for (int64_t i = 0; i < n; ++i) {
        if (bits[i] != 2 && bits[i] != 4 && bits[i] != 8) return ORACLE_EBITS;
        if (peer_of_slot[i] < 0 || peer_of_slot[i] >= n_peers) return ORACLE_EINVAL;
        if (i > 0 && peer_of_slot[i] < peer_of_slot[i - 1]) return ORACLE_EINVAL;
    }
    int64_t k = 0, offset = 0, begin = 0;
    for (int32_t p = 0; p < n_peers; ++p) {
        int64_t end = begin;
        while (end < n && peer_of_slot[end] == p) ++end;
        peer_byte_ptr[p] = offset;
        for (int w = 0; w < 3; ++w)
            for (int64_t i = begin; i < end; ++i)
                if (bits[i] == widths[w]) {
                    perm[k] = i;
                    row_offset[k] = offset;
                    offset += oracle_row_stride(dim, widths[w]);
                    ++k;
                }
        begin = end;
    }
    peer_byte_ptr[n_peers] = offset;
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------------ */
/* Quantise + pack (Eq. 4 with R1-R6).  codes_out (optional, [n_send * dim]) receives the unpacked codes.   */
/* slot_base: slot number of the first entry of the arrays (the random stream is keyed by slot number), so  */
/* that any contiguous run of slots - or a single one - can be computed on its own.                        */
/* ------------------------------------------------------------------------------------------------------ */
int oracle_quantize_pack(const float *feat, int64_t ld, int32_t dim,
                         const int32_t *send_idx, const uint8_t *bits, const int64_t *row_offset,
                         int64_t n_send, uint64_t seed, int64_t slot_base,
                         uint8_t *packed, float *params, uint8_t *codes_out)
{
    if (n_send < 0 || dim <= 0 || ld < dim) return ORACLE_EINVAL;
    for (int64_t s = 0; s < n_send; ++s) {
        const int b = bits[s];
        if (b != 2 && b != 4 && b != 8) return ORACLE_EBITS;
        const float *h = feat + (int64_t)send_idx[s] * ld;
        const float levels = (float)((1 << b) - 1);

        float mn = h[0], mx = h[0];
        for (int32_t j = 1; j < dim; ++j) {
            if (h[j] < mn) mn = h[j];
            if (h[j] > mx) mx = h[j];
        }
        const float Z = mn + 0.0f;                 /* R4 */
        const float range = (mx + 0.0f) - Z;
        float S = 0.0f, inv = 0.0f;
        if (range > 0.0f) {
            S = range / levels;                    /* Eq. 4: scale */
            inv = levels / range;                  /* R1 */
            if (!(inv <= FLT_MAX)) {               /* R4: range below (2^b-1)/FLT_MAX, the reciprocal is not an fp32 */
                S = 0.0f;                          /* number - the row counts as constant */
                inv = 0.0f;
            }
        }
        params[2 * s + 0] = Z;                     /* R6 */
        params[2 * s + 1] = S;

        uint8_t *row = packed + row_offset[s];
        memset(row, 0, (size_t)oracle_row_stride(dim, b));
        for (int32_t j = 0; j < dim; ++j) {
            float x = (h[j] - Z) * inv;            /* position on the integer grid, >= 0 */
            if (x > levels) x = levels;            /* R1: the top element may overshoot by an ulp */
            const uint32_t t = (uint32_t)(x * 65536.0f);          /* R2: 16.16 fixed point, truncated */
            const uint32_t code = (t + oracle_rand16(seed, (uint64_t)(slot_base + s), (uint32_t)j)) >> 16;
            if (codes_out) codes_out[s * (int64_t)dim + j] = (uint8_t)code;
            const int64_t bit = (int64_t)j * b;    /* R5 */
            row[bit >> 3] |= (uint8_t)(code << (bit & 7));
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------------ */
/* Trace for the bit-width assigner (Sec. 4.2): beta_k = (sum_v alpha_{k,v}^2) * D * (max(h_k) - min(h_k))^2 / 6, */
/* the numerator of message k's term in the variance objective (Eq. 8).  alpha_sq[s] is the per-message sum   */
/* of squared coefficients (an input: it lives on the target device).  fp32, in the order written.           */
/* ------------------------------------------------------------------------------------------------------ */
int oracle_trace_beta(const float *feat, int64_t ld, int32_t dim, const int32_t *send_idx,
                      const float *alpha_sq, int64_t n_send, float *beta)
{
    if (n_send < 0 || dim <= 0 || ld < dim) return ORACLE_EINVAL;
    for (int64_t s = 0; s < n_send; ++s) {
        const float *h = feat + (int64_t)send_idx[s] * ld;
        float mn = h[0], mx = h[0];
        for (int32_t j = 1; j < dim; ++j) {
            if (h[j] < mn) mn = h[j];
            if (h[j] > mx) mx = h[j];
        }
        const float range = (mx + 0.0f) - (mn + 0.0f);
        const float wd = alpha_sq[s] * (float)dim;
        const float r2 = range * range;
        beta[s] = (wd * r2) / 6.0f;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------------ */
/* Unpack + de-quantise into the halo rows (Eq. 5).  codes_out optional as above.                           */
/* ------------------------------------------------------------------------------------------------------ */
int oracle_unpack_dequant(const uint8_t *packed, const float *params,
                          const uint8_t *bits, const int64_t *row_offset, const int32_t *halo_idx,
                          int64_t n_recv, int32_t dim, float *feat, int64_t ld, uint8_t *codes_out)
{
    if (n_recv < 0 || dim <= 0 || ld < dim) return ORACLE_EINVAL;
    for (int64_t t = 0; t < n_recv; ++t) {
        const int b = bits[t];
        if (b != 2 && b != 4 && b != 8) return ORACLE_EBITS;
        const float Z = params[2 * t + 0], S = params[2 * t + 1];
        const uint8_t *row = packed + row_offset[t];
        float *h = feat + (int64_t)halo_idx[t] * ld;
        for (int32_t j = 0; j < dim; ++j) {
            const int64_t bit = (int64_t)j * b;
            const uint32_t code = ((uint32_t)row[bit >> 3] >> (bit & 7)) & ((1u << b) - 1u);
            if (codes_out) codes_out[t * (int64_t)dim + j] = (uint8_t)code;
            const float scaled = (float)code * S;  /* Eq. 5, two roundings: product, then sum */
            h[j] = scaled + Z;
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------------ */
/* Backward receive (Sec. 3.1: in the backward pass the embedding gradients of remote neighbours travel back   */
/* to the owner of the node, quantised the same way; the owner de-quantises them, Eq. 5, and adds them to the   */
/* gradient row of that node).  Slots are applied in slot order: grad[dst[t]] = grad[dst[t]] + h^_t, one fp32   */
/* addition per element and slot, so a node that hears from several peers accumulates them in slot order.      */
/* ------------------------------------------------------------------------------------------------------ */
int oracle_unpack_dequant_add(const uint8_t *packed, const float *params,
                              const uint8_t *bits, const int64_t *row_offset, const int32_t *dst_idx,
                              int64_t n_recv, int32_t dim, float *grad, int64_t ld)
{
    if (n_recv < 0 || dim <= 0 || ld < dim) return ORACLE_EINVAL;
    for (int64_t t = 0; t < n_recv; ++t) {
        const int b = bits[t];
        if (b != 2 && b != 4 && b != 8) return ORACLE_EBITS;
        const float Z = params[2 * t + 0], S = params[2 * t + 1];
        const uint8_t *row = packed + row_offset[t];
        float *g = grad + (int64_t)dst_idx[t] * ld;
        for (int32_t j = 0; j < dim; ++j) {
            const int64_t bit = (int64_t)j * b;
            const uint32_t code = ((uint32_t)row[bit >> 3] >> (bit & 7)) & ((1u << b) - 1u);
            const float scaled = (float)code * S;
            const float value = scaled + Z;        /* Eq. 5 */
            g[j] = g[j] + value;
        }
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------------------------------------------ */
/* Neighbour aggregation (Eq. 3, inner sum) over rows [row_begin, row_end) of a CSR matrix, accumulated in   */
/* double in CSR order.  out may be NULL; out64 / abs64 (optional, indexed from row_begin, [rows * dim])     */
/* receive the double sum and the sum of |terms| that scales the comparison tolerance.                      */
/* ------------------------------------------------------------------------------------------------------ */
int oracle_spmm_csr(const int64_t *rowptr, const int32_t *col, const float *val,
                    int64_t row_begin, int64_t row_end,
                    const float *H, int64_t ldh, int32_t dim,
                    float *out, int64_t ldo, double *out64, double *abs64)
{
    if (row_begin < 0 || row_end < row_begin || dim <= 0 || ldh < dim) return ORACLE_EINVAL;
    if (out && ldo < dim) return ORACLE_EINVAL;
    double acc[dim], mag[dim];                      /* one output row at a time */
    for (int64_t v = row_begin; v < row_end; ++v) {
        for (int32_t j = 0; j < dim; ++j) { acc[j] = 0.0; mag[j] = 0.0; }
        for (int64_t k = rowptr[v]; k < rowptr[v + 1]; ++k) {
            const float *h = H + (int64_t)col[k] * ldh;
            for (int32_t j = 0; j < dim; ++j) {
                const double term = (double)val[k] * (double)h[j];
                acc[j] += term;
                mag[j] += fabs(term);
            }
        }
        for (int32_t j = 0; j < dim; ++j) {
            if (out) out[v * ldo + j] = (float)acc[j];
            if (out64) out64[(v - row_begin) * (int64_t)dim + j] = acc[j];
            if (abs64) abs64[(v - row_begin) * (int64_t)dim + j] = mag[j];
        }
    }
    return ORACLE_OK;
}
