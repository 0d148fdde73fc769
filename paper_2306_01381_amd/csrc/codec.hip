// Message codec for gfx950: quantise + pack (Sec. 2.3 Eq. 4, App. A.1, Sec. 5 "Implementation") and
// unpack + de-quantise (Sec. 2.3 Eq. 5).
//
// Both kernels are HBM-streaming: the send side reads 4*dim bytes per slot and writes dim*b/8, the receive
// side does the reverse.  Nothing is a dense contraction, so the matrix cores are not used.
//
// Send side, one pass over memory.  A row of dim floats is cut into "granules" of 8 consecutive columns;
// a granule is the unit of everything: 32 bytes of input, one Philox4x32-10 call (its 128 bits are the
// eight 16-bit rounding values), b bytes of output.  A row is owned by LPR = 2^k lanes of a wave, lane l
// holding granules l, l + LPR, l + 2*LPR, ... (GPL of them) in registers, so that at each step the LPR
// lanes of a row read LPR*32 contiguous bytes.  LPR and GPL are chosen on the host so that LPR*GPL barely
// exceeds dim/8 (D=602: 16 x 5, D=256: 8 x 4, D=300: 8 x 5, D=128: 4 x 4); a wave carries 64/LPR rows.
// min / max are reduced in registers and over the row's lanes with xor shuffles, (Z, S, inv) are computed
// redundantly by every lane, the codes are packed in registers and stored.
// 32-bit integer multiplies issue at full rate on gfx950 (measured), so a Philox call costs about 60 VALU
// issue slots per lane, the rest of a granule about as much again.
//
// fp32 arithmetic is written operation by operation and the file is compiled with -ffp-contract=off: the
// integer codes depend on every rounding.
#include "common.hpp"
#include "adaqp_probe.h"

namespace adaqp {
namespace {

// ---------------------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  The key schedule is wave-uniform (it only depends on the seed).
// ---------------------------------------------------------------------------------------------------------
struct Rand128 { uint32_t w0, w1, w2, w3; };

// a ^ b ^ c in one instruction: gfx950's v_bitop3_b32 with the truth table of the three-input xor (the compiler
// does not form it from two xors)
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
}

__device__ __forceinline__ Rand128 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1)
{
    constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
    constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t pA = (uint64_t)kMulA * c0;            // one v_mad_u64_u32 each
        const uint64_t pB = (uint64_t)kMulB * c2;
        c0 = xor3((uint32_t)(pB >> 32), c1, k0);
        c1 = (uint32_t)pB;
        c2 = xor3((uint32_t)(pA >> 32), c3, k1);
        c3 = (uint32_t)pA;
        k0 += kWeylA;
        k1 += kWeylB;
    }
    return Rand128{c0, c1, c2, c3};
}

constexpr uint32_t kCounterTag = 0x41645150u;


struct QuantArgs {
    const float *feat;
    int64_t n_feat_rows, ld;
    int32_t dim, n_granules;
    const int32_t *send_idx;
    const uint8_t *bits;
    const int64_t *row_offset;
    int64_t n_send;
    uint32_t seed_lo, seed_hi;
    uint8_t *packed;
    int64_t packed_bytes;
    float *params;
    const float *alpha_sq;      // optional trace input / output (both or none)
    float *beta;
    int32_t lpr_log2;
};

template <int VW> struct VecOf;
template <> struct VecOf<1> { using type = float; };
template <> struct VecOf<2> { using type = float2; };
template <> struct VecOf<4> { using type = float4; };

template <int VW>
__device__ __forceinline__ void load_vec(const float *p, float *dst)
{
    using V = typename VecOf<VW>::type;
    const V v = *reinterpret_cast<const V *>(p);
    if constexpr (VW == 1) { dst[0] = v; }
    if constexpr (VW == 2) { dst[0] = v.x; dst[1] = v.y; }
    if constexpr (VW == 4) { dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w; }
}

template <int VW>
__device__ __forceinline__ void store_vec(float *p, const float *src)
{
    using V = typename VecOf<VW>::type;
    if constexpr (VW == 1) { *p = src[0]; }
    if constexpr (VW == 2) { *reinterpret_cast<V *>(p) = make_float2(src[0], src[1]); }
    if constexpr (VW == 4) { *reinterpret_cast<V *>(p) = make_float4(src[0], src[1], src[2], src[3]); }
}

// A row that is read once: the non-temporal hint.
template <int VW>
__device__ __forceinline__ void load_vec_streaming(const float *p, float *dst)
{
    typedef float vec_t __attribute__((ext_vector_type(VW)));
    const vec_t v = __builtin_nontemporal_load(reinterpret_cast<const vec_t *>(p));
#pragma unroll
    for (int k = 0; k < VW; ++k) dst[k] = v[k];
}

// The backward receive reads a gradient row once and writes it back: with whole-line rows both accesses carry the
// non-temporal hint (measured on 102 000 rows of 256 columns: 58 us with ordinary accesses, 55 us with the stores
// alone hinted, 43 us with both).
template <int VW, bool STREAM>
__device__ __forceinline__ void load_row_vec(const float *p, float *dst)
{
    if (STREAM) load_vec_streaming<VW>(p, dst);
    else        load_vec<VW>(p, dst);
}

// Same, marked non-temporal.  For rows that are written once in whole 128-byte lines and not read back by the
// kernel this is worth a quarter of the kernel's time on MI355X (measured: 19.7 -> 15.0 us for 30 000 rows of 602
// columns, 29.7 -> 21.1 us for 120 000 rows of 256): the lines go out without being kept in the L2.
template <int VW>
__device__ __forceinline__ void store_vec_streaming(float *p, const float *src)
{
    typedef float vec_t __attribute__((ext_vector_type(VW)));
    vec_t v;
#pragma unroll
    for (int k = 0; k < VW; ++k) v[k] = src[k];
    __builtin_nontemporal_store(v, reinterpret_cast<vec_t *>(p));
}

// Codes of one granule (8 columns) at width B, merged little-endian into lo (and hi for B == 8).
// The definition is trunc(min((x - Z) * inv, L) * 2^16).  With scale = inv * 2^16 and top = L * 2^16 the last
// multiplication folds into the first: scaling by a power of two commutes with fp32 rounding, so
// trunc(min((x - Z) * scale, top)) is the same integer - as long as inv * 2^16 is an fp32 number.  For the rare
// row where it overflows (range below about 2^-104) TWO_STEP takes the definition as written, with scale = inv
// and top = L; for every other row the two forms agree, so a wave may take either for all its rows.
// MASK: zero the codes of columns >= dim (only the last granule step of a row can need it).
template <int B, bool MASK, bool TWO_STEP>
__device__ __forceinline__ void quantise_granule(const float (&x)[8], float Z, float scale, float top,
                                                 const Rand128 &rnd, int32_t col0, int32_t dim,
                                                 uint32_t &lo, uint32_t &hi)
{
    const uint32_t words[4] = {rnd.w0, rnd.w1, rnd.w2, rnd.w3};
    lo = 0u;
    hi = 0u;
    // Last column first: the code (bits 16 .. 16+B-1 of the sum) is moved to the top of its word and funnelled into
    // the packed word from the right (v_alignbit_b32: shift, extract and merge in one instruction), so column 0
    // ends up in the lowest bits.
#pragma unroll
    for (int k = 7; k >= 0; --k) {
        float pos = (x[k] - Z) * scale;                       // Eq. 4 argument (in 16.16 fixed point), >= 0
        pos = fminf(pos, top);                                // the top element may overshoot by an ulp
        if (TWO_STEP) pos = pos * 65536.0f;
        const uint32_t fixed = (uint32_t)pos;                 // truncated
        const uint32_t r16 = (k & 1) ? (words[k >> 1] >> 16) : (words[k >> 1] & 0xFFFFu);
        uint32_t sum = (fixed + r16) << (16 - B);             // App. A.1: up with probability frac; code = top B bits
        if (MASK) sum = (col0 + k < dim) ? sum : 0u;          // padding bits are zero
        if (B * k < 32) lo = __builtin_amdgcn_alignbit(lo, sum, 32 - B);
        else            hi = __builtin_amdgcn_alignbit(hi, sum, 32 - B);
    }
}

template <int B>
__device__ __forceinline__ void store_granule(uint8_t *row, int32_t g, int32_t n_granules, int64_t stride,
                                              uint32_t lo, uint32_t hi)
{
    if constexpr (B == 2) {
        *reinterpret_cast<uint16_t *>(row + 2 * (int64_t)g) = (uint16_t)lo;
        if (g == n_granules - 1 && 2 * (int64_t)(g + 1) < stride)       // odd granule count: two pad bytes
            *reinterpret_cast<uint16_t *>(row + 2 * (int64_t)(g + 1)) = (uint16_t)0;
    }
    if constexpr (B == 4) {
        *reinterpret_cast<uint32_t *>(row + 4 * (int64_t)g) = lo;
    }
    if constexpr (B == 8) {
        *reinterpret_cast<uint32_t *>(row + 8 * (int64_t)g) = lo;
        if (8 * (int64_t)g + 4 < stride) *reinterpret_cast<uint32_t *>(row + 8 * (int64_t)g + 4) = hi;
    }
}

struct RowScale { float Z, S, inv, inv16, range; };

constexpr float kFltMax = 3.402823466e+38f;

__device__ __forceinline__ RowScale row_scale(float mn, float mx, float levels)
{
    RowScale rs;
    rs.Z = mn + 0.0f;                     // -0 -> +0, so that any reduction order gives the same zero-point
    const float range = (mx + 0.0f) - rs.Z;
    rs.range = range;
    rs.S = 0.0f;
    rs.inv = 0.0f;
    rs.inv16 = 0.0f;
    if (range > 0.0f) {
        const float inv = levels / range;
        if (inv <= kFltMax) {             // else: the reciprocal is not an fp32 number, the row counts as constant
            rs.S = range / levels;        // Eq. 4 scale, correctly rounded fp32 division
            rs.inv = inv;
            rs.inv16 = inv * 65536.0f;    // may overflow: then the wave takes the two-step form
        }
    }
    return rs;
}

// Trace for the bit-width assigner (Sec. 4.2): the numerator of the message's term in the variance objective.
__device__ __forceinline__ float trace_beta(float alpha_sq, int32_t dim, float range)
{
    const float wd = alpha_sq * (float)dim;
    const float r2 = range * range;
    return (wd * r2) / 6.0f;
}

template <int B, int GPL, bool TWO_STEP>
__device__ __forceinline__ void quantise_row(const float (&x)[GPL][8], const Rand128 (&rnd)[GPL],
                                             const RowScale &rs, int lpr, int l, int32_t dim, int32_t n_granules,
                                             uint8_t *row, int64_t stride, bool valid)
{
    const float levels = (float)((1 << B) - 1);
    const float scale = TWO_STEP ? rs.inv : rs.inv16;
    const float top = TWO_STEP ? levels : levels * 65536.0f;
#pragma unroll
    for (int i = 0; i < GPL; ++i) {
        const int32_t g = i * lpr + l;
        uint32_t lo, hi;
        if (i < GPL - 1) quantise_granule<B, false, TWO_STEP>(x[i], rs.Z, scale, top, rnd[i], g * 8, dim, lo, hi);
        else             quantise_granule<B, true, TWO_STEP>(x[i], rs.Z, scale, top, rnd[i], g * 8, dim, lo, hi);
        if (valid && g < n_granules) store_granule<B>(row, g, n_granules, stride, lo, hi);
    }
}

// The widths of a wave's rows: slots are sorted by (peer, width), so nearly every wave holds a single width and
// takes one of the three bodies; a wave on a seam runs the bodies of the widths it holds, each under its lanes.
template <int GPL, bool TWO_STEP>
__device__ __forceinline__ void quantise_rows(const float (&x)[GPL][8], const Rand128 (&rnd)[GPL],
                                              const RowScale &rs, int lpr, int l, int32_t dim, int32_t n_granules,
                                              uint8_t *row, int64_t stride, bool valid, int32_t b)
{
    if (b == 4)      quantise_row<4, GPL, TWO_STEP>(x, rnd, rs, lpr, l, dim, n_granules, row, stride, valid);
    else if (b == 2) quantise_row<2, GPL, TWO_STEP>(x, rnd, rs, lpr, l, dim, n_granules, row, stride, valid);
    else if (b == 8) quantise_row<8, GPL, TWO_STEP>(x, rnd, rs, lpr, l, dim, n_granules, row, stride, valid);
}

// Pins a value to this point of the program: the optimiser may neither sink its computation below nor
// rematerialise it later.
__device__ __forceinline__ void pin(Rand128 &r)
{
    asm volatile("" : "+v"(r.w0), "+v"(r.w1), "+v"(r.w2), "+v"(r.w3));
}

// ---------------------------------------------------------------------------------------------------------
// Register-resident rows: GPL granules per lane, LPR = 2^lpr_log2 lanes per row, 64/LPR rows per wave.
// Order of work inside a wave: (1) issue the loads of the slots' index entries; (2) with four or more granules
// per lane, run Philox for the first two while those are in flight - the rounding values depend only on (seed,
// slot, column), not on memory; (3) issue all row loads; (4) Philox for the remaining granules while the rows
// stream in; (5) min / max, scale, codes, stores.
// ---------------------------------------------------------------------------------------------------------
// PROBE: the measurement twin - the same grid, index loads, row loads and stores (same instructions, same
// addresses), but no generator, no min / max reduction, no codes: what is stored is derived from the loaded values
// with two operations per granule.  Its time is the floor of this access pattern.
template <int GPL, int VW, bool PROBE>
__global__ __launch_bounds__(kBlock) void quantize_pack_kernel(const QuantArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int lpr = 1 << a.lpr_log2;
    const int rows_per_wave = kWave >> a.lpr_log2;
    const int64_t s = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * rows_per_wave + (lane >> a.lpr_log2);
    const int l = lane & (lpr - 1);

    // (1) the slot's index entries
    const bool in_range = s < a.n_send;
    const int64_t s_safe = in_range ? s : 0;
    const int32_t r_raw = a.send_idx[s_safe];
    const int32_t b = a.bits[s_safe];
    const int64_t off = a.row_offset[s_safe];

    // (2) rounding values of the lane's first granules (the barriers and pins keep the compiler from sinking
    // the arithmetic behind the wait for the rows)
    constexpr int kEarly = (PROBE || GPL <= 3) ? 0 : 2;  // light waves: the row loads go out first, the generator runs under them
    Rand128 rnd[GPL];
    const uint32_t s_lo = (uint32_t)s, s_hi = (uint32_t)((uint64_t)s >> 32);
#pragma unroll
    for (int i = 0; i < kEarly; ++i) {
        rnd[i] = philox4x32_10((uint32_t)(i * lpr + l), s_lo, s_hi, kCounterTag, a.seed_lo, a.seed_hi);
        pin(rnd[i]);
    }

    const int64_t stride = 4 * (((int64_t)a.dim * b + 31) >> 5);
    const bool valid = in_range && r_raw >= 0 && r_raw < a.n_feat_rows && (b == 2 || b == 4 || b == 8) &&
                       off >= 0 && (off & 3) == 0 && off + stride <= a.packed_bytes;
    // lanes without a valid slot read row 0 and store nothing: every load below is unconditional
    const float *h = a.feat + (valid ? (int64_t)r_raw * a.ld : 0);

    // (3) gather the lane's granules.  Only the last step can reach past the row; there the column is clamped
    // to the vector holding the row's last element, and elements past dim (row padding, the pitch is a
    // multiple of VW) are replaced by that vector's first element: only real elements enter min and max.
    float x[GPL][8];
    const int32_t last_vec = ((a.dim - 1) / VW) * VW;
#pragma unroll
    for (int i = 0; i < GPL; ++i) {
        const int32_t c0 = (i * lpr + l) * 8;
#pragma unroll
        for (int v = 0; v < 8 / VW; ++v) {
            int32_t c = c0 + v * VW;
            if (i == GPL - 1) c = c < last_vec ? c : last_vec;
            load_vec<VW>(h + c, &x[i][v * VW]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (PROBE) {
        float m = x[0][0];
#pragma unroll
        for (int i = 0; i < GPL; ++i) m = fmaxf(m, x[i][3]);
        if (valid && l == 0) *reinterpret_cast<float2 *>(a.params + 2 * s) = make_float2(m, m);
        uint8_t *prow = a.packed + (valid ? off : 0);
#pragma unroll
        for (int i = 0; i < GPL; ++i) {
            const int32_t g = i * lpr + l;
            const uint32_t word = __builtin_bit_cast(uint32_t, x[i][0]) ^ __builtin_bit_cast(uint32_t, x[i][5]);
            if (valid && g < a.n_granules) {
                if (b == 4)      store_granule<4>(prow, g, a.n_granules, stride, word, word);
                else if (b == 2) store_granule<2>(prow, g, a.n_granules, stride, word, word);
                else             store_granule<8>(prow, g, a.n_granules, stride, word, word);
            }
        }
        return;
    }
    // (4)
#pragma unroll
    for (int i = kEarly; i < GPL; ++i) {
        rnd[i] = philox4x32_10((uint32_t)(i * lpr + l), s_lo, s_hi, kCounterTag, a.seed_lo, a.seed_hi);
        pin(rnd[i]);
    }
    __builtin_amdgcn_sched_barrier(0);

    // (5) row minimum / maximum
    if (VW > 1) {
        const int32_t c0 = ((GPL - 1) * lpr + l) * 8;
#pragma unroll
        for (int v = 0; v < 8 / VW; ++v) {
            int32_t c = c0 + v * VW;
            c = c < last_vec ? c : last_vec;
#pragma unroll
            for (int k = 1; k < VW; ++k)
                if (c + k >= a.dim) x[GPL - 1][v * VW + k] = x[GPL - 1][v * VW];
        }
    }
    float mn = x[0][0], mx = x[0][0];
#pragma unroll
    for (int i = 0; i < GPL; ++i)
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            mn = fminf(mn, x[i][k]);
            mx = fmaxf(mx, x[i][k]);
        }
    for (int m = 1; m < lpr; m <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, m, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, m, kWave));
    }
    if (__ballot(valid) == 0) return;

    const float levels = (float)((1 << (b & 15)) - 1);
    const RowScale rs = row_scale(mn, mx, levels);
    // a row whose scale overflows once the 2^16 is folded in sends its whole wave down the two-step form
    const bool two_step = __ballot(valid && !(rs.inv16 <= kFltMax)) != 0;      // no cross-lane operation below
    if (valid && l == 0) {
        *reinterpret_cast<float2 *>(a.params + 2 * s) = make_float2(rs.Z, rs.S);
        if (a.beta) a.beta[s] = trace_beta(a.alpha_sq[s], a.dim, rs.range);
    }

    uint8_t *row = a.packed + (valid ? off : 0);
    if (!two_step) quantise_rows<GPL, false>(x, rnd, rs, lpr, l, a.dim, a.n_granules, row, stride, valid, b);
    else           quantise_rows<GPL, true>(x, rnd, rs, lpr, l, a.dim, a.n_granules, row, stride, valid, b);
}

// ---------------------------------------------------------------------------------------------------------
// Rows too wide for registers (dim > 8 * 64 * kMaxGpl): one wave per row, two passes over the row (the
// second one is served by the caches).
// ---------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void quantize_pack_wide_kernel(const QuantArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t s = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);     // wave-uniform
    if (s >= a.n_send) return;
    const int32_t r = a.send_idx[s];
    const int32_t b = a.bits[s];
    const int64_t off = a.row_offset[s];
    const int64_t stride = 4 * (((int64_t)a.dim * b + 31) >> 5);
    if (!(r >= 0 && r < a.n_feat_rows && (b == 2 || b == 4 || b == 8) && off >= 0 && (off & 3) == 0 &&
          off + stride <= a.packed_bytes))
        return;
    const float *h = a.feat + (int64_t)r * a.ld;

    float mn = h[0], mx = mn;
    for (int32_t c = lane; c < a.dim; c += kWave) {
        const float v = h[c];
        mn = fminf(mn, v);
        mx = fmaxf(mx, v);
    }
    for (int m = 1; m < kWave; m <<= 1) {
        mn = fminf(mn, __shfl_xor(mn, m, kWave));
        mx = fmaxf(mx, __shfl_xor(mx, m, kWave));
    }
    const float levels = (float)((1 << b) - 1);
    const RowScale rs = row_scale(mn, mx, levels);
    const bool two_step = !(rs.inv16 <= kFltMax);                       // wave-uniform: one row per wave
    const float scale = two_step ? rs.inv : rs.inv16;
    const float top = two_step ? levels : levels * 65536.0f;
    if (lane == 0) {
        *reinterpret_cast<float2 *>(a.params + 2 * s) = make_float2(rs.Z, rs.S);
        if (a.beta) a.beta[s] = trace_beta(a.alpha_sq[s], a.dim, rs.range);
    }

    uint8_t *row = a.packed + off;
    const uint32_t s_lo = (uint32_t)s, s_hi = (uint32_t)((uint64_t)s >> 32);
    for (int32_t g = lane; g < a.n_granules; g += kWave) {
        float x[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) x[k] = (g * 8 + k < a.dim) ? h[g * 8 + k] : mn;
        const Rand128 rnd = philox4x32_10((uint32_t)g, s_lo, s_hi, kCounterTag, a.seed_lo, a.seed_hi);
        uint32_t lo, hi;
        if (b == 4) {
            if (two_step) quantise_granule<4, true, true>(x, rs.Z, scale, top, rnd, g * 8, a.dim, lo, hi);
            else          quantise_granule<4, true, false>(x, rs.Z, scale, top, rnd, g * 8, a.dim, lo, hi);
            store_granule<4>(row, g, a.n_granules, stride, lo, hi);
        } else if (b == 2) {
            if (two_step) quantise_granule<2, true, true>(x, rs.Z, scale, top, rnd, g * 8, a.dim, lo, hi);
            else          quantise_granule<2, true, false>(x, rs.Z, scale, top, rnd, g * 8, a.dim, lo, hi);
            store_granule<2>(row, g, a.n_granules, stride, lo, hi);
        } else {
            if (two_step) quantise_granule<8, true, true>(x, rs.Z, scale, top, rnd, g * 8, a.dim, lo, hi);
            else          quantise_granule<8, true, false>(x, rs.Z, scale, top, rnd, g * 8, a.dim, lo, hi);
            store_granule<8>(row, g, a.n_granules, stride, lo, hi);
        }
    }
}

// ---------------------------------------------------------------------------------------------------------
// Receive side.  A lane turns VW consecutive codes into VW floats and stores them as one vector, so a wave
// writes 64*VW*4 contiguous bytes per step; VW*b divides 32, so the codes of one vector never straddle a
// 32-bit word of the packed row.  A wave owns R consecutive slots, R chosen so that it writes about 4 KB (light
// waves stream best here): their index entries are fetched in one go, then all R*NV packed words are requested
// before the first one is decoded, so a wave pays two memory latencies for R rows.
// ---------------------------------------------------------------------------------------------------------
struct DequantArgs {
    const uint8_t *packed;
    int64_t packed_bytes;
    const float *params;
    const uint8_t *bits;
    const int64_t *row_offset;
    const int32_t *halo_idx;
    const int32_t *order;       // optional: slot handled at position k (ascending destination rows)
    int64_t n_recv;
    int32_t dim, write_dim;     // write_dim > dim: columns [dim, write_dim) receive zeros (whole 128-byte lines)
    float *feat;
    int64_t n_feat_rows, ld;
};

__device__ __forceinline__ int64_t readlane_i64(int64_t v, int lane_id)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int32_t)(uint32_t)v, lane_id);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int32_t)(uint32_t)((uint64_t)v >> 32), lane_id);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// SCALAR: the wave's slot numbers are wave-uniform, so the index entries of its R slots can come through the scalar
// cache (R <= 2); otherwise lanes 0..R-1 fetch them with one vector load each and broadcast them (R = 4).
// STREAM: rows are written in whole lines (line-padded layout): non-temporal stores.
template <int VW, int NV, int R, bool SCALAR, bool STREAM>
__global__ __launch_bounds__(kBlock) void unpack_dequant_kernel(const DequantArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int64_t t0 = ((int64_t)blockIdx.x * kWavesPerBlock + wave) * R;                    // wave-uniform
    if (t0 >= a.n_recv) return;

    int32_t r_of[R], b_of[R];
    int64_t off_of[R];
    float z_of[R], s_of[R];
    if (SCALAR) {
#pragma unroll
        for (int k = 0; k < R; ++k) {
            int64_t t = t0 + k < a.n_recv ? t0 + k : a.n_recv - 1;
            bool in_list = t0 + k < a.n_recv;
            if (a.order) {
                const int32_t o = a.order[t];
                in_list = in_list && o >= 0 && o < a.n_recv;
                t = in_list ? o : 0;
            }
            const int32_t r = a.halo_idx[t];
            const int32_t b = a.bits[t];
            const int64_t off = a.row_offset[t];
            const float2 zs = *reinterpret_cast<const float2 *>(a.params + 2 * t);
            const int64_t stride = 4 * (((int64_t)a.dim * b + 31) >> 5);
            const bool ok = in_list && r >= 0 && r < a.n_feat_rows && (b == 2 || b == 4 || b == 8) && off >= 0 &&
                            (off & 3) == 0 && off + stride <= a.packed_bytes;
            r_of[k] = ok ? r : -1;
            b_of[k] = b;
            off_of[k] = off;
            z_of[k] = zs.x;
            s_of[k] = zs.y;
        }
    } else {
        // lane k < R: index entries of the slot at position t0 + k
        int64_t t_mine = t0 + lane < a.n_recv ? t0 + lane : a.n_recv - 1;
        int32_t my_r = -1, my_b = 0;
        int64_t my_off = 0;
        float my_z = 0.0f, my_s = 0.0f;
        if (lane < R) {
            bool in_list = true;
            if (a.order) {
                const int32_t o = a.order[t_mine];
                in_list = o >= 0 && o < a.n_recv;
                t_mine = in_list ? o : 0;
            }
            my_r = a.halo_idx[t_mine];
            my_b = a.bits[t_mine];
            my_off = a.row_offset[t_mine];
            const float2 zs = *reinterpret_cast<const float2 *>(a.params + 2 * t_mine);
            my_z = zs.x;
            my_s = zs.y;
            const int64_t stride = 4 * (((int64_t)a.dim * my_b + 31) >> 5);
            const bool ok = in_list && t0 + lane < a.n_recv && my_r >= 0 && my_r < a.n_feat_rows &&
                            (my_b == 2 || my_b == 4 || my_b == 8) && my_off >= 0 && (my_off & 3) == 0 &&
                            my_off + stride <= a.packed_bytes;
            if (!ok) my_r = -1;
        }
#pragma unroll
        for (int k = 0; k < R; ++k) {
            r_of[k] = __builtin_amdgcn_readlane(my_r, k);
            b_of[k] = __builtin_amdgcn_readlane(my_b, k);
            off_of[k] = readlane_i64(my_off, k);
            z_of[k] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_z), k));
            s_of[k] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_s), k));
        }
    }

    const bool last_ok = ((NV - 1) * kWave + lane) * VW < a.write_dim;
    // Every packed word is requested before the first one is looked at.  The loads are unconditional (a lane
    // past the row re-reads the row's last word, a skipped slot reads the buffer's first word) so that they
    // form one straight run of instructions with a single wait behind it.
    uint32_t w[R][NV];
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int32_t r = r_of[k];
        const uint32_t *words = reinterpret_cast<const uint32_t *>(a.packed + (r >= 0 ? off_of[k] : 0));
        const uint32_t last_word = r >= 0 ? (uint32_t)(((int64_t)a.dim * b_of[k] - 1) >> 5) : 0u;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const uint32_t bit = (uint32_t)((v * kWave + lane) * VW) * (uint32_t)b_of[k];
            const uint32_t idx = (bit >> 5) < last_word ? (bit >> 5) : last_word;
            w[k][v] = words[idx];
        }
    }
#pragma unroll
    for (int k = 0; k < R; ++k) {
        const int32_t r = r_of[k];
        if (r < 0) continue;
        const float Z = z_of[k], S = s_of[k];
        const int32_t b = b_of[k];
        const uint32_t mask = (1u << b) - 1u;
        float *h = a.feat + (int64_t)r * a.ld;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (v < NV - 1 || last_ok) {
                float y[VW];
                const uint32_t bit = (uint32_t)((v * kWave + lane) * VW) * (uint32_t)b;
                const uint32_t word = w[k][v] >> (bit & 31u);
#pragma unroll
                for (int q = 0; q < VW; ++q) {
                    const uint32_t code = (word >> (q * b)) & mask;
                    const float scaled = (float)code * S;          // Eq. 5: product rounded, then sum rounded
                    y[q] = scaled + Z;
                    if (v == NV - 1 && (v * kWave + lane) * VW + q >= a.dim) y[q] = 0.0f;   // row padding
                }
                if (STREAM) store_vec_streaming<VW>(h + (v * kWave + lane) * VW, y);
                else        store_vec<VW>(h + (v * kWave + lane) * VW, y);
            }
        }
    }
}

// Any row length: one wave per slot, looping over the row.
template <int VW>
__global__ __launch_bounds__(kBlock) void unpack_dequant_long_kernel(const DequantArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    int64_t t = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);           // wave-uniform
    if (t >= a.n_recv) return;
    if (a.order) {
        t = a.order[t];
        if (t < 0 || t >= a.n_recv) return;
    }
    const int32_t r = a.halo_idx[t];
    const int32_t b = a.bits[t];
    const int64_t off = a.row_offset[t];
    const int64_t stride = 4 * (((int64_t)a.dim * b + 31) >> 5);
    if (!(r >= 0 && r < a.n_feat_rows && (b == 2 || b == 4 || b == 8) && off >= 0 && (off & 3) == 0 &&
          off + stride <= a.packed_bytes))
        return;
    const float2 zs = *reinterpret_cast<const float2 *>(a.params + 2 * t);
    const float Z = zs.x, S = zs.y;
    const uint32_t *words = reinterpret_cast<const uint32_t *>(a.packed + off);
    float *h = a.feat + (int64_t)r * a.ld;
    const uint32_t mask = (1u << b) - 1u;

    for (int32_t c = lane * VW; c < a.dim; c += kWave * VW) {
        const uint32_t bit = (uint32_t)c * (uint32_t)b;
        const uint32_t w = words[bit >> 5] >> (bit & 31u);
        float y[VW];
#pragma unroll
        for (int k = 0; k < VW; ++k) {
            const uint32_t code = (w >> (k * b)) & mask;
            const float scaled = (float)code * S;          // Eq. 5: product rounded, then sum rounded
            y[k] = scaled + Z;
        }
        store_vec<VW>(h + c, y);
    }
    for (int32_t c = a.dim + lane; c < a.write_dim; c += kWave) h[c] = 0.0f;           // row padding
}

// ---------------------------------------------------------------------------------------------------------
// Backward receive: one wave per destination row.  The slots that target the row (a node hears from every peer
// that holds it as a halo node) were grouped on the host; the wave stages their index entries in lanes, loads
// the row, adds the de-quantised messages in slot order (one fp32 addition per slot and element: the order is
// part of the result) and stores the row once.  Rows wider than 64*VW*4 columns are walked in column chunks.
// ---------------------------------------------------------------------------------------------------------
struct DequantAddArgs {
    const uint8_t *packed;
    int64_t packed_bytes;
    const float *params;
    const uint8_t *bits;
    const int64_t *row_offset;
    const int32_t *dst_idx;
    int64_t n_recv;
    const int32_t *seg_order;
    const int64_t *seg_ptr;
    int64_t n_seg;
    int32_t dim;
    float *grad;
    int64_t n_grad_rows, ld;
};

// One destination segment g, worked on by a whole wave.
template <int VW, int NV, bool STREAM>       // NV: vectors per lane and column chunk; STREAM: non-temporal row stores
__device__ void add_one_segment(const DequantAddArgs &a, int64_t g, int lane)
{
    constexpr int G = 4;        // slots whose packed words are requested together
    int64_t k0 = a.seg_ptr[g], k1 = a.seg_ptr[g + 1];
    k0 = k0 < 0 ? 0 : (k0 > a.n_recv ? a.n_recv : k0);
    k1 = k1 < k0 ? k0 : (k1 > a.n_recv ? a.n_recv : k1);
    if (k0 >= k1) return;

    int32_t r = -1;             // the segment's destination row: that of its first slot
    float *row = nullptr;
    for (int32_t c0 = 0; c0 < a.dim; c0 += kWave * VW * NV) {
        float acc[NV][VW];
        for (int64_t win = k0; win < k1; win += kWave) {
            // index entries of up to 64 slots of the segment: lane j <-> slot win + j ("skip" = width 0)
            const int32_t n_win = (int32_t)(k1 - win < kWave ? k1 - win : kWave);
            int32_t my_t = -1, my_dst = -1, my_b = 0;
            int64_t my_off = 0;
            float my_z = 0.0f, my_s = 0.0f;
            if (lane < n_win) {
                my_t = a.seg_order[win + lane];
                if (my_t >= 0 && my_t < a.n_recv) {
                    my_dst = a.dst_idx[my_t];
                    my_b = a.bits[my_t];
                    my_off = a.row_offset[my_t];
                    const float2 zs = *reinterpret_cast<const float2 *>(a.params + 2 * (int64_t)my_t);
                    my_z = zs.x;
                    my_s = zs.y;
                }
            }
            if (win == k0) {
                r = __builtin_amdgcn_readlane(my_dst, 0);
                if (r < 0 || r >= a.n_grad_rows) return;
                row = a.grad + (int64_t)r * a.ld;
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    const int32_t c = c0 + (v * kWave + lane) * VW;
#pragma unroll
                    for (int q = 0; q < VW; ++q) acc[v][q] = 0.0f;
                    if (c < a.dim) load_row_vec<VW, STREAM>(row + c, acc[v]);
                }
            }
            {
                const int64_t stride = 4 * (((int64_t)a.dim * my_b + 31) >> 5);
                const bool ok = my_dst == r && (my_b == 2 || my_b == 4 || my_b == 8) && my_off >= 0 &&
                                (my_off & 3) == 0 && my_off + stride <= a.packed_bytes;
                if (!ok) { my_b = 0; my_off = 0; }
            }
            for (int32_t j0 = 0; j0 < n_win; j0 += G) {
                // packed words of up to G slots in one run of loads (a skipped slot reads the buffer's first word)
                uint32_t w[G][NV];
#pragma unroll
                for (int u = 0; u < G; ++u) {
                    const int32_t j = j0 + u < n_win ? j0 + u : n_win - 1;
                    const int32_t b = __builtin_amdgcn_readlane(my_b, j);
                    const int64_t off = readlane_i64(my_off, j);
                    const uint32_t *words = reinterpret_cast<const uint32_t *>(a.packed + off);
                    const uint32_t last_word = b ? (uint32_t)(((int64_t)a.dim * b - 1) >> 5) : 0u;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const uint32_t bit = (uint32_t)(c0 + (v * kWave + lane) * VW) * (uint32_t)b;
                        const uint32_t idx = (bit >> 5) < last_word ? (bit >> 5) : last_word;
                        w[u][v] = words[idx];
                    }
                }
#pragma unroll
                for (int u = 0; u < G; ++u) {
                    if (j0 + u >= n_win) break;
                    const int32_t b = __builtin_amdgcn_readlane(my_b, j0 + u);
                    if (b == 0) continue;
                    const float Z = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_z), j0 + u));
                    const float S = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_s), j0 + u));
                    const uint32_t mask = (1u << b) - 1u;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const uint32_t bit = (uint32_t)(c0 + (v * kWave + lane) * VW) * (uint32_t)b;
                        const uint32_t word = w[u][v] >> (bit & 31u);
#pragma unroll
                        for (int q = 0; q < VW; ++q) {
                            const uint32_t code = (word >> (q * b)) & mask;
                            const float scaled = (float)code * S;      // Eq. 5: product rounded, then sum rounded
                            const float value = scaled + Z;
                            acc[v][q] = acc[v][q] + value;
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int32_t c = c0 + (v * kWave + lane) * VW;
            if (c < a.dim) {
                if (STREAM) store_vec_streaming<VW>(row + c, acc[v]);
                else        store_vec<VW>(row + c, acc[v]);
            }
        }
    }
}

template <int VW, int NV, bool STREAM>
__global__ __launch_bounds__(kBlock) void unpack_dequant_add_kernel(const DequantAddArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t g = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);             // wave-uniform
    if (g >= a.n_seg) return;
    add_one_segment<VW, NV, STREAM>(a, g, lane);
}

// Rows of at most two vectors per lane: a wave takes S = 4 consecutive segments at once.  Most destination rows
// hear from one or two peers, so a wave per row spends its life waiting on a chain of dependent loads (segment
// bounds -> slot numbers -> index entries -> row and packed words); here the chain is walked once for S rows,
// and their row loads and packed words are all in flight together.  Same arithmetic and order per row as above.
// PROBE: the no-compute twin - the same loads and stores at the same addresses, but a message's words are xor-ed
// into its row instead of being decoded and added (the rows end up holding meaningless bits).
template <int VW, int NV, int S, bool STREAM, bool PROBE>
__global__ __launch_bounds__(kBlock) void unpack_dequant_add4_kernel(const DequantAddArgs a)
{
    constexpr int G = 4;
    static_assert(NV * S <= 8, "register budget: S rows of NV vectors");
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t g0 = ((int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)) * S;      // wave-uniform
    if (g0 >= a.n_seg) return;
    const int ns = (int)(a.n_seg - g0 < S ? a.n_seg - g0 : S);

    // segment bounds, clamped and made monotone
    int64_t my_sp = 0;
    if (lane <= ns) {
        my_sp = a.seg_ptr[g0 + lane];
        my_sp = my_sp < 0 ? 0 : (my_sp > a.n_recv ? a.n_recv : my_sp);
    }
    int64_t sp[S + 1];
    sp[0] = readlane_i64(my_sp, 0);
#pragma unroll
    for (int i = 1; i <= S; ++i) {
        const int64_t v = i <= ns ? readlane_i64(my_sp, i) : sp[i - 1];
        sp[i] = v < sp[i - 1] ? sp[i - 1] : v;
    }
    const int64_t total = sp[S] - sp[0];
    if (total <= 0) return;
    if (total > kWave) {                                    // a crowd on one of the rows: one segment at a time
        for (int i = 0; i < ns; ++i) add_one_segment<VW, NV, STREAM>(a, g0 + i, lane);
        return;
    }
    const int n_win = (int)total;

    // index entries: lane j <-> slot sp[0] + j
    int32_t my_t = -1, my_dst = -1, my_b = 0, my_seg = 0;
    int64_t my_off = 0;
    float my_z = 0.0f, my_s = 0.0f;
    if (lane < n_win) {
        my_t = a.seg_order[sp[0] + lane];
#pragma unroll
        for (int i = 1; i < S; ++i) my_seg += sp[i] <= sp[0] + lane ? 1 : 0;
        if (my_t >= 0 && my_t < a.n_recv) {
            my_dst = a.dst_idx[my_t];
            my_b = a.bits[my_t];
            my_off = a.row_offset[my_t];
            const float2 zs = *reinterpret_cast<const float2 *>(a.params + 2 * (int64_t)my_t);
            my_z = zs.x;
            my_s = zs.y;
        }
    }
    // each segment's destination row is that of its first slot; its rows are requested before any packed word
    int32_t r[S];
    bool live[S];
    float acc[S][NV][VW];
    int32_t my_r = -1;
#pragma unroll
    for (int i = 0; i < S; ++i) {
        live[i] = sp[i + 1] > sp[i];
        r[i] = live[i] ? __builtin_amdgcn_readlane(my_dst, (int)(sp[i] - sp[0])) : -1;
        live[i] = live[i] && r[i] >= 0 && r[i] < a.n_grad_rows;
        if (my_seg == i) my_r = live[i] ? r[i] : -1;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int32_t c = (v * kWave + lane) * VW;
#pragma unroll
            for (int q = 0; q < VW; ++q) acc[i][v][q] = 0.0f;
            if (live[i] && c < a.dim) load_row_vec<VW, STREAM>(a.grad + (int64_t)r[i] * a.ld + c, acc[i][v]);
        }
    }
    {
        const int64_t stride = 4 * (((int64_t)a.dim * my_b + 31) >> 5);
        const bool ok = lane < n_win && my_r >= 0 && my_dst == my_r && (my_b == 2 || my_b == 4 || my_b == 8) &&
                        my_off >= 0 && (my_off & 3) == 0 && my_off + stride <= a.packed_bytes;
        if (!ok) { my_b = 0; my_off = 0; }
    }
    for (int32_t j0 = 0; j0 < n_win; j0 += G) {
        uint32_t w[G][NV];
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const int32_t j = j0 + u < n_win ? j0 + u : n_win - 1;
            const int32_t b = __builtin_amdgcn_readlane(my_b, j);
            const int64_t off = readlane_i64(my_off, j);
            const uint32_t *words = reinterpret_cast<const uint32_t *>(a.packed + off);
            const uint32_t last_word = b ? (uint32_t)(((int64_t)a.dim * b - 1) >> 5) : 0u;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const uint32_t bit = (uint32_t)((v * kWave + lane) * VW) * (uint32_t)b;
                const uint32_t idx = (bit >> 5) < last_word ? (bit >> 5) : last_word;
                w[u][v] = words[idx];
            }
        }
#pragma unroll
        for (int u = 0; u < G; ++u) {
            if (j0 + u >= n_win) break;
            const int32_t b = __builtin_amdgcn_readlane(my_b, j0 + u);
            if (b == 0) continue;
            const int32_t seg = __builtin_amdgcn_readlane(my_seg, j0 + u);
            if (PROBE) {
#pragma unroll
                for (int i = 0; i < S; ++i)
                    if (seg == i)
#pragma unroll
                        for (int v = 0; v < NV; ++v)
                            acc[i][v][0] = __builtin_bit_cast(float, __builtin_bit_cast(uint32_t, acc[i][v][0]) ^ w[u][v]);
                continue;
            }
            const float Z = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_z), j0 + u));
            const float Sc = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_s), j0 + u));
            const uint32_t mask = (1u << b) - 1u;
            float value[NV][VW];
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const uint32_t bit = (uint32_t)((v * kWave + lane) * VW) * (uint32_t)b;
                const uint32_t word = w[u][v] >> (bit & 31u);
#pragma unroll
                for (int q = 0; q < VW; ++q) {
                    const uint32_t code = (word >> (q * b)) & mask;
                    const float scaled = (float)code * Sc;      // Eq. 5: product rounded, then sum rounded
                    value[v][q] = scaled + Z;
                }
            }
#pragma unroll
            for (int i = 0; i < S; ++i)
                if (seg == i)                                   // wave-uniform
#pragma unroll
                    for (int v = 0; v < NV; ++v)
#pragma unroll
                        for (int q = 0; q < VW; ++q) acc[i][v][q] = acc[i][v][q] + value[v][q];
        }
    }
#pragma unroll
    for (int i = 0; i < S; ++i) {
        if (!live[i]) continue;
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int32_t c = (v * kWave + lane) * VW;
            if (c < a.dim) {
                if (STREAM) store_vec_streaming<VW>(a.grad + (int64_t)r[i] * a.ld + c, acc[i][v]);
                else        store_vec<VW>(a.grad + (int64_t)r[i] * a.ld + c, acc[i][v]);
            }
        }
    }
}

constexpr int kMaxGpl = 8;

// Largest vector width (floats) such that every row start is naturally aligned.  `whole_vectors`: the width
// must also divide dim (needed where a vector may not spill into the row's padding).
int vector_width(const void *base, int64_t ld, int32_t dim, bool whole_vectors)
{
    if (ld % 4 == 0 && aligned_to(base, 16) && (!whole_vectors || dim % 4 == 0)) return 4;
    if (ld % 2 == 0 && aligned_to(base, 8) && (!whole_vectors || dim % 2 == 0)) return 2;
    return 1;
}

// Rows start on 128-byte lines and the pitch is a whole number of lines: the layout this library is built for.
bool line_padded(const void *base, int64_t ld) { return ld % 32 == 0 && aligned_to(base, 128); }

template <int VW, bool PROBE = false>
hipError_t launch_quantize(const QuantArgs &a, int gpl, dim3 grid, hipStream_t st)
{
    switch (gpl) {
#define ADAQP_CASE(G) case G: hipLaunchKernelGGL((quantize_pack_kernel<G, VW, PROBE>), grid, dim3(kBlock), 0, st, a); break;
        ADAQP_CASE(1) ADAQP_CASE(2) ADAQP_CASE(3) ADAQP_CASE(4)
        ADAQP_CASE(5) ADAQP_CASE(6) ADAQP_CASE(7) ADAQP_CASE(8)
#undef ADAQP_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

constexpr int kMaxDequantNv = 8;

// Slots per wave on the receive side: four rows of one vector per lane, two of two, else one (measured on 256-,
// 300- and 602-column rows: 21.1 / 19.5 / 14.4 us against 25.4 / 21.1 / 15.0 us for the next best choice).
inline int dequant_rows_per_wave(int nv) { return nv == 1 ? 4 : (nv == 2 ? 2 : 1); }

template <int VW, bool STREAM>
hipError_t launch_dequant(const DequantArgs &a, int nv, int64_t n_waves, hipStream_t st)
{
    const dim3 grid((unsigned)((n_waves + kWavesPerBlock - 1) / kWavesPerBlock));
    switch (nv) {
        case 1: hipLaunchKernelGGL((unpack_dequant_kernel<VW, 1, 4, false, STREAM>), grid, dim3(kBlock), 0, st, a); break;
        case 2: hipLaunchKernelGGL((unpack_dequant_kernel<VW, 2, 2, true, STREAM>), grid, dim3(kBlock), 0, st, a); break;
#define ADAQP_CASE(N) case N: hipLaunchKernelGGL((unpack_dequant_kernel<VW, N, 1, true, STREAM>), grid, dim3(kBlock), 0, st, a); break;
        ADAQP_CASE(3) ADAQP_CASE(4) ADAQP_CASE(5) ADAQP_CASE(6) ADAQP_CASE(7) ADAQP_CASE(8)
#undef ADAQP_CASE
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace
}  // namespace adaqp

using namespace adaqp;

extern "C" int adaqp_quantize_pack(const float *feat_dev, int64_t n_feat_rows, int64_t ld, int32_t dim,
                                   const int32_t *send_idx_dev, const uint8_t *bits_dev,
                                   const int64_t *row_offset_dev, int64_t n_send, uint64_t seed,
                                   uint8_t *packed_dev, int64_t packed_bytes, float *params_dev, void *stream)
{
    return adaqp_quantize_pack_trace(feat_dev, n_feat_rows, ld, dim, send_idx_dev, bits_dev, row_offset_dev, n_send,
                                     seed, packed_dev, packed_bytes, params_dev, nullptr, nullptr, stream);
}

namespace {

// Argument checks, launch shape and launch of the send side; `probe` launches the measurement twin of the kernel.
int quantize_pack_launch(const float *feat_dev, int64_t n_feat_rows, int64_t ld, int32_t dim,
                         const int32_t *send_idx_dev, const uint8_t *bits_dev, const int64_t *row_offset_dev,
                         int64_t n_send, uint64_t seed, uint8_t *packed_dev, int64_t packed_bytes, float *params_dev,
                         const float *alpha_sq_dev, float *beta_dev, void *stream, bool probe)
{
    if ((alpha_sq_dev == nullptr) != (beta_dev == nullptr)) return ADAQP_EINVAL;
    if (!aligned_to(alpha_sq_dev, 4) || !aligned_to(beta_dev, 4)) return ADAQP_EINVAL;
    if (n_send < 0 || dim <= 0 || ld < dim || n_feat_rows < 0 || packed_bytes < 0) return ADAQP_EINVAL;
    if (n_send == 0) return ADAQP_OK;
    if (!feat_dev || !send_idx_dev || !bits_dev || !row_offset_dev || !packed_dev || !params_dev)
        return ADAQP_EINVAL;
    if (n_feat_rows == 0) return ADAQP_EINVAL;
    if (!aligned_to(feat_dev, 4) || !aligned_to(params_dev, 8) || !aligned_to(packed_dev, 4) ||
        !aligned_to(send_idx_dev, 4) || !aligned_to(row_offset_dev, 8))
        return ADAQP_EINVAL;
    if (n_send > ((int64_t)1 << 40)) return ADAQP_ESIZE;

    QuantArgs a;
    a.feat = feat_dev;
    a.n_feat_rows = n_feat_rows;
    a.ld = ld;
    a.dim = dim;
    a.n_granules = (dim + 7) / 8;
    a.send_idx = send_idx_dev;
    a.bits = bits_dev;
    a.row_offset = row_offset_dev;
    a.n_send = n_send;
    a.seed_lo = (uint32_t)seed;
    a.seed_hi = (uint32_t)(seed >> 32);
    a.packed = packed_dev;
    a.packed_bytes = packed_bytes;
    a.params = params_dev;
    a.alpha_sq = alpha_sq_dev;
    a.beta = beta_dev;
    a.lpr_log2 = 0;
    hipStream_t st = (hipStream_t)stream;

    // Lanes per row / granules per lane.  Light waves do best (measured on c1-c4-shaped inputs: a wave that carries 2-5
    // KB of rows beats one that carries 8-10 KB by 3-6 %): two or three granules per lane if that leaves at most a
    // quarter of the lanes' granule slots idle (602 columns -> 32 x 3, 300 -> 16 x 3, 256 -> 16 x 2, 128 -> 8 x 2);
    // otherwise least padding first, then the count closest to four granules.
    int best_k = -1, best_gpl = 0;
    int64_t best_waste = INT64_MAX;
    for (int k = 0; k <= 6; ++k) {
        const int lpr = 1 << k;
        const int gpl = (a.n_granules + lpr - 1) / lpr;
        if (gpl > 3 || gpl < 2) continue;
        const int64_t waste = (int64_t)lpr * gpl - a.n_granules;
        if (4 * waste > (int64_t)lpr * gpl) continue;
        if (waste < best_waste || (waste == best_waste && gpl > best_gpl)) {
            best_waste = waste;
            best_k = k;
            best_gpl = gpl;
        }
    }
    if (best_k < 0) {
        for (int k = 0; k <= 6; ++k) {
            const int lpr = 1 << k;
            const int gpl = (a.n_granules + lpr - 1) / lpr;
            if (gpl > kMaxGpl) continue;
            const int64_t waste = (int64_t)lpr * gpl - a.n_granules;
            const bool closer = (gpl > 4 ? gpl - 4 : 4 - gpl) < (best_gpl > 4 ? best_gpl - 4 : 4 - best_gpl);
            if (waste < best_waste || (waste == best_waste && closer)) {
                best_waste = waste;
                best_k = k;
                best_gpl = gpl;
            }
        }
    }
    if (best_k < 0) {
        if (probe) return ADAQP_EINVAL;                 // rows too wide for registers have no twin
        const int64_t blocks = (n_send + kWavesPerBlock - 1) / kWavesPerBlock;
        if (blocks > INT32_MAX) return ADAQP_ESIZE;
        hipLaunchKernelGGL(quantize_pack_wide_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, st, a);
        ADAQP_HIP_TRY(hipGetLastError());
        return ADAQP_OK;
    }
    a.lpr_log2 = best_k;
    const int64_t rows_per_block = (int64_t)kWavesPerBlock * (kWave >> best_k);
    const int64_t blocks = (n_send + rows_per_block - 1) / rows_per_block;
    if (blocks > INT32_MAX) return ADAQP_ESIZE;
    const dim3 grid((unsigned)blocks);
    const int vw = vector_width(feat_dev, ld, dim, false);
    hipError_t err;
    if (probe) {
        if (vw != 4) return ADAQP_EINVAL;               // the twin exists for 16-byte-aligned rows only
        err = launch_quantize<4, true>(a, best_gpl, grid, st);
    } else if (vw == 4) err = launch_quantize<4>(a, best_gpl, grid, st);
    else if (vw == 2) err = launch_quantize<2>(a, best_gpl, grid, st);
    else err = launch_quantize<1>(a, best_gpl, grid, st);
    ADAQP_HIP_TRY(err);
    return ADAQP_OK;
}

}  // namespace

extern "C" int adaqp_quantize_pack_trace(const float *feat_dev, int64_t n_feat_rows, int64_t ld, int32_t dim,
                                         const int32_t *send_idx_dev, const uint8_t *bits_dev,
                                         const int64_t *row_offset_dev, int64_t n_send, uint64_t seed,
                                         uint8_t *packed_dev, int64_t packed_bytes, float *params_dev,
                                         const float *alpha_sq_dev, float *beta_dev, void *stream)
{
    return quantize_pack_launch(feat_dev, n_feat_rows, ld, dim, send_idx_dev, bits_dev, row_offset_dev, n_send, seed,
                                packed_dev, packed_bytes, params_dev, alpha_sq_dev, beta_dev, stream, false);
}

extern "C" int adaqp_probe_quantize_pack(const float *feat_dev, int64_t n_feat_rows, int64_t ld, int32_t dim,
                                         const int32_t *send_idx_dev, const uint8_t *bits_dev,
                                         const int64_t *row_offset_dev, int64_t n_send,
                                         uint8_t *packed_dev, int64_t packed_bytes, float *params_dev, void *stream)
{
    return quantize_pack_launch(feat_dev, n_feat_rows, ld, dim, send_idx_dev, bits_dev, row_offset_dev, n_send, 0,
                                packed_dev, packed_bytes, params_dev, nullptr, nullptr, stream, true);
}

extern "C" int adaqp_unpack_dequant(const uint8_t *packed_dev, int64_t packed_bytes, const float *params_dev,
                                    const uint8_t *bits_dev, const int64_t *row_offset_dev,
                                    const int32_t *halo_idx_dev, const int32_t *order_dev, int64_t n_recv,
                                    int32_t dim, float *feat_dev, int64_t n_feat_rows, int64_t ld, void *stream)
{
    if (n_recv < 0 || dim <= 0 || ld < dim || n_feat_rows < 0 || packed_bytes < 0) return ADAQP_EINVAL;
    if (n_recv == 0) return ADAQP_OK;
    if (!packed_dev || !params_dev || !bits_dev || !row_offset_dev || !halo_idx_dev || !feat_dev)
        return ADAQP_EINVAL;
    if (n_feat_rows == 0) return ADAQP_EINVAL;
    if (!aligned_to(feat_dev, 4) || !aligned_to(params_dev, 8) || !aligned_to(packed_dev, 4) ||
        !aligned_to(halo_idx_dev, 4) || !aligned_to(row_offset_dev, 8) || !aligned_to(order_dev, 4))
        return ADAQP_EINVAL;
    if (order_dev && n_recv > INT32_MAX) return ADAQP_ESIZE;
    if (packed_bytes < 4) return ADAQP_OK;          // no row fits: every slot would be skipped
    const int64_t blocks = (n_recv + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > INT32_MAX) return ADAQP_ESIZE;

    DequantArgs a;
    a.packed = packed_dev;
    a.packed_bytes = packed_bytes;
    a.params = params_dev;
    a.bits = bits_dev;
    a.row_offset = row_offset_dev;
    a.halo_idx = halo_idx_dev;
    a.order = order_dev;
    a.n_recv = n_recv;
    a.dim = dim;
    a.write_dim = dim;
    a.feat = feat_dev;
    a.n_feat_rows = n_feat_rows;
    a.ld = ld;
    hipStream_t st = (hipStream_t)stream;
    // line-padded rows are written in whole 128-byte lines (the padding receives zeros): partial-line
    // writes cost a read-modify-write in the memory system
    const bool whole_lines = line_padded(feat_dev, ld);
    const int32_t write_dim = whole_lines ? (int32_t)((((int64_t)dim + 31) / 32) * 32) : dim;
    const int vw = vector_width(feat_dev, ld, dim, !whole_lines);
    const int nv = (write_dim + kWave * vw - 1) / (kWave * vw);
    if (nv <= kMaxDequantNv) {
        a.write_dim = write_dim;
        const int rows = dequant_rows_per_wave(nv);
        const int64_t waves = (n_recv + rows - 1) / rows;
        hipError_t err;
        // whole-line writes go out as non-temporal stores; rows that share lines with their neighbours stay with
        // ordinary stores, which the L2 merges
        if (whole_lines) {
            err = launch_dequant<4, true>(a, nv, waves, st);            // line-padded rows take 16-byte vectors
        } else {
            if (vw == 4) err = launch_dequant<4, false>(a, nv, waves, st);
            else if (vw == 2) err = launch_dequant<2, false>(a, nv, waves, st);
            else err = launch_dequant<1, false>(a, nv, waves, st);
        }
        ADAQP_HIP_TRY(err);
        return ADAQP_OK;
    }
    const dim3 grid((unsigned)blocks);
    a.write_dim = write_dim;
    const int vw_long = vector_width(feat_dev, ld, dim, true);
    if (vw_long == 4) hipLaunchKernelGGL(unpack_dequant_long_kernel<4>, grid, dim3(kBlock), 0, st, a);
    else if (vw_long == 2) hipLaunchKernelGGL(unpack_dequant_long_kernel<2>, grid, dim3(kBlock), 0, st, a);
    else hipLaunchKernelGGL(unpack_dequant_long_kernel<1>, grid, dim3(kBlock), 0, st, a);
    ADAQP_HIP_TRY(hipGetLastError());
    return ADAQP_OK;
}

static int dequant_add_launch(const uint8_t *packed_dev, int64_t packed_bytes, const float *params_dev,
                              const uint8_t *bits_dev, const int64_t *row_offset_dev, const int32_t *dst_idx_dev,
                              int64_t n_recv, const int32_t *seg_order_dev, const int64_t *seg_ptr_dev, int64_t n_seg,
                              int32_t dim, float *grad_dev, int64_t n_grad_rows, int64_t ld, void *stream, bool probe)
{
    if (n_recv < 0 || n_seg < 0 || dim <= 0 || ld < dim || n_grad_rows < 0 || packed_bytes < 0) return ADAQP_EINVAL;
    if (n_recv == 0 || n_seg == 0) return ADAQP_OK;
    if (!packed_dev || !params_dev || !bits_dev || !row_offset_dev || !dst_idx_dev || !seg_order_dev ||
        !seg_ptr_dev || !grad_dev)
        return ADAQP_EINVAL;
    if (n_grad_rows == 0 || n_seg > n_recv) return ADAQP_EINVAL;
    if (!aligned_to(grad_dev, 4) || !aligned_to(params_dev, 8) || !aligned_to(packed_dev, 4) ||
        !aligned_to(dst_idx_dev, 4) || !aligned_to(row_offset_dev, 8) || !aligned_to(seg_order_dev, 4) ||
        !aligned_to(seg_ptr_dev, 8))
        return ADAQP_EINVAL;
    if (n_recv > INT32_MAX) return ADAQP_ESIZE;
    if (packed_bytes < 4) return ADAQP_OK;          // no row fits: every slot would be skipped
    const int64_t blocks = (n_seg + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > INT32_MAX) return ADAQP_ESIZE;

    DequantAddArgs a;
    a.packed = packed_dev;
    a.packed_bytes = packed_bytes;
    a.params = params_dev;
    a.bits = bits_dev;
    a.row_offset = row_offset_dev;
    a.dst_idx = dst_idx_dev;
    a.n_recv = n_recv;
    a.seg_order = seg_order_dev;
    a.seg_ptr = seg_ptr_dev;
    a.n_seg = n_seg;
    a.dim = dim;
    a.grad = grad_dev;
    a.n_grad_rows = n_grad_rows;
    a.ld = ld;
    hipStream_t st = (hipStream_t)stream;
    const dim3 grid((unsigned)blocks);
    const int vw = vector_width(grad_dev, ld, dim, true);
    const int nv = (dim + kWave * vw - 1) / (kWave * vw);          // rows wider than 4 vectors per lane: chunks of 4
    const int seg_per_wave = 4;     // measured on 150 000 messages: two per wave the same, one + 20 %, eight + 9 %
    const dim3 grid4((unsigned)((n_seg + seg_per_wave * kWavesPerBlock - 1) / (seg_per_wave * kWavesPerBlock)));
#define ADAQP_ADD(VW_, ST_)                                                                                        \
    do {                                                                                                           \
        if (nv == 1) hipLaunchKernelGGL((unpack_dequant_add4_kernel<VW_, 1, 4, ST_, false>), grid4, dim3(kBlock), 0, st, a);   \
        else if (nv == 2) hipLaunchKernelGGL((unpack_dequant_add4_kernel<VW_, 2, 4, ST_, false>), grid4, dim3(kBlock), 0, st, a); \
        else if (nv == 3) hipLaunchKernelGGL((unpack_dequant_add_kernel<VW_, 3, ST_>), grid, dim3(kBlock), 0, st, a);   \
        else hipLaunchKernelGGL((unpack_dequant_add_kernel<VW_, 4, ST_>), grid, dim3(kBlock), 0, st, a);                \
    } while (0)
    // rows that are whole 128-byte lines (line-padded layout, dim a multiple of 32) are written back non-temporally
    const bool whole_lines = line_padded(grad_dev, ld) && dim % 32 == 0;
    if (probe) {
        // the twin exists for the shape the full-size workloads take: whole-line rows of at most 512 columns
        if (vw != 4 || !whole_lines || nv > 2) return ADAQP_EINVAL;
        if (nv == 1) hipLaunchKernelGGL((unpack_dequant_add4_kernel<4, 1, 4, true, true>), grid4, dim3(kBlock), 0, st, a);
        else hipLaunchKernelGGL((unpack_dequant_add4_kernel<4, 2, 4, true, true>), grid4, dim3(kBlock), 0, st, a);
        ADAQP_HIP_TRY(hipGetLastError());
        return ADAQP_OK;
    }
    if (vw == 4 && whole_lines) ADAQP_ADD(4, true);
    else if (vw == 4) ADAQP_ADD(4, false);
    else if (vw == 2) ADAQP_ADD(2, false);
    else ADAQP_ADD(1, false);
#undef ADAQP_ADD
    ADAQP_HIP_TRY(hipGetLastError());
    return ADAQP_OK;
}

extern "C" int adaqp_unpack_dequant_add(const uint8_t *packed_dev, int64_t packed_bytes, const float *params_dev,
                                        const uint8_t *bits_dev, const int64_t *row_offset_dev,
                                        const int32_t *dst_idx_dev, int64_t n_recv, const int32_t *seg_order_dev,
                                        const int64_t *seg_ptr_dev, int64_t n_seg, int32_t dim, float *grad_dev,
                                        int64_t n_grad_rows, int64_t ld, void *stream)
{
    return dequant_add_launch(packed_dev, packed_bytes, params_dev, bits_dev, row_offset_dev, dst_idx_dev, n_recv,
                              seg_order_dev, seg_ptr_dev, n_seg, dim, grad_dev, n_grad_rows, ld, stream, false);
}

extern "C" int adaqp_probe_unpack_dequant_add(const uint8_t *packed_dev, int64_t packed_bytes, const float *params_dev,
                                              const uint8_t *bits_dev, const int64_t *row_offset_dev,
                                              const int32_t *dst_idx_dev, int64_t n_recv,
                                              const int32_t *seg_order_dev, const int64_t *seg_ptr_dev, int64_t n_seg,
                                              int32_t dim, float *grad_dev, int64_t n_grad_rows, int64_t ld,
                                              void *stream)
{
    return dequant_add_launch(packed_dev, packed_bytes, params_dev, bits_dev, row_offset_dev, dst_idx_dev, n_recv,
                              seg_order_dev, seg_ptr_dev, n_seg, dim, grad_dev, n_grad_rows, ld, stream, true);
}
