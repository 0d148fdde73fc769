// Neighbour aggregation out_v = sum_u alpha(u,v) h_u (Sec. 2.1 Eq. 3, inner sum) as a CSR SpMM for gfx950.
//
// Work split.  Degrees follow a power law (the largest row is ~50x the mean), so rows are not the unit of
// work.  The CSR is walked as a merge path: the list of row ends and the list of entries are merged, the
// path of length n_rows + nnz is cut into equal pieces, one piece per wave.  A wave finds its two end points
// with a 64-ary search over rowptr (every lane probes one position), then walks its piece:
//   * entries are staged 64 at a time, lane e holding (col, alpha) of entry e; the wave-uniform column of
//     the entry being processed is fetched with v_readlane, so the neighbour row's address is scalar and
//     every lane loads its VW-float slice of that row with one vector load;
//   * row ends are staged the same way, 64 rows at a time;
//   * U entries are in flight at once (U * NV vector loads per lane) before the first is consumed;
//   * a row that ends inside the piece is stored directly; what a piece has accumulated for a row that
//     continues into the next piece goes to a carry slot in the workspace.
// A second, tiny kernel adds the carries of each split row in piece order.  The summation order therefore
// depends only on the launch geometry: results are bit-identical from run to run and across schedules.
//
// The kernel is a gather: per entry it reads 8 bytes of (col, alpha) and 4*dim bytes of H.  It is bound by
// how fast H rows come out of L2 / Infinity Cache / HBM, not by arithmetic, so there is no MFMA use.
#include <mutex>

#include "common.hpp"

namespace adaqp {
namespace {

struct SpmmArgs {
    const int64_t *rowptr;      // already offset: rowptr[0] is the start of the first row of the range
    const int32_t *col;
    const float *val;
    int64_t nnz;                // capacity of col / val
    int32_t n_rows;             // rows in the range
    const float *H;
    int64_t n_cols, ldh;
    int32_t dim, wdim;          // wdim >= dim: columns [dim, wdim) of a written row receive zeros (whole lines)
    float *out;                 // already offset to the first row of the range
    int64_t ldo;
    int32_t *carry_row;         // [n_items]
    float *carry;               // [n_items, carry_ld]
    int64_t carry_ld;
    int32_t n_items;
    // optional: rows of H that are still packed (received halo rows, de-quantised on the fly)
    const int32_t *slot_of_row; // [n_cols], -1 = read the row from H
    const uint8_t *packed;
    int64_t packed_bytes;
    const float *params;
    const uint8_t *bits;
    const int64_t *row_offset;
    int64_t n_slots;
    int32_t col0, full_dim;     // first column of this launch's chunk and the row length of the packed layout
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

// Same, marked non-temporal: output rows are written once and not read again by this kernel.
template <int VW>
__device__ __forceinline__ void store_vec_streaming(float *p, const float *src)
{
    typedef float vec_t __attribute__((ext_vector_type(VW)));
    vec_t v;
    for (int k = 0; k < VW; ++k) v[k] = src[k];
    __builtin_nontemporal_store(v, reinterpret_cast<vec_t *>(p));
}

__device__ __forceinline__ int64_t clamp64(int64_t v, int64_t lo, int64_t hi) { return v < lo ? lo : (v > hi ? hi : v); }

__device__ __forceinline__ int32_t uniform_i32(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ int64_t uniform_i64(int64_t v)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int32_t)(uint32_t)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

__device__ __forceinline__ int64_t readlane_i64(int64_t v, int lane_id)
{
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int32_t)(uint32_t)v, lane_id);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int32_t)(uint32_t)((uint64_t)v >> 32), lane_id);
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Merge-path split point on diagonal d: the number of row ends that precede d path steps.  Row end i (its
// entry count relative to the range is end_i) precedes entry j iff end_i <= j; on diagonal d this reads
// end_i + i + 1 <= d, which is increasing in i, so the answer is the first i for which it fails.
// All 64 lanes take part; the result is wave-uniform.
__device__ int64_t split_rows(const SpmmArgs &a, int64_t d, int64_t base, int64_t nnz_r, int lane)
{
    int64_t lo = d - nnz_r > 0 ? d - nnz_r : 0;
    int64_t hi = d < a.n_rows ? d : a.n_rows;
    while (lo < hi) {
        const int64_t n = hi - lo;
        const int64_t step = (n + kWave - 1) / kWave;
        const int64_t probes = (n + step - 1) / step;          // <= 64
        const int64_t p = lo + lane * step;
        bool before = false;
        if (lane < probes) {
            const int64_t end_p = clamp64(a.rowptr[p + 1], base, base + nnz_r) - base;
            before = end_p + p + 1 <= d;
        }
        const int cnt = __popcll(__ballot(before));
        const int64_t new_lo = cnt > 0 ? lo + (int64_t)(cnt - 1) * step + 1 : lo;
        const int64_t new_hi = cnt < probes ? lo + (int64_t)cnt * step : hi;
        lo = new_lo;
        hi = new_hi;
    }
    return lo;
}

constexpr int32_t kNoRow = -1;
constexpr int32_t kFar = 0x7FFFFFFF;

// PACKED: entries whose column has a slot in slot_of_row take the neighbour row from the packed receive buffer
// and de-quantise it in registers, (float)code * S + Z as in Sec. 2.3 Eq. 5 (product rounded, then sum rounded),
// so the result is bit-identical to de-quantising into H first - without writing and re-reading those rows.
template <int VW, int NV, int U, bool PACKED>
__global__ __launch_bounds__(kBlock) void spmm_merge_kernel(const SpmmArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t item = uniform_i32((int32_t)(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)));
    if (item >= a.n_items) return;

    // extent of the range on the device: the host only sized the launch
    const int64_t base = uniform_i64(clamp64(a.rowptr[0], 0, a.nnz));
    const int64_t nnz_r = uniform_i64(clamp64(a.rowptr[a.n_rows], base, a.nnz)) - base;
    const int64_t total = (int64_t)a.n_rows + nnz_r;
    const int64_t per = (total + a.n_items - 1) / a.n_items;
    const int64_t d0 = (int64_t)item * per < total ? (int64_t)item * per : total;
    const int64_t d1 = d0 + per < total ? d0 + per : total;
    if (d0 >= d1) {
        if (lane == 0) a.carry_row[item] = kNoRow;
        return;
    }
    const int64_t i0 = uniform_i64(split_rows(a, d0, base, nnz_r, lane));
    const int64_t i1 = uniform_i64(split_rows(a, d1, base, nnz_r, lane));
    const int64_t j0 = d0 - i0;                             // first entry of the piece, relative to base
    const int32_t n_edges = (int32_t)((d1 - i1) - j0);      // entries in the piece

    // per-lane slice of a row: vectors v*64 + lane, v < NV; only the last one can fall off the row
    const bool last_ok = ((NV - 1) * kWave + lane) * VW < a.wdim;

    float acc[NV][VW];
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int k = 0; k < VW; ++k) acc[v][k] = 0.0f;

    // row-end staging: lane q holds the end (relative to j0) of row row_blk + q
    int64_t row = i0, row_blk = i0;
    int32_t my_end = kFar;
    auto stage_rows = [&]() {
        my_end = kFar;
        const int64_t q = row_blk + lane;
        if (q < a.n_rows) {
            const int64_t e = clamp64(a.rowptr[q + 1], base, base + nnz_r) - base - j0;
            my_end = e > kFar ? kFar : (e < 0 ? 0 : (int32_t)e);
        }
    };
    stage_rows();
    int32_t cur_end = __builtin_amdgcn_readlane(my_end, 0);
    bool dirty = false;

    auto flush_row = [&]() {
        float *o = a.out + row * a.ldo;
        if (a.wdim > a.dim) {                                   // row padding: whatever was gathered there is dropped
#pragma unroll
            for (int k = 0; k < VW; ++k)
                if (((NV - 1) * kWave + lane) * VW + k >= a.dim) acc[NV - 1][k] = 0.0f;
        }
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            if (v < NV - 1 || last_ok) store_vec_streaming<VW>(o + (v * kWave + lane) * VW, acc[v]);
#pragma unroll
            for (int k = 0; k < VW; ++k) acc[v][k] = 0.0f;
        }
        dirty = false;
        ++row;
        if (row - row_blk == kWave) {
            row_blk = row;
            stage_rows();
        }
        cur_end = __builtin_amdgcn_readlane(my_end, (int)(row - row_blk));
    };

    const int32_t *colp = a.col + base + j0;
    const float *valp = a.val + base + j0;
    int32_t j = 0;                                          // entries consumed, relative to j0
    while (j < n_edges) {
        const int32_t nb = n_edges - j < kWave ? n_edges - j : kWave;
        int32_t my_col = 0;
        float my_val = 0.0f;
        int32_t my_b = 0;                                   // PACKED: width of the entry's packed row, 0 = plain row
        int64_t my_off = 0;
        float my_z = 0.0f, my_s = 0.0f;
        if (lane < nb) {
            my_col = __builtin_nontemporal_load(colp + j + lane);     // streamed once: keep the caches for H
            my_val = __builtin_nontemporal_load(valp + j + lane);
            if (my_col < 0 || my_col >= a.n_cols) { my_col = 0; my_val = 0.0f; }   // out-of-range entry: skipped
            if (PACKED) {
                const int32_t slot = a.slot_of_row[my_col];
                if (slot >= 0 && slot < a.n_slots) {
                    my_b = a.bits[slot];
                    my_off = a.row_offset[slot];
                    const float2 zs = *reinterpret_cast<const float2 *>(a.params + 2 * (int64_t)slot);
                    my_z = zs.x;
                    my_s = zs.y;
                    const int64_t stride = 4 * (((int64_t)a.full_dim * my_b + 31) >> 5);
                    const bool ok = (my_b == 2 || my_b == 4 || my_b == 8) && my_off >= 0 && (my_off & 3) == 0 &&
                                    my_off + stride <= a.packed_bytes;
                    if (!ok) my_b = 0;                      // broken slot: fall back to the row in H
                }
            }
        }
        for (int32_t e = 0; e < nb; e += U) {
            float h[U][NV][VW];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int32_t eu = e + u < nb ? e + u : nb - 1;                    // tail repeats the last entry
                const int32_t c = __builtin_amdgcn_readlane(my_col, eu);
                const int32_t pb = PACKED ? __builtin_amdgcn_readlane(my_b, eu) : 0;
                if (PACKED && pb != 0) {                                           // wave-uniform
                    // one 32-bit word holds the VW codes of a lane's vector (VW * b <= 32 and divides 32)
                    const uint32_t *words = reinterpret_cast<const uint32_t *>(a.packed + readlane_i64(my_off, eu));
                    const uint32_t last_word = (uint32_t)(((int64_t)a.full_dim * pb - 1) >> 5);
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const uint32_t bit = (uint32_t)(a.col0 + (v * kWave + lane) * VW) * (uint32_t)pb;
                        const uint32_t idx = (bit >> 5) < last_word ? (bit >> 5) : last_word;
#pragma unroll
                        for (int k = 0; k < VW; ++k) h[u][v][k] = 0.0f;
                        h[u][v][0] = __builtin_bit_cast(float, words[idx]);
                    }
                } else {
                    const float *hrow = a.H + (int64_t)c * a.ldh;
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        if (v < NV - 1 || last_ok) {
                            load_vec<VW>(hrow + (v * kWave + lane) * VW, h[u][v]);
                        } else {
#pragma unroll
                            for (int k = 0; k < VW; ++k) h[u][v][k] = 0.0f;
                        }
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (e + u < nb) {
                    while (j >= cur_end && row < i1) flush_row();    // rows that end before this entry
                    const float alpha = __builtin_bit_cast(
                        float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_val), e + u));
                    const int32_t pb = PACKED ? __builtin_amdgcn_readlane(my_b, e + u) : 0;
                    if (PACKED && pb != 0) {
                        const float Z = __builtin_bit_cast(
                            float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_z), e + u));
                        const float S = __builtin_bit_cast(
                            float, __builtin_amdgcn_readlane(__builtin_bit_cast(int32_t, my_s), e + u));
                        const uint32_t mask = (1u << pb) - 1u;
#pragma unroll
                        for (int v = 0; v < NV; ++v) {
                            const uint32_t bit = (uint32_t)(a.col0 + (v * kWave + lane) * VW) * (uint32_t)pb;
                            const uint32_t word = __builtin_bit_cast(uint32_t, h[u][v][0]) >> (bit & 31u);
#pragma unroll
                            for (int k = 0; k < VW; ++k) {
                                const uint32_t code = (word >> (k * pb)) & mask;
                                const float scaled = (float)code * S;      // Eq. 5: product rounded, then sum rounded
                                const float value = scaled + Z;
                                acc[v][k] = fmaf(alpha, value, acc[v][k]);
                            }
                        }
                    } else {
#pragma unroll
                        for (int v = 0; v < NV; ++v)
#pragma unroll
                            for (int k = 0; k < VW; ++k) acc[v][k] = fmaf(alpha, h[u][v][k], acc[v][k]);
                    }
                    ++j;
                    dirty = true;
                }
            }
        }
    }
    while (row < i1) flush_row();                           // rows that end at the piece's last entry, empty rows

    // what is left belongs to a row that continues in the next piece
    if (dirty && row < a.n_rows) {
        float *cslot = a.carry + (int64_t)item * a.carry_ld;
#pragma unroll
        for (int v = 0; v < NV; ++v)
            if (v < NV - 1 || last_ok) store_vec<VW>(cslot + (v * kWave + lane) * VW, acc[v]);
        if (lane == 0) a.carry_row[item] = (int32_t)row;
    } else {
        if (lane == 0) a.carry_row[item] = kNoRow;
    }
}

// Adds the carries of every split row to the part stored by the piece that finished the row, in piece order.
// One wave per piece; only the wave of a row's first carry does the work.  Lanes own the same column slices
// as in the main kernel, and several carries are in flight at once.
template <int VW, int NV>
__global__ __launch_bounds__(kBlock) void spmm_carry_kernel(const SpmmArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t item = uniform_i32((int32_t)(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)));
    if (item >= a.n_items) return;
    const int32_t r = uniform_i32(a.carry_row[item]);
    if (r < 0 || r >= a.n_rows) return;
    if (item > 0 && uniform_i32(a.carry_row[item - 1]) == r) return;
    int32_t last = item + 1;
    while (last < a.n_items && uniform_i32(a.carry_row[last]) == r) ++last;

    const bool last_ok = ((NV - 1) * kWave + lane) * VW < a.wdim;
    float sum[NV][VW];
#pragma unroll
    for (int v = 0; v < NV; ++v)
#pragma unroll
        for (int k = 0; k < VW; ++k) sum[v][k] = 0.0f;
    constexpr int kAhead = 4;
    for (int32_t w0 = item; w0 < last; w0 += kAhead) {
        float c[kAhead][NV][VW];
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            const int32_t w = w0 + u < last ? w0 + u : last - 1;
            const float *slot = a.carry + (int64_t)w * a.carry_ld;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                if (v < NV - 1 || last_ok) {
                    load_vec<VW>(slot + (v * kWave + lane) * VW, c[u][v]);
                } else {
#pragma unroll
                    for (int k = 0; k < VW; ++k) c[u][v][k] = 0.0f;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kAhead; ++u)
            if (w0 + u < last)
#pragma unroll
                for (int v = 0; v < NV; ++v)
#pragma unroll
                    for (int k = 0; k < VW; ++k) sum[v][k] += c[u][v][k];
    }
    float *o = a.out + (int64_t)r * a.ldo;
#pragma unroll
    for (int v = 0; v < NV; ++v) {
        if (v < NV - 1 || last_ok) {
            float cur[VW];
            load_vec<VW>(o + (v * kWave + lane) * VW, cur);
#pragma unroll
            for (int k = 0; k < VW; ++k) {
                cur[k] = cur[k] + sum[v][k];
                if (v == NV - 1 && (v * kWave + lane) * VW + k >= a.dim) cur[k] = 0.0f;      // row padding
            }
            store_vec<VW>(o + (v * kWave + lane) * VW, cur);
        }
    }
}

// Scratch of adaqp_spmm_csr_noalloc: one copy per GPU the library runs on, held until the process ends.  In host
// code the array's name is only a handle for hipGetSymbolAddress, never an address to pass to a kernel.
static __device__ __align__(256) unsigned char scratch[ADAQP_SPMM_NOALLOC_SCRATCH_BYTES];

// Geometry shared by the workspace query and the launch.
struct Geometry { int32_t n_items; int64_t carry_ld; int64_t bytes; int64_t carry_off; };

bool geometry(int64_t n_rows, int64_t nnz, int32_t dim, Geometry *g)
{
    const int64_t total = n_rows + nnz;
    if (total <= 0) { *g = Geometry{0, 0, 0, 0}; return true; }
    // path steps per wave: enough pieces to fill 256 CUs several times over, few enough that the search
    // and the carry are amortised
    int64_t per = 32;
    while (per < 512 && total / per > 65536) per *= 2;
    const int64_t items = (total + per - 1) / per;
    if (items > (int64_t)1 << 30) return false;
    g->n_items = (int32_t)items;
    g->carry_ld = ((int64_t)dim + 31) / 32 * 32;
    g->carry_off = (items * 4 + 255) / 256 * 256;
    g->bytes = g->carry_off + (items * g->carry_ld * 4 + 255) / 256 * 256;
    return true;
}

template <int VW, int NV>
hipError_t launch_merge(const SpmmArgs &a, dim3 grid, hipStream_t st)
{
    constexpr int U = NV >= 4 ? 4 : (NV >= 2 ? 8 : 16);
    if (a.slot_of_row) hipLaunchKernelGGL((spmm_merge_kernel<VW, NV, U, true>), grid, dim3(kBlock), 0, st, a);
    else hipLaunchKernelGGL((spmm_merge_kernel<VW, NV, U, false>), grid, dim3(kBlock), 0, st, a);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((spmm_carry_kernel<VW, NV>), grid, dim3(kBlock), 0, st, a);
    return hipGetLastError();
}

template <int VW>
hipError_t launch_merge_nv(const SpmmArgs &a, int nv, dim3 grid, hipStream_t st)
{
    switch (nv) {
        case 1: return launch_merge<VW, 1>(a, grid, st);
        case 2: return launch_merge<VW, 2>(a, grid, st);
        case 3: return launch_merge<VW, 3>(a, grid, st);
        case 4: return launch_merge<VW, 4>(a, grid, st);
        case 5: return launch_merge<VW, 5>(a, grid, st);
        case 6: return launch_merge<VW, 6>(a, grid, st);
        case 7: return launch_merge<VW, 7>(a, grid, st);
        case 8: return launch_merge<VW, 8>(a, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace
}  // namespace adaqp

using namespace adaqp;

extern "C" int adaqp_spmm_workspace_bytes(int64_t n_rows, int64_t nnz, int32_t dim, int64_t *bytes_out)
{
    if (!bytes_out || n_rows < 0 || nnz < 0 || dim <= 0) return ADAQP_EINVAL;
    Geometry g;
    if (!geometry(n_rows, nnz, dim, &g)) return ADAQP_ESIZE;
    *bytes_out = g.bytes;
    return ADAQP_OK;
}

extern "C" int adaqp_spmm_csr(const int64_t *rowptr_dev, const int32_t *col_dev, const float *val_dev,
                              int64_t nnz, int64_t row_begin, int64_t row_end, int64_t nnz_range,
                              const float *H_dev, int64_t n_cols, int64_t ldh, int32_t dim,
                              float *out_dev, int64_t ldo, void *workspace_dev, int64_t workspace_bytes,
                              void *stream)
{
    return adaqp_spmm_csr_packed(rowptr_dev, col_dev, val_dev, nnz, row_begin, row_end, nnz_range, H_dev, n_cols, ldh,
                                 dim, out_dev, ldo, nullptr, nullptr, 0, nullptr, nullptr, nullptr, 0, workspace_dev,
                                 workspace_bytes, stream);
}

extern "C" int adaqp_spmm_csr_packed(const int64_t *rowptr_dev, const int32_t *col_dev, const float *val_dev,
                                     int64_t nnz, int64_t row_begin, int64_t row_end, int64_t nnz_range,
                                     const float *H_dev, int64_t n_cols, int64_t ldh, int32_t dim,
                                     float *out_dev, int64_t ldo,
                                     const int32_t *slot_of_row_dev, const uint8_t *packed_dev, int64_t packed_bytes,
                                     const float *params_dev, const uint8_t *bits_dev, const int64_t *row_offset_dev,
                                     int64_t n_slots,
                                     void *workspace_dev, int64_t workspace_bytes, void *stream)
{
    if (slot_of_row_dev) {
        if (!packed_dev || !params_dev || !bits_dev || !row_offset_dev || packed_bytes < 4 || n_slots <= 0)
            return ADAQP_EINVAL;
        if (!aligned_to(slot_of_row_dev, 4) || !aligned_to(packed_dev, 4) || !aligned_to(params_dev, 8) ||
            !aligned_to(row_offset_dev, 8))
            return ADAQP_EINVAL;
    }
    if (row_begin < 0 || row_end < row_begin || nnz < 0 || dim <= 0 || ldh < dim || ldo < dim || n_cols < 0)
        return ADAQP_EINVAL;
    const int64_t n_rows = row_end - row_begin;
    if (n_rows == 0) return ADAQP_OK;
    if (!rowptr_dev || !out_dev) return ADAQP_EINVAL;
    if (nnz > 0 && (!col_dev || !val_dev || !H_dev || n_cols == 0)) return ADAQP_EINVAL;
    if (n_rows > INT32_MAX - 1) return ADAQP_ESIZE;
    if (!aligned_to(rowptr_dev, 8) || !aligned_to(col_dev, 4) || !aligned_to(val_dev, 4) ||
        !aligned_to(H_dev, 4) || !aligned_to(out_dev, 4))
        return ADAQP_EINVAL;
    if (nnz_range < 0 || nnz_range > nnz) nnz_range = nnz;

    Geometry g;
    if (!geometry(n_rows, nnz_range, dim, &g)) return ADAQP_ESIZE;
    if (g.bytes > 0 && (!workspace_dev || !aligned_to(workspace_dev, 256))) return ADAQP_EINVAL;
    if (workspace_bytes < g.bytes) return ADAQP_ESIZE;

    // vector width: every row start of H and out and of the carry slots must be naturally aligned, and a
    // vector must not spill past dim - unless both matrices are line-padded (rows start on 128-byte lines,
    // pitch a whole number of lines): then rows are read and written in whole lines, padding written as zero
    const bool whole_lines = ldh % 32 == 0 && ldo % 32 == 0 && aligned_to(H_dev, 128) && aligned_to(out_dev, 128);
    int vw = 1;
    if (whole_lines) vw = 4;
    else if (dim % 4 == 0 && ldh % 4 == 0 && ldo % 4 == 0 && aligned_to(H_dev, 16) && aligned_to(out_dev, 16)) vw = 4;
    else if (dim % 2 == 0 && ldh % 2 == 0 && ldo % 2 == 0 && aligned_to(H_dev, 8) && aligned_to(out_dev, 8)) vw = 2;

    hipStream_t st = (hipStream_t)stream;
    const int32_t chunk_cap = kWave * vw * 8;               // columns one launch covers (NV <= 8)
    for (int32_t c0 = 0; c0 < dim; c0 += chunk_cap) {
        const int32_t cdim = dim - c0 < chunk_cap ? dim - c0 : chunk_cap;
        SpmmArgs a;
        a.rowptr = rowptr_dev + row_begin;
        a.col = col_dev;
        a.val = val_dev;
        a.nnz = nnz;
        a.n_rows = (int32_t)n_rows;
        a.H = H_dev + c0;
        a.n_cols = n_cols;
        a.ldh = ldh;
        a.dim = cdim;
        a.wdim = whole_lines ? (cdim + 31) / 32 * 32 : cdim;
        a.out = out_dev + row_begin * ldo + c0;
        a.ldo = ldo;
        a.carry_row = reinterpret_cast<int32_t *>(workspace_dev);
        a.carry = reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(workspace_dev) + g.carry_off);
        a.carry_ld = g.carry_ld;
        a.n_items = g.n_items;
        a.slot_of_row = slot_of_row_dev;
        a.col0 = c0;
        a.full_dim = dim;
        a.packed = packed_dev;
        a.packed_bytes = packed_bytes;
        a.params = params_dev;
        a.bits = bits_dev;
        a.row_offset = row_offset_dev;
        a.n_slots = n_slots;
        const int nv = (a.wdim + kWave * vw - 1) / (kWave * vw);
        const dim3 grid((unsigned)((g.n_items + kWavesPerBlock - 1) / kWavesPerBlock));
        hipError_t err;
        if (vw == 4) err = launch_merge_nv<4>(a, nv, grid, st);
        else if (vw == 2) err = launch_merge_nv<2>(a, nv, grid, st);
        else err = launch_merge_nv<1>(a, nv, grid, st);
        ADAQP_HIP_TRY(err);
    }
    return ADAQP_OK;
}

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each GPU, looked up once per GPU

// Address of the current device's copy of `scratch`.  The first call on a device asks the runtime for it (which
// may load the code object); later calls only read the table.
int scratch_of_current_device(void **ptr_out)
{
    int dev = -1;
    ADAQP_HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ADAQP_ESIZE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        ADAQP_HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return note_hip_error(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
        g_scratch_ptr[dev] = p;
    }
    *ptr_out = g_scratch_ptr[dev];
    return ADAQP_OK;
}

}  // namespace

extern "C" int adaqp_spmm_csr_noalloc(const int64_t *rowptr_dev, const int32_t *col_dev, const float *val_dev,
                                      int64_t nnz, int64_t row_begin, int64_t row_end, int64_t nnz_range,
                                      const float *H_dev, int64_t n_cols, int64_t ldh, int32_t dim,
                                      float *out_dev, int64_t ldo, void *stream)
{
    // the same checks, in the same order, as adaqp_spmm_csr makes before it looks at its workspace
    if (row_begin < 0 || row_end < row_begin || nnz < 0 || dim <= 0 || ldh < dim || ldo < dim || n_cols < 0)
        return ADAQP_EINVAL;
    const int64_t n_rows = row_end - row_begin;
    if (n_rows == 0) return ADAQP_OK;
    if (!rowptr_dev || !out_dev) return ADAQP_EINVAL;
    if (nnz > 0 && (!col_dev || !val_dev || !H_dev || n_cols == 0)) return ADAQP_EINVAL;
    if (n_rows > INT32_MAX - 1) return ADAQP_ESIZE;
    if (!aligned_to(rowptr_dev, 8) || !aligned_to(col_dev, 4) || !aligned_to(val_dev, 4) ||
        !aligned_to(H_dev, 4) || !aligned_to(out_dev, 4))
        return ADAQP_EINVAL;
    Geometry g;
    if (!geometry(n_rows, (nnz_range < 0 || nnz_range > nnz) ? nnz : nnz_range, dim, &g)) return ADAQP_ESIZE;
    if (g.bytes > (int64_t)ADAQP_SPMM_NOALLOC_SCRATCH_BYTES) return ADAQP_ESIZE;     // beyond the built-in scratch
    void *ptr = nullptr;
    const int rc = scratch_of_current_device(&ptr);
    if (rc != ADAQP_OK) return rc;
    return adaqp_spmm_csr(rowptr_dev, col_dev, val_dev, nnz, row_begin, row_end, nnz_range, H_dev, n_cols, ldh, dim,
                          out_dev, ldo, ptr, (int64_t)ADAQP_SPMM_NOALLOC_SCRATCH_BYTES, stream);
}
