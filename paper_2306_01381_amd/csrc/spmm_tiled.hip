// Neighbour aggregation (Sec. 2.1 Eq. 3: out[v] = sum_u alpha(u, v) * H[u]) for graphs whose rows are long
// enough that every row of H is used hundreds of times - the regime of the paper's densest dataset (mean
// degree near 500), where the merge-path kernel streams the same 240 MB operand 290 times.
//
// MI355X has eight XCDs with a private 4 MB L2 each, and workgroups are dealt to XCDs round-robin.  The columns
// of the graph are cut into eight ranges ("tiles", equal entry counts, planned on the host once per graph) and
// the feature columns into chunks of 64 or 128; workgroup i works on tile i mod 8, so an XCD only ever touches
// one tile's rows of H, and with the chunk index outermost its working set at any time is one tile x one chunk:
// a few MB that stay in its L2 (hit rate 84-87 % on the Reddit-shaped workload against 5-7 % untiled).  A gather
// of that shape runs at about 25 TB/s on this part against 8-9 TB/s when the same rows come through the fabric.
// The price: every (row, tile) segment leaves a partial sum in a workspace, added up in tile order by a second
// kernel (deterministic), and the entries are re-read once per chunk.  Two choices of the plan keep that price
// down: rows shorter than ADAQP_SPMM_TILED_SHORT_ROW are not cut up (each goes whole to one tile), and the chunk
// is narrowed to 64 columns when a 128-column chunk of the widest column range would not fit an L2.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <type_traits>
#include <vector>

#include "adaqp.h"
#include "common.hpp"

namespace adaqp {
namespace {

constexpr int kTiles = ADAQP_SPMM_TILES;

struct TiledArgs {
    const int64_t *rowptr;      // already offset to row_begin: rowptr[0..n_rows]
    const int32_t *col;
    const float *val;
    int64_t nnz;
    int32_t n_rows;
    const int32_t *tile_off;    // [n_rows][kTiles + 1]: entries of the row that precede each tile
    const float *H;
    int64_t n_cols, ldh;
    int32_t dim, wdim;          // wdim = dim rounded up to whole 128-byte lines
    float *out;                 // already offset to row_begin
    int64_t ldo;
    float *partial;             // [kTiles][n_rows][wdim]
    uint32_t n_row_blocks;
    int32_t rows_per_wave;
};

__device__ __forceinline__ int32_t uniform_i32(int32_t v) { return __builtin_amdgcn_readfirstlane(v); }

__device__ __forceinline__ int64_t clamp64(int64_t v, int64_t lo, int64_t hi) { return v < lo ? lo : (v > hi ? hi : v); }

// Entries of row r that fall into `tile`, clamped so that a corrupt plan or rowptr cannot lead outside the arrays.
__device__ __forceinline__ void segment(const TiledArgs &a, int64_t r, int tile, int64_t *first, int32_t *count)
{
    const int64_t lo = clamp64(a.rowptr[r], 0, a.nnz);
    const int64_t hi = clamp64(a.rowptr[r + 1], lo, a.nnz);
    const int32_t *off = a.tile_off + r * (kTiles + 1) + tile;
    const int64_t s = clamp64(lo + off[0], lo, hi);
    const int64_t e = clamp64(lo + off[1], s, hi);
    const int64_t n = e - s;
    *first = s;
    *count = n > 0x7FFFFFFF ? 0x7FFFFFFF : (int32_t)n;
}

typedef float float4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store4_streaming(float *p, const float *v)
{
    float4_t x = {v[0], v[1], v[2], v[3]};
    __builtin_nontemporal_store(x, reinterpret_cast<float4_t *>(p));
}

__device__ __forceinline__ void load4_streaming(const float *p, float *v)
{
    const float4_t x = __builtin_nontemporal_load(reinterpret_cast<const float4_t *>(p));
    v[0] = x[0];
    v[1] = x[1];
    v[2] = x[2];
    v[3] = x[3];
}

__device__ __forceinline__ int32_t shuffle_i32(int32_t v, int src_lane)
{
    return __builtin_amdgcn_ds_bpermute(src_lane << 2, v);
}

__device__ __forceinline__ float shuffle_f32(float v, int src_lane)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src_lane << 2, __builtin_bit_cast(int32_t, v)));
}

// LPE lanes share one entry; each lane holds VPL vectors of four columns, LPE * 4 columns apart, so a chunk is
// CW = LPE * 4 * VPL columns and every load instruction reads whole 128-byte lines.  One "step" fetches
// SLOTS = 64 / LPE entries with VPL loads that share the column lookup and the address arithmetic; up to
// 8 / VPL steps (8 KB per wave) are in flight, and the tail of a segment is issued in groups of 4, 2 and 1 steps
// so that a row with two entries in this tile costs one load, not eight.  The inner loop is branch-free: per
// step two cross-lane reads (column, coefficient), one 32 x 32 -> 64-bit multiply-add for the address, VPL loads,
// 4 * VPL multiply-adds.  Measured on this part the kernel is bound by the rate at which a CU's vector memory
// pipeline takes 16-byte-per-lane gathers (about 22 TB/s over the chip with every row L1-resident), not by L2.
template <int LPE, int VPL>
__global__ __launch_bounds__(kBlock) void spmm_tiled_kernel(const TiledArgs a)
{
    constexpr int SLOTS = kWave / LPE;
    constexpr int CW = LPE * 4 * VPL;
    constexpr int UMAX = 8 / VPL;                           // load steps in flight: 8 KB per wave
    static_assert(LPE % UMAX == 0, "a batch of 64 entries is LPE load steps: a whole number of full groups");
    const int lane = threadIdx.x & (kWave - 1);
    const int q = lane / LPE, l = lane % LPE;
    // the tile is the fastest-running index: consecutive workgroups land on consecutive XCDs
    const uint32_t tile = blockIdx.x % kTiles;
    const uint32_t rest = blockIdx.x / kTiles;
    const uint32_t rb = rest % a.n_row_blocks;
    const uint32_t chunk = rest / a.n_row_blocks;
    const int32_t c0 = (int32_t)chunk * CW + l * 4;         // first vector of the lane; vector v is LPE * 4 columns on
    bool live[VPL];                                         // wdim is a multiple of 32: a live vector is whole
#pragma unroll
    for (int v = 0; v < VPL; ++v) live[v] = c0 + v * LPE * 4 < a.wdim;
    const int wave = uniform_i32((int32_t)(threadIdx.x >> 6));
    const int64_t r_begin = ((int64_t)rb * kWavesPerBlock + wave) * a.rows_per_wave;
    if (r_begin >= a.n_rows) return;
    const int32_t n_mine = (int32_t)(r_begin + a.rows_per_wave < a.n_rows ? a.rows_per_wave : a.n_rows - r_begin);
    // a vector past the row's end is read from the start of the row instead and never stored: no masked loads
    const float *hlane[VPL];
#pragma unroll
    for (int v = 0; v < VPL; ++v) hlane[v] = a.H + (live[v] ? c0 + v * LPE * 4 : 0);
    const uint32_t pitch = (uint32_t)a.ldh * 4u;            // bytes; the host checks that it fits

    // lanes 0..n_mine-1 look up their row's segment (one memory round trip for all the wave's rows)
    int64_t my_first = 0;
    int32_t my_count = 0;
    if (lane < n_mine) segment(a, r_begin + lane, (int)tile, &my_first, &my_count);
    const int32_t my_first_lo = (int32_t)(uint32_t)my_first, my_first_hi = (int32_t)(my_first >> 32);
    uint64_t todo = __ballot(my_count > 0);                 // rows that have entries in this tile
    if (todo == 0) return;                                  // the reduction skips these partials as well

    // the wave's work as a sequence of batches of up to 64 entries of one row; the next batch's (col, val) are
    // requested before the current batch is worked on
    int32_t row = (int32_t)__builtin_ctzll(todo);           // relative to r_begin
    int64_t first = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane(my_first_hi, row) << 32) |
                              (uint32_t)__builtin_amdgcn_readlane(my_first_lo, row));
    int32_t count = __builtin_amdgcn_readlane(my_count, row);
    int32_t j = 0;
    auto request = [&](int32_t *col_out, float *val_out) {
        // lane i holds entry j + i.  A lane without an entry repeats the batch's first entry with a zero
        // coefficient (a row that is being fetched anyway); an out-of-range column reads row 0 likewise
        const int32_t nb = count - j < kWave ? count - j : kWave;
        const int32_t mine = lane < nb ? lane : 0;
        *col_out = __builtin_nontemporal_load(a.col + first + j + mine);
        *val_out = __builtin_nontemporal_load(a.val + first + j + mine);
    };
    int32_t nx_col;
    float nx_val;
    request(&nx_col, &nx_val);

    float acc[VPL][4];
#pragma unroll
    for (int v = 0; v < VPL; ++v)
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[v][k] = 0.0f;

    for (;;) {
        const int32_t nb = count - j < kWave ? count - j : kWave;
        const int32_t this_row = row;
        const bool row_ends = j + kWave >= count;
        int32_t my_col = nx_col;
        float my_val = nx_val;
        if (lane >= nb) my_val = 0.0f;
        if ((uint32_t)my_col >= (uint32_t)a.n_cols) { my_col = 0; my_val = 0.0f; }
        // move on and request the next batch
        bool more = true;
        if (!row_ends) {
            j += kWave;
        } else {
            todo &= todo - 1;
            if (todo != 0) {
                row = (int32_t)__builtin_ctzll(todo);
                first = (int64_t)(((uint64_t)(uint32_t)__builtin_amdgcn_readlane(my_first_hi, row) << 32) |
                                  (uint32_t)__builtin_amdgcn_readlane(my_first_lo, row));
                count = __builtin_amdgcn_readlane(my_count, row);
                j = 0;
            } else {
                more = false;
            }
        }
        if (more) request(&nx_col, &nx_val);

        const int32_t n_it = (nb + SLOTS - 1) / SLOTS;
        // UU load steps at once, starting at step `it`
        auto group = [&](auto uu_tag, int32_t it) {
            constexpr int UU = decltype(uu_tag)::value;
            float h[UU][VPL][4];
            float alpha[UU];
#pragma unroll
            for (int u = 0; u < UU; ++u) {
                const int e = ((it + u) * SLOTS + q) & (kWave - 1);            // < 64: it + u < LPE
                const uint32_t c = (uint32_t)shuffle_i32(my_col, e);
                alpha[u] = shuffle_f32(my_val, e);
                const uint64_t off = (uint64_t)c * pitch;                      // one 32 x 32 -> 64 multiply
#pragma unroll
                for (int v = 0; v < VPL; ++v) {
                    const float4 x = *reinterpret_cast<const float4 *>(
                        reinterpret_cast<const char *>(hlane[v]) + off);
                    h[u][v][0] = x.x;
                    h[u][v][1] = x.y;
                    h[u][v][2] = x.z;
                    h[u][v][3] = x.w;
                }
            }
#pragma unroll
            for (int u = 0; u < UU; ++u)
#pragma unroll
                for (int v = 0; v < VPL; ++v)
#pragma unroll
                    for (int k = 0; k < 4; ++k) acc[v][k] = fmaf(alpha[u], h[u][v][k], acc[v][k]);
        };
        int32_t it = 0;
        for (; it + UMAX <= n_it; it += UMAX) group(std::integral_constant<int, UMAX>(), it);
        if constexpr (UMAX >= 8) {
            if (it + 4 <= n_it) {
                group(std::integral_constant<int, 4>(), it);
                it += 4;
            }
        }
        if constexpr (UMAX >= 4) {
            if (it + 2 <= n_it) {
                group(std::integral_constant<int, 2>(), it);
                it += 2;
            }
        }
        if constexpr (UMAX >= 2) {
            if (it < n_it) group(std::integral_constant<int, 1>(), it);
        }

        if (row_ends) {
            // the SLOTS partial sums of the row, combined pairwise in a fixed order
#pragma unroll
            for (int step = LPE; step < kWave; step <<= 1)
#pragma unroll
                for (int v = 0; v < VPL; ++v)
#pragma unroll
                    for (int k = 0; k < 4; ++k) acc[v][k] += shuffle_f32(acc[v][k], lane ^ step);
            if (q == 0) {
                float *p = a.partial + ((int64_t)tile * a.n_rows + r_begin + this_row) * a.wdim + c0;
#pragma unroll
                for (int v = 0; v < VPL; ++v)
                    if (live[v]) store4_streaming(p + v * LPE * 4, acc[v]);
            }
#pragma unroll
            for (int v = 0; v < VPL; ++v)
#pragma unroll
                for (int k = 0; k < 4; ++k) acc[v][k] = 0.0f;
        }
        if (!more) break;
    }
}

// out[r] = sum over the tiles that hold entries of row r, in tile order; whole lines, row padding zero.
__global__ __launch_bounds__(kBlock) void spmm_tiled_reduce_kernel(const TiledArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (r >= a.n_rows) return;
    if (a.tile_off[r * (kTiles + 1)] < 0) return;           // a row struck from the table: someone else's to write
    uint32_t present = 0;
    for (int t = 0; t < kTiles; ++t) {
        int64_t first;
        int32_t count;
        segment(a, r, t, &first, &count);
        if (count > 0) present |= 1u << t;
    }
    present = (uint32_t)uniform_i32((int32_t)present);
    float *o = a.out + r * a.ldo;
    for (int32_t c = lane * 4; c < a.wdim; c += kWave * 4) {
        float x[kTiles][4];
#pragma unroll
        for (int t = 0; t < kTiles; ++t) {
            if (present & (1u << t)) {
                load4_streaming(a.partial + ((int64_t)t * a.n_rows + r) * a.wdim + c, x[t]);
            } else {
                x[t][0] = x[t][1] = x[t][2] = x[t][3] = 0.0f;
            }
        }
        float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int t = 0; t < kTiles; ++t)
            if (present & (1u << t))
#pragma unroll
                for (int k = 0; k < 4; ++k) sum[k] += x[t][k];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (c + k >= a.dim) sum[k] = 0.0f;              // row padding
        store4_streaming(o + c, sum);
    }
}

int64_t tiled_bytes(int64_t n_rows, int32_t dim)
{
    const int64_t wdim = ((int64_t)dim + 31) / 32 * 32;
    return ((int64_t)kTiles * n_rows * wdim * 4 + 255) / 256 * 256;
}

}  // namespace
}  // namespace adaqp

using namespace adaqp;

extern "C" int adaqp_plan_spmm_tiles(const int64_t *rowptr_host, const int32_t *col_host, int64_t row_begin,
                                     int64_t row_end, int64_t n_cols, int32_t *col_bounds_out,
                                     int32_t *tile_off_out)
{
    if (row_begin < 0 || row_end < row_begin || n_cols < 0 || n_cols > INT32_MAX) return ADAQP_EINVAL;
    if (!rowptr_host || !col_bounds_out) return ADAQP_EINVAL;
    const int64_t n_rows = row_end - row_begin;
    if (n_rows > 0 && !tile_off_out) return ADAQP_EINVAL;
    const int64_t e0 = rowptr_host[row_begin], e1 = rowptr_host[row_end];
    if (e0 < 0 || e1 < e0) return ADAQP_EINVAL;
    if (e1 > e0 && !col_host) return ADAQP_EINVAL;
    // entries per column, then boundaries at equal entry counts
    std::vector<int64_t> uses((size_t)n_cols + 1, 0);
    for (int64_t r = row_begin; r < row_end; ++r) {
        const int64_t s = rowptr_host[r], e = rowptr_host[r + 1];
        if (e < s || e - s > INT32_MAX) return ADAQP_EINVAL;
        for (int64_t j = s; j < e; ++j) {
            const int32_t c = col_host[j];
            if (c < 0 || c >= n_cols) return ADAQP_EINVAL;
            if (j > s && col_host[j - 1] >= c) return ADAQP_EINVAL;        // rows must list ascending, distinct columns
            ++uses[(size_t)c];
        }
    }
    const int64_t total = e1 - e0;
    col_bounds_out[0] = 0;
    {
        int64_t seen = 0;
        int32_t c = 0;
        for (int t = 1; t < kTiles; ++t) {
            const int64_t want = (total * t + kTiles - 1) / kTiles;
            while (c < n_cols && seen < want) seen += uses[(size_t)c++];
            col_bounds_out[t] = c;
        }
        // the last range ends after the last column that is referenced (a row range may use only part of
        // the columns: central rows never point at halo columns)
        int64_t last = n_cols;
        while (last > 0 && uses[(size_t)last - 1] == 0) --last;
        col_bounds_out[kTiles] = (int32_t)std::max<int64_t>(last, c);
    }
    for (int64_t r = row_begin; r < row_end; ++r) {
        const int32_t *cb = col_host + rowptr_host[r];
        const int32_t *ce = col_host + rowptr_host[r + 1];
        int32_t *off = tile_off_out + (r - row_begin) * (kTiles + 1);
        const int32_t degree = (int32_t)(ce - cb);
        if (degree < ADAQP_SPMM_TILED_SHORT_ROW) {
            // a short row is not worth eight segments: all of it goes to one tile (rows take turns), its few
            // neighbour rows outside that tile's column range are fetched past the L2
            const int home = (int)((r - row_begin) % kTiles);
            for (int t = 0; t <= kTiles; ++t) off[t] = t <= home ? 0 : degree;
        } else {
            for (int t = 0; t <= kTiles; ++t) off[t] = (int32_t)(std::lower_bound(cb, ce, col_bounds_out[t]) - cb);
        }
    }
    return ADAQP_OK;
}

extern "C" int32_t adaqp_spmm_tiled_pays(int64_t n_rows, int64_t nnz)
{
    // a partial row per (row, tile) with entries, written and read back, against one neighbour row per entry
    // fetched 2-3 times faster: worth it from a mean row length of about a hundred entries (measured: wins
    // at 440-520, loses at 9-43)
    return n_rows > 0 && nnz >= ADAQP_SPMM_TILED_MIN_MEAN_ROW * n_rows ? 1 : 0;
}

extern "C" int32_t adaqp_spmm_tiled_chunk_cols(const int32_t *col_bounds_host, int32_t dim)
{
    if (!col_bounds_host || dim <= 0) return 0;
    if (dim <= 96) return 64;                               // narrower than one wide chunk
    int64_t widest = 0;
    for (int t = 0; t < kTiles; ++t)
        widest = std::max<int64_t>(widest, (int64_t)col_bounds_host[t + 1] - col_bounds_host[t]);
    // an XCD's live working set is (rows of H in its column range) x (chunk bytes); past about 5 MB the 4 MB L2
    // misses often enough that halving the chunk pays for the extra pass over the entries
    return widest * 512 > (int64_t)5 << 20 ? 64 : 128;
}

extern "C" int adaqp_spmm_tiled_workspace_bytes(int64_t n_rows, int32_t dim, int64_t *bytes_out)
{
    if (!bytes_out || n_rows < 0 || dim <= 0) return ADAQP_EINVAL;
    if (n_rows > INT32_MAX - 1) return ADAQP_ESIZE;
    *bytes_out = tiled_bytes(n_rows, dim);
    return ADAQP_OK;
}

extern "C" int adaqp_spmm_csr_tiled(const int64_t *rowptr_dev, const int32_t *col_dev, const float *val_dev,
                                    int64_t nnz, int64_t row_begin, int64_t row_end, const float *H_dev,
                                    int64_t n_cols, int64_t ldh, int32_t dim, float *out_dev, int64_t ldo,
                                    const int32_t *tile_off_dev, int32_t chunk_cols, void *workspace_dev,
                                    int64_t workspace_bytes, void *stream)
{
    if (chunk_cols != 0 && chunk_cols != 64 && chunk_cols != 128) return ADAQP_EINVAL;
    if (row_begin < 0 || row_end < row_begin || nnz < 0 || dim <= 0 || ldh < dim || ldo < dim || n_cols < 0)
        return ADAQP_EINVAL;
    const int64_t n_rows = row_end - row_begin;
    if (n_rows == 0) return ADAQP_OK;
    if (!rowptr_dev || !out_dev || !tile_off_dev) return ADAQP_EINVAL;
    if (nnz > 0 && (!col_dev || !val_dev || !H_dev || n_cols == 0)) return ADAQP_EINVAL;
    if (n_rows > INT32_MAX - 1) return ADAQP_ESIZE;
    if (!aligned_to(rowptr_dev, 8) || !aligned_to(col_dev, 4) || !aligned_to(val_dev, 4) ||
        !aligned_to(tile_off_dev, 4))
        return ADAQP_EINVAL;
    // this kernel exists for the line-padded layout only: whole 128-byte lines in and out
    if (ldh % 32 != 0 || ldo % 32 != 0 || !aligned_to(H_dev, 128) || !aligned_to(out_dev, 128)) return ADAQP_EINVAL;
    if (ldh >= ((int64_t)1 << 30)) return ADAQP_ESIZE;                          // the row pitch in bytes stays in 32 bits
    const int64_t need = tiled_bytes(n_rows, dim);
    if (!workspace_dev || !aligned_to(workspace_dev, 256)) return ADAQP_EINVAL;
    if (workspace_bytes < need) return ADAQP_ESIZE;

    TiledArgs a;
    a.rowptr = rowptr_dev + row_begin;
    a.col = col_dev;
    a.val = val_dev;
    a.nnz = nnz;
    a.n_rows = (int32_t)n_rows;
    a.tile_off = tile_off_dev;
    a.H = H_dev;
    a.n_cols = n_cols;
    a.ldh = ldh;
    a.dim = dim;
    a.wdim = (dim + 31) / 32 * 32;
    a.out = out_dev + row_begin * ldo;
    a.ldo = ldo;
    a.partial = reinterpret_cast<float *>(workspace_dev);
    a.rows_per_wave = 4;                                    // <= 64: a wave keeps its rows' segments in lanes
    const int64_t rows_per_block = (int64_t)a.rows_per_wave * kWavesPerBlock;
    a.n_row_blocks = (uint32_t)((n_rows + rows_per_block - 1) / rows_per_block);
    // 128-column chunks (32 lanes x one vector per entry) unless the caller asks for 64 or the rows are narrower
    const bool wide = a.wdim >= 128 && chunk_cols != 64;
    const int cw = wide ? 128 : 64;
    const int64_t n_chunks = (a.wdim + cw - 1) / cw;
    const int64_t blocks = (int64_t)a.n_row_blocks * kTiles * n_chunks;
    if (blocks > 0x7FFFFFFF) return ADAQP_ESIZE;
    hipStream_t st = (hipStream_t)stream;
    if (wide) hipLaunchKernelGGL((spmm_tiled_kernel<32, 1>), dim3((unsigned)blocks), dim3(kBlock), 0, st, a);
    else hipLaunchKernelGGL((spmm_tiled_kernel<16, 1>), dim3((unsigned)blocks), dim3(kBlock), 0, st, a);
    ADAQP_HIP_TRY(hipGetLastError());
    const int64_t rblocks = (n_rows + kWavesPerBlock - 1) / kWavesPerBlock;
    hipLaunchKernelGGL(spmm_tiled_reduce_kernel, dim3((unsigned)rblocks), dim3(kBlock), 0, st, a);
    ADAQP_HIP_TRY(hipGetLastError());
    return ADAQP_OK;
}
