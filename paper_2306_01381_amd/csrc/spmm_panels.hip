// Neighbour aggregation (Sec. 2.1 Eq. 3: out[v] = sum_u alpha(u, v) * H[u]) for the longest rows of a power-law
// graph, as a dense product on the fp32 matrix cores.
//
// In the Reddit-shaped workload (Sec. 5: mean degree near 500) about a thousand rows per row range hold more
// than four fifths of the entries, and 32 such rows taken together reference each of their columns 5-7 times.
// The host plan groups them into panels of 32 rows: the sorted distinct columns of the panel and a dense
// [columns][32] table of coefficients.  out[panel rows] = table^T x H[columns] is then a [32 x K] x [K x dim]
// product with K in the tens of thousands.  Against the entry-by-entry kernels this fetches a row of H once per
// panel instead of once per entry and moves the multiply-adds from the vector ALUs (one 16-byte load and four
// FMAs per entry and lane) to v_mfma_f32_32x32x2_f32, at the price of multiplying by the table's zeros (its
// density is 15-20 %).  It pays only for rows with thousands of entries; everything else stays with the tiled
// kernel.
//
// Work decomposition: the panel's columns are cut at the same eight column bounds as the tiled kernel's plan
// and further into pieces of about a thousand columns; workgroup i works on pieces of tile i mod 8, so that
// each XCD's L2 keeps seeing one column range of H (chunk index outermost: one range x 128 feature columns at
// a time).  One wave = one piece x one 128-column chunk: per group of 8 panel columns it loads 4 x 16 bytes
// per lane of H (lane n of each half-wave: feature columns 4n..4n+3 of one row) and issues 16 MFMAs
// (4 k-steps x 4 interleaved 32 x 32 output tiles, tile t = feature columns 4n + t).  Each piece leaves a
// [32][dim] partial in the workspace; a second kernel adds the pieces of a panel in a fixed order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdint>
#include <cstring>
#include <vector>

#include "adaqp.h"
#include "common.hpp"

namespace adaqp {
namespace {

constexpr int kTiles = ADAQP_SPMM_TILES;
constexpr int kPanelRows = ADAQP_SPMM_PANEL_ROWS;
constexpr int kChunk = 128;                 // feature columns per wave
constexpr int kLdsPerCu = 160 * 1024;       // gfx950
constexpr int kPanelIdleLds = kLdsPerCu / 3 + 1024;     // two workgroups fit a CU, three do not

typedef float float16_t __attribute__((ext_vector_type(16)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef int int4_t __attribute__((ext_vector_type(4)));

struct PanelArgs {
    const int32_t *pcol;        // [n_groups][2][4]
    const float *palpha;        // [n_groups][64][4]
    const int32_t *piece;       // [kTiles][n_per_tile][2]
    const int32_t *panel_rows;  // [n_panels * 32]
    const int32_t *panel_piece_ptr;
    const int32_t *panel_piece;
    int32_t n_panels, n_per_tile;
    int32_t n_groups;
    int32_t n_panel_pieces;
    const float *H;
    int32_t n_cols;
    int64_t ldh;
    int32_t dim, wdim;          // wdim = dim rounded up to whole 128-byte lines
    float *out;
    int64_t ldo;
    int64_t row_begin, row_end;
    float *ppartial;            // [kTiles * n_per_tile][32][wdim]
};

// One wave: one piece x one chunk of 128 feature columns (the last chunk of a row may be 32, 64 or 96 wide).
//
// v_mfma_f32_32x32x2_f32 computes D[32][32] += A[32][2] * B[2][32] with A's element (m, k) in lane 32k + m,
// B's element (k, n) in lane 32k + n, and D's element (8 * (v / 4) + 4 * (lane / 32) + v % 4, lane % 32) in value
// v of the lane's 16.  Here m = panel row, k = panel column, n = feature column.
//
// T = output tiles of 32 feature columns: lane n of each half-wave takes feature columns T * n .. T * n + T - 1 of
// one row of H, value t of those is the B operand of tile t.  T = 4 everywhere but in a narrower last chunk, which
// then costs T / 4 of the matrix instructions instead of multiplying padding.
template <int T>
__device__ __forceinline__ void panel_piece(const PanelArgs &a, int64_t pid, int32_t g0, int32_t g1, uint32_t chunk,
                                            int lane)
{
    const int half = lane >> 5, n = lane & 31;
    const int32_t c0 = (int32_t)chunk * kChunk + T * n;     // < wdim: the chunk is 32 * T columns wide
    const float *hbase = a.H + c0;
    const uint32_t last_col = (uint32_t)a.n_cols - 1u;

    float16_t acc[T];
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.0f;

    auto meta = [&](int32_t g, int4_t *cols, float4_t *al) {
        *cols = *reinterpret_cast<const int4_t *>(a.pcol + ((int64_t)g * 2 + half) * 4);
        *al = *reinterpret_cast<const float4_t *>(a.palpha + ((int64_t)g * kWave + lane) * 4);
    };
    int4_t cols, ncols;
    float4_t al, nal;
    meta(g0, &cols, &al);
    ncols = cols;
    nal = al;
    for (int32_t g = g0; g < g1; ++g) {
        float x[4][T];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t c = min((uint32_t)cols[u], last_col);            // a corrupt plan cannot lead outside H
            const float *src = hbase + (int64_t)c * a.ldh;
            if (T == 4) {
                const float4_t v4 = *reinterpret_cast<const float4_t *>(src);
#pragma unroll
                for (int t = 0; t < T; ++t) x[u][t] = v4[t];
            } else {
#pragma unroll
                for (int t = 0; t < T; ++t) x[u][t] = src[t];
            }
        }
        if (g + 1 < g1) meta(g + 1, &ncols, &nal);                          // in flight during the MFMAs
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int t = 0; t < T; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(al[u], x[u][t], acc[t], 0, 0, 0);
        cols = ncols;
        al = nal;
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int m = 8 * (v / 4) + 4 * half + (v % 4);
        float *dst = a.ppartial + (pid * kPanelRows + m) * a.wdim + c0;
        if (T == 4) {
            float4_t r = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
            __builtin_nontemporal_store(r, reinterpret_cast<float4_t *>(dst));
        } else {
#pragma unroll
            for (int t = 0; t < T; ++t) __builtin_nontemporal_store(acc[t][v], dst + t);
        }
    }
}

__global__ __launch_bounds__(kBlock) void spmm_panel_kernel(const PanelArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const uint32_t tile = blockIdx.x % kTiles;              // = the XCD this workgroup lands on
    const uint32_t rest = blockIdx.x / kTiles;
    const uint32_t blocks_per_tile = ((uint32_t)a.n_per_tile + kWavesPerBlock - 1) / kWavesPerBlock;
    const uint32_t chunk = rest / blocks_per_tile;          // outermost: an XCD works through one chunk at a time
    const int32_t i = (int32_t)((rest % blocks_per_tile) * kWavesPerBlock + wave);
    if (i >= a.n_per_tile) return;
    const int64_t pid = (int64_t)tile * a.n_per_tile + i;
    int32_t g0 = a.piece[pid * 2], g1 = a.piece[pid * 2 + 1];
    g0 = max(0, min(g0, a.n_groups));
    g1 = min(g1, a.n_groups);
    if (g0 >= g1) return;
    // width of this chunk in tiles of 32 columns (wdim is a multiple of 32): 4 but possibly for the last chunk
    const int32_t left = a.wdim - (int32_t)chunk * kChunk;
    if (left >= kChunk) panel_piece<4>(a, pid, g0, g1, chunk, lane);
    else if (left == 96) panel_piece<3>(a, pid, g0, g1, chunk, lane);
    else if (left == 64) panel_piece<2>(a, pid, g0, g1, chunk, lane);
    else if (left == 32) panel_piece<1>(a, pid, g0, g1, chunk, lane);
}

// out[row of (panel, m)] = sum of the panel's pieces, in a fixed order; whole lines, row padding zero.
// One workgroup per (panel row, strip of 256 columns).  Its four waves take every fourth piece each (ascending, eight
// loads in flight) and leave their sums in LDS; wave 0 adds the four in wave order and stores.  A panel has 50-100
// pieces: one wave walking them all is a chain of a dozen dependent round trips with little else in flight.
__global__ __launch_bounds__(kBlock) void spmm_panel_reduce_kernel(const PanelArgs a, int32_t n_strips)
{
    __shared__ float4_t part[kWavesPerBlock][kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x >> 6;
    const int64_t pr = blockIdx.x / (uint32_t)n_strips;     // panel * 32 + m
    const int32_t strip = (int32_t)(blockIdx.x % (uint32_t)n_strips);
    const int32_t panel = (int32_t)(pr / kPanelRows);
    const int32_t m = (int32_t)(pr % kPanelRows);
    const int64_t row = a.panel_rows[pr];
    if (row < a.row_begin || row >= a.row_end) return;      // the whole workgroup: no barrier is skipped by a part
    int32_t s = a.panel_piece_ptr[panel], e = a.panel_piece_ptr[panel + 1];
    s = max(0, min(s, a.n_panel_pieces));
    e = max(s, min(e, a.n_panel_pieces));
    const int32_t n_slots = kTiles * a.n_per_tile;
    const int32_t c = strip * (kWave * 4) + lane * 4;
    const bool live = c < a.wdim;
    float4_t sum = {0.0f, 0.0f, 0.0f, 0.0f};
    if (live) {
        for (int32_t j = s + wave; j < e; j += 8 * kWavesPerBlock) {
            float4_t x[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const int32_t jq = j + q * kWavesPerBlock;
                if (jq < e) {
                    const int32_t pid = max(0, min(a.panel_piece[jq], n_slots - 1));
                    x[q] = __builtin_nontemporal_load(
                        reinterpret_cast<const float4_t *>(a.ppartial + ((int64_t)pid * kPanelRows + m) * a.wdim + c));
                }
            }
#pragma unroll
            for (int q = 0; q < 8; ++q)
                if (j + q * kWavesPerBlock < e) sum += x[q];
        }
    }
    part[wave][lane] = sum;
    __syncthreads();
    if (wave == 0 && live) {
        float4_t total = part[0][lane];
#pragma unroll
        for (int w = 1; w < kWavesPerBlock; ++w) total += part[w][lane];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (c + k >= a.dim) total[k] = 0.0f;            // row padding
        __builtin_nontemporal_store(total, reinterpret_cast<float4_t *>(a.out + row * a.ldo + c));
    }
}

int64_t panels_bytes(int64_t n_per_tile, int32_t dim)
{
    const int64_t wdim = ((int64_t)dim + 31) / 32 * 32;
    return ((int64_t)kTiles * n_per_tile * kPanelRows * wdim * 4 + 255) / 256 * 256;
}

}  // namespace
}  // namespace adaqp

using namespace adaqp;

extern "C" int adaqp_plan_spmm_panels(const int64_t *rowptr_host, const int32_t *col_host, const float *val_host,
                                      int64_t row_begin, int64_t row_end, int64_t n_cols,
                                      const int32_t *col_bounds_host, int32_t min_row_len, int32_t piece_cols,
                                      int64_t *sizes_out, int32_t *tile_off_inout, int32_t *panel_rows_out,
                                      int32_t *pcol_out, float *palpha_out, int32_t *piece_out,
                                      int32_t *panel_piece_ptr_out, int32_t *panel_piece_out)
{
    if (row_begin < 0 || row_end < row_begin || n_cols < 0 || n_cols > INT32_MAX) return ADAQP_EINVAL;
    if (!rowptr_host || !col_bounds_host || !sizes_out) return ADAQP_EINVAL;
    if (min_row_len < 1 || piece_cols < 8 || piece_cols % 8 != 0) return ADAQP_EINVAL;
    const bool fill = panel_rows_out != nullptr;
    if (fill && (!pcol_out || !palpha_out || !piece_out || !panel_piece_ptr_out || !panel_piece_out || !val_host))
        return ADAQP_EINVAL;
    for (int t = 0; t < kTiles; ++t)
        if (col_bounds_host[t] < 0 || col_bounds_host[t + 1] < col_bounds_host[t] || col_bounds_host[t + 1] > n_cols)
            return ADAQP_EINVAL;

    // the rows that go into panels: longest first
    std::vector<int64_t> heavy;
    for (int64_t r = row_begin; r < row_end; ++r) {
        const int64_t s = rowptr_host[r], e = rowptr_host[r + 1];
        if (s < 0 || e < s || e - s > INT32_MAX) return ADAQP_EINVAL;
        if (e - s >= min_row_len) heavy.push_back(r);
    }
    std::stable_sort(heavy.begin(), heavy.end(), [&](int64_t x, int64_t y) {
        return rowptr_host[x + 1] - rowptr_host[x] > rowptr_host[y + 1] - rowptr_host[y];
    });
    const int64_t n_heavy = (int64_t)heavy.size();
    const int64_t n_panels = (n_heavy + kPanelRows - 1) / kPanelRows;
    if (n_panels > INT32_MAX / kPanelRows) return ADAQP_ESIZE;
    if (n_heavy > 0 && !col_host) return ADAQP_EINVAL;

    if (fill) {
        if (sizes_out[2] < 0 || sizes_out[2] > INT32_MAX - 1) return ADAQP_EINVAL;
        std::memset(palpha_out, 0, (size_t)sizes_out[2] * kWave * 4 * sizeof(float));
    }
    struct Piece {
        int32_t panel, g0, g1, first_col;
    };
    std::vector<Piece> lists[kTiles];
    std::vector<uint8_t> used((size_t)n_cols, 0);
    std::vector<int64_t> where(fill ? (size_t)n_cols : 0, 0);   // panel column (padded numbering) of a column of H
    std::vector<int32_t> distinct;
    const int32_t piece_groups = piece_cols / 8;
    int64_t n_groups = 0;
    for (int64_t p = 0; p < n_panels; ++p) {
        const int64_t m_end = std::min<int64_t>(kPanelRows, n_heavy - p * kPanelRows);
        int32_t lo = INT32_MAX, hi = -1;
        for (int64_t m = 0; m < m_end; ++m) {
            const int64_t r = heavy[(size_t)(p * kPanelRows + m)];
            for (int64_t j = rowptr_host[r]; j < rowptr_host[r + 1]; ++j) {
                const int32_t c = col_host[j];
                if (c < 0 || c >= n_cols) return ADAQP_EINVAL;
                if (j > rowptr_host[r] && col_host[j - 1] >= c) return ADAQP_EINVAL;
                used[(size_t)c] = 1;
                lo = std::min(lo, c);
                hi = std::max(hi, c);
            }
        }
        distinct.clear();
        for (int32_t c = lo; c <= hi; ++c)
            if (used[(size_t)c]) {
                distinct.push_back(c);
                used[(size_t)c] = 0;
            }
        // cut at the tile bounds (the last tile also takes anything at or beyond its upper bound)
        size_t at = 0;
        for (int t = 0; t < kTiles; ++t) {
            size_t end = at;
            if (t == kTiles - 1) end = distinct.size();
            else while (end < distinct.size() && distinct[end] < col_bounds_host[t + 1]) ++end;
            const int64_t len = (int64_t)(end - at);
            if (len > 0) {
                const int64_t ng = (len + 7) / 8;
                if (n_groups + ng > INT32_MAX - 1) return ADAQP_ESIZE;
                if (fill && n_groups + ng > sizes_out[2]) return ADAQP_EINVAL;      // arrays sized for another plan
                if (fill) {
                    for (int64_t k = 0; k < ng * 8; ++k) {
                        // padding repeats the last column (with coefficient 0)
                        const int32_t c = distinct[at + (size_t)std::min<int64_t>(k, len - 1)];
                        const int64_t G = n_groups * 8 + k;
                        const int64_t g = G / 8, h = G % 2, u = (G % 8) / 2;
                        pcol_out[(g * 2 + h) * 4 + u] = c;
                        if (k < len) where[(size_t)c] = G;
                    }
                }
                // as few pieces as piece_cols allows, equal to within one group (pieces of one size finish together)
                const int64_t n_cut = (ng + piece_groups - 1) / piece_groups;
                for (int64_t q = 0; q < n_cut; ++q) {
                    const int64_t s0 = ng * q / n_cut, s1 = ng * (q + 1) / n_cut;
                    lists[t].push_back(Piece{(int32_t)p, (int32_t)(n_groups + s0), (int32_t)(n_groups + s1),
                                             distinct[at + (size_t)(s0 * 8)]});
                }
                n_groups += ng;
            }
            at = end;
        }
        if (fill) {
            // coefficients: zero everywhere (cleared above), then the entries of the panel's rows
            for (int64_t m = 0; m < m_end; ++m) {
                const int64_t r = heavy[(size_t)(p * kPanelRows + m)];
                for (int64_t j = rowptr_host[r]; j < rowptr_host[r + 1]; ++j) {
                    const int64_t G = where[(size_t)col_host[j]];
                    const int64_t g = G / 8, h = G % 2, u = (G % 8) / 2;
                    palpha_out[((g * kWave) + h * 32 + m) * 4 + u] = val_host[j];
                }
            }
        }
    }
    // within a tile, pieces in order of their first column: the pieces of different panels that walk the same
    // rows of H are launched next to each other (a few percent faster than panel by panel)
    for (int t = 0; t < kTiles; ++t)
        std::stable_sort(lists[t].begin(), lists[t].end(),
                         [](const Piece &x, const Piece &y) { return x.first_col < y.first_col; });
    size_t n_per_tile = 0, n_pieces = 0;
    for (int t = 0; t < kTiles; ++t) {
        n_per_tile = std::max(n_per_tile, lists[t].size());
        n_pieces += lists[t].size();
    }
    if ((int64_t)n_per_tile * kTiles > INT32_MAX) return ADAQP_ESIZE;
    if (!fill) {
        sizes_out[0] = n_heavy;
        sizes_out[1] = n_panels;
        sizes_out[2] = n_groups;
        sizes_out[3] = (int64_t)n_per_tile;
        sizes_out[4] = (int64_t)n_pieces;
        return ADAQP_OK;
    }
    if (sizes_out[0] != n_heavy || sizes_out[1] != n_panels || sizes_out[2] != n_groups ||
        sizes_out[3] != (int64_t)n_per_tile || sizes_out[4] != (int64_t)n_pieces)
        return ADAQP_EINVAL;                                // the arrays were sized for another plan
    for (int64_t k = 0; k < n_panels * kPanelRows; ++k)
        panel_rows_out[k] = k < n_heavy ? (int32_t)heavy[(size_t)k] : -1;
    std::fill(piece_out, piece_out + (size_t)kTiles * n_per_tile * 2, 0);
    std::vector<int32_t> count((size_t)n_panels + 1, 0);
    for (int t = 0; t < kTiles; ++t)
        for (size_t i = 0; i < lists[t].size(); ++i) {
            piece_out[((size_t)t * n_per_tile + i) * 2] = lists[t][i].g0;
            piece_out[((size_t)t * n_per_tile + i) * 2 + 1] = lists[t][i].g1;
            ++count[(size_t)lists[t][i].panel + 1];
        }
    for (int64_t p = 0; p < n_panels; ++p) count[(size_t)p + 1] += count[(size_t)p];
    std::copy(count.begin(), count.end(), panel_piece_ptr_out);
    std::vector<int32_t> next(count.begin(), count.end() - 1);
    for (int t = 0; t < kTiles; ++t)                        // ascending piece number within each panel
        for (size_t i = 0; i < lists[t].size(); ++i)
            panel_piece_out[next[(size_t)lists[t][i].panel]++] = (int32_t)((size_t)t * n_per_tile + i);
    if (tile_off_inout)
        for (int64_t k = 0; k < n_heavy; ++k)
            std::fill_n(tile_off_inout + (heavy[(size_t)k] - row_begin) * (kTiles + 1), kTiles + 1, -1);
    return ADAQP_OK;
}

extern "C" int32_t adaqp_spmm_panels_pay(int64_t n_panel_pieces, int32_t dim)
{
    if (n_panel_pieces <= 0 || dim <= 0) return 0;
    const int64_t chunks = ((int64_t)dim + 127) / 128;
    return n_panel_pieces * chunks >= ADAQP_SPMM_PANEL_MIN_WAVES ? 1 : 0;
}

extern "C" int adaqp_spmm_panels_workspace_bytes(int32_t n_per_tile, int32_t dim, int64_t *bytes_out)
{
    if (!bytes_out || n_per_tile < 0 || dim <= 0) return ADAQP_EINVAL;
    *bytes_out = panels_bytes(n_per_tile, dim);
    return ADAQP_OK;
}

extern "C" int adaqp_spmm_csr_panels(const adaqp_spmm_panels *p, int64_t row_begin, int64_t row_end,
                                     const float *H_dev, int64_t n_cols, int64_t ldh, int32_t dim, float *out_dev,
                                     int64_t ldo, void *workspace_dev, int64_t workspace_bytes, void *stream)
{
    if (!p) return ADAQP_EINVAL;
    if (p->n_panels < 0 || p->n_per_tile < 0 || p->n_groups < 0 || p->n_panel_pieces < 0) return ADAQP_EINVAL;
    if (row_begin < 0 || row_end < row_begin || dim <= 0 || ldh < dim || ldo < dim || n_cols < 0) return ADAQP_EINVAL;
    if (p->n_panels == 0 || p->n_per_tile == 0 || row_end == row_begin) return ADAQP_OK;
    if (p->n_groups > INT32_MAX - 1 || p->n_panel_pieces > INT32_MAX || n_cols > INT32_MAX) return ADAQP_ESIZE;
    if (p->n_panels > INT32_MAX / kPanelRows || (int64_t)p->n_per_tile * kTiles > INT32_MAX) return ADAQP_ESIZE;
    if (p->n_panel_pieces > (int64_t)p->n_per_tile * kTiles) return ADAQP_EINVAL;
    if (!p->panel_rows_dev || !p->pcol_dev || !p->palpha_dev || !p->piece_dev || !p->panel_piece_ptr_dev ||
        !p->panel_piece_dev || !H_dev || !out_dev || n_cols == 0)
        return ADAQP_EINVAL;
    if (!aligned_to(p->panel_rows_dev, 4) || !aligned_to(p->pcol_dev, 16) || !aligned_to(p->palpha_dev, 16) ||
        !aligned_to(p->piece_dev, 4) || !aligned_to(p->panel_piece_ptr_dev, 4) || !aligned_to(p->panel_piece_dev, 4))
        return ADAQP_EINVAL;
    if (ldh % 32 != 0 || ldo % 32 != 0 || !aligned_to(H_dev, 128) || !aligned_to(out_dev, 128)) return ADAQP_EINVAL;
    const int64_t need = panels_bytes(p->n_per_tile, dim);
    if (!workspace_dev || !aligned_to(workspace_dev, 256)) return ADAQP_EINVAL;
    if (workspace_bytes < need) return ADAQP_ESIZE;

    PanelArgs a;
    a.pcol = p->pcol_dev;
    a.palpha = p->palpha_dev;
    a.piece = p->piece_dev;
    a.panel_rows = p->panel_rows_dev;
    a.panel_piece_ptr = p->panel_piece_ptr_dev;
    a.panel_piece = p->panel_piece_dev;
    a.n_panels = p->n_panels;
    a.n_per_tile = p->n_per_tile;
    a.n_groups = (int32_t)p->n_groups;
    a.n_panel_pieces = (int32_t)p->n_panel_pieces;
    a.H = H_dev;
    a.n_cols = (int32_t)n_cols;
    a.ldh = ldh;
    a.dim = dim;
    a.wdim = (dim + 31) / 32 * 32;
    a.out = out_dev;
    a.ldo = ldo;
    a.row_begin = row_begin;
    a.row_end = row_end;
    a.ppartial = reinterpret_cast<float *>(workspace_dev);
    const int64_t n_chunks = (a.wdim + kChunk - 1) / kChunk;
    const int64_t blocks_per_tile = ((int64_t)p->n_per_tile + kWavesPerBlock - 1) / kWavesPerBlock;
    const int64_t blocks = blocks_per_tile * kTiles * n_chunks;
    if (blocks > 0x7FFFFFFF) return ADAQP_ESIZE;
    hipStream_t st = (hipStream_t)stream;
    // Two workgroups per CU, i.e. two waves per SIMD: kPanelIdleLds bytes of dynamic LDS that the kernel never
    // touches keep a third workgroup off the CU.  Measured on MI355X: a SIMD's fp32 MFMA rate is 98 % of peak with
    // one to three waves issuing MFMAs back to back and 80 % with four, the kernel alone is 5 % faster at two waves
    // than at the four its registers allow, and next to the tiled kernel (adaqp_layer_step's two-stream schedules)
    // the registers it leaves free let more of that kernel's waves onto the SIMD.
    hipLaunchKernelGGL(spmm_panel_kernel, dim3((unsigned)blocks), dim3(kBlock), (size_t)kPanelIdleLds, st, a);
    ADAQP_HIP_TRY(hipGetLastError());
    const int64_t n_strips = (a.wdim + kWave * 4 - 1) / (kWave * 4);
    const int64_t rblocks = (int64_t)p->n_panels * kPanelRows * n_strips;
    if (rblocks > 0x7FFFFFFF) return ADAQP_ESIZE;
    hipLaunchKernelGGL(spmm_panel_reduce_kernel, dim3((unsigned)rblocks), dim3(kBlock), 0, st, a, (int32_t)n_strips);
    ADAQP_HIP_TRY(hipGetLastError());
    return ADAQP_OK;
}
