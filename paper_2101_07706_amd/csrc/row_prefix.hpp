// Degrees of a set of rows, their exclusive prefix (the flat edge numbering of the edge passes) and
// the CSR start of every row: one tile of ROW_TILE rows per block, tile offsets by the single-pass
// scan across blocks.  Used by the row_prefix kernel (rows given by the caller) and by the
// adjacency kernel's spare blocks (rows = the node set just sampled, prepared for the next layer).
#pragma once
#include "lookback.hpp"

namespace csgs {

constexpr int RP_ITEMS = 4;                  // rows per thread
static_assert(ROW_TILE == 256 * RP_ITEMS, "row tile");

// Tile t of the rows S[0 .. nS).  Called by all 256 threads of a block; blocks with t >= number of
// tiles must not call.  Leaves in `meta` (by the last tile): row count, edge count (0 when above
// edge_cap: treated as empty), true edge count; in bound_note [chunk_cap + 2] what stage_slice_bounds() reads.
__device__ inline void row_prefix_tile(const int64_t *__restrict__ rowptr, int64_t n_nodes,
                                       const int32_t *__restrict__ S, int32_t nS, int64_t t, int64_t n_tiles,
                                       const TileState<1> &ts, unsigned long long tag, int64_t *__restrict__ eoff,
                                       int64_t *__restrict__ rowstart, int64_t *__restrict__ meta, int64_t edge_cap,
                                       int2 *__restrict__ bound_note, int64_t chunk_cap, int32_t *__restrict__ status)
{
    __shared__ int64_t lds[17];
    __shared__ int32_t s_deg[ROW_TILE];
    __shared__ unsigned long long s_lb[1];
    const int32_t r0 = (int32_t)(t * ROW_TILE);
    bool bad = false;
    // degrees are fetched striped (coalesced, all loads independent) and handed through LDS to a
    // blocked arrangement for the scan
#pragma unroll
    for (int k = 0; k < RP_ITEMS; ++k) {
        const int32_t a = r0 + k * 256 + (int32_t)threadIdx.x;
        int64_t deg = 0, beg = 0;
        if (a < nS) {
            const int32_t i = S[a];
            if (i >= 0 && i < n_nodes) {
                beg = rowptr[i];
                deg = rowptr[i + 1] - beg;
                if (deg < 0 || deg > 0x7FFFFFFFll) deg = 0;
            } else {
                bad = true;
            }
            rowstart[a] = beg;
        }
        s_deg[k * 256 + threadIdx.x] = (int32_t)deg;
    }
    __syncthreads();
    int32_t d[RP_ITEMS];
    int64_t sum = 0;
#pragma unroll
    for (int k = 0; k < RP_ITEMS; ++k) {
        d[k] = s_deg[threadIdx.x * RP_ITEMS + k];
        sum += d[k];
    }
    int64_t tile_total;
    int64_t ex = block_exclusive_scan<int64_t>(sum, lds, &tile_total);
    unsigned long long local[1] = {(unsigned long long)tile_total}, excl[1];
    lookback_publish<1>(ts, tag, t, local);
    lookback_resolve<1>(ts, tag, t, n_tiles, local, excl, s_lb, status);
    ex += (int64_t)excl[0];
#pragma unroll
    for (int k = 0; k < RP_ITEMS; ++k) {
        const int32_t a = r0 + (int32_t)threadIdx.x * RP_ITEMS + k;
        if (a < nS) {
            eoff[a] = ex;
            // Edge positions t * EDGE_TILE inside (ex, ex + deg]: a chunk that starts there starts in this row --
            // or, if the row ends exactly there, with the next one -- and the first row whose offset is at
            // or beyond the position is the next one.  The edge passes read this instead of searching eoff.
            const int64_t e1 = ex + d[k];
            for (int64_t tb = ex / EDGE_TILE + 1; tb <= e1 / EDGE_TILE && tb <= chunk_cap; ++tb)
                bound_note[tb] = make_int2(e1 == tb * EDGE_TILE ? a + 1 : a, a + 1);
        }
        ex += d[k];
    }
    if (bad) atomicOr(status, CSGS_ST_BAD_NODE_ID);
    if (t == n_tiles - 1 && threadIdx.x == 0) {
        const int64_t total = (int64_t)excl[0] + tile_total;
        // an edge count the workspace cannot hold is treated as empty (the weight scan reports it)
        const int64_t usable = total > edge_cap ? 0 : total;
        eoff[nS] = usable;
        meta[META_ROWS] = nS;
        meta[META_EDGES] = usable;
        meta[META_EDGES_TRUE] = total;
    }
}

// Number of tiles for nS rows: an empty row set still has one, which writes the end markers.
__device__ inline int64_t row_tiles(int32_t nS)
{
    const int64_t n = ((int64_t)nS + ROW_TILE - 1) / ROW_TILE;
    return n < 1 ? 1 : n;
}

// Fraction bits of the fixed-point weights for nS rows: the sum of nS weights must stay below
// 2^61 / (s_fx rmax); shift_base = 61 - ceil(log2 s_fx) - ceil(log2 rmax).
__device__ inline int32_t shift_for_rows(int32_t shift_base, int64_t nS)
{
    int32_t lg = 0;
    while (lg < 31 && (1ll << lg) < nS) ++lg;
    const int32_t shift = shift_base - lg;
    return shift > 52 ? 52 : shift;
}

}  // namespace csgs
