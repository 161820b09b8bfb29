// Shared device helpers and the workspace layout of the csgs library (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "csgs.h"
#include "profile.hpp"

namespace csgs {

constexpr int WAVE = 64;

#define CSGS_LAUNCH_CHECK()                                   \
    do {                                                      \
        if (hipGetLastError() != hipSuccess) return CSGS_ELAUNCH; \
    } while (0)

__host__ __device__ inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---------------------------------------------------------------- workspace
// "clean" sections are all-zero between calls and come first.  The per-edge sections come
// last; how many edges they can hold follows from the size the caller passed.
constexpr int CAND_TILE = 1024;   // node ids per block in the candidate scan
constexpr int EDGE_TILE = 1024;   // edges per chunk in the flat edge passes
constexpr int EDGE_GRID = 2048;   // blocks of a flat edge pass (grid-stride over chunks)

struct Workspace {
    uint64_t *wtable;    // [n_nodes]  clean: per-node fixed-point weight accumulator
    uint8_t *tileflag;   // [ceil(n_nodes/64)] clean: 1 = some node of this 64-id word was touched
    int32_t *rank;       // [n_nodes]  clean: position in S_next + 1
    uint32_t *hit;       // [n_nodes]  clean: draws per candidate position
    uint64_t *cbitmap;   // [ceil(n_nodes/64)] clean: bit set = candidate position was drawn
    uint64_t *partial;   // [4 * n_tiles] per-tile partial sums of the candidate scan
    int64_t *eoff;       // [nS + 1] exclusive prefix of the degrees of the rows of S
    int64_t *rowstart;   // [nS]     rowptr[S[a]]
    int32_t *hitpos;     // [B]      candidate position of the k-th distinct hit
    double *pdbl;        // [B]      inclusion probabilities in double
    int64_t *chunkbase;  // [edge_chunks + 1] kept edges per chunk, then their exclusive prefix
    uint64_t *keepmask;  // [edge_cap / 64] bit = edge survives into the sampled adjacency
    int64_t edge_cap;    // edges the per-edge sections can hold (multiple of EDGE_TILE)
    size_t fixed_bytes;  // everything except the per-edge sections
    size_t bytes;
};

// Layout for a workspace of `ws_bytes` bytes; pass ws_bytes = 0 together with edges_max to size one.
__host__ inline Workspace carve(void *base, int64_t n_nodes, int64_t nS, int64_t B, size_t ws_bytes, int64_t edges_max)
{
    Workspace w;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return (char *)base + o;
    };
    const size_t words = (size_t)(n_nodes + 63) / 64;
    const size_t tiles = (size_t)(n_nodes + CAND_TILE - 1) / CAND_TILE;
    w.wtable = (uint64_t *)take((size_t)n_nodes * 8);
    w.tileflag = (uint8_t *)take(words);
    w.rank = (int32_t *)take((size_t)n_nodes * 4);
    w.hit = (uint32_t *)take((size_t)n_nodes * 4);
    w.cbitmap = (uint64_t *)take(words * 8);
    w.partial = (uint64_t *)take(tiles * 4 * 8);
    w.eoff = (int64_t *)take((size_t)(nS + 1) * 8);
    w.rowstart = (int64_t *)take((size_t)nS * 8);
    w.hitpos = (int32_t *)take((size_t)B * 4);
    w.pdbl = (double *)take((size_t)B * 8);
    w.fixed_bytes = off;
    // per-edge part: 8 bytes per chunk (+1 entry) and 1 bit per edge
    auto per_edge_bytes = [](int64_t chunks) {
        return align_up((size_t)(chunks + 1) * 8, 256) + align_up((size_t)chunks * (EDGE_TILE / 8), 256);
    };
    int64_t chunks;
    if (ws_bytes == 0) {
        chunks = (edges_max + EDGE_TILE - 1) / EDGE_TILE;
        if (chunks < 1) chunks = 1;
    } else {
        // largest chunk count that fits (per_edge_bytes is monotone; 136 bytes per chunk plus padding)
        const size_t room = ws_bytes > off ? ws_bytes - off : 0;
        chunks = (int64_t)(room / (8 + EDGE_TILE / 8));
        while (chunks > 0 && per_edge_bytes(chunks) > room) --chunks;
    }
    w.chunkbase = (int64_t *)take((size_t)(chunks + 1) * 8);
    w.keepmask = (uint64_t *)take((size_t)chunks * (EDGE_TILE / 8));
    w.edge_cap = chunks * EDGE_TILE;
    w.bytes = off;
    return w;
}

// ---------------------------------------------------------------- wave helpers
__device__ inline int lane_id() { return (int)(threadIdx.x & (WAVE - 1)); }

template <typename T>
__device__ inline T wave_sum(T v)
{
#pragma unroll
    for (int off = WAVE / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, WAVE);
    return v;
}

template <typename T>
__device__ inline T wave_inclusive_scan(T v)
{
    const int lane = lane_id();
#pragma unroll
    for (int off = 1; off < WAVE; off <<= 1) {
        T t = __shfl_up(v, off, WAVE);
        if (lane >= off) v += t;
    }
    return v;
}

// Exclusive scan over the threads of a block (blockDim.x a multiple of 64, at most 1024).
// Returns the exclusive prefix; *block_total receives the sum over the block.
template <typename T>
__device__ inline T block_exclusive_scan(T v, T *lds /*[17]*/, T *block_total)
{
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int nwaves = (int)(blockDim.x >> 6);
    T incl = wave_inclusive_scan(v);
    __syncthreads();  // lds may still be read from a previous use
    if (lane == WAVE - 1) lds[wave] = incl;
    __syncthreads();
    if (wave == 0) {
        T t = lane < nwaves ? lds[lane] : T(0);
        T s = wave_inclusive_scan(t);
        if (lane < nwaves) lds[lane] = s - t;
        if (lane == nwaves - 1) lds[16] = s;
    }
    __syncthreads();
    *block_total = lds[16];
    return incl - v + lds[wave];
}

// first index in [0, n) with a[idx] >= key (n if none)
__device__ inline int64_t lower_bound_i64(const int64_t *a, int64_t n, int64_t key)
{
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t m = (lo + hi) >> 1;
        if (a[m] >= key) hi = m; else lo = m + 1;
    }
    return lo;
}

// ---------------------------------------------------------------- flat edge chunks
// The edges of the rows of S, concatenated in row order, form one sequence of E edges; position
// e belongs to the row a with eoff[a] <= e < eoff[a+1] and sits at rowstart[a] + (e - eoff[a])
// in the CSR arrays.  A block works on chunks of EDGE_TILE consecutive positions, so the work
// per block does not depend on the degree distribution.  The rows that overlap a chunk are
// staged in LDS once per chunk.
constexpr int SLICE_MAX = EDGE_TILE + 2;

struct RowSlice {
    int32_t off[SLICE_MAX];     // eoff[a_first + r] - c0 (first entry may be negative)
    int64_t start[SLICE_MAX];   // rowstart[a_first + r]
    int32_t a_first;            // first staged row
    int32_t R;                  // staged rows; rows [a_first, a_first + R) overlap or start in the chunk
    bool in_lds;                // false: too many (empty) rows for LDS, read eoff / rowstart directly
};

// Called by all threads of the block.  c0 < c1 <= eoff[nS].
__device__ inline void stage_slice(RowSlice &s, const int64_t *__restrict__ eoff, const int64_t *__restrict__ rowstart,
                                   int32_t nS, int64_t c0, int64_t c1)
{
    __syncthreads();  // previous chunk's readers are done
    const int64_t lb0 = lower_bound_i64(eoff, (int64_t)nS + 1, c0);
    const int64_t a_first = (eoff[lb0] == c0) ? lb0 : lb0 - 1;
    const int64_t lb1 = lower_bound_i64(eoff, (int64_t)nS + 1, c1);
    const int64_t R = lb1 - a_first;
    if (threadIdx.x == 0) {
        s.a_first = (int32_t)a_first;
        s.R = (int32_t)R;
        s.in_lds = R <= SLICE_MAX;
    }
    if (R <= SLICE_MAX) {
        for (int64_t r = threadIdx.x; r < R; r += blockDim.x) {
            s.off[r] = (int32_t)(eoff[a_first + r] - c0);
            s.start[r] = (a_first + r < nS) ? rowstart[a_first + r] : 0;
        }
    }
    __syncthreads();
}

// CSR position of chunk-relative edge x (0 <= x < c1 - c0); *r_out = staged row index.
__device__ inline int64_t edge_address(const RowSlice &s, const int64_t *__restrict__ eoff,
                                       const int64_t *__restrict__ rowstart, int64_t c0, int32_t x, int32_t *r_out)
{
    int32_t lo = 0, hi = s.R;  // last r with off[r] <= x; off[0] <= 0 <= x always
    if (s.in_lds) {
        while (hi - lo > 1) {
            const int32_t m = (lo + hi) >> 1;
            if (s.off[m] <= x) lo = m; else hi = m;
        }
        *r_out = lo;
        return s.start[lo] + (x - s.off[lo]);
    }
    const int64_t a0 = s.a_first;
    while (hi - lo > 1) {
        const int32_t m = (lo + hi) >> 1;
        if (eoff[a0 + m] - c0 <= (int64_t)x) lo = m; else hi = m;
    }
    *r_out = lo;
    return rowstart[a0 + lo] + ((int64_t)x - (eoff[a0 + lo] - c0));
}

}  // namespace csgs
