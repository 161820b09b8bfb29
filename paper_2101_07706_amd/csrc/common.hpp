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
// Sections whose offsets depend on n_nodes only come first; the tail depends on nS and B.
// "clean" sections are all-zero between calls.
struct Workspace {
    uint64_t *wtable;   // [n_nodes]  clean: per-node fixed-point weight accumulator
    uint64_t *nbitmap;  // [ceil(n_nodes/64)] clean: bit set = node is a candidate
    int32_t *rank;      // [n_nodes]  clean: position in S_next + 1
    uint32_t *hit;      // [n_nodes]  clean: draws per candidate position
    uint64_t *cbitmap;  // [ceil(n_nodes/64)] clean: bit set = candidate position was drawn
    uint64_t *partial;  // [4 * n_tiles] per-tile partial sums of the candidate scan
    int32_t *rowcnt;    // [nS + 1]
    double *pdbl;       // [B] inclusion probabilities in double
    size_t bytes;
};

constexpr int CAND_TILE = 1024;  // node ids per block in the candidate scan

__host__ inline Workspace carve(void *base, int64_t n_nodes, int64_t nS, int64_t B)
{
    Workspace w;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return (char *)base + o;
    };
    size_t words = (size_t)(n_nodes + 63) / 64;
    size_t tiles = (size_t)(n_nodes + CAND_TILE - 1) / CAND_TILE;
    w.wtable = (uint64_t *)take((size_t)n_nodes * 8);
    w.nbitmap = (uint64_t *)take(words * 8);
    w.rank = (int32_t *)take((size_t)n_nodes * 4);
    w.hit = (uint32_t *)take((size_t)n_nodes * 4);
    w.cbitmap = (uint64_t *)take(words * 8);
    w.partial = (uint64_t *)take(tiles * 4 * 8);
    w.rowcnt = (int32_t *)take((size_t)(nS + 1) * 4);
    w.pdbl = (double *)take((size_t)B * 8);
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

}  // namespace csgs
