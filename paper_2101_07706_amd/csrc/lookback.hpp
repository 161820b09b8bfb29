// Single-pass prefix sums across the blocks of one kernel.
//
// A kernel that must place its output at positions given by a running sum over all earlier tiles
// (stream compaction, CDF) normally needs three launches: per-tile sums, a scan of the sums, and
// the pass that uses them.  Here every block publishes its tile's sum and then adds up what the
// earlier tiles published, in three short hops so that no block waits on a chain of other blocks
// and no flag is polled by more than 64 readers (polls are served by the memory-side cache, and a
// flag polled by every block was measured to serialise there):
//   1. tiles form groups of 64; a tile reads the (at most 63) sums of the earlier tiles of its group;
//   2. the last tile of a group publishes the group's total;
//   3. the first tile of a group adds the totals of all earlier groups and publishes that prefix
//      for its group; the other tiles of the group read just this one value.
//
// Every wait ends.  A tile publishes its own sum (lookback_publish) before it waits for anything
// (lookback_resolve), and nothing a block does between the two halves waits for another block; a group total
// depends only on sums of lower tiles, the prefix only on group totals and sums of lower tiles.
// So a block makes progress as long as the blocks that own lower tiles run, which holds in both
// ways these kernels are launched:
//   - one tile per block, grid = number of tiles: the hardware walks a 1-D grid in ascending
//     block id, so the owners of all lower tiles were dispatched earlier and run or have finished;
//   - a grid of at most resident_grid() blocks, all resident at once, block b taking tiles b,
//     b + grid, ... in ascending order (used when the tile count is known only on the device).
// Each poll loop is also bounded (LOOKBACK_SPIN_LIMIT polls, or what csgs_workspace_wait_limit set);
// on a timeout (which would need another workload to keep lower blocks off the device for seconds)
// the block sets CSGS_ST_INTERNAL and carries on with a zero prefix; every store is
// capacity-checked and every edge address derived from a prefix is checked against the graph.
//
// Memory ordering.  Tile sums and flags are exchanged only through device-scope relaxed atomic
// loads and stores, which the hardware serves at the memory-side cache shared by all XCDs, so they
// are coherent without fences.  The writer waits until its value stores have been acknowledged
// before it stores the flag; a reader loads values only after its flag load has returned the tag.
// Full release / acquire fences are deliberately not used here: at device scope they write back
// and invalidate the whole L2 of the XCD on every use, which was measured to cost tens of
// microseconds per tile.  Everything else a tile writes is consumed by later kernels only.
//
// The flags live in the caller's workspace and are never cleared: a flag counts only if it carries
// the tag of the current call.  Tags come from a call counter that lives in the workspace itself
// (device memory): a kernel reads it when it starts, and the last kernel of every library call
// advances it at its very end, when all blocks that use the tag have read it.  Nothing about a
// tag is fixed at launch time, so a captured sequence of calls can be replayed.
#pragma once
#include "common.hpp"

namespace csgs {

constexpr int LOOKBACK_SPIN_LIMIT = 1 << 22;

// words of Workspace::epoch
constexpr int EPOCH_CALLS = 0;   // library calls completed on this workspace
constexpr int EPOCH_DRAW = 1;    // value of (calls + 1) during the latest draw: tags the rank table
constexpr int EPOCH_WAIT = 2;    // 0, or 1 + the number of polls a wait may take (set through csgs_workspace_wait_limit)
// one tag space per scan-state region, so the kernels of one call never mistake each other's flags
enum TagSlot { SLOT_ROWS = 1, SLOT_CAND = 2, SLOT_HITS = 3, SLOT_ADJ = 4, SLOT_ROWS_NEXT = 5, SLOT_STAGE = 6 };

__device__ inline int wait_limit(const uint64_t *epoch)
{
    const uint64_t v = epoch[EPOCH_WAIT];
    return v ? (int)(v - 1ull) : LOOKBACK_SPIN_LIMIT;
}
__device__ inline unsigned long long call_number(const uint64_t *epoch) { return epoch[EPOCH_CALLS] + 1ull; }
__device__ inline unsigned long long call_tag(unsigned long long call, int slot) { return call * 16ull + (unsigned long long)slot; }

__device__ inline unsigned long long ld_relaxed(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void st_relaxed(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline uint32_t ld_relaxed32(const uint32_t *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ inline void st_relaxed32(uint32_t *p, uint32_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
// Blocks until every earlier load and store of this wavefront has been acknowledged.
__device__ inline void wait_memory_ops() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Stores the flag after the value stores issued before it have reached the coherent level.
__device__ inline void st_flag(unsigned long long *p, unsigned long long v)
{
    wait_memory_ops();
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

constexpr int LB_GROUP = 64;

// flag[t] / agg[t * NV + v]: sums of tile t;  gflag[g] / gagg[g * NV + v]: sums of group g;
// pflag[g] / gpre[g * NV + v]: sums of all groups before g.
template <int NV>
struct TileState {
    unsigned long long *flag, *agg, *gflag, *gagg, *pflag, *gpre;
    int limit;   // polls a wait may take
    __device__ TileState(uint64_t *mem, int64_t tiles, int poll_limit) : limit(poll_limit)
    {
        const int64_t groups = tiles / LB_GROUP + 2;
        flag = (unsigned long long *)mem;
        agg = flag + tiles;
        gflag = agg + (int64_t)NV * tiles;
        gagg = gflag + groups;
        pflag = gagg + (int64_t)NV * groups;
        gpre = pflag + groups;
    }
};

// Waits (bounded, with growing pauses) until *p carries `tag`; returns false on a timeout.
__device__ inline bool wait_tag(const unsigned long long *p, unsigned long long tag, int limit)
{
    unsigned long long f = ld_relaxed(p);
    int spins = 0;
    while (f != tag && spins < limit) {
        if (spins < 4) __builtin_amdgcn_s_sleep(2); else __builtin_amdgcn_s_sleep(16);
        f = ld_relaxed(p);
        ++spins;
    }
    wait_memory_ops();  // the flag has arrived before any value load is issued
    return f == tag;
}

// First half: publishes `local` (the block-uniform sums of tile t).  Called by all threads; what a
// block does between the two halves (issuing loads that do not depend on the prefix, arithmetic in
// wavefronts other than the first) overlaps with the hops of the second half.
template <int NV>
__device__ inline void lookback_publish(const TileState<NV> &ts, unsigned long long tag, long long t,
                                        const unsigned long long (&local)[NV])
{
    if (threadIdx.x == 0) {
#pragma unroll
        for (int v = 0; v < NV; ++v) st_relaxed(&ts.agg[t * NV + v], local[v]);
        st_flag(&ts.flag[t], tag);
    }
}

// Second half: returns in `excl` the sums over tiles 0..t-1 (block-uniform).  Called by all threads
// after lookback_publish of the same tile; the first wavefront does the hops, the block meets at
// a barrier at the end.  `lds` holds NV words; between two calls that use the same `lds` the block
// must pass a barrier of its own.
template <int NV>
__device__ inline void lookback_resolve(const TileState<NV> &ts, unsigned long long tag, long long t, long long n_tiles,
                                        const unsigned long long (&local)[NV], unsigned long long (&excl)[NV],
                                        unsigned long long *lds, int32_t *status)
{
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    if (wave == 0) {
        const long long g = t / LB_GROUP;
        const int r = (int)(t % LB_GROUP);
        bool ok = true;
        unsigned long long run[NV];
        // hop 1: earlier tiles of my group
        {
            const bool mine = lane < r;
            const long long j = g * LB_GROUP + lane;
            if (mine) ok = wait_tag(&ts.flag[j], tag, ts.limit);
#pragma unroll
            for (int v = 0; v < NV; ++v) run[v] = wave_sum((mine && ok) ? ld_relaxed(&ts.agg[j * NV + v]) : 0ull);
        }
        // hop 2: the last tile of a group publishes the group's total
        if ((r == LB_GROUP - 1 || t == n_tiles - 1) && lane == 0) {
#pragma unroll
            for (int v = 0; v < NV; ++v) st_relaxed(&ts.gagg[g * NV + v], run[v] + local[v]);
            st_flag(&ts.gflag[g], tag);
        }
        // hop 3: the first tile of a group sums the totals of the earlier groups for everyone in it.
        // Nothing lies before the first group: its tiles neither wait nor publish here, so scans of
        // at most 64 tiles are done after one hop.
        unsigned long long pre[NV];
        if (g == 0) {
#pragma unroll
            for (int v = 0; v < NV; ++v) pre[v] = 0ull;
        } else if (r == 0) {
#pragma unroll
            for (int v = 0; v < NV; ++v) pre[v] = 0ull;
            for (long long g0 = 0; g0 < g; g0 += WAVE) {
                const long long gj = g0 + lane;
                const bool mine = gj < g;
                bool okg = true;
                if (mine) okg = wait_tag(&ts.gflag[gj], tag, ts.limit);
                ok = ok && okg;
#pragma unroll
                for (int v = 0; v < NV; ++v) pre[v] += wave_sum((mine && okg) ? ld_relaxed(&ts.gagg[gj * NV + v]) : 0ull);
            }
            if (lane == 0) {
#pragma unroll
                for (int v = 0; v < NV; ++v) st_relaxed(&ts.gpre[g * NV + v], pre[v]);
                st_flag(&ts.pflag[g], tag);
            }
        } else {
            bool okp = true;
            if (lane == 0) okp = wait_tag(&ts.pflag[g], tag, ts.limit);
            ok = ok && okp;
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const unsigned long long x = (lane == 0 && okp) ? ld_relaxed(&ts.gpre[g * NV + v]) : 0ull;
                pre[v] = __shfl(x, 0, WAVE);
            }
        }
        if (__ballot(!ok)) {
            if (lane == 0) atomicOr(status, CSGS_ST_INTERNAL);
#pragma unroll
            for (int v = 0; v < NV; ++v) { run[v] = 0ull; pre[v] = 0ull; }
        }
        if (lane == 0) {
#pragma unroll
            for (int v = 0; v < NV; ++v) lds[v] = run[v] + pre[v];
        }
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < NV; ++v) excl[v] = lds[v];
}

}  // namespace csgs
