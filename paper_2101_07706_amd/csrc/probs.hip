// csgs_build_probs: importance weights over the neighbors of S_l (Section 4.1) and the skewed
// linear weighted sampling distribution (Section 4.2, Eq. 10) as an integer CDF.
//
// Kernels:
//   row_prefix     per tile of 1024 rows of S: degrees, their exclusive prefix (the flat edge
//                  numbering; tile offsets by the single-pass scan across blocks), CSR start of
//                  every row; the last tile leaves the row count and the edge counts for
//                  the kernels that follow
//   scan_edges     flat over the edges of S (chunks of 1024, rows of a chunk staged in LDS, so
//                  hub rows and short rows cost the same per edge): square each edge value
//                  exactly, round to the fixed-point grid, add into a per-node 64-bit accumulator
//                  -- remote targets with fire-and-forget integer atomics, targets in the local id
//                  range (in launches large enough to be bound by the atomic rate) through owner
//                  blocks that sum in LDS (see the kernel); flag the group of 8 node ids of the
//                  target (one 64-byte piece of the accumulator table) with a plain byte store, so
//                  that the candidate kernels fetch only touched pieces
//   cand_partials  per tile of 1024 node ids: candidate count, local count, local and remote
//                  weight sums of the flagged words (unskewed, so they do not depend on s); the
//                  last tile of each group of 64 adds up its group (it waits for the other
//                  tiles' flags)
//   cand_emit      per tile: prefix = group sums before my group + tile sums before me in my
//                  group (plain loads: the producers are earlier kernels); the skew multiplier is
//                  fixed by the caller, or taken from the grand totals by the rule of Theorem 1
//                  (Eq. 12), or zero for remote nodes ("Local" version of Section 5.1); the
//                  tile's candidates are packed into LDS in id order (ballot popcount), then the
//                  packed list gets its skewed weights, their inclusive running sum and q, and goes
//                  out as contiguous runs of cand_id / cand_w / cdf / q; restores accumulator and
//                  flags to zero; the last tile writes the stats
#include <math.h>
#include "common.hpp"
#include "lookback.hpp"
#include "row_prefix.hpp"

namespace csgs {

// Rows given by the caller: one tile per block, grid = tiles of the row capacity; with a device-side
// count the blocks past it leave at once.
__global__ __launch_bounds__(256) void row_prefix(const int64_t *__restrict__ rowptr, int64_t n_nodes,
                                                  const int32_t *__restrict__ S, int32_t nS_bound,
                                                  const int32_t *__restrict__ nS_dev, const uint64_t *__restrict__ epoch,
                                                  uint64_t *__restrict__ ts_mem, int64_t ts_tiles,
                                                  int64_t *__restrict__ eoff, int64_t *__restrict__ rowstart,
                                                  int64_t *__restrict__ meta, int64_t edge_cap,
                                                  int2 *__restrict__ bound_note, int32_t *__restrict__ status, InstStride is)
{
    bound_note = inst_ptr(bound_note, is.ws);
    S = inst_ptr(S, is.buf); nS_dev = inst_ptr(nS_dev, is.buf); status = inst_ptr(status, is.buf);
    epoch = inst_ptr(epoch, is.ws); ts_mem = inst_ptr(ts_mem, is.ws); eoff = inst_ptr(eoff, is.ws);
    rowstart = inst_ptr(rowstart, is.ws); meta = inst_ptr(meta, is.ws);
    const TileState<1> ts(ts_mem, ts_tiles, wait_limit(epoch));
    const int32_t nS = resolve_count(nS_bound, nS_dev);
    const int64_t n_tiles = row_tiles(nS);
    if ((int64_t)blockIdx.x >= n_tiles) return;
    row_prefix_tile(rowptr, n_nodes, S, nS, blockIdx.x, n_tiles, ts, call_tag(call_number(epoch), SLOT_ROWS), eoff, rowstart,
                    meta, edge_cap, bound_note, edge_cap / EDGE_TILE, status);
}

// Arguments of the hand-over inside the weight scan (see scan_edges).
struct Stage {
    uint64_t *w;
    uint32_t *c, *off;
    unsigned long long *done;
    int64_t chunks;     // chunks the hand-over arrays can hold
    int32_t lo, hi;     // local id range
    int32_t owners;     // owner blocks at the end of the grid (0: every edge goes through device-scope atomics)
    int32_t mode;       // 0: hand over when the launch has enough chunks to be bound by the atomic rate; 1: never; 2: always
};
// chunks (over all instances of the launch) from which the hand-over pays: below, the launch is
// bound by latency and the owners' last round only adds to it
constexpr int64_t STAGE_MIN_CHUNKS = 1024;

// The weight scan.  Two kinds of blocks in one grid:
//  * chunk blocks (the first gridDim.x - owners, grid-stride over chunks of EDGE_TILE edges): stage the
//    rows of the chunk, fetch column and value of every edge, square and round.  An edge whose
//    target lies outside the local id range is added to the per-node accumulator with a
//    device-scope atomic.  The others -- most edges: the partition holds most neighbors -- are
//    counting-sorted by owner inside the block and written to the chunk's piece of the hand-over
//    arrays, then the chunk's flag is raised.  Scattered device-scope atomics run at about 23 G/s on
//    this part whatever their scope or target range; LDS atomics are two orders faster.
//  * owner blocks (the last `owners` of the grid): block r owns local ids [lo + r SUB_IDS, + SUB_IDS),
//    sums in LDS what the chunks hand it (64 chunks at a time per wavefront, one per lane, as their
//    flags come up), and stores the non-zero sums and their touch flags with plain stores: nobody
//    else writes those entries.
// Owners wait only for chunk blocks, which have lower block ids and wait for nobody.  Integer sums:
// the result does not depend on which way an edge went or in what order.  The hand-over is used
// when the call's edges fit its arrays and are many enough (see STAGE_MIN_CHUNKS); all blocks take
// that decision from the same words.
__global__ __launch_bounds__(256) void scan_edges(const int32_t *__restrict__ colidx, const float *__restrict__ val,
                                                  int64_t n_nodes, int64_t nnz, int32_t shift_base,
                                                  const int64_t *__restrict__ meta, int64_t edge_cap,
                                                  const int64_t *__restrict__ eoff,
                                                  const int64_t *__restrict__ rowstart,
                                                  uint64_t *__restrict__ wtable, uint8_t *__restrict__ tileflag,
                                                  int2 *__restrict__ chunk_note, const int2 *__restrict__ bound_note,
                                                  int32_t *__restrict__ status,
                                                  const uint64_t *__restrict__ epoch, Stage stg, InstStride is)
{
    __shared__ RowSlice slice;
    __shared__ unsigned long long acc[SUB_IDS];
    __shared__ uint32_t hist[SUB_MAX + 1];
    meta = inst_ptr(meta, is.ws); eoff = inst_ptr(eoff, is.ws); rowstart = inst_ptr(rowstart, is.ws);
    wtable = inst_ptr(wtable, is.ws); tileflag = inst_ptr(tileflag, is.ws); chunk_note = inst_ptr(chunk_note, is.ws); bound_note = inst_ptr(bound_note, is.ws);
    epoch = inst_ptr(epoch, is.ws);
    stg.w = inst_ptr(stg.w, is.ws); stg.c = inst_ptr(stg.c, is.ws); stg.off = inst_ptr(stg.off, is.ws);
    stg.done = inst_ptr(stg.done, is.ws);
    status = inst_ptr(status, is.buf);
    const int32_t nS = (int32_t)meta[META_ROWS];
    const double scale = ldexp(1.0, shift_for_rows(shift_base, nS));
    const int64_t E = meta[META_EDGES];
    const int64_t n_chunks = (E + EDGE_TILE - 1) / EDGE_TILE;
    const bool staged = stg.owners > 0 && n_chunks <= stg.chunks && stg.mode != 1 &&
                        (stg.mode == 2 || n_chunks * (int64_t)gridDim.z >= STAGE_MIN_CHUNKS);
    const unsigned long long tag = call_tag(call_number(epoch), SLOT_STAGE);
    const int32_t chunk_blocks = (int32_t)gridDim.x - stg.owners;
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);

    if ((int32_t)blockIdx.x >= chunk_blocks) {   // ---------------- owner
        if (!staged) return;
        const int32_t r = (int32_t)blockIdx.x - chunk_blocks;
        const int32_t base_id = stg.lo + r * SUB_IDS;
        const int limit = wait_limit(epoch);
        for (int i = threadIdx.x; i < SUB_IDS; i += blockDim.x) acc[i] = 0ull;
        __syncthreads();
        bool timed_out = false;
        for (int64_t cb = (int64_t)wave * WAVE; cb < n_chunks; cb += (int64_t)(blockDim.x >> 6) * WAVE) {
            // one chunk per lane: where my group lies in its piece
            const int64_t c = cb + lane;
            int32_t beg = 0, end = 0;
            if (c < n_chunks) {
                if (wait_tag(&stg.done[c], tag, limit)) {
                    const uint32_t pr = ld_relaxed32(&stg.off[c * SUB_MAX + r]);
                    beg = (int32_t)(pr & 0xFFFFu);
                    end = (int32_t)(pr >> 16);
                    if (end > EDGE_TILE || beg > end) beg = end = 0;   // (only after a failed wait elsewhere)
                } else {
                    timed_out = true;
                }
            }
            // the 64 groups as one sequence, one entry per lane and step: entry j belongs to the first
            // lane whose running count exceeds j
            const int32_t n = end - beg;
            const int32_t incl = wave_inclusive_scan<int32_t>(n);
            const int32_t excl = incl - n;
            const int32_t total = __builtin_amdgcn_readlane(incl, WAVE - 1);
            for (int32_t j0 = 0; j0 < total; j0 += 4 * WAVE) {
                unsigned long long wv[4];
                uint32_t cv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int32_t j = j0 + u * WAVE + lane;
                    int lo_l = 0, hi_l = WAVE - 1;
#pragma unroll
                    for (int it = 0; it < 6; ++it) {
                        const int mid = (lo_l + hi_l) >> 1;
                        if (__shfl(incl, mid, WAVE) > j) hi_l = mid; else lo_l = mid + 1;
                    }
                    const int src = lo_l < WAVE ? lo_l : WAVE - 1;
                    const int64_t pos = (cb + src) * EDGE_TILE + __shfl(beg, src, WAVE) + (j - __shfl(excl, src, WAVE));
                    // unconditional (entry 0 stands in past the end and is dropped below), so that the four
                    // steps' loads are on their way together
                    const int64_t at = j < total ? pos : 0;
                    wv[u] = ld_relaxed((const unsigned long long *)&stg.w[at]);
                    cv[u] = ld_relaxed32(&stg.c[at]);
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t x = (int64_t)cv[u] - base_id;
                    if (j0 + u * WAVE + lane < total && x >= 0 && x < SUB_IDS) atomicAdd(&acc[x], wv[u]);
                }
            }
        }
        if (timed_out) atomicOr(status, CSGS_ST_INTERNAL);
        __syncthreads();
        for (int i = threadIdx.x; i < SUB_IDS; i += blockDim.x) {
            const unsigned long long v = acc[i];
            const int64_t id = (int64_t)base_id + i;
            if (v && id < stg.hi && id < n_nodes) {
                wtable[id] = v;
                tileflag[id >> 3] = 1;
            }
        }
        return;
    }

    // ---------------- chunk blocks
    if (blockIdx.x == 0 && threadIdx.x == 0 && meta[META_EDGES_TRUE] > edge_cap) atomicOr(status, CSGS_ST_EDGE_OVERFLOW);
    bool bad = false;
    for (int64_t t = blockIdx.x; t < n_chunks; t += chunk_blocks) {
        const int64_t c0 = t * EDGE_TILE;
        const int64_t c1 = (c0 + EDGE_TILE < E) ? c0 + EDGE_TILE : E;
        stage_slice_bounds(slice, eoff, rowstart, nS, t, c0, c1, bound_note, chunk_note + t);   // (starts with a barrier)
        if (staged) {
            for (int i = threadIdx.x; i <= SUB_MAX; i += blockDim.x) hist[i] = 0u;
            __syncthreads();
        }
        const int32_t len = (int32_t)(c1 - c0);
        unsigned long long hq[EDGE_TILE / 256];
        int32_t hc[EDGE_TILE / 256], hb[EDGE_TILE / 256];
        uint32_t hr[EDGE_TILE / 256];
        // All of a thread's edges go through each step together -- their addresses, then their columns and
        // values with unconditional loads (an edge that does not exist reads entry 0 and is dropped) -- so
        // the loads of the four edges travel at the same time instead of one after the other.
        int64_t ek[EDGE_TILE / 256];
        bool live[EDGE_TILE / 256];
#pragma unroll
        for (int k = 0; k < EDGE_TILE / 256; ++k) {
            const int32_t x = (int32_t)threadIdx.x + k * 256;
            ek[k] = 0;
            live[k] = x < len;
            if (live[k]) {
                int32_t r;
                ek[k] = edge_address(slice, eoff, rowstart, c0, x, &r);
                if (ek[k] < 0 || ek[k] >= nnz) {   // only after a failed wait in the prefix kernel: stay inside the graph
                    bad = true;
                    ek[k] = 0;
                    live[k] = false;
                }
            }
        }
        int32_t ck[EDGE_TILE / 256];
        float vk[EDGE_TILE / 256];
#pragma unroll
        for (int k = 0; k < EDGE_TILE / 256; ++k) {
            ck[k] = colidx[ek[k]];
            vk[k] = val[ek[k]];
        }
        // Everything that reads a loaded value comes before the first update: an update issued between two
        // such reads would have to be acknowledged before the second value counts as arrived.
        long long qk[EDGE_TILE / 256];
#pragma unroll
        for (int k = 0; k < EDGE_TILE / 256; ++k) {
            const bool sound = isfinite(vk[k]) && ck[k] >= 0 && ck[k] < n_nodes;
            if (live[k] && !sound) bad = true;
            live[k] = live[k] && sound;
            const double sq = (double)vk[k] * (double)vk[k];   // exact: 24 x 24 bit product
            qk[k] = live[k] ? __double2ll_rn(sq * scale) : 0;  // scale is a power of two: exact, then RNE
            if (qk[k] < 1) qk[k] = 1;                          // every candidate stays drawable
        }
#pragma unroll
        for (int k = 0; k < EDGE_TILE / 256; ++k) {
            hb[k] = -1;
            hq[k] = 0ull; hc[k] = 0; hr[k] = 0u;
            if (!live[k]) continue;
            const int32_t c = ck[k];
            if (staged && c >= stg.lo && c < stg.hi) {
                hb[k] = (c - stg.lo) / SUB_IDS;           // < owners <= SUB_MAX
                hq[k] = (unsigned long long)qk[k];
                hc[k] = c;
                hr[k] = atomicAdd(&hist[hb[k]], 1u);      // place inside the owner's group (any order)
            } else {
                hb[k] = -2;   // goes through a device-scope atomic, issued after the chunk's hand-over (below)
            }
        }
        if (staged) {
            __syncthreads();
            if (wave == 0) {   // counts -> begin of every owner's group; two owners per lane
                const uint32_t a = hist[2 * lane], b = (2 * lane + 1 <= SUB_MAX) ? hist[2 * lane + 1] : 0u;
                const uint32_t incl = wave_inclusive_scan<uint32_t>(a + b);
                const uint32_t ex = incl - (a + b);
                hist[2 * lane] = ex;
                hist[2 * lane + 1] = ex + a;
                if (lane == WAVE - 1) hist[SUB_MAX] = incl;   // edges handed over by this chunk
                // begin | end << 16 for the owners' lookups
                st_relaxed32(&stg.off[t * SUB_MAX + 2 * lane], ex | ((ex + a) << 16));
                st_relaxed32(&stg.off[t * SUB_MAX + 2 * lane + 1], (ex + a) | ((ex + a + b) << 16));
            }
            __syncthreads();
            // grouped by owner in LDS first (the owner blocks' sum array is free here), then out in
            // order: full 64-byte pieces instead of one scattered store per edge
            static_assert(SUB_IDS * 8 >= EDGE_TILE * 12, "the sort buffer lives in the owners' sum array");
            unsigned long long *s_w = acc;                                           // [EDGE_TILE]
            uint32_t *s_c = reinterpret_cast<uint32_t *>(acc + EDGE_TILE);           // [EDGE_TILE]
#pragma unroll
            for (int k = 0; k < EDGE_TILE / 256; ++k) {
                if (hb[k] < 0) continue;
                const uint32_t slot = hist[hb[k]] + hr[k];    // < EDGE_TILE: the groups partition the chunk's local edges
                s_w[slot] = hq[k];
                s_c[slot] = (uint32_t)hc[k];
            }
            __syncthreads();
            const uint32_t n_handed = hist[SUB_MAX];
            for (uint32_t i = threadIdx.x; i < n_handed; i += blockDim.x) {
                st_relaxed((unsigned long long *)&stg.w[t * EDGE_TILE + i], s_w[i]);
                st_relaxed32(&stg.c[t * EDGE_TILE + i], s_c[i]);
            }
            wait_memory_ops();     // this wavefront's hand-over stores have been acknowledged
            __syncthreads();
            if (threadIdx.x == 0) st_flag(&stg.done[t], tag);
        }
        // The edges that end outside the local range (all edges without the hand-over).  After the flag: the wait above
        // would otherwise include these updates, which take far longer to be acknowledged than the stores, and the
        // owners would start that much later.
#pragma unroll
        for (int k = 0; k < EDGE_TILE / 256; ++k) {
            if (hb[k] != -2) continue;
            const int32_t c = ck[k];
            (void)__hip_atomic_fetch_add((unsigned long long *)&wtable[c], (unsigned long long)qk[k], __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
            tileflag[c >> 3] = 1;  // same value from every writer
        }
    }
    if (bad) atomicOr(status, CSGS_ST_BAD_EDGE_VALUE);
}

// Skew policy, resolved on the device once the candidate counts are known.
struct SkewPolicy {
    int mode;          // 0: s_fx given; 1: Theorem 1 from (D, B), clamped to [16, s_fx_max]; 2: remote weight 0
    uint64_t s_fx;     // mode 0: local multiplier in 1/16 units
    double D;          // mode 1
    int64_t B;         // mode 1
    uint64_t s_fx_max; // mode 1
};

// Multipliers of local and remote weights (Eq. 10 numerators in 1/16 units).
__device__ inline void resolve_skew(const SkewPolicy &pol, uint64_t n_cand, uint64_t n_remote, uint64_t *m_local,
                                    uint64_t *m_remote)
{
    *m_remote = 16ull;
    if (pol.mode == 0) {
        *m_local = pol.s_fx;
    } else if (pol.mode == 1) {
        // s = D (|N(S_l)| - B) / |R| + 1/2 (Eq. 12), at least 1, no remote candidates -> 1
        double sk = 1.0;
        if (n_remote > 0) sk = pol.D * (double)((int64_t)n_cand - pol.B) / (double)n_remote + 0.5;
        if (!(sk >= 1.0)) sk = 1.0;
        double fx = floor(sk * 16.0 + 0.5);
        if (fx > (double)pol.s_fx_max) fx = (double)pol.s_fx_max;
        *m_local = (uint64_t)fx;
    } else {
        *m_local = 16ull;
        *m_remote = 0ull;
    }
}

constexpr int CAND_WORDS = CAND_TILE / WAVE;  // 16 words per tile, 4 per wave

// Tile sums, and -- by the last tile of every group of 64 -- the group's sums.  That tile waits
// for the flags of the (at most 63) lower tiles of its group, which were dispatched before it
// (ascending block ids) or belong to its own block and are published before the wait, and which
// wait for nobody, so the wait ends.  A block takes CAND_PART_TILES consecutive tiles and asks for
// the flags of all their words, then for all their pieces of the table: two load latencies per block.
constexpr int CAND_PART_TILES = 2;
__global__ __launch_bounds__(256) void cand_partials(const uint64_t *__restrict__ wtable,
                                                     const uint8_t *__restrict__ tileflag, int64_t n_words,
                                                     int64_t n_nodes, int64_t n_tiles, int32_t lo, int32_t hi,
                                                     const uint64_t *__restrict__ epoch, unsigned long long *__restrict__ cand_flag,
                                                     unsigned long long *__restrict__ partial,
                                                     uint64_t *__restrict__ gtot, int32_t *__restrict__ status, InstStride is)
{
    constexpr int TPB = CAND_PART_TILES, W = CAND_WORDS / 4;   // tiles per block, words per wavefront and tile
    __shared__ uint64_t lds[TPB][4][3];
    wtable = inst_ptr(wtable, is.ws); tileflag = inst_ptr(tileflag, is.ws); epoch = inst_ptr(epoch, is.ws);
    cand_flag = inst_ptr(cand_flag, is.ws); partial = inst_ptr(partial, is.ws); gtot = inst_ptr(gtot, is.ws);
    status = inst_ptr(status, is.buf);
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t t0 = (int64_t)blockIdx.x * TPB;
    const unsigned long long tag = call_tag(call_number(epoch), SLOT_CAND);
    uint64_t f8[TPB][W], w[TPB][W];
#pragma unroll
    for (int h = 0; h < TPB; ++h)
#pragma unroll
        for (int k = 0; k < W; ++k) {
            const int64_t word_idx = (t0 + h) * CAND_WORDS + wave * W + k;
            f8[h][k] = word_idx < n_words ? reinterpret_cast<const uint64_t *>(tileflag)[word_idx] : 0ull;   // the word's eight group flags
        }
#pragma unroll
    for (int h = 0; h < TPB; ++h)
#pragma unroll
        for (int k = 0; k < W; ++k) {
            const uint32_t id = ((uint32_t)(t0 + h) * CAND_WORDS + wave * W + k) * 64u + lane;   // below 2^31 + 1024
            // only the touched groups of 8 ids (one 64-byte piece of the table each) are fetched
            w[h][k] = (((f8[h][k] >> (8 * (lane >> 3))) & 0xFFull) && id < (uint32_t)n_nodes) ? wtable[id] : 0ull;
        }
    const uint32_t lo_u = lo > 0 ? (uint32_t)lo : 0u, hi_u = hi > 0 ? (uint32_t)hi : 0u;
#pragma unroll
    for (int h = 0; h < TPB; ++h) {
        // counts from the ballots (scalar work), weights as the sum over everything and over the local ids: two
        // wave-wide 64-bit sums per tile instead of three
        uint64_t cn = 0, wl = 0, wa = 0;   // cn packs (candidates << 32) | local candidates
#pragma unroll
        for (int k = 0; k < W; ++k) {
            const uint32_t id = ((uint32_t)(t0 + h) * CAND_WORDS + wave * W + k) * 64u + lane;
            const bool local = id >= lo_u && id < hi_u;
            cn += ((uint64_t)__popcll(__ballot(w[h][k] != 0)) << 32) | (uint64_t)__popcll(__ballot(w[h][k] != 0 && local));
            wa += w[h][k];
            wl += local ? w[h][k] : 0ull;
        }
        wl = wave_sum(wl); wa = wave_sum(wa);
        if (lane == 0) { lds[h][wave][0] = cn; lds[h][wave][1] = wl; lds[h][wave][2] = wa - wl; }
    }
    __syncthreads();
    if (wave != 0) return;
    // packed count halves cannot carry: each is at most 1024 per tile
    unsigned long long mine = 0ull;   // of the block's last tile
    int64_t t = t0;
#pragma unroll
    for (int h = 0; h < TPB; ++h) {
        if (t0 + h >= n_tiles) break;
        t = t0 + h;
        mine = lane < 3 ? lds[h][0][lane] + lds[h][1][lane] + lds[h][2][lane] + lds[h][3][lane] : 0ull;
        if (lane < 3) st_relaxed(&partial[t * 4 + lane], mine);
        if (lane == 0) st_flag(&cand_flag[t], tag);   // after the wavefront's value stores have been acknowledged
    }
    // the last tile of a group (and the last tile of all) is odd-numbered or the last: always a block's last tile
    static_assert(LB_GROUP % CAND_PART_TILES == 0, "a group's last tile must be a block's last tile");
    const int r = (int)(t % LB_GROUP);
    if (r != LB_GROUP - 1 && t != n_tiles - 1) return;
    const int64_t g = t / LB_GROUP;
    bool ok = true;
    if (lane < r) ok = wait_tag(&cand_flag[g * LB_GROUP + lane], tag, wait_limit(epoch));
    unsigned long long sum[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const unsigned long long own = __shfl(mine, i, WAVE);
        sum[i] = own + wave_sum((lane < r && ok) ? ld_relaxed(&partial[(g * LB_GROUP + lane) * 4 + i]) : 0ull);
    }
    if (__ballot(!ok) && lane == 0) atomicOr(status, CSGS_ST_INTERNAL);
    if (lane < 3) gtot[g * 4 + lane] = lane == 0 ? sum[0] : (lane == 1 ? sum[1] : sum[2]);
}

__global__ __launch_bounds__(256) void cand_emit(uint64_t *__restrict__ wtable, uint8_t *__restrict__ tileflag,
                                                 int64_t n_words, int64_t n_nodes, int64_t n_tiles, int32_t lo,
                                                 int32_t hi, SkewPolicy pol, const uint64_t *__restrict__ partial,
                                                 const uint64_t *__restrict__ gtot,
                                                 const int64_t *__restrict__ meta, int32_t shift_base,
                                                 uint64_t *__restrict__ epoch,
                                                 csgs_prob_stats *__restrict__ stats, int32_t *__restrict__ status,
                                                 int32_t *__restrict__ cand_id, uint64_t *__restrict__ cand_w,
                                                 uint64_t *__restrict__ cdf, float *__restrict__ q, int64_t cap, InstStride is)
{
    __shared__ uint32_t s_cnt[4];
    __shared__ uint32_t s_id[4][CAND_TILE / 4];    // the tile's candidates, packed: ids ...
    __shared__ uint64_t s_wt[4][CAND_TILE / 4];    // ... and fixed-point weights, per wavefront in id order
    wtable = inst_ptr(wtable, is.ws); tileflag = inst_ptr(tileflag, is.ws); partial = inst_ptr(partial, is.ws);
    gtot = inst_ptr(gtot, is.ws); meta = inst_ptr(meta, is.ws); epoch = inst_ptr(epoch, is.ws);
    stats = inst_ptr(stats, is.buf); status = inst_ptr(status, is.buf); cand_id = inst_ptr(cand_id, is.buf);
    cand_w = inst_ptr(cand_w, is.buf); cdf = inst_ptr(cdf, is.buf); q = inst_ptr(q, is.buf);
    __shared__ uint64_t s_w[4];
    __shared__ uint64_t s_red[4][6];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t t = blockIdx.x;
    const int64_t g = t / 64, n_groups = (n_tiles + 63) / 64;
    // Loads are issued in the order flags, prefix inputs, accumulators, and consumed only after
    // all are in flight, so the tile's own data travels while the prefix is being summed.
    uint64_t flagged[CAND_WORDS / 4];   // the eight group flags of each 64-id word (one byte per 8 ids)
#pragma unroll
    for (int k = 0; k < CAND_WORDS / 4; ++k) {
        const int64_t word_idx = t * CAND_WORDS + wave * (CAND_WORDS / 4) + k;
        flagged[k] = word_idx < n_words ? reinterpret_cast<const uint64_t *>(tileflag)[word_idx] : 0ull;
    }
    // sums over everything (tot) and over what lies before this tile (pre): group sums before my
    // group, then tile sums before me inside my group
    uint64_t gv[3] = {0, 0, 0}, pv[3] = {0, 0, 0};
    if ((int64_t)threadIdx.x < n_groups) {
#pragma unroll
        for (int i = 0; i < 3; ++i) gv[i] = gtot[(int64_t)threadIdx.x * 4 + i];
    }
    {
        const int64_t j = g * 64 + threadIdx.x;
        if (threadIdx.x < 64 && j < t) {
#pragma unroll
            for (int i = 0; i < 3; ++i) pv[i] = partial[j * 4 + i];
        }
    }
    uint64_t w[CAND_WORDS / 4];
#pragma unroll
    for (int k = 0; k < CAND_WORDS / 4; ++k) {
        // node ids are below 2^31 and a tile adds at most 1023: 32-bit arithmetic, half the instructions
        const uint32_t id = ((uint32_t)t * CAND_WORDS + wave * (CAND_WORDS / 4) + k) * 64u + lane;
        w[k] = (((flagged[k] >> (8 * (lane >> 3))) & 0xFFull) && id < (uint32_t)n_nodes) ? wtable[id] : 0ull;
    }
    uint64_t tot[3], pre[3];
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        tot[i] = gv[i];
        pre[i] = ((int64_t)threadIdx.x < g ? gv[i] : 0ull) + pv[i];
    }
    for (int64_t j = (int64_t)threadIdx.x + blockDim.x; j < n_groups; j += blockDim.x) {  // more than 256 groups
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            const uint64_t v = gtot[j * 4 + i];
            tot[i] += v;
            if (j < g) pre[i] += v;
        }
    }
    // group j's sums are held by thread j and the in-group tile sums by the first 64 threads: with fewer
    // than 64 groups only the first wavefront has anything to add up (the others hold zeros)
    if ((int64_t)wave * WAVE < n_groups) {
#pragma unroll
        for (int i = 0; i < 3; ++i) { tot[i] = wave_sum(tot[i]); pre[i] = wave_sum(pre[i]); }
    }
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < 3; ++i) { s_red[wave][i] = tot[i]; s_red[wave][3 + i] = pre[i]; }
    }
    __syncthreads();
    {   // lanes 0 .. 5 add up one of the six sums each; the others get them by lane broadcast (not every lane all 24 terms)
        const uint64_t mine = lane < 6 ? s_red[0][lane] + s_red[1][lane] + s_red[2][lane] + s_red[3][lane] : 0ull;
#pragma unroll
        for (int i = 0; i < 3; ++i) {
            tot[i] = __shfl(mine, i, WAVE);
            pre[i] = __shfl(mine, 3 + i, WAVE);
        }
    }
    const uint64_t n_cand = tot[0] >> 32, n_local = tot[0] & 0xFFFFFFFFull;
    uint64_t m_local, m_remote;
    resolve_skew(pol, n_cand, n_cand - n_local, &m_local, &m_remote);
    const uint64_t total_w = tot[1] * m_local + tot[2] * m_remote;
    const double total_d = (double)total_w;

    // The tile's candidates (about one id in fifteen in a sparse neighbourhood) are first packed into LDS, every
    // wavefront its own four words in id order, the accumulators and flags going back to their clean state on the way.
    // Everything that costs instructions per candidate -- the skewed weight, the 64-bit running sum, q, the five
    // stores -- is then done on the packed list, by as many wavefronts as it fills, with contiguous stores.
    uint32_t my_cnt = 0;
#pragma unroll
    for (int k = 0; k < CAND_WORDS / 4; ++k) {
        const int slot = wave * (CAND_WORDS / 4) + k;
        const uint32_t id = ((uint32_t)t * CAND_WORDS + slot) * 64u + lane;
        const uint64_t word = __ballot(w[k] != 0);
        if (w[k] != 0) {
            const uint32_t at = my_cnt + (uint32_t)__popcll(word & ((1ull << lane) - 1ull));
            s_id[wave][at] = id;
            s_wt[wave][at] = w[k];
            wtable[id] = 0ull;  // back to the clean state
        }
        my_cnt += (uint32_t)__popcll(word);
        if (flagged[k] && lane == 0) reinterpret_cast<uint64_t *>(tileflag)[t * CAND_WORDS + slot] = 0ull;  // back to the clean state
    }
    if (lane == 0) s_cnt[wave] = my_cnt;
    __syncthreads();
    const uint32_t c0 = s_cnt[0], c1 = c0 + s_cnt[1], c2 = c1 + s_cnt[2], n_t = c2 + s_cnt[3];
    const uint32_t lo_u = lo > 0 ? (uint32_t)lo : 0u, hi_u = hi > 0 ? (uint32_t)hi : 0u;
    const int64_t base_cnt = (int64_t)(pre[0] >> 32);
    uint64_t run_w = pre[1] * m_local + pre[2] * m_remote;   // skewed weight before the packed candidate at pass_base
    for (uint32_t pass_base = 0; pass_base < n_t; pass_base += 256u) {   // one pass unless the tile holds more than 256 candidates
        const uint32_t i = pass_base + threadIdx.x;
        const bool have = i < n_t;
        const bool wave_has = pass_base + (uint32_t)wave * WAVE < n_t;   // the same for the whole wavefront
        uint32_t id = 0;
        uint64_t wi = 0, wsk = 0, incl = 0;
        if (wave_has) {
            if (have) {
                const int src = i < c0 ? 0 : (i < c1 ? 1 : (i < c2 ? 2 : 3));
                const uint32_t at = i - (src == 0 ? 0u : (src == 1 ? c0 : (src == 2 ? c1 : c2)));
                id = s_id[src][at];
                wi = s_wt[src][at];
                wsk = wi * ((id >= lo_u && id < hi_u) ? m_local : m_remote);
            }
            incl = wave_inclusive_scan(wsk);
            if (lane == WAVE - 1) s_w[wave] = incl;
        } else if (lane == WAVE - 1) {
            s_w[wave] = 0ull;
        }
        __syncthreads();
        uint64_t before = run_w;
        for (int w2 = 0; w2 < wave; ++w2) before += s_w[w2];
        if (have) {
            const int64_t pos = base_cnt + i;
            if (pos < cap) {
                cand_id[pos] = (int32_t)id;
                cand_w[pos] = wi;
                cdf[pos] = before + incl;
                if (q) q[pos] = (float)((double)wsk / total_d);
            }
        }
        run_w += s_w[0] + s_w[1] + s_w[2] + s_w[3];
        __syncthreads();   // s_w is written again in the next pass
    }
    if (t == n_tiles - 1 && threadIdx.x == 0) {
        stats->n_cand = (int64_t)n_cand;
        stats->n_local = (int64_t)n_local;
        stats->n_remote = (int64_t)(n_cand - n_local);
        stats->w_local = tot[1];
        stats->w_remote = tot[2];
        stats->total = total_w;
        stats->shift = shift_for_rows(shift_base, meta[META_ROWS]);
        stats->edges_scanned = meta[META_EDGES_TRUE];
        stats->skew_fx = (int32_t)m_local * (m_remote ? 1 : -1);
        int32_t st = 0;
        if (n_cand == 0 || total_w == 0) st |= CSGS_ST_EMPTY_CANDIDATES;
        if ((int64_t)n_cand > cap) st |= CSGS_ST_CAND_OVERFLOW;
        if (st) atomicOr(status, st);
        epoch[EPOCH_CALLS] += 1ull;  // last kernel of the call; no block of this kernel reads the counter
    }
}

__global__ void fill_zero(uint64_t *p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0ull;
}

static int ceil_log2_u64(uint64_t n)
{
    int e = 0;
    while (e < 63 && (1ull << e) < n) ++e;
    return e;
}

// 61 - ceil(log2 s_fx) - ceil(log2 rmax): the fraction bits a single row could use
static int shift_base_for(int64_t s_fx, float rownorm2_max)
{
    int e_r = 0;
    while (e_r < 64 && ldexp(1.0, e_r) < (double)rownorm2_max) ++e_r;
    return 61 - ceil_log2_u64((uint64_t)s_fx) - e_r;
}

}  // namespace csgs

int csgs::launch_row_prefix(const int64_t *rowptr, int64_t n_nodes, const int32_t *S, int32_t nS, const int32_t *nS_dev,
                            const Workspace &w, const RowOffsets &rows, int32_t *status, hipStream_t st)
{
    const unsigned tiles = (unsigned)(((int64_t)nS + ROW_TILE - 1) / ROW_TILE);
    CSGS_LAUNCH(K_ROW_PREFIX, row_prefix, dim3(tiles, 1, (unsigned)w.n_inst), dim3(256), st, rowptr, n_nodes, S, nS, nS_dev,
                w.epoch, w.rp_ts, w.rp_tiles, rows.eoff, rows.rowstart, rows.meta, w.chunk_cap * EDGE_TILE, rows.bound_note, status,
                inst_stride(w));
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

using namespace csgs;

extern "C" size_t csgs_workspace_bytes(int64_t n_nodes, int32_t nS_max, int32_t B_max, int64_t edges_max)
{
    if (n_nodes <= 0 || n_nodes > 0x7FFFFFFFll || nS_max <= 0 || B_max <= 0 || edges_max <= 0) return 0;
    return carve(nullptr, n_nodes, nS_max, B_max, edges_max).bytes;
}

extern "C" size_t csgs_workspace_clean_bytes(int64_t n_nodes)
{
    if (n_nodes <= 0) return 0;
    return carve(nullptr, n_nodes, 1, 1, 1).clean_bytes;
}

extern "C" int csgs_workspace_init(csgs_workspace *ws, void *stream)
{
    if (!ws) return CSGS_EINVAL;
    ws->rows_buf = 0;
    ws->has_draw = 0;
    ws->has_next = 0;
    ws->draw_B = 0;
    Workspace w;
    const int rc = open_workspace(ws, ws->n_nodes, 1, 1, &w);
    if (rc != CSGS_OK) return rc;
    const size_t n = w.bytes * (size_t)w.n_inst / 8;
    const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    CSGS_LAUNCH(K_FILL_ZERO, fill_zero, dim3(blocks), dim3(256), (hipStream_t)stream, (uint64_t *)ws->base, n);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

namespace csgs {
// one block per instance
__global__ void set_word(uint64_t *p, uint64_t v, int64_t stride) { *(uint64_t *)((char *)p + (int64_t)blockIdx.x * stride) = v; }
}  // namespace csgs

extern "C" int csgs_workspace_wait_limit(csgs_workspace *ws, int64_t polls, void *stream)
{
    if (!ws) return CSGS_EINVAL;
    Workspace w;
    const int rc = open_workspace(ws, ws->n_nodes, 1, 1, &w);
    if (rc != CSGS_OK) return rc;
    const uint64_t v = polls < 0 ? 0ull : (uint64_t)(polls > 0x7FFFFFF0ll ? 0x7FFFFFF0ll : polls) + 1ull;
    CSGS_LAUNCH(K_FILL_ZERO, csgs::set_word, dim3((unsigned)w.n_inst), dim3(1), (hipStream_t)stream, w.epoch + EPOCH_WAIT, v,
                (int64_t)w.bytes);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

// Fixed-point parameters.  shift = min(52, 61 - ceil(log2 nS) - ceil(log2 s_fx) - ceil(log2 rmax)):
// the skewed total is at most nS * rmax * 2^shift * s_fx plus rounding slack, below 2^63.
extern "C" int csgs_fixed_point(int32_t nS, float skew, float rownorm2_max, int32_t *shift, int64_t *s_fx)
{
    if (nS <= 0 || !(skew >= 1.0f) || skew > 1048576.0f || !(rownorm2_max > 0.0f) || !isfinite(rownorm2_max))
        return CSGS_EINVAL;
    const int64_t sfx = llround((double)skew * 16.0);
    int sh = shift_base_for(sfx, rownorm2_max) - ceil_log2_u64((uint64_t)nS);
    if (sh > 52) sh = 52;
    if (shift) *shift = sh;
    if (s_fx) *s_fx = sfx;
    return sh < 24 ? CSGS_ERANGE : CSGS_OK;
}

static int build_probs_impl(const csgs_graph *g, const int32_t *S, int32_t nS, const int32_t *nS_dev,
                            float shift_skew, SkewPolicy pol,
                            int32_t *cand_id, uint64_t *cand_w, uint64_t *cdf, float *q, int64_t cap,
                            csgs_prob_stats *stats, csgs_workspace *ws, int32_t *status, void *stream)
{
    if (!g || !g->rowptr || !g->colidx || !g->val || g->n_nodes <= 0 || g->n_nodes > 0x7FFFFFFFll ||
        g->local_lo > g->local_hi || nS <= 0 || !cand_id || !cand_w || !cdf || cap <= 0 || !stats || !ws || !status)
        return CSGS_EINVAL;
    // S == NULL: the rows are the node set of the latest csgs_sample_layer on this workspace, whose
    // offsets that call has prepared; nS must be its capacity (the B of that draw)
    if (ws->scan_mode < 0 || ws->scan_mode > 2) return CSGS_EINVAL;
    const bool chained = S == nullptr;
    if (chained && (!ws->has_next || nS_dev || nS != ws->draw_B)) return CSGS_EINVAL;
    int32_t shift;
    int64_t s_fx;
    int rc = csgs_fixed_point(nS, shift_skew, g->rownorm2_max, &shift, &s_fx);
    if (rc != CSGS_OK) return rc;
    if (pol.mode == 0) pol.s_fx = (uint64_t)s_fx;
    if (pol.mode == 1) pol.s_fx_max = (uint64_t)s_fx;
    Workspace w;
    rc = open_workspace(ws, g->n_nodes, nS, 1, &w);
    if (rc != CSGS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int64_t n_words = (g->n_nodes + 63) / 64;

    // the shift for nS rows has passed the range check; fewer rows on the device only widen it
    const int32_t shift_base = shift_base_for(s_fx, g->rownorm2_max);
    if (chained) {
        ws->rows_buf ^= 1;      // the set the adjacency pass prepared
    } else {
        rc = launch_row_prefix(g->rowptr, g->n_nodes, S, nS, nS_dev, w, w.rows[ws->rows_buf & 1], status, st);
        if (rc != CSGS_OK) return rc;
    }
    ws->has_next = 0;
    const RowOffsets &rows = w.rows[ws->rows_buf & 1];
    const unsigned nz = (unsigned)w.n_inst;
    const InstStride is = inst_stride(w);
    // owner blocks for the local id range, when it is one the hand-over can cover
    const int64_t n_local = (int64_t)g->local_hi - (int64_t)g->local_lo;
    const int32_t owners = (n_local > 0 && n_local <= (int64_t)SUB_IDS * SUB_MAX && g->local_lo >= 0 && g->local_hi <= g->n_nodes)
                               ? (int32_t)((n_local + SUB_IDS - 1) / SUB_IDS) : 0;
    const Stage stg{w.stage_w, w.stage_c, w.stage_off, (unsigned long long *)w.stage_done, w.stage_chunks, g->local_lo,
                    g->local_hi, owners, ws->scan_mode};
    CSGS_LAUNCH(K_SCAN_EDGES, scan_edges, dim3((unsigned)(EDGE_GRID + owners), 1, nz), dim3(256), st, g->colidx, g->val,
                g->n_nodes, g->nnz, shift_base, rows.meta, w.chunk_cap * EDGE_TILE, rows.eoff, rows.rowstart, w.wtable,
                w.tileflag, rows.chunk_note, rows.bound_note, status, w.epoch, stg, is);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_CAND_PARTIALS, cand_partials, dim3((unsigned)((w.n_tiles + CAND_PART_TILES - 1) / CAND_PART_TILES), 1, nz), dim3(256), st, w.wtable, w.tileflag, n_words,
                g->n_nodes, w.n_tiles, g->local_lo, g->local_hi, w.epoch, (unsigned long long *)w.cand_flag,
                (unsigned long long *)w.partial, w.gtot, status, is);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_CAND_EMIT, cand_emit, dim3((unsigned)w.n_tiles, 1, nz), dim3(256), st, w.wtable, w.tileflag, n_words,
                g->n_nodes, w.n_tiles, g->local_lo, g->local_hi, pol, w.partial, w.gtot, rows.meta, shift_base, w.epoch, stats, status, cand_id,
                cand_w, cdf, q, cap, is);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_build_probs(const csgs_graph *g, const int32_t *S, int32_t nS, const int32_t *nS_dev, float skew,
                                int32_t *cand_id,
                                uint64_t *cand_w, uint64_t *cdf, float *q, int64_t cap, csgs_prob_stats *stats,
                                csgs_workspace *ws, int32_t *status, void *stream)
{
    SkewPolicy pol = {0, 0, 0.0, 0, 0};
    float shift_skew = skew;
    if (isinf(skew) && skew > 0) {   // "Local" version: remote candidates get probability zero
        pol.mode = 2;
        shift_skew = 1.0f;
    }
    return build_probs_impl(g, S, nS, nS_dev, shift_skew, pol, cand_id, cand_w, cdf, q, cap, stats, ws, status, stream);
}

extern "C" int csgs_build_probs_auto(const csgs_graph *g, const int32_t *S, int32_t nS, const int32_t *nS_dev, float D,
                                     int32_t B,
                                     float skew_max, int32_t *cand_id, uint64_t *cand_w, uint64_t *cdf, float *q,
                                     int64_t cap, csgs_prob_stats *stats, csgs_workspace *ws, int32_t *status,
                                     void *stream)
{
    if (!(D >= 0.0f) || !isfinite(D) || B <= 0) return CSGS_EINVAL;
    SkewPolicy pol = {1, 0, (double)D, (int64_t)B, 0};
    return build_probs_impl(g, S, nS, nS_dev, skew_max, pol, cand_id, cand_w, cdf, q, cap, stats, ws, status, stream);
}
