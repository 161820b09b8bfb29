// csgs_draw_nodes, csgs_sampled_adjacency, csgs_sample_layer and csgs_remote_count.
//
// B draws with replacement from the skewed distribution (Section 4.1: the sampling is run B
// times), deduplicated; inclusion probability p_j = 1 - (1 - q_j)^B (Eq. 8); sampled adjacency
// with every kept edge divided by p_j (Eq. 3); number of sampled remote nodes (Eq. 4).
//
// Kernels:
//   draw          one thread per draw: Philox4x32-10 word -> u = mulhi(r, total) -> first cdf
//                 entry above u.  The top levels of the search run on a strided sample of the
//                 CDF staged in LDS, the rest is an 8-ary search on the global array (seven
//                 independent probes per round).  Hits are counted per candidate position with
//                 integer atomics; first hits set a position bitmap.
//   hits_fused    single pass over the position bitmap (tiles of 256 words): ordered list of
//                 the tile's hits in LDS, prefix over earlier tiles by the single-pass scan
//                 across blocks, then one thread per distinct hit: S_next ascending, mult,
//                 p_incl, node -> rank table.  Everything but the output position is fetched
//                 and computed while the prefix is being resolved.
//   adj_fused     flat over the edges of S (same chunking as the weight scan), single pass: keep
//                 = the target was sampled; the kept edges in flat order ARE the CSR of P~ (rows
//                 in the order of S, columns ascending), so position = prefix of the chunk +
//                 popcount of earlier keep bits, and the row pointers are the positions at the
//                 row starts.  The node -> rank table is never cleared: its entries carry the
//                 tag of the draw that wrote them.
//   remote_count_k  S_next ascends and the local partition is one id range: two searches by a
//                 whole wavefront place every element (see the kernel)
#include <math.h>
#include "common.hpp"
#include "lookback.hpp"
#include "row_prefix.hpp"

namespace csgs {

// Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11): each round multiplies two
// counter words by fixed odd constants, swaps halves around and xors in the key, then the key
// advances by two Weyl increments.
__device__ inline uint64_t philox_word(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0;
        const uint32_t n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return (uint64_t)c0 | ((uint64_t)c1 << 32);
}

constexpr int DRAW_BLOCK = 256;
constexpr int TOP = 2048;  // CDF samples staged in LDS per block (16 KB)

__global__ __launch_bounds__(DRAW_BLOCK) void draw(const uint64_t *__restrict__ cdf,
                                                   const csgs_prob_stats *__restrict__ stats, int64_t cand_cap,
                                                   int32_t B, uint32_t seed_lo, uint32_t seed_hi, uint64_t iter,
                                                   const uint64_t *__restrict__ iter_dev, uint32_t layer,
                                                   uint32_t *__restrict__ hit, uint64_t *__restrict__ cbitmap,
                                                   const uint64_t *__restrict__ epoch, uint64_t *__restrict__ rank,
                                                   uint64_t *__restrict__ member, int64_t n_nodes, InstStride is)
{
    __shared__ uint64_t top[TOP];
    cdf = inst_ptr(cdf, is.buf); stats = inst_ptr(stats, is.buf);
    hit = inst_ptr(hit, is.ws); cbitmap = inst_ptr(cbitmap, is.ws); epoch = inst_ptr(epoch, is.ws); rank = inst_ptr(rank, is.ws);
    member = inst_ptr(member, is.ws);
    // rank entries and membership words carry the low 32 bits of the call number; when those wrap, stale
    // entries could look current, so both tables are wiped once every 2^32 calls (the compaction kernel that
    // follows writes the new entries)
    if ((call_number(epoch) & 0xFFFFFFFFull) == 0) {
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_nodes; i += (int64_t)gridDim.x * blockDim.x) {
            rank[i] = 0ull;
            if (i < (n_nodes + 31) / 32) member[i] = 0ull;
        }
    }
    if (iter_dev) iter = *iter_dev;
    iter += blockIdx.z;   // consecutive instances are consecutive iterations
    const uint32_t iter_lo = (uint32_t)iter, iter_hi = (uint32_t)(iter >> 32);
    int64_t n = stats->n_cand;
    if (n > cand_cap) n = cand_cap;
    if (n <= 0) return;
    const uint64_t total = stats->total;   // = cdf[n - 1], without waiting for a second dependent load
    if (total == 0) return;
    // top[i] = cdf[(i + 1) * stride - 1] for the i with that index inside the array
    const int64_t stride = (n + TOP - 1) / TOP;
    const int64_t n_top = n / stride;  // number of complete strides
    for (int64_t i = threadIdx.x; i < n_top; i += blockDim.x) top[i] = cdf[(i + 1) * stride - 1];
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= B) return;
    const uint64_t r = philox_word((uint32_t)t, layer, iter_lo, iter_hi, seed_lo, seed_hi);
    const uint64_t u = __umul64hi(r, total);
    // first sample above u: the answer lies in stride block a
    int64_t a = 0, b = n_top;
    while (a < b) {
        const int64_t m = (a + b) >> 1;
        if (top[m] > u) b = m; else a = m + 1;
    }
    int64_t lo = a * stride;
    int64_t hi = (a < n_top) ? (a + 1) * stride - 1 : n - 1;  // cdf[hi] > u is known; the answer is in [lo, hi]
    // 8-ary search on the global array: 7 independent probes per round instead of one
    while (hi - lo >= 8) {
        const int64_t len = hi - lo;  // candidates lo .. hi, hi already known to be above u
        uint64_t pv[7];
#pragma unroll
        for (int i = 0; i < 7; ++i) pv[i] = cdf[lo + (len * (i + 1)) / 8];
        int below = 0;                // pivots that are <= u (they ascend, so these are the first ones)
#pragma unroll
        for (int i = 0; i < 7; ++i) below += pv[i] <= u ? 1 : 0;
        const int64_t new_lo = below ? lo + (len * below) / 8 + 1 : lo;
        const int64_t new_hi = below < 7 ? lo + (len * (below + 1)) / 8 : hi;
        lo = new_lo;
        hi = new_hi;
    }
    {
        // at most 8 entries left: fetch them together, take the first above u
        uint64_t v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (lo + i < hi) ? cdf[lo + i] : ~0ull;
        int skip = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) skip += v[i] <= u ? 1 : 0;
        lo += skip;  // entries ascend; cdf[hi] > u bounds the result by hi
        if (lo > hi) lo = hi;
    }
    // both updates are fire-and-forget (no returned value to wait for); setting an already set bit is harmless
    (void)__hip_atomic_fetch_add(&hit[lo], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    (void)__hip_atomic_fetch_or((unsigned long long *)&cbitmap[lo >> 6], 1ull << (lo & 63), __ATOMIC_RELAXED,
                                __HIP_MEMORY_SCOPE_AGENT);
}

// The membership words: word id / 32 holds (tag << 32) | one bit per id, set when the id is in S_next of the draw
// with that tag; the adjacency pass looks an edge's column up here (612 KB for 2.4 M nodes: it stays in the L2s)
// and goes to the 8-byte-per-node rank table only for the one column in twenty that is a member.
// Merging bits into a word that other wavefronts may write as well: a word of an older draw counts as empty.  Two
// updates nobody waits for: a 64-bit maximum with (tag << 32) replaces an older draw's word by the empty word of this
// draw and leaves a current one alone (tags ascend from draw to draw; the table is wiped when they wrap), then the
// bits are or-ed in.  Updates of one address by one lane take effect in program order.
__device__ inline void member_merge(uint64_t *word, uint32_t bits, uint32_t tag32)
{
    unsigned long long *p = reinterpret_cast<unsigned long long *>(word);
    (void)__hip_atomic_fetch_max(p, (unsigned long long)tag32 << 32, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    (void)__hip_atomic_fetch_or(p, (unsigned long long)bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Every lane of a wavefront calls this with the id of its hit (-1: none).  The hits of a wavefront are consecutive
// entries of the ascending list, so the ids that share a word sit in neighbouring lanes: their bits are put
// together by lane exchanges and the first lane of the run stores the word.  All ids of a word that lies strictly
// inside the wavefront's hits are in this wavefront, so that store is a plain one; a run next to a lane without a
// hit, or at either end of the wavefront, may go on in another wavefront and is merged atomically.
__device__ inline void mark_members(uint64_t *__restrict__ member, int32_t id, uint32_t tag32)
{
    const int lane = lane_id();
    const int32_t w = id >= 0 ? id >> 5 : -1;
    uint32_t bits = id >= 0 ? 1u << (id & 31) : 0u;
    const int32_t wp = __shfl_up(w, 1, WAVE), wn = __shfl_down(w, 1, WAVE);
    const bool head = w >= 0 && (lane == 0 || wp != w);
    uint32_t open = (w >= 0 && (lane == WAVE - 1 || wn < 0)) ? 1u : 0u;   // matters in the run's last lane: nothing valid follows it here
#pragma unroll
    for (int d = 1; d <= 16; d <<= 1) {   // a run has at most 32 lanes
        const uint32_t ob = __shfl_down(bits, d, WAVE), oo = __shfl_down(open, d, WAVE);
        const int32_t w2 = __shfl_down(w, d, WAVE);
        if (lane + d < WAVE && w2 == w) { bits |= ob; open |= oo; }
    }
    if (head) {
        if (open || lane == 0 || wp < 0) member_merge(&member[w], bits, tag32);
        else member[w] = ((uint64_t)tag32 << 32) | bits;
    }
}

__global__ __launch_bounds__(256) void hits_fused(const int32_t *__restrict__ cand_id,
                                                  const uint64_t *__restrict__ cdf,
                                                  const csgs_prob_stats *__restrict__ stats, int64_t cand_cap,
                                                  int64_t n_nodes, int32_t B, uint64_t *__restrict__ epoch,
                                                  uint64_t *__restrict__ ts_mem, int64_t ts_tiles,
                                                  uint32_t *__restrict__ hit, uint64_t *__restrict__ cbitmap,
                                                  uint64_t *__restrict__ rank, uint64_t *__restrict__ member,
                                                  int32_t *__restrict__ S_next,
                                                  int32_t *__restrict__ mult, float *__restrict__ p_incl,
                                                  double *__restrict__ pdbl, int32_t *__restrict__ n_next,
                                                  int32_t *__restrict__ status, InstStride is)
{
    __shared__ uint32_t lds[17];
    member = inst_ptr(member, is.ws);
    cand_id = inst_ptr(cand_id, is.buf); cdf = inst_ptr(cdf, is.buf); stats = inst_ptr(stats, is.buf);
    S_next = inst_ptr(S_next, is.buf); mult = inst_ptr(mult, is.buf); p_incl = inst_ptr(p_incl, is.buf);
    n_next = inst_ptr(n_next, is.buf); status = inst_ptr(status, is.buf);
    epoch = inst_ptr(epoch, is.ws); ts_mem = inst_ptr(ts_mem, is.ws); hit = inst_ptr(hit, is.ws);
    cbitmap = inst_ptr(cbitmap, is.ws); rank = inst_ptr(rank, is.ws); pdbl = inst_ptr(pdbl, is.ws);
    __shared__ unsigned long long s_lb[1];
    __shared__ uint16_t s_list[HIT_TILE_WORDS * 64];   // drawn positions of the tile, ascending
    const TileState<1> ts(ts_mem, ts_tiles, wait_limit(epoch));
    const unsigned long long call = call_number(epoch);
    const unsigned long long tag = call_tag(call, SLOT_HITS);
    int64_t n = stats->n_cand;
    if (n > cand_cap) n = cand_cap;
    if (n < 0) n = 0;
    const int64_t n_words = (n + 63) / 64;
    const int64_t n_tiles = (n_words + HIT_TILE_WORDS - 1) / HIT_TILE_WORDS;
    if (n_tiles == 0) {
        if (blockIdx.x == 0 && threadIdx.x == 0) {  // no candidates at all
            *n_next = 0;
            epoch[EPOCH_DRAW] = call;
            epoch[EPOCH_CALLS] = call;
        }
        return;
    }
    const double total = (double)stats->total;   // = cdf[n - 1]
    const uint64_t rank_tag = (call & 0xFFFFFFFFull) << 32;
    for (int64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        // one bitmap word per thread -> ordered list of the tile's drawn positions in LDS
        const int64_t wi = t * HIT_TILE_WORDS + threadIdx.x;
        uint64_t word = wi < n_words ? cbitmap[wi] : 0ull;
        const uint32_t cnt = (uint32_t)__popcll(word);
        uint32_t tile_total;
        uint32_t ex = block_exclusive_scan<uint32_t>(cnt, lds, &tile_total);
        if (word) cbitmap[wi] = 0ull;  // back to the clean state
        while (word) {
            const int bit = __ffsll((unsigned long long)word) - 1;
            word &= word - 1;
            s_list[ex++] = (uint16_t)(threadIdx.x * 64 + bit);
        }
        unsigned long long local[1] = {tile_total}, excl[1];
        lookback_publish<1>(ts, tag, t, local);
        __syncthreads();  // s_list complete
        // One thread per distinct hit.  Everything except the output position is ready before the
        // prefix is: fetch and compute it now.  The tile's first hits go to the last threads, so
        // that the arithmetic runs in other wavefronts than the one that does the hops.
        const uint32_t i0 = (uint32_t)(blockDim.x - 1 - threadIdx.x);
        int64_t kpos0 = 0;
        uint32_t m0 = 0;
        int32_t id0 = -1;
        double pk0 = 0.0;
        if (i0 < tile_total) {
            kpos0 = t * (HIT_TILE_WORDS * 64) + s_list[i0];
            m0 = hit[kpos0];
            hit[kpos0] = 0u;
            const uint64_t wk = cdf[kpos0] - (kpos0 ? cdf[kpos0 - 1] : 0ull);
            const double qk = (double)wk / total;
            pk0 = (qk >= 1.0) ? 1.0 : -expm1((double)B * log1p(-qk));
            id0 = cand_id[kpos0];
        }
        lookback_resolve<1>(ts, tag, t, n_tiles, local, excl, s_lb, status);
        int32_t member_id = -1;
        if (i0 < tile_total) {
            const uint64_t pos = excl[0] + i0;
            if (pos < (uint64_t)B) {  // at most B distinct hits exist; the guard keeps stores in bounds regardless
                S_next[pos] = id0;
                mult[pos] = (int32_t)m0;
                p_incl[pos] = (float)pk0;
                pdbl[pos] = pk0;
                if (id0 >= 0 && id0 < n_nodes) {
                    rank[id0] = rank_tag | (pos + 1);
                    member_id = id0;
                }
            }
        }
        mark_members(member, member_id, (uint32_t)(rank_tag >> 32));
        for (uint32_t i_base = blockDim.x; i_base < tile_total; i_base += blockDim.x) {  // crowded tiles (every lane goes round together)
            const uint32_t i = i_base + threadIdx.x;
            int32_t marked = -1;
            if (i < tile_total) {
                const int64_t kpos = t * (HIT_TILE_WORDS * 64) + s_list[i];
                const uint64_t pos = excl[0] + i;
                const uint32_t m = hit[kpos];
                hit[kpos] = 0u;
                if (pos < (uint64_t)B) {
                    const uint64_t wk = cdf[kpos] - (kpos ? cdf[kpos - 1] : 0ull);
                    const double qk = (double)wk / total;
                    const double pk = (qk >= 1.0) ? 1.0 : -expm1((double)B * log1p(-qk));
                    const int32_t id = cand_id[kpos];
                    S_next[pos] = id;
                    mult[pos] = (int32_t)m;
                    p_incl[pos] = (float)pk;
                    pdbl[pos] = pk;
                    if (id >= 0 && id < n_nodes) {
                        rank[id] = rank_tag | (pos + 1);
                        marked = id;
                    }
                }
            }
            mark_members(member, marked, (uint32_t)(rank_tag >> 32));
        }
        if (t == n_tiles - 1 && threadIdx.x == 0) {
            const uint64_t tot = excl[0] + tile_total;
            *n_next = (int32_t)(tot < (uint64_t)B ? tot : (uint64_t)B);
            // Last kernel of the draw: advance the call counter.  Every block that owns a tile has
            // read it by now (this tile's prefix needed all their sums), the others never use it.
            epoch[EPOCH_DRAW] = call;
            epoch[EPOCH_CALLS] = call;
        }
        __syncthreads();  // s_list is reused by the next tile
    }
}

// S_next ascends and the local partition is one id range, so the sampled remote nodes are the
// entries before the first id >= lo and from the first id >= hi on: two searches give every
// element its place, no scan needed.
constexpr int REMOTE_BLOCKS = 64;

struct RemoteArgs {
    const int32_t *S_next, *n_next;
    int32_t lo, hi;
    const int32_t *part_bounds;
    int32_t P;
    int64_t *remote_total, *per_part;
    int32_t *src_row, *remote_ids;
    int32_t blocks;   // blocks of 256 threads that do this work (as leading blocks of another kernel: 0 = none)
};

// `block` of `n_blocks` blocks of 256 threads
__device__ inline void remote_count_body(const RemoteArgs &r_, int32_t block, int32_t n_blocks)
{
    const int32_t *__restrict__ S_next = r_.S_next;
    const int32_t lo = r_.lo, hi = r_.hi, P = r_.P;
    const int32_t *__restrict__ part_bounds = r_.part_bounds;
    int64_t *__restrict__ remote_total = r_.remote_total, *__restrict__ per_part = r_.per_part;
    int32_t *__restrict__ src_row = r_.src_row, *__restrict__ remote_ids = r_.remote_ids;
    int32_t n = *r_.n_next;
    if (n < 0) n = 0;
    const int32_t a = wave_lower_bound(S_next, n, lo);   // ids below the local range
    const int32_t b = wave_lower_bound(S_next, n, hi);   // first id above it
    const int32_t n_local = b - a;
    const int32_t tid = (int32_t)(block * blockDim.x + threadIdx.x);
    const int32_t stride = (int32_t)(n_blocks * blockDim.x);
    if (tid == 0) *remote_total = (int64_t)(n - n_local);
    if (src_row || remote_ids) {
        for (int32_t k = tid; k < n; k += stride) {
            const int32_t j = S_next[k];
            if (k >= a && k < b) {
                if (src_row) src_row[k] = j - lo;
            } else {
                const int32_t r = k < a ? k : k - n_local;
                if (src_row) src_row[k] = -1 - r;
                if (remote_ids && r >= 0 && r < n) remote_ids[r] = j;   // (r leaves [0, n) only if S_next does not ascend)
            }
        }
    }
    // partition p holds the ids between two lower bounds; one wavefront per partition
    if (per_part) {
        const int32_t wave = tid >> 6, n_waves = stride >> 6;
        for (int32_t p = wave; p < P; p += n_waves) {
            const int32_t c0 = wave_lower_bound(S_next, n, part_bounds[p]);
            const int32_t c1 = wave_lower_bound(S_next, n, part_bounds[p + 1]);
            if (lane_id() == 0) per_part[p] = (int64_t)(c1 > c0 ? c1 - c0 : 0);
        }
    }
}

__global__ __launch_bounds__(256) void remote_count_k(RemoteArgs r) { remote_count_body(r, (int32_t)blockIdx.x, (int32_t)gridDim.x); }

// Work of the adjacency kernel's second group of spare blocks: the row offsets of the node set just
// sampled, for a following csgs_build_probs on those rows (one tile of rows per block).
struct NextRows {
    const int64_t *rowptr;
    int64_t n_nodes;
    const int32_t *S_next, *n_next;
    int32_t bound;        // capacity of S_next (the B of the draw)
    uint64_t *ts_mem;
    int64_t ts_tiles;
    int64_t *eoff, *rowstart, *meta;
    int2 *bound_note;
    int64_t edge_cap;
    int32_t blocks;       // 0 = none
};

template <bool FROM_NOTE>
__global__ __launch_bounds__(256) void adj_fused(const int32_t *__restrict__ colidx, const float *__restrict__ val,
                                                 int64_t n_nodes, int64_t nnz, const int64_t *__restrict__ meta,
                                                 const int64_t *__restrict__ eoff,
                                                 const int64_t *__restrict__ rowstart,
                                                 const uint64_t *__restrict__ rank, const uint64_t *__restrict__ member,
                                                 const double *__restrict__ pdbl,
                                                 uint64_t *__restrict__ epoch, uint64_t *__restrict__ ts_mem, int64_t chunk_cap,
                                                 int2 *__restrict__ chunk_note, int32_t *__restrict__ adj_rowptr,
                                                 int32_t *__restrict__ adj_col, float *__restrict__ adj_val,
                                                 int64_t adj_cap, int64_t *__restrict__ adj_nnz,
                                                 int32_t *__restrict__ status, RemoteArgs rem, NextRows nxt, InstStride is)
{
    status = inst_ptr(status, is.buf);
    epoch = inst_ptr(epoch, is.ws);
    // The leading rem.blocks blocks split the new node set into local and remote (what
    // csgs_remote_count does: it needs only S_next / n_next, complete since the previous kernel) so
    // that a layer step is one launch shorter; they wait for nobody and nobody waits for them.
    if ((int32_t)blockIdx.x < rem.blocks) {
        rem.S_next = inst_ptr(rem.S_next, is.buf); rem.n_next = inst_ptr(rem.n_next, is.buf);
        rem.remote_total = inst_ptr(rem.remote_total, is.buf); rem.per_part = inst_ptr(rem.per_part, is.buf);
        rem.src_row = inst_ptr(rem.src_row, is.buf); rem.remote_ids = inst_ptr(rem.remote_ids, is.buf);
        remote_count_body(rem, (int32_t)blockIdx.x, rem.blocks);
        return;
    }
    // The next nxt.blocks blocks lay out the rows of the new node set.  They wait only for each other
    // (lower tiles, dispatched before them); their flags are tagged with the draw's call number,
    // which the previous kernel wrote, so the counter this kernel advances at its end does not matter.
    if ((int32_t)blockIdx.x < rem.blocks + nxt.blocks) {
        nxt.S_next = inst_ptr(nxt.S_next, is.buf); nxt.n_next = inst_ptr(nxt.n_next, is.buf);
        nxt.ts_mem = inst_ptr(nxt.ts_mem, is.ws); nxt.eoff = inst_ptr(nxt.eoff, is.ws);
        nxt.rowstart = inst_ptr(nxt.rowstart, is.ws); nxt.meta = inst_ptr(nxt.meta, is.ws);
        nxt.bound_note = inst_ptr(nxt.bound_note, is.ws);
        const int32_t n = resolve_count(nxt.bound, nxt.n_next);
        const int64_t t = (int64_t)blockIdx.x - rem.blocks, n_tiles = row_tiles(n);
        if (t < n_tiles) {
            const TileState<1> rts(nxt.ts_mem, nxt.ts_tiles, wait_limit(epoch));
            row_prefix_tile(nxt.rowptr, nxt.n_nodes, nxt.S_next, n, t, n_tiles, rts, call_tag(epoch[EPOCH_DRAW], SLOT_ROWS_NEXT),
                            nxt.eoff, nxt.rowstart, nxt.meta, nxt.edge_cap, nxt.bound_note, nxt.edge_cap / EDGE_TILE, status);
        }
        return;
    }
    meta = inst_ptr(meta, is.ws); eoff = inst_ptr(eoff, is.ws); rowstart = inst_ptr(rowstart, is.ws);
    rank = inst_ptr(rank, is.ws); member = inst_ptr(member, is.ws); pdbl = inst_ptr(pdbl, is.ws); ts_mem = inst_ptr(ts_mem, is.ws);
    chunk_note = inst_ptr(chunk_note, is.ws);
    adj_rowptr = inst_ptr(adj_rowptr, is.buf); adj_col = inst_ptr(adj_col, is.buf); adj_val = inst_ptr(adj_val, is.buf);
    adj_nnz = inst_ptr(adj_nnz, is.buf);
    const int64_t bid = (int64_t)blockIdx.x - rem.blocks - nxt.blocks;
    const int64_t n_bids = (int64_t)gridDim.x - rem.blocks - nxt.blocks;
    __shared__ RowSlice slice;
    __shared__ uint64_t s_mask[EDGE_TILE / 64];
    __shared__ int32_t s_pre[EDGE_TILE / 64 + 1];
    __shared__ unsigned long long s_lb[1];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const TileState<1> ts(ts_mem, chunk_cap, wait_limit(epoch));
    const unsigned long long call = call_number(epoch);
    const unsigned long long tag = call_tag(call, SLOT_ADJ);
    const uint64_t rank_tag = (epoch[EPOCH_DRAW] & 0xFFFFFFFFull) << 32;
    const int32_t nS = (int32_t)meta[META_ROWS];
    // Row pointers never exceed what adj_col / adj_val can hold: when the kept edges overflow the
    // capacity (status bit), later kernels that walk the rows still stay inside the arrays.
    const int64_t ptr_max = adj_cap < 0x7FFFFFFFll ? adj_cap : 0x7FFFFFFFll;
    int64_t E = meta[META_EDGES];
    int64_t n_chunks = (E + EDGE_TILE - 1) / EDGE_TILE;
    bool overflow = false;
    if (n_chunks > chunk_cap) {  // the workspace cannot describe this many chunks: report, emit nothing
        overflow = true;
        E = 0;
        n_chunks = 0;
    }
    if (n_chunks == 0) {
        if (bid == 0) {
            for (int32_t a = threadIdx.x; a <= nS; a += blockDim.x) adj_rowptr[a] = 0;
            if (threadIdx.x == 0) {
                *adj_nnz = 0;
                if (overflow) atomicOr(status, CSGS_ST_EDGE_OVERFLOW);
                epoch[EPOCH_CALLS] = call;
            }
        }
        return;
    }
    // all blocks are resident; block b takes chunks b, b + grid, ... in ascending order
    for (int64_t t = bid; t < n_chunks; t += n_bids) {
        const int64_t c0 = t * EDGE_TILE;
        const int64_t c1 = (c0 + EDGE_TILE < E) ? c0 + EDGE_TILE : E;
        stage_slice<FROM_NOTE>(slice, eoff, rowstart, nS, c0, c1, FROM_NOTE ? chunk_note + t : nullptr);
        const int32_t len = (int32_t)(c1 - c0);
        // wave w owns positions [w * 256, w * 256 + 256): four 64-edge words
        // A lane's four edges go through each step together, and no load sits under a condition (an edge that does
        // not exist reads entry 0 and is dropped): the four columns travel at the same time, then the four table
        // lookups, instead of eight trips one after the other.
        int32_t rk[4];
        int64_t ea[4];
        bool live[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int32_t x = wave * 256 + k * 64 + lane;
            ea[k] = 0;
            live[k] = false;
            if (x < len) {
                int32_t r;
                const int64_t a = edge_address(slice, eoff, rowstart, c0, x, &r);
                if (a >= 0 && a < nnz) {   // (an address outside the graph can only follow a failed wait)
                    ea[k] = a;
                    live[k] = true;
                }
            }
        }
        int32_t ck[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) ck[k] = colidx[ea[k]];
        // the membership word of every column first (a small table that stays in the L2s), then the rank entry, which
        // only a member's lane reads from its own place (the others read entry 0)
        uint64_t mw[4], re[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            live[k] = live[k] && ck[k] >= 0 && ck[k] < n_nodes;
            mw[k] = member[live[k] ? ck[k] >> 5 : 0];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            live[k] = live[k] && (mw[k] & 0xFFFFFFFF00000000ull) == rank_tag && ((mw[k] >> (ck[k] & 31)) & 1ull);
            re[k] = rank[live[k] ? ck[k] : 0];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            rk[k] = (live[k] && (re[k] & 0xFFFFFFFF00000000ull) == rank_tag) ? (int32_t)(re[k] & 0xFFFFFFFFull) : 0;
            const uint64_t m = __ballot(rk[k] > 0);
            if (lane == 0) s_mask[wave * 4 + k] = m;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int32_t acc = 0;
            for (int i = 0; i < EDGE_TILE / 64; ++i) { s_pre[i] = acc; acc += __popcll(s_mask[i]); }
            s_pre[EDGE_TILE / 64] = acc;
        }
        __syncthreads();
        const int32_t tile_cnt = s_pre[EDGE_TILE / 64];
        unsigned long long local[1] = {(unsigned long long)tile_cnt}, excl[1];
        lookback_publish<1>(ts, tag, t, local);
        // values of the kept edges do not depend on the prefix: fetch and divide while it is resolved
        float pv[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {   // (unconditional loads again: entry 0 stands in for an edge that was not kept)
            const float vv = val[ea[k]];
            const double pp = pdbl[rk[k] > 0 ? rk[k] - 1 : 0];
            pv[k] = rk[k] > 0 ? (float)((double)vv / pp) : 0.f;
        }
        lookback_resolve<1>(ts, tag, t, n_chunks, local, excl, s_lb, status);
        const int64_t base = (int64_t)excl[0];
        // row pointers of the rows that start inside this chunk: kept edges before the row start
        const int32_t R = slice.R;
        const int64_t a_first = slice.a_first;
        for (int32_t r = threadIdx.x; r < R; r += blockDim.x) {
            const int64_t off = slice.in_lds ? (int64_t)slice.off[r] : eoff[a_first + r] - c0;
            if (off >= 0 && off < len) {
                const int64_t v = base + s_pre[off >> 6] + __popcll(s_mask[off >> 6] & ((1ull << (off & 63)) - 1ull));
                adj_rowptr[a_first + r] = (int32_t)(v < ptr_max ? v : ptr_max);
            }
        }
        if (tile_cnt) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (rk[k] <= 0) continue;
                const int32_t word = wave * 4 + k;
                const int64_t pos = base + s_pre[word] + __popcll(s_mask[word] & ((1ull << lane) - 1ull));
                if (pos < adj_cap) {
                    adj_col[pos] = rk[k] - 1;
                    adj_val[pos] = pv[k];
                }
            }
        }
        if (t == n_chunks - 1) {
            // rows that start at or after the last edge (trailing empty rows, and the end pointer)
            const int64_t total = base + tile_cnt;
            const int32_t clamp = (int32_t)(total < ptr_max ? total : ptr_max);
            const int64_t first_tail = wave_lower_bound(eoff, (int64_t)nS + 1, E);
            for (int64_t a = first_tail + threadIdx.x; a <= nS; a += blockDim.x) adj_rowptr[a] = clamp;
            if (threadIdx.x == 0) {
                *adj_nnz = total;
                if (total > adj_cap || total > 0x7FFFFFFFll) atomicOr(status, CSGS_ST_ADJ_OVERFLOW);
                epoch[EPOCH_CALLS] = call;  // last kernel of the call, last chunk: all chunk owners have read the counter
            }
        }
    }
}

}  // namespace csgs
using namespace csgs;

extern "C" int csgs_draw_nodes(int64_t n_nodes, const int32_t *cand_id, const uint64_t *cdf, int64_t cand_cap,
                               const csgs_prob_stats *stats, int32_t B, uint64_t seed, uint64_t iter,
                               const uint64_t *iter_dev, uint32_t layer, int32_t *S_next, int32_t *mult, float *p_incl,
                               int32_t *n_next, csgs_workspace *ws, int32_t *status, void *stream)
{
    if (n_nodes <= 0 || n_nodes > 0x7FFFFFFFll || !cand_id || !cdf || cand_cap <= 0 || !stats || B <= 0 || !S_next ||
        !mult || !p_incl || !n_next || !ws || !status)
        return CSGS_EINVAL;
    Workspace w;
    const int rc = open_workspace(ws, n_nodes, 1, B, &w);
    if (rc != CSGS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (cand_cap > n_nodes) cand_cap = n_nodes;  // there are never more candidates than nodes

    const unsigned nz = (unsigned)w.n_inst;
    const InstStride is = inst_stride(w);
    CSGS_LAUNCH(K_DRAW, draw, dim3((unsigned)((B + DRAW_BLOCK - 1) / DRAW_BLOCK), 1, nz), dim3(DRAW_BLOCK), st, cdf, stats,
                cand_cap, B, (uint32_t)seed, (uint32_t)(seed >> 32), iter, iter_dev, layer, w.hit, w.cbitmap, w.epoch, w.rank, w.member,
                n_nodes, is);
    CSGS_LAUNCH_CHECK();
    const int64_t cap_words = (cand_cap + 63) / 64;
    const int64_t hit_tiles = (cap_words + HIT_TILE_WORDS - 1) / HIT_TILE_WORDS;
    const unsigned hit_blocks = (unsigned)(hit_tiles < resident_grid(1) ? hit_tiles : resident_grid(1));
    CSGS_LAUNCH(K_HITS_FUSED, hits_fused, dim3(hit_blocks, 1, nz), dim3(256), st, cand_id, cdf, stats, cand_cap, n_nodes, B,
                w.epoch, w.hit_ts, w.hit_tiles, w.hit, w.cbitmap, w.rank, w.member, S_next, mult, p_incl, w.pdbl, n_next, status, is);
    CSGS_LAUNCH_CHECK();
    ws->has_draw = 1;
    ws->draw_B = B;
    ws->has_next = 0;   // offsets prepared for an earlier node set are void
    return CSGS_OK;
}

// rows == nullptr: reuse the row offsets that csgs_build_probs left in the workspace for the same rows
static int sampled_adjacency_impl(const csgs_graph *g, const int32_t *rows, int32_t n_rows, const int32_t *n_rows_dev,
                                  bool reuse_offsets,
                                  int32_t *adj_rowptr, int32_t *adj_col, float *adj_val, int64_t adj_cap,
                                  int64_t *adj_nnz, csgs_workspace *ws, int32_t *status, const RemoteArgs &rem,
                                  const int32_t *S_next, const int32_t *n_next, void *stream)
{
    if (!g || !g->rowptr || !g->colidx || !g->val || g->n_nodes <= 0 || g->n_nodes > 0x7FFFFFFFll || (!rows && !reuse_offsets) ||
        n_rows <= 0 ||
        !adj_rowptr || !adj_col || !adj_val || adj_cap <= 0 || !adj_nnz || !ws || !status)
        return CSGS_EINVAL;
    if (!ws->has_draw) return CSGS_EINVAL;  // no csgs_draw_nodes has run on this workspace
    Workspace w;
    const int rc = open_workspace(ws, g->n_nodes, n_rows, ws->draw_B, &w);
    if (rc != CSGS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const RowOffsets &cur = w.rows[ws->rows_buf & 1];
    if (!reuse_offsets) {
        const int rc2 = launch_row_prefix(g->rowptr, g->n_nodes, rows, n_rows, n_rows_dev, w, cur, status, st);
        if (rc2 != CSGS_OK) return rc2;
    }
    // prepare the other set of row offsets for the new node set, if it fits there
    NextRows nxt{};
    if (S_next && ws->draw_B <= ws->nS_max) {
        const RowOffsets &o = w.rows[(ws->rows_buf & 1) ^ 1];
        nxt = NextRows{g->rowptr, g->n_nodes, S_next, n_next, ws->draw_B, w.rp_ts, w.rp_tiles, o.eoff, o.rowstart, o.meta,
                       o.bound_note, w.chunk_cap * EDGE_TILE, (int32_t)((ws->draw_B + ROW_TILE - 1) / ROW_TILE)};
    }
    ws->has_next = nxt.blocks > 0;
    // after csgs_build_probs on the same rows the weight scan has left every chunk's row slice in the workspace
    const dim3 grid((unsigned)(resident_grid(2) + rem.blocks + nxt.blocks), 1, (unsigned)w.n_inst);
    const InstStride is = inst_stride(w);
    if (reuse_offsets)
        CSGS_LAUNCH(K_ADJ_FUSED, adj_fused<true>, grid, dim3(256), st, g->colidx, g->val, g->n_nodes,
                    g->nnz, cur.meta, cur.eoff, cur.rowstart, w.rank, w.member, w.pdbl, w.epoch, w.adj_ts, w.chunk_cap, cur.chunk_note,
                    adj_rowptr, adj_col, adj_val, adj_cap, adj_nnz, status, rem, nxt, is);
    else
        CSGS_LAUNCH(K_ADJ_FUSED, adj_fused<false>, grid, dim3(256), st, g->colidx, g->val, g->n_nodes,
                    g->nnz, cur.meta, cur.eoff, cur.rowstart, w.rank, w.member, w.pdbl, w.epoch, w.adj_ts, w.chunk_cap, cur.chunk_note,
                    adj_rowptr, adj_col, adj_val, adj_cap, adj_nnz, status, rem, nxt, is);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_sampled_adjacency(const csgs_graph *g, const int32_t *rows, int32_t n_rows,
                                      const int32_t *n_rows_dev, int32_t *adj_rowptr, int32_t *adj_col, float *adj_val, int64_t adj_cap, int64_t *adj_nnz,
                                      csgs_workspace *ws, int32_t *status, void *stream)
{
    return sampled_adjacency_impl(g, rows, n_rows, n_rows_dev, false, adj_rowptr, adj_col, adj_val, adj_cap, adj_nnz, ws, status,
                                  RemoteArgs{}, nullptr, nullptr, stream);
}

extern "C" int csgs_sample_layer(const csgs_graph *g, const int32_t *S, int32_t nS, const int32_t *cand_id,
                                 const uint64_t *cdf, int64_t cand_cap, const csgs_prob_stats *stats, int32_t B, uint64_t seed,
                                 uint64_t iter, const uint64_t *iter_dev, uint32_t layer, int32_t *S_next, int32_t *mult, float *p_incl,
                                 int32_t *n_next, int32_t *adj_rowptr, int32_t *adj_col, float *adj_val,
                                 int64_t adj_cap, int64_t *adj_nnz, const csgs_remote_out *remote,
                                 csgs_workspace *ws, int32_t *status, void *stream)
{
    if (!g || nS <= 0 || !adj_rowptr || !adj_col || !adj_val || adj_cap <= 0 || !adj_nnz) return CSGS_EINVAL;
    RemoteArgs rem{};
    if (remote) {
        if (!remote->remote_total || remote->local_lo > remote->local_hi ||
            (remote->per_part && (!remote->part_bounds || remote->P <= 0)))
            return CSGS_EINVAL;
        rem = RemoteArgs{S_next, n_next, remote->local_lo, remote->local_hi, remote->part_bounds,
                         remote->per_part ? remote->P : 0, remote->remote_total, remote->per_part, remote->src_row,
                         remote->remote_ids, REMOTE_BLOCKS};
    }
    const int rc = csgs_draw_nodes(g->n_nodes, cand_id, cdf, cand_cap, stats, B, seed, iter, iter_dev, layer, S_next, mult, p_incl,
                                   n_next, ws, status, stream);
    if (rc != CSGS_OK) return rc;
    return sampled_adjacency_impl(g, S, nS, nullptr, true, adj_rowptr, adj_col, adj_val, adj_cap, adj_nnz, ws, status, rem, S_next, n_next, stream);
}

extern "C" int csgs_remote_count(const int32_t *S_next, const int32_t *n_next, int32_t local_lo, int32_t local_hi,
                                 const int32_t *part_bounds, int32_t P, int64_t *remote_total, int64_t *per_part,
                                 int32_t *src_row, int32_t *remote_ids, void *stream)
{
    if (!S_next || !n_next || local_lo > local_hi || !remote_total) return CSGS_EINVAL;
    if (per_part && (!part_bounds || P <= 0)) return CSGS_EINVAL;
    // the element count is known only on the device; REMOTE_BLOCKS blocks of 256 cover the usual budgets
    // in one sweep and stride over larger ones
    const RemoteArgs rem{S_next, n_next, local_lo, local_hi, part_bounds, per_part ? P : 0, remote_total, per_part, src_row,
                         remote_ids, REMOTE_BLOCKS};
    CSGS_LAUNCH(K_REMOTE_COUNT, remote_count_k, dim3(REMOTE_BLOCKS), dim3(256), (hipStream_t)stream, rem);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}
