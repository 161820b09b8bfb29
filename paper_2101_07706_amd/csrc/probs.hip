// csgs_build_probs: importance weights over the neighbors of S_l (Section 4.1) and the skewed
// linear weighted sampling distribution (Section 4.2, Eq. 10) as an integer CDF.
//
// Kernels:
//   scan_edges     one wavefront per row of S: square each edge value exactly, round to the
//                  fixed-point grid, add into a per-node 64-bit accumulator with integer atomics
//                  (order-independent), mark first touches in a node bitmap
//   cand_partials  per tile of 1024 node ids: candidate count and weight sums
//   cand_scan      one block: exclusive scan of the tile partials, writes the stats
//   cand_emit      per tile: positions by bitmap popcount, inclusive wave scan of the skewed
//                  weights -> cand_id / cand_w / cdf / q; restores the accumulator and bitmap to zero
#include <math.h>
#include "common.hpp"

namespace csgs {

__global__ __launch_bounds__(256) void scan_edges(const int64_t *__restrict__ rowptr,
                                                  const int32_t *__restrict__ colidx,
                                                  const float *__restrict__ val, int64_t n_nodes,
                                                  const int32_t *__restrict__ S, int32_t nS, double scale,
                                                  uint64_t *__restrict__ wtable,
                                                  uint64_t *__restrict__ nbitmap,
                                                  int32_t *__restrict__ status)
{
    const int lane = lane_id();
    const int64_t row = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    if (row >= nS) return;
    const int32_t i = S[row];
    if (i < 0 || i >= n_nodes) {
        if (lane == 0) atomicOr(status, CSGS_ST_BAD_NODE_ID);
        return;
    }
    const int64_t beg = rowptr[i], end = rowptr[i + 1];
    bool bad = false;
    for (int64_t e = beg + lane; e < end; e += WAVE) {
        const int32_t c = colidx[e];
        const float v = val[e];
        if (!isfinite(v) || c < 0 || c >= n_nodes) {
            bad = true;
            continue;
        }
        const double sq = (double)v * (double)v;      // exact: 24 x 24 bit product
        long long x = __double2ll_rn(sq * scale);     // scale is a power of two: exact, then RNE
        if (x < 1) x = 1;                             // every candidate stays drawable
        const unsigned long long old = atomicAdd((unsigned long long *)&wtable[c], (unsigned long long)x);
        if (old == 0) atomicOr((unsigned long long *)&nbitmap[c >> 6], 1ull << (c & 63));
    }
    if (bad) atomicOr(status, CSGS_ST_BAD_EDGE_VALUE);
}

struct TileSums {
    uint32_t count, n_local;
    uint64_t wskew, wlocal, wremote;
};

// Loads the accumulator of node `id` if its bitmap bit is set.
__device__ inline uint64_t node_weight(const uint64_t *wtable, uint64_t word, int lane, int64_t id)
{
    return ((word >> lane) & 1ull) ? wtable[id] : 0ull;
}

__global__ __launch_bounds__(256) void cand_partials(const uint64_t *__restrict__ wtable,
                                                     const uint64_t *__restrict__ nbitmap, int64_t n_words,
                                                     int32_t lo, int32_t hi, uint64_t s_fx,
                                                     uint64_t *__restrict__ partial)
{
    __shared__ uint64_t lds[4][4];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    uint64_t cnt = 0, nloc = 0, wskew = 0, wloc = 0, wrem = 0;
    constexpr int WORDS = CAND_TILE / WAVE;  // 16 words per block, 4 per wave
    for (int k = 0; k < WORDS / 4; ++k) {
        const int64_t word_idx = (int64_t)blockIdx.x * WORDS + wave * (WORDS / 4) + k;
        if (word_idx >= n_words) break;
        const uint64_t word = nbitmap[word_idx];
        if (word == 0) continue;
        const int64_t id = word_idx * 64 + lane;
        const uint64_t w = node_weight(wtable, word, lane, id);
        const bool local = id >= lo && id < hi;
        if (w) {
            cnt += 1;
            if (local) { nloc += 1; wloc += w; wskew += w * s_fx; }
            else       { wrem += w; wskew += w * 16ull; }
        }
    }
    cnt = wave_sum(cnt); nloc = wave_sum(nloc); wskew = wave_sum(wskew);
    wloc = wave_sum(wloc); wrem = wave_sum(wrem);
    if (lane == 0) {
        lds[wave][0] = (cnt << 32) | nloc; lds[wave][1] = wskew; lds[wave][2] = wloc; lds[wave][3] = wrem;
    }
    __syncthreads();
    if (threadIdx.x < 4) {
        uint64_t a = lds[0][threadIdx.x], b = lds[1][threadIdx.x], c = lds[2][threadIdx.x], d = lds[3][threadIdx.x];
        partial[(int64_t)blockIdx.x * 4 + threadIdx.x] = a + b + c + d;  // count|nloc halves cannot carry: <= 1024 each
    }
}

__global__ __launch_bounds__(1024) void cand_scan(uint64_t *__restrict__ partial, int64_t n_tiles,
                                                  const int64_t *__restrict__ rowptr,
                                                  const int32_t *__restrict__ S, int32_t nS, int64_t n_nodes,
                                                  int32_t shift, int64_t cap, csgs_prob_stats *__restrict__ stats,
                                                  int32_t *__restrict__ status)
{
    __shared__ uint64_t lds[17];
    // running totals carried across chunks of 1024 tiles
    uint64_t base_cnt = 0, base_w = 0, tot_loc = 0, tot_wloc = 0, tot_wrem = 0;
    for (int64_t t0 = 0; t0 < n_tiles; t0 += blockDim.x) {
        const int64_t t = t0 + threadIdx.x;
        uint64_t cn = 0, wsk = 0, wl = 0, wr = 0;
        if (t < n_tiles) {
            cn = partial[t * 4 + 0]; wsk = partial[t * 4 + 1]; wl = partial[t * 4 + 2]; wr = partial[t * 4 + 3];
        }
        const uint64_t cnt = cn >> 32, nloc = cn & 0xFFFFFFFFull;
        uint64_t tot;
        const uint64_t ex_cnt = block_exclusive_scan<uint64_t>(cnt, lds, &tot);
        const uint64_t chunk_cnt = tot;
        const uint64_t ex_w = block_exclusive_scan<uint64_t>(wsk, lds, &tot);
        const uint64_t chunk_w = tot;
        block_exclusive_scan<uint64_t>(nloc, lds, &tot); tot_loc += tot;
        block_exclusive_scan<uint64_t>(wl, lds, &tot);   tot_wloc += tot;
        block_exclusive_scan<uint64_t>(wr, lds, &tot);   tot_wrem += tot;
        if (t < n_tiles) {
            partial[t * 4 + 0] = base_cnt + ex_cnt;   // candidates before this tile
            partial[t * 4 + 1] = base_w + ex_w;       // skewed weight before this tile
        }
        base_cnt += chunk_cnt;
        base_w += chunk_w;
    }
    // edges scanned = sum of the degrees of the rows of S
    uint64_t deg = 0;
    for (int32_t a = threadIdx.x; a < nS; a += blockDim.x) {
        const int32_t i = S[a];
        if (i >= 0 && i < n_nodes) deg += (uint64_t)(rowptr[i + 1] - rowptr[i]);
    }
    uint64_t edges;
    block_exclusive_scan<uint64_t>(deg, lds, &edges);
    if (threadIdx.x == 0) {
        stats->n_cand = (int64_t)base_cnt;
        stats->n_local = (int64_t)tot_loc;
        stats->n_remote = (int64_t)(base_cnt - tot_loc);
        stats->edges_scanned = (int64_t)edges;
        stats->w_local = tot_wloc;
        stats->w_remote = tot_wrem;
        stats->total = base_w;
        stats->shift = shift;
        stats->pad_ = 0;
        int32_t st = 0;
        if (base_cnt == 0) st |= CSGS_ST_EMPTY_CANDIDATES;
        if ((int64_t)base_cnt > cap) st |= CSGS_ST_CAND_OVERFLOW;
        if (st) atomicOr(status, st);
    }
}

__global__ __launch_bounds__(256) void cand_emit(uint64_t *__restrict__ wtable, uint64_t *__restrict__ nbitmap,
                                                 int64_t n_words, int32_t lo, int32_t hi, uint64_t s_fx,
                                                 const uint64_t *__restrict__ partial,
                                                 const csgs_prob_stats *__restrict__ stats,
                                                 int32_t *__restrict__ cand_id, uint64_t *__restrict__ cand_w,
                                                 uint64_t *__restrict__ cdf, float *__restrict__ q, int64_t cap)
{
    constexpr int WORDS = CAND_TILE / WAVE;  // 16
    __shared__ uint32_t s_cnt[WORDS];
    __shared__ uint64_t s_w[WORDS];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    uint64_t words[WORDS / 4], w[WORDS / 4], wsk_incl[WORDS / 4];
    // pass 1: per-word totals
#pragma unroll
    for (int k = 0; k < WORDS / 4; ++k) {
        const int slot = wave * (WORDS / 4) + k;
        const int64_t word_idx = (int64_t)blockIdx.x * WORDS + slot;
        uint64_t word = word_idx < n_words ? nbitmap[word_idx] : 0ull;
        const int64_t id = word_idx * 64 + lane;
        uint64_t wv = word ? node_weight(wtable, word, lane, id) : 0ull;
        const bool local = id >= lo && id < hi;
        const uint64_t wsk = wv * (local ? s_fx : 16ull);
        words[k] = word; w[k] = wv;
        wsk_incl[k] = wave_inclusive_scan(wsk);
        if (lane == WAVE - 1) { s_cnt[slot] = (uint32_t)__popcll(word); s_w[slot] = wsk_incl[k]; }
    }
    __syncthreads();
    // prefix over the 16 words of the tile (tiny: done redundantly by every thread)
    uint64_t base_cnt = partial[(int64_t)blockIdx.x * 4 + 0];
    uint64_t base_w = partial[(int64_t)blockIdx.x * 4 + 1];
    for (int s = 0; s < wave * (WORDS / 4); ++s) { base_cnt += s_cnt[s]; base_w += s_w[s]; }
    const double total = (double)stats->total;
#pragma unroll
    for (int k = 0; k < WORDS / 4; ++k) {
        const int slot = wave * (WORDS / 4) + k;
        const int64_t word_idx = (int64_t)blockIdx.x * WORDS + slot;
        const uint64_t word = words[k];
        if (word) {
            const int64_t id = word_idx * 64 + lane;
            const bool set = (word >> lane) & 1ull;
            const int64_t pos = (int64_t)base_cnt + __popcll(word & ((1ull << lane) - 1ull));
            if (set) {
                wtable[id] = 0ull;  // back to the clean state
                if (pos < cap) {
                    const bool local = id >= lo && id < hi;
                    cand_id[pos] = (int32_t)id;
                    cand_w[pos] = w[k];
                    cdf[pos] = base_w + wsk_incl[k];
                    if (q) q[pos] = (float)((double)(w[k] * (local ? s_fx : 16ull)) / total);
                }
            }
            if (lane == 0) nbitmap[word_idx] = 0ull;
        }
        base_cnt += s_cnt[slot];
        base_w += s_w[slot];
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

}  // namespace csgs

using namespace csgs;

extern "C" size_t csgs_workspace_bytes(int64_t n_nodes, int32_t nS_max, int32_t B_max)
{
    if (n_nodes <= 0 || nS_max <= 0 || B_max <= 0) return 0;
    return carve(nullptr, n_nodes, nS_max, B_max).bytes;
}

extern "C" size_t csgs_workspace_clean_bytes(int64_t n_nodes)
{
    if (n_nodes <= 0) return 0;
    const Workspace w = carve(nullptr, n_nodes, 1, 1);
    return (size_t)((char *)w.partial - (char *)nullptr);
}

extern "C" int csgs_workspace_init(void *ws, size_t ws_bytes, void *stream)
{
    if (!ws || ws_bytes == 0 || ((uintptr_t)ws & 255) || (ws_bytes & 7)) return CSGS_EINVAL;
    const size_t n = ws_bytes / 8;
    const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    CSGS_LAUNCH(K_FILL_ZERO, fill_zero, dim3(blocks), dim3(256), (hipStream_t)stream, (uint64_t *)ws, n);
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
    int e_r = 0;
    while (e_r < 64 && ldexp(1.0, e_r) < (double)rownorm2_max) ++e_r;
    int sh = 61 - ceil_log2_u64((uint64_t)nS) - ceil_log2_u64((uint64_t)sfx) - e_r;
    if (sh > 52) sh = 52;
    if (shift) *shift = sh;
    if (s_fx) *s_fx = sfx;
    return sh < 24 ? CSGS_ERANGE : CSGS_OK;
}

extern "C" int csgs_build_probs(const csgs_graph *g, const int32_t *S, int32_t nS, float skew, int32_t *cand_id,
                                uint64_t *cand_w, uint64_t *cdf, float *q, int64_t cap, csgs_prob_stats *stats,
                                void *ws, size_t ws_bytes, int32_t *status, void *stream)
{
    if (!g || !g->rowptr || !g->colidx || !g->val || g->n_nodes <= 0 || g->n_nodes > 0x7FFFFFFFll ||
        g->local_lo > g->local_hi || !S || nS <= 0 || !cand_id || !cand_w || !cdf || cap <= 0 || !stats || !ws ||
        !status || ((uintptr_t)ws & 255))
        return CSGS_EINVAL;
    int32_t shift;
    int64_t s_fx;
    int rc = csgs_fixed_point(nS, skew, g->rownorm2_max, &shift, &s_fx);
    if (rc != CSGS_OK) return rc;
    Workspace w = carve(ws, g->n_nodes, nS, 1);
    if (w.bytes > ws_bytes) return CSGS_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const int64_t n_words = (g->n_nodes + 63) / 64;
    const int64_t n_tiles = (g->n_nodes + CAND_TILE - 1) / CAND_TILE;

    const int64_t scan_blocks = ((int64_t)nS * WAVE + 255) / 256;
    CSGS_LAUNCH(K_SCAN_EDGES, scan_edges, dim3((unsigned)scan_blocks), dim3(256), st, g->rowptr, g->colidx, g->val,
                       g->n_nodes, S, nS, ldexp(1.0, shift), w.wtable, w.nbitmap, status);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_CAND_PARTIALS, cand_partials, dim3((unsigned)n_tiles), dim3(256), st, w.wtable, w.nbitmap, n_words,
                       g->local_lo, g->local_hi, (uint64_t)s_fx, w.partial);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_CAND_SCAN, cand_scan, dim3(1), dim3(1024), st, w.partial, n_tiles, g->rowptr, S, nS, g->n_nodes,
                       shift, cap, stats, status);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_CAND_EMIT, cand_emit, dim3((unsigned)n_tiles), dim3(256), st, w.wtable, w.nbitmap, n_words,
                       g->local_lo, g->local_hi, (uint64_t)s_fx, w.partial, stats, cand_id, cand_w, cdf, q, cap);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}
