// csgs_build_probs: importance weights over the neighbors of S_l (Section 4.1) and the skewed
// linear weighted sampling distribution (Section 4.2, Eq. 10) as an integer CDF.
//
// Kernels:
//   row_prefix     one block: degrees of the rows of S, their exclusive prefix (the flat edge
//                  numbering), CSR start of every row, total edges
//   scan_edges     flat over the edges of S (chunks of 1024, rows of a chunk staged in LDS, so
//                  hub rows and short rows cost the same per edge): square each edge value
//                  exactly, round to the fixed-point grid, add into a per-node 64-bit accumulator
//                  with fire-and-forget integer atomics (order-independent); flag the 64-node
//                  word of the target with a plain byte store
//   cand_fused     per tile of 1024 node ids, single pass: candidate count and weight sums of the
//                  flagged words, prefix over earlier tiles by decoupled look-back, positions by
//                  ballot popcount, inclusive wave scan of the skewed weights -> cand_id / cand_w /
//                  cdf; restores accumulator and flags to zero; the last tile writes the stats
//   fill_q         only when q is requested: skewed weight / total (the total is known only after
//                  the last tile)
#include <math.h>
#include "common.hpp"
#include "lookback.hpp"

namespace csgs {

constexpr int RP_ITEMS = 8;  // rows per thread and round in row_prefix

__global__ __launch_bounds__(1024) void row_prefix(const int64_t *__restrict__ rowptr, int64_t n_nodes,
                                                   const int32_t *__restrict__ S, int32_t nS,
                                                   int64_t *__restrict__ eoff, int64_t *__restrict__ rowstart,
                                                   int64_t edge_cap, csgs_prob_stats *__restrict__ stats,
                                                   int32_t *__restrict__ status)
{
    __shared__ int64_t lds[17];
    __shared__ int32_t s_deg[1024 * RP_ITEMS];
    bool bad = false;
    int64_t base = 0;
    // rounds of 8192 rows: degrees are fetched striped (coalesced, all loads independent), handed
    // through LDS to a blocked arrangement, and scanned with one block scan per round
    for (int32_t r0 = 0; r0 < nS; r0 += 1024 * RP_ITEMS) {
        __syncthreads();
#pragma unroll
        for (int k = 0; k < RP_ITEMS; ++k) {
            const int32_t a = r0 + k * 1024 + (int32_t)threadIdx.x;
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
            s_deg[k * 1024 + threadIdx.x] = (int32_t)deg;
        }
        __syncthreads();
        int32_t d[RP_ITEMS];
        int64_t sum = 0;
#pragma unroll
        for (int k = 0; k < RP_ITEMS; ++k) {
            d[k] = s_deg[threadIdx.x * RP_ITEMS + k];
            sum += d[k];
        }
        int64_t total;
        int64_t ex = base + block_exclusive_scan<int64_t>(sum, lds, &total);
#pragma unroll
        for (int k = 0; k < RP_ITEMS; ++k) {
            const int32_t a = r0 + (int32_t)threadIdx.x * RP_ITEMS + k;
            if (a < nS) eoff[a] = ex;
            ex += d[k];
        }
        base += total;
    }
    if (bad) atomicOr(status, CSGS_ST_BAD_NODE_ID);
    if (threadIdx.x == 0) {
        stats->edges_scanned = base;
        // an edge count the workspace cannot hold is reported and treated as empty
        if (base > edge_cap) {
            atomicOr(status, CSGS_ST_EDGE_OVERFLOW);
            base = 0;
        }
        eoff[nS] = base;
    }
}

__global__ __launch_bounds__(256) void scan_edges(const int32_t *__restrict__ colidx, const float *__restrict__ val,
                                                  int64_t n_nodes, int32_t nS, const int64_t *__restrict__ eoff,
                                                  const int64_t *__restrict__ rowstart, double scale,
                                                  uint64_t *__restrict__ wtable, uint8_t *__restrict__ tileflag,
                                                  int32_t *__restrict__ status)
{
    __shared__ RowSlice slice;
    const int64_t E = eoff[nS];
    bool bad = false;
    for (int64_t c0 = (int64_t)blockIdx.x * EDGE_TILE; c0 < E; c0 += (int64_t)gridDim.x * EDGE_TILE) {
        const int64_t c1 = (c0 + EDGE_TILE < E) ? c0 + EDGE_TILE : E;
        stage_slice(slice, eoff, rowstart, nS, c0, c1);
        const int32_t len = (int32_t)(c1 - c0);
#pragma unroll
        for (int k = 0; k < EDGE_TILE / 256; ++k) {
            const int32_t x = (int32_t)threadIdx.x + k * 256;
            if (x >= len) break;
            int32_t r;
            const int64_t e = edge_address(slice, eoff, rowstart, c0, x, &r);
            const int32_t c = colidx[e];
            const float v = val[e];
            if (!isfinite(v) || c < 0 || c >= n_nodes) {
                bad = true;
                continue;
            }
            const double sq = (double)v * (double)v;      // exact: 24 x 24 bit product
            long long q = __double2ll_rn(sq * scale);     // scale is a power of two: exact, then RNE
            if (q < 1) q = 1;                             // every candidate stays drawable
            (void)__hip_atomic_fetch_add((unsigned long long *)&wtable[c], (unsigned long long)q, __ATOMIC_RELAXED,
                                         __HIP_MEMORY_SCOPE_AGENT);
            tileflag[c >> 6] = 1;  // same value from every writer
        }
    }
    if (bad) atomicOr(status, CSGS_ST_BAD_EDGE_VALUE);
}

__global__ __launch_bounds__(256) void cand_fused(uint64_t *__restrict__ wtable, uint8_t *__restrict__ tileflag,
                                                  int64_t n_words, int64_t n_nodes, int64_t n_tiles, int32_t lo,
                                                  int32_t hi, uint64_t s_fx, unsigned long long tag,
                                                  uint64_t *__restrict__ ts_mem, int32_t shift,
                                                  csgs_prob_stats *__restrict__ stats, int32_t *__restrict__ status,
                                                  int32_t *__restrict__ cand_id, uint64_t *__restrict__ cand_w,
                                                  uint64_t *__restrict__ cdf, int64_t cap)
{
    constexpr int WORDS = CAND_TILE / WAVE;  // 16 words per tile, 4 per wave
    __shared__ uint32_t s_cnt[WORDS];
    __shared__ uint64_t s_w[WORDS];
    __shared__ uint64_t s_aux[4][3];
    __shared__ unsigned long long s_lb[4];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const TileState<4> ts(ts_mem, n_tiles);
    // one tile per block (the loop also covers a smaller, fully resident grid)
    for (int64_t t = blockIdx.x; t < n_tiles; t += gridDim.x) {
        uint64_t words[WORDS / 4], w[WORDS / 4], wsk_incl[WORDS / 4];
        uint64_t nloc = 0, wl = 0, wr = 0;
#pragma unroll
        for (int k = 0; k < WORDS / 4; ++k) {
            const int slot = wave * (WORDS / 4) + k;
            const int64_t word_idx = t * WORDS + slot;
            const bool flagged = word_idx < n_words && tileflag[word_idx] != 0;
            const int64_t id = word_idx * 64 + lane;
            const uint64_t wv = (flagged && id < n_nodes) ? wtable[id] : 0ull;
            const bool local = id >= lo && id < hi;
            const uint64_t wsk = wv * (local ? s_fx : 16ull);
            if (wv) {
                if (local) { nloc += 1; wl += wv; } else { wr += wv; }
            }
            words[k] = __ballot(wv != 0);
            w[k] = wv;
            wsk_incl[k] = wave_inclusive_scan(wsk);
            if (lane == WAVE - 1) { s_cnt[slot] = (uint32_t)__popcll(words[k]); s_w[slot] = wsk_incl[k]; }
            if (flagged && lane == 0) tileflag[word_idx] = 0;  // back to the clean state
        }
        nloc = wave_sum(nloc); wl = wave_sum(wl); wr = wave_sum(wr);
        if (lane == 0) { s_aux[wave][0] = nloc; s_aux[wave][1] = wl; s_aux[wave][2] = wr; }
        __syncthreads();
        // tile totals (tiny: computed redundantly by every thread)
        uint64_t tile_cnt = 0, tile_w = 0, my_cnt = 0, my_w = 0;
        for (int sl = 0; sl < WORDS; ++sl) {
            if (sl == wave * (WORDS / 4)) { my_cnt = tile_cnt; my_w = tile_w; }
            tile_cnt += s_cnt[sl]; tile_w += s_w[sl];
        }
        unsigned long long local[4], excl[4];
        local[0] = (tile_cnt << 32) | (s_aux[0][0] + s_aux[1][0] + s_aux[2][0] + s_aux[3][0]);  // both halves stay below 2^31
        local[1] = tile_w;
        local[2] = s_aux[0][1] + s_aux[1][1] + s_aux[2][1] + s_aux[3][1];
        local[3] = s_aux[0][2] + s_aux[1][2] + s_aux[2][2] + s_aux[3][2];
        lookback<4>(ts, tag, t, n_tiles, local, excl, s_lb, status);
        uint64_t base_cnt = (excl[0] >> 32) + my_cnt;
        uint64_t base_w = excl[1] + my_w;
#pragma unroll
        for (int k = 0; k < WORDS / 4; ++k) {
            const int slot = wave * (WORDS / 4) + k;
            const int64_t word_idx = t * WORDS + slot;
            const uint64_t word = words[k];
            if (word) {
                const int64_t id = word_idx * 64 + lane;
                const bool set = (word >> lane) & 1ull;
                const int64_t pos = (int64_t)base_cnt + __popcll(word & ((1ull << lane) - 1ull));
                if (set) {
                    wtable[id] = 0ull;  // back to the clean state
                    if (pos < cap) {
                        cand_id[pos] = (int32_t)id;
                        cand_w[pos] = w[k];
                        cdf[pos] = base_w + wsk_incl[k];
                    }
                }
            }
            base_cnt += s_cnt[slot];
            base_w += s_w[slot];
        }
        if (t == n_tiles - 1 && threadIdx.x == 0) {
            const uint64_t tot_cnt = (excl[0] >> 32) + tile_cnt;
            const uint64_t tot_loc = (excl[0] & 0xFFFFFFFFull) + (local[0] & 0xFFFFFFFFull);
            stats->n_cand = (int64_t)tot_cnt;
            stats->n_local = (int64_t)tot_loc;
            stats->n_remote = (int64_t)(tot_cnt - tot_loc);
            stats->w_local = excl[2] + local[2];
            stats->w_remote = excl[3] + local[3];
            stats->total = excl[1] + tile_w;
            stats->shift = shift;
            stats->pad_ = 0;
            int32_t st = 0;
            if (tot_cnt == 0) st |= CSGS_ST_EMPTY_CANDIDATES;
            if ((int64_t)tot_cnt > cap) st |= CSGS_ST_CAND_OVERFLOW;
            if (st) atomicOr(status, st);
        }
        __syncthreads();  // the shared arrays are reused by the next tile
    }
}

__global__ __launch_bounds__(256) void fill_q(const uint64_t *__restrict__ cdf,
                                              const csgs_prob_stats *__restrict__ stats, int64_t cap,
                                              float *__restrict__ q)
{
    int64_t n = stats->n_cand;
    if (n > cap) n = cap;
    const double total = (double)stats->total;
    for (int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; k < n; k += (int64_t)gridDim.x * blockDim.x) {
        const uint64_t wsk = cdf[k] - (k ? cdf[k - 1] : 0ull);
        q[k] = (float)((double)wsk / total);
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
    ws->epoch = 0;
    Workspace w;
    const int rc = open_workspace(ws, ws->n_nodes, 1, 1, &w);
    if (rc != CSGS_OK) return rc;
    const size_t n = w.bytes / 8;
    const int blocks = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
    CSGS_LAUNCH(K_FILL_ZERO, fill_zero, dim3(blocks), dim3(256), (hipStream_t)stream, (uint64_t *)ws->base, n);
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
                                csgs_workspace *ws, int32_t *status, void *stream)
{
    if (!g || !g->rowptr || !g->colidx || !g->val || g->n_nodes <= 0 || g->n_nodes > 0x7FFFFFFFll ||
        g->local_lo > g->local_hi || !S || nS <= 0 || !cand_id || !cand_w || !cdf || cap <= 0 || !stats || !ws || !status)
        return CSGS_EINVAL;
    int32_t shift;
    int64_t s_fx;
    int rc = csgs_fixed_point(nS, skew, g->rownorm2_max, &shift, &s_fx);
    if (rc != CSGS_OK) return rc;
    Workspace w;
    rc = open_workspace(ws, g->n_nodes, nS, 1, &w);
    if (rc != CSGS_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int64_t n_words = (g->n_nodes + 63) / 64;

    CSGS_LAUNCH(K_ROW_PREFIX, row_prefix, dim3(1), dim3(1024), st, g->rowptr, g->n_nodes, S, nS, w.eoff, w.rowstart,
                w.chunk_cap * EDGE_TILE, stats, status);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_SCAN_EDGES, scan_edges, dim3(EDGE_GRID), dim3(256), st, g->colidx, g->val, g->n_nodes, nS, w.eoff,
                w.rowstart, ldexp(1.0, shift), w.wtable, w.tileflag, status);
    CSGS_LAUNCH_CHECK();
    const unsigned long long tag = ++ws->epoch;
    const int64_t cand_grid = w.n_tiles;  // one tile per block, dispatched in ascending order
    CSGS_LAUNCH(K_CAND_FUSED, cand_fused, dim3((unsigned)cand_grid), dim3(256), st, w.wtable, w.tileflag, n_words,
                g->n_nodes, w.n_tiles, g->local_lo, g->local_hi, (uint64_t)s_fx, tag, w.cand_ts, shift, stats, status,
                cand_id, cand_w, cdf, cap);
    CSGS_LAUNCH_CHECK();
    if (q) {
        const int64_t qn = cap < g->n_nodes ? cap : g->n_nodes;
        const unsigned qb = (unsigned)((qn + 255) / 256 < 2048 ? (qn + 255) / 256 : 2048);
        CSGS_LAUNCH(K_FILL_Q, fill_q, dim3(qb), dim3(256), st, cdf, stats, cap, q);
        CSGS_LAUNCH_CHECK();
    }
    return CSGS_OK;
}
