// csgs_sample_layer and csgs_remote_count.
//
// B draws with replacement from the skewed distribution (Section 4.1: the sampling is run B
// times), deduplicated; inclusion probability p_j = 1 - (1 - q_j)^B (Eq. 8); sampled adjacency
// with every kept edge divided by p_j (Eq. 3); number of sampled remote nodes (Eq. 4).
//
// Kernels:
//   draw          one thread per draw: Philox4x32-10 word -> u = mulhi(r, total) -> first cdf
//                 entry above u.  The top levels of the search run on a strided sample of the
//                 CDF staged in LDS, the rest on the global array.  Hits are counted per
//                 candidate position with integer atomics; first hits set a position bitmap.
//   compact_hits  one block: bitmap -> ordered list of hit positions, then one thread per distinct
//                 hit: S_next ascending, mult, p_incl, node -> rank table
//   adj_flag      flat over the edges of S (same chunking as the weight scan): keep = the target
//                 was sampled; keep bits per 64 edges and the kept count per chunk
//   adj_scan      one block: exclusive scan of the chunk counts
//   adj_emit      flat again: the kept edges in flat order ARE the CSR of P~ (rows in the order
//                 of S, columns ascending), so position = chunk base + popcount of earlier keep
//                 bits; row pointers are the positions at the row starts
//   rank_clear    restores the rank table
//   remote_count  one block
#include <math.h>
#include "common.hpp"

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

constexpr int DRAW_BLOCK = 1024;
constexpr int TOP = 4096;  // CDF samples staged in LDS per block (32 KB)

__global__ __launch_bounds__(DRAW_BLOCK) void draw(const uint64_t *__restrict__ cdf,
                                                   const csgs_prob_stats *__restrict__ stats, int64_t cand_cap,
                                                   int32_t B, uint32_t seed_lo, uint32_t seed_hi, uint32_t iter_lo,
                                                   uint32_t iter_hi, uint32_t layer, uint32_t *__restrict__ hit,
                                                   uint64_t *__restrict__ cbitmap)
{
    __shared__ uint64_t top[TOP];
    int64_t n = stats->n_cand;
    if (n > cand_cap) n = cand_cap;
    if (n <= 0) return;
    const uint64_t total = cdf[n - 1];
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
    int64_t hi = (a < n_top) ? (a + 1) * stride - 1 : n - 1;  // cdf[hi] > u is known
    while (lo < hi) {
        const int64_t m = (lo + hi) >> 1;
        if (cdf[m] > u) hi = m; else lo = m + 1;
    }
    const uint32_t old = atomicAdd(&hit[lo], 1u);
    if (old == 0) atomicOr((unsigned long long *)&cbitmap[lo >> 6], 1ull << (lo & 63));
}

__global__ __launch_bounds__(1024) void compact_hits(const int32_t *__restrict__ cand_id,
                                                     const uint64_t *__restrict__ cdf,
                                                     const csgs_prob_stats *__restrict__ stats, int64_t cand_cap,
                                                     int64_t n_nodes, int32_t B, uint32_t *__restrict__ hit,
                                                     uint64_t *__restrict__ cbitmap, int32_t *__restrict__ rank,
                                                     int32_t *__restrict__ hitpos, int32_t *__restrict__ S_next,
                                                     int32_t *__restrict__ mult, float *__restrict__ p_incl,
                                                     double *__restrict__ pdbl, int32_t *__restrict__ n_next)
{
    __shared__ uint32_t lds[17];
    int64_t n = stats->n_cand;
    if (n > cand_cap) n = cand_cap;
    if (n < 0) n = 0;
    const int64_t n_words = (n + 63) / 64;
    const double total = n > 0 ? (double)cdf[n - 1] : 1.0;
    // phase 1: contiguous run of words per thread, so that list order = ascending position
    const int64_t per = (n_words + blockDim.x - 1) / blockDim.x;
    const int64_t w0 = (int64_t)threadIdx.x * per;
    const int64_t w1 = (w0 + per < n_words) ? w0 + per : n_words;
    uint32_t cnt = 0;
    for (int64_t w = w0; w < w1; ++w) cnt += (uint32_t)__popcll(cbitmap[w]);
    uint32_t tot;
    uint32_t pos = block_exclusive_scan<uint32_t>(cnt, lds, &tot);
    if (cnt) {
        for (int64_t w = w0; w < w1; ++w) {
            uint64_t word = cbitmap[w];
            if (!word) continue;
            cbitmap[w] = 0ull;
            while (word) {
                const int bit = __ffsll((unsigned long long)word) - 1;
                word &= word - 1;
                if (pos < (uint32_t)B) hitpos[pos] = (int32_t)(w * 64 + bit);  // at most B distinct hits exist
                ++pos;
            }
        }
    }
    __syncthreads();  // hitpos (global) written above is read by other threads of this block below
    const uint32_t n_hit = tot < (uint32_t)B ? tot : (uint32_t)B;
    // phase 2: one thread per distinct hit
    for (uint32_t r = threadIdx.x; r < n_hit; r += blockDim.x) {
        const int64_t k = hitpos[r];
        const uint32_t m = hit[k];
        hit[k] = 0u;
        const uint64_t wk = cdf[k] - (k ? cdf[k - 1] : 0ull);
        const double qk = (double)wk / total;
        const double pk = (qk >= 1.0) ? 1.0 : -expm1((double)B * log1p(-qk));
        const int32_t id = cand_id[k];
        S_next[r] = id;
        mult[r] = (int32_t)m;
        p_incl[r] = (float)pk;
        pdbl[r] = pk;
        if (id >= 0 && id < n_nodes) rank[id] = (int32_t)r + 1;
    }
    if (threadIdx.x == 0) *n_next = (int32_t)n_hit;
}

__global__ __launch_bounds__(256) void adj_flag(const int32_t *__restrict__ colidx, int64_t n_nodes, int32_t nS,
                                                const int64_t *__restrict__ eoff,
                                                const int64_t *__restrict__ rowstart,
                                                const int32_t *__restrict__ rank, int64_t edge_cap,
                                                uint64_t *__restrict__ keepmask, int64_t *__restrict__ chunkcnt,
                                                int32_t *__restrict__ status)
{
    __shared__ RowSlice slice;
    __shared__ int32_t wave_cnt[4];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t E = eoff[nS];
    if (E > edge_cap) {  // the per-edge scratch cannot hold this step
        if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(status, CSGS_ST_EDGE_OVERFLOW);
        return;
    }
    for (int64_t c0 = (int64_t)blockIdx.x * EDGE_TILE; c0 < E; c0 += (int64_t)gridDim.x * EDGE_TILE) {
        const int64_t c1 = (c0 + EDGE_TILE < E) ? c0 + EDGE_TILE : E;
        stage_slice(slice, eoff, rowstart, nS, c0, c1);
        const int32_t len = (int32_t)(c1 - c0);
        int32_t cnt = 0;
        // wave w owns positions [w * 256, w * 256 + 256): four 64-edge words
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int32_t x = wave * 256 + k * 64 + lane;
            bool keep = false;
            if (x < len) {
                int32_t r;
                const int64_t e = edge_address(slice, eoff, rowstart, c0, x, &r);
                const int32_t c = colidx[e];
                keep = c >= 0 && c < n_nodes && rank[c] != 0;
            }
            const uint64_t m = __ballot(keep);
            if (lane == 0) keepmask[(c0 >> 6) + wave * 4 + k] = m;
            cnt += __popcll(m);
        }
        if (lane == 0) wave_cnt[wave] = cnt;
        __syncthreads();
        if (threadIdx.x == 0) chunkcnt[c0 / EDGE_TILE] = (int64_t)(wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3]);
    }
}

// chunkbase[c] holds the kept count of chunk c on entry and the exclusive prefix on exit.
__global__ __launch_bounds__(1024) void adj_scan(int64_t *__restrict__ chunkbase, int32_t nS,
                                                 const int64_t *__restrict__ eoff, int64_t edge_cap,
                                                 int32_t *__restrict__ adj_rowptr, int64_t adj_cap,
                                                 int64_t *__restrict__ adj_nnz, int32_t *__restrict__ status)
{
    __shared__ int64_t lds[17];
    int64_t E = eoff[nS];
    if (E > edge_cap) E = 0;
    const int64_t n_chunks = (E + EDGE_TILE - 1) / EDGE_TILE;
    const int64_t per = (n_chunks + blockDim.x - 1) / blockDim.x;
    const int64_t t0 = (int64_t)threadIdx.x * per;
    const int64_t t1 = (t0 + per < n_chunks) ? t0 + per : n_chunks;
    int64_t sum = 0;
    for (int64_t t = t0; t < t1; ++t) sum += chunkbase[t];
    int64_t total;
    int64_t ex = block_exclusive_scan<int64_t>(sum, lds, &total);
    for (int64_t t = t0; t < t1; ++t) {
        const int64_t c = chunkbase[t];
        chunkbase[t] = ex;
        ex += c;
    }
    // rows that start at or after the last edge (trailing empty rows, and the end pointer)
    const int32_t clamp = (int32_t)(total < 0x7FFFFFFFll ? total : 0x7FFFFFFFll);
    const int64_t first_tail = E > 0 ? lower_bound_i64(eoff, (int64_t)nS + 1, E) : 0;
    for (int64_t a = first_tail + threadIdx.x; a <= nS; a += blockDim.x) adj_rowptr[a] = clamp;
    if (threadIdx.x == 0) {
        *adj_nnz = total;
        if (total > adj_cap || total > 0x7FFFFFFFll) atomicOr(status, CSGS_ST_ADJ_OVERFLOW);
    }
}

__global__ __launch_bounds__(256) void adj_emit(const int32_t *__restrict__ colidx, const float *__restrict__ val,
                                                int32_t nS, const int64_t *__restrict__ eoff,
                                                const int64_t *__restrict__ rowstart,
                                                const int32_t *__restrict__ rank, const double *__restrict__ pdbl,
                                                int64_t edge_cap, const uint64_t *__restrict__ keepmask,
                                                const int64_t *__restrict__ chunkbase,
                                                int32_t *__restrict__ adj_rowptr, int32_t *__restrict__ adj_col,
                                                float *__restrict__ adj_val, int64_t adj_cap)
{
    __shared__ RowSlice slice;
    __shared__ uint64_t s_mask[EDGE_TILE / 64];
    __shared__ int32_t s_pre[EDGE_TILE / 64 + 1];
    const int lane = lane_id();
    const int wave = (int)(threadIdx.x >> 6);
    const int64_t E = eoff[nS];
    if (E > edge_cap) return;
    for (int64_t c0 = (int64_t)blockIdx.x * EDGE_TILE; c0 < E; c0 += (int64_t)gridDim.x * EDGE_TILE) {
        const int64_t c1 = (c0 + EDGE_TILE < E) ? c0 + EDGE_TILE : E;
        stage_slice(slice, eoff, rowstart, nS, c0, c1);
        if (threadIdx.x < EDGE_TILE / 64) s_mask[threadIdx.x] = keepmask[(c0 >> 6) + threadIdx.x];
        __syncthreads();
        if (threadIdx.x == 0) {
            int32_t acc = 0;
            for (int i = 0; i < EDGE_TILE / 64; ++i) { s_pre[i] = acc; acc += __popcll(s_mask[i]); }
            s_pre[EDGE_TILE / 64] = acc;
        }
        __syncthreads();
        const int64_t base = chunkbase[c0 / EDGE_TILE];
        const int32_t len = (int32_t)(c1 - c0);
        // row pointers of the rows that start inside this chunk: kept edges before the row start
        const int32_t R = slice.R;
        const int64_t a_first = slice.a_first;
        for (int32_t r = threadIdx.x; r < R; r += blockDim.x) {
            const int64_t off = slice.in_lds ? (int64_t)slice.off[r] : eoff[a_first + r] - c0;
            if (off >= 0 && off < len) {
                const int64_t v = base + s_pre[off >> 6] + __popcll(s_mask[off >> 6] & ((1ull << (off & 63)) - 1ull));
                adj_rowptr[a_first + r] = (int32_t)(v < 0x7FFFFFFFll ? v : 0x7FFFFFFFll);
            }
        }
        if (s_pre[EDGE_TILE / 64] == 0) continue;  // nothing kept in this chunk (uniform over the block)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int32_t word = wave * 4 + k;
            const uint64_t m = s_mask[word];
            if (!((m >> lane) & 1ull)) continue;
            const int32_t x = word * 64 + lane;
            int32_t r;
            const int64_t e = edge_address(slice, eoff, rowstart, c0, x, &r);
            const int64_t pos = base + s_pre[word] + __popcll(m & ((1ull << lane) - 1ull));
            const int32_t rk = rank[colidx[e]];
            if (pos < adj_cap && rk > 0) {
                adj_col[pos] = rk - 1;
                adj_val[pos] = (float)((double)val[e] / pdbl[rk - 1]);
            }
        }
    }
}

__global__ void rank_clear(const int32_t *__restrict__ S_next, const int32_t *__restrict__ n_next, int32_t B,
                           int64_t n_nodes, int32_t *__restrict__ rank)
{
    int32_t n = *n_next;
    if (n > B) n = B;
    for (int32_t k = blockIdx.x * blockDim.x + threadIdx.x; k < n; k += gridDim.x * blockDim.x) {
        const int32_t id = S_next[k];
        if (id >= 0 && id < n_nodes) rank[id] = 0;
    }
}

__global__ __launch_bounds__(1024) void remote_count_k(const int32_t *__restrict__ S_next,
                                                       const int32_t *__restrict__ n_next, int32_t lo, int32_t hi,
                                                       const int32_t *__restrict__ part_bounds, int32_t P,
                                                       int64_t *__restrict__ remote_total,
                                                       int64_t *__restrict__ per_part, int32_t *__restrict__ src_row,
                                                       int32_t *__restrict__ remote_ids)
{
    __shared__ uint32_t lds[17];
    const int32_t n = *n_next;
    // every thread owns a contiguous run of the (ascending) sampled ids: one block scan in total
    const int32_t per = (n + (int32_t)blockDim.x - 1) / (int32_t)blockDim.x;
    const int32_t k0 = (int32_t)threadIdx.x * per;
    const int32_t k1 = (k0 + per < n) ? k0 + per : n;
    uint32_t rem = 0;
    for (int32_t k = k0; k < k1; ++k) {
        const int32_t j = S_next[k];
        rem += (j < lo || j >= hi) ? 1u : 0u;
    }
    uint32_t tot;
    uint32_t ex = block_exclusive_scan<uint32_t>(rem, lds, &tot);
    if (src_row || remote_ids) {
        for (int32_t k = k0; k < k1; ++k) {
            const int32_t j = S_next[k];
            if (j < lo || j >= hi) {
                if (src_row) src_row[k] = -1 - (int32_t)ex;
                if (remote_ids) remote_ids[ex] = j;
                ++ex;
            } else if (src_row) {
                src_row[k] = j - lo;
            }
        }
    }
    if (threadIdx.x == 0) *remote_total = (int64_t)tot;
    // S_next ascends, so partition p holds the ids between two lower bounds
    if (per_part) {
        for (int p = threadIdx.x; p < P; p += blockDim.x) {
            int32_t cut[2];
            for (int s = 0; s < 2; ++s) {
                const int32_t key = part_bounds[p + s];
                int32_t a = 0, b = n;
                while (a < b) {
                    const int32_t m = (a + b) >> 1;
                    if (S_next[m] >= key) b = m; else a = m + 1;
                }
                cut[s] = a;
            }
            per_part[p] = (int64_t)(cut[1] > cut[0] ? cut[1] - cut[0] : 0);
        }
    }
}

}  // namespace csgs

using namespace csgs;

extern "C" int csgs_sample_layer(const csgs_graph *g, const int32_t *S, int32_t nS, const int32_t *cand_id,
                                 const uint64_t *cdf, int64_t cand_cap, const csgs_prob_stats *stats, int32_t B, uint64_t seed,
                                 uint64_t iter, uint32_t layer, int32_t *S_next, int32_t *mult, float *p_incl,
                                 int32_t *n_next, int32_t *adj_rowptr, int32_t *adj_col, float *adj_val,
                                 int64_t adj_cap, int64_t *adj_nnz, void *ws, size_t ws_bytes, int32_t *status,
                                 void *stream)
{
    if (!g || !g->rowptr || !g->colidx || !g->val || g->n_nodes <= 0 || g->n_nodes > 0x7FFFFFFFll || !S || nS <= 0 ||
        !cand_id || !cdf || cand_cap <= 0 || !stats || B <= 0 || !S_next || !mult || !p_incl || !n_next || !adj_rowptr || !adj_col ||
        !adj_val || adj_cap <= 0 || !adj_nnz || !ws || !status || ((uintptr_t)ws & 255))
        return CSGS_EINVAL;
    Workspace w = carve(ws, g->n_nodes, nS, B, ws_bytes, 0);
    if (w.fixed_bytes > ws_bytes || w.edge_cap < EDGE_TILE) return CSGS_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    if (cand_cap > g->n_nodes) cand_cap = g->n_nodes;  // there are never more candidates than nodes

    CSGS_LAUNCH(K_DRAW, draw, dim3((unsigned)((B + DRAW_BLOCK - 1) / DRAW_BLOCK)), dim3(DRAW_BLOCK), st, cdf, stats,
                cand_cap, B, (uint32_t)seed, (uint32_t)(seed >> 32), (uint32_t)iter, (uint32_t)(iter >> 32), layer, w.hit,
                w.cbitmap);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_COMPACT_HITS, compact_hits, dim3(1), dim3(1024), st, cand_id, cdf, stats, cand_cap, g->n_nodes, B,
                w.hit, w.cbitmap, w.rank, w.hitpos, S_next, mult, p_incl, w.pdbl, n_next);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_ADJ_FLAG, adj_flag, dim3(EDGE_GRID), dim3(256), st, g->colidx, g->n_nodes, nS, w.eoff, w.rowstart,
                w.rank, w.edge_cap, w.keepmask, w.chunkbase, status);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_ADJ_SCAN, adj_scan, dim3(1), dim3(1024), st, w.chunkbase, nS, w.eoff, w.edge_cap, adj_rowptr,
                adj_cap, adj_nnz, status);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_ADJ_EMIT, adj_emit, dim3(EDGE_GRID), dim3(256), st, g->colidx, g->val, nS, w.eoff, w.rowstart,
                w.rank, w.pdbl, w.edge_cap, w.keepmask, w.chunkbase, adj_rowptr, adj_col, adj_val, adj_cap);
    CSGS_LAUNCH_CHECK();
    const unsigned clr_blocks = (unsigned)((B + 255) / 256 < 1024 ? (B + 255) / 256 : 1024);
    CSGS_LAUNCH(K_RANK_CLEAR, rank_clear, dim3(clr_blocks), dim3(256), st, S_next, n_next, B, g->n_nodes, w.rank);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_remote_count(const int32_t *S_next, const int32_t *n_next, int32_t local_lo, int32_t local_hi,
                                 const int32_t *part_bounds, int32_t P, int64_t *remote_total, int64_t *per_part,
                                 int32_t *src_row, int32_t *remote_ids, void *stream)
{
    if (!S_next || !n_next || local_lo > local_hi || !remote_total) return CSGS_EINVAL;
    if (per_part && (!part_bounds || P <= 0)) return CSGS_EINVAL;
    CSGS_LAUNCH(K_REMOTE_COUNT, remote_count_k, dim3(1), dim3(1024), (hipStream_t)stream, S_next, n_next, local_lo, local_hi,
                       part_bounds, per_part ? P : 0, remote_total, per_part, src_row, remote_ids);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}
