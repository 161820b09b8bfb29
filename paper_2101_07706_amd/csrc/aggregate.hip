// csgs_aggregate: Z = P~ sigma?(X)  (Section 3, Eq. 1 with the sampled operator P~).
//
// A group of G lanes (16, 32 or 64) owns one output row and spreads over the feature dimension
// with V-element vector loads, so every gathered source row is read as one contiguous burst.
// The row's edges (column, value, resolved source pointer) are fetched G at a time, one edge per
// lane, and broadcast lane-to-lane.  Products are accumulated in double, in ascending edge order,
// and rounded to float once: sampled rows carry 1/p_j discounts of 10^2..10^3, so near-cancelling
// outputs would lose the 1e-5 absolute tolerance with a float accumulator; the kernel is bound
// by memory traffic, so the wider adds are free.  Rows with many kept edges (hubs) are taken by
// all wavefronts of the block that owns them, after its ordinary rows.
//
// Also here: csgs_gather_rows (staging of the sampled remote feature rows) and csgs_aggregate_grad
// (dH_prev = (P~^T dZ) .* [H_prev > 0]: the same kernel on a per-call transpose of P~).
#include "common.hpp"

namespace csgs {

template <int V>
struct Vec {
    float x[V];
};

template <typename T, int V>
__device__ inline Vec<V> load_row(const T *p);

template <>
__device__ inline Vec<1> load_row<float, 1>(const float *p) { return Vec<1>{{p[0]}}; }
template <>
__device__ inline Vec<2> load_row<float, 2>(const float *p)
{
    const float2 v = *reinterpret_cast<const float2 *>(p);
    return Vec<2>{{v.x, v.y}};
}
template <>
__device__ inline Vec<4> load_row<float, 4>(const float *p)
{
    const float4 v = *reinterpret_cast<const float4 *>(p);
    return Vec<4>{{v.x, v.y, v.z, v.w}};
}
// bfloat16 bit patterns: widening is a 16-bit left shift
template <>
__device__ inline Vec<1> load_row<uint16_t, 1>(const uint16_t *p) { return Vec<1>{{__uint_as_float((uint32_t)p[0] << 16)}}; }
template <>
__device__ inline Vec<2> load_row<uint16_t, 2>(const uint16_t *p)
{
    const uint32_t v = *reinterpret_cast<const uint32_t *>(p);
    return Vec<2>{{__uint_as_float(v << 16), __uint_as_float(v & 0xFFFF0000u)}};
}
template <>
__device__ inline Vec<4> load_row<uint16_t, 4>(const uint16_t *p)
{
    const uint2 v = *reinterpret_cast<const uint2 *>(p);
    return Vec<4>{{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16),
                   __uint_as_float(v.y & 0xFFFF0000u)}};
}

constexpr int LONG_ROW = 32;    // rows with more kept edges than this are taken by whole blocks
constexpr int UNR = 4;          // gathered rows in flight per lane: with 8 the kernel needs more than 64 registers, which
                                // halves the blocks a compute unit holds, and the rows in flight on the device set its rate
constexpr int AGG_BLOCK = 256;  // threads per block.  Small blocks on purpose: beside kernels of other streams a 1024-thread
                                // block waits until one compute unit has 16 wavefront places free at once and the kernel starves
constexpr int AGG_WAVES = AGG_BLOCK / WAVE;

// Resolves edge e to (source row pointer, weight); a null pointer marks an edge that must not be read.
template <typename T>
__device__ inline void resolve_edge(int32_t e, const int32_t *__restrict__ adj_col, const float *__restrict__ adj_val,
                                    int64_t n_cols, const int32_t *__restrict__ src_row, const T *__restrict__ Xl,
                                    int64_t ldl, int64_t rows_l, const T *__restrict__ Xr, int64_t ldr, int64_t rows_r,
                                    const T **src, float *w)
{
    *src = nullptr;
    *w = 0.f;
    const int32_t c = adj_col[e];
    const float val = adj_val[e];   // asked for together with the column: one load latency, not two
    // a column or source row outside the tables contributes nothing (keeps every load in bounds)
    if (c >= 0 && c < n_cols) {
        const int64_t sr = src_row ? (int64_t)src_row[c] : (int64_t)c;
        if (sr >= 0 && sr < rows_l) {
            *src = Xl + sr * ldl;
            *w = val;
        } else if (sr < 0 && -1 - sr < rows_r) {
            *src = Xr + (-1 - sr) * ldr;
            *w = val;
        }
    }
}

// acc += sum over the n_max staged edges (held one per lane, group base lane `gbase`) of w * x[f..f+V).
// Loads are issued UNR at a time so that a row with many edges is not a chain of load latencies.
template <typename T, int V, bool RELU>
__device__ inline void accumulate_staged(double (&acc)[V], const T *src, float w, int gbase, int32_t n_here,
                                         int32_t n_max, bool active, int32_t f)
{
    for (int32_t j0 = 0; j0 < n_max; j0 += UNR) {
        Vec<V> x[UNR];
        float wj[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int srcl = gbase + ((j0 + u) & (WAVE - 1));
            const uint64_t pj = __shfl((uint64_t)(uintptr_t)src, srcl, WAVE);
            wj[u] = __shfl(w, srcl, WAVE);
            const bool ok = active && (j0 + u) < n_here && pj != 0;
            if (ok) {
                x[u] = load_row<T, V>(reinterpret_cast<const T *>((uintptr_t)pj) + f);
            } else {
                wj[u] = 0.f;
#pragma unroll
                for (int v = 0; v < V; ++v) x[u].x[v] = 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
#pragma unroll
            for (int v = 0; v < V; ++v) {
                float xv = x[u].x[v];
                if (RELU) xv = xv > 0.f ? xv : 0.f;
                acc[v] = fma((double)wj[u], (double)xv, acc[v]);
            }
        }
    }
}

// Zeroes the components whose mask entry is not positive (the derivative of ReLU at the layer's input).
template <int V>
__device__ inline void apply_mask(double (&acc)[V], const float *__restrict__ m)
{
#pragma unroll
    for (int v = 0; v < V; ++v)
        if (!(m[v] > 0.f)) acc[v] = 0.0;
}

template <int V>
__device__ inline void store_row(float *z, const double (&acc)[V])
{
    if (V == 4)
        *reinterpret_cast<float4 *>(z) = make_float4((float)acc[0], (float)acc[1], (float)acc[V > 2 ? 2 : 0],
                                                     (float)acc[V > 3 ? 3 : 0]);
    else if (V == 2)
        *reinterpret_cast<float2 *>(z) = make_float2((float)acc[0], (float)acc[V > 1 ? 1 : 0]);
    else
        z[0] = (float)acc[0];
}

// Ordinary rows: block `bid` of AGG_BLOCK threads owns AGG_BLOCK / G consecutive rows.
template <typename T, int V, int G, bool RELU>
__device__ inline bool aggregate_rows(int64_t bid, const int32_t *__restrict__ adj_rowptr,
                                      const int32_t *__restrict__ adj_col, const float *__restrict__ adj_val,
                                      int32_t nS_bound, const int32_t *__restrict__ nS_dev,
                                      const int32_t *__restrict__ n_cols_p, int64_t n_cols_default, int32_t *nS_out,
                                      int64_t *n_cols_out, const T *__restrict__ Xl, int64_t ldl, int64_t rows_l,
                                      const T *__restrict__ Xr, int64_t ldr, int64_t rows_r,
                                      const int32_t *__restrict__ src_row, int32_t F, float *__restrict__ Z, int64_t ldz,
                                      const float *__restrict__ mask, int64_t ldm)
{
    const int tid = (int)threadIdx.x;
    const int g = tid & (G - 1);  // lane within the row group
    const int gbase = tid & (WAVE - 1) & ~(G - 1);
    const int64_t row = (bid * AGG_BLOCK + tid) / G;
    // The two counts that may live on the device and the row's extent are asked for together, before any of
    // them is used: one load latency instead of three in a row.  The row pointers have nS_bound + 1 entries
    // whatever the count says; a count that is not given is read from a stand-in address and dropped.
    const int64_t row_c = row < nS_bound ? row : (int64_t)nS_bound - 1;
    const int32_t nS_raw = *(nS_dev ? nS_dev : adj_rowptr);
    const int32_t n_cols_raw = *(n_cols_p ? n_cols_p : adj_rowptr);
    int32_t beg = adj_rowptr[row_c], end = adj_rowptr[row_c + 1];
    const int32_t nS = !nS_dev ? nS_bound : (nS_raw < 0 ? 0 : (nS_raw < nS_bound ? nS_raw : nS_bound));
    const int64_t n_cols = n_cols_p ? (int64_t)n_cols_raw : n_cols_default;
    *nS_out = nS;
    *n_cols_out = n_cols;
    // Rows past the end, and long rows (left to the block's second pass), take part in the lane broadcasts of
    // their wavefront with an empty range.
    if (row >= nS) { beg = 0; end = 0; }
    const bool is_long = row < nS && (end - beg) > LONG_ROW;
    const bool mine = row < nS && !is_long;
    if (!mine) end = beg;
    // trip count of the edge loop must be uniform over the wavefront when G < 64
    const int32_t len = end - beg;
    int32_t maxlen = len;
    if (G < 64) {
#pragma unroll
        for (int off = G; off < WAVE; off <<= 1) {
            const int32_t o = __shfl_xor(maxlen, off, WAVE);
            maxlen = o > maxlen ? o : maxlen;
        }
    }
    {   // feature chunk blockIdx.y: wide rows are spread over several blocks instead of walked chunk by chunk
        const int32_t f0 = (int32_t)blockIdx.y * G * V;
        const int32_t f = f0 + g * V;
        const bool active = f < F;  // F is a multiple of V (checked on the host)
        double acc[V];
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] = 0.0;
        for (int32_t c0 = 0; c0 < maxlen; c0 += G) {
            // stage up to G edges of this row: one per lane
            const int32_t e = beg + c0 + g;
            const T *src = nullptr;
            float w = 0.f;
            if (e < end) resolve_edge<T>(e, adj_col, adj_val, n_cols, src_row, Xl, ldl, rows_l, Xr, ldr, rows_r, &src, &w);
            const int32_t n_here = (len - c0) < G ? (len - c0) : G;  // edges of my row in this chunk (may be <= 0)
            const int32_t n_max = (maxlen - c0) < G ? (maxlen - c0) : G;
            accumulate_staged<T, V, RELU>(acc, src, w, gbase, n_here, n_max, active, f);
        }
        if (active && mine) {
            if (mask) apply_mask<V>(acc, mask + row * ldm + f);
            store_row<V>(Z + row * ldz + f, acc);
        }
    }
    return is_long;
}

// Rows with more than LONG_ROW kept edges (hubs among the rows of S): the block's wavefronts
// work on one such row at a time, each wavefront takes a contiguous share of the row's edges,
// partial sums are added in wavefront order through LDS (fixed order: the result does not depend
// on timing).  Block `bid` takes the long ones among its own `per` rows, in row order.
template <typename T, int V, bool RELU>
__device__ inline void aggregate_long_rows(int64_t bid, int32_t per, const int32_t *__restrict__ adj_rowptr,
                                           const int32_t *__restrict__ adj_col, const float *__restrict__ adj_val,
                                           int32_t nS, int64_t n_cols, const T *__restrict__ Xl, int64_t ldl,
                                           int64_t rows_l, const T *__restrict__ Xr, int64_t ldr, int64_t rows_r,
                                           const int32_t *__restrict__ src_row, int32_t F, float *__restrict__ Z,
                                           int64_t ldz, const float *__restrict__ mask, int64_t ldm)
{
    __shared__ double part[AGG_WAVES][WAVE * V];
    __shared__ int32_t long_rows[WAVE];   // per <= 64 rows, one lane each
    __shared__ int32_t n_long;
    const int tid = (int)threadIdx.x;
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    if (wave == 0) {   // one lane per row of the block; the list keeps row order
        const int64_t row = bid * per + lane;
        const bool is_long = lane < per && row < nS && adj_rowptr[row + 1] - adj_rowptr[row] > LONG_ROW;
        const uint64_t m = __ballot(is_long);
        if (is_long) long_rows[__popcll(m & ((1ull << lane) - 1ull))] = (int32_t)row;
        if (lane == 0) n_long = __popcll(m);
    }
    __syncthreads();
    const int32_t cnt = n_long;
    for (int32_t li = 0; li < cnt; ++li) {
        const int32_t row = long_rows[li];
        const int32_t beg = adj_rowptr[row], end = adj_rowptr[row + 1];
        const int32_t share = (end - beg + AGG_WAVES - 1) / AGG_WAVES;
        const int32_t wbeg = beg + wave * share;
        const int32_t wend = (wbeg + share < end) ? wbeg + share : end;
        const int32_t len = wend > wbeg ? wend - wbeg : 0;
        {
            const int32_t f0 = (int32_t)blockIdx.y * WAVE * V;
            const int32_t f = f0 + lane * V;
            const bool active = f < F;
            double acc[V];
#pragma unroll
            for (int v = 0; v < V; ++v) acc[v] = 0.0;
            for (int32_t c0 = 0; c0 < len; c0 += WAVE) {
                const int32_t e = wbeg + c0 + lane;
                const T *src = nullptr;
                float w = 0.f;
                if (e < wend) resolve_edge<T>(e, adj_col, adj_val, n_cols, src_row, Xl, ldl, rows_l, Xr, ldr, rows_r, &src, &w);
                const int32_t n_here = (len - c0) < WAVE ? (len - c0) : WAVE;
                accumulate_staged<T, V, RELU>(acc, src, w, 0, n_here, n_here, active, f);
            }
            __syncthreads();  // part[] of the previous feature chunk / row has been read
#pragma unroll
            for (int v = 0; v < V; ++v) part[wave][lane * V + v] = acc[v];
            __syncthreads();
            if (wave == 0 && active) {
                double sum[V];
#pragma unroll
                for (int v = 0; v < V; ++v) sum[v] = 0.0;
                for (int w2 = 0; w2 < AGG_WAVES; ++w2) {
#pragma unroll
                    for (int v = 0; v < V; ++v) sum[v] += part[w2][lane * V + v];
                }
                if (mask) apply_mask<V>(sum, mask + (int64_t)row * ldm + f);
                store_row<V>(Z + (int64_t)row * ldz + f, sum);
            }
        }
    }
}

constexpr int DENSE_AVG = 16;      // kept edges per row, on average, from which on leading blocks take the long rows of a large grid
constexpr int MANY_ROWS = 32768;   // rows per call (and instance) from which on such a grid has leading blocks at all

// A block first takes the ordinary ones among its AGG_BLOCK / G rows, one group of lanes each, then,
// all wavefronts together, the long ones among them (a block-wide vote says whether there are any):
// no block has to look for long rows, which matters when the grid takes many rounds and few rows are long.
// Or the long rows go to n_long_blocks leading blocks instead, `per` rows to look through each, which
// start together with the ordinary ones: always when the whole grid is resident at once (the longest
// path counts there, not the number of blocks); in a larger grid when the rows are dense (many blocks
// would otherwise end with wavefronts that wait for the one with the longest ordinary row before the
// long rows start), and then the leading blocks of a sparse call return at once.
template <typename T, int V, int G, bool RELU, bool ADAPT>
__global__ __launch_bounds__(AGG_BLOCK) void aggregate_k(const int32_t *__restrict__ adj_rowptr,
                                                         const int32_t *__restrict__ adj_col,
                                                         const float *__restrict__ adj_val, int32_t nS_bound,
                                                         const int32_t *__restrict__ nS_dev,
                                                         const int32_t *__restrict__ n_cols_p,
                                                         const T *__restrict__ Xl, int64_t ldl, int64_t rows_l,
                                                         const T *__restrict__ Xr, int64_t ldr, int64_t rows_r,
                                                         const int32_t *__restrict__ src_row, int32_t F,
                                                         float *__restrict__ Z, int64_t ldz,
                                                         const float *__restrict__ mask, int64_t ldm,
                                                         int32_t n_long_blocks, int32_t per, int32_t dense_avg, CompStride cs)
{
    adj_rowptr = inst_ptr(adj_rowptr, cs.adj); adj_col = inst_ptr(adj_col, cs.adj); adj_val = inst_ptr(adj_val, cs.adj);
    nS_dev = inst_ptr(nS_dev, cs.adj); n_cols_p = inst_ptr(n_cols_p, cs.adj); src_row = inst_ptr(src_row, cs.adj);
    Xl = inst_ptr(Xl, cs.x); Xr = inst_ptr(Xr, cs.xr); Z = inst_ptr(Z, cs.out);
    // Who takes the long rows: the leading blocks if there are any and (ADAPT) the rows hold more than
    // dense_avg kept edges on average; else the blocks that own them.  The same for the whole grid.
    bool leading = n_long_blocks > 0;
    if (ADAPT) {
        const int32_t n = resolve_count(nS_bound, nS_dev);
        leading = leading && n > 0 && (int64_t)adj_rowptr[n] > (int64_t)dense_avg * n;
    }
    if ((int32_t)blockIdx.x < n_long_blocks) {
        if (ADAPT && !leading) return;
        const int64_t n_cols = n_cols_p ? (int64_t)*n_cols_p : (src_row ? 0x7FFFFFFFll : rows_l);
        aggregate_long_rows<T, V, RELU>((int64_t)blockIdx.x, per, adj_rowptr, adj_col, adj_val, resolve_count(nS_bound, nS_dev),
                                        n_cols, Xl, ldl, rows_l, Xr, ldr, rows_r, src_row, F, Z, ldz, mask, ldm);
        return;
    }
    const int64_t bid = (int64_t)blockIdx.x - n_long_blocks;
    int32_t nS;
    int64_t n_cols;
    const bool is_long = aggregate_rows<T, V, G, RELU>(bid, adj_rowptr, adj_col, adj_val, nS_bound, nS_dev,
                                                       n_cols_p, src_row ? 0x7FFFFFFFll : rows_l, &nS, &n_cols, Xl, ldl,
                                                       rows_l, Xr, ldr, rows_r, src_row, F, Z, ldz, mask, ldm);
    if ((ADAPT ? !leading : n_long_blocks == 0) && __syncthreads_or(is_long ? 1 : 0))
        aggregate_long_rows<T, V, RELU>(bid, AGG_BLOCK / G, adj_rowptr, adj_col, adj_val, nS, n_cols, Xl, ldl,
                                        rows_l, Xr, ldr, rows_r, src_row, F, Z, ldz, mask, ldm);
}

template <typename T, int V, int G>
static int launch_agg(const int32_t *rp, const int32_t *col, const float *val, int32_t nS, const int32_t *nsd, const int32_t *ncp, const void *Xl,
                      int64_t ldl, int64_t rl, const void *Xr, int64_t ldr, int64_t rr, const int32_t *src_row, int32_t F, int relu, float *Z, int64_t ldz,
                      const float *mask, int64_t ldm, int kid, hipStream_t st, const CompInst &ci = CompInst{})
{
    const int rows_per_block = AGG_BLOCK / G;
    const int64_t blocks = ((int64_t)nS + rows_per_block - 1) / rows_per_block;
    // the feature dimension in chunks of G * V (G = 64 whenever there is more than one chunk)
    const int64_t chunks = (F + G * V - 1) / (G * V);
    // Leading blocks for the long rows.  When the row blocks are resident at once, or nearly (8 blocks of
    // 256 threads per compute unit), 4 rows each to look through, and they always take the long rows.
    // For a call with very many rows 8 rows each, and the kernel decides by the density of the rows (every
    // block then reads the edge total first).  In between none: measured, the leading blocks and the extra
    // read cost more there than they bring (launches for 8 mini-batches of 2 K to 8 K rows each).
    const bool small_grid = (blocks + ((int64_t)nS + 3) / 4) * chunks * ci.n <= 2 * 8 * 256;
    const bool many_rows = nS >= MANY_ROWS;
    const int64_t per = small_grid ? 4 : 8;
    const int64_t lblocks = (small_grid || many_rows) ? ((int64_t)nS + per - 1) / per : 0;
    const int32_t dense_avg = (many_rows && !small_grid) ? DENSE_AVG : 0;   // > 0: the kernel decides
    const dim3 grid((unsigned)(blocks + lblocks), (unsigned)chunks, (unsigned)ci.n);
#define CSGS_AGG_LAUNCH(RELU, ADAPT)                                                                                              \
    CSGS_LAUNCH_ID(kid, (aggregate_k<T, V, G, RELU, ADAPT>), grid, dim3(AGG_BLOCK), st, rp, col, val, nS, nsd, ncp, (const T *)Xl, ldl, \
                   rl, (const T *)Xr, ldr, rr, src_row, F, Z, ldz, mask, ldm, (int32_t)lblocks, (int32_t)per, dense_avg, ci.cs)
    if (dense_avg > 0) {
        if (relu) CSGS_AGG_LAUNCH(true, true); else CSGS_AGG_LAUNCH(false, true);
    } else {
        if (relu) CSGS_AGG_LAUNCH(true, false); else CSGS_AGG_LAUNCH(false, false);
    }
#undef CSGS_AGG_LAUNCH
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

template <typename T, int V>
static int pick_group(const int32_t *rp, const int32_t *col, const float *val, int32_t nS, const int32_t *nsd, const int32_t *ncp, const void *Xl,
                      int64_t ldl, int64_t rl, const void *Xr, int64_t ldr, int64_t rr, const int32_t *src_row, int32_t F, int relu, float *Z, int64_t ldz,
                      const float *mask, int64_t ldm, int kid, hipStream_t st, const CompInst &ci = CompInst{})
{
    if (F <= 16 * V) return launch_agg<T, V, 16>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, F, relu, Z, ldz, mask, ldm, kid, st, ci);
    if (F <= 32 * V) return launch_agg<T, V, 32>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, F, relu, Z, ldz, mask, ldm, kid, st, ci);
    return launch_agg<T, V, 64>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, F, relu, Z, ldz, mask, ldm, kid, st, ci);
}

template <typename T>
static int pick_vec(const int32_t *rp, const int32_t *col, const float *val, int32_t nS, const int32_t *nsd, const int32_t *ncp, const void *Xl,
                    int64_t ldl, int64_t rl, const void *Xr, int64_t ldr, int64_t rr, const int32_t *src_row, int32_t F, int relu, float *Z, int64_t ldz,
                    const float *mask, int64_t ldm, int kid, hipStream_t st, const CompInst &ci = CompInst{})
{
    // widest vector for which every row start and F are aligned
    auto ok = [&](int v) {
        const uintptr_t bytes = (uintptr_t)v * sizeof(T);
        return F % v == 0 && (!Xl || (ldl % v == 0 && ((uintptr_t)Xl % bytes) == 0)) &&
               (!Xr || (ldr % v == 0 && ((uintptr_t)Xr % bytes) == 0)) && ldz % v == 0 &&
               ((uintptr_t)Z % ((uintptr_t)v * sizeof(float))) == 0;
    };
    if (ok(4)) return pick_group<T, 4>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, F, relu, Z, ldz, mask, ldm, kid, st, ci);
    if (ok(2)) return pick_group<T, 2>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, F, relu, Z, ldz, mask, ldm, kid, st, ci);
    return pick_group<T, 1>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, F, relu, Z, ldz, mask, ldm, kid, st, ci);
}

// ------------------------------------------------------------------ gradient of the aggregation
// dH_prev = (P~^T dZ) .* [H_prev > 0].  P~ is held by rows; its transpose is built per call in the
// caller's scratch: entries per column counted with integer atomics, a block scan turns the
// counts into column offsets, a second pass drops every entry into its column in arrival order,
// and a third puts each column's entries into ascending row order (ranks by counting inside a
// wavefront for columns of up to 64 entries, through a bitmap over the rows in LDS for longer ones).
// Then the forward kernel runs on the transposed structure with dZ as the gathered table and the
// ReLU derivative as an output mask.  Every column is summed in ascending row order, in double, with
// one rounding: the result does not depend on timing.

// one wavefront per row of P~: counts[c] += 1 for every entry of the row
__global__ __launch_bounds__(256) void adjT_count(const int32_t *__restrict__ adj_rowptr,
                                                  const int32_t *__restrict__ adj_col, int32_t nS_bound,
                                                  const int32_t *__restrict__ nS_dev, int32_t n_cols_bound,
                                                  const int32_t *__restrict__ n_cols_dev, int64_t cap,
                                                  int32_t *__restrict__ counts)
{
    const int32_t nS = resolve_count(nS_bound, nS_dev), n_cols = resolve_count(n_cols_bound, n_cols_dev);
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r = wave; r < nS; r += n_waves) {
        const int32_t beg = adj_rowptr[r] < 0 ? 0 : adj_rowptr[r];
        const int32_t end = adj_rowptr[r + 1] < cap ? adj_rowptr[r + 1] : (int32_t)cap;   // stay inside adj_col whatever the pointers say
        for (int32_t e = beg + lane; e < end; e += WAVE) {
            const int32_t c = adj_col[e];
            if (c >= 0 && c < n_cols) atomicAdd(&counts[c], 1);
        }
    }
}

// one block: colptr = exclusive prefix of counts (rounds of 8192), counts reset to zero so that the
// fill pass can use them as per-column cursors
__global__ __launch_bounds__(1024) void adjT_prefix(int32_t *__restrict__ counts, int32_t n_cols_bound,
                                                    const int32_t *__restrict__ n_cols_dev,
                                                    int32_t *__restrict__ colptr)
{
    __shared__ int32_t lds[17];
    const int32_t n_cols = resolve_count(n_cols_bound, n_cols_dev);
    int32_t base = 0;
    for (int32_t c0 = 0; c0 < n_cols; c0 += 8192) {
        int32_t v[8], sum = 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int32_t c = c0 + (int32_t)threadIdx.x * 8 + k;
            v[k] = c < n_cols ? counts[c] : 0;
            sum += v[k];
        }
        int32_t total;
        int32_t ex = base + block_exclusive_scan<int32_t>(sum, lds, &total);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int32_t c = c0 + (int32_t)threadIdx.x * 8 + k;
            if (c < n_cols) {
                colptr[c] = ex;
                counts[c] = 0;
            }
            ex += v[k];
        }
        base += total;
    }
    if (threadIdx.x == 0) colptr[n_cols] = base;
}

// one wavefront per row of P~: entry (r, c, v) goes to slot colptr[c] + cursor[c]++ of the unordered list
__global__ __launch_bounds__(256) void adjT_fill(const int32_t *__restrict__ adj_rowptr,
                                                 const int32_t *__restrict__ adj_col, const float *__restrict__ adj_val,
                                                 int32_t nS_bound, const int32_t *__restrict__ nS_dev,
                                                 int32_t n_cols_bound, const int32_t *__restrict__ n_cols_dev,
                                                 const int32_t *__restrict__ colptr, int32_t *__restrict__ cursor,
                                                 uint2 *__restrict__ unordered, int64_t cap)
{
    const int32_t nS = resolve_count(nS_bound, nS_dev), n_cols = resolve_count(n_cols_bound, n_cols_dev);
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t r = wave; r < nS; r += n_waves) {
        const int32_t beg = adj_rowptr[r] < 0 ? 0 : adj_rowptr[r];
        const int32_t end = adj_rowptr[r + 1] < cap ? adj_rowptr[r + 1] : (int32_t)cap;
        for (int32_t e = beg + lane; e < end; e += WAVE) {
            const int32_t c = adj_col[e];
            if (c >= 0 && c < n_cols) {
                const int64_t slot = (int64_t)colptr[c] + atomicAdd(&cursor[c], 1);
                if (slot < cap) unordered[slot] = make_uint2((uint32_t)r, __float_as_uint(adj_val[e]));
            }
        }
    }
}

// Puts the entries of every column into ascending row order: (row, value) from the unordered list into
// rowT / valT.  A block owns ORD_COLS consecutive columns.  Columns of up to 64 entries are taken by one
// wavefront each, an entry's place being the number of entries of its column with a smaller row (rows are
// distinct inside a column).  Longer columns (hubs among the sampled nodes) are then taken by the whole
// block one at a time: the rows present are marked in a bitmap in LDS, ORD_TILE_ROWS rows at a time, and an
// entry's place is the number of marked rows below its own.
constexpr int ORD_COLS = 64;
constexpr int ORD_TILE_ROWS = 65536;
constexpr int ORD_TILE_WORDS = ORD_TILE_ROWS / 32;

__global__ __launch_bounds__(256) void adjT_order(const int32_t *__restrict__ colptr, int32_t n_cols_bound,
                                                  const int32_t *__restrict__ n_cols_dev, int32_t nS_bound,
                                                  const int32_t *__restrict__ nS_dev, const uint2 *__restrict__ unordered,
                                                  int32_t *__restrict__ rowT, float *__restrict__ valT, int64_t cap)
{
    __shared__ uint32_t bm[ORD_TILE_WORDS];
    __shared__ int32_t below[ORD_TILE_WORDS];   // marked rows in the words before this one
    __shared__ int32_t long_cols[ORD_COLS];
    __shared__ int32_t n_long;
    __shared__ int32_t scan_lds[17];
    const int32_t n_cols = resolve_count(n_cols_bound, n_cols_dev), nS = resolve_count(nS_bound, nS_dev);
    const int tid = (int)threadIdx.x, lane = tid & (WAVE - 1), wave = tid >> 6;
    if (tid == 0) n_long = 0;
    __syncthreads();
    auto extent = [&](int32_t c, int32_t *beg, int32_t *end) {   // stays inside the lists whatever the offsets say
        const int32_t b = colptr[c], e = colptr[c + 1];
        *beg = b < 0 ? 0 : b;
        *end = e < cap ? e : (int32_t)cap;
    };
    for (int k = wave; k < ORD_COLS; k += AGG_WAVES) {
        const int64_t c = (int64_t)blockIdx.x * ORD_COLS + k;
        if (c >= n_cols) break;
        int32_t beg, end;
        extent((int32_t)c, &beg, &end);
        const int32_t len = end - beg;
        if (len <= 0) continue;
        if (len > WAVE) {
            if (lane == 0) long_cols[atomicAdd(&n_long, 1)] = (int32_t)c;   // in any order: the columns do not meet
            continue;
        }
        const uint2 v = lane < len ? unordered[beg + lane] : make_uint2(0xFFFFFFFFu, 0u);
        int32_t place = 0;
        for (int32_t j = 0; j < len; ++j) place += __shfl(v.x, j, WAVE) < v.x ? 1 : 0;
        if (lane < len) {
            rowT[beg + place] = (int32_t)v.x;
            valT[beg + place] = __uint_as_float(v.y);
        }
    }
    __syncthreads();
    const int32_t cnt = n_long;
    for (int32_t li = 0; li < cnt; ++li) {
        int32_t beg, end;
        extent(long_cols[li], &beg, &end);
        int32_t base = 0;   // entries of this column with rows below the tile
        for (int64_t lo = 0; lo < nS; lo += ORD_TILE_ROWS) {
            const int32_t words = (int32_t)((nS - lo + 31) / 32 < ORD_TILE_WORDS ? (nS - lo + 31) / 32 : ORD_TILE_WORDS);
            for (int32_t w = tid; w < words; w += AGG_BLOCK) bm[w] = 0u;
            __syncthreads();
            for (int32_t e = beg + tid; e < end; e += AGG_BLOCK) {
                const int64_t d = (int64_t)unordered[e].x - lo;
                if (d >= 0 && d < (int64_t)words * 32) atomicOr(&bm[d >> 5], 1u << (d & 31));
            }
            __syncthreads();
            int32_t pc[ORD_TILE_WORDS / AGG_BLOCK], sum = 0;
#pragma unroll
            for (int k = 0; k < ORD_TILE_WORDS / AGG_BLOCK; ++k) {
                const int32_t w = tid * (ORD_TILE_WORDS / AGG_BLOCK) + k;
                pc[k] = w < words ? __popc(bm[w]) : 0;
                sum += pc[k];
            }
            int32_t total;
            int32_t ex = block_exclusive_scan<int32_t>(sum, scan_lds, &total);
#pragma unroll
            for (int k = 0; k < ORD_TILE_WORDS / AGG_BLOCK; ++k) {
                below[tid * (ORD_TILE_WORDS / AGG_BLOCK) + k] = ex;
                ex += pc[k];
            }
            __syncthreads();
            for (int32_t e = beg + tid; e < end; e += AGG_BLOCK) {
                const uint2 v = unordered[e];
                const int64_t d = (int64_t)v.x - lo;
                if (d >= 0 && d < (int64_t)words * 32) {
                    const int32_t place = base + below[d >> 5] + __popc(bm[d >> 5] & ((1u << (d & 31)) - 1u));
                    if (place < end - beg) {
                        rowT[beg + place] = (int32_t)v.x;
                        valT[beg + place] = __uint_as_float(v.y);
                    }
                }
            }
            base += total;
            __syncthreads();   // the bitmap is cleared for the next tile or column
        }
    }
}

__global__ void fill_zero_i32(int32_t *p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = 0;
}

struct GradScratch {
    int32_t *counts, *colptr, *rowT;
    float *valT;
    uint2 *unordered;   // (row, value bits) of every entry, grouped by column, in arrival order inside a column
    size_t bytes;
};

__host__ inline GradScratch carve_grad(void *base, int32_t n_cols_cap, int64_t adj_cap)
{
    GradScratch g;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return (char *)base + o;
    };
    g.counts = (int32_t *)take((size_t)n_cols_cap * 4);
    g.colptr = (int32_t *)take(((size_t)n_cols_cap + 1) * 4);
    g.rowT = (int32_t *)take((size_t)adj_cap * 4);
    g.valT = (float *)take((size_t)adj_cap * 4);
    g.unordered = (uint2 *)take((size_t)adj_cap * 8);
    g.bytes = off;
    return g;
}

// out[k, :] = X[ids[k], :] in units of U (the widest type every row start is aligned to); one
// wavefront per row, rows strided over the grid.  An id outside the table gives a zero row.
template <typename U>
__global__ __launch_bounds__(256) void gather_rows_k(const U *__restrict__ X, int64_t ld_u, int64_t rows, int32_t row_u,
                                                     const int32_t *__restrict__ ids, int64_t cap,
                                                     const int64_t *__restrict__ n_dev, U *__restrict__ out,
                                                     int64_t ldo_u, CompStride cs)
{
    X = inst_ptr(X, cs.x); ids = inst_ptr(ids, cs.adj); n_dev = inst_ptr(n_dev, cs.adj); out = inst_ptr(out, cs.out);
    int64_t n = cap;
    if (n_dev) {
        const int64_t d = *n_dev;
        n = d < 0 ? 0 : (d < cap ? d : cap);
    }
    const int lane = lane_id();
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t n_waves = ((int64_t)gridDim.x * blockDim.x) >> 6;
    for (int64_t k = wave; k < n; k += n_waves) {
        const int64_t id = ids[k];
        const bool ok = id >= 0 && id < rows;
        for (int32_t f = lane; f < row_u; f += WAVE) out[k * ldo_u + f] = ok ? X[id * ld_u + f] : U{};
    }
}

template <typename U>
static void launch_gather(const void *X, int64_t ld_b, int64_t rows, int64_t row_b, const int32_t *ids, int64_t cap,
                          const int64_t *n_dev, void *out, int64_t ldo_b, hipStream_t st, const CompInst &ci)
{
    const int64_t waves = cap < 8192 ? cap : 8192;
    const unsigned blocks = (unsigned)((waves + 3) / 4);
    CSGS_LAUNCH(K_GATHER_ROWS, gather_rows_k<U>, dim3(blocks, 1, (unsigned)ci.n), dim3(256), st, (const U *)X,
                ld_b / (int64_t)sizeof(U), rows, (int32_t)(row_b / (int64_t)sizeof(U)), ids, cap, n_dev, (U *)out,
                ldo_b / (int64_t)sizeof(U), ci.cs);
}

}  // namespace csgs

using namespace csgs;

extern "C" int csgs_gather_rows_n(const csgs_inst_strides *inst, const void *X, int64_t ld, int64_t rows, int32_t F, int dtype,
                                  const int32_t *ids, int64_t cap, const int64_t *n_dev, void *out, int64_t ldo, void *stream)
{
    if (!X || !ids || !out || rows <= 0 || F <= 0 || ld < F || ldo < F || cap <= 0) return CSGS_EINVAL;
    CompInst ci;
    if (open_instances(inst, &ci) != CSGS_OK) return CSGS_EINVAL;
    if (dtype != CSGS_F32 && dtype != CSGS_BF16) return CSGS_EUNSUPPORTED;
    const int64_t elt = dtype == CSGS_F32 ? 4 : 2;
    const int64_t row_b = (int64_t)F * elt, ld_b = ld * elt, ldo_b = ldo * elt;
    hipStream_t st = (hipStream_t)stream;
    auto aligned = [&](int64_t a) {
        return row_b % a == 0 && ld_b % a == 0 && ldo_b % a == 0 && ((uintptr_t)X % (uintptr_t)a) == 0 &&
               ((uintptr_t)out % (uintptr_t)a) == 0;
    };
    if (aligned(16)) launch_gather<uint4>(X, ld_b, rows, row_b, ids, cap, n_dev, out, ldo_b, st, ci);
    else if (aligned(8)) launch_gather<uint2>(X, ld_b, rows, row_b, ids, cap, n_dev, out, ldo_b, st, ci);
    else if (aligned(4)) launch_gather<uint32_t>(X, ld_b, rows, row_b, ids, cap, n_dev, out, ldo_b, st, ci);
    else launch_gather<uint16_t>(X, ld_b, rows, row_b, ids, cap, n_dev, out, ldo_b, st, ci);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_gather_rows(const void *X, int64_t ld, int64_t rows, int32_t F, int dtype, const int32_t *ids,
                                int64_t cap, const int64_t *n_dev, void *out, int64_t ldo, void *stream)
{
    return csgs_gather_rows_n(nullptr, X, ld, rows, F, dtype, ids, cap, n_dev, out, ldo, stream);
}

extern "C" int csgs_aggregate(const int32_t *adj_rowptr, const int32_t *adj_col, const float *adj_val, int32_t nS,
                              const int32_t *nS_dev, const int32_t *n_next, const void *X_local, int64_t ld_local, int64_t rows_local,
                              const void *X_remote, int64_t ld_remote, int64_t rows_remote, const int32_t *src_row,
                              int32_t F, int dtype, int relu_on_input, float *Z, int64_t ldz, void *stream)
{
    return csgs_aggregate_n(nullptr, adj_rowptr, adj_col, adj_val, nS, nS_dev, n_next, X_local, ld_local, rows_local, X_remote,
                            ld_remote, rows_remote, src_row, F, dtype, relu_on_input, Z, ldz, stream);
}

extern "C" int csgs_aggregate_n(const csgs_inst_strides *inst, const int32_t *adj_rowptr, const int32_t *adj_col,
                                const float *adj_val, int32_t nS, const int32_t *nS_dev, const int32_t *n_next,
                                const void *X_local, int64_t ld_local, int64_t rows_local, const void *X_remote,
                                int64_t ld_remote, int64_t rows_remote, const int32_t *src_row, int32_t F, int dtype,
                                int relu_on_input, float *Z, int64_t ldz, void *stream)
{
    CompInst ci;
    if (open_instances(inst, &ci) != CSGS_OK) return CSGS_EINVAL;
    if (!adj_rowptr || !adj_col || !adj_val || nS <= 0 || F <= 0 || rows_local < 0 || (rows_local > 0 && !X_local) ||
        (X_local && ld_local < F) || !Z || ldz < F || (X_remote && (ld_remote < F || rows_remote < 0)))
        return CSGS_EINVAL;
    if (!X_remote) rows_remote = 0;
    if (!X_local || rows_local == 0) { X_local = nullptr; rows_local = 0; ld_local = F; }
    if (dtype != CSGS_F32 && dtype != CSGS_BF16) return CSGS_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == CSGS_F32)
        return pick_vec<float>(adj_rowptr, adj_col, adj_val, nS, nS_dev, n_next, X_local, ld_local, rows_local, X_remote,
                               ld_remote, rows_remote, src_row, F, relu_on_input, Z, ldz, nullptr, 0, prof::K_AGGREGATE, st, ci);
    return pick_vec<uint16_t>(adj_rowptr, adj_col, adj_val, nS, nS_dev, n_next, X_local, ld_local, rows_local, X_remote,
                              ld_remote, rows_remote, src_row, F, relu_on_input, Z, ldz, nullptr, 0, prof::K_AGGREGATE, st, ci);
}

extern "C" size_t csgs_aggregate_grad_scratch_bytes(int32_t n_cols, int64_t adj_cap)
{
    if (n_cols <= 0 || adj_cap <= 0) return 0;
    return carve_grad(nullptr, n_cols, adj_cap).bytes;
}

extern "C" int csgs_aggregate_grad(const int32_t *adj_rowptr, const int32_t *adj_col, const float *adj_val, int64_t adj_cap,
                                   int32_t nS, const int32_t *nS_dev, int32_t n_cols, const int32_t *n_cols_dev, const float *dZ,
                                   int64_t lddz, int32_t F, const float *H_prev, int64_t ldh, float *dH_prev, int64_t ldd,
                                   void *scratch, size_t scratch_bytes, void *stream)
{
    if (!adj_rowptr || !adj_col || !adj_val || adj_cap <= 0 || adj_cap > 0x7FFFFFFFll || nS <= 0 || n_cols <= 0 || !dZ ||
        lddz < F || F <= 0 || (H_prev && ldh < F) || !dH_prev || ldd < F || !scratch || ((uintptr_t)scratch & 255))
        return CSGS_EINVAL;
    const GradScratch g = carve_grad(scratch, n_cols, adj_cap);
    if (scratch_bytes < g.bytes) return CSGS_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    const unsigned zb = (unsigned)(((int64_t)n_cols + 255) / 256 < 1024 ? ((int64_t)n_cols + 255) / 256 : 1024);
    CSGS_LAUNCH(K_FILL_ZERO, fill_zero_i32, dim3(zb), dim3(256), st, g.counts, (int64_t)n_cols);
    CSGS_LAUNCH_CHECK();
    const unsigned rb = (unsigned)(((int64_t)nS + 3) / 4 < 4096 ? ((int64_t)nS + 3) / 4 : 4096);   // 4 rows (wavefronts) per block
    CSGS_LAUNCH(K_ADJT_COUNT, adjT_count, dim3(rb), dim3(256), st, adj_rowptr, adj_col, nS, nS_dev, n_cols, n_cols_dev, adj_cap, g.counts);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_ADJT_PREFIX, adjT_prefix, dim3(1), dim3(1024), st, g.counts, n_cols, n_cols_dev, g.colptr);
    CSGS_LAUNCH_CHECK();
    CSGS_LAUNCH(K_ADJT_FILL, adjT_fill, dim3(rb), dim3(256), st, adj_rowptr, adj_col, adj_val, nS, nS_dev, n_cols, n_cols_dev,
                (const int32_t *)g.colptr, g.counts, g.unordered, adj_cap);
    CSGS_LAUNCH_CHECK();
    const unsigned ob = (unsigned)(((int64_t)n_cols + ORD_COLS - 1) / ORD_COLS);
    CSGS_LAUNCH(K_ADJT_ORDER, adjT_order, dim3(ob), dim3(AGG_BLOCK), st, (const int32_t *)g.colptr, n_cols, n_cols_dev, nS, nS_dev,
                (const uint2 *)g.unordered, g.rowT, g.valT, adj_cap);
    CSGS_LAUNCH_CHECK();
    // the forward kernel on the transposed structure: rows = columns of P~, gathered table = dZ
    // (its rows are bounded by the row count of P~), output mask = [H_prev > 0]
    return pick_vec<float>(g.colptr, g.rowT, g.valT, n_cols, n_cols_dev, nS_dev, dZ, lddz, (int64_t)nS, nullptr, (int64_t)F, 0,
                           nullptr, F, 0, dH_prev, ldd, H_prev, ldh, prof::K_AGGREGATE_GRAD, st);
}
