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
#include "aggregate_tile.hpp"

namespace csgs {


// Block b of the grid: row block b / slots (four tiles of TR consecutive output rows, one per wavefront) and
// feature slice b % slots (G * V features; slots = the slice count rounded up to a multiple of 8 when there is more
// than one slice, blocks beyond the slice count leave at once).  The hardware deals consecutive blocks
// round-robin to the 8 XCDs, so all blocks of slice s run on XCD s mod 8: that XCD's L2 sees only slice s of the
// gathered table, an eighth of it for rows of 1 KB, and a row that several output rows refer to is fetched
// from memory once.
template <typename T, int V, int G, bool RELU>
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
                                                         int32_t n_slices, int32_t slots, CompStride cs)
{
    constexpr int TR = tile_rows(G);
    __shared__ WaveStage<TR> stage[AGG_WAVES];
    __shared__ double heads[AGG_WAVES][WAVE * V], carries[AGG_WAVES][2 * G * V];
    const int32_t slice = (int32_t)(blockIdx.x % (unsigned)slots);
    if (slice >= n_slices) return;
    const int64_t block_row0 = (int64_t)(blockIdx.x / (unsigned)slots) * (AGG_WAVES * TR);
    adj_rowptr = inst_ptr(adj_rowptr, cs.adj); adj_col = inst_ptr(adj_col, cs.adj); adj_val = inst_ptr(adj_val, cs.adj);
    nS_dev = inst_ptr(nS_dev, cs.adj); n_cols_p = inst_ptr(n_cols_p, cs.adj); src_row = inst_ptr(src_row, cs.adj);
    Xl = inst_ptr(Xl, cs.x); Xr = inst_ptr(Xr, cs.xr); Z = inst_ptr(Z, cs.out);
    // the two counts that may live on the device are asked for together; a count that is not given is read from a
    // stand-in address and dropped
    const int32_t nS_raw = *(nS_dev ? nS_dev : adj_rowptr);
    const int32_t n_cols_raw = *(n_cols_p ? n_cols_p : adj_rowptr);
    const int32_t nS = !nS_dev ? nS_bound : (nS_raw < 0 ? 0 : (nS_raw < nS_bound ? nS_raw : nS_bound));
    const int64_t n_cols = n_cols_p ? (int64_t)n_cols_raw : (src_row ? 0x7FFFFFFFll : rows_l);
    if (block_row0 >= nS) return;
    const int tid = (int)threadIdx.x;
    const int wave = tid >> 6;
    const int32_t slice0 = slice * G * V;
    const int32_t f = slice0 + (tid % G) * V;
    const bool active = f < F;  // F is a multiple of V (checked on the host)
    const bool is_long = aggregate_tile<T, V, G, RELU>(stage[wave], heads[wave], carries[wave], block_row0 + (int64_t)wave * TR, 0, slice0, f,
                                                       active, adj_rowptr, adj_col, adj_val, nS_bound, nS, n_cols, Xl, ldl, rows_l,
                                                       Xr, ldr, rows_r, src_row, Z, ldz, mask, ldm);
    if (__syncthreads_or(is_long ? 1 : 0))
        aggregate_long_rows<T, V, G, RELU>(&heads[0][0], block_row0, 0, is_long, f, active, adj_rowptr, adj_col, adj_val, n_cols, Xl, ldl,
                                           rows_l, Xr, ldr, rows_r, src_row, Z, ldz, mask, ldm);
}

template <typename T, int V, int G>
static int launch_agg(const int32_t *rp, const int32_t *col, const float *val, int32_t nS, const int32_t *nsd, const int32_t *ncp, const void *Xl,
                      int64_t ldl, int64_t rl, const void *Xr, int64_t ldr, int64_t rr, const int32_t *src_row, int32_t F, int relu, float *Z, int64_t ldz,
                      const float *mask, int64_t ldm, int kid, hipStream_t st, const CompInst &ci = CompInst{})
{
    constexpr int BLOCK_ROWS = AGG_WAVES * tile_rows(G);
    const int64_t row_blocks = ((int64_t)nS + BLOCK_ROWS - 1) / BLOCK_ROWS;
    const int64_t n_slices = (F + G * V - 1) / (G * V);
    const int64_t slots = n_slices > 1 ? (n_slices + 7) / 8 * 8 : 1;
    if (row_blocks * slots > 0x7FFFFFFFll) return CSGS_EUNSUPPORTED;
    const dim3 grid((unsigned)(row_blocks * slots), 1, (unsigned)ci.n);
#define CSGS_AGG_LAUNCH(RELU)                                                                                                     \
    CSGS_LAUNCH_ID(kid, (aggregate_k<T, V, G, RELU>), grid, dim3(AGG_BLOCK), st, rp, col, val, nS, nsd, ncp, (const T *)Xl, ldl, rl, \
                   (const T *)Xr, ldr, rr, src_row, F, Z, ldz, mask, ldm, (int32_t)n_slices, (int32_t)slots, ci.cs)
    if (relu) CSGS_AGG_LAUNCH(true); else CSGS_AGG_LAUNCH(false);
#undef CSGS_AGG_LAUNCH
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

// Lanes per row and slice.  Rows of 1 KB and more are cut into (about) eight slices, one per XCD; shorter rows
// are taken whole by the smallest group of lanes that covers them.
template <typename T, int V>
static int pick_group(const int32_t *rp, const int32_t *col, const float *val, int32_t nS, const int32_t *nsd, const int32_t *ncp, const void *Xl,
                      int64_t ldl, int64_t rl, const void *Xr, int64_t ldr, int64_t rr, const int32_t *src_row, int32_t F, int relu, float *Z, int64_t ldz,
                      const float *mask, int64_t ldm, int kid, hipStream_t st, const CompInst &ci = CompInst{})
{
    const int64_t vecs = (F + V - 1) / V;
    const int64_t want = (int64_t)F * (int64_t)sizeof(T) >= 1024 ? (vecs + 7) / 8 : vecs;
#define CSGS_AGG_G(GG) launch_agg<T, V, GG>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, F, relu, Z, ldz, mask, ldm, kid, st, ci)
    if (want <= 4) return CSGS_AGG_G(4);
    if (want <= 8) return CSGS_AGG_G(8);
    if (want <= 16) return CSGS_AGG_G(16);
    if (want <= 32) return CSGS_AGG_G(32);
    return CSGS_AGG_G(64);
#undef CSGS_AGG_G
}

template <typename T>
static int pick_vec(const int32_t *rp, const int32_t *col, const float *val, int32_t nS, const int32_t *nsd, const int32_t *ncp, const void *Xl,
                    int64_t ldl, int64_t rl, const void *Xr, int64_t ldr, int64_t rr, const int32_t *src_row, int32_t F, int relu, float *Z, int64_t ldz,
                    const float *mask, int64_t ldm, int kid, hipStream_t st, const CompInst &ci = CompInst{})
{
    // widest vector for which every row start and F are aligned (8 floats are read as two pieces of 4)
    auto ok = [&](int v) {
        const int piece = (v == 8 && sizeof(T) == 4) ? 4 : v;
        const uintptr_t bytes = (uintptr_t)piece * sizeof(T);
        const int zpiece = v == 8 ? 4 : v;
        return F % v == 0 && (!Xl || (ldl % piece == 0 && ((uintptr_t)Xl % bytes) == 0)) &&
               (!Xr || (ldr % piece == 0 && ((uintptr_t)Xr % bytes) == 0)) && ldz % zpiece == 0 &&
               ((uintptr_t)Z % ((uintptr_t)zpiece * sizeof(float))) == 0 && (!mask || ldm % 1 == 0);
    };
    if (ok(8)) return pick_group<T, 8>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, F, relu, Z, ldz, mask, ldm, kid, st, ci);
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
    if (rows_remote > 0x7FFFFFFEll) return CSGS_EUNSUPPORTED;   // staged rows are addressed as -1 - row in 32 bits
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
