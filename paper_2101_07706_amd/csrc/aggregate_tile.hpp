// Device code of the aggregation Z = P~ sigma?(X) (Section 3, Eq. 1): one wavefront takes a tile of output rows,
// stages the kept edges of those rows in LDS and streams through the gathered rows.  Shared by the aggregation
// kernel and by the kernel that goes on to the layer product without writing Z to memory.
#pragma once
#include "common.hpp"

namespace csgs {

template <int V>
struct Vec {
    float x[V];
};

// Rows of the gathered tables are read through pointers that come out of LDS or a lane exchange as plain
// integers; the loads say that they go to global memory (a pointer of unknown kind would be read with the
// slower flat instructions, which every wait for LDS data would then wait for as well).
#define CSGS_GLOBAL __attribute__((address_space(1)))
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
template <typename U>
__device__ inline U load_global(const void *p)
{
    return *reinterpret_cast<const CSGS_GLOBAL U *>((uintptr_t)p);
}

template <typename T, int V>
__device__ inline Vec<V> load_row(const T *p);

template <>
__device__ inline Vec<1> load_row<float, 1>(const float *p) { return Vec<1>{{load_global<float>(p)}}; }
template <>
__device__ inline Vec<2> load_row<float, 2>(const float *p)
{
    const f32x2 v = load_global<f32x2>(p);
    return Vec<2>{{v.x, v.y}};
}
template <>
__device__ inline Vec<4> load_row<float, 4>(const float *p)
{
    const f32x4 v = load_global<f32x4>(p);
    return Vec<4>{{v.x, v.y, v.z, v.w}};
}
template <>
__device__ inline Vec<8> load_row<float, 8>(const float *p)   // two 16-byte loads
{
    const f32x4 a = load_global<f32x4>(p), b = load_global<f32x4>(p + 4);
    return Vec<8>{{a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w}};
}
// bfloat16 bit patterns: widening is a 16-bit left shift
template <>
__device__ inline Vec<1> load_row<uint16_t, 1>(const uint16_t *p) { return Vec<1>{{__uint_as_float((uint32_t)load_global<uint16_t>(p) << 16)}}; }
template <>
__device__ inline Vec<2> load_row<uint16_t, 2>(const uint16_t *p)
{
    const uint32_t v = load_global<uint32_t>(p);
    return Vec<2>{{__uint_as_float(v << 16), __uint_as_float(v & 0xFFFF0000u)}};
}
template <>
__device__ inline Vec<4> load_row<uint16_t, 4>(const uint16_t *p)
{
    const u32x2 v = load_global<u32x2>(p);
    return Vec<4>{{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16),
                   __uint_as_float(v.y & 0xFFFF0000u)}};
}
template <>
__device__ inline Vec<8> load_row<uint16_t, 8>(const uint16_t *p)
{
    const u32x4 v = load_global<u32x4>(p);
    return Vec<8>{{__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xFFFF0000u), __uint_as_float(v.y << 16),
                   __uint_as_float(v.y & 0xFFFF0000u), __uint_as_float(v.z << 16), __uint_as_float(v.z & 0xFFFF0000u),
                   __uint_as_float(v.w << 16), __uint_as_float(v.w & 0xFFFF0000u)}};
}

constexpr int LONG_ROW = 256;   // rows with more kept edges than this are taken by the whole block, after its tiles
template <int V>
constexpr int unr() { return V >= 8 ? 2 : 4; }   // gathered row pieces asked for at a time per lane (and as many again before those are used): 64 bytes
constexpr int AGG_BLOCK = 256;  // threads per block.  Small blocks on purpose: beside kernels of other streams a 1024-thread
                                // block waits until one compute unit has 16 wavefront places free at once and the kernel starves
constexpr int AGG_WAVES = AGG_BLOCK / WAVE;
constexpr int POOL = 256;       // edges a wavefront stages at a time

// Reads that must not count (an edge whose column or source row lies outside the tables, a lane whose share of
// the edges has ended) go here: zeros, so that they add 0 * 0 without a test.  At least 64 lanes x 8 floats.
static __device__ __align__(256) uint32_t g_zero_row[512];

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
    constexpr int UNR = unr<V>();
    for (int32_t j0 = 0; j0 < n_max; j0 += UNR) {
        Vec<V> x[UNR];
        float wj[UNR];
#pragma unroll
        for (int u = 0; u < UNR; ++u) {
            const int srcl = gbase + ((j0 + u) & (WAVE - 1));
            const uint64_t pj = __shfl((uint64_t)(uintptr_t)src, srcl, WAVE);
            wj[u] = __shfl(w, srcl, WAVE);
            // (no load under a condition: what must not count reads the zero row with weight 0, and the compiler
            // keeps exact count of the loads in flight)
            const bool ok = active && (j0 + u) < n_here && pj != 0;
            if (!ok) wj[u] = 0.f;
            x[u] = load_row<T, V>(ok ? reinterpret_cast<const T *>((uintptr_t)pj) + f : reinterpret_cast<const T *>(g_zero_row));
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

// ZLDS: `z` points into LDS (the tile of Z that the layer product reads next); the stores then say so, instead of
// going through the flat path that a pointer of unknown kind takes.
#define CSGS_LDS __attribute__((address_space(3)))
// Stores to global memory that the compiler does not keep count of.  Loads and stores share one counter of outstanding
// operations on this part, and loads come back in order only among themselves: with a store of its own outstanding the
// compiler waits for everything before it uses any loaded value, so a row's store inside a loop that keeps the next
// loads in flight would drain them at every turn.  A store it does not see leaves its count of the loads exact, and
// the extra outstanding operation only makes a wait for "all but the last n" longer, never shorter.  Only for memory
// that the kernel itself never reads again.
__device__ inline void store_untracked(float *p, float v)
{
    asm volatile("global_store_dword %0, %1, off" : : "v"(p), "v"(v) : "memory");
}
__device__ inline void store_untracked(float *p, f32x2 v)
{
    asm volatile("global_store_dwordx2 %0, %1, off" : : "v"(p), "v"(v) : "memory");
}
__device__ inline void store_untracked(float *p, f32x4 v)
{
    asm volatile("global_store_dwordx4 %0, %1, off" : : "v"(p), "v"(v) : "memory");
}

template <int V, bool ZLDS = false>
__device__ inline void store_row(float *z, const double (&acc)[V])
{
    if (ZLDS) {
#pragma unroll
        for (int v = 0; v < V; ++v) ((CSGS_LDS float *)z)[v] = (float)acc[v];   // consecutive words: the compiler merges them
        return;
    }
    if (V >= 4) {
#pragma unroll
        for (int q = 0; q + 4 <= V; q += 4)
            store_untracked(z + q, f32x4{(float)acc[q], (float)acc[q + 1 < V ? q + 1 : 0], (float)acc[q + 2 < V ? q + 2 : 0],
                                         (float)acc[q + 3 < V ? q + 3 : 0]});
    } else if (V == 2) {
        store_untracked(z, f32x2{(float)acc[0], (float)acc[V > 1 ? 1 : 0]});
    } else {
        store_untracked(z, (float)acc[0]);
    }
}

// A staged edge: where its piece of the gathered row starts (source row resolved, the block's feature slice added;
// a lane adds its own offset inside the slice), its P~ value, and where it stands in its row.
struct __align__(16) StagedEdge {
    uint64_t ptr;
    float w;
    uint32_t tag;   // row in the tile << 2 | first edge of its row << 1 | last edge of its row
};

// What a wavefront keeps in LDS about its tile of TR output rows.  The kept edges of the tile's ordinary rows
// are staged here in row order, already resolved, up to POOL at a time.  The NG lane groups of the wavefront
// (G lanes each, spread over the slice's features) then take equal shares of the staged edges, whatever rows
// they belong to, and stream through them; a row whose edges fall into several shares is put together from the
// groups' partial sums afterwards, in group order.
template <int TR, int PL = POOL>
struct WaveStage {
    StagedEdge pool[PL + 1];     // [PL]: the edge that does not count (zeros, weight 0, ends no row)
    int32_t beg[TR];             // first edge of the row
    int32_t len[TR];             // staged edges of the row: 0 for rows past the end and for long rows
    int32_t xs[TR + 1];          // exclusive prefix of len over the tile
    int32_t head_state[16];      // per group: how its share begins (see HEAD_*)
    int32_t carry_row;           // row (in the tile) of the partial sum carried into the next POOL edges, -1: none
    uint8_t ordinary[TR];        // 1: a row of this call that is not long
};
enum { HEAD_NONE = 0,    // the share begins with the first edge of a row
       HEAD_CLOSED = 1,  // it begins inside a row, and that row's last edge is in the share: head = the row's edges in the share
       HEAD_OPEN = 2 };  // every edge of the share (possibly none) belongs to a row that began earlier and goes on: head = all of them

constexpr int tile_rows(int G) { return (WAVE / G) * 8 < WAVE ? (WAVE / G) * 8 : WAVE; }   // about 8 rows per lane group
constexpr int ilog2(int n) { return n <= 1 ? 0 : 1 + ilog2(n / 2); }

// One wavefront, one tile of TR output rows, one slice of G * V features starting at feature `slice0`.
// head: LDS, WAVE * V doubles; carry: LDS, 2 * G * V doubles.
// Row r of the call is stored at Z + (r - out_row0) * ldz.  ZLDS: Z is a tile in LDS.  PL: edges staged at a time.
// WHOLE (G = 64: the wavefront is one lane group): the sum of a row that goes on beyond the staged edges stays in
// the registers, and neither `head` nor `carry` is used (null).
template <typename T, int V, int G, bool RELU, int PL = POOL, bool ZLDS = false, bool WHOLE = false>
__device__ inline bool aggregate_tile(WaveStage<tile_rows(G), PL> &st, double *__restrict__ head, double *__restrict__ carry, int64_t row0, int64_t out_row0,
                                      int32_t slice0, int32_t f, bool active, const int32_t *__restrict__ adj_rowptr,
                                      const int32_t *__restrict__ adj_col, const float *__restrict__ adj_val, int32_t nS_bound,
                                      int32_t nS, int64_t n_cols, const T *__restrict__ Xl, int64_t ldl, int64_t rows_l,
                                      const T *__restrict__ Xr, int64_t ldr, int64_t rows_r, const int32_t *__restrict__ src_row,
                                      float *__restrict__ Z, int64_t ldz, const float *__restrict__ mask, int64_t ldm)
{
    constexpr int NG = WAVE / G;   // lane groups per wavefront
    constexpr int TR = tile_rows(G);
    constexpr int UNR = unr<V>();
    static_assert(!WHOLE || G == WAVE, "whole rows: one lane group per wavefront");
    constexpr int ROUNDS = PL >= 2 * WAVE ? 2 : 1;   // staging rounds whose loads are asked for together
    const int lane = lane_id();
    // ---- lane l < TR looks at row l of the tile
    const int64_t row = row0 + lane;
    const int64_t row_c = row < nS_bound ? row : (int64_t)nS_bound - 1;   // the row pointers have nS_bound + 1 entries
    const int32_t rbeg = adj_rowptr[row_c], rend = adj_rowptr[row_c + 1];
    const bool in_call = lane < TR && row < nS;
    const int32_t full_len = in_call ? rend - rbeg : 0;
    const bool is_long = full_len > LONG_ROW;
    const int32_t len = (is_long || full_len < 0) ? 0 : full_len;
    const int32_t incl = wave_inclusive_scan(len);
    if (lane < TR) {
        st.beg[lane] = rbeg;
        st.len[lane] = len;
        st.xs[lane + 1] = incl;
        st.ordinary[lane] = (in_call && !is_long) ? 1 : 0;
    }
    if (lane == 0) {
        st.xs[0] = 0;
        st.carry_row = -1;
        st.pool[PL] = StagedEdge{(uint64_t)(uintptr_t)g_zero_row, 0.f, 0u};
    }
    const int32_t total = __builtin_amdgcn_readlane(incl, WAVE - 1);
    const int grp = lane / G;
    int par = 0;   // which half of `carry` the next round reads
    const uint32_t lane_off = active ? (uint32_t)((lane % G) * V * (int)sizeof(T)) : 0u;   // a lane past the last feature reads the slice's start and stores nothing
    __builtin_amdgcn_wave_barrier();
    // ---- rows without kept edges are zero rows
    for (int rr = grp; rr < TR; rr += NG) {
        if (st.ordinary[rr] && st.len[rr] == 0 && active) {
            double zero[V];
#pragma unroll
            for (int v = 0; v < V; ++v) zero[v] = 0.0;
            store_row<V, ZLDS>(Z + (row0 - out_row0 + rr) * ldz + f, zero);
        }
    }
    auto finish_row = [&](double (&sum)[V], int r) {   // rounds and stores row r of the tile
        const int64_t out = row0 + r;
        if (active) {
            if (mask) apply_mask<V>(sum, mask + out * ldm + f);
            store_row<V, ZLDS>(Z + (out - out_row0) * ldz + f, sum);
        }
    };
    double acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.0;
    for (int32_t cb = 0; cb < total; cb += PL) {
        const int32_t S = (total - cb) < PL ? (total - cb) : PL;   // edges staged this time: wave-uniform
        __builtin_amdgcn_wave_barrier();
        // ---- stage them: one edge per lane and round, two rounds at a time with their loads asked for together
        // (column and value, then the source row)
        for (int32_t s0 = 0; s0 < S; s0 += ROUNDS * WAVE) {
            uint32_t e[ROUNDS], tg[ROUNDS];
            int32_t c[ROUNDS];
            float w[ROUNDS];
#pragma unroll
            for (int k = 0; k < ROUNDS; ++k) {
                const int32_t s = s0 + k * WAVE + lane;
                const int32_t sa = cb + (s < S ? s : S - 1);   // a lane beyond the end repeats the last edge and stores nothing
                int lo = 0, hi = TR;   // the row r with xs[r] <= sa < xs[r + 1]
#pragma unroll
                for (int step = 0; step < ilog2(TR); ++step) {
                    const int m = (lo + hi) >> 1;
                    if (st.xs[m] <= sa) lo = m; else hi = m;
                }
                const int32_t d = sa - st.xs[lo];
                e[k] = (uint32_t)(st.beg[lo] + d);
                tg[k] = ((uint32_t)lo << 2) | (d == 0 ? 2u : 0u) | (d + 1 == st.len[lo] ? 1u : 0u);
            }
#pragma unroll
            for (int k = 0; k < ROUNDS; ++k) {
                c[k] = adj_col[e[k]];
                w[k] = adj_val[e[k]];
            }
#pragma unroll
            for (int k = 0; k < ROUNDS; ++k) {
                const bool col_ok = c[k] >= 0 && c[k] < n_cols;
                const uint32_t cc = col_ok ? (uint32_t)c[k] : 0u;
                c[k] = src_row ? src_row[cc] : (int32_t)cc;        // from here on: the source row
                if (!col_ok) c[k] = (int32_t)0x80000000;
            }
#pragma unroll
            for (int k = 0; k < ROUNDS; ++k) {
                const int32_t s = s0 + k * WAVE + lane;
                if (s < S) {
                    StagedEdge se;
                    se.ptr = (uint64_t)(uintptr_t)g_zero_row;
                    se.w = 0.f;
                    if (c[k] != (int32_t)0x80000000) {
                        if (c[k] >= 0 && c[k] < rows_l) {
                            se.ptr = (uint64_t)(uintptr_t)(Xl + (int64_t)c[k] * ldl + slice0);
                            se.w = w[k];
                        } else if (c[k] < 0 && -1 - (int64_t)c[k] < rows_r) {
                            se.ptr = (uint64_t)(uintptr_t)(Xr + (-1 - (int64_t)c[k]) * ldr + slice0);
                            se.w = w[k];
                        }
                    }
                    se.tag = tg[k];
                    st.pool[s] = se;
                }
            }
        }
        __builtin_amdgcn_wave_barrier();
        // ---- every group streams through its share [lo, hi) of the staged edges: UNR pieces of gathered rows asked for
        // per lane, and UNR more before those are used; sums in double in edge order
        const int32_t lo = (int32_t)(((int64_t)grp * S) / NG), hi = (int32_t)(((int64_t)(grp + 1) * S) / NG);
        const int32_t L = hi - lo;
        const int32_t Lmax = (S + NG - 1) / NG;   // no share is longer
        if (!WHOLE) {
#pragma unroll
            for (int v = 0; v < V; ++v) acc[v] = 0.0;
        }
        // my share begins inside a row that an earlier share (or the edges staged before) began; a wavefront that
        // takes whole rows has the beginning of such a row in its registers
        bool in_head = !WHOLE && (L == 0 || !(st.pool[lo].tag & 2u));
        int32_t my_head = in_head ? HEAD_OPEN : HEAD_NONE;
        struct Batch {
            Vec<V> x[UNR];
            float w[UNR];
            uint32_t tg[UNR];
        };
        auto issue = [&](int32_t t0, Batch &bt) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
                const int32_t t = t0 + u;
                const StagedEdge se = st.pool[t < L ? lo + t : PL];   // beyond my share: the edge that does not count
                bt.w[u] = se.w;
                bt.tg[u] = se.tag;
                bt.x[u] = load_row<T, V>(reinterpret_cast<const T *>((uintptr_t)(se.ptr + lane_off)));
            }
        };
        auto consume = [&](const Batch &bt) {
#pragma unroll
            for (int u = 0; u < UNR; ++u) {
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float xv = bt.x[u].x[v];
                    if (RELU) xv = xv > 0.f ? xv : 0.f;
                    acc[v] = fma((double)bt.w[u], (double)xv, acc[v]);
                }
                if (bt.tg[u] & 1u) {         // the row ends here
                    if (in_head) {           // its beginning lies in an earlier share: leave my part for whoever holds that
#pragma unroll
                        for (int v = 0; v < V; ++v) head[lane * V + v] = acc[v];
                        in_head = false;
                        my_head = HEAD_CLOSED;
                    } else {
                        finish_row(acc, (int)(bt.tg[u] >> 2));
                    }
#pragma unroll
                    for (int v = 0; v < V; ++v) acc[v] = 0.0;
                }
            }
        };
        {
            // No load of this loop sits under a condition (a batch beyond the share asks for the edge that does not
            // count: cached zeros), and the rows' stores are ones the compiler does not count: it then knows how many
            // loads are in flight at every point and waits for the batch it consumes, not for the one just asked for.
            Batch a, b2;
            issue(0, a);
            for (int32_t t0 = 0; t0 < Lmax; t0 += 2 * UNR) {
                issue(t0 + UNR, b2);
                consume(a);
                issue(t0 + 2 * UNR, a);
                consume(b2);
            }
        }
        if (WHOLE) continue;   // a row that goes on stays in `acc`
        if (in_head) {   // the whole share lies inside a row that goes on
#pragma unroll
            for (int v = 0; v < V; ++v) head[lane * V + v] = acc[v];
        }
        if ((lane % G) == 0) st.head_state[grp] = my_head;
        const uint32_t end_tag = L > 0 ? st.pool[hi - 1].tag : 1u;
        const bool has_tail = !in_head && !(end_tag & 1u);   // acc holds the beginning of a row that goes on in later shares
        const int32_t c_row = st.carry_row;                  // a row carried in from the edges staged before
        double *carry_in = carry + (par ? G * V : 0), *carry_out = carry + (par ? 0 : G * V);
        par ^= 1;
        __builtin_amdgcn_wave_barrier();
        // ---- rows cut by share boundaries: whoever holds a row's beginning adds the later shares' heads, in share
        // order.  A row that goes on beyond the edges staged this time (at most one) is carried into the next round.
        auto add_heads = [&](double (&sum)[V], int k, int r) -> bool {   // true: the row was completed and stored
            for (; k < NG; ++k) {
                const int32_t hs = st.head_state[k];
                const int src = k * G + (lane % G);
#pragma unroll
                for (int v = 0; v < V; ++v) sum[v] += head[src * V + v];
                if (hs == HEAD_CLOSED) break;
            }
            if (k < NG) {
                finish_row(sum, r);
                return true;
            }
#pragma unroll
            for (int v = 0; v < V; ++v) carry_out[(lane % G) * V + v] = sum[v];
            return false;
        };
        int32_t next_carry = -1;
        if (has_tail && !add_heads(acc, grp + 1, (int)(end_tag >> 2))) next_carry = (int32_t)(end_tag >> 2);
        if (grp == 0 && c_row >= 0) {   // the row carried in: group 0's lanes put it together the same way
            double sum[V];
#pragma unroll
            for (int v = 0; v < V; ++v) sum[v] = carry_in[(lane % G) * V + v];
            if (!add_heads(sum, 0, c_row)) next_carry = c_row;
        }
        // every lane of the one group that carries on holds the row; all others hold -1
        int32_t nc = next_carry;
#pragma unroll
        for (int off = WAVE / 2; off >= 1; off >>= 1) {
            const int32_t o = __shfl_xor(nc, off, WAVE);
            nc = o > nc ? o : nc;
        }
        if (lane == 0) st.carry_row = nc;
    }
    return is_long;
}

// Rows with more than LONG_ROW kept edges (hubs among the rows of S): the whole block works on one such row at
// a time, each of its 256 / G lane groups takes a contiguous share of the row's edges, and the groups' sums are
// added in group order through LDS (fixed order: the result does not depend on timing).
template <typename T, int V, int G, bool RELU, bool ZLDS = false>
__device__ inline void aggregate_long_rows(double *__restrict__ part /* LDS, AGG_BLOCK * V */, int64_t block_row0, int64_t out_row0, bool is_long, int32_t f,
                                           bool active, const int32_t *__restrict__ adj_rowptr, const int32_t *__restrict__ adj_col,
                                           const float *__restrict__ adj_val, int64_t n_cols, const T *__restrict__ Xl,
                                           int64_t ldl, int64_t rows_l, const T *__restrict__ Xr, int64_t ldr, int64_t rows_r,
                                           const int32_t *__restrict__ src_row, float *__restrict__ Z, int64_t ldz,
                                           const float *__restrict__ mask, int64_t ldm)
{
    constexpr int UNITS = AGG_BLOCK / G;
    constexpr int TR = tile_rows(G);
    __shared__ int32_t long_rows[AGG_WAVES * TR];   // row in the block, in row order
    __shared__ int32_t wave_cnt[AGG_WAVES];
    const int tid = (int)threadIdx.x;
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    const uint64_t m = __ballot(is_long);
    if (lane == 0) wave_cnt[wave] = __popcll(m);
    __syncthreads();
    int32_t base = 0, cnt = 0;
    for (int w2 = 0; w2 < AGG_WAVES; ++w2) {
        if (w2 < wave) base += wave_cnt[w2];
        cnt += wave_cnt[w2];
    }
    if (is_long) long_rows[base + __popcll(m & ((1ull << lane) - 1ull))] = wave * TR + lane;
    __syncthreads();
    const int unit = tid / G, g = tid % G;
    const int gbase = lane & ~(G - 1);
    for (int32_t li = 0; li < cnt; ++li) {
        const int64_t row = block_row0 + long_rows[li];
        const int32_t beg = adj_rowptr[row], end = adj_rowptr[row + 1];
        const int32_t share = (end - beg + UNITS - 1) / UNITS;
        const int32_t ub = beg + unit * share;
        const int32_t ue = (ub + share < end) ? ub + share : end;
        double acc[V];
#pragma unroll
        for (int v = 0; v < V; ++v) acc[v] = 0.0;
        for (int32_t k0 = 0; k0 < share; k0 += G) {   // the same trip count for every group of the block
            const int32_t e = ub + k0 + g;
            const T *src = nullptr;
            float w = 0.f;
            if (e < ue) resolve_edge<T>(e, adj_col, adj_val, n_cols, src_row, Xl, ldl, rows_l, Xr, ldr, rows_r, &src, &w);
            const int32_t left = ue - (ub + k0);
            const int32_t n_here = left < 0 ? 0 : (left < G ? left : G);
            const int32_t n_max = (share - k0) < G ? (share - k0) : G;
            accumulate_staged<T, V, RELU>(acc, src, w, gbase, n_here, n_max, active, f);
        }
        __syncthreads();  // part[] of the previous row has been read
#pragma unroll
        for (int v = 0; v < V; ++v) part[tid * V + v] = acc[v];
        __syncthreads();
        if (tid < G && active) {
            double sum[V];
#pragma unroll
            for (int v = 0; v < V; ++v) sum[v] = 0.0;
            for (int u = 0; u < UNITS; ++u) {
#pragma unroll
                for (int v = 0; v < V; ++v) sum[v] += part[(u * G + tid) * V + v];
            }
            if (mask) apply_mask<V>(sum, mask + row * ldm + f);
            store_row<V, ZLDS>(Z + (row - out_row0) * ldz + f, sum);
        }
    }
}

}  // namespace csgs
