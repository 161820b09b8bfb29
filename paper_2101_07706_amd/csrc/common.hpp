// Shared device helpers and the workspace layout of the csgs library (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>
#include <type_traits>
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
// "clean" sections are all-zero between calls and come first.  The per-edge sections come
// last; how many edges they can hold follows from the size the caller passed.
constexpr int CAND_TILE = 1024;   // node ids per block in the candidate scan
constexpr int EDGE_TILE = 1024;   // edges per chunk in the flat edge passes
constexpr int EDGE_GRID = 512;    // chunk blocks of the weight scan (grid-stride over chunks, they wait for nobody): two per compute unit
constexpr int HIT_TILE_WORDS = 256;   // 64-position bitmap words per block in the hit compaction
constexpr int ROW_TILE = 1024;    // rows of S per block in the degree prefix
// Weight scan through owners: edges that end in the local id range are handed, chunk by chunk, to
// blocks that each own SUB_IDS consecutive local ids and add them up in LDS.
constexpr int SUB_IDS = 2048;                     // ids per owner block (16 KB of 64-bit sums)
constexpr int SUB_MAX = 128;                      // most owner blocks: local ranges up to SUB_IDS * SUB_MAX ids
constexpr int64_t STAGE_EDGES_MAX = 8ll << 20;    // most edges of a call that are handed over this way
constexpr int META_WORDS = 4;
constexpr int META_ROWS = 0;          // rows the latest row_prefix covered (the count behind eoff / rowstart)
constexpr int META_EDGES = 1;         // eoff[rows]: edges of those rows (0 when above the workspace's capacity)
constexpr int META_EDGES_TRUE = 2;    // their true number

// Words of workspace a single-pass scan over at most `tiles` tiles with nv sums per tile needs
// (one tag word and nv sums per tile, and twice that per group of 64 tiles).
__host__ __device__ inline size_t scan_state_words(int64_t tiles, int nv)
{
    return (size_t)(1 + nv) * (size_t)(tiles + 2 * (tiles / 64 + 2));
}

struct RowOffsets {
    int64_t *eoff;       // [nS + 1] exclusive prefix of the degrees of the rows
    int64_t *rowstart;   // [nS + 1] rowptr[S[a]]
    int64_t *meta;       // [META_WORDS] resolved on the device: row count, edge count, true edge count
    int2 *chunk_note;    // [chunk_cap] (first row, rows) of every edge chunk, left by the weight scan for the adjacency pass
    int2 *bound_note;    // [chunk_cap + 2] for the edge position t * EDGE_TILE: (first row of a chunk that starts there, first row
                         // whose offset is at or beyond it), left by the row pass for the weight scan
};

struct Workspace {
    // clean: all-zero whenever no call is in flight
    uint64_t *wtable;    // [n_nodes]  per-node fixed-point weight accumulator
    uint8_t *tileflag;   // [8 * ceil(n_nodes/64)] byte g = 1: some node of ids 8g .. 8g+7 was touched (read 8 at a time: one 64-id word)
    uint32_t *hit;       // [n_nodes]  draws per candidate position
    uint64_t *cbitmap;   // [ceil(n_nodes/64)] bit set = candidate position was drawn
    // persistent: zeroed once, then never cleared; an entry counts only if it carries the tag of
    // the current call
    uint64_t *rank;      // [n_nodes]  (tag << 32) | (position in S_next + 1)
    uint64_t *member;    // [(n_nodes + 31) / 32]  (tag << 32) | one bit per id of the word's 32: in S_next of the draw with that tag
    uint64_t *partial;   // [4 * n_tiles] per-tile candidate counts and weight sums
    uint64_t *gtot;      // [4 * ceil(n_tiles / 64)] the same per group of 64 tiles
    uint64_t *cand_flag; // [n_tiles] tag of the call whose partial sums a tile holds
    uint64_t *epoch;     // [4] call counter and draw tag (see lookback.hpp); advanced on the device
    uint64_t *hit_ts;    // scan state of the hit tiles (1 sum per tile)
    // per call.  The row offsets exist twice: while the adjacency pass of one layer reads one set,
    // its spare blocks prepare the other for the next layer (rows = the node set just sampled).
    RowOffsets rows[2];
    uint64_t *adj_ts;    // scan state of the edge chunks (1 sum per chunk of 1024 edges)
    uint64_t *rp_ts;     // scan state of the row tiles (1 sum per tile of ROW_TILE rows)
    double *pdbl;        // [B]      inclusion probabilities in double
    // hand-over of local-range edges from the chunk blocks of the weight scan to the owner blocks
    uint64_t *stage_w;   // [stage_chunks * EDGE_TILE] fixed-point weight of a handed-over edge
    uint32_t *stage_c;   // [stage_chunks * EDGE_TILE] its target id; a chunk's edges lie grouped by owner
    uint32_t *stage_off; // [stage_chunks * SUB_MAX]   per chunk and owner: begin | end << 16 of its group
    uint64_t *stage_done;// [stage_chunks] persistent: tag of the call whose hand-over of this chunk is complete
    int64_t stage_chunks;
    int64_t chunk_cap;   // chunks of EDGE_TILE edges the adjacency scan can describe
    int64_t n_tiles, hit_tiles, rp_tiles;
    size_t clean_bytes;  // size of the clean part
    size_t bytes;        // size of one instance's workspace (a multiple of 256)
    int32_t n_inst;      // instances a call on this workspace processes (set by open_workspace)
    int64_t buf_stride;  // bytes between consecutive instances' caller buffers
};

// Several independent instances of a call run in the same launches: blockIdx.z selects the
// instance, and every per-instance pointer moves by that instance's stride in bytes -- `ws` for
// what lives in the workspace (instance k's workspace follows instance k - 1's), `buf` for the
// caller's arrays.  The graph is shared.  With one instance blockIdx.z is 0 and nothing moves.
struct InstStride {
    int64_t ws, buf;
};
template <typename T>
__device__ inline T *inst_ptr(T *p, int64_t stride)
{
    // (pointer arithmetic, not integer arithmetic: the result is still known to point to global memory, so loads
    // through it are global loads and not the slower flat ones)
    return p ? (T *)((char *)const_cast<typename std::remove_const<T>::type *>(p) + (int64_t)blockIdx.z * stride) : p;   // null stays null
}
constexpr int MAX_INSTANCES = 64;

// The same for the layer compute calls, whose arrays come in four groups with a stride each.
struct CompStride {
    int64_t adj;   // what the sampling calls wrote: adjacency arrays, row counts, source-row map, id lists
    int64_t x;     // the input matrix (0: one table shared by all instances)
    int64_t xr;    // staged remote rows
    int64_t out;   // the output matrix
};
struct CompInst {
    int32_t n = 1;
    CompStride cs = {0, 0, 0, 0};
};
// Checks a caller's csgs_inst_strides (null: one instance).
__host__ inline int open_instances(const csgs_inst_strides *d, CompInst *out)
{
    *out = CompInst{};
    if (!d) return CSGS_OK;
    if (d->n_inst < 1 || d->n_inst > MAX_INSTANCES || d->adj < 0 || d->x < 0 || d->x_remote < 0 || d->out < 0 ||
        ((d->adj | d->x | d->x_remote | d->out) & 15))
        return CSGS_EINVAL;
    out->n = d->n_inst;
    out->cs = CompStride{d->adj, d->x, d->x_remote, d->out};
    return CSGS_OK;
}

// Layout of a workspace sized for (n_nodes, nS_max, B_max, edges_max).  Every call carves with the
// same four numbers (they travel in the caller's csgs_workspace descriptor), so the persistent
// parts never move.
__host__ inline Workspace carve(void *base, int64_t n_nodes, int64_t nS_max, int64_t B_max, int64_t edges_max)
{
    Workspace w;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return (char *)base + o;
    };
    const size_t words = (size_t)(n_nodes + 63) / 64;
    w.n_tiles = (n_nodes + CAND_TILE - 1) / CAND_TILE;
    w.hit_tiles = ((int64_t)words + HIT_TILE_WORDS - 1) / HIT_TILE_WORDS;
    w.chunk_cap = (edges_max + EDGE_TILE - 1) / EDGE_TILE;
    if (w.chunk_cap < 1) w.chunk_cap = 1;
    w.wtable = (uint64_t *)take((size_t)n_nodes * 8);
    w.tileflag = (uint8_t *)take(words * 8);
    w.hit = (uint32_t *)take((size_t)n_nodes * 4);
    w.cbitmap = (uint64_t *)take(words * 8);
    w.clean_bytes = off;
    w.rank = (uint64_t *)take((size_t)n_nodes * 8);
    w.member = (uint64_t *)take((size_t)((n_nodes + 31) / 32) * 8);
    w.partial = (uint64_t *)take((size_t)w.n_tiles * 4 * 8);
    w.gtot = (uint64_t *)take((size_t)((w.n_tiles + 63) / 64) * 4 * 8);
    w.cand_flag = (uint64_t *)take((size_t)w.n_tiles * 8);
    w.epoch = (uint64_t *)take(4 * 8);
    w.hit_ts = (uint64_t *)take(scan_state_words(w.hit_tiles, 1) * 8);
    w.adj_ts = (uint64_t *)take(scan_state_words(w.chunk_cap, 1) * 8);
    w.rp_tiles = (nS_max + ROW_TILE - 1) / ROW_TILE;
    w.rp_ts = (uint64_t *)take(scan_state_words(w.rp_tiles, 1) * 8);
    for (int b = 0; b < 2; ++b) {
        w.rows[b].eoff = (int64_t *)take((size_t)(nS_max + 1) * 8);
        w.rows[b].rowstart = (int64_t *)take((size_t)(nS_max + 1) * 8);
        w.rows[b].meta = (int64_t *)take(META_WORDS * 8);
        w.rows[b].chunk_note = (int2 *)take((size_t)w.chunk_cap * sizeof(int2));
        w.rows[b].bound_note = (int2 *)take((size_t)(w.chunk_cap + 2) * sizeof(int2));
    }
    w.pdbl = (double *)take((size_t)B_max * 8);
    w.stage_chunks = w.chunk_cap < STAGE_EDGES_MAX / EDGE_TILE ? w.chunk_cap : STAGE_EDGES_MAX / EDGE_TILE;
    w.stage_w = (uint64_t *)take((size_t)w.stage_chunks * EDGE_TILE * 8);
    w.stage_c = (uint32_t *)take((size_t)w.stage_chunks * EDGE_TILE * 4);
    w.stage_off = (uint32_t *)take((size_t)w.stage_chunks * SUB_MAX * 4);
    w.stage_done = (uint64_t *)take((size_t)w.stage_chunks * 8);
    w.bytes = off;
    w.n_inst = 1;
    w.buf_stride = 0;
    return w;
}

// Checks a descriptor against a call's sizes and carves it.  Returns CSGS_OK or an error code.
__host__ inline int open_workspace(csgs_workspace *d, int64_t n_nodes, int64_t nS, int64_t B, Workspace *out)
{
    if (!d || !d->base || ((uintptr_t)d->base & 255) || d->n_nodes != n_nodes || d->nS_max <= 0 || d->B_max <= 0 ||
        d->edges_max <= 0)
        return CSGS_EINVAL;
    if (nS > d->nS_max || B > d->B_max) return CSGS_EWORKSPACE;
    const int32_t n_inst = d->n_inst > 1 ? d->n_inst : 1;
    if (n_inst > MAX_INSTANCES || (n_inst > 1 && (d->inst_stride <= 0 || (d->inst_stride & 255)))) return CSGS_EINVAL;
    *out = carve(d->base, d->n_nodes, d->nS_max, d->B_max, d->edges_max);
    out->n_inst = n_inst;
    out->buf_stride = n_inst > 1 ? d->inst_stride : 0;
    return out->bytes * (size_t)n_inst <= d->bytes ? CSGS_OK : CSGS_EWORKSPACE;
}

__host__ inline InstStride inst_stride(const Workspace &w) { return InstStride{(int64_t)w.bytes, w.buf_stride}; }

// Grid of a kernel whose blocks wait for each other and stride over a tile count known only on
// the device: resident_grid(per_cu) blocks of 256 threads, per_cu per compute unit.  Such a kernel
// must have all its blocks resident at once.  Alone on the device that is certain (registers and
// LDS allow several times as many).  Beside kernels of other streams it still holds as long as the
// waiting kernels in flight fit together, because every other kernel drains by itself: the
// compaction of drawn positions (33 KB of LDS) runs 1 block per unit and the adjacency filter
// (13 KB) 2, so four call sequences on four workspaces can be in flight on one device within the
// 2048 threads and 160 KB of a compute unit.  That is the documented limit.
// With several instances per call (blockIdx.z) the grid is that many times as large, but blocks
// wait only for blocks of their own instance and the hardware hands out a grid's blocks in
// ascending x, then y, then z: an instance is dispatched completely before the next one starts, a
// completely dispatched instance finishes by itself and frees its places, and at most one instance
// per kernel is ever partly dispatched -- so what must fit at once is still one instance per
// waiting kernel in flight.
__host__ inline int resident_grid(int per_cu)
{
    static std::atomic<int> cached[64];   // compute units per device, 0 = not asked yet (zero-initialised)
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 32 * per_cu;
    int cus = cached[dev].load(std::memory_order_relaxed);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 32;
        cached[dev].store(cus, std::memory_order_relaxed);   // every thread would store the same value
    }
    return per_cu * cus;
}

// Degrees of the rows S, their exclusive prefix and CSR starts into `rows`.  The row count is
// min(*nS_dev, nS) when nS_dev is given; the kernel leaves it, and the edge count, in rows.meta for
// the kernels that follow.  Defined with the weight scan.
int launch_row_prefix(const int64_t *rowptr, int64_t n_nodes, const int32_t *S, int32_t nS, const int32_t *nS_dev,
                      const Workspace &w, const RowOffsets &rows, int32_t *status, hipStream_t st);

// A row count given on the host (n) or, when n_dev is not null, on the device with n as its bound.
__device__ inline int32_t resolve_count(int32_t n, const int32_t *__restrict__ n_dev)
{
    if (!n_dev) return n;
    const int32_t d = *n_dev;
    return d < 0 ? 0 : (d < n ? d : n);
}

// ---------------------------------------------------------------- wave helpers
__device__ inline int lane_id() { return (int)(threadIdx.x & (WAVE - 1)); }

// Lane exchanges of the wave-wide scan run on the data-parallel-primitive path of the vector ALU
// (no LDS round trip): shifts by 1, 2, 4, 8 inside each row of 16 lanes with zero fill, then lane
// 15 of a row broadcast to the next row (rows 1 and 3), then lane 31 to rows 2 and 3.
template <int CTRL, int ROW_MASK>
__device__ inline uint32_t dpp_move(uint32_t v)
{
    // old = 0: lanes outside ROW_MASK, and lanes whose source falls outside the row, receive 0
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, 0xF, true);
}

template <typename T, int CTRL, int ROW_MASK>
__device__ inline T dpp_move_t(T v)
{
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit integers");
    if (sizeof(T) == 4) return (T)dpp_move<CTRL, ROW_MASK>((uint32_t)v);
    const uint64_t x = (uint64_t)v;
    const uint32_t lo = dpp_move<CTRL, ROW_MASK>((uint32_t)x), hi = dpp_move<CTRL, ROW_MASK>((uint32_t)(x >> 32));
    return (T)(((uint64_t)hi << 32) | lo);
}

// One step of the scan on a 64-bit value held as two halves: v += (v moved by the step's pattern), as an
// add with carry whose first operand comes through the DPP path -- two instructions, where a moved copy
// (two moves, each with its zero fill) and a 64-bit add take five.  Lanes the pattern leaves out are not
// written and keep v, which is what adding the zero fill gave.  The carry travels in VCC.  A DPP read of a
// register needs two wait states after the vector instruction that wrote it; inside an asm statement the
// compiler does not count them, hence the s_nop in front.
#define CSGS_SCAN_STEP64(lo, hi, PATTERN)                                                      \
    asm volatile("s_nop 1\n\t"                                                                 \
                 "v_add_co_u32_dpp %0, vcc, %0, %0 " PATTERN "\n\t"                              \
                 "v_addc_co_u32_dpp %1, vcc, %1, %1, vcc " PATTERN                               \
                 : "+v"(lo), "+v"(hi)                                                          \
                 :                                                                             \
                 : "vcc")
template <int STEP>
__device__ inline void scan_step64(uint32_t &lo, uint32_t &hi)
{
    if (STEP == 0) CSGS_SCAN_STEP64(lo, hi, "row_shr:1 row_mask:0xf bank_mask:0xf bound_ctrl:1");
    if (STEP == 1) CSGS_SCAN_STEP64(lo, hi, "row_shr:2 row_mask:0xf bank_mask:0xf bound_ctrl:1");
    if (STEP == 2) CSGS_SCAN_STEP64(lo, hi, "row_shr:4 row_mask:0xf bank_mask:0xf bound_ctrl:1");
    if (STEP == 3) CSGS_SCAN_STEP64(lo, hi, "row_shr:8 row_mask:0xf bank_mask:0xf bound_ctrl:1");
    if (STEP == 4) CSGS_SCAN_STEP64(lo, hi, "row_bcast:15 row_mask:0xa bank_mask:0xf");
    if (STEP == 5) CSGS_SCAN_STEP64(lo, hi, "row_bcast:31 row_mask:0xc bank_mask:0xf");
}

__device__ inline uint64_t wave_inclusive_scan64(uint64_t v)
{
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
    scan_step64<0>(lo, hi); scan_step64<1>(lo, hi); scan_step64<2>(lo, hi);
    scan_step64<3>(lo, hi); scan_step64<4>(lo, hi); scan_step64<5>(lo, hi);
    return ((uint64_t)hi << 32) | lo;
}

template <typename T>
__device__ inline T wave_inclusive_scan(T v)
{
    if (sizeof(T) == 8) return (T)wave_inclusive_scan64((uint64_t)v);
    v += dpp_move_t<T, 0x111, 0xF>(v);  // row_shr:1
    v += dpp_move_t<T, 0x112, 0xF>(v);  // row_shr:2
    v += dpp_move_t<T, 0x114, 0xF>(v);  // row_shr:4
    v += dpp_move_t<T, 0x118, 0xF>(v);  // row_shr:8
    v += dpp_move_t<T, 0x142, 0xA>(v);  // row_bcast:15 into rows 1 and 3
    v += dpp_move_t<T, 0x143, 0xC>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

// Sum over the wavefront, the same value in every lane.
template <typename T>
__device__ inline T wave_sum(T v)
{
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "32- or 64-bit integers");
    const T s = wave_inclusive_scan(v);
    if (sizeof(T) == 4) return (T)__builtin_amdgcn_readlane((int)s, WAVE - 1);
    const uint64_t x = (uint64_t)s;
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, WAVE - 1);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), WAVE - 1);
    return (T)(((uint64_t)hi << 32) | lo);
}

// K independent inclusive scans; written step by step across the chains so that they interleave.
template <typename T, int K>
__device__ inline void wave_inclusive_scan_multi(T (&v)[K])
{
    if (sizeof(T) == 8) {
        uint32_t lo[K], hi[K];
#pragma unroll
        for (int k = 0; k < K; ++k) { lo[k] = (uint32_t)(uint64_t)v[k]; hi[k] = (uint32_t)((uint64_t)v[k] >> 32); }
#pragma unroll
        for (int k = 0; k < K; ++k) scan_step64<0>(lo[k], hi[k]);
#pragma unroll
        for (int k = 0; k < K; ++k) scan_step64<1>(lo[k], hi[k]);
#pragma unroll
        for (int k = 0; k < K; ++k) scan_step64<2>(lo[k], hi[k]);
#pragma unroll
        for (int k = 0; k < K; ++k) scan_step64<3>(lo[k], hi[k]);
#pragma unroll
        for (int k = 0; k < K; ++k) scan_step64<4>(lo[k], hi[k]);
#pragma unroll
        for (int k = 0; k < K; ++k) scan_step64<5>(lo[k], hi[k]);
#pragma unroll
        for (int k = 0; k < K; ++k) v[k] = (T)(((uint64_t)hi[k] << 32) | lo[k]);
        return;
    }
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] += dpp_move_t<T, 0x111, 0xF>(v[k]);
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] += dpp_move_t<T, 0x112, 0xF>(v[k]);
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] += dpp_move_t<T, 0x114, 0xF>(v[k]);
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] += dpp_move_t<T, 0x118, 0xF>(v[k]);
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] += dpp_move_t<T, 0x142, 0xA>(v[k]);
#pragma unroll
    for (int k = 0; k < K; ++k) v[k] += dpp_move_t<T, 0x143, 0xC>(v[k]);
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

// First index in [0, n) with a[idx] >= key, found by the whole wavefront: every round the 64 lanes
// probe the ends of 64 equal segments at once, so an array of 8192 entries takes 3 dependent loads
// instead of 13.  All lanes must call it with the same arguments; all get the result.
template <typename T, typename I>
__device__ inline I wave_lower_bound(const T *__restrict__ a, I n, T key)
{
    const int lane = lane_id();
    I lo = 0, hi = n;
    while (hi > lo) {
        const I len = hi - lo;
        const I step = (len + WAVE - 1) / WAVE;
        const I seg_end = lo + ((lane + 1) * step < len ? (lane + 1) * step : len);  // exclusive
        const I seg_beg = lo + (lane * step < len ? lane * step : len);
        bool ge = true;  // empty segments sit past the end: treat as "all remaining entries are >= key"
        if (seg_end > seg_beg) ge = a[seg_end - 1] >= key;
        const uint64_t m = __ballot(ge);
        const int first = m ? __ffsll((unsigned long long)m) - 1 : WAVE;
        const I fb = lo + (first * step < len ? first * step : len);
        const I fe = lo + ((first + 1) * step < len ? (first + 1) * step : len);
        if (fe <= fb) {          // no segment ends at or above key: every entry is below it
            lo = hi;
        } else if (step == 1) {  // segments are single entries: entry fb is the first >= key
            return fb;
        } else {                 // a[fe - 1] >= key and everything before fb is below key
            lo = fb;
            hi = fe;
        }
    }
    return lo;
}

// ---------------------------------------------------------------- flat edge chunks
// The edges of the rows of S, concatenated in row order, form one sequence of E edges; position
// e belongs to the row a with eoff[a] <= e < eoff[a+1] and sits at rowstart[a] + (e - eoff[a])
// in the CSR arrays.  A block works on chunks of EDGE_TILE consecutive positions, so the work
// per block does not depend on the degree distribution.  The rows that overlap a chunk are
// staged in LDS once per chunk.
constexpr int SLICE_MAX = EDGE_TILE + 2;

struct RowSlice {
    int32_t off[SLICE_MAX];     // eoff[a_first + r] - c0 (first entry may be negative)
    int64_t start[SLICE_MAX];   // rowstart[a_first + r]
    int32_t a_first;            // first staged row
    int32_t R;                  // staged rows; rows [a_first, a_first + R) overlap or start in the chunk
    bool in_lds;                // false: too many (empty) rows for LDS, read eoff / rowstart directly
};

// Second half of staging a chunk: rows [a_first, a_first + R) into LDS.  Called by all threads.
__device__ inline void stage_rows(RowSlice &s, const int64_t *__restrict__ eoff, const int64_t *__restrict__ rowstart,
                                  int32_t nS, int64_t c0, int64_t a_first, int64_t R)
{
    // A prefix broken by a failed wait, or a stale note (the caller skipped the scan that writes it),
    // must not lead outside eoff / rowstart: rows [a_first, a_first + R) stay within [0, nS].
    if (a_first < 0) a_first = 0;
    if (a_first > nS) a_first = nS;
    if (R < 0) R = 0;
    if (R > (int64_t)nS + 1 - a_first) R = (int64_t)nS + 1 - a_first;
    if (threadIdx.x == 0) {
        s.a_first = (int32_t)a_first;
        s.R = (int32_t)R;
        s.in_lds = R <= SLICE_MAX;
    }
    if (R <= SLICE_MAX) {
        for (int64_t r = threadIdx.x; r < R; r += blockDim.x) {
            s.off[r] = (int32_t)(eoff[a_first + r] - c0);
            s.start[r] = (a_first + r < nS) ? rowstart[a_first + r] : 0;
        }
    }
    __syncthreads();
}

// Called by all threads of the block (at least two wavefronts).  c0 < c1 <= eoff[nS].
// `note` (nullable) points at this chunk's entry of the workspace's chunk table: with FROM_NOTE the
// first row and row count are read from it (one load) instead of being searched for (four dependent
// loads); otherwise they are searched for and, if `note` is given, left there for a later pass over
// the same chunks.
template <bool FROM_NOTE>
__device__ inline void stage_slice(RowSlice &s, const int64_t *__restrict__ eoff, const int64_t *__restrict__ rowstart,
                                   int32_t nS, int64_t c0, int64_t c1, int2 *note)
{
    __syncthreads();  // previous chunk's readers are done
    int64_t a_first, R;
    if (FROM_NOTE) {
        const int2 v = *note;
        a_first = v.x;
        R = v.y;
    } else {
        // the two searches run side by side, each by one whole wavefront (3 dependent loads for 8192
        // rows where a per-thread binary search takes 14)
        const int wave = (int)(threadIdx.x >> 6);
        if (wave == 0) {
            int64_t lb0 = wave_lower_bound(eoff, (int64_t)nS + 1, c0);
            if (lb0 > nS) lb0 = nS;   // cannot happen with a sound prefix (c0 < eoff[nS])
            if (lane_id() == 0) s.a_first = (int32_t)((eoff[lb0] == c0) ? lb0 : lb0 - 1);
        } else if (wave == 1) {
            const int64_t lb1 = wave_lower_bound(eoff, (int64_t)nS + 1, c1);
            if (lane_id() == 0) s.R = (int32_t)lb1;  // turned into a count below
        }
        __syncthreads();
        a_first = s.a_first;
        R = (int64_t)s.R - a_first;
        __syncthreads();  // everyone has read the end index before it is replaced by the count
        if (note && threadIdx.x == 0) *note = make_int2((int)a_first, (int)R);
    }
    stage_rows(s, eoff, rowstart, nS, c0, a_first, R);
}

// The same from what the row pass left per chunk boundary (bound[t] belongs to edge position
// t * EDGE_TILE): chunk t starts at bound[t].x (row 0 for t = 0) and ends before bound[t + 1].y -- two
// independent loads instead of the searches.  The last chunk, when it ends short of a boundary, still
// searches for its end.  Leaves (first row, rows) in `note` like the searching form.
__device__ inline void stage_slice_bounds(RowSlice &s, const int64_t *__restrict__ eoff,
                                          const int64_t *__restrict__ rowstart, int32_t nS, int64_t t, int64_t c0,
                                          int64_t c1, const int2 *__restrict__ bound, int2 *note)
{
    __syncthreads();  // previous chunk's readers are done
    const bool ends_on_bound = c1 == c0 + EDGE_TILE;
    const int64_t a_first = t == 0 ? 0 : (int64_t)bound[t].x;
    int64_t lb1;
    if (ends_on_bound) {
        lb1 = bound[t + 1].y;
    } else {
        if (threadIdx.x < WAVE) {
            const int64_t lb = wave_lower_bound(eoff, (int64_t)nS + 1, c1);
            if (lane_id() == 0) s.R = (int32_t)lb;
        }
        __syncthreads();
        lb1 = s.R;
        __syncthreads();  // everyone has read the end index before it is replaced by the count
    }
    const int64_t R = lb1 - a_first;
    if (note && threadIdx.x == 0) *note = make_int2((int)a_first, (int)R);
    stage_rows(s, eoff, rowstart, nS, c0, a_first, R);
}

// CSR position of chunk-relative edge x (0 <= x < c1 - c0); *r_out = staged row index.
__device__ inline int64_t edge_address(const RowSlice &s, const int64_t *__restrict__ eoff,
                                       const int64_t *__restrict__ rowstart, int64_t c0, int32_t x, int32_t *r_out)
{
    int32_t lo = 0, hi = s.R;  // last r with off[r] <= x; off[0] <= 0 <= x always
    if (s.in_lds) {
        while (hi - lo > 1) {
            const int32_t m = (lo + hi) >> 1;
            if (s.off[m] <= x) lo = m; else hi = m;
        }
        *r_out = lo;
        return s.start[lo] + (x - s.off[lo]);
    }
    const int64_t a0 = s.a_first;
    while (hi - lo > 1) {
        const int32_t m = (lo + hi) >> 1;
        if (eoff[a0 + m] - c0 <= (int64_t)x) lo = m; else hi = m;
    }
    *r_out = lo;
    return rowstart[a0 + lo] + ((int64_t)x - (eoff[a0 + lo] - c0));
}

}  // namespace csgs
