// csgs_layer_forward: H = (P~ sigma?(X)) W  (Section 3, Eq. 1) in one kernel: the rows of Z = P~ sigma?(X) that a
// block aggregates stay in LDS and feed the matrix cores there, so Z is neither written to memory nor read back
// (optionally it is also written, for the weight gradient of a training step).
//
// A block of four wavefronts owns 32 consecutive rows of the sampled layer.
//   1. Aggregation: each wavefront takes 8 of the rows, all 64 lanes spread over the (at most 256) input features
//      of one gathered row at a time; sums in double in edge order, one rounding to float into the LDS tile.  Rows
//      with more than 256 kept edges are taken by the whole block afterwards.  This is the code of csgs_aggregate
//      with one lane group per wavefront.
//   2. Product: wavefront w computes the 16-column tiles w, w + 4, ... of H for all 32 rows.  A comes from the LDS
//      tile (two 128-bit reads per 16 rows and K chunk of 32, the k order permuted as in csgs_layer_gemm: lane group
//      g feeds k = 8 g + s at step s).  B needs no LDS: in that order lane (g, n) multiplies exactly W[8 g + s][n],
//      s = 0..7, so every lane loads its own eight weights of the next chunk from global memory (W is small and
//      stays in L2) while the current chunk's MFMAs run.  The wavefronts of a block do not wait for each other in
//      this phase.  Operands are widened to double (exact), v_mfma_f64_16x16x4_f64 accumulates in double, one
//      rounding to float: the arithmetic of csgs_layer_gemm.
// Blocks of one compute unit are at different points of their life, so one block's gathers overlap another's MFMAs.
#include "common.hpp"
#include "aggregate_tile.hpp"
#include "gemm_tile.hpp"

namespace csgs {

constexpr int FUSED_ROWS = 32;   // rows of Z per block: one 8-row tile per wavefront
constexpr int FUSED_POOL = 64;   // edges a wavefront stages at a time (8 rows hold a few dozen)

// KP: capacity of the LDS tile in features (64, 128 or 256); a lane holds V = KP / 64 consecutive features.
template <typename T, int KP, bool RELU>
__global__ __launch_bounds__(AGG_BLOCK, 3) void layer_forward_k(const int32_t *__restrict__ adj_rowptr,
                                                                const int32_t *__restrict__ adj_col,
                                                                const float *__restrict__ adj_val, int32_t nS_bound,
                                                                const int32_t *__restrict__ nS_dev,
                                                                const int32_t *__restrict__ n_cols_p,
                                                                const T *__restrict__ Xl, int64_t ldl, int64_t rows_l,
                                                                const T *__restrict__ Xr, int64_t ldr, int64_t rows_r,
                                                                const int32_t *__restrict__ src_row, int32_t K,
                                                                const float *__restrict__ W, int64_t ldw, int32_t N,
                                                                float *__restrict__ H, int64_t ldh,
                                                                float *__restrict__ Zout, int64_t ldz, CompStride cs, int64_t z_stride)
{
    constexpr int V = KP / WAVE;
    constexpr int G = WAVE;
    constexpr int TR = tile_rows(G);
    static_assert(AGG_WAVES * TR == FUSED_ROWS, "one tile per wavefront");
    constexpr int ZS = KP + 4;    // words per row of the tile: 16 rows' 128-bit reads of one k range fall on all banks
    constexpr int RT = FUSED_ROWS / 16;
    typedef WaveStage<TR, FUSED_POOL> Stage;
    constexpr size_t STAGE_BYTES = sizeof(Stage) * AGG_WAVES, PART_BYTES = sizeof(double) * AGG_BLOCK * V;
    __shared__ __attribute__((aligned(16))) float Zt[FUSED_ROWS * ZS];
    // the staged edges of the tiles, then (when the tiles are done) the partial sums of the long rows
    __shared__ __attribute__((aligned(16))) unsigned char work[STAGE_BYTES > PART_BYTES ? STAGE_BYTES : PART_BYTES];
    Stage *stage = reinterpret_cast<Stage *>(work);
    double *part = reinterpret_cast<double *>(work);

    const int64_t block_row0 = (int64_t)blockIdx.x * FUSED_ROWS;
    adj_rowptr = inst_ptr(adj_rowptr, cs.adj); adj_col = inst_ptr(adj_col, cs.adj); adj_val = inst_ptr(adj_val, cs.adj);
    nS_dev = inst_ptr(nS_dev, cs.adj); n_cols_p = inst_ptr(n_cols_p, cs.adj); src_row = inst_ptr(src_row, cs.adj);
    Xl = inst_ptr(Xl, cs.x); Xr = inst_ptr(Xr, cs.xr); H = inst_ptr(H, cs.out); Zout = inst_ptr(Zout, z_stride);
    const int32_t nS_raw = *(nS_dev ? nS_dev : adj_rowptr);
    const int32_t n_cols_raw = *(n_cols_p ? n_cols_p : adj_rowptr);
    const int32_t nS = !nS_dev ? nS_bound : (nS_raw < 0 ? 0 : (nS_raw < nS_bound ? nS_raw : nS_bound));
    const int64_t n_cols = n_cols_p ? (int64_t)n_cols_raw : (src_row ? 0x7FFFFFFFll : rows_l);
    if (block_row0 >= nS) return;
    const int tid = (int)threadIdx.x;
    const int lane = tid & (WAVE - 1), wave = tid >> 6;
    const int n_chunks = (K + BK - 1) / BK;

    // ---- columns K .. 32 * n_chunks of the tile are zeros (the product multiplies whole chunks)
    {
        const int pad = n_chunks * BK - K;
        for (int i = tid; i < FUSED_ROWS * pad; i += AGG_BLOCK) Zt[(i / pad) * ZS + K + (i % pad)] = 0.f;
    }
    // ---- 1. the rows of Z
    const int32_t f = lane * V;
    const bool active = f < K;   // K is a multiple of V (checked on the host)
    const bool is_long = aggregate_tile<T, V, G, RELU, FUSED_POOL, true, true>(
        stage[wave], nullptr, nullptr, block_row0 + (int64_t)wave * TR, block_row0, 0, f, active, adj_rowptr, adj_col, adj_val, nS_bound, nS,
        n_cols, Xl, ldl, rows_l, Xr, ldr, rows_r, src_row, Zt, ZS, nullptr, 0);
    if (__syncthreads_or(is_long ? 1 : 0))
        aggregate_long_rows<T, V, G, RELU, true>(part, block_row0, block_row0, is_long, f, active, adj_rowptr, adj_col, adj_val, n_cols, Xl,
                                                 ldl, rows_l, Xr, ldr, rows_r, src_row, Zt, ZS, nullptr, 0);

    // ---- 2. the product.  Tile t of 16 columns, chunk c of 32 k; this wavefront takes the tiles wave, wave + 4, ...
    const int grp = lane >> 4, l16 = lane & 15;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    const int n_tiles16 = (N + 15) / 16;
    const int my_tiles = n_tiles16 > wave_u ? (n_tiles16 - wave_u + AGG_WAVES - 1) / AGG_WAVES : 0;
    // Lane (g, n) needs W[32 c + 8 g + s][first column of the tile + n], s = 0..7.  The address is a part that the whole
    // wavefront shares (chunk and tile: scalar arithmetic) plus a lane's own byte offset that never changes, so a
    // fetch costs no vector arithmetic.  A ragged last tile is moved left to end at column N (its first columns repeat
    // the tile before and are not stored; with fewer than 16 columns in all, lanes beyond N read column N - 1).  In a
    // ragged last chunk a k that does not exist reads the last real one and is dropped when used.
    const int lc = N >= 16 ? l16 : (l16 < N ? l16 : N - 1);
    const int k_last0 = (n_chunks - 1) * BK;
    uint32_t off[8], off_last[8];
    bool k_real[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int k = 8 * grp + s;
        off[s] = (uint32_t)(((int64_t)k * ldw + lc) * 4);      // ldw is below 2^24 (checked on the host)
        k_real[s] = k_last0 + k < K;
        off_last[s] = (uint32_t)(((int64_t)(k_real[s] ? k : K - 1 - k_last0) * ldw + lc) * 4);
    }
    auto tile_col0 = [&](int tl) {   // first column of this wavefront's tile tl
        const int c0 = (wave_u + tl * AGG_WAVES) * 16;
        return N >= 16 ? (c0 < N - 16 ? c0 : N - 16) : 0;
    };
    // The weights of the next PF steps are on their way while a step's MFMAs run (one step is 16 or 32 MFMAs, far less
    // than a trip to L2): a ring of PF register sets, set d serving the chunks c with c % PF = d.  PF divides the chunks
    // of a tile (4, 2 or 1), and neither a fetch nor a store sits under a condition: the wavefront's memory operations
    // then come in one fixed order, and each wait is for exactly the set that is needed, with the later ones
    // still in flight.
    // NT: column tiles a wavefront works on at a time.  RAGGED: K is no multiple of 32 (only then the last chunk
    // needs its own offsets and drops values).
    const int a_off = l16 * ZS + 8 * grp;
    auto run = [&](auto pf, auto nt, auto ragged) {
        constexpr int PF = decltype(pf)::value;
        constexpr int NT = decltype(nt)::value;
        constexpr bool RAGGED = decltype(ragged)::value;
        const int my_groups = my_tiles / NT;
        doublex4 acc[NT][RT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int r = 0; r < RT; ++r) acc[t][r] = doublex4{0.0, 0.0, 0.0, 0.0};
        int ft = 0, fc = 0;   // tile group and chunk of the next fetch
        auto fetch_b = [&](float (&bv)[NT][8]) {
            const bool last = RAGGED && fc + 1 == n_chunks;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const char *base = reinterpret_cast<const char *>(W) + ((int64_t)fc * BK * ldw + tile_col0(ft * NT + t)) * 4;
#pragma unroll
                for (int s = 0; s < 8; ++s) bv[t][s] = *reinterpret_cast<const float *>(base + (last ? off_last[s] : off[s]));
            }
            // on to the next step; past the last one the position stays, and the fetch is repeated
            const bool wrap = fc + 1 == n_chunks;
            const int nft = ft + (wrap ? 1 : 0), nfc = wrap ? 0 : fc + 1;
            const bool end = nft >= my_groups;
            ft = end ? ft : nft;
            fc = end ? fc : nfc;
        };
        auto mfma_chunk = [&](int c, const float (&bj)[NT][8]) {
            float av[RT][8];
#pragma unroll
            for (int r = 0; r < RT; ++r) {
                const float *ap = &Zt[a_off + r * 16 * ZS + c * BK];
                const float4 x = *reinterpret_cast<const float4 *>(ap), y = *reinterpret_cast<const float4 *>(ap + 4);
                av[r][0] = x.x; av[r][1] = x.y; av[r][2] = x.z; av[r][3] = x.w;
                av[r][4] = y.x; av[r][5] = y.y; av[r][6] = y.z; av[r][7] = y.w;
            }
            // (no step is skipped, not even one of the last chunk in which every k is padding: a branch inside the loop
            // makes the compiler lose count of the fetches in flight, and it then waits for all of them at every step)
            const bool last = RAGGED && c + 1 == n_chunks;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                double a[RT];
#pragma unroll
                for (int r = 0; r < RT; ++r) a[r] = (double)av[r][s];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const float bs = (!last || k_real[s]) ? bj[t][s] : 0.f;
                    const double b = (double)bs;
#pragma unroll
                    for (int r = 0; r < RT; ++r) acc[t][r] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[r], b, acc[t][r], 0, 0, 0);
                }
            }
        };
        float bq[PF][NT][8];
        if (my_groups > 0) {
#pragma unroll
            for (int d = 0; d < PF; ++d) fetch_b(bq[d]);   // on their way while the block gathers its last rows
        }
        __syncthreads();                          // the tile is complete
        for (int tl = 0; tl < my_groups; ++tl) {
            for (int c0 = 0; c0 < n_chunks; c0 += PF) {
#pragma unroll
                for (int d = 0; d < PF; ++d) {
                    mfma_chunk(c0 + d, bq[d]);
                    fetch_b(bq[d]);               // this set's next turn
                }
            }
            // accumulator element i of lane l holds row l / 16 + 4 i, column l % 16 of its 16 x 16 tile
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int first_new = (wave_u + (tl * NT + t) * AGG_WAVES) * 16;   // columns before it belong to the tile before
                const int64_t col = (int64_t)tile_col0(tl * NT + t) + l16;
                const bool col_ok = col >= first_new && col < N;
#pragma unroll
                for (int r = 0; r < RT; ++r) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int64_t row = block_row0 + r * 16 + grp + 4 * i;
                        if (row < nS && col_ok) store_untracked(H + row * ldh + col, (float)acc[t][r][i]);
                    }
                    acc[t][r] = doublex4{0.0, 0.0, 0.0, 0.0};
                }
            }
        }
    };
    using std::integral_constant;
    auto pick_pf = [&](auto nt, auto ragged) {
        if (n_chunks % 4 == 0) run(integral_constant<int, 4>{}, nt, ragged);
        else if (n_chunks % 2 == 0) run(integral_constant<int, 2>{}, nt, ragged);
        else run(integral_constant<int, 1>{}, nt, ragged);
    };
    // (two column tiles at a time per wavefront, the conversions of A shared by two MFMAs, were measured: 168 instead
    // of 118 registers and no faster)
    if (K % BK == 0) pick_pf(integral_constant<int, 1>{}, std::false_type{});
    else pick_pf(integral_constant<int, 1>{}, std::true_type{});
    if (Zout) {   // the caller wants Z as well: rows below the count, K floats each (the tile is still whole)
        const int32_t rows_here = nS - block_row0 < FUSED_ROWS ? (int32_t)(nS - block_row0) : FUSED_ROWS;
        for (int i = tid; i < rows_here * K; i += AGG_BLOCK) {
            const int r = i / K, k = i % K;
            Zout[(block_row0 + r) * ldz + k] = Zt[r * ZS + k];
        }
    }
}

template <typename T, int KP>
static int launch_fused(const int32_t *rp, const int32_t *col, const float *val, int32_t nS, const int32_t *nsd, const int32_t *ncp,
                        const void *Xl, int64_t ldl, int64_t rl, const void *Xr, int64_t ldr, int64_t rr, const int32_t *src_row,
                        int32_t K, int relu, const float *W, int64_t ldw, int32_t N, float *H, int64_t ldh, float *Z, int64_t ldz,
                        int64_t z_stride, hipStream_t st, const CompInst &ci)
{
    const int64_t row_blocks = ((int64_t)nS + FUSED_ROWS - 1) / FUSED_ROWS;
    const dim3 grid((unsigned)row_blocks, 1, (unsigned)ci.n);
#define CSGS_FUSED_LAUNCH(RELU)                                                                                                  \
    CSGS_LAUNCH(K_LAYER_FORWARD, (layer_forward_k<T, KP, RELU>), grid, dim3(AGG_BLOCK), st, rp, col, val, nS, nsd, ncp, (const T *)Xl, ldl, \
                rl, (const T *)Xr, ldr, rr, src_row, K, W, ldw, N, H, ldh, Z, ldz, ci.cs, z_stride)
    if (relu) CSGS_FUSED_LAUNCH(true); else CSGS_FUSED_LAUNCH(false);
#undef CSGS_FUSED_LAUNCH
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

// Features per lane for an input width K (0: this kernel does not take it): 64 lanes cover a gathered row
static int fused_vec(int32_t K)
{
    if (K <= 64) return 1;
    if (K <= 128 && K % 2 == 0) return 2;
    if (K <= 256 && K % 4 == 0) return 4;
    return 0;
}

template <typename T>
static int pick_fused(int v, const int32_t *rp, const int32_t *col, const float *val, int32_t nS, const int32_t *nsd, const int32_t *ncp,
                      const void *Xl, int64_t ldl, int64_t rl, const void *Xr, int64_t ldr, int64_t rr, const int32_t *src_row, int32_t K,
                      int relu, const float *W, int64_t ldw, int32_t N, float *H, int64_t ldh, float *Z, int64_t ldz, int64_t z_stride,
                      hipStream_t st, const CompInst &ci)
{
#define CSGS_FUSED_KP(KP) launch_fused<T, KP>(rp, col, val, nS, nsd, ncp, Xl, ldl, rl, Xr, ldr, rr, src_row, K, relu, W, ldw, N, H, ldh, Z, ldz, z_stride, st, ci)
    if (v == 1) return CSGS_FUSED_KP(64);
    if (v == 2) return CSGS_FUSED_KP(128);
    return CSGS_FUSED_KP(256);
#undef CSGS_FUSED_KP
}

}  // namespace csgs

using namespace csgs;

extern "C" int csgs_layer_forward_supported(int32_t F_in, int dtype, int64_t ld_local, int64_t ld_remote)
{
    const int v = fused_vec(F_in);
    if (F_in <= 0 || v == 0 || (dtype != CSGS_F32 && dtype != CSGS_BF16)) return 0;
    return ld_local % v == 0 && ld_remote % v == 0 ? 1 : 0;
}

extern "C" int csgs_layer_forward_n(const csgs_inst_strides *inst, const int32_t *adj_rowptr, const int32_t *adj_col,
                                    const float *adj_val, int32_t nS, const int32_t *nS_dev, const int32_t *n_next,
                                    const void *X_local, int64_t ld_local, int64_t rows_local, const void *X_remote,
                                    int64_t ld_remote, int64_t rows_remote, const int32_t *src_row, int32_t F_in, int dtype,
                                    int relu_on_input, const float *W, int64_t ldw, int32_t F_out, float *H, int64_t ldh,
                                    float *Z, int64_t ldz, int64_t z_stride, void *stream)
{
    CompInst ci;
    if (open_instances(inst, &ci) != CSGS_OK) return CSGS_EINVAL;
    if (!adj_rowptr || !adj_col || !adj_val || nS <= 0 || F_in <= 0 || F_out <= 0 || rows_local < 0 || (rows_local > 0 && !X_local) ||
        (X_local && ld_local < F_in) || (X_remote && (ld_remote < F_in || rows_remote < 0)) || !W || ldw < F_out || !H || ldh < F_out ||
        (Z && ldz < F_in) || z_stride < 0 || (z_stride & 15))
        return CSGS_EINVAL;
    if (!X_remote) rows_remote = 0;
    if (!X_local || rows_local == 0) { X_local = nullptr; rows_local = 0; ld_local = F_in; }
    if (dtype != CSGS_F32 && dtype != CSGS_BF16) return CSGS_EUNSUPPORTED;
    if (rows_remote > 0x7FFFFFFEll) return CSGS_EUNSUPPORTED;   // staged rows are addressed as -1 - row in 32 bits
    const int v = fused_vec(F_in);
    if (v == 0 || ldw >= (1ll << 24)) return CSGS_EUNSUPPORTED;   // (the kernel keeps byte offsets into a 32-row chunk of W in 32 bits)
    // every gathered row must start on a multiple of the lanes' load width
    const uintptr_t bytes = (uintptr_t)v * (dtype == CSGS_F32 ? 4 : 2);
    if ((X_local && (ld_local % v != 0 || (uintptr_t)X_local % bytes != 0)) || (X_remote && (ld_remote % v != 0 || (uintptr_t)X_remote % bytes != 0)))
        return CSGS_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    if (dtype == CSGS_F32)
        return pick_fused<float>(v, adj_rowptr, adj_col, adj_val, nS, nS_dev, n_next, X_local, ld_local, rows_local, X_remote, ld_remote,
                                 rows_remote, src_row, F_in, relu_on_input, W, ldw, F_out, H, ldh, Z, ldz, z_stride, st, ci);
    return pick_fused<uint16_t>(v, adj_rowptr, adj_col, adj_val, nS, nS_dev, n_next, X_local, ld_local, rows_local, X_remote, ld_remote,
                                rows_remote, src_row, F_in, relu_on_input, W, ldw, F_out, H, ldh, Z, ldz, z_stride, st, ci);
}

extern "C" int csgs_layer_forward(const int32_t *adj_rowptr, const int32_t *adj_col, const float *adj_val, int32_t nS,
                                  const int32_t *nS_dev, const int32_t *n_next, const void *X_local, int64_t ld_local,
                                  int64_t rows_local, const void *X_remote, int64_t ld_remote, int64_t rows_remote,
                                  const int32_t *src_row, int32_t F_in, int dtype, int relu_on_input, const float *W, int64_t ldw,
                                  int32_t F_out, float *H, int64_t ldh, float *Z, int64_t ldz, void *stream)
{
    return csgs_layer_forward_n(nullptr, adj_rowptr, adj_col, adj_val, nS, nS_dev, n_next, X_local, ld_local, rows_local, X_remote,
                                ld_remote, rows_remote, src_row, F_in, dtype, relu_on_input, W, ldw, F_out, H, ldh, Z, ldz, 0, stream);
}
