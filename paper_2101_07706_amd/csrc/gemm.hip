// csgs_layer_gemm: H = Z W (Section 3, Eq. 1), fp32 in, fp32 out, fp64 matrix-core accumulation.
//
// Why double: sampled rows carry 1/p_j discounts that compound over the layers, so the products
// z*w of a near-cancelling output reach magnitude 10 and more while the tolerance is 1e-5
// absolute.  fp32 MFMA with double master accumulators over runs of 32 k was measured to miss it
// (5.9e-5 against 3.5e-5 allowed on one output of the largest configuration).  The operands are
// widened to double after the LDS read (exact), products of two 24-bit mantissas are exact in
// double, and v_mfma_f64_16x16x4_f64 accumulates in double, so the only rounding is the final
// conversion to float.
//
// Block tile BM (128, or 64 where that would leave too few blocks) x BN (64 or 32), K chunks of 32,
// four wavefronts stacked along M, each owning a BM/4 x BN strip = BM/64 x BN/16 MFMA tiles of
// 16 x 16.  Global -> register -> LDS with the next chunk's loads in flight during the current
// chunk's MFMAs (two LDS buffers).  Every load of a tile is unconditional (a piece that does not
// exist reads a clamped address and becomes zero on the way to LDS); a row count that lives on the
// device gates only the early exit and the stores.
//
// LDS layout (fp32): A row-major [BM][36], B transposed [BN][36] (k contiguous, 16-byte aligned
// rows whose stride of 36 words spreads 16 lanes' 128-bit reads over all 64 banks); in the
// 128 x 64 blocks of the forward product B has rows of 32 words with the 16-byte columns swizzled
// instead, which brings a block to 52-53 KB and three blocks onto a compute unit.  The k order
// inside a chunk is permuted -- the lane group l / 16 = g feeds k = 8 g + s at step s, for both
// operands alike, which leaves the sum unchanged -- so that every lane fetches the 8 values it
// needs per operand row with two 128-bit LDS reads.
//
// Block ids are remapped so that consecutive tiles (same rows of Z, neighbouring column tiles)
// land on the same XCD and share its L2.
#include <type_traits>
#include "common.hpp"

#include "gemm_tile.hpp"

namespace csgs {

// TAIL (forward product only, K = 32 n + 1 .. 4 with n >= 1): the last 1 .. 4 k do not get a chunk of
// their own, whose loads, barrier and LDS reads would cost as much as a full one (100 input features
// are three chunks and four k).  They are loaded once, before the first barrier, into the four padding
// words of the rows of the LDS buffer that will hold the last chunk, and take one MFMA step after it,
// in which lane group g feeds k = 32 n + g.
template <int BN, int MODE, int V, bool FULL, bool TAIL = false, int BM_ = 128>
__global__ __launch_bounds__(256, (MODE == MODE_FWD && BM_ == 128 && BN == 64) ? 3 : 2) void gemm_f32_k(const float *__restrict__ A, int64_t lda,
                                                  const float *__restrict__ Bm, int64_t ldb, float *__restrict__ C,
                                                  int64_t ldc, double *__restrict__ partial, int M_bound, int N,
                                                  int K_bound, const int32_t *__restrict__ rows_dev, int n_tiles_n,
                                                  int n_tiles, int k_split, CompStride cs)
{
    A = inst_ptr(A, cs.x); C = inst_ptr(C, cs.out); rows_dev = inst_ptr(rows_dev, cs.adj);   // B (the weights) is shared
    constexpr int NT = BN / 16;   // 16-column MFMA tiles per wavefront
    constexpr int RT = BM_ / 64;  // 16-row MFMA tiles per wavefront: the four wavefronts are stacked along M
    static_assert(BM_ == 128 || BM_ == 64, "block tiles of 128 or 64 rows");
    constexpr bool A_KMAJOR = MODE != MODE_DW, B_KMAJOR = MODE == MODE_DZ;
    __shared__ __attribute__((aligned(16))) float As[2][BM_ * LDS_STRIDE];
    // The B tile of the forward product's 128 x 64 blocks is swizzled instead of padded: 52-53 KB of LDS per block
    // instead of 54, which lets a third block onto a compute unit (the launch bound asks the compiler for the
    // 168 registers that go with it)
    constexpr bool SWZ = MODE == MODE_FWD && BM_ == 128 && BN == 64;
    constexpr int B_STRIDE = SWZ ? BK : LDS_STRIDE;
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * B_STRIDE];
    __shared__ float Bt[(TAIL && SWZ) ? BN * 4 : 1];   // the K tail of B where its rows have no padding
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int grp = lane >> 4, l16 = lane & 15;
    // XCD-aware tile order: hardware deals consecutive block ids round-robin to the 8 XCDs
    const int bid = (int)blockIdx.x;
    const int per_xcd = (n_tiles + 7) / 8;
    // (rotated by the instance: the row tiles beyond a mini-batch's row count are the last ones, and with the
    // same order for every instance they would all fall to the same XCD, which then idles)
    const int tile = (((bid & 7) + (int)blockIdx.z) & 7) * per_xcd + (bid >> 3);
    if (tile >= n_tiles) return;
    const int64_t m0 = (int64_t)(tile / n_tiles_n) * BM_, n0 = (int64_t)(tile % n_tiles_n) * BN;
    // the row count of the sampled layer may live on the device: it bounds M, or K for dW.  As a bound
    // of M it is only needed once the first chunk's loads are on their way (see below)
    const int m_dev = (MODE != MODE_DW && rows_dev) ? *rows_dev : M_bound;
    const int K = MODE == MODE_DW ? resolve_count(K_bound, rows_dev) : K_bound;
    const int k_begin = MODE == MODE_DW ? (int)blockIdx.y * k_split : 0;
    const int k_end = MODE == MODE_DW ? (k_begin + k_split < K ? k_begin + k_split : K) : K;
    static_assert(!TAIL || MODE == MODE_FWD, "the folded tail is for forward products");
    const int n_chunks = TAIL ? (k_end - k_begin) / BK : (k_end > k_begin ? (k_end - k_begin + BK - 1) / BK : 0);

    doublex4 acc[RT][NT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = doublex4{0.0, 0.0, 0.0, 0.0};
    float4 ra[BM_ / 32], rb[BN / 32];
    uint32_t oka = 0, okb = 0;
    // Rows of A up to M_bound are the caller's memory whatever the device count says, and a row of A
    // only reaches its own row of C, which is not stored beyond the count: so the count never masks a
    // load, and the first chunk's loads need not wait for it.
    const bool a_whole = m0 + BM_ <= M_bound, b_whole = n0 + BN <= N;
    bool k_whole = false;   // of the chunk in the registers
    auto fetch = [&](int k0) {
        k_whole = k0 + BK <= k_end;
        if (A_KMAJOR) fetch_kmajor<BM_, V, FULL>(A, lda, M_bound, k_end, m0, k0, tid, ra, oka);
        else fetch_rmajor<BM_, FULL>(A, lda, M_bound, k_end, m0, k0, tid, ra, oka);
        if (B_KMAJOR) fetch_kmajor<BN, V, FULL>(Bm, ldb, N, k_end, n0, k0, tid, rb, okb);
        else fetch_rmajor<BN, FULL>(Bm, ldb, N, k_end, n0, k0, tid, rb, okb);
    };
    auto stash = [&](int buf) {
        stash_tile<BM_, A_KMAJOR, FULL>(As[buf], tid, ra, oka, a_whole && k_whole);
        stash_tile<BN, B_KMAJOR, FULL, SWZ>(Bs[buf], tid, rb, okb, b_whole && k_whole);
    };
    if (n_chunks > 0) fetch(k_begin);
    // the K tail's loads travel with the first chunk's (unconditional, clamped addresses; threads beyond the
    // tail's extent read a stand-in and store nothing): one load latency before the first barrier, not two
    float ta0 = 0.f, ta1 = 0.f, tb = 0.f;
    const int kt = k_begin + n_chunks * BK, tail = k_end - kt;
    const int tr = (tid >> 1) < BM_ ? (tid >> 1) : BM_ - 1, tj0 = (tid & 1) * 2;   // A: BM_ rows x 4 k, two floats per thread
    const int tn = tid % BN, tj = (tid / BN) & 3;                                  // B: 4 k x BN columns, one float per thread
    if (TAIL) {
        const int64_t gr = m0 + tr;
        const float *row = A + (gr < M_bound ? gr : (int64_t)M_bound - 1) * lda;
        ta0 = row[tj0 < tail ? kt + tj0 : k_end - 1];
        ta1 = row[tj0 + 1 < tail ? kt + tj0 + 1 : k_end - 1];
        const int64_t gn = n0 + tn;
        tb = Bm[(int64_t)(tj < tail ? kt + tj : k_end - 1) * ldb + (gn < N ? gn : (int64_t)N - 1)];
    }
    const int M = m_dev < 0 ? 0 : (m_dev < M_bound ? m_dev : M_bound);
    if (m0 >= M) return;  // the whole block leaves together, before any barrier
    if (n_chunks > 0) stash(0);
    if (TAIL) {
        const int last = (n_chunks - 1) & 1;
        if (tid < BM_ * 2) {
            const bool row_ok = m0 + tr < M_bound;
            As[last][tr * LDS_STRIDE + BK + tj0] = (row_ok && tj0 < tail) ? ta0 : 0.f;
            As[last][tr * LDS_STRIDE + BK + tj0 + 1] = (row_ok && tj0 + 1 < tail) ? ta1 : 0.f;
        }
        if (tid < BN * 4) {
            const bool ok = n0 + tn < N && tj < tail;
            if (SWZ) Bt[tn * 4 + tj] = ok ? tb : 0.f;
            else Bs[last][tn * LDS_STRIDE + BK + tj] = ok ? tb : 0.f;
        }
    }
    __syncthreads();
    const int a_off = (wave * (BM_ / 4) + l16) * LDS_STRIDE + 8 * grp;
    const int b_off = l16 * LDS_STRIDE + 8 * grp;
    const int bx_off = l16 * BK + (((2 * grp) ^ ((l16 >> 1) & 7)) << 2), by_off = l16 * BK + (((2 * grp + 1) ^ ((l16 >> 1) & 7)) << 2);
    // 16-column MFMA tiles of this block that hold any real column (47 output classes fill 3 of 4), and
    // k steps of the last chunk that hold any real k (lane group g feeds k = 8 g + s at step s, so with
    // k_left <= 8 only the first k_left steps of group 0 are not padding): the rest would multiply zeros
    // (a regular shape has neither: then nothing in the chunk loop sits under a condition, and the compiler is free to
    // order the conversions, the MFMAs and the next chunk's loads)
    const int nt_valid = FULL ? NT : (int)(N - n0 >= BN ? NT : (N - n0 + 15) / 16);
    const int k_left = n_chunks > 0 ? (k_end - k_begin) - (n_chunks - 1) * BK : 0;
    const int s_last = (FULL || k_left >= 8) ? 8 : k_left;
    for (int c = 0; c < n_chunks; ++c) {
        const int cur = c & 1;
        if (c + 1 < n_chunks) fetch(k_begin + (c + 1) * BK);
        float av[RT][8], bv[NT][8];
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            const float *ap = &As[cur][a_off + r * 16 * LDS_STRIDE];
            const float4 x = *reinterpret_cast<const float4 *>(ap), y = *reinterpret_cast<const float4 *>(ap + 4);
            av[r][0] = x.x; av[r][1] = x.y; av[r][2] = x.z; av[r][3] = x.w;
            av[r][4] = y.x; av[r][5] = y.y; av[r][6] = y.z; av[r][7] = y.w;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float4 x, y;
            if (SWZ) {   // row 16 t + l16: its swizzle (row >> 1) & 7 does not depend on t
                x = *reinterpret_cast<const float4 *>(&Bs[cur][bx_off + t * 16 * BK]);
                y = *reinterpret_cast<const float4 *>(&Bs[cur][by_off + t * 16 * BK]);
            } else {
                const float *bp = &Bs[cur][b_off + t * 16 * LDS_STRIDE];
                x = *reinterpret_cast<const float4 *>(bp);
                y = *reinterpret_cast<const float4 *>(bp + 4);
            }
            bv[t][0] = x.x; bv[t][1] = x.y; bv[t][2] = x.z; bv[t][3] = x.w;
            bv[t][4] = y.x; bv[t][5] = y.y; bv[t][6] = y.z; bv[t][7] = y.w;
        }
        const int s_end = (FULL || c + 1 < n_chunks) ? 8 : s_last;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            if (FULL || s < s_end) {
                double a[RT];
#pragma unroll
                for (int r = 0; r < RT; ++r) a[r] = (double)av[r][s];
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    if (FULL || t < nt_valid) {
                        const double b = (double)bv[t][s];
#pragma unroll
                        for (int r = 0; r < RT; ++r) acc[r][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[r], b, acc[r][t], 0, 0, 0);
                    }
                }
            }
        }
        if (c + 1 < n_chunks) {
            stash(cur ^ 1);
            __syncthreads();
        }
    }
    if (TAIL) {
        const int last = (n_chunks - 1) & 1;
        double a[RT];
#pragma unroll
        for (int r = 0; r < RT; ++r) a[r] = (double)As[last][(wave * (BM_ / 4) + r * 16 + l16) * LDS_STRIDE + BK + grp];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (FULL || t < nt_valid) {
                const double b = (double)(SWZ ? Bt[(t * 16 + l16) * 4 + grp] : Bs[last][(t * 16 + l16) * LDS_STRIDE + BK + grp]);
#pragma unroll
                for (int r = 0; r < RT; ++r) acc[r][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[r], b, acc[r][t], 0, 0, 0);
            }
        }
    }
    // accumulator element i of lane l holds row l / 16 + 4 * i, column l % 16 of its 16 x 16 tile
    auto store = [&](auto whole) {
        constexpr bool WHOLE = decltype(whole)::value;
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int64_t row = m0 + wave * (BM_ / 4) + r * 16 + grp + 4 * i;
                if (WHOLE || row < M) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) {
                        const int64_t col = n0 + t * 16 + l16;
                        if (WHOLE || col < N) {
                            if (MODE == MODE_DW)
                                partial[((int64_t)blockIdx.y * M_bound + row) * N + col] = acc[r][t][i];
                            else
                                C[row * ldc + col] = (float)acc[r][t][i];
                        }
                    }
                }
            }
    };
    if (m0 + BM_ <= M && (FULL || n0 + BN <= N)) store(std::true_type{});
    else store(std::false_type{});
}

// dW[i] = sum over the K parts, in ascending part order (fixed: the result does not depend on timing)
__global__ __launch_bounds__(256) void gemm_reduce_parts(const double *__restrict__ partial, int parts, int64_t count,
                                                         int N, float *__restrict__ C, int64_t ldc)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= count) return;
    double s = 0.0;
    int p = 0;
    for (; p + 8 <= parts; p += 8) {   // eight loads in flight, added in ascending part order
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(p + u) * count + i];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; p < parts; ++p) s += partial[(int64_t)p * count + i];
    C[(i / N) * ldc + (i % N)] = (float)s;
}

// Widest vector (in floats) that loads rows of `k` floats, `ld` apart, in whole pieces
static int widest(const float *p, int64_t ld, int k)
{
    if (ld % 4 == 0 && k % 4 == 0 && ((uintptr_t)p & 15) == 0) return 4;
    if (ld % 2 == 0 && k % 2 == 0 && ((uintptr_t)p & 7) == 0) return 2;
    return 1;
}

template <int BMF, int BN>
static void launch_fwd(const float *Z, int64_t ldz, int M, const int32_t *M_dev, int K, const float *W, int64_t ldw, int N, float *H,
                       int64_t ldh, hipStream_t st, const CompInst &ci)
{
    const int tm = (M + BMF - 1) / BMF, tn = (N + BN - 1) / BN;
    const int n_tiles = tm * tn;
    const dim3 grid((unsigned)(((n_tiles + 7) / 8) * 8), 1, (unsigned)ci.n);
    const int va = widest(Z, ldz, K);
    const bool fold = K > BK && K % BK >= 1 && K % BK <= 4;   // see TAIL
    // regular shape (of the bounds: a device count only gates the stores); a folded tail leaves whole chunks
    const bool full = M % BMF == 0 && N % BN == 0 && (K % BK == 0 || fold) && va == 4;
    double *none = nullptr;
#define CSGS_GEMM_FWD(V, FULL, TAIL) \
    CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, MODE_FWD, V, FULL, TAIL, BMF>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, none, M, N, K, M_dev, tn, n_tiles, 0, ci.cs)
    if (full && fold) CSGS_GEMM_FWD(4, true, true);
    else if (full) CSGS_GEMM_FWD(4, true, false);
    else if (fold && va == 4) CSGS_GEMM_FWD(4, false, true);
    else if (fold && va == 2) CSGS_GEMM_FWD(2, false, true);
    else if (fold) CSGS_GEMM_FWD(1, false, true);
    else if (va == 4) CSGS_GEMM_FWD(4, false, false);
    else if (va == 2) CSGS_GEMM_FWD(2, false, false);
    else CSGS_GEMM_FWD(1, false, false);
#undef CSGS_GEMM_FWD
}

template <int BN>
static void launch_dz(const float *G, int64_t ldg, int M, const int32_t *M_dev, int K, const float *W, int64_t ldw, int N, float *dZ,
                      int64_t lddz, hipStream_t st)
{
    const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
    const int n_tiles = tm * tn;
    const dim3 grid((unsigned)(((n_tiles + 7) / 8) * 8));
    const int v = widest(G, ldg, K) == 4 && widest(W, ldw, K) == 4 ? 4 : 1;
    double *none = nullptr;
    if (v == 4)
        CSGS_LAUNCH(K_GEMM_DZ, (gemm_f32_k<BN, MODE_DZ, 4, false>), grid, dim3(256), st, G, ldg, W, ldw, dZ, lddz, none, M, N, K, M_dev, tn, n_tiles, 0, CompStride{0, 0, 0, 0});
    else
        CSGS_LAUNCH(K_GEMM_DZ, (gemm_f32_k<BN, MODE_DZ, 1, false>), grid, dim3(256), st, G, ldg, W, ldw, dZ, lddz, none, M, N, K, M_dev, tn, n_tiles, 0, CompStride{0, 0, 0, 0});
}

// Parts of the reduction dimension for dW = Z^T G with `rows` rows: enough blocks to fill the device,
// each part a multiple of the K chunk.
static void dw_split(int rows, int tiles, int *parts, int *k_split)
{
    int want = (512 + tiles - 1) / tiles;
    const int max_parts = (rows + BK - 1) / BK;
    if (want > max_parts) want = max_parts;
    if (want < 1) want = 1;
    int ks = ((rows + want - 1) / want + BK - 1) / BK * BK;
    if (ks < BK) ks = BK;
    *k_split = ks;
    *parts = (rows + ks - 1) / ks;
    if (*parts < 1) *parts = 1;
}

}  // namespace csgs

using namespace csgs;

extern "C" int csgs_layer_gemm(const float *Z, int64_t ldz, int32_t M, const int32_t *M_dev, int32_t K, const float *W, int64_t ldw,
                               int32_t Nout, float *H, int64_t ldh, void *stream)
{
    return csgs_layer_gemm_n(nullptr, Z, ldz, M, M_dev, K, W, ldw, Nout, H, ldh, stream);
}

extern "C" int csgs_layer_gemm_n(const csgs_inst_strides *inst, const float *Z, int64_t ldz, int32_t M, const int32_t *M_dev,
                                 int32_t K, const float *W, int64_t ldw, int32_t Nout, float *H, int64_t ldh, void *stream)
{
    if (!Z || !W || !H || M <= 0 || K <= 0 || Nout <= 0 || ldz < K || ldw < Nout || ldh < Nout) return CSGS_EINVAL;
    CompInst ci;
    if (open_instances(inst, &ci) != CSGS_OK) return CSGS_EINVAL;
    const int64_t tm = ((int64_t)M + BM - 1) / BM;
    if (tm * (((int64_t)Nout + 31) / 32) > 0x3FFFFFFF) return CSGS_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    // Tiles of 128 x 64 where they give at least two blocks per compute unit; else 64 rows (twice the
    // blocks: 18 against 20 us per launch for one mini-batch of the named configuration; with 512 tiles
    // of 128 rows, the narrow output layer of 8 mini-batches, 64-row tiles are 2 us slower); narrow column
    // tiles when even those would leave fewer than two blocks per compute unit
    const int64_t wide_tiles = tm * (((int64_t)Nout + 63) / 64);
    const int64_t tm64 = ((int64_t)M + 63) / 64;
    if (wide_tiles * ci.n >= 512 && Nout > 32)
        launch_fwd<128, 64>(Z, ldz, M, M_dev, K, W, ldw, Nout, H, ldh, st, ci);
    else if (tm64 * (((int64_t)Nout + 63) / 64) * ci.n >= 512 && Nout > 32)
        launch_fwd<64, 64>(Z, ldz, M, M_dev, K, W, ldw, Nout, H, ldh, st, ci);
    else
        launch_fwd<64, 32>(Z, ldz, M, M_dev, K, W, ldw, Nout, H, ldh, st, ci);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_layer_gemm_grad_z(const float *G, int64_t ldg, int32_t M, const int32_t *M_dev, int32_t Nout, const float *W,
                                      int64_t ldw, int32_t K, float *dZ, int64_t lddz, void *stream)
{
    if (!G || !W || !dZ || M <= 0 || K <= 0 || Nout <= 0 || ldg < Nout || ldw < Nout || lddz < K) return CSGS_EINVAL;
    const int64_t tm = ((int64_t)M + BM - 1) / BM;
    if (tm * (((int64_t)K + 31) / 32) > 0x3FFFFFFF) return CSGS_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    // output [M x K]; the reduction runs over the Nout columns of G
    const int64_t wide_tiles = tm * (((int64_t)K + 63) / 64);
    if (wide_tiles >= 512 && K > 32)
        launch_dz<64>(G, ldg, M, M_dev, Nout, W, ldw, K, dZ, lddz, st);
    else
        launch_dz<32>(G, ldg, M, M_dev, Nout, W, ldw, K, dZ, lddz, st);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" size_t csgs_layer_gemm_grad_w_scratch_bytes(int32_t M, int32_t K, int32_t Nout)
{
    if (M <= 0 || K <= 0 || Nout <= 0) return 0;
    const int tiles = ((K + BM - 1) / BM) * ((Nout + 31) / 32);
    int parts, ks;
    dw_split(M, tiles, &parts, &ks);
    return (size_t)parts * (size_t)K * (size_t)Nout * sizeof(double);
}

// dW = Z^T G with the partial sums in `parts` (device, at least csgs_layer_gemm_grad_w_scratch_bytes bytes)
static int grad_w_launch(const float *Z, int64_t ldz, const float *G, int64_t ldg, int32_t M, const int32_t *M_dev, int32_t K,
                         int32_t Nout, float *dW, int64_t lddw, double *parts_buf, hipStream_t st)
{
    // kernel terms: output [K x Nout], reduction over the M rows (their count may live on the device)
    const int tm = (K + BM - 1) / BM, tn = (Nout + 31) / 32;
    const int n_tiles = tm * tn;
    int parts, ks;
    dw_split(M, n_tiles, &parts, &ks);
    const dim3 grid((unsigned)(((n_tiles + 7) / 8) * 8), (unsigned)parts);
    float *none = nullptr;
    CSGS_LAUNCH(K_GEMM_DW, (gemm_f32_k<32, MODE_DW, 1, false>), grid, dim3(256), st, Z, ldz, G, ldg, none, (int64_t)0,
                parts_buf, K, Nout, M, M_dev, tn, n_tiles, ks, CompStride{0, 0, 0, 0});
    CSGS_LAUNCH_CHECK();
    const int64_t count = (int64_t)K * Nout;
    CSGS_LAUNCH(K_GEMM_DW_REDUCE, gemm_reduce_parts, dim3((unsigned)((count + 255) / 256)), dim3(256), st,
                (const double *)parts_buf, parts, count, Nout, dW, lddw);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_layer_gemm_grad_w(const float *Z, int64_t ldz, const float *G, int64_t ldg, int32_t M, const int32_t *M_dev,
                                      int32_t K, int32_t Nout, float *dW, int64_t lddw, void *scratch, size_t scratch_bytes,
                                      void *stream)
{
    if (!Z || !G || !dW || M <= 0 || K <= 0 || Nout <= 0 || ldz < K || ldg < Nout || lddw < Nout || !scratch ||
        ((uintptr_t)scratch & 7))
        return CSGS_EINVAL;
    if (scratch_bytes < csgs_layer_gemm_grad_w_scratch_bytes(M, K, Nout)) return CSGS_EWORKSPACE;
    return grad_w_launch(Z, ldz, G, ldg, M, M_dev, K, Nout, dW, lddw, (double *)scratch, (hipStream_t)stream);
}

// ---------------------------------------------------------------- the same without any allocation
// The partial sums of csgs_layer_gemm_grad_w_static live in this array, which is part of the library's
// device image: every device the library runs on holds its own copy, at its own address, until the
// process ends.  Host code never uses the array's name as an address; the address on the current
// device is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[CSGS_GRAD_W_STATIC_BYTES];
static std::atomic<void *> g_static_scratch[64];   // per device; null = not looked up yet (zero-initialised)

// Address of `scratch` on the current device, or null.
static void *static_scratch_ptr()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    void *p = g_static_scratch[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_static_scratch[dev].store(p, std::memory_order_release);   // every thread would store the same address
    }
    return p;
}

extern "C" int csgs_layer_gemm_grad_w_static(const float *Z, int64_t ldz, const float *G, int64_t ldg, int32_t M,
                                             const int32_t *M_dev, int32_t K, int32_t Nout, float *dW, int64_t lddw, void *stream)
{
    if (!Z || !G || !dW || M <= 0 || K <= 0 || Nout <= 0 || ldz < K || ldg < Nout || lddw < Nout) return CSGS_EINVAL;
    if (csgs_layer_gemm_grad_w_scratch_bytes(M, K, Nout) > (size_t)CSGS_GRAD_W_STATIC_BYTES) return CSGS_EWORKSPACE;
    void *parts_buf = static_scratch_ptr();
    if (!parts_buf) return CSGS_ELAUNCH;
    // every part that the reduction reads is written by the product kernel of the same call: nothing to clear
    return grad_w_launch(Z, ldz, G, ldg, M, M_dev, K, Nout, dW, lddw, (double *)parts_buf, (hipStream_t)stream);
}

static const char *const kErr[] = {"ok",
                                   "invalid argument",
                                   "workspace too small",
                                   "unsupported dtype or dimension",
                                   "fixed-point format out of range",
                                   "kernel launch failed"};

extern "C" const char *csgs_strerror(int code)
{
    const int i = -code;
    return (i >= 0 && i < (int)(sizeof(kErr) / sizeof(kErr[0]))) ? kErr[i] : "unknown error";
}
