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
// Block tile 128 (M) x BN (64 or 32), K chunks of 32, four wavefronts stacked along M, each
// owning a 32 x BN strip = 2 x BN/16 MFMA tiles of 16 x 16.  Global -> register -> LDS with the
// next chunk's loads in flight during the current chunk's MFMAs (two LDS buffers).
//
// LDS layout (fp32): A row-major [128][36], B transposed [BN][36] (k contiguous, 16-byte aligned
// rows whose stride of 36 words spreads 16 lanes' 128-bit reads over all 64 banks).  The k order
// inside a chunk is permuted -- the lane group l / 16 = g feeds k = 8 g + s at step s, for both
// operands alike, which leaves the sum unchanged -- so that every lane fetches the 8 values it
// needs per operand row with two 128-bit LDS reads.
//
// Block ids are remapped so that consecutive tiles (same rows of Z, neighbouring column tiles)
// land on the same XCD and share its L2.
#include "common.hpp"

namespace csgs {

typedef double doublex4 __attribute__((ext_vector_type(4)));

constexpr int BM = 128, BK = 32;
constexpr int LDS_STRIDE = BK + 4;

template <int V>
__device__ inline float4 load4(const float *__restrict__ p)
{
    if (V == 4) return *reinterpret_cast<const float4 *>(p);
    if (V == 2) {
        const float2 a = *reinterpret_cast<const float2 *>(p);
        const float2 b = *reinterpret_cast<const float2 *>(p + 2);
        return make_float4(a.x, a.y, b.x, b.y);
    }
    return make_float4(p[0], p[1], p[2], p[3]);
}

// A chunk: 128 rows x 32 k = 1024 groups of 4 consecutive k; thread t takes groups t + 256 i.
template <int VA, bool FULL>
__device__ inline void fetch_a(const float *__restrict__ A, int64_t lda, int M, int K, int64_t m0, int k0, int tid,
                               float4 (&ra)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + i * 256;
        const int r = idx >> 3, kq = (idx & 7) * 4;
        const int64_t gm = m0 + r;
        const int gk = k0 + kq;
        if (FULL || (gm < M && gk + 3 < K)) {
            ra[i] = load4<VA>(A + gm * lda + gk);
        } else {
            float t[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) t[j] = (gm < M && gk + j < K) ? A[gm * lda + gk + j] : 0.f;
            ra[i] = make_float4(t[0], t[1], t[2], t[3]);
        }
    }
}

// B chunk: 32 k x BN columns.  Lane <-> column (coalesced across lanes), each thread takes runs of
// 4 consecutive k of one column, which become one 128-bit store into the transposed LDS tile.
template <int BN, bool FULL>
__device__ inline void fetch_b(const float *__restrict__ Bm, int64_t ldb, int K, int N, int k0, int64_t n0, int tid,
                               float4 (&rb)[BN / 32])
{
#pragma unroll
    for (int i = 0; i < BN / 32; ++i) {
        const int idx = tid + i * 256;          // BN * 8 groups
        const int n = idx % BN, kg = (idx / BN) * 4;
        const int64_t gn = n0 + n;
        const int gk = k0 + kg;
        float t[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) t[j] = (FULL || (gn < N && gk + j < K)) ? Bm[(int64_t)(gk + j) * ldb + gn] : 0.f;
        rb[i] = make_float4(t[0], t[1], t[2], t[3]);
    }
}

template <int BN>
__device__ inline void stash(float *As, float *Bs, int tid, const float4 (&ra)[4], const float4 (&rb)[BN / 32])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int idx = tid + i * 256;
        const int r = idx >> 3, kq = (idx & 7) * 4;
        *reinterpret_cast<float4 *>(&As[r * LDS_STRIDE + kq]) = ra[i];
    }
#pragma unroll
    for (int i = 0; i < BN / 32; ++i) {
        const int idx = tid + i * 256;
        const int n = idx % BN, kg = (idx / BN) * 4;
        *reinterpret_cast<float4 *>(&Bs[n * LDS_STRIDE + kg]) = rb[i];
    }
}

template <int BN, int VA, bool FULL>
__global__ __launch_bounds__(256) void gemm_f32_k(const float *__restrict__ A, int64_t lda,
                                                  const float *__restrict__ Bm, int64_t ldb, float *__restrict__ C,
                                                  int64_t ldc, int M_bound, const int32_t *__restrict__ M_dev, int N,
                                                  int K, int n_tiles_n, int n_tiles)
{
    constexpr int NT = BN / 16;   // 16-column MFMA tiles per wavefront (times 2 row tiles)
    __shared__ __attribute__((aligned(16))) float As[2][BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * LDS_STRIDE];
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int grp = lane >> 4, l16 = lane & 15;
    // XCD-aware tile order: hardware deals consecutive block ids round-robin to the 8 XCDs
    const int bid = (int)blockIdx.x;
    const int per_xcd = (n_tiles + 7) / 8;
    const int tile = (bid & 7) * per_xcd + (bid >> 3);
    if (tile >= n_tiles) return;
    const int64_t m0 = (int64_t)(tile / n_tiles_n) * BM, n0 = (int64_t)(tile % n_tiles_n) * BN;
    const int M = resolve_count(M_bound, M_dev);
    if (m0 >= M) return;  // the whole block leaves together, before any barrier

    doublex4 acc[2][NT];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = doublex4{0.0, 0.0, 0.0, 0.0};
    float4 ra[4], rb[BN / 32];
    const int n_chunks = (K + BK - 1) / BK;
    fetch_a<VA, FULL>(A, lda, M, K, m0, 0, tid, ra);
    fetch_b<BN, FULL>(Bm, ldb, K, N, 0, n0, tid, rb);
    stash<BN>(As[0], Bs[0], tid, ra, rb);
    __syncthreads();
    const int a_off = (wave * 32 + l16) * LDS_STRIDE + 8 * grp;
    const int b_off = l16 * LDS_STRIDE + 8 * grp;
    for (int c = 0; c < n_chunks; ++c) {
        const int cur = c & 1;
        if (c + 1 < n_chunks) {
            fetch_a<VA, FULL>(A, lda, M, K, m0, (c + 1) * BK, tid, ra);
            fetch_b<BN, FULL>(Bm, ldb, K, N, (c + 1) * BK, n0, tid, rb);
        }
        float av[2][8], bv[NT][8];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const float *ap = &As[cur][a_off + r * 16 * LDS_STRIDE];
            const float4 x = *reinterpret_cast<const float4 *>(ap), y = *reinterpret_cast<const float4 *>(ap + 4);
            av[r][0] = x.x; av[r][1] = x.y; av[r][2] = x.z; av[r][3] = x.w;
            av[r][4] = y.x; av[r][5] = y.y; av[r][6] = y.z; av[r][7] = y.w;
        }
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const float *bp = &Bs[cur][b_off + t * 16 * LDS_STRIDE];
            const float4 x = *reinterpret_cast<const float4 *>(bp), y = *reinterpret_cast<const float4 *>(bp + 4);
            bv[t][0] = x.x; bv[t][1] = x.y; bv[t][2] = x.z; bv[t][3] = x.w;
            bv[t][4] = y.x; bv[t][5] = y.y; bv[t][6] = y.z; bv[t][7] = y.w;
        }
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const double a0 = (double)av[0][s], a1 = (double)av[1][s];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const double b = (double)bv[t][s];
                acc[0][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b, acc[0][t], 0, 0, 0);
                acc[1][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b, acc[1][t], 0, 0, 0);
            }
        }
        if (c + 1 < n_chunks) {
            stash<BN>(As[cur ^ 1], Bs[cur ^ 1], tid, ra, rb);
            __syncthreads();
        }
    }
    // accumulator element i of lane l holds row l / 16 + 4 * i, column l % 16 of its 16 x 16 tile
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int64_t row = m0 + wave * 32 + r * 16 + grp + 4 * i;
            if (FULL || row < M) {
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const int64_t col = n0 + t * 16 + l16;
                    if (FULL || col < N) C[row * ldc + col] = (float)acc[r][t][i];
                }
            }
        }
}

static int widest(const float *p, int64_t ld)
{
    if (ld % 4 == 0 && ((uintptr_t)p & 15) == 0) return 4;
    if (ld % 2 == 0 && ((uintptr_t)p & 7) == 0) return 2;
    return 1;
}

template <int BN>
static void launch_gemm(const float *Z, int64_t ldz, int M, const int32_t *M_dev, int K, const float *W, int64_t ldw, int N, float *H,
                        int64_t ldh, hipStream_t st)
{
    const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
    const int n_tiles = tm * tn;
    const dim3 grid((unsigned)(((n_tiles + 7) / 8) * 8));
    const int va = widest(Z, ldz);
    const bool full = !M_dev && M % BM == 0 && N % BN == 0 && K % BK == 0 && va == 4;
    if (full)
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, 4, true>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, M_dev, N, K, tn, n_tiles);
    else if (va == 4)
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, 4, false>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, M_dev, N, K, tn, n_tiles);
    else if (va == 2)
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, 2, false>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, M_dev, N, K, tn, n_tiles);
    else
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, 1, false>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, M_dev, N, K, tn, n_tiles);
}

}  // namespace csgs

using namespace csgs;

extern "C" int csgs_layer_gemm(const float *Z, int64_t ldz, int32_t M, const int32_t *M_dev, int32_t K, const float *W, int64_t ldw,
                               int32_t Nout, float *H, int64_t ldh, void *stream)
{
    if (!Z || !W || !H || M <= 0 || K <= 0 || Nout <= 0 || ldz < K || ldw < Nout || ldh < Nout) return CSGS_EINVAL;
    const int64_t tm = ((int64_t)M + BM - 1) / BM;
    if (tm * (((int64_t)Nout + 31) / 32) > 0x3FFFFFFF) return CSGS_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    // narrow column tiles when wide ones would leave fewer than two blocks per compute unit
    const int64_t wide_tiles = tm * (((int64_t)Nout + 63) / 64);
    if (wide_tiles >= 512 && Nout > 32)
        launch_gemm<64>(Z, ldz, M, M_dev, K, W, ldw, Nout, H, ldh, st);
    else
        launch_gemm<32>(Z, ldz, M, M_dev, K, W, ldw, Nout, H, ldh, st);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
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
