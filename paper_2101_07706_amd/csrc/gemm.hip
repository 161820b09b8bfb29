// csgs_layer_gemm: H = Z W (Section 3, Eq. 1), fp32 in, fp32 out.
//
// Products and short partial sums (32 consecutive k) come from fp32 MFMA
// (v_mfma_f32_32x32x2_f32); the partial sums are folded into double master accumulators, which
// keeps the rounding error of a near-cancelling output below the 1e-5 absolute tolerance even
// for K in the hundreds and products of magnitude 1 (error ~ sqrt(32 K) / 2.8 * 2^-24 * |z w|).
//
// Block tile 128 (M) x BN (64 or 32), K chunks of 32, four wavefronts stacked along M, each
// owning a 32 x BN strip (BN / 32 MFMA tiles that share the A operand).  Global -> register ->
// LDS with the next chunk's loads in flight during the current chunk's MFMAs (two LDS buffers).
//
// LDS layout: A row-major [128][36], B transposed [BN][36] (k contiguous, 16-byte aligned rows
// whose stride of 36 words spreads 16 lanes' 128-bit reads over all 64 banks).  The k order
// inside a run of 16 is permuted -- lanes 0..31 feed k = 0..7 of the run, lanes 32..63 feed
// k = 8..15, for both operands alike, which leaves the sum unchanged -- so that every lane
// fetches its 8 operand values of a run with two 128-bit LDS reads.
//
// Block ids are remapped so that consecutive tiles (same rows of Z, neighbouring column tiles)
// land on the same XCD and share its L2.
#include "common.hpp"

namespace csgs {

typedef float floatx16 __attribute__((ext_vector_type(16)));

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
                                                  int64_t ldc, int M, int N, int K, int n_tiles_n, int n_tiles)
{
    constexpr int NT = BN / 32;   // MFMA tiles per wavefront
    __shared__ __attribute__((aligned(16))) float As[2][BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) float Bs[2][BN * LDS_STRIDE];
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    // XCD-aware tile order: hardware deals consecutive block ids round-robin to the 8 XCDs
    const int bid = (int)blockIdx.x;
    const int per_xcd = (n_tiles + 7) / 8;
    const int tile = (bid & 7) * per_xcd + (bid >> 3);
    if (tile >= n_tiles) return;
    const int64_t m0 = (int64_t)(tile / n_tiles_n) * BM, n0 = (int64_t)(tile % n_tiles_n) * BN;

    double master[NT][16];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 16; ++i) master[t][i] = 0.0;
    float4 ra[4], rb[NT];
    const int n_chunks = (K + BK - 1) / BK;
    fetch_a<VA, FULL>(A, lda, M, K, m0, 0, tid, ra);
    fetch_b<BN, FULL>(Bm, ldb, K, N, 0, n0, tid, rb);
    stash<BN>(As[0], Bs[0], tid, ra, rb);
    __syncthreads();
    const int a_off = (wave * 32 + l32) * LDS_STRIDE + 8 * half;
    const int b_off = l32 * LDS_STRIDE + 8 * half;
    for (int c = 0; c < n_chunks; ++c) {
        const int cur = c & 1;
        if (c + 1 < n_chunks) {
            fetch_a<VA, FULL>(A, lda, M, K, m0, (c + 1) * BK, tid, ra);
            fetch_b<BN, FULL>(Bm, ldb, K, N, (c + 1) * BK, n0, tid, rb);
        }
        floatx16 acc[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[t][i] = 0.f;
#pragma unroll
        for (int run = 0; run < 2; ++run) {   // two runs of 16 k
            const float *ap = &As[cur][a_off + run * 16];
            const float4 a0 = *reinterpret_cast<const float4 *>(ap), a1 = *reinterpret_cast<const float4 *>(ap + 4);
            const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
            float bv[NT][8];
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const float *bp = &Bs[cur][b_off + t * 32 * LDS_STRIDE + run * 16];
                const float4 b0 = *reinterpret_cast<const float4 *>(bp), b1 = *reinterpret_cast<const float4 *>(bp + 4);
                bv[t][0] = b0.x; bv[t][1] = b0.y; bv[t][2] = b0.z; bv[t][3] = b0.w;
                bv[t][4] = b1.x; bv[t][5] = b1.y; bv[t][6] = b1.z; bv[t][7] = b1.w;
            }
#pragma unroll
            for (int s = 0; s < 8; ++s)
#pragma unroll
                for (int t = 0; t < NT; ++t) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s], bv[t][s], acc[t], 0, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < 16; ++i) master[t][i] += (double)acc[t][i];
        if (c + 1 < n_chunks) {
            stash<BN>(As[cur ^ 1], Bs[cur ^ 1], tid, ra, rb);
            __syncthreads();
        }
    }
    // accumulator register i of lane l holds row 8 * (i / 4) + 4 * (l / 32) + i % 4, column l % 32
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t row = m0 + wave * 32 + 8 * (i / 4) + 4 * half + (i % 4);
        if (FULL || row < M) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                const int64_t col = n0 + t * 32 + l32;
                if (FULL || col < N) C[row * ldc + col] = (float)master[t][i];
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
static void launch_gemm(const float *Z, int64_t ldz, int M, int K, const float *W, int64_t ldw, int N, float *H,
                        int64_t ldh, hipStream_t st)
{
    const int tm = (M + BM - 1) / BM, tn = (N + BN - 1) / BN;
    const int n_tiles = tm * tn;
    const dim3 grid((unsigned)(((n_tiles + 7) / 8) * 8));
    const int va = widest(Z, ldz);
    const bool full = M % BM == 0 && N % BN == 0 && K % BK == 0 && va == 4;
    if (full)
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, 4, true>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, N, K, tn, n_tiles);
    else if (va == 4)
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, 4, false>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, N, K, tn, n_tiles);
    else if (va == 2)
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, 2, false>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, N, K, tn, n_tiles);
    else
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<BN, 1, false>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, N, K, tn, n_tiles);
}

}  // namespace csgs

using namespace csgs;

extern "C" int csgs_layer_gemm(const float *Z, int64_t ldz, int32_t M, int32_t K, const float *W, int64_t ldw,
                               int32_t Nout, float *H, int64_t ldh, void *stream)
{
    if (!Z || !W || !H || M <= 0 || K <= 0 || Nout <= 0 || ldz < K || ldw < Nout || ldh < Nout) return CSGS_EINVAL;
    const int64_t tm = ((int64_t)M + BM - 1) / BM;
    if (tm * (((int64_t)Nout + 31) / 32) > 0x3FFFFFFF) return CSGS_EUNSUPPORTED;
    hipStream_t st = (hipStream_t)stream;
    // narrow column tiles when wide ones would leave fewer than two blocks per compute unit
    const int64_t wide_tiles = tm * (((int64_t)Nout + 63) / 64);
    if (wide_tiles >= 512 && Nout > 32)
        launch_gemm<64>(Z, ldz, M, K, W, ldw, Nout, H, ldh, st);
    else
        launch_gemm<32>(Z, ldz, M, K, W, ldw, Nout, H, ldh, st);
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
