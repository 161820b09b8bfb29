// csgs_layer_gemm: H = Z W (Section 3, Eq. 1), fp32 in, fp32 out.
//
// Products and short partial sums (16 consecutive k) come from fp32 MFMA
// (v_mfma_f32_32x32x2_f32); the partial sums are folded into double master accumulators, which
// keeps the rounding error of a near-cancelling output far below the 1e-5 absolute tolerance even
// for K in the hundreds and inputs of magnitude 10.  Two fp32 accumulator sets alternate so that
// the fold of one runs in the shadow of the MFMAs of the other.
//
// Block tile 128 (M) x 64 (N), K chunks of 32, four wavefronts stacked along M, each owning a
// 32 x 64 strip (two 32 x 32 MFMA tiles that share the A operand).  Global -> register -> LDS
// with the next chunk's loads in flight during the current chunk's MFMAs (two LDS buffers).
// A is kept row-major in LDS with an odd row stride, B k-major: both operand fetches
// (lane l -> row/col l % 32, k-slice l / 32) are conflict free.  Block ids are remapped so that
// consecutive tiles (same rows of Z, neighbouring column tiles) land on the same XCD and share
// its L2.
#include "common.hpp"

namespace csgs {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 64, BK = 32;
constexpr int A_STRIDE = BK + 1;   // odd: 32 consecutive rows at one k hit 32 different banks
constexpr int B_STRIDE = BN + 4;
constexpr int A_PER_THREAD = BM * BK / 256;  // 16 floats
constexpr int B_PER_THREAD = BK * BN / 256;  // 8 floats

template <int V>
__device__ inline void load_vec(const float *__restrict__ p, float *dst)
{
    if (V == 4) {
        const float4 v = *reinterpret_cast<const float4 *>(p);
        dst[0] = v.x; dst[1] = v.y; dst[2] = v.z; dst[3] = v.w;
    } else if (V == 2) {
        const float2 a = *reinterpret_cast<const float2 *>(p);
        const float2 b = *reinterpret_cast<const float2 *>(p + 2);
        dst[0] = a.x; dst[1] = a.y; dst[2] = b.x; dst[3] = b.y;
    } else {
        dst[0] = p[0]; dst[1] = p[1]; dst[2] = p[2]; dst[3] = p[3];
    }
}

// Chunk loaders: every thread fetches groups of 4 consecutive elements along the contiguous
// dimension (k for A, n for B); groups that cross the matrix edge are fetched element-wise with
// zero fill.  VA / VB = widest aligned vector the leading dimension and base pointer allow.
template <int VA>
__device__ inline void fetch_a(const float *__restrict__ A, int64_t lda, int M, int K, int64_t m0, int k0, int tid,
                               float (&ra)[A_PER_THREAD])
{
#pragma unroll
    for (int i = 0; i < A_PER_THREAD / 4; ++i) {
        const int idx = tid + i * 256;          // 1024 groups: 128 rows x 8 groups
        const int r = idx >> 3, kq = (idx & 7) * 4;
        const int64_t gm = m0 + r;
        const int gk = k0 + kq;
        float *dst = &ra[i * 4];
        if (gm < M && gk + 3 < K) {
            load_vec<VA>(A + gm * lda + gk, dst);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[j] = (gm < M && gk + j < K) ? A[gm * lda + gk + j] : 0.f;
        }
    }
}

template <int VB>
__device__ inline void fetch_b(const float *__restrict__ Bm, int64_t ldb, int K, int N, int k0, int64_t n0, int tid,
                               float (&rb)[B_PER_THREAD])
{
#pragma unroll
    for (int i = 0; i < B_PER_THREAD / 4; ++i) {
        const int idx = tid + i * 256;          // 512 groups: 32 k x 16 groups
        const int kk = idx >> 4, nq = (idx & 15) * 4;
        const int gk = k0 + kk;
        const int64_t gn = n0 + nq;
        float *dst = &rb[i * 4];
        if (gk < K && gn + 3 < N) {
            load_vec<VB>(Bm + (int64_t)gk * ldb + gn, dst);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) dst[j] = (gk < K && gn + j < N) ? Bm[(int64_t)gk * ldb + gn + j] : 0.f;
        }
    }
}

__device__ inline void stash(float *As, float *Bs, int tid, const float (&ra)[A_PER_THREAD],
                             const float (&rb)[B_PER_THREAD])
{
#pragma unroll
    for (int i = 0; i < A_PER_THREAD / 4; ++i) {
        const int idx = tid + i * 256;
        const int r = idx >> 3, kq = (idx & 7) * 4;
#pragma unroll
        for (int j = 0; j < 4; ++j) As[r * A_STRIDE + kq + j] = ra[i * 4 + j];
    }
#pragma unroll
    for (int i = 0; i < B_PER_THREAD / 4; ++i) {
        const int idx = tid + i * 256;
        const int kk = idx >> 4, nq = (idx & 15) * 4;
        *reinterpret_cast<float4 *>(&Bs[kk * B_STRIDE + nq]) = make_float4(rb[i * 4], rb[i * 4 + 1], rb[i * 4 + 2], rb[i * 4 + 3]);
    }
}

// 8 MFMA k-steps (16 consecutive k starting at kbase) for the wavefront's 32 x 64 strip.
__device__ inline void mfma_run(const float *As, const float *Bs, int wave, int lane, int kbase, floatx16 &c0,
                                floatx16 &c1)
{
    const int half = lane >> 5, l32 = lane & 31;
    const float *ap = As + (wave * 32 + l32) * A_STRIDE + kbase + half;
    const float *bp = Bs + (kbase + half) * B_STRIDE + l32;
    floatx16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    {
        const float a = ap[0], b0 = bp[0], b1 = bp[32];
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, z, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, z, 0, 0, 0);
    }
#pragma unroll
    for (int s = 1; s < 8; ++s) {
        const float a = ap[2 * s], b0 = bp[2 * s * B_STRIDE], b1 = bp[2 * s * B_STRIDE + 32];
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, c1, 0, 0, 0);
    }
}

__device__ inline void fold(double (&m0)[16], double (&m1)[16], const floatx16 &c0, const floatx16 &c1)
{
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        m0[i] += (double)c0[i];
        m1[i] += (double)c1[i];
    }
}

template <int VA, int VB>
__global__ __launch_bounds__(256) void gemm_f32_k(const float *__restrict__ A, int64_t lda,
                                                  const float *__restrict__ Bm, int64_t ldb, float *__restrict__ C,
                                                  int64_t ldc, int M, int N, int K, int n_tiles_n, int n_tiles)
{
    __shared__ float As[2][BM * A_STRIDE];
    __shared__ __attribute__((aligned(16))) float Bs[2][BK * B_STRIDE];
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    // XCD-aware tile order: hardware deals consecutive block ids round-robin to the 8 XCDs
    const int bid = (int)blockIdx.x;
    const int per_xcd = (n_tiles + 7) / 8;
    const int tile = (bid & 7) * per_xcd + (bid >> 3);
    if (tile >= n_tiles) return;
    const int64_t m0 = (int64_t)(tile / n_tiles_n) * BM, n0 = (int64_t)(tile % n_tiles_n) * BN;

    double ma[16], mb[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) { ma[i] = 0.0; mb[i] = 0.0; }
    float ra[A_PER_THREAD], rb[B_PER_THREAD];
    const int n_chunks = (K + BK - 1) / BK;
    fetch_a<VA>(A, lda, M, K, m0, 0, tid, ra);
    fetch_b<VB>(Bm, ldb, K, N, 0, n0, tid, rb);
    stash(As[0], Bs[0], tid, ra, rb);
    __syncthreads();
    for (int c = 0; c < n_chunks; ++c) {
        const int cur = c & 1;
        if (c + 1 < n_chunks) {
            fetch_a<VA>(A, lda, M, K, m0, (c + 1) * BK, tid, ra);
            fetch_b<VB>(Bm, ldb, K, N, (c + 1) * BK, n0, tid, rb);
        }
        floatx16 p0, p1, q0, q1;
        mfma_run(As[cur], Bs[cur], wave, lane, 0, p0, p1);
        mfma_run(As[cur], Bs[cur], wave, lane, 16, q0, q1);
        fold(ma, mb, p0, p1);   // runs while the second run's MFMAs drain
        fold(ma, mb, q0, q1);
        if (c + 1 < n_chunks) {
            stash(As[cur ^ 1], Bs[cur ^ 1], tid, ra, rb);
            __syncthreads();
        }
    }
    // accumulator register i of lane l holds row 8 * (i / 4) + 4 * (l / 32) + i % 4, column l % 32
    const int64_t col0 = n0 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t row = m0 + wave * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i % 4);
        if (row < M) {
            if (col0 < N) C[row * ldc + col0] = (float)ma[i];
            if (col0 + 32 < N) C[row * ldc + col0 + 32] = (float)mb[i];
        }
    }
}

static int widest(const float *p, int64_t ld)
{
    if (ld % 4 == 0 && ((uintptr_t)p & 15) == 0) return 4;
    if (ld % 2 == 0 && ((uintptr_t)p & 7) == 0) return 2;
    return 1;
}

}  // namespace csgs

using namespace csgs;

extern "C" int csgs_layer_gemm(const float *Z, int64_t ldz, int32_t M, int32_t K, const float *W, int64_t ldw,
                               int32_t Nout, float *H, int64_t ldh, void *stream)
{
    if (!Z || !W || !H || M <= 0 || K <= 0 || Nout <= 0 || ldz < K || ldw < Nout || ldh < Nout) return CSGS_EINVAL;
    const int64_t tm = ((int64_t)M + BM - 1) / BM, tn = ((int64_t)Nout + BN - 1) / BN;
    if (tm * tn > 0x3FFFFFFF) return CSGS_EUNSUPPORTED;
    const int n_tiles = (int)(tm * tn);
    const dim3 grid((unsigned)(((n_tiles + 7) / 8) * 8));
    hipStream_t st = (hipStream_t)stream;
    const int va = widest(Z, ldz), vb = widest(W, ldw);
#define CSGS_GEMM_CASE(VA_, VB_)                                                                                     \
    if (va == VA_ && vb == VB_)                                                                                      \
        CSGS_LAUNCH(K_GEMM, (gemm_f32_k<VA_, VB_>), grid, dim3(256), st, Z, ldz, W, ldw, H, ldh, M, Nout, K, (int)tn, \
                    n_tiles)
    CSGS_GEMM_CASE(4, 4); CSGS_GEMM_CASE(4, 2); CSGS_GEMM_CASE(4, 1);
    CSGS_GEMM_CASE(2, 4); CSGS_GEMM_CASE(2, 2); CSGS_GEMM_CASE(2, 1);
    CSGS_GEMM_CASE(1, 4); CSGS_GEMM_CASE(1, 2); CSGS_GEMM_CASE(1, 1);
#undef CSGS_GEMM_CASE
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
