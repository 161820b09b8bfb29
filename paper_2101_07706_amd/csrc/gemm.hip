// csgs_layer_gemm: H = Z W (Section 3, Eq. 1), fp32 in, fp32 out.  Products and short partial
// sums (16 consecutive k) come from fp32 MFMA; the partial sums are folded into double master
// accumulators, which keeps the rounding error of a near-cancelling output far below the 1e-5
// absolute tolerance even for K in the hundreds and inputs of magnitude 10.
//
// Block tile 64 x 64, four wavefronts, each owning one 32 x 32 accumulator tile computed with
// v_mfma_f32_32x32x2_f32.  A and B tiles pass through LDS in k-major order so that the operand
// fetch of a wavefront (lane l -> row/col l % 32, k-slice l / 32) is bank-conflict free.
#include "common.hpp"

namespace csgs {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BM = 64, BN = 64, BK = 16, LDS_PAD = 4;

__global__ __launch_bounds__(256) void gemm_f32_k(const float *__restrict__ A, int64_t lda,
                                                  const float *__restrict__ Bm, int64_t ldb, float *__restrict__ C,
                                                  int64_t ldc, int M, int N, int K)
{
    __shared__ float As[BK][BM + LDS_PAD];
    __shared__ float Bs[BK][BN + LDS_PAD];
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int64_t m0 = (int64_t)blockIdx.y * BM, n0 = (int64_t)blockIdx.x * BN;
    double master[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) master[i] = 0.0;

    for (int k0 = 0; k0 < K; k0 += BK) {
        // A tile: 64 rows x 16 k, read along k (row-major source), stored k-major
#pragma unroll
        for (int i = 0; i < (BM * BK) / 256; ++i) {
            const int idx = tid + i * 256;
            const int r = idx / BK, kk = idx % BK;
            const int64_t gm = m0 + r;
            const int gk = k0 + kk;
            As[kk][r] = (gm < M && gk < K) ? A[gm * lda + gk] : 0.f;
        }
        // B tile: 16 k x 64 cols
#pragma unroll
        for (int i = 0; i < (BK * BN) / 256; ++i) {
            const int idx = tid + i * 256;
            const int kk = idx / BN, c = idx % BN;
            const int gk = k0 + kk;
            const int64_t gn = n0 + c;
            Bs[kk][c] = (gk < K && gn < N) ? Bm[(int64_t)gk * ldb + gn] : 0.f;
        }
        __syncthreads();
        floatx16 acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 2) {
            const float a = As[kk + (lane >> 5)][wm * 32 + (lane & 31)];
            const float b = Bs[kk + (lane >> 5)][wn * 32 + (lane & 31)];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) master[i] += (double)acc[i];
        __syncthreads();
    }
    // accumulator register i of lane l holds row 8 * (i / 4) + 4 * (l / 32) + i % 4, column l % 32
    const int64_t col = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const int64_t row = m0 + wm * 32 + 8 * (i / 4) + 4 * (lane >> 5) + (i % 4);
        if (row < M && col < N) C[row * ldc + col] = (float)master[i];
    }
}

}  // namespace csgs

using namespace csgs;

extern "C" int csgs_layer_gemm(const float *Z, int64_t ldz, int32_t M, int32_t K, const float *W, int64_t ldw,
                               int32_t Nout, float *H, int64_t ldh, void *stream)
{
    if (!Z || !W || !H || M <= 0 || K <= 0 || Nout <= 0 || ldz < K || ldw < Nout || ldh < Nout) return CSGS_EINVAL;
    const dim3 grid((unsigned)((Nout + BN - 1) / BN), (unsigned)((M + BM - 1) / BM));
    if (grid.y > 65535u) return CSGS_EUNSUPPORTED;
    CSGS_LAUNCH(K_GEMM, gemm_f32_k, grid, dim3(256), (hipStream_t)stream, Z, ldz, W, ldw, H, ldh, M, Nout, K);
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
