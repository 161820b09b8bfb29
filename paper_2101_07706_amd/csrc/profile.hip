// Per-kernel timing: every launch made while timing is enabled carries a pair of HIP events that
// the runtime stamps with the start and the end of that very dispatch (hipExtLaunchKernelGGL), so
// the elapsed time is the kernel's own duration as the command processor sees it, without the
// cost of separate event packets; csgs_profile_collect() (after the caller synchronised) sums
// the elapsed times per kernel.  Process-wide state, one thread at a time.
#include <vector>
#include "common.hpp"
#include "csgs_bench.h"
#include "profile.hpp"

namespace csgs {
namespace prof {

bool g_enabled = false;

struct Pair {
    hipEvent_t a, b;
    int kid;
};
static std::vector<Pair> g_pool;   // created once, reused
static size_t g_used = 0;
static const size_t kMaxPairs = 1 << 16;

static const char *const kNames[K_COUNT] = {"row_prefix", "scan_edges", "cand_partials", "cand_emit", "draw", "hits_fused",
                                            "adj_fused", "remote_count", "aggregate",
                                            "layer_gemm", "gather_rows", "gemm_grad_z", "gemm_grad_w", "gemm_grad_w_reduce",
                                            "adjT_count", "adjT_prefix", "adjT_fill", "adjT_order", "aggregate_grad", "fill_zero", "copy", "atomics", "mfma_f64", "lookups", "layer_forward"};

bool next_pair(int kid, hipEvent_t *start, hipEvent_t *stop)
{
    if (g_used >= kMaxPairs) return false;
    if (g_used == g_pool.size()) {
        Pair p;
        if (hipEventCreate(&p.a) != hipSuccess) return false;
        if (hipEventCreate(&p.b) != hipSuccess) { (void)hipEventDestroy(p.a); return false; }
        g_pool.push_back(p);
    }
    g_pool[g_used].kid = kid;
    *start = g_pool[g_used].a;
    *stop = g_pool[g_used].b;
    ++g_used;
    return true;
}

}  // namespace prof
}  // namespace csgs

namespace csgs {
// Plain streaming copy, 16 bytes per thread and step: the yardstick for achievable HBM bandwidth
// and the known-size kernel against which byte counters are calibrated.
__global__ __launch_bounds__(256) void copy_k(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n16)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n16; i += stride) dst[i] = src[i];
}
// n fire-and-forget 64-bit integer atomic adds at device scope to pseudo-random entries of a table:
// the yardstick for the weight scan, whose accumulators are updated the same way.
__global__ __launch_bounds__(256) void atomics_k(unsigned long long *__restrict__ table, uint64_t n_table, uint64_t n)
{
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) {
        uint64_t h = (i + 1) * 0x9E3779B97F4A7C15ull;   // Fibonacci hashing: consecutive i land far apart
        h ^= h >> 29;
        (void)__hip_atomic_fetch_add(&table[h % n_table], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}
// n independent 8-byte reads of pseudo-random entries of a table (the same sequence of entries as atomics_k):
// what one random lookup costs in fetched bytes and time -- the adjacency pass looks up one such entry per edge.
__global__ __launch_bounds__(256) void lookups_k(const unsigned long long *__restrict__ table, uint64_t n_table, uint64_t n,
                                                 unsigned long long *__restrict__ sink)
{
    uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x, me = i;
    unsigned long long s = 0;
    for (; i < n; i += stride) {
        uint64_t h = (i + 1) * 0x9E3779B97F4A7C15ull;
        h ^= h >> 29;
        s += table[h % n_table];
    }
    sink[me] = s;   // keeps the reads
}
// Back-to-back v_mfma_f64_16x16x4_f64 on eight independent accumulators per wavefront, 64 per loop
// iteration: the yardstick for the layer GEMM, whose inner loop is the same instruction stream.
// FROM_LDS = false: operands stay in registers (the matrix cores' issue rate under load and at the
// clock the device sustains).  FROM_LDS = true: per iteration every lane reads 6 x 8 floats from LDS
// with 128-bit reads and widens them, as the GEMM does per K chunk of 32, without its global loads
// and barriers.
typedef double calib_d4 __attribute__((ext_vector_type(4)));
template <bool FROM_LDS>
__global__ __launch_bounds__(256) void mfma_f64_k(double *__restrict__ sink, int64_t iters)
{
    constexpr int STRIDE = 36;
    __shared__ __attribute__((aligned(16))) float tile[2][64 * STRIDE];
    const int tid = (int)threadIdx.x, lane = tid & 63;
    for (int i = tid; i < 2 * 64 * STRIDE; i += 256) (&tile[0][0])[i] = 1.0f / (float)(1 + (i & 1023));
    __syncthreads();
    calib_d4 acc[2][4];
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[r][t] = calib_d4{0.0, 0.0, 0.0, 0.0};
    double a0 = 1.0 / (double)(lane + 1), a1 = 1.0 / (double)(lane + 65), b = 1.0 / (double)(lane + 129);
    const int off = (lane & 15) * STRIDE + 8 * (lane >> 4);
    for (int64_t it = 0; it < iters; ++it) {
        if (FROM_LDS) {
            const float *base = &tile[it & 1][off];
            float av[2][8], bv[4][8];
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const float4 x = *reinterpret_cast<const float4 *>(base + r * 16 * STRIDE);
                const float4 y = *reinterpret_cast<const float4 *>(base + r * 16 * STRIDE + 4);
                av[r][0] = x.x; av[r][1] = x.y; av[r][2] = x.z; av[r][3] = x.w;
                av[r][4] = y.x; av[r][5] = y.y; av[r][6] = y.z; av[r][7] = y.w;
            }
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const float4 x = *reinterpret_cast<const float4 *>(base + t * 16 * STRIDE);   // rows 16 t + lane % 16 < 64
                const float4 y = *reinterpret_cast<const float4 *>(base + t * 16 * STRIDE + 4);
                bv[t][0] = x.x; bv[t][1] = x.y; bv[t][2] = x.z; bv[t][3] = x.w;
                bv[t][4] = y.x; bv[t][5] = y.y; bv[t][6] = y.z; bv[t][7] = y.w;
            }
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const double x0 = (double)av[0][s], x1 = (double)av[1][s];
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const double y = (double)bv[t][s];
                    acc[0][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(x0, y, acc[0][t], 0, 0, 0);
                    acc[1][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(x1, y, acc[1][t], 0, 0, 0);
                }
            }
        } else {
#pragma unroll
            for (int s = 0; s < 8; ++s)
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    acc[0][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a0, b, acc[0][t], 0, 0, 0);
                    acc[1][t] = __builtin_amdgcn_mfma_f64_16x16x4f64(a1, b, acc[1][t], 0, 0, 0);
                }
        }
    }
    double sum = 0.0;
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
        for (int t = 0; t < 4; ++t) sum += acc[r][t][0] + acc[r][t][1] + acc[r][t][2] + acc[r][t][3];
    sink[(size_t)blockIdx.x * 256 + tid] = sum;
}
}  // namespace csgs

using namespace csgs::prof;

extern "C" int csgs_calib_mfma_f64(double *sink, size_t n_sink, int64_t iters, int32_t from_lds, void *stream)
{
    if (!sink || ((uintptr_t)sink & 7) || iters <= 0 || iters > (1 << 24) || n_sink < (size_t)CSGS_CALIB_MFMA_BLOCKS * 256)
        return CSGS_EINVAL;
    if (from_lds)
        CSGS_LAUNCH(K_MFMA_F64, csgs::mfma_f64_k<true>, dim3(CSGS_CALIB_MFMA_BLOCKS), dim3(256), (hipStream_t)stream, sink, iters);
    else
        CSGS_LAUNCH(K_MFMA_F64, csgs::mfma_f64_k<false>, dim3(CSGS_CALIB_MFMA_BLOCKS), dim3(256), (hipStream_t)stream, sink, iters);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_calib_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || bytes == 0 || (bytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) return CSGS_EINVAL;
    const size_t n16 = bytes / 16;
    const unsigned blocks = (unsigned)((n16 + 255) / 256 < 16384 ? (n16 + 255) / 256 : 16384);
    CSGS_LAUNCH(K_COPY, csgs::copy_k, dim3(blocks), dim3(256), (hipStream_t)stream, (const uint4 *)src, (uint4 *)dst, n16);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_calib_atomics(uint64_t *table, size_t n_table, size_t n_updates, void *stream)
{
    if (!table || n_table == 0 || n_updates == 0 || ((uintptr_t)table & 7)) return CSGS_EINVAL;
    const size_t want = (n_updates + 255) / 256;
    const unsigned blocks = (unsigned)(want < 16384 ? want : 16384);
    CSGS_LAUNCH(K_ATOMICS, csgs::atomics_k, dim3(blocks), dim3(256), (hipStream_t)stream, (unsigned long long *)table,
                (uint64_t)n_table, (uint64_t)n_updates);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_calib_lookups(const uint64_t *table, size_t n_table, size_t n_reads, uint64_t *sink, size_t n_sink, void *stream)
{
    const size_t want = (n_reads + 255) / 256;
    const unsigned blocks = (unsigned)(want < 16384 ? want : 16384);
    if (!table || n_table == 0 || n_reads == 0 || !sink || n_sink < (size_t)blocks * 256 || ((uintptr_t)table & 7) || ((uintptr_t)sink & 7))
        return CSGS_EINVAL;
    CSGS_LAUNCH(K_LOOKUPS, csgs::lookups_k, dim3(blocks), dim3(256), (hipStream_t)stream, (const unsigned long long *)table,
                (uint64_t)n_table, (uint64_t)n_reads, (unsigned long long *)sink);
    CSGS_LAUNCH_CHECK();
    return CSGS_OK;
}

extern "C" int csgs_profile_enable(int on)
{
    g_enabled = on != 0;
    return CSGS_OK;
}

extern "C" int csgs_profile_kernel_count(void) { return K_COUNT; }

extern "C" const char *csgs_profile_kernel_name(int kid) { return (kid >= 0 && kid < K_COUNT) ? kNames[kid] : ""; }

extern "C" int csgs_profile_samples(float *ms, int32_t *kernel, int64_t cap, int64_t *n_out)
{
    if (!ms || !kernel || cap < 0 || !n_out) return CSGS_EINVAL;
    *n_out = (int64_t)g_used;
    for (size_t i = 0; i < g_used && (int64_t)i < cap; ++i) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, g_pool[i].a, g_pool[i].b) != hipSuccess) t = -1.f;   // (not yet complete: the caller did not synchronise)
        ms[i] = t;
        kernel[i] = g_pool[i].kid;
    }
    return CSGS_OK;
}

extern "C" int csgs_profile_collect(double *ms_sum, int64_t *launches)
{
    if (!ms_sum || !launches) return CSGS_EINVAL;
    for (int k = 0; k < K_COUNT; ++k) { ms_sum[k] = 0.0; launches[k] = 0; }
    for (size_t i = 0; i < g_used; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, g_pool[i].a, g_pool[i].b) == hipSuccess) {
            ms_sum[g_pool[i].kid] += (double)ms;
            launches[g_pool[i].kid] += 1;
        }
    }
    g_used = 0;
    return CSGS_OK;
}
