// Per-kernel timing: every launch made while timing is enabled carries a pair of HIP events that
// the runtime stamps with the start and the end of that very dispatch (hipExtLaunchKernelGGL), so
// the elapsed time is the kernel's own duration as the command processor sees it, without the
// cost of separate event packets; csgs_profile_collect() (after the caller synchronised) sums
// the elapsed times per kernel.  Process-wide state, one thread at a time.
#include <vector>
#include "common.hpp"
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
                                            "adjT_count", "adjT_prefix", "adjT_fill", "aggregate_grad", "fill_zero", "copy", "atomics"};

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
}  // namespace csgs

using namespace csgs::prof;

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
