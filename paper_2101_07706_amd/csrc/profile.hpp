// Optional per-kernel timing with HIP events (off by default; a measuring aid for benchmarks).
#pragma once
#include <hip/hip_runtime.h>

namespace csgs {
namespace prof {

enum Kid {
    K_ROW_PREFIX = 0, K_SCAN_EDGES, K_CAND_PARTIALS, K_CAND_EMIT, K_DRAW, K_HITS_FUSED, K_ADJ_FUSED, K_REMOTE_COUNT,
    K_AGGREGATE, K_GEMM, K_GATHER_ROWS, K_FILL_ZERO, K_COPY, K_COUNT
};

extern bool g_enabled;
void record(int kid, hipStream_t st, bool start);

struct Scope {
    int kid;
    hipStream_t st;
    Scope(int k, hipStream_t s) : kid(k), st(s) { if (g_enabled) record(kid, st, true); }
    ~Scope() { if (g_enabled) record(kid, st, false); }
};

}  // namespace prof
}  // namespace csgs

// Launch `kernel` on `stream`; when timing is enabled the launch is bracketed by two events.
#define CSGS_LAUNCH(kid, kernel, grid, block, stream, ...)                     \
    do {                                                                       \
        ::csgs::prof::Scope scope_(::csgs::prof::kid, stream);                 \
        hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);       \
    } while (0)
