// Optional per-kernel timing with HIP events (off by default; a measuring aid for benchmarks).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

namespace csgs {
namespace prof {

enum Kid {
    K_ROW_PREFIX = 0, K_SCAN_EDGES, K_CAND_PARTIALS, K_CAND_EMIT, K_DRAW, K_HITS_FUSED, K_ADJ_FUSED, K_REMOTE_COUNT,
    K_AGGREGATE, K_GEMM, K_GATHER_ROWS, K_GEMM_DZ, K_GEMM_DW, K_GEMM_DW_REDUCE, K_ADJT_COUNT, K_ADJT_PREFIX, K_ADJT_FILL, K_ADJT_ORDER,
    K_AGGREGATE_GRAD, K_FILL_ZERO, K_COPY, K_ATOMICS, K_MFMA_F64, K_LOOKUPS, K_LAYER_FORWARD, K_COUNT
};

extern bool g_enabled;
// Hands out the next pooled event pair for a launch of kernel `kid`; false when none is available.
bool next_pair(int kid, hipEvent_t *start, hipEvent_t *stop);

}  // namespace prof
}  // namespace csgs

// Launch `kernel` on `stream`; when timing is enabled the dispatch is stamped with two events.
// `kid_expr` is any int expression naming the kernel's slot in the timing table.
#define CSGS_LAUNCH_ID(kid_expr, kernel, grid, block, stream, ...)                                 \
    do {                                                                                           \
        hipEvent_t ev0_ = nullptr, ev1_ = nullptr;                                                 \
        if (::csgs::prof::g_enabled && ::csgs::prof::next_pair((int)(kid_expr), &ev0_, &ev1_))     \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, stream, ev0_, ev1_, 0, __VA_ARGS__);     \
        else                                                                                       \
            hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);                       \
    } while (0)
#define CSGS_LAUNCH(kid, kernel, grid, block, stream, ...) \
    CSGS_LAUNCH_ID(::csgs::prof::kid, kernel, grid, block, stream, __VA_ARGS__)
