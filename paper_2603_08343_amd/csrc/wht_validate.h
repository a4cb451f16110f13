// Argument validation of the C ABI (include/wht_affine.h), free of any GPU call so that it also
// compiles with a host compiler alone (csrc/validate_selftest.cpp runs it under the sanitizers).
// Every entry point validates before anything is enqueued: a failed call has no side effects.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "../../include/wht_affine.h"

namespace wht {

// What a width d is to the library: log2 of the number of slots the schedule runs on, and whether
// the row is a power of two or 12 * 2^m.
struct Width { int logd; bool twelve; };

inline int log2_exact(int32_t d) {
    if (d < 1 || (d & (d - 1)) != 0) return -1;
    int l = 0;
    while ((1 << l) < d) ++l;
    return l;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int check_dims(int64_t N, int32_t d, int32_t dtype, Width* w) {
    if (dtype != WHT_DTYPE_F32 && dtype != WHT_DTYPE_BF16) return WHT_ERR_BAD_DTYPE;
    if (N < 0) return WHT_ERR_BAD_DIM;
    const int l = log2_exact(d);
    if (l >= 0) {
        if (d < WHT_MIN_D || d > WHT_MAX_D) return WHT_ERR_BAD_DIM;
        if (dtype == WHT_DTYPE_F32 && d > WHT_MAX_D_F32) return WHT_ERR_BAD_DIM;
        *w = Width{l, false};
        return WHT_OK;
    }
    // 12 * 2^m: bfloat16 only, 768 .. 12288
    if (d % 12 != 0 || dtype != WHT_DTYPE_BF16 || d < WHT_MIN_D_TWELVE || d > WHT_MAX_D_TWELVE)
        return WHT_ERR_BAD_DIM;
    const int m = log2_exact(d / 12);
    if (m < 0) return WHT_ERR_BAD_DIM;
    *w = Width{m + 4, true};
    return WHT_OK;
}

// Forward entry points (with_resid / with_stats: the fused variants' extra arguments).
inline int validate_forward(const void* x, const float* alpha, const float* beta, const void* resid,
                            bool with_resid, const void* y, const float* sumsq, bool with_stats, int64_t N,
                            int32_t d, int32_t dtype, Width* w) {
    if (!x || !alpha || !beta || !y || (with_resid && !resid) || (with_stats && !sumsq))
        return WHT_ERR_NULL_PTR;
    if (int rc = check_dims(N, d, dtype, w)) return rc;
    if (!aligned16(x) || !aligned16(y) || !aligned16(alpha) || !aligned16(beta) ||
        (with_resid && !aligned16(resid)) ||
        (with_stats && (reinterpret_cast<uintptr_t>(sumsq) & 3u) != 0))
        return WHT_ERR_MISALIGNED;
    return WHT_OK;
}

// Backward entry points, up to the workspace (whose size depends on the launch shape).
inline int validate_backward(const void* dy, const void* x, const float* alpha, const void* dx,
                             const float* dalpha, const float* dbeta, int64_t N, int32_t d, int32_t dtype,
                             Width* w) {
    const bool grads = dalpha != nullptr || dbeta != nullptr;
    if (!dy || !alpha) return WHT_ERR_NULL_PTR;
    if (grads && (!dalpha || !dbeta || !x)) return WHT_ERR_NULL_PTR;   // the two sums come together
    if (!grads && !dx) return WHT_ERR_NULL_PTR;                        // nothing asked for
    if (int rc = check_dims(N, d, dtype, w)) return rc;
    if (!aligned16(dy) || !aligned16(x) || !aligned16(alpha) || !aligned16(dx) || !aligned16(dalpha) ||
        !aligned16(dbeta))
        return WHT_ERR_MISALIGNED;
    return WHT_OK;
}

// The caller's workspace against what the call needs.
inline int validate_workspace(const void* workspace, size_t workspace_bytes, size_t need) {
    if (!workspace || workspace_bytes < need) return WHT_ERR_WORKSPACE;
    if (!aligned16(workspace)) return WHT_ERR_MISALIGNED;
    return WHT_OK;
}

}  // namespace wht
