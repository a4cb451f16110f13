// C ABI (include/wht_affine.h) and host-side dispatch of the Walsh-Hadamard output layer
//     y = alpha (.) (H x) + beta                                   (paper Sec. 4.1, Eq. 1)
// for gfx950.  The kernels live in wht_device.h, the stage schedules in wht_plan.h.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "../../include/wht_affine.h"
#include "wht_device.h"
#include "wht_validate.h"

namespace wht {

// ------------------------------------------------------------------------------------------------
// host side: launch shapes and dispatch

constexpr int kNumCU = 256;             // MI355X

// Workgroups launched per CU: the grid is persistent, each workgroup strides over token groups.  The
// per-configuration figures (C::kFwdGroupsPerCU, C::kBwdGroupsPerCU) are measured optima; the launch
// shape, and with it the backward workspace size, depends on (N, d, dtype) alone.
template <class C>
static int grid_for(int64_t N, bool backward) {
    const int64_t groups = (N + C::G - 1) / C::G;
    const int64_t cap = (int64_t)kNumCU * (backward ? C::kBwdGroupsPerCU : C::kFwdGroupsPerCU);
    return (int)(groups < cap ? groups : cap);
}

// Workgroups per cluster of the forward kernel: the configuration's figure when the grid divides
// into such clusters and every workgroup has several token groups to walk, else the whole grid.
template <class C>
static int forward_cluster(int64_t N, int grid, bool resid) {
    const int64_t groups = (N + C::G - 1) / C::G;
    const int want = resid ? C::kFwdClusterResid : C::kFwdCluster;
    if (want > 0 && grid % want == 0 && grid > want && groups >= 4 * (int64_t)grid) return want;
    return grid;
}

// Few tokens (decoding, short prefills): one token group per workgroup and no token loop.  Measured
// under HIP-graph replay, bfloat16: 2.1 against 3.2 us per call for one token of 4096 elements.  The
// persistent kernel takes over where the two break even: 2^22 elements per call at d >= 4096 (and for
// the butterfly schedule), 2^24 for the matrix-core schedule at d = 1024 and 2048 (16384 tokens of
// 1024 elements: 12.0 against 13.3 us), 2^21 for rows of 12 * 2^m elements.  Both kernels do the same
// arithmetic on a token in the same order, so the switch is invisible in y (the norm statistic is
// summed in the order of the launch shape: its last bits may differ between the two).
template <class C>
static bool few_tokens(int64_t N) {
    const int64_t limit = C::kTwelve ? (1 << 21) : ((C::kMfma && C::n <= 11) ? (1 << 24) : (1 << 22));
    return N * C::kRow <= limit;
}

template <class C>
static int launch_forward_once(const void* x, const float* alpha, const float* beta, const void* resid,
                               void* y, float* sumsq, int64_t N, hipStream_t stream) {
    using T = typename C::io::elem_t;
    const int grid = (int)((N + C::G - 1) / C::G);
    if (resid && sumsq)
        hipLaunchKernelGGL((forward_once_kernel<C, true, true>), dim3(grid), dim3(C::BT), 0, stream,
                           static_cast<const T*>(x), alpha, beta, static_cast<const T*>(resid), static_cast<T*>(y),
                           sumsq, N);
    else if (resid)
        hipLaunchKernelGGL((forward_once_kernel<C, true>), dim3(grid), dim3(C::BT), 0, stream,
                           static_cast<const T*>(x), alpha, beta, static_cast<const T*>(resid), static_cast<T*>(y),
                           static_cast<float*>(nullptr), N);
    else
        hipLaunchKernelGGL((forward_once_kernel<C, false>), dim3(grid), dim3(C::BT), 0, stream,
                           static_cast<const T*>(x), alpha, beta, static_cast<const T*>(nullptr), static_cast<T*>(y),
                           static_cast<float*>(nullptr), N);
    return hipGetLastError() == hipSuccess ? WHT_OK : WHT_ERR_LAUNCH;
}

template <class C>
static int launch_forward(const void* x, const float* alpha, const float* beta, const void* resid, void* y,
                          float* sumsq, int64_t N, hipStream_t stream) {
    using T = typename C::io::elem_t;
    const int grid = grid_for<C>(N, false);
    const int cluster = forward_cluster<C>(N, grid, resid != nullptr);
    if (resid && sumsq)
        hipLaunchKernelGGL((forward_kernel<C, true, true>), dim3(grid), dim3(C::BT), 0, stream,
                           static_cast<const T*>(x), alpha, beta, static_cast<const T*>(resid),
                           static_cast<T*>(y), sumsq, N, cluster);
    else if (resid)
        hipLaunchKernelGGL((forward_kernel<C, true>), dim3(grid), dim3(C::BT), 0, stream,
                           static_cast<const T*>(x), alpha, beta, static_cast<const T*>(resid),
                           static_cast<T*>(y), static_cast<float*>(nullptr), N, cluster);
    else
        hipLaunchKernelGGL((forward_kernel<C, false>), dim3(grid), dim3(C::BT), 0, stream,
                           static_cast<const T*>(x), alpha, beta, static_cast<const T*>(nullptr),
                           static_cast<T*>(y), static_cast<float*>(nullptr), N, cluster);
    return hipGetLastError() == hipSuccess ? WHT_OK : WHT_ERR_LAUNCH;
}

template <class C>
static int launch_backward(const void* dy, const void* x, const float* alpha, void* dx, float* dalpha,
                           float* dbeta, int64_t N, void* workspace, hipStream_t stream) {
    using T = typename C::io::elem_t;
    const bool grads = dalpha != nullptr;
    const int grid = grid_for<C>(N, grads);      // dx alone streams like a forward pass

    if (grads && dx) {
        if constexpr (C::kBwdTeams)
            hipLaunchKernelGGL((backward_teams_kernel<C>), dim3(grid), dim3(3 * C::BT), 0, stream,
                               static_cast<const T*>(dy), static_cast<const T*>(x), alpha, static_cast<T*>(dx),
                               static_cast<float*>(workspace), N);
        else
            hipLaunchKernelGGL((backward_kernel<C, true, true>), dim3(grid), dim3(C::BT), 0, stream,
                               static_cast<const T*>(dy), static_cast<const T*>(x), alpha, static_cast<T*>(dx),
                               static_cast<float*>(workspace), N);
    } else if (grads)
        hipLaunchKernelGGL((backward_kernel<C, true, false>), dim3(grid), dim3(C::BT), 0, stream,
                           static_cast<const T*>(dy), static_cast<const T*>(x), alpha, static_cast<T*>(nullptr),
                           static_cast<float*>(workspace), N);
    else
        hipLaunchKernelGGL((backward_kernel<C, false, true>), dim3(grid), dim3(C::BT), 0, stream,
                           static_cast<const T*>(dy), static_cast<const T*>(nullptr), alpha, static_cast<T*>(dx),
                           static_cast<float*>(nullptr), N);
    if (hipGetLastError() != hipSuccess) return WHT_ERR_LAUNCH;
    if (!grads) return WHT_OK;
    if constexpr (C::kRow >= 4096)
        hipLaunchKernelGGL(reduce_partials_kernel<16>, dim3((C::kRow + 63) / 64, 2), dim3(1024), 0, stream,
                           static_cast<const float*>(workspace), grid, C::kRow, dalpha, dbeta);
    else
        hipLaunchKernelGGL(reduce_partials_kernel<4>, dim3((C::kRow + 15) / 16, 2), dim3(1024), 0, stream,
                           static_cast<const float*>(workspace), grid, C::kRow, dalpha, dbeta);
    return hipGetLastError() == hipSuccess ? WHT_OK : WHT_ERR_LAUNCH;
}

template <class C>
static size_t workspace_for(int64_t N) { return (size_t)grid_for<C>(N, true) * 2 * C::kRow * sizeof(float); }

enum class Op { Forward, Backward, Workspace };

struct Args {
    const void* x; const void* dy; const void* resid; const float* alpha; const float* beta;
    void* y; void* dx; float* dalpha; float* dbeta; float* sumsq;
    int64_t N; void* workspace; hipStream_t stream;
    size_t workspace_out;
};

// CF: configuration of the forward kernels, CB: of the backward kernels (and its workspace), CO: of
// the forward kernel for few tokens.
template <class CF, class CB = CF, class CO = CF>
static int run(Op op, Args& a) {
    switch (op) {
    case Op::Forward:
        if (few_tokens<CO>(a.N))
            return launch_forward_once<CO>(a.x, a.alpha, a.beta, a.resid, a.y, a.sumsq, a.N, a.stream);
        return launch_forward<CF>(a.x, a.alpha, a.beta, a.resid, a.y, a.sumsq, a.N, a.stream);
    case Op::Backward: return launch_backward<CB>(a.dy, a.x, a.alpha, a.dx, a.dalpha, a.dbeta, a.N,
                                                  a.workspace, a.stream);
    default:           a.workspace_out = workspace_for<CB>(a.N); return WHT_OK;
    }
}

// Schedule choice: bfloat16 tokens of 1024 elements or more take the matrix-core schedule, the
// rest the butterfly schedule.  WHT_AFFINE_SCHEDULE=butterfly in the environment (read once per
// process; the library's only environment variable) forces the butterfly schedule for those too:
// it exists so that both schedules of one build can be tested and profiled against each other.
static bool use_mfma() {
    static const bool on = [] {
        const char* v = getenv("WHT_AFFINE_SCHEDULE");
        return !(v && strcmp(v, "butterfly") == 0);
    }();
    return on;
}

template <class Io, int LOGD>
static int run_d(Op op, Args& a) {
    if constexpr (std::is_same<Io, IoBF16>::value && LOGD >= 10) {
        if (use_mfma())
            return run<MfmaCfg<LOGD, mfma_log_tiles(LOGD, false)>, MfmaCfg<LOGD, mfma_log_tiles(LOGD, true)>,
                       MfmaCfg<LOGD, mfma_log_tiles_few(LOGD)>>(op, a);
    }
    return run<Cfg<LOGD, log_e_for(LOGD, Io::kLogVec), Io>>(op, a);
}

// The debug build that poisons LDS after every read (WHT_POISON_LDS, libwht_affine_poison.so, loaded
// by one GPU test only) carries a few widths that between them use every kernel and every kind of
// LDS hand-over; the others are left out of it to keep its compile time short.
#ifdef WHT_POISON_LDS
#define WHT_ALL_WIDTHS 0
#else
#define WHT_ALL_WIDTHS 1
#endif

template <class Io>
static int dispatch_d(int logd, Op op, Args& a) {
    switch (logd) {
#if WHT_ALL_WIDTHS
    case 5:  return run_d<Io, 5>(op, a);
    case 6:  return run_d<Io, 6>(op, a);
    case 7:  return run_d<Io, 7>(op, a);
    case 8:  return run_d<Io, 8>(op, a);
    case 10: return run_d<Io, 10>(op, a);
    case 11: return run_d<Io, 11>(op, a);
#endif
    case 9:  return run_d<Io, 9>(op, a);
    case 12: return run_d<Io, 12>(op, a);
    case 13: return run_d<Io, 13>(op, a);
    case 14:
        if constexpr (std::is_same<Io, IoBF16>::value) return run_d<Io, 14>(op, a);
        return WHT_ERR_BAD_DIM;
    default: return WHT_ERR_BAD_DIM;
    }
}

// Rows of 12 * 2^m elements (bfloat16): matrix-core schedule on 16 * 2^m slots.
template <int LOGS>
static int run_twelve(Op op, Args& a) {
    return run<MfmaCfg<LOGS, mfma_log_tiles(LOGS, false), true>, MfmaCfg<LOGS, mfma_log_tiles(LOGS, true), true>,
               MfmaCfg<LOGS, mfma_log_tiles_few(LOGS), true>>(op, a);
}

static int dispatch_twelve(int logslots, Op op, Args& a) {
    switch (logslots) {
#if WHT_ALL_WIDTHS
    case 10: return run_twelve<10>(op, a);
    case 11: return run_twelve<11>(op, a);
    case 12: return run_twelve<12>(op, a);
    case 14: return run_twelve<14>(op, a);
#endif
    case 13: return run_twelve<13>(op, a);
    default: return WHT_ERR_BAD_DIM;
    }
}

static int dispatch(Width w, int dtype, Op op, Args& a) {
    if (w.twelve) return dispatch_twelve(w.logd, op, a);
    return dtype == WHT_DTYPE_F32 ? dispatch_d<IoF32>(w.logd, op, a) : dispatch_d<IoBF16>(w.logd, op, a);
}

// ------------------------------------------------------------------------------------------------
// Partial-sum scratch that lives in the library's own code object, for wht_affine_backward_static:
// callers that cannot allocate pass no workspace.  Every GPU the library runs on holds its own copy
// of the array, at its own address, until the process ends.  In host code the array's name is only a
// handle for hipGetSymbolAddress: what kernels and copies take is the device address it returns.
static __device__ __align__(256) unsigned char scratch[WHT_STATIC_WORKSPACE_BYTES];

constexpr int kMaxDevices = 64;
static std::mutex scratch_mutex;
static void* scratch_address[kMaxDevices];       // per device, filled on the first call there

// Device address of the current device's copy of `scratch`, or nullptr if it cannot be had.
static void* static_scratch() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_address[dev]) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        scratch_address[dev] = ptr;
    }
    return scratch_address[dev];
}

}  // namespace wht

// ------------------------------------------------------------------------------------------------
// C ABI

extern "C" {

static int forward_common(const void* x, const float* alpha, const float* beta, const void* resid,
                          bool with_resid, void* y, float* sumsq, bool with_stats, int64_t N, int32_t d,
                          int32_t dtype, void* stream) {
    using namespace wht;
    Width w{};
    if (int rc = validate_forward(x, alpha, beta, resid, with_resid, y, sumsq, with_stats, N, d, dtype, &w)) return rc;
    if (N == 0) return WHT_OK;
    Args a{};
    a.x = x; a.alpha = alpha; a.beta = beta; a.resid = with_resid ? resid : nullptr; a.y = y; a.N = N;
    a.sumsq = with_stats ? sumsq : nullptr;
    a.stream = static_cast<hipStream_t>(stream);
    return dispatch(w, dtype, Op::Forward, a);
}

int wht_affine_forward(const void* x, const float* alpha, const float* beta, void* y, int64_t N,
                       int32_t d, int32_t dtype, void* stream) {
    return forward_common(x, alpha, beta, nullptr, false, y, nullptr, false, N, d, dtype, stream);
}

int wht_affine_forward_residual(const void* x, const float* alpha, const float* beta, const void* resid,
                                void* y, int64_t N, int32_t d, int32_t dtype, void* stream) {
    return forward_common(x, alpha, beta, resid, true, y, nullptr, false, N, d, dtype, stream);
}

int wht_affine_forward_residual_stats(const void* x, const float* alpha, const float* beta,
                                      const void* resid, void* y, float* sumsq, int64_t N, int32_t d,
                                      int32_t dtype, void* stream) {
    return forward_common(x, alpha, beta, resid, true, y, sumsq, true, N, d, dtype, stream);
}

size_t wht_affine_backward_workspace_bytes(int64_t N, int32_t d, int32_t dtype) {
    using namespace wht;
    Width w{};
    if (check_dims(N, d, dtype, &w) != WHT_OK || N == 0) return 0;
    Args a{};
    a.N = N;
    dispatch(w, dtype, Op::Workspace, a);
    return a.workspace_out;
}

// Both backward entry points: `own_scratch` takes the partial-sum workspace from the library's
// static buffer instead of the caller.
static int backward_common(const void* dy, const void* x, const float* alpha, void* dx, float* dalpha,
                           float* dbeta, int64_t N, int32_t d, int32_t dtype, void* workspace,
                           size_t workspace_bytes, bool own_scratch, void* stream) {
    using namespace wht;
    const bool grads = dalpha != nullptr || dbeta != nullptr;
    Width w{};
    if (int rc = validate_backward(dy, x, alpha, dx, dalpha, dbeta, N, d, dtype, &w)) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (N == 0) {
        if (!grads) return WHT_OK;
        hipLaunchKernelGGL(zero_kernel, dim3((d + 255) / 256), dim3(256), 0, s, dalpha, dbeta, d);
        return hipGetLastError() == hipSuccess ? WHT_OK : WHT_ERR_LAUNCH;
    }
    if (grads) {
        const size_t need = wht_affine_backward_workspace_bytes(N, d, dtype);
        if (own_scratch) {
            if (need > (size_t)WHT_STATIC_WORKSPACE_BYTES) return WHT_ERR_WORKSPACE;
            workspace = static_scratch();
            if (!workspace) return WHT_ERR_LAUNCH;
        } else {
            if (int rc = validate_workspace(workspace, workspace_bytes, need)) return rc;
        }
    }
    Args a{};
    a.dy = dy; a.x = x; a.alpha = alpha; a.dx = dx; a.dalpha = dalpha; a.dbeta = dbeta; a.N = N;
    a.workspace = workspace; a.stream = s;
    return dispatch(w, dtype, Op::Backward, a);
}

int wht_affine_backward(const void* dy, const void* x, const float* alpha, void* dx, float* dalpha,
                        float* dbeta, int64_t N, int32_t d, int32_t dtype, void* workspace,
                        size_t workspace_bytes, void* stream) {
    return backward_common(dy, x, alpha, dx, dalpha, dbeta, N, d, dtype, workspace, workspace_bytes, false, stream);
}

int wht_affine_backward_static(const void* dy, const void* x, const float* alpha, void* dx, float* dalpha,
                               float* dbeta, int64_t N, int32_t d, int32_t dtype, void* stream) {
    return backward_common(dy, x, alpha, dx, dalpha, dbeta, N, d, dtype, nullptr, 0, true, stream);
}

const char* wht_affine_status_string(int status) {
    switch (status) {
    case WHT_OK:             return "ok";
    case WHT_ERR_NULL_PTR:   return "a required pointer is NULL";
    case WHT_ERR_BAD_DIM:    return "d must be a power of two in [WHT_MIN_D, WHT_MAX_D] (WHT_MAX_D_F32 for float32) or, for bfloat16, 12*2^m in [WHT_MIN_D_TWELVE, WHT_MAX_D_TWELVE]; N >= 0";
    case WHT_ERR_BAD_DTYPE:  return "dtype must be WHT_DTYPE_F32 or WHT_DTYPE_BF16";
    case WHT_ERR_MISALIGNED: return "tensor pointers must be 16-byte aligned";
    case WHT_ERR_WORKSPACE:  return "workspace is NULL or smaller than wht_affine_backward_workspace_bytes (wht_affine_backward_static: the call needs more than WHT_STATIC_WORKSPACE_BYTES)";
    case WHT_ERR_LAUNCH:     return "the HIP runtime refused a kernel launch";
    default:                 return "unknown status";
    }
}

int wht_affine_version(void) { return 100; }

}  // extern "C"
