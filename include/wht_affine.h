/*
 * wht_affine.h -- C ABI of the Walsh-Hadamard output layer for AMD MI355X (gfx950).
 *
 * The layer replaces the dense attention output projection W_O (paper Sec. 4.1, Eq. 1):
 * for every token n, with x[n,:] the concatenated head outputs (d = heads * d_head),
 *
 *     z[n,:] = H x[n,:]                    H = H_raw / sqrt(d),  H_raw[j][k] = (-1)^popcount(j & k)
 *     y[n,:] = alpha (.) z[n,:] + beta     (Eq. 1; alpha, beta in R^d are the only parameters)
 *
 * For d a power of two, H is the normalised Walsh-Hadamard matrix in Sylvester (natural) order --
 * the sign block drawn in Fig. 1 -- so H^T H = I (Sec. 4.1) and H is symmetric.  It is never
 * stored: the kernels run the log2(d) add/subtract butterfly stages of Fig. 2.
 *
 * Widths d = 12 * 2^m.  The paper also trains d = 768 and d = 1536 (Table 2) and does not say which
 * matrix it uses there.  This library's reading, for bfloat16 tensors and d = 768 ... 12288:
 *
 *     H_raw = P12 (x) S_{2^m}      H_raw[j][k] = P12[j / 2^m][k / 2^m] * (-1)^popcount(j & k & (2^m - 1))
 *
 * i.e. the Sylvester transform inside each of the 12 contiguous blocks of 2^m features, and P12
 * across the blocks; P12 is the symmetric order-12 Hadamard matrix of Paley's second construction
 * over GF(5) with first row and column +1 (rows, as +/-):
 *     ++++++++++++  +--+-+-+-+-+  +-+-++----++  ++--+--+-++-  +-+++-++----  +++---+--+-+
 *     +---+++-++--  ++-++---+--+  +-----+++-++  ++-+-++---+-  +-++----+++-  +++--+-++---
 * H = H_raw / sqrt(d) is again symmetric and orthogonal with entries +-1/sqrt(d), so Eq. 1 and the
 * backward formulas below hold unchanged.
 *
 * Backward (the paper gives only the O(d log d) cost, Table 1; the formulas are Eq. 1's chain rule):
 *
 *     dx[n,:]   = H (alpha (.) dy[n,:])
 *     dalpha[j] = sum_n dy[n,j] * z[n,j]        z is recomputed from x, never stored
 *     dbeta[j]  = sum_n dy[n,j]
 *
 * Conventions for every entry point
 *   - Every pointer is a DEVICE pointer owned by the caller (the `stream` handle aside).  The
 *     library never allocates, frees or synchronises; work is enqueued on `stream` (a hipStream_t
 *     passed as void*, NULL = the default stream) and the call returns at once.
 *   - x, y, dy, dx are row-major [N, d], contiguous (leading dimension d), of type `dtype`.
 *     alpha, beta, dalpha, dbeta are float32 [d] whatever `dtype` is.
 *   - bfloat16 tensors are computed in float32 internally and rounded to nearest-even on store.
 *     For bfloat16 tensors of d >= 1024 (and all 12 * 2^m widths) ten of the log2(d) stages run on
 *     the matrix cores as products with +-1 matrices: exact products, float32 accumulation, and a
 *     float32 value entering such a product is represented as the sum of two bfloat16 terms, which
 *     carries it to a relative error of at most 2^-17 (five hundred times finer than the bfloat16
 *     output's own rounding).  float32 tensors never take this path.
 *   - Non-finite inputs: NaN propagates.  An infinite input makes the token's outputs +-Inf or NaN
 *     with float32 tensors (Inf - Inf in a butterfly) and NaN with bfloat16 tensors of d >= 1024
 *     (the two-term representation of Inf is Inf + NaN).
 *   - All tensor pointers must be 16-byte aligned.  y may alias x exactly, dx may alias dy or x
 *     exactly; partial overlap is undefined.
 *   - The return value is a wht_status_t.  Arguments are validated before anything is enqueued, so
 *     a failed call has no side effects.  N = 0 is valid (backward then zero-fills dalpha, dbeta).
 *   - d must be a power of two with WHT_MIN_D <= d <= WHT_MAX_D (WHT_MAX_D_F32 for float32
 *     tensors, whose token groups take twice the LDS), or, for bfloat16 tensors only, 12 * 2^m with
 *     WHT_MIN_D_TWELVE <= d <= WHT_MAX_D_TWELVE; anything else is WHT_ERR_BAD_DIM.
 */
#ifndef WHT_AFFINE_H
#define WHT_AFFINE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define WHT_MIN_D 32
#define WHT_MAX_D 16384        /* bfloat16 tensors */
#define WHT_MAX_D_F32 8192     /* float32 tensors */
#define WHT_MIN_D_TWELVE 768   /* d = 12 * 2^m, bfloat16 tensors: 768, 1536, 3072, 6144, 12288 */
#define WHT_MAX_D_TWELVE 12288

typedef enum {
    WHT_DTYPE_F32  = 0,   /* x, y, dy, dx are IEEE binary32 */
    WHT_DTYPE_BF16 = 1    /* x, y, dy, dx are bfloat16 (upper half of binary32) */
} wht_dtype_t;

typedef enum {
    WHT_OK             = 0,
    WHT_ERR_NULL_PTR   = 1,   /* a required pointer is NULL */
    WHT_ERR_BAD_DIM    = 2,   /* d outside the widths listed above for this dtype, or N < 0 */
    WHT_ERR_BAD_DTYPE  = 3,
    WHT_ERR_MISALIGNED = 4,   /* a tensor pointer is not 16-byte aligned */
    WHT_ERR_WORKSPACE  = 5,   /* workspace NULL or smaller than wht_affine_backward_workspace_bytes */
    WHT_ERR_LAUNCH     = 6    /* the HIP runtime refused a launch (hipGetLastError() != hipSuccess) */
} wht_status_t;

/*
 * Forward, Eq. 1:  y = alpha (.) (H x) + beta.
 *   x      in   [N,d] dtype     read once
 *   alpha  in   [d]   float32
 *   beta   in   [d]   float32
 *   y      out  [N,d] dtype     written once
 */
int wht_affine_forward(const void *x, const float *alpha, const float *beta, void *y,
                       int64_t N, int32_t d, int32_t dtype, void *stream);

/*
 * Forward with the attention block's residual add fused into the epilogue:
 *     y = resid + alpha (.) (H x) + beta.
 * (Eq. 1; the layer's output feeds the residual connection that follows the attention block, and
 * Sec. 6 of the paper names missing operator fusion as what keeps its measured speed-ups below the
 * operation count.)  One more [N,d] stream is read; the separate read-modify-write pass over y that
 * a framework would otherwise run is saved.
 *   resid  in   [N,d] dtype.   y may alias resid or x exactly.
 * The gradient with respect to resid is dy itself, so wht_affine_backward serves this call too.
 */
int wht_affine_forward_residual(const void *x, const float *alpha, const float *beta,
                                const void *resid, void *y,
                                int64_t N, int32_t d, int32_t dtype, void *stream);

/*
 * The same, and the statistic of an RMS normalisation that follows the residual stream:
 *     y = resid + alpha (.) (H x) + beta,      sumsq[n] = sum_j y[n,j]^2.
 * (Sec. 6 of the paper leaves the interplay of the layer with RMSNorm open; with the statistic
 * delivered by the layer's epilogue, the normalisation has no reduction pass of its own and can be
 * folded into its consumer.)  The squares are taken from the float32 values before they are rounded
 * to `dtype` for the store, and summed in float32 in a fixed order (bit-reproducible).
 *   sumsq  out  [N]  float32, 4-byte aligned, overwritten.
 * Its backward is wht_affine_backward as well: the statistic's own gradient belongs to the
 * normalisation that consumes it.
 */
int wht_affine_forward_residual_stats(const void *x, const float *alpha, const float *beta,
                                      const void *resid, void *y, float *sumsq,
                                      int64_t N, int32_t d, int32_t dtype, void *stream);

/*
 * Bytes of device scratch wht_affine_backward needs for (N, d, dtype): per-workgroup partial sums
 * of dalpha and dbeta, float32.  Depends on d only through the launch shape; 0 when N = 0 or when
 * the arguments are invalid.  Needs no GPU.
 */
size_t wht_affine_backward_workspace_bytes(int64_t N, int32_t d, int32_t dtype);

/*
 * Backward of Eq. 1 (see the header comment).
 *   dy      in   [N,d] dtype
 *   x       in   [N,d] dtype      the forward input; z = H x is recomputed
 *   alpha   in   [d]   float32
 *   dx      out  [N,d] dtype      written once
 *   dalpha  out  [d]   float32    overwritten (not accumulated into)
 *   dbeta   out  [d]   float32    overwritten
 *   workspace    device scratch, 16-byte aligned, at least ..._workspace_bytes(N, d, dtype) bytes;
 *                contents on entry are ignored, contents on return are unspecified
 * The reduction over tokens has a fixed order: results are bit-reproducible run to run.
 *
 * Outputs may be left out:
 *   dalpha = dbeta = NULL   only dx is computed (frozen parameters).  x and workspace are then not
 *                           used and may be NULL; the call moves the bytes of a forward pass.
 *   dx = NULL               only dalpha and dbeta are computed.
 * dalpha and dbeta come together: exactly one of them NULL, or all three outputs NULL, is
 * WHT_ERR_NULL_PTR.  The values of the outputs that are computed do not depend on which others are.
 */
int wht_affine_backward(const void *dy, const void *x, const float *alpha,
                        void *dx, float *dalpha, float *dbeta,
                        int64_t N, int32_t d, int32_t dtype,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * wht_affine_backward for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, outputs and results (bit for
 * bit) as wht_affine_backward, without the workspace: the per-workgroup partial sums go to a buffer
 * of WHT_STATIC_WORKSPACE_BYTES that is part of the library's code object (every GPU the library
 * runs on holds one until the process ends).  The call allocates and frees nothing.
 *   - A call that would need more than WHT_STATIC_WORKSPACE_BYTES of partial sums
 *     (wht_affine_backward_workspace_bytes(N, d, dtype); today: d > 8192) returns WHT_ERR_WORKSPACE
 *     and enqueues nothing.
 *   - All calls on one GPU share that GPU's buffer.  Calls on one stream are ordered and safe; two
 *     calls that may run at the same time on one GPU (different streams) race on it -- give those
 *     their own workspaces through wht_affine_backward.  The buffer's contents between calls are
 *     unspecified; nothing in it has to start at zero.
 *   - The first call on a GPU looks the buffer's address up once (with that GPU current); if that
 *     fails the call returns WHT_ERR_LAUNCH.
 */
#define WHT_STATIC_WORKSPACE_BYTES (16u << 20)
int wht_affine_backward_static(const void *dy, const void *x, const float *alpha,
                               void *dx, float *dalpha, float *dbeta,
                               int64_t N, int32_t d, int32_t dtype, void *stream);

/* Static, NUL-terminated description of a wht_status_t (host memory, never freed). */
const char *wht_affine_status_string(int status);

/* Library version, major * 10000 + minor * 100 + patch. */
int wht_affine_version(void);

#ifdef __cplusplus
}
#endif
#endif /* WHT_AFFINE_H */
