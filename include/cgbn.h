/*
 * libcgbn -- Cross-GPU Batch Normalization (CGBN) forward and backward for one
 * MI355X (gfx950), with the method's n devices appearing as K "virtual
 * devices": K contiguous, equal sub-batch shards of one activation tensor.
 *
 * Method: MegDet, section 3.3 "Cross-GPU Batch Normalization", Algorithm 1.
 *   steps 1-3   device sums            s[k,c] = sum over shard k of x
 *   steps 4-5   reduce + broadcast     mean[c] = (sum_k s[k,c]) / M
 *   steps 6-8   device variance sums   v[k,c] = sum over shard k of (x - mean[c])^2
 *   steps 9-10  reduce + broadcast     var[c]  = (sum_k v[k,c]) / M   (biased)
 *   step 11     y = gamma (x - mean)/sqrt(var + eps) + beta
 * with M = N*H*W the pooled count per channel.  The paper gives no backward;
 * the one here is the chain rule through the pooled mean and variance:
 *   a[k,c] = sum over shard k of dy,   b[k,c] = sum over shard k of dy*xhat
 *   dbeta = sum_k a,  dgamma = sum_k b,  xhat = (x - mean) * invstd
 *   dx = gamma * invstd * (dy - dbeta/M - xhat * dgamma/M)
 *
 * Conventions common to every entry point
 *   - Every tensor/vector pointer is a DEVICE pointer owned by the caller; the
 *     library never allocates, frees or keeps device memory.  Scratch is the
 *     caller's `workspace` (size from cgbn_workspace_bytes, contents undefined
 *     after a call).  Activation tensors (x, y, dy, dx) are dense in `layout`
 *     with element type `dtype`, their base address 16-byte aligned.  Per-channel
 *     vectors are float[C]; shard partials are double[K*C], index k*C + c.
 *   - Shard k holds images [k*N/K, (k+1)*N/K); 1 <= K <= N and N % K == 0.
 *   - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream).  No call synchronises, reads back or allocates, and scratch is
 *     cleared by kernels, so a sequence of calls can be captured into a HIP graph and
 *     replayed (with the same pointers).
 *   - Errors: the return code only.  Argument errors are found on the host
 *     before any launch and leave every output untouched.  CGBN_ERR_HIP wraps a
 *     failed launch.  NaN/Inf in the data are not errors; they propagate within
 *     their channel.  Per-row partial sums are floats (cross-row sums doubles), so
 *     a channel's squared deviations must stay inside float range (|x - mean| up
 *     to about 1e18) for the stated accuracy.
 *   - Aliasing: y may be exactly x, dx may be exactly dy; any other overlap of
 *     an output with another argument is undefined.
 *   - `mean_lo` (optional, may be NULL everywhere): float[C] holding the part of
 *     the pooled mean that does not fit `mean`'s float, mean + mean_lo being the
 *     mean to about double precision.  The forward uses it internally in any
 *     case; exporting it lets the backward see the same mean when |mean| is
 *     orders of magnitude above the channel's spread.
 *   - Concurrency: calls on ONE stream, or on several streams as long as they do not run at
 *     the same time, need nothing special.  cgbn_forward / cgbn_backward calls that may
 *     overlap in time on one device (different streams, each with its own workspace) must
 *     set the "cooperative" knob first: their single-launch kernels wait for sibling
 *     workgroups, and two such grids dispatched together could each end up half resident and
 *     starve the other until the bounded waits give up (error word set, NaN statistics).
 *     A workspace must never be shared by calls that can overlap.
 *   - Results are bitwise reproducible run to run (fixed summation order, no
 *     floating-point atomics) and depend on K only through rounding.
 */
#ifndef CGBN_H
#define CGBN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Status, layout and dtype travel as plain ints (any value a caller passes is representable; values outside
 * the lists below are answered with CGBN_ERR_ENUM, or "unknown status"). */
typedef int cgbn_status;
enum {
    CGBN_OK = 0,
    CGBN_ERR_NULL = 1,       /* a required pointer is NULL */
    CGBN_ERR_SHAPE = 2,      /* a dimension is < 1 or the tensor is too large to index */
    CGBN_ERR_SHARD = 3,      /* K < 1, K > N or N % K != 0 */
    CGBN_ERR_ENUM = 4,       /* layout or dtype out of range */
    CGBN_ERR_EPS = 5,        /* eps is not finite and > 0 */
    CGBN_ERR_WORKSPACE = 6,  /* workspace NULL, misaligned (256 B) or too small */
    CGBN_ERR_ALIGN = 7,      /* an activation tensor is not 16-byte aligned */
    CGBN_ERR_HIP = 8,        /* the HIP runtime refused a launch */
    CGBN_ERR_TUNING = 9,     /* unknown tuning key or value out of range */
    CGBN_ERR_MOMENTUM = 10,  /* momentum outside [0, 1] */
    CGBN_ERR_ALIAS = 11,     /* two outputs that must differ are the same buffer */
    CGBN_ERR_SCRATCH = 12    /* cgbn_forward_static: the problem needs more than CGBN_STATIC_SCRATCH_BYTES */
};

typedef int cgbn_layout;
enum { CGBN_NCHW = 0, CGBN_NHWC = 1 };
typedef int cgbn_dtype;      /* of x, y, dy, dx */
enum { CGBN_F32 = 0, CGBN_BF16 = 1 };

/* Bytes of workspace any entry point below needs for this problem (a multiple
 * of 256; the workspace itself must be 256-byte aligned).  Returns 0 if the
 * arguments are invalid.  Host-only, launches nothing. */
size_t cgbn_workspace_bytes(int N, int C, int H, int W, cgbn_layout layout,
                            cgbn_dtype dtype, int K);

/* Byte offset, inside a workspace, of a 32-bit word that is 0 after cgbn_forward /
 * cgbn_backward unless a bounded device-side wait gave up (it cannot when the launch is
 * sound; if it does, the statistics of the affected channels are NaN).  The offset is the
 * same for every problem; (size_t)-1 if the arguments are invalid.  Callers that do not
 * want to read workspace memory themselves use cgbn_workspace_status. */
size_t cgbn_workspace_error_offset(int N, int C, int H, int W, cgbn_layout layout,
                                   cgbn_dtype dtype, int K);

/* The first-class way to learn of such a give-up: enqueues on `stream` a one-thread kernel
 * that sets *gave_up (a DEVICE int owned by the caller) to 1 if the error word of
 * `workspace` is up, and leaves it untouched otherwise.  Call it after the cgbn_forward /
 * cgbn_backward (or their ReLU variants) it is to watch, on the same stream and before the
 * next call that uses the workspace (every such call clears the word when it starts).  Zero
 * *gave_up once, let any number of layers raise it, and read it when the host next
 * synchronises anyway (once per training step, say): a non-zero value means that some
 * statistics of that step are NaN because the device was shared with other kernels in a way
 * the launch could not cope with (see "Concurrency" above and the "cooperative" knob). */
cgbn_status cgbn_workspace_status(const void* workspace, int* gave_up, void* stream);

/* Algorithm 1, all steps.  In: x, gamma[C], beta[C], eps.  Out: y (same shape,
 * layout and dtype as x; bf16 rounded to nearest-even), mean[C], invstd[C] =
 * 1/sqrt(var + eps), and mean_lo[C] if not NULL. */
cgbn_status cgbn_forward(const void* x, int N, int C, int H, int W, cgbn_layout layout, int K,
                         const float* gamma, const float* beta, float eps,
                         void* y, float* mean, float* invstd,
                         cgbn_dtype dtype, float* mean_lo,
                         void* workspace, size_t workspace_bytes, void* stream);

/* cgbn_forward for callers that can neither allocate device memory nor bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * kernels and results as cgbn_forward, without `workspace` / `workspace_bytes`: the scratch is a
 * static device array of CGBN_STATIC_SCRATCH_BYTES inside the library (each GPU the library runs
 * on holds one until the process ends).  The call allocates and frees nothing, on the device or
 * through any allocating library routine.
 *   - A problem whose cgbn_workspace_bytes exceeds CGBN_STATIC_SCRATCH_BYTES is refused with
 *     CGBN_ERR_SCRATCH before anything is launched (the five detector-shaped workloads of this
 *     repository need 0.01 to 8.1 MiB).
 *   - The array's device address is looked up on the first call on each device; make that call
 *     outside a graph capture.
 *   - Every call on a GPU uses that GPU's one array: calls that can overlap in time on one GPU
 *     (different streams) race on it and must not be made; back-to-back calls on one stream are
 *     fine (whatever must start cleared is cleared by kernels of the call itself).
 *   - The give-up word of the single-launch kernels lives in the array too; there is no
 *     workspace pointer to pass to cgbn_workspace_status, so watch it through NaN statistics. */
#define CGBN_STATIC_SCRATCH_BYTES (16u << 20)
cgbn_status cgbn_forward_static(const void* x, int N, int C, int H, int W, cgbn_layout layout, int K,
                                const float* gamma, const float* beta, float eps,
                                void* y, float* mean, float* invstd,
                                cgbn_dtype dtype, float* mean_lo, void* stream);

/* Backward of Algorithm 1's last step through the pooled statistics.  In: dy, x,
 * mean[C], invstd[C] as written by cgbn_forward, gamma[C], mean_lo[C] or NULL.
 * Out: dx, dgamma[C], dbeta[C]. */
cgbn_status cgbn_backward(const void* dy, const void* x, const float* mean, const float* invstd,
                          const float* gamma, void* dx, float* dgamma, float* dbeta,
                          int N, int C, int H, int W, cgbn_layout layout, int K,
                          cgbn_dtype dtype, const float* mean_lo,
                          void* workspace, size_t workspace_bytes, void* stream);

/* ---- CGBN followed by a shortcut add and a ReLU, the two placements of a normalization
 * layer in the detector's backbone (ResNet-50, section 4): y = max(0, z) inside a block,
 * y = max(0, z + shortcut) at a block's end, z being Algorithm 1's output.  The paper does
 * not discuss the activation; fusing it here saves the separate sweeps over y and dy. ---- */

/* As cgbn_forward, then y = max(0, z + shortcut).  `shortcut` (same shape, layout and
 * dtype as x) may be NULL: y = max(0, z).  The statistics are those of x alone.
 * y may be exactly x or exactly shortcut. */
cgbn_status cgbn_forward_relu(const void* x, const void* shortcut, int N, int C, int H, int W,
                              cgbn_layout layout, int K, const float* gamma, const float* beta, float eps,
                              void* y, float* mean, float* invstd, cgbn_dtype dtype, float* mean_lo,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Its backward.  `y` is the output cgbn_forward_relu stored: gradient passes where y > 0
 * (dz = dy there, 0 elsewhere), then dbeta, dgamma, dx as in cgbn_backward with dz for dy.
 * `dshortcut`, if not NULL, receives dz (the gradient of the shortcut).  dx may be exactly
 * dy, or dshortcut may be exactly dy; dx and dshortcut must differ (CGBN_ERR_ALIAS). */
cgbn_status cgbn_backward_relu(const void* dy, const void* y, const void* x,
                               const float* mean, const float* invstd, const float* gamma,
                               void* dx, void* dshortcut, float* dgamma, float* dbeta,
                               int N, int C, int H, int W, cgbn_layout layout, int K,
                               cgbn_dtype dtype, const float* mean_lo,
                               void* workspace, size_t workspace_bytes, void* stream);

/* ---- The same path one step at a time, one sweep over the tensor per call.
 * cgbn_forward and cgbn_backward run these kernels back to back where a shape
 * does not qualify for their single-launch kernels (and always when the
 * "fused" knob is 0).  Meant for tests and measurement. ---- */

/* Algorithm 1 steps 1-3: s[k*C + c] = sum over shard k of x. */
cgbn_status cgbn_shard_sum(const void* x, int N, int C, int H, int W, cgbn_layout layout, int K,
                           cgbn_dtype dtype, double* s,
                           void* workspace, size_t workspace_bytes, void* stream);

/* Steps 4-5: mean[c] = (sum_k s[k,c]) / M, with M given as a count.  mean_lo optional. */
cgbn_status cgbn_reduce_mean(const double* s, int K, int C, long long M,
                             float* mean, float* mean_lo, void* stream);

/* Steps 6-8: v[k*C + c] = sum over shard k of (x - mean[c])^2 (mean_lo optional). */
cgbn_status cgbn_shard_sqdev(const void* x, int N, int C, int H, int W, cgbn_layout layout, int K,
                             cgbn_dtype dtype, const float* mean, const float* mean_lo, double* v,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Steps 9-10: invstd[c] = 1/sqrt((sum_k v[k,c])/M + eps). */
cgbn_status cgbn_reduce_invstd(const double* v, int K, int C, long long M, float eps,
                               float* invstd, void* stream);

/* Step 11: y = gamma*(x - mean)*invstd + beta. */
cgbn_status cgbn_normalize(const void* x, int N, int C, int H, int W, cgbn_layout layout,
                           cgbn_dtype dtype, const float* mean, const float* mean_lo,
                           const float* invstd, const float* gamma, const float* beta,
                           void* y, void* stream);

/* Backward device sums: a[k*C + c] = sum dy, b[k*C + c] = sum dy*xhat over shard k. */
cgbn_status cgbn_backward_shard_sums(const void* dy, const void* x, int N, int C, int H, int W,
                                     cgbn_layout layout, int K, cgbn_dtype dtype,
                                     const float* mean, const float* mean_lo, const float* invstd,
                                     double* a, double* b,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* Backward reduce: dbeta[c] = sum_k a[k,c], dgamma[c] = sum_k b[k,c]. */
cgbn_status cgbn_backward_reduce(const double* a, const double* b, int K, int C,
                                 float* dbeta, float* dgamma, void* stream);

/* dx = gamma*invstd*(dy - dbeta/M - xhat*dgamma/M). */
cgbn_status cgbn_backward_dx(const void* dy, const void* x, int N, int C, int H, int W,
                             cgbn_layout layout, cgbn_dtype dtype,
                             const float* mean, const float* mean_lo, const float* invstd,
                             const float* gamma, const float* dgamma, const float* dbeta,
                             void* dx, void* stream);

/* ---- Fixed-statistics ("frozen") mode: the layer the paper's baseline detectors use
 * (section 3.1; opening of section 3.3; Table 3, row "16-base", BN size 0), where the
 * statistics are constants computed beforehand.  One elementwise sweep each; no
 * workspace.  The paper does not say how the constants come about; the update below is
 * the exponential moving average of the batch-normalization work section 3.3 builds on,
 * with `momentum` and `unbiased` left to the caller. ---- */

/* y = gamma*(x - fixed_mean)/sqrt(fixed_var + eps) + beta: the formula of Algorithm 1's last
 * step with constants for the statistics.  fixed_mean[C], fixed_var[C] (variances, not
 * their inverse roots), gamma[C], beta[C].  y may be exactly x. */
cgbn_status cgbn_frozen_forward(const void* x, int N, int C, int H, int W, cgbn_layout layout,
                                cgbn_dtype dtype, const float* fixed_mean, const float* fixed_var,
                                const float* gamma, const float* beta, float eps,
                                void* y, void* stream);

/* Its backward.  Statistics and affine parameters are constants of the layer, so
 * dx = dy*gamma/sqrt(fixed_var + eps) and there is no dgamma/dbeta.  dx may be exactly dy. */
cgbn_status cgbn_frozen_backward(const void* dy, int N, int C, int H, int W, cgbn_layout layout,
                                 cgbn_dtype dtype, const float* fixed_var, const float* gamma,
                                 float eps, void* dx, void* stream);

/* After a cgbn_forward with the same eps over M = N*H*W values per channel:
 *   running_mean <- (1-momentum)*running_mean + momentum*(mean + mean_lo)
 *   running_var  <- (1-momentum)*running_var  + momentum*var*(unbiased ? M/(M-1) : 1)
 * in place, with var = 1/invstd^2 - eps (accurate to about 2e-7*(var + eps)).  mean_lo may
 * be NULL.  0 <= momentum <= 1, else CGBN_ERR_MOMENTUM; unbiased needs M >= 2. */
cgbn_status cgbn_update_running_stats(const float* mean, const float* mean_lo, const float* invstd,
                                      float eps, long long M, int C, float momentum, int unbiased,
                                      float* running_mean, float* running_var, void* stream);

/* ---- housekeeping ---- */

/* Static, never NULL. */
const char* cgbn_status_string(cgbn_status status);

/* Launch-shape knobs for measurement sweeps.  They are process-wide; reading and writing
 * them is serialised, and every call of the library works on ONE copy of them taken when it
 * starts, so calls from several host threads are safe and a call never sees half of a
 * change.  The workspace size depends on some of them: re-query cgbn_workspace_bytes after
 * a change (a call whose workspace is too small for the knobs it runs under returns
 * CGBN_ERR_WORKSPACE before launching anything).
 *   "chunk_bytes"      NCHW: bytes of one plane handled by one workgroup
 *   "wave_plane_bytes" NCHW: planes up to this size are handled by one wavefront
 *   "tiny_planes"      0/1 (default 1): NCHW planes of at most 2 KiB, C a multiple of 8: a workgroup of the
 *                      multi-sweep kernels takes a run of 8 ... 256 planes of consecutive channels at once
 *   "piece_bytes"      NHWC reductions: bytes of one pixel range handled by one workgroup (0, the default:
 *                      chosen per shape so that the grid fills the device's compute units evenly)
 *   "map_piece_bytes"  NHWC normalise / dx: the same for the elementwise sweeps (0, the default: 128 KiB for
 *                      bfloat16; for float 64 KiB where the sweep reads one tensor, 32 KiB where it reads more)
 *   "reverse"          0/1: alternate the sweep direction between consecutive sweeps
 *   "nt_store"         0/1: non-temporal stores for y and dx
 *   "fused"            0/1: register-resident single-launch forward/backward (NCHW)
 *   "one_sweep_stats"  0/1 (default 1): where cgbn_forward runs as separate sweeps, steps 1-10 come from ONE sweep
 *                      over x: each row partial is the sum about a per-channel pivot and M2, the squared
 *                      deviations from the row's own mean (formed chunk by chunk in registers, never as a
 *                      difference of large sums); the combine step turns them into Algorithm 1's sums about the
 *                      pooled mean by the pairwise update.  3 tensor sweeps instead of 4, same results up to
 *                      rounding.  0: one sweep for the sums, a second for the squared deviations (what the
 *                      step-by-step entry points below always do)
 *   "cooperative"      0/1 (default 0): launch the single-launch kernels cooperatively, so that the runtime
 *                      guarantees the whole grid is resident; needed only if such calls can overlap on
 *                      different streams; costs about 15 us per launch
 *   "big_lds"          0/1 (default 1): NCHW shapes with at most 384 rows and 48 (large planes) or 128 (small
 *                      planes) shards use variants of the single-launch kernels that stage few rows and keep
 *                      more unit data in LDS
 *   "fused_groups"     workgroups of that launch (0 = all that are resident at once)
 *   "stagger"          0/1 (default 1): the single-launch kernels start their channel slots class by class, so
 *                      that the slots' load, hand-over and write-out phases interleave
 *   "stagger_us"       microseconds by which the last class starts after the first (0, the default: chosen
 *                      per launch, none for short launches)
 *   "stagger_phases"   number of such classes (2..64, default 16)
 *   "spin_limit"       polls before a device-side wait gives up (0: at once; for tests of that path)
 *   "wait_us"          microseconds of wall-clock time before it gives up (default 100000); once one wait
 *                      of a launch has given up, its later waits do so at once
 * cgbn_get_tuning returns -1 for an unknown key. */
cgbn_status cgbn_set_tuning(const char* key, long long value);
/* also readable: "last_forward_fused", "last_backward_fused" (1 if the last
 * cgbn_forward / cgbn_backward took the single-launch path) */
long long cgbn_get_tuning(const char* key);

/* One number of the launch plan the library would use for this problem under the current
 * knobs; host-only, launches nothing, -1 for invalid arguments or an unknown key.  For tests
 * of the host-side planning (every kernel trusts these numbers for its indexing).
 * Multi-sweep kernels: "grid" (workgroups of a reduction sweep), "gridm" (of a channels-last
 * elementwise sweep), "rows" / "rps" (row partials per channel / per shard), "G" (lanes adding
 * one shard's rows), "part_bytes" / "shard_bytes" (workspace bytes of one array of row partials /
 * of shard sums); NCHW: "wave_mode" (one wavefront per plane), "L" / "sp" (chunk elements, chunks
 * per plane); NHWC: "vec" (elements per access), "cv" (accesses per pixel), "TW" / "ctiles"
 * (accesses per pixel handled by one workgroup, workgroups per pixel), "rpp" (pixels per pass),
 * "PL" / "pps" (pixels per piece, pieces per shard; reductions), "PLm" / "ppsm" (elementwise).
 * Single-launch kernels, prefix "fwd_" or "bwd_": "ok" (the shape qualifies), "LB" (bytes per
 * access), "LPPC" (register slots per small plane; 0: large planes), "LPP" (slots a plane fills),
 * "IPU" (images per unit), "U" (units per channel), "tp" / "TL" (tiles per large plane, tile
 * elements), "rows", "rps", "G", "big" (0, or which LDS variant), "total_units". */
long long cgbn_plan_get(int N, int C, int H, int W, cgbn_layout layout, cgbn_dtype dtype, int K,
                        const char* key);

/* A plain device-to-device copy of `bytes` bytes (a multiple of 16, both
 * pointers 16-byte aligned) by a kernel of this library: it reads and writes a
 * known number of bytes, which is what hardware traffic counters are calibrated
 * against when the library's kernels are profiled. */
cgbn_status cgbn_calibration_copy(const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CGBN_H */
