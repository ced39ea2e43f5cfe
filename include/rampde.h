/*
 * rampde.h -- C ABI of the MI355X (gfx950) mixed-precision neural-ODE time stepper.
 *
 * One library, two compute entry points:
 *   rampde_odeint_fwd : explicit Runge-Kutta forward pass with low-precision velocity
 *                       evaluations, fp32 solution accumulation and a low-precision
 *                       state trajectory (paper Algorithm 1).
 *   rampde_odeint_bwd : discrete adjoint of that forward pass: stage recomputation from the
 *                       stored states, low-precision vector-Jacobian products, dynamic
 *                       power-of-two adjoint scaling with overflow detection, fp32
 *                       accumulation of the adjoint and of the parameter gradient
 *                       (paper Algorithm 2 and eq. (vjp); update formulas of Sec. 3).
 *
 * Conventions
 *   - "dev" pointers are device (HBM) pointers owned by the caller, 16-byte aligned (RAMPDE_EINVAL
 *     otherwise); "host" pointers are ordinary host memory.  The library allocates no device memory: all scratch comes
 *     from the caller's workspace (size from rampde_workspace_bytes).
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*, may be NULL
 *     for the default stream).  rampde_odeint_fwd never synchronises.  rampde_odeint_bwd
 *     synchronises the stream once before returning when it has to read something back: under
 *     DYNAMIC / NONE_SAFE scaling (the outcome of the overflow detector), or when scale_hist /
 *     stats are requested -- and once more per detected overflow, to retry from that step.
 *     Under SCALE_NONE with scale_hist = stats = NULL it does not synchronise at all.
 *   - Return value: 0 on success, otherwise a rampde_status code; rampde_strerror gives
 *     a message.  No exceptions.  Process-global state: the optional timing facility below, and
 *     one helper stream with a pool of events (default priority, created on first use, kept until
 *     the process ends) on which rampde_odeint_bwd runs the parameter-gradient kernels of narrow
 *     networks beside the adjoint kernels; it is joined into `hip_stream` before the call returns
 *     its last work, so callers see ordinary stream order.
 *   - Calls that share a workspace must not overlap; distinct workspaces on distinct streams may.
 *     The host side is not thread safe: calls from several host threads must be serialised by
 *     the caller.
 *   - theta layout (flat fp32, also the layout of grad_theta):
 *       MLP  : for each layer l: W_l[out_l][in_l] row-major, then b_l[out_l];
 *              layer 1 has in_1 = d + 1 when time_input is set (time column LAST).
 *       CONV2: W1[C][C+time_input][3][3], b1[C], W2[C][C+time_input][3][3], b2[C]
 *              (time channel LAST); zero padding 1, stride 1.
 *       PARABOLIC: for each piece q = 0 .. n_intervals-1: W_q[C][C][3][3], b_q[C].
 *     Activation is tanh after every layer but the last (MLP, CONV2); ReLU in PARABOLIC.
 *   - State layout at the boundary (y0, yN, grad_yN, grad_y0, grad_ys), fp32:
 *       MLP [B][d];  CNF [B][d+1] (l last);  CONV2 and PARABOLIC NCHW [B][C][H][W].
 *   - Checkpoint layout (ckpt, written by fwd, read by bwd; element type = policy.low):
 *       MLP [N+1][B][d];  CNF [N+1][B][d+1];  CONV2 and PARABOLIC channels-last [N+1][B][H][W][C].
 */
#ifndef RAMPDE_H
#define RAMPDE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { RAMPDE_F32 = 0, RAMPDE_F16 = 1, RAMPDE_BF16 = 2 } rampde_dtype;

/* Backward variants (paper Sec. 5, "three backward pass implementations"). */
typedef enum {
  RAMPDE_SCALE_NONE = 0,      /* unscaled: S = 1, no overflow checks                       */
  RAMPDE_SCALE_NONE_SAFE = 1, /* unscaled-safe: S = 1, overflow => gradients filled with +inf */
  RAMPDE_SCALE_DYNAMIC = 2,   /* dynamic adjoint scaling, Algorithm 2                      */
  RAMPDE_SCALE_AUTO = 3       /* F32/BF16 -> NONE, F16 -> DYNAMIC                          */
} rampde_scaling;

/* Velocity kinds.  PARABOLIC is the convolution block of the paper's image classifier,
 * f(y) = -W^T N(relu(W y + b))  (Sec. 6.3, eq. (NODE_STL10)): W a 3x3 convolution with C input and C
 * output channels (zero padding 1), W^T its exact transpose with the same weights, N the instance
 * normalisation (per sample and channel over the H*W pixels, biased variance, eps = 1e-5, no affine
 * parameters; statistics and arithmetic in fp32, result rounded to `low`).  No time input; instead the
 * parameters are piecewise constant in time: step i of an N-step grid uses piece i * n_intervals / N
 * (integer division) for all of its stages.
 * CNF is the augmented state of a continuous normalising flow (Sec. 6.1): y = [z; l] with d + 1 columns,
 * dz/dt = v(t, z) = W2 tanh(W1 [z; t] + b1) + b2 (n_layers = 2, widths = {d, H, d}), dl/dt = -tr(dv/dz)
 * formed analytically (sum_h c_h (1 - a_h^2), c_h = sum_i W2[i,h] W1[h,i], in fp32 from the rounded
 * weights and activations, rounded to `low` like the other slope entries).  theta is that of the MLP. */
typedef enum { RAMPDE_VEL_MLP = 0, RAMPDE_VEL_CONV2 = 1, RAMPDE_VEL_PARABOLIC = 2, RAMPDE_VEL_CNF = 3 } rampde_vel_kind;

typedef enum {
  RAMPDE_OK = 0,
  RAMPDE_EINVAL = 1,       /* null pointer, N < 1, non-increasing grid, tableau not strictly lower triangular, ... */
  RAMPDE_EUNSUPPORTED = 2, /* dtype / velocity kind / shape not built                        */
  RAMPDE_EWORKSPACE = 3,   /* workspace too small or misaligned (256 B)                      */
  RAMPDE_ESCALE = 4,       /* dynamic adjoint scaling failed at step stats.failed_step (Alg. 2, error branch) */
  RAMPDE_EHIP = 5          /* HIP runtime error                                              */
} rampde_status;

/* policy.flags */
#define RAMPDE_ROUND_INCREMENT 1u /* round sum_j b_j k_j to `low` before the fp32 add (the literal update line of Alg. 1) */
#define RAMPDE_GROW_RAW_NORM 2u   /* growth test on the unscaled norm ||a|| <= 1/(2 u_L) (literal Alg. 2)     */
#define RAMPDE_PER_LAYER_KERNELS 4u /* dense networks: use one kernel per layer instead of the row-tile-persistent kernels */
#define RAMPDE_NAIVE_STATE 8u       /* comparison baseline, not the paper's scheme: the state y and the adjoint a are
                                     themselves kept in low precision (rounded after every update), i.e. without
                                     the fp32 accumulators of Algorithms 1-2 (the "naive" rows of the paper's Table 5) */

/* Explicit Butcher tableau, host memory, fp64.  A is s*s row-major; only the strictly
 * lower triangle may be non-zero (checked).  Consistency (sum b = 1, ...) is not checked. */
typedef struct {
  int s;
  const double *A;
  const double *b;
  const double *c;
} rampde_tableau;

/* Velocity network descriptor (host memory). */
typedef struct {
  rampde_vel_kind kind;
  int n_layers;      /* MLP: number of linear layers (>= 1)                           */
  const int *widths; /* MLP: n_layers + 1 entries, widths[0] = widths[n_layers] = d   */
  int C, H, W;       /* CONV2, PARABOLIC: channels and spatial size; kernel 3x3, padding 1 */
  int time_input;    /* 1: append t as last input column (MLP, layer 1) / channel (each conv); PARABOLIC: 0 */
  int n_intervals;   /* PARABOLIC: pieces of the piecewise-constant parameters (0 or 1: constant in time) */
} rampde_velocity;

typedef struct {
  rampde_dtype low;       /* precision of velocity evaluations, stage values and checkpoints */
  rampde_scaling scaling;
  int k_max;              /* max attempts per step under DYNAMIC (Alg. 2); <= 0 means 16     */
  unsigned flags;
  /* Launch-shape choices; 0 = let the library choose.  They change how the work is cut into
   * kernels, never what is computed (results agree to fp32 summation order). */
  int step_group;         /* dense networks, fixed scale (SCALE_NONE): cap on the adjoint steps that one
                             launch runs (default: as many as about 4 GiB of workspace hold, at most 64).
                             With overflow detection the adjoint runs step by step; where wgrad_tile = 256
                             applies this is the number of accepted steps whose parameter gradients one launch
                             forms (default: as many as keep their buffers in the memory-side cache) */
  int row_tile;           /* dense networks: batch rows per workgroup of the row-tile kernels: 16, 32 or 64.
                             64 selects the kernels built for 512-wide networks (state width 128) where
                             they apply; values that do not apply fall back to the automatic choice  */
  int wgrad_tile;         /* dense networks, row-tile kernels, one launch per adjoint step: which kernel forms the
                             parameter gradients.  128: workgroups with a 128 x 128 block of dW_l; 256: wavefronts
                             with a 128 x 128 block each, operands streamed through LDS by direct loads (built for
                             long batch contractions).  0: chosen by the contraction length (stages x batch rows).
                             Convolutions with 64 channels, or PARABOLIC with channel counts in multiples of 128, and W in {16, 32, 64}: 64 keeps the
                             convolution weight-gradient kernel with 64 x 64 channel blocks per workgroup instead of
                             the one with 128 x 128 x 3-tap blocks built on transposing LDS reads (the default there),
                             and the convolution kernel that fetches an input slab per tap instead of the one that
                             stages the input by image lines */
  /* Scope of the adjoint scale within a batch (Alg. 2 is stated for one sample).  0: one scale S for the
   * whole batch (the default).  G > 0: every G consecutive samples (the last group: the remainder) share a
   * scale of their own -- initial value from the group's own max-norm, own overflow retries, own growth --
   * and the group's share of dL/dtheta (and dL/dt) is unscaled with its own h / S before it is added to
   * the other groups'.  Absent overflow and underflow the result is that of G = 0 up to fp32 summation
   * order.  G times the number of state elements of a sample must be a multiple of 8 (every group's
   * slice of the caller's buffers starts 16-byte aligned; RAMPDE_EINVAL otherwise).  This field changes
   * WHAT is computed, unlike the three above. */
  int scale_group;
} rampde_policy;

typedef struct {
  int status;        /* 0 ok; 1 = overflow under NONE_SAFE (gradients are +inf); 2 = scaling failed */
  int failed_step;   /* step index i of the failure, -1 if none                                  */
  int retries;       /* number of halvings over the whole pass                                   */
  float s_first;     /* S_N                                                                      */
  float s_last;      /* accepted S_0                                                             */
  float s_min, s_max;
} rampde_stats;

/* Number of parameters P implied by a velocity descriptor (0 if invalid). */
int64_t rampde_num_params(const rampde_velocity *vel);

/* Bytes of device workspace needed by fwd (is_backward = 0) or bwd (= 1). 0 if invalid.
 * The size depends on the policy: with a fixed scale (SCALE_NONE) the backward pass of a dense
 * network keeps the low-precision stage inputs, activations and cotangents of a whole group of
 * steps (up to 64 steps or about 4 GiB) so that their parameter gradients are one contraction;
 * with overflow detection it keeps those of two steps.  Pass the same policy to the query and
 * to the call. */
size_t rampde_workspace_bytes(const rampde_velocity *vel, int64_t B, int N,
                              const rampde_tableau *tab, const rampde_policy *pol,
                              int is_backward);

/* Forward pass, Algorithm 1.
 *   theta   dev, P fp32 (master weights; rounded to `low` once inside: the weight rounding of Alg. 1)
 *   y0      dev, B*d fp32
 *   tgrid   host, N+1 strictly increasing fp64
 *   ckpt    dev, (N+1)*B*d elements of `low`, written: ckpt[i] = Q_low(y_i)
 *   yN      dev, B*d fp32, written: the fp32 accumulator after the last step
 *   workspace dev, >= rampde_workspace_bytes(..., 0) bytes, 256-byte aligned
 * Asynchronous on hip_stream. */
int rampde_odeint_fwd(const rampde_velocity *vel, const float *theta, const float *y0,
                      int64_t B, const double *tgrid, int N, const rampde_tableau *tab,
                      const rampde_policy *pol, void *ckpt, float *yN, void *workspace,
                      size_t workspace_bytes, void *hip_stream);

/* rampde_odeint_fwd for callers that cannot allocate device memory or size a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and stream behaviour as rampde_odeint_fwd (the same kernels run), but the workspace is a static
 * device array of RAMPDE_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held until the
 * process ends.  The call performs no hipMalloc / hipFree and creates no events (the optional timing
 * facility does not record it).  The first call on each device looks the array's address up (that
 * may load the library's code object): make it once before capturing.
 *   - RAMPDE_EWORKSPACE, with nothing launched, if rampde_workspace_bytes(vel, B, N, tab, pol, 0)
 *     exceeds RAMPDE_STATIC_SCRATCH_BYTES.  (Full-size dense workloads of the paper fit; the
 *     128 x 64 x 32 x 32 convolutional one does not.)
 *   - All calls on one GPU share that GPU's array, on whatever stream: calls that overlap in time on
 *     one GPU race.  Nothing in the array has to survive from one call to the next, and nothing in it
 *     is assumed to be zero at entry. */
#define RAMPDE_STATIC_SCRATCH_BYTES ((size_t)32 << 20)
int rampde_odeint_fwd_static(const rampde_velocity *vel, const float *theta, const float *y0,
                             int64_t B, const double *tgrid, int N, const rampde_tableau *tab,
                             const rampde_policy *pol, void *ckpt, float *yN, void *hip_stream);

/* Backward pass, Algorithm 2 (without the time-grid gradient: see rampde_odeint_bwd_tgrid).
 *   ckpt       dev, read: the trajectory written by rampde_odeint_fwd with the same arguments
 *   grad_yN    dev, B*d fp32: dL/dy_N (the terminal-cost gradient, formed by the caller)
 *   grad_ys    dev or NULL: (N+1)*B*d fp32 per-step cotangents dL/dy_i of a running cost,
 *              added to the adjoint in fp32 (entry N at initialisation, entry i after step i)
 *   grad_y0    dev, B*d fp32, written: dL/dy_0
 *   grad_theta dev, P fp32, ACCUMULATED into (Alg. 2 starts g at the caller's dL/dtheta):
 *              zero it for a plain gradient
 *   scale_hist host or NULL, N+1 floats: [N] = S_N, [i] = accepted S_i; with policy.scale_group = G in
 *              (0, B): ceil(B / G) * (N+1) floats, one such row per group, in batch order
 *   stats      host or NULL; with scale groups: retries summed, s_min / s_max over all groups, s_first /
 *              s_last of the first group, status / failed_step of the worst group (the groups run one after
 *              the other on the caller's stream and workspace; workspace size from rampde_workspace_bytes
 *              with the same policy)
 * Returns RAMPDE_ESCALE if no finite scale was found within k_max attempts at some step
 * (outputs then undefined).  Under NONE_SAFE an overflow is not an error: grad_y0 and
 * grad_theta are filled with +inf and stats.status = 1. */
int rampde_odeint_bwd(const rampde_velocity *vel, const float *theta, int64_t B,
                      const double *tgrid, int N, const rampde_tableau *tab,
                      const rampde_policy *pol, const void *ckpt, const float *grad_yN,
                      const float *grad_ys, float *grad_y0, float *grad_theta,
                      float *scale_hist, rampde_stats *stats, void *workspace,
                      size_t workspace_bytes, void *hip_stream);

/* Backward pass that also forms the time-grid gradient dL/dt (paper Sec. 3, the update lines of
 * t'_i and t'_{i+1}; Alg. 2 returns dL/dt beside dL/dx and dL/dtheta).  Arguments as for
 * rampde_odeint_bwd, plus
 *   grad_t   dev or NULL, N+1 fp32, ACCUMULATED into (Alg. 2 starts t' at the caller's explicit
 *            dL/dt): zero it for a plain gradient.  NULL: exactly rampde_odeint_bwd.
 * With h = t[i+1] - t[i] and the step y_{i+1} = y_i + h Phi(y_i, t_i, h), per accepted step
 *   dt = lambda^T dPhi/dt,  dh = lambda^T dPhi/dh   from the same low-precision cotangent chain
 *   as the state and parameter cotangents, summed in fp32 and not rounded to 16 bits,
 *   t'_i += (h/S)(dt - dh) - Phi^T a_{i+1},   t'_{i+1} += (h/S) dh + Phi^T a_{i+1},
 * Phi = sum_j b_j k_j from the low-precision slopes, a_{i+1} the fp32 adjoint before the step's
 * update.  Sums over the batch: every workgroup writes a slot of its own and a one-workgroup kernel folds a launch's
 * slots in a fixed order (no floating-point atomics): two calls on the same inputs give the same bits. */
int rampde_odeint_bwd_tgrid(const rampde_velocity *vel, const float *theta, int64_t B,
                            const double *tgrid, int N, const rampde_tableau *tab,
                            const rampde_policy *pol, const void *ckpt, const float *grad_yN,
                            const float *grad_ys, float *grad_y0, float *grad_theta,
                            float *grad_t, float *scale_hist, rampde_stats *stats,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

const char *rampde_strerror(int code);

/* Library/ABI version, e.g. 100 = 1.0.0. */
int rampde_version(void);

/* Optional per-kernel timing, a measurement aid for benchmarks (off by default).
 * While enabled, every launch of the kernel classes below is bracketed by two HIP events on
 * the caller's stream (this perturbs end-to-end time slightly: measure throughput with it off).
 * Process-global and not thread safe.
 *   rampde_timing_enable(on) : drops all recorded events, then switches recording on/off.
 *   rampde_timing_read(cls, out) : waits for the recorded events of class cls and sums them:
 *       out->ms       total elapsed milliseconds of the launches,
 *       out->launches number of launches,
 *       out->work     algorithmic work of those launches: floating-point operations
 *                     (2 * M * N * K of the padded contraction) for the GEMM classes, bytes
 *                     for the streaming classes (per state element: forward update reads y (4),
 *                     s slopes (2 each), writes y (4) and the checkpoint (2); adjoint update
 *                     reads a (4), s stage cotangents (2 each), writes a (4)).            */
typedef enum {
  RAMPDE_K_VELOCITY_GEMM = 0,  /* forward layers, recomputation and input-cotangent products (Alg. 1: low-precision evaluation of Phi; eq. (vjp)) */
  RAMPDE_K_WGRAD_GEMM = 1,     /* parameter-gradient contractions over the batch (update of g, Sec. 3) */
  RAMPDE_K_COMBINE_STORE = 2,  /* fp32 solution update + low-precision checkpoint store (Alg. 1: accumulate and store) */
  RAMPDE_K_ADJOINT_UPDATE = 3, /* fp32 adjoint update + max-norm (Alg. 2, update of a) */
  RAMPDE_K_FUSED_FORWARD = 4,  /* dense networks: whole forward pass of a row tile, all steps, one launch (Alg. 1);
                                  work = flops of all its layer contractions */
  RAMPDE_K_FUSED_ADJOINT_STEP = 5, /* dense networks: recomputation + cotangent chain + adjoint update of one step (Alg. 2) */
  RAMPDE_K_CLASSES = 6
} rampde_kernel_class;
typedef struct {
  double ms;
  int64_t launches;
  double work;
} rampde_kernel_time;
int rampde_timing_enable(int on);
int rampde_timing_read(int kernel_class, rampde_kernel_time *out);

#ifdef __cplusplus
}
#endif
#endif /* RAMPDE_H */
