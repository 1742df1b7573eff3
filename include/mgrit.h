/*
 * mgrit.h -- C ABI of the MI355X (gfx950) layer-parallel hot path.
 *
 * The library solves the layer ODE of a pre-layer-norm transformer,
 *     Z_{n+1} = Z_n + h F(Z_n, theta_n),   n = 0 .. N-1          (paper sec. 3.1),
 * and its discrete adjoint  lambda_n = lambda_{n+1} + h (dF/dZ(Z_n))^T lambda_{n+1}
 * (sec. 3.1, the backward problem), with multigrid-reduction-in-time over the layer
 * index (sec. 3.2, Fig. 2, Appendix A): F- or FCF-relaxation batched over all
 * coarse intervals, injection restriction, full-approximation coarse equation,
 * serial coarsest solve, correction, recursion into V-cycles for more levels.
 *
 * General rules for every entry point
 *  - All pointers named "device" are HIP device pointers on the current device;
 *    "host" pointers are ordinary host memory.  The caller owns every buffer.
 *  - The library never allocates, frees or synchronises.  All work is enqueued on
 *    `stream` (a hipStream_t passed as void*; NULL = the null stream); outputs are
 *    valid once the caller has synchronised that stream.
 *  - Scratch memory comes from the caller's `workspace` (device, 256-byte aligned);
 *    query its size first.  Its contents are undefined afterwards.
 *  - Return value: MGRIT_OK (0) or a negative mgrit_status.  On MGRIT_INVALID_ARG,
 *    MGRIT_UNSUPPORTED and MGRIT_WORKSPACE_TOO_SMALL nothing has been enqueued or
 *    written.  No exception or abort crosses this boundary.
 *  - Results are run-to-run bit-identical (no atomics feed any state).
 *  - Threads: entry points that enqueue work may be called from several host threads; they
 *    serialise on a process-wide lock while they enqueue (a call holds it for its host-side
 *    duration, not for the GPU work), because the helper stream and the events of the two-lane
 *    mode exist once per device and are shared by all calls.  Calls issued on different caller
 *    streams are then ordered on the helper lane in the order the lock was taken; their results do
 *    not depend on it.  The tuning knobs below (lanes, groups per launch, adjoint cache, debug
 *    hooks) are process-global and unsynchronised: set them while no call is in progress, and
 *    query workspace sizes under the same settings as the call.  The last-error code is per thread.
 *
 * State layout: a state is [T, d_model] row-major fp32 with T = batch*seq tokens,
 * sequence b owning rows b*seq .. (b+1)*seq-1.  States, lambda, and every
 * residual update stay fp32 in both dtypes (the Euler sum is an accumulation).
 */
#ifndef MGRIT_H
#define MGRIT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mgrit_status {
  MGRIT_OK = 0,
  MGRIT_INVALID_ARG = -1,        /* null pointer, bad size, N not divisible by cf^(levels-1), ... */
  MGRIT_UNSUPPORTED = -2,        /* valid request this build has no kernel for */
  MGRIT_WORKSPACE_TOO_SMALL = -3,
  MGRIT_HIP_ERROR = -4           /* a HIP call failed; see mgrit_last_hip_error() */
} mgrit_status;

enum { MGRIT_ARCH_ENCODER = 0,   /* self-attention, no mask          (eq. "encoder") */
       MGRIT_ARCH_CAUSAL  = 1,   /* causal self-attention            (decoder-only)  */
       MGRIT_ARCH_CROSS   = 2 }; /* causal self-attn + cross-attn    (eq. "decoder") */

enum { MGRIT_DTYPE_F32  = 0,     /* fp32 parameters and matmul operands                      */
       MGRIT_DTYPE_BF16 = 1 };   /* bf16 matrices and matmul operands, fp32 accumulate,      */
                                 /* fp32 vectors (biases, LayerNorm), fp32 state             */

enum { MGRIT_RELAX_F = 0, MGRIT_RELAX_FCF = 1 };

/* Model shape (paper Table 2 families).  F is the pre-LN block of sec. 3.1:
 * LayerNorm eps = ln_eps with biased variance, exact erf GELU, a bias on every
 * projection, attention scale 1/sqrt(d_model/n_heads). */
typedef struct mgrit_model_desc {
  int32_t arch;
  int32_t d_model, n_heads, d_ff;
  int32_t batch, seq;
  int32_t mem_seq;               /* cross-attention memory length, 0 unless MGRIT_ARCH_CROSS */
  int32_t dtype;
  float   ln_eps;
} mgrit_model_desc;

/* MGRIT knobs (sec. 3.2, Table 3): N fine steps of size h, coarsening factor cf,
 * `levels` grid levels (level l has N/cf^l steps of size cf^l h), `iters`
 * V-cycles (at least 1 unless the run is serial: MGRIT_INVALID_ARG otherwise).  levels == 1 or
 * cf == 1 means plain serial propagation.
 * init_guess: 0 = the initial value copied into every C-point; 1 = the caller has
 * filled rows 1..N of the output array with a guess (row 0 is overwritten). */
typedef struct mgrit_opts {
  int32_t N;
  float   h;
  int32_t cf, levels, iters;
  int32_t relax;
  int32_t init_guess;
} mgrit_opts;

/* ---- packed parameter block of one layer ------------------------------------
 * One contiguous device block per layer.  Tensors, in this order:
 *   vectors (always fp32): ln1_g[d] ln1_b[d] bqkv[3d] bo[d] ln2_g[d] ln2_b[d] b1[f] b2[d]
 *                          (+ arch 2: ln3_g[d] ln3_b[d] bq_c[d] bkv_c[2d] bo_c[d])
 *   matrices (fp32 or bf16 by dtype), each [out_features, in_features] row-major
 *   (y = x W^T + b; reduction dimension contiguous):
 *                          Wqkv[3d,d] Wo[d,d] W1[f,d] W2[d,f]
 *                          (+ arch 2: Wq_c[d,d] Wkv_c[2d,d] Wo_c[d,d])
 * Wqkv rows are Q | K | V, head j owning rows j*d_h..(j+1)*d_h of each third;
 * Wkv_c rows are K | V likewise.  Every tensor starts on a 16-byte boundary; the
 * block itself must be 16-byte aligned.  mgrit_theta_layout() reports offsets. */
enum { MGRIT_P_LN1_G = 0, MGRIT_P_LN1_B, MGRIT_P_BQKV, MGRIT_P_BO, MGRIT_P_LN2_G, MGRIT_P_LN2_B,
       MGRIT_P_B1, MGRIT_P_B2, MGRIT_P_LN3_G, MGRIT_P_LN3_B, MGRIT_P_BQ_C, MGRIT_P_BKV_C,
       MGRIT_P_BO_C,
       MGRIT_P_WQKV, MGRIT_P_WO, MGRIT_P_W1, MGRIT_P_W2, MGRIT_P_WQ_C, MGRIT_P_WKV_C, MGRIT_P_WO_C,
       MGRIT_P_COUNT };

typedef struct mgrit_theta_layout_t {
  int64_t block_bytes;                    /* size of one layer's block                 */
  int64_t offset[MGRIT_P_COUNT];          /* byte offset of each tensor, -1 if absent   */
  int32_t rows[MGRIT_P_COUNT];            /* out_features (or length for vectors)       */
  int32_t cols[MGRIT_P_COUNT];            /* in_features  (1 for vectors)               */
  int32_t elem_bytes[MGRIT_P_COUNT];      /* 4 or 2                                     */
} mgrit_theta_layout_t;

/* Fills *out for the given model.  Host only, no GPU needed. */
int mgrit_theta_layout(const mgrit_model_desc* desc, mgrit_theta_layout_t* out);

/* Workspace sizes in bytes (0 on invalid arguments).  Host only.
 * mgrit_workspace_bytes: adjoint = 0 for mgrit_forward, 1 for mgrit_adjoint, 2 for
 * mgrit_adjoint called with dtheta or dmemory (the gradient pass needs transposed operand
 * copies and per-layer terms). */
size_t mgrit_workspace_bytes(const mgrit_model_desc* desc, const mgrit_opts* opts, int adjoint);
size_t mgrit_layer_step_workspace_bytes(const mgrit_model_desc* desc, int adjoint, int n_groups);

/* Number of layer-step evaluations (Phi or Psi, all levels, each on T tokens) that
 * mgrit_forward / mgrit_adjoint enqueue for these options; -1 on invalid
 * arguments.  The adjoint count excludes its one-off N-layer linearisation pass.
 * Host only. */
int64_t mgrit_step_evaluations(const mgrit_opts* opts);

/* Number of batched sweeps those evaluations are enqueued in: a sweep advances all its
 * intervals at once (one evaluation deep) and needs the sweep before it, so this is the
 * length of the dependent chain of layer steps, to set against the N of serial propagation
 * (sec. 3.2: relaxation sweeps are parallel over the intervals, the coarsest level is a chain
 * of N / cf^(levels-1) steps).  -1 on invalid arguments.  Host only. */
int64_t mgrit_step_depth(const mgrit_opts* opts);

/* MGRIT forward propagation (sec. 3.2.1).
 *   Z0        device, [T,d] fp32: initial value (embedded input)
 *   theta     HOST array of N device pointers, one packed block per layer
 *   memory    device, [batch*mem_seq, d] fp32 encoder output (arch 2), else NULL
 *   Z_all     device, [(N+1),T,d] fp32 out: row n = Z_n after `iters` V-cycles;
 *             row 0 = copy of Z0, row N = the network output.  F-points are
 *             consistent with their C-point (each cycle ends with an F-relaxation).
 *   resnorm   device, [iters] fp32 out or NULL: 2-norm of the level-0 residual at the
 *             C-points after relaxation in each V-cycle (ratio of consecutive entries
 *             = the convergence factor of sec. 3.2.3).  Untouched when the run is serial.
 */
int mgrit_forward(const mgrit_model_desc* desc, const mgrit_opts* opts,
                  const void* Z0, const void* const* theta, const void* memory,
                  void* Z_all, float* resnorm,
                  void* workspace, size_t workspace_bytes, void* stream);

/* MGRIT adjoint propagation (sec. 3.2.2): the same algorithm on the reversed layer
 * index with the transposed, linearised step.
 *   Z_all      device, [(N+1),T,d] fp32: forward states to linearise about (exact or inexact)
 *   lambda_N   device, [T,d] fp32: dL/dZ_N
 *   lambda_all device, [(N+1),T,d] fp32 out: row n = lambda_n; row N = copy of lambda_N,
 *              row 0 = dL/dZ_0
 *   memory     as in mgrit_forward (required for arch 2: the decoder is linearised with it)
 *   dtheta     NULL, or HOST array of N device pointers to gradient blocks (out).  Block n
 *              receives  h * (dF/dtheta_n (Z_n))^T lambda_{n+1}  (sec. 3.1: with the adjoint
 *              states of the Euler network this is dL/dtheta_n; with MGRIT's inexact Z and
 *              lambda, the paper's inexact gradient), computed from the final lambda in one
 *              pass batched over all layers.  A gradient block is laid out like the fp32
 *              parameter block of the same model (mgrit_theta_layout on a copy of desc with
 *              dtype = MGRIT_DTYPE_F32), every entry fp32, whatever desc->dtype is; entries
 *              are overwritten, not accumulated.
 *   dmemory    NULL, or device [batch*mem_seq, d] fp32 out (arch 2 only, MGRIT_INVALID_ARG for
 *              the other block types): dL/dE = sum over layers of h * (dF/dE (Y_n))^T lambda_{n+1},
 *              the gradient with respect to the cross-attention memory (the encoder output),
 *              from the same pass; overwritten.
 *              Either output needs the workspace of mgrit_workspace_bytes(desc, opts, 2).
 */
int mgrit_adjoint(const mgrit_model_desc* desc, const mgrit_opts* opts,
                  const void* Z_all, const void* const* theta, const void* memory,
                  const void* lambda_N, void* lambda_all,
                  void* dmemory, void* const* dtheta, float* resnorm,
                  void* workspace, size_t workspace_bytes, void* stream);

/* The same two solves for a training step, where the adjoint follows the forward solve (sec. 3.2.2:
 * the adjoint is linearised about the forward iterate): the adjoint keeps the internals of every
 * layer's step at Z_n (a linearisation cache of N entries at the start of its workspace), and the
 * level-0 steps of the forward solve's closing F-relaxation (sec. 3.2.1; every step of a serial run)
 * evaluate exactly those internals at the final Z_n, for every layer but the last of each coarse
 * interval.  mgrit_forward_linearising is mgrit_forward whose closing relaxation also leaves them in
 * `adjoint_workspace`; mgrit_adjoint_linearised is mgrit_adjoint that takes them from its workspace
 * and evaluates only the remaining N / cf layers (none in a serial run) before it starts.  Z_all,
 * lambda_all, gradients and residual norms are bit-identical to those of the plain pair.
 *   adjoint_workspace        device, at least mgrit_workspace_bytes(desc, opts, with_gradients ? 2 : 1)
 *   with_gradients           non-zero iff the adjoint call will ask for dtheta or dmemory (the cache
 *                            then also keeps the feed-forward pre-activation)
 * The caller guarantees, between the two calls: the same desc, opts, theta and memory; Z_all of the
 * adjoint is the unmodified output of the forward call; `workspace` of the adjoint is the forward
 * call's `adjoint_workspace`, untouched in between, and with_gradients matches; the adjoint is
 * enqueued after the forward call on the same stream; the linearisation cache is switched on
 * (mgrit_set_adjoint_cache, the default; MGRIT_INVALID_ARG otherwise).  None of this can be checked
 * by the library: a violation gives wrong lambda without an error.  Everything else as above. */
int mgrit_forward_linearising(const mgrit_model_desc* desc, const mgrit_opts* opts,
                              const void* Z0, const void* const* theta, const void* memory,
                              void* Z_all, float* resnorm,
                              void* workspace, size_t workspace_bytes,
                              void* adjoint_workspace, size_t adjoint_workspace_bytes, int with_gradients,
                              void* stream);
int mgrit_adjoint_linearised(const mgrit_model_desc* desc, const mgrit_opts* opts,
                             const void* Z_all, const void* const* theta, const void* memory,
                             const void* lambda_N, void* lambda_all,
                             void* dmemory, void* const* dtheta, float* resnorm,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Buffer layers (Appendix "Buffer layers"): the first n_open and the last n_close layers of the
 * network are propagated serially (exactly) with their own step size h_buffer (the paper uses 1),
 * and only the N = opts->N layers in between by MGRIT with step opts->h (the paper: 1 / N).
 * theta, dtheta: n_open + N + n_close blocks in network order; Z_all, lambda_all:
 * [(n_open + N + n_close + 1), T, d] fp32, row n = state after n layers; resnorm: the MGRIT part's
 * residual norms.  Everything else as in mgrit_forward / mgrit_adjoint; n_open = n_close = 0
 * reduces to them.  Workspace: mgrit_buffered_workspace_bytes (adjoint as in mgrit_workspace_bytes). */
typedef struct {
  int32_t n_open, n_close;
  float   h_buffer;
} mgrit_buffer_opts;
size_t mgrit_buffered_workspace_bytes(const mgrit_model_desc* desc, const mgrit_opts* opts,
                                      const mgrit_buffer_opts* buf, int adjoint);
int mgrit_forward_buffered(const mgrit_model_desc* desc, const mgrit_opts* opts, const mgrit_buffer_opts* buf,
                           const void* Z0, const void* const* theta, const void* memory,
                           void* Z_all, float* resnorm,
                           void* workspace, size_t workspace_bytes, void* stream);
int mgrit_adjoint_buffered(const mgrit_model_desc* desc, const mgrit_opts* opts, const mgrit_buffer_opts* buf,
                           const void* Z_all, const void* const* theta, const void* memory,
                           const void* lambda_N, void* lambda_all,
                           void* dmemory, void* const* dtheta, float* resnorm,
                           void* workspace, size_t workspace_bytes, void* stream);
/* The buffered pair for a training step, as mgrit_forward_linearising / mgrit_adjoint_linearised (same
 * contract between the two calls).  The three segments' adjoint solves then cannot share one workspace:
 * `adjoint_workspace` (the `workspace` of the adjoint call) holds one region per segment,
 * mgrit_buffered_linearised_workspace_bytes in all.  The serial open and close segments are stepped
 * through completely by the forward solve, so their adjoints evaluate no layer internals of their own. */
size_t mgrit_buffered_linearised_workspace_bytes(const mgrit_model_desc* desc, const mgrit_opts* opts,
                                                 const mgrit_buffer_opts* buf, int with_gradients);
int mgrit_forward_buffered_linearising(const mgrit_model_desc* desc, const mgrit_opts* opts,
                                       const mgrit_buffer_opts* buf,
                                       const void* Z0, const void* const* theta, const void* memory,
                                       void* Z_all, float* resnorm,
                                       void* workspace, size_t workspace_bytes,
                                       void* adjoint_workspace, size_t adjoint_workspace_bytes, int with_gradients,
                                       void* stream);
int mgrit_adjoint_buffered_linearised(const mgrit_model_desc* desc, const mgrit_opts* opts,
                                      const mgrit_buffer_opts* buf,
                                      const void* Z_all, const void* const* theta, const void* memory,
                                      const void* lambda_N, void* lambda_all,
                                      void* dmemory, void* const* dtheta, float* resnorm,
                                      void* workspace, size_t workspace_bytes, void* stream);

/* Stacked encoder-decoder system (sec. 3.1, eq. "fp_transformer"): one MGRIT grid over the
 * N = opts->N = N_enc + N_dec layers of an encoder followed by a cross-attention decoder.  The
 * state of a grid point is Z_n = [X_n ; Y_n]: the batch*mem_seq encoder tokens, then the
 * batch*seq decoder tokens, each d_model wide.  For n < n_enc the step is the encoder block on
 * the X rows (Y rows copied); from n_enc on it is the decoder block on the Y rows, whose
 * cross-attention reads the X rows of the same input state (X rows copied).  A coarse step takes
 * the type and the parameters of the fine layer it starts at.  The transposed decoder step also
 * adds the memory cotangent to the X rows of the adjoint state.
 *   desc       the decoder's description: arch must be MGRIT_ARCH_CROSS; the encoder is the
 *              arch-0 block of the same d_model, n_heads, d_ff, batch, dtype with seq = mem_seq
 *   n_enc      1 <= n_enc < opts->N
 *   theta      host array of N device pointers: the first n_enc blocks in the encoder's layout
 *              (mgrit_theta_layout of the encoder description), the others in the decoder's
 *   Z0, lambda_N           device [batch*(mem_seq+seq), d] fp32
 *   Z_all, lambda_all      device [(N+1), batch*(mem_seq+seq), d] fp32, row n = grid point n
 *   dtheta     NULL, or host array of N device pointers to fp32 gradient blocks (layouts of the
 *              fp32 encoder / decoder descriptions), as in mgrit_adjoint
 * Everything else (resnorm, workspace, stream, errors, ownership) as in mgrit_forward /
 * mgrit_adjoint.  Workspace: mgrit_stacked_workspace_bytes (adjoint as in mgrit_workspace_bytes). */
size_t mgrit_stacked_workspace_bytes(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc, int adjoint);
int mgrit_forward_stacked(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc,
                          const void* Z0, const void* const* theta,
                          void* Z_all, float* resnorm,
                          void* workspace, size_t workspace_bytes, void* stream);
int mgrit_adjoint_stacked(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc,
                          const void* Z_all, const void* const* theta,
                          const void* lambda_N, void* lambda_all,
                          void* const* dtheta, float* resnorm,
                          void* workspace, size_t workspace_bytes, void* stream);
/* The stacked pair for a training step, as mgrit_forward_linearising / mgrit_adjoint_linearised (same
 * contract between the two calls): the closing relaxation of the forward solve leaves the internals of
 * the encoder and decoder layers it steps through in the caches of `adjoint_workspace`
 * (mgrit_stacked_workspace_bytes(desc, opts, n_enc, with_gradients ? 2 : 1)). */
int mgrit_forward_stacked_linearising(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc,
                                      const void* Z0, const void* const* theta,
                                      void* Z_all, float* resnorm,
                                      void* workspace, size_t workspace_bytes,
                                      void* adjoint_workspace, size_t adjoint_workspace_bytes, int with_gradients,
                                      void* stream);
int mgrit_adjoint_stacked_linearised(const mgrit_model_desc* desc, const mgrit_opts* opts, int n_enc,
                                     const void* Z_all, const void* const* theta,
                                     const void* lambda_N, void* lambda_all,
                                     void* const* dtheta, float* resnorm,
                                     void* workspace, size_t workspace_bytes, void* stream);

/* One batched layer step over n_groups independent (state, layer) pairs -- the
 * launch that F-/C-relaxation of Algorithm 1 is made of.
 *   adjoint == 0:  out[g] = in[g] + hstep * F(in[g]; theta[g])            (+ rhs[g])
 *   adjoint != 0:  out[g] = in[g] + hstep * (dF/dZ(lin_state[g]; theta[g]))^T in[g]  (+ rhs[g])
 * in, out, theta, lin_state, rhs: HOST arrays of n_groups device pointers
 * ([T,d] fp32 states; packed blocks).  rhs may be NULL (no right-hand side);
 * lin_state is required iff adjoint.  out[g] must not alias any in[], lin_state[] or
 * rhs[] of the same call. */
int layer_step_batched(const mgrit_model_desc* desc, int adjoint, int n_groups,
                             const void* const* in, void* const* out,
                             const void* const* theta, const void* const* lin_state,
                             const void* const* rhs, const void* memory, float hstep,
                             void* workspace, size_t workspace_bytes, void* stream);

/* layer_step_batched for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as layer_step_batched without the workspace: the scratch memory is a fixed array of
 * MGRIT_STATIC_SCRATCH_BYTES inside the library's device code (each GPU the library is loaded on
 * holds its own copy until the process ends).  The call allocates nothing -- no device or host
 * memory, no stream, no event -- and enqueues every launch on `stream` alone (no helper lane).
 *   - Sizes whose scratch need, mgrit_layer_step_static_bytes(), exceeds MGRIT_STATIC_SCRATCH_BYTES are
 *     rejected with MGRIT_WORKSPACE_TOO_SMALL (0 from the query = invalid arguments); nothing is enqueued.
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents (no kernel
 *     reads a scratch location before writing it, so nothing needs clearing).  Calls that overlap in
 *     time on one GPU -- two streams, two host threads -- race on it: serialise them.
 *   - The first call on a device looks up the array's device address (hipGetSymbolAddress, no
 *     allocation); make that call outside stream capture.
 * Results are bit-identical to layer_step_batched run with mgrit_set_lanes(1). */
#define MGRIT_STATIC_SCRATCH_BYTES (256u << 20)
size_t mgrit_layer_step_static_bytes(const mgrit_model_desc* desc, int adjoint, int n_groups);
int layer_step_batched_static(const mgrit_model_desc* desc, int adjoint, int n_groups,
                              const void* const* in, void* const* out,
                              const void* const* theta, const void* const* lin_state,
                              const void* const* rhs, const void* memory, float hstep, void* stream);

/* ---- adaptive control of the inexactness (sec. 3.2.3), host only ---------------------------
 * The convergence factor of MGRIT iteration k is ||r^(k+1)|| / ||r^(k)||, the ratio of consecutive
 * entries of the `resnorm` output above.  Policy of the paper: every `probe_every` batches run one
 * batch with twice the iterations and look at the factor of its final iteration; above `threshold`
 * (1 in the paper) the iteration count is no longer effective, and either the count is raised or
 * training switches to serial propagation.  The caller owns the struct (plain data, may be copied
 * or checkpointed) and drives it around its own calls of mgrit_forward / mgrit_adjoint (one
 * indicator per direction, as in the paper's Fig. 5):
 *     it = mgrit_indicator_begin_batch(&ind);     // iterations for this batch; 0 = run serial
 *     opts.iters = it; opts.levels = it ? L : 1;  mgrit_forward(..., resnorm_dev, ...);
 *     copy resnorm to the host if ind.probing;    mgrit_indicator_end_batch(&ind, resnorm_host, it);
 * Where the paper leaves the policy open: batches are counted from 0 and batch b is a probe when
 * (b + 1) is a multiple of probe_every; MGRIT_MITIGATE_MORE_ITERATIONS doubles `iters` (the count
 * the probe just ran) while that stays <= max_iters and falls back to serial beyond;
 * MGRIT_MITIGATE_SERIAL switches at the first failing probe; serial is final.  A probe whose last
 * residual is not finite fails; one whose residuals are both zero passes. */
enum { MGRIT_MITIGATE_SERIAL = 0, MGRIT_MITIGATE_MORE_ITERATIONS = 1 };
typedef struct {
  int32_t iters;          /* iterations on ordinary batches (doubled on probes)                 */
  int32_t probe_every;    /* probe period in batches, 0 = never probe                           */
  int32_t mitigation;     /* MGRIT_MITIGATE_*                                                   */
  int32_t max_iters;      /* ceiling of `iters` under MGRIT_MITIGATE_MORE_ITERATIONS            */
  float   threshold;      /* failing convergence factor                                         */
  float   last_factor;    /* factor seen by the last probe, -1 before the first                 */
  int64_t batch;          /* batches finished                                                   */
  int32_t serial;         /* 1 once switched to serial propagation                              */
  int32_t probing;        /* 1 between begin_batch and end_batch of a probe batch               */
  int32_t failures;       /* probes that failed so far                                          */
  int32_t reserved;
} mgrit_indicator;
/* Returns MGRIT_OK or MGRIT_INVALID_ARG (iters < 1, negative period or ceiling, threshold <= 0). */
int mgrit_indicator_init(mgrit_indicator* ind, int iters, int probe_every, int mitigation, int max_iters,
                         float threshold);
/* Iterations to run for the coming batch: 2*iters on a probe, iters otherwise, 0 = serial. */
int mgrit_indicator_begin_batch(mgrit_indicator* ind);
/* resnorm: HOST array of the n residual norms of the batch just run (ignored unless it was a
 * probe).  Returns 1 if the policy changed (iters raised or switched to serial), 0 if not,
 * MGRIT_INVALID_ARG on bad arguments. */
int mgrit_indicator_end_batch(mgrit_indicator* ind, const float* resnorm, int n);

const char* mgrit_status_string(int status);
int         mgrit_last_hip_error(void);          /* hipError_t of the last MGRIT_HIP_ERROR */

/* Tuning knob: at most this many groups go into one kernel launch (larger sweeps
 * are split into chunks that run one after another).  0 restores the default, which the library
 * chooses per model and sweep width (3..6 for bf16 models: the count whose projection GEMMs fill
 * their last round of tiles best; 4 for fp32); mgrit_default_groups_per_launch reports it for
 * sweeps of `sweep` groups (opts->N / opts->cf intervals on level 0).  Host only. */
void mgrit_set_max_groups_per_launch(int n);
int  mgrit_default_groups_per_launch(const mgrit_model_desc* desc, int sweep);

/* Tuning knob: 2 (default) lets the independent launch chunks of a sweep alternate between the
 * caller's stream and one helper stream, forked from and joined back into the caller's stream
 * with events before the call's remaining work is enqueued (stream-ordered semantics for the
 * caller are unchanged); with two lanes the serial solve on the coarsest level also overlaps the
 * right-hand sides before it and the F-relaxation after it, handed over chunk by chunk through
 * events (same results, bit for bit); 1 keeps everything on the caller's stream.  The helper
 * stream and its events (34, no timing) are created once per device on first use.  Both knobs
 * change the workspace size: set them before querying it. */
void mgrit_set_lanes(int n);

/* Memory knob of mgrit_adjoint (and of the buffered and stacked forms): 1 (default) keeps the block
 * internals of all N layers at their linearisation states in the workspace -- filled once per call by
 * one forward pass batched over the layers, about 24 d_model bytes per token and layer (5 GB at the
 * BERT shape, 10 GB at the GPT-2 shape) -- so that every transposed step is pure backward work.
 * 0 is for callers who cannot spend that memory: the workspace then holds the internals of one launch
 * chunk per lane only, and every chunk of transposed steps first recomputes those of its own layers
 * (the forward block up to the FFN activation).  Results are identical bit for bit; the workspace
 * shrinks by the cache; an adjoint evaluation costs one partial forward evaluation more.  Process-
 * global like the other knobs, and it changes the workspace size: set it before querying. */
void mgrit_set_adjoint_cache(int on);

/* ---- instrumentation (benchmark and tests; not needed for normal use) ------------------
 * Per-launch timing with HIP events recorded on the launch stream around every kernel of
 * a class.  mgrit_profile_enable(n > 0) creates a pool of n records (this call allocates
 * events; do it outside timed regions) and starts recording; n = 0 stops and frees it.
 * After synchronising the stream, mgrit_profile_read() returns the totals of one class
 * since the last mgrit_profile_reset(): summed kernel time, algorithmic flops and bytes,
 * launches.  Classes: 0 generic GEMM, 1 attention fwd, 2 attention bwd, 3 LayerNorm fwd,
 * 4 LayerNorm VJP (3, 4: launches over several groups; 6, 7: the same over a single group),
 * 5 other elementwise, 8+e MFMA grouped GEMM with epilogue e launched over
 * several groups (relaxation sweeps), 16+e the same over a single group (the serial coarse
 * chain); e: 0 store, 1 bias+GELU, 2 sublayer sum, 3 Euler update, 4 multiply by GELU',
 * 5 fp32 store, 6 GELU' of the cache pass.
 * Returns 0, -1 for a bad class, -3 if the pool overflowed. */
int  mgrit_profile_enable(int max_records);
void mgrit_profile_reset(void);
int  mgrit_profile_read(int cls, double* total_ms, double* flops, double* bytes, int64_t* launches);

/* Measured ceilings of the device, for stating a kernel's rate as a fraction of what the box
 * reaches as well as of the datasheet: a register-resident 32x32x16 bf16 MFMA loop on every
 * compute unit (`scratch`: device, at least 512 KiB, overwritten; `iters` MFMA rounds, 1..2^20;
 * result in TFLOP/s) and a grid-stride copy of `bytes` (a multiple of 16, at least 1 MiB) from
 * `src` to `dst` (device, not overlapping; result = bytes read + written per second, in GB/s, the
 * best of three grid sizes: few resident blocks keep the chip's accesses inside a small window of
 * DRAM pages and reach the higher rate).
 * Both enqueue on `stream`, wait for it and create two events meanwhile; 0 on success, -1 on
 * bad arguments, -4 on a HIP error. */
int mgrit_measure_mfma_ceiling(void* scratch, size_t scratch_bytes, int iters, double* tflops, void* stream);
int mgrit_measure_copy_ceiling(const void* src, void* dst, size_t bytes, double* gbs, void* stream);
/* What the per-launch timing above adds to a launch: the median time, in microseconds, between two
 * events recorded around a kernel that does nothing (64 launches on `stream`, then a wait for it).
 * Subtracting it from a bracketed launch gives its duration as a kernel trace shows it, to within a
 * microsecond; it matters for launches of 10-30 us.  0 on success, -1 / -4 as above. */
int mgrit_measure_event_bracket(double* us, void* stream);

/* Test hook: route GEMMs (first flag) / attention (second flag) to the generic kernels. */
void mgrit_debug_force_simple_kernels(int gemm, int attn);

/* Tuning hook: tile configuration of the MFMA grouped GEMM (0 = chosen by shape, the default;
 * 1 = 256x256x64 and 3 = 256x192x64, one block per CU; 4 = 128x128x64 and 2 = 256x128x32, two
 * blocks per CU).  A configuration that does not fit a shape falls back to configuration 2. */
void mgrit_debug_gemm_tile_config(int cfg);

/* Tuning hook: which attention kernels use 256-row blocks.  Bits 0-2: forward, dQ pass, dK/dV
 * pass at d_head = 128 (sequences of more than 128 tokens; the backward passes only when the
 * last block is more than half full); bits 4-6: the same at d_head = 64 (512 tokens or more;
 * measured slower, off by default).  Default 7; 0 keeps 128-row blocks everywhere. */
void mgrit_debug_attention_wide_blocks(int mask);

/* Tuning hook: 1 (default) overlaps the serial solve on the coarsest level with the F-relaxation
 * that follows it (needs the two lanes); 0 runs them one after the other.  Results are identical. */
void mgrit_debug_pipeline_coarse_solve(int on);

/* Tuning hook: intervals per hand-over of the overlapped coarse solve (0 = the launch chunk, the
 * default; values above the launch chunk are ignored). */
void mgrit_debug_pipeline_chunk(int n);

#ifdef __cplusplus
}
#endif
#endif /* MGRIT_H */
