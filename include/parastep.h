/*
 * parastep.h -- C ABI of the MI355X (gfx950) hot path of reuse-then-predict
 * diffusion denoising.
 *
 * The paper states the problem as  eps_t = eps_theta(x_t, t, c);
 * x_{t-1} = Scheduler(x_t, t, eps_t)  (Preliminaries, "Denoising computation"),
 * measures similarity with the relative MAE of Eq. (1), and wraps the loop in the
 * round-based reuse-then-predict procedure of Appendix A, Algorithm 1 (batched on one
 * device in Section 3.3).  Each entry point below is one of those operations.
 *
 * Conventions for every function:
 *  - returns PS_OK (0) or a negative ps_status; never throws, exits or prints;
 *  - arguments are validated on the host before any launch, so a failing call has
 *    no side effects on device memory;
 *  - "DEVICE" pointers are HIP device memory owned by the caller (e.g. PyTorch
 *    tensors); the library never allocates, frees or keeps device memory.  "HOST"
 *    pointers are ordinary host memory read during the call only;
 *  - work is enqueued on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *    default stream) and the call returns without synchronising; outputs, including
 *    device-side sums, are valid once the caller has synchronised that stream;
 *  - results are deterministic: no floating-point atomics, fixed reduction order;
 *  - a sample's result does not depend on the batch it is computed in: every sample of a
 *    batch is tiled and summed exactly as if it were alone (Section 3.3: the batched step
 *    must reproduce the per-step process), so dit_forward on B samples equals B calls bit
 *    for bit;
 *  - the library keeps no process-wide mutable state: kernels are selected per call from
 *    the shapes and from the kernel path of the handle (dit_set_kernel_path) or of the
 *    call (attn3d, dit_linear);
 *  - calls on one `dit` handle must not overlap; distinct handles/streams may.
 *
 * Shape limits (anything beyond them is PS_ERR_SHAPE at dit_create, never a slow or wrong
 * path): layers <= 64, hidden <= 2048 and a multiple of 8, head_dim in {16, 32, 64},
 * mlp_ratio <= 8, batch <= 16, in_channels*patch^2 <= 1024, at most 2^24 tokens per sample
 * and, for bf16, tokens * hidden * max(mlp_ratio, 3) < 2^31.  The MFMA kernels serve bf16
 * with K % 64 == 0 and at least 64 outputs (projections) and head_dim 64 (attention);
 * every other accepted shape runs on generic fp32-FMA kernels.
 */
#ifndef PARASTEP_H
#define PARASTEP_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__)
#define PS_API __attribute__((visibility("default")))
#else
#define PS_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    PS_OK = 0,
    PS_ERR_NULL = -1,       /* a required pointer is NULL */
    PS_ERR_SHAPE = -2,      /* inconsistent or unsupported sizes */
    PS_ERR_DTYPE = -3,      /* unknown ps_dtype */
    PS_ERR_WORKSPACE = -4,  /* workspace missing, misaligned (256 B) or too small */
    PS_ERR_SCHEDULE = -5,   /* invalid sampling schedule */
    PS_ERR_HIP = -6         /* a HIP runtime call or launch failed */
} ps_status;

/* Storage / operand type of matrices and activations fed to contractions.
 * Accumulators, LayerNorm statistics, softmax statistics, the residual stream,
 * modulation vectors, biases, latents and eps are always fp32. */
typedef enum { PS_F32 = 0, PS_BF16 = 1 } ps_dtype;

/* Static message for a status code. */
PS_API const char* ps_strerror(int status);

/* ------------------------------------------------------------------ noise predictor
 * eps_theta is a DiT with full 3D attention (Section 1: cost quadratic in spatial and
 * temporal length).  Tokens are the text tokens followed by one token per
 * (frame, patch row, patch col) of the latent, patch vector ordered (c, dy, dx).
 * Requirements: hidden == heads*head_dim, head_dim % 16 == 0 (3D RoPE splits it
 * d/4, 3d/8, 3d/8 into interleaved pairs), height and width divisible by patch,
 * hidden even, text_tokens >= 0, layers <= 64. */
typedef struct {
    int layers, hidden, heads, head_dim, mlp_ratio;
    int in_channels, patch, frames, height, width;   /* latent [C, F, H, W] */
    int text_tokens, time_embed_dim;
    int dtype;                                        /* ps_dtype */
    float ln_eps, rope_theta;
} dit_config;

typedef struct dit dit;   /* opaque host object */

/* Number of weight tensors dit_create expects for `layers` layers: 6 + 10*layers + 4. */
PS_API int dit_num_weights(int layers);

/* Create a predictor.  `weights` is a HOST array of n_weights DEVICE pointers in the
 * order  W_pe b_pe W_t1 b_t1 W_t2 b_t2, then per layer  W_mod b_mod W_qkv b_qkv W_o
 * b_o W_1 b_1 W_2 b_2,  then  W_fm b_fm W_out b_out.  Matrices are row-major
 * [out_features, in_features] in cfg->dtype; biases are fp32.  The tensors are
 * borrowed: the caller keeps them alive and unchanged while the handle exists.
 * The handle owns only host memory and a few HIP events. */
PS_API int dit_create(const dit_config* cfg, const void* const* weights, int n_weights, dit** out);
PS_API int dit_destroy(dit* d);

/* Kernel path of a handle (0 after dit_create), used by every later call on it.  Low byte = mode:
 * 0 the fastest kernel for each shape, 1 the generic fp32-FMA kernels, 2 bf16 attention without
 * the key split of its last partial round of workgroups, 3 bf16 head-dim-64 attention always
 * through the kernel that tracks a softmax reference (the one without is not tried first),
 * 4 projections whose last partial round of workgroups is not divided along k.  Bits 8-11: tile variant of the bf16
 * MFMA projections (0 automatic, 1: 256x256, 2: 128x128, 3: 192x256, 4: 192x128); the variant
 * decides which workgroup computes an output and, for k >= 4096, which outputs of the last partial
 * round are summed in k pieces (a different rounding of those); nothing else.  Other values:
 * PS_ERR_SHAPE.
 * dit_workspace_bytes does not depend on the path. */
PS_API int dit_set_kernel_path(dit* d, int path);
PS_API int dit_get_kernel_path(const dit* d);    /* the handle's path, PS_ERR_NULL for NULL */

/* Bytes of DEVICE workspace dit_forward needs for `batch` samples (0 on bad input). */
PS_API size_t dit_workspace_bytes(const dit* d, int batch);

/* eps_out[b] = eps_theta(x[b], t_host[b], ctx[b]) for b < batch.
 *   x        DEVICE fp32 [B, C, F, H, W]
 *   ctx      DEVICE cfg.dtype [B, text_tokens, hidden]; may be NULL iff text_tokens == 0
 *   t_host   HOST int32 [B], per-sample timestep (0 <= t < 100000)
 *   eps_out  DEVICE fp32 [B, C, F, H, W]; must not alias x
 *   workspace DEVICE, 256-byte aligned, >= dit_workspace_bytes(d, batch); scratch only */
PS_API int dit_forward(dit* d, const float* x, const void* ctx, const int32_t* t_host, float* eps_out,
                int batch, void* workspace, size_t workspace_bytes, void* hip_stream);

/* Optional per-kernel-class timing of dit_forward with HIP events on its stream.
 * Classes: 0 attention, 1 qkv GEMM, 2 out-proj GEMM, 3 fc1 GEMM, 4 fc2 GEMM,
 * 5 LayerNorm+modulate, 6 everything else.  dit_profile_read synchronises the
 * recorded events and returns accumulated milliseconds and launch counts since the
 * last dit_profile_enable(d, on > 0); both arrays are HOST [7].
 * on: 0 off, 1 every class (two events per launch: about 1.5 % of a 30-layer forward at
 * 17776 tokens), 2 the attention class only (0.3 %); other values: PS_ERR_SHAPE. */
PS_API int dit_profile_enable(dit* d, int on);
PS_API int dit_profile_read(dit* d, double* ms_out, int64_t* launches_out);

/* Measurement aid: one launch of nothing but bf16 matrix instructions (v_mfma_f32_16x16x32_bf16 on
 * register operands, two waves per SIMD on every compute unit, `iters` x 8 instructions per wave).
 * Timed by the caller, *flops_out (HOST) / time is the rate the matrix pipes sustain on this chip
 * under load -- the practical ceiling next to the nominal peak.  sink: DEVICE float[1], never
 * written in practice.  1 <= iters <= 2^24. */
PS_API int ps_mfma_probe(int iters, float* sink, double* flops_out, void* hip_stream);

/* Stand-alone full attention: for every batch and head, O = softmax(scale*Q K^T) V
 * over all `seq` tokens (no mask, Section 1's "3D attention": one token axis holding
 * text tokens and the flattened frame/row/col grid).  q, k, v, o: DEVICE
 * [B, seq, heads, head_dim] contiguous in `dtype`, 16-byte aligned; o must not alias
 * the inputs.  seq >= 1, scale > 0, head_dim in {16, 32, 64}; rows past the end are never
 * read, but V must be finite (masked keys multiply V by an exact 0).
 * workspace: DEVICE, 256-byte aligned, >= attn3d_workspace_bytes(...) (may be NULL when
 * that is 0); scratch only.  It is non-zero for bf16 with head_dim 64: the kernel that needs no
 * running maximum checks its own sums and marks, per (batch, head), what it could not do there
 * (a second kernel that tracks a softmax reference recomputes those heads), and the workgroups
 * that split their keys in the last, partial round leave their partial sums there (merged by
 * that second launch).
 * kernel_path: as for dit_set_kernel_path (0 = default); the workspace size does not depend on it. */
PS_API size_t attn3d_workspace_bytes(int batch, int seq, int heads, int head_dim, int dtype);
PS_API int attn3d(const void* q, const void* k, const void* v, void* o,
           int batch, int seq, int heads, int head_dim, float scale, int dtype, int kernel_path,
           void* workspace, size_t workspace_bytes, void* hip_stream);

/* The projection every DiT sub-layer uses, exposed for per-kernel parity and timing:
 * out[M, n_out] = act(a[M, k] * w[n_out, k]^T + bias), act 0 = none, 1 = tanh-GELU.
 * a, w, out DEVICE in `dtype`, row-major, 16-byte aligned; bias DEVICE fp32 [n_out],
 * 16-byte aligned.  n_out even, k % 8 == 0; bf16 shapes of the MFMA kernel (k % 64 == 0,
 * n_out % 4 == 0, n_out >= 64) need m * n_out < 2^31.
 * workspace: DEVICE scratch, 256-byte aligned, or NULL.  With at least
 * dit_linear_workspace_bytes(...) of it, shapes whose output tiles do not fill the last round
 * of workgroups split those tiles along k (fp32 partial sums pass through the workspace and
 * are added in a fixed order); with NULL or less the call computes the same product unsplit.
 * The two differ only in summation order.
 * kernel_path: as for dit_set_kernel_path (0 = default); it enters the workspace size. */
PS_API size_t dit_linear_workspace_bytes(int m, int n_out, int k, int dtype, int kernel_path);
PS_API int dit_linear(const void* a, const void* w, const float* bias, void* out, int m, int n_out, int k,
               int act, int dtype, int kernel_path, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------- scheduler and metric
 * Fused DDIM update  x_out = a*x + b*eps  (the element-wise Scheduler of the paper's
 * Section 3) and, if sums4 != NULL, the four sums behind the adjacent-step relative
 * MAEs of Eq. (1):  sums4 = { sum|x_out-x|, sum|x_out|, sum|eps-eps_prev|, sum|eps| }
 * (the last two use eps_prev; with eps_prev == NULL they are 0 and sum|eps|).
 * The coefficients are doubles because a -> 1 towards the end of a run: the kernel works
 * in fp32 on the increment  d = (a-1)*x + b*eps,  x_out = x + d,  sum|x_out-x| = sum|d|,
 * with (a-1) rounded to fp32 only after the subtraction.
 * x_out may alias x.  workspace: DEVICE, >= sampler_step_workspace_bytes(n), only
 * needed when sums4 != NULL.  n may be 0: x, eps and x_out are then not looked at (NULL
 * is accepted) and the sums are zero. */
PS_API size_t sampler_step_workspace_bytes(size_t n);
PS_API int sampler_step(const float* x, const float* eps, const float* eps_prev, float* x_out,
                 double a, double b, size_t n, float* sums4,
                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* sampler_step for callers that cannot allocate device memory or carry a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels
 * and results as sampler_step (bit for bit), but the partial sums of the reduction live in a
 * file-scope device array of the library (1 MiB on every GPU the library runs on, held until the
 * process ends) instead of a workspace; the call allocates and frees nothing.
 * n <= SAMPLER_STEP_NOALLOC_MAX_N, larger sizes are PS_ERR_SHAPE.  The device current at the call
 * must be the one `hip_stream` belongs to (the array's address is looked up per device, on first
 * use with sums4 != NULL: a caller that captures its stream into a graph makes one such call on the
 * device beforehand).  Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams,
 * two threads) race on it; calls in order on one stream do not. */
#define SAMPLER_STEP_NOALLOC_MAX_N ((size_t)1 << 31)
PS_API int sampler_step_noalloc(const float* x, const float* eps, const float* eps_prev, float* x_out,
                         double a, double b, size_t n, float* sums4, void* hip_stream);

/* Relative MAE of Eq. (1): out3 = { sum|a-b|, sum|a|, sum|a-b| / sum|a| } (DEVICE fp32).
 * The denominator is the FIRST argument; a zero denominator yields inf or nan.
 * n may be 0 (a and b are then not looked at, NULL is accepted): { 0, 0, nan }. */
PS_API size_t rel_mae_workspace_bytes(size_t n);
PS_API int rel_mae(const float* a, const float* b, size_t n, float* out3,
            void* workspace, size_t workspace_bytes, void* hip_stream);

/* Host-only: DDIM grid and coefficients for a linear beta schedule, computed in
 * double.  tau_i = (steps-1-i)*floor(train_steps/steps); a_i = sqrt(abar_prev/abar_tau),
 * b_i = sqrt(1-abar_prev) - a_i*sqrt(1-abar_tau), abar_prev = 1 after the last step.
 * Outputs are HOST arrays of length `steps`. */
PS_API int ddim_coefficients(int train_steps, double beta_start, double beta_end, int steps,
                      int32_t* timesteps_out, double* a_out, double* b_out);

/* Host-only tables of two other deterministic schedulers the paper runs its method under; both
 * are x' = a*x + b*eps for the same fused kernel and the same loop.
 * euler_discrete_coefficients: the Euler step in sigma space (the scheduler Section 4.2 names
 * for SVD), for samples held as x = x0 + sigma*eps: on the DDIM grid tau_i, with
 * sigma_t = sqrt((1 - abar_t) / abar_t) and sigma = 0 after the last step,
 * a_i = 1, b_i = sigma_next - sigma_tau_i.
 * flow_euler_coefficients: Flow Matching's discretised ODE (Preliminaries, "Flow Matching"),
 * z_{t+dt} = z_t + dt*v(z_t, t), t from 0 (reference sample) to 1 on a uniform grid:
 * a_i = 1, b_i = 1/steps; the predictor is given the time index floor(i*train_steps/steps),
 * which ascends.  Outputs are HOST arrays of length `steps`. */
PS_API int euler_discrete_coefficients(int train_steps, double beta_start, double beta_end, int steps,
                                int32_t* timesteps_out, double* a_out, double* b_out);
PS_API int flow_euler_coefficients(int train_steps, int steps, int32_t* timesteps_out, double* a_out,
                            double* b_out);

/* ------------------------------------------------------------- reuse-then-predict run
 * Algorithm 1 with all ranks of a cycle simulated on one device.
 *   warmup     first `warmup` steps run the original process; must be >= 1 unless
 *              every cycle has length 1
 *   cycle_len  HOST [n_cycles] cycle length (= parallel degree p) of each cycle after
 *              warm-up; they must cover steps - warmup; the last may be cut short
 *   batched    0: one predictor call per step (rank == round evaluates);
 *              1: one call per cycle with batch = cycle length (Section 3.3)
 *   mode       0 reuse-then-predict (Algorithm 1: a rank reuses the eps it predicted itself),
 *              1 direct reuse (predict only in round 0; not with batched),
 *              2 reuse-then-predict in which every rank's cache is refreshed, at the end of
 *                each cycle, with the eps rank 0 applied in the cycle's last step (what a
 *                single device, or ranks that also exchange eps, can do; equals mode 0 when
 *                every cycle has length <= 2) */
typedef struct {
    int steps;
    const int32_t* timesteps;   /* HOST [steps], strictly monotonic (descending for diffusion grids) */
    const double* coef_a;       /* HOST [steps] */
    const double* coef_b;       /* HOST [steps] */
    int warmup;
    int n_cycles;
    const int32_t* cycle_len;
    int batched;
    int mode;
} sampler_schedule;

PS_API size_t sampler_workspace_bytes(const dit* d, const sampler_schedule* s);

/* x_T, x0_out: DEVICE fp32 [C,F,H,W] (one sample; may alias each other).
 * ctx as in dit_forward with B = 1 (it is shared by all ranks).
 * step_sums: DEVICE fp32 [steps][4] or NULL; row i holds sampler_step's sums4 for the
 * update rank 0 takes at step i (row 0's eps_prev terms are 0, sum|eps|).
 * trajectory_out: DEVICE fp32 [steps][C,F,H,W] or NULL; slice i receives the sample after
 * step i (rank 0's, i.e. the one the run returns at the end), so that two runs can be
 * compared step by step with rel_mae (the deviation curves of Section 3.1's comparison of
 * direct reuse with reuse-then-predict).  It must not overlap x_T or x0_out.
 * calls_out: HOST, optional; receives the number of predictor launches. */
PS_API int sampler_run(dit* d, const sampler_schedule* s, const float* x_T, const void* ctx,
                float* x0_out, float* step_sums, float* trajectory_out, int* calls_out,
                void* workspace, size_t workspace_bytes, void* hip_stream);

/* ------------------------------------------------------------- a run in pieces (split / resume)
 * What Algorithm 1 carries from one step to the next is the step count, the round within the
 * cycle, and per rank its sample and its eps_cache (plus, for the adjacent-step sums, the eps of
 * the last step).  sampler_run_steps advances a run from state->step to stop_step and leaves that
 * state behind: the position in `state` (HOST, plain data) and the tensors in the first
 * sampler_state_bytes(d, s) bytes of the workspace.  A run taken in pieces -- in one process with
 * the workspace left alone in between, or in another process from a stored copy of the struct and
 * of those bytes put at the head of a workspace of the same size, with the same schedule and
 * weights -- is bit-identical to sampler_run's.
 *   state      in/out.  step == 0 starts a run (the other fields are ignored and x_T is read);
 *              otherwise it must be what an earlier call with this schedule left: a state whose
 *              cycle, round or slots do not fit the schedule is PS_ERR_SCHEDULE
 *   stop_step  state->step < stop_step <= steps.  With batched == 1 a cycle is one predictor call,
 *              so a run can only pause inside warm-up or between cycles (else PS_ERR_SCHEDULE)
 *   x_T        needed iff state->step == 0;  x_out (optional) receives rank 0's sample after
 *              stop_step steps;  step_sums / trajectory_out as in sampler_run, rows
 *              state->step .. stop_step-1 are written. */
typedef struct {
    int32_t step;       /* steps taken so far */
    int32_t cycle;      /* cycle (after warm-up) and round within it at which the next step runs */
    int32_t round;
    int32_t toggle;     /* which of the two eps buffers rank 0's next prediction goes to */
    int32_t eps_prev;   /* where the last step's eps lives: -1 nowhere yet, 0 / 1 eps buffer, 2 + r rank r's cache */
    int32_t calls;      /* predictor launches so far */
    int32_t src[16];    /* rank r's current sample is in sample slot src[r] (0 after a broadcast, else r) */
} sampler_state;
PS_API size_t sampler_state_bytes(const dit* d, const sampler_schedule* s);
PS_API int sampler_run_steps(dit* d, const sampler_schedule* s, sampler_state* state, int stop_step,
                      const float* x_T, const void* ctx, float* x_out, float* step_sums,
                      float* trajectory_out, void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PARASTEP_H */
