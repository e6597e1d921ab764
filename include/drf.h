/*
 * drf.h -- C ABI of libdrf: DRiffusion draft-and-refine sampling on one MI355X.
 *
 * The paper states the problem as: given sampled noise x_T, a number of sampling
 * steps T and a block size k, produce x_0 (Algorithm 1 / Algorithm 2, "Require /
 * Ensure").  Its three building blocks are the calls below:
 *   - the noise predictor eps_theta(x, t), evaluated on k drafts at once
 *     (Algorithm 1, the "concurrently" loop): drf_eps_batched;
 *   - the skip transition x_{t-k} = Skip(x_t, eps_t) (Eq. ddim_skip_reverse, with or
 *     without variance; Eq. ddpm_skip_reverse; the Euler skip of the ODE solvers):
 *     drf_skip_transition, drf_skip_transition_noise;
 *   - the standard denoising update that refines the drafts (Algorithm 1, second
 *     loop): drf_refine_step;
 * and drf_sample / drf_sample_noise run the whole draft-and-refine loop in either mode.
 * On one GPU the paper's k devices are k groups of batch slots of one forward pass.
 *
 * Conventions
 *   - Every pointer is marked HOST or DEVICE.  Device buffers belong to the caller;
 *     the library never frees or reallocates them.  All work is enqueued on the
 *     given HIP stream (a hipStream_t passed as void*; NULL = the default stream)
 *     and is asynchronous unless stated otherwise.
 *   - Every call returns a drf_status; nothing throws or aborts across the ABI.
 *     drf_last_error() gives a thread-local message for the last failure.
 *     Asynchronous HIP faults surface at the caller's next synchronisation.
 *   - One denoiser handle may be used by one stream at a time, and only one handle per
 *     process may have work in flight: a call on a handle while another handle's last call is
 *     still running on a different stream returns DRF_EUNSUPPORTED (the kernels are sized for
 *     sole occupancy of the GPU and the handles' work would interleave).  Handles used one
 *     after the other on the same stream, or after a synchronisation, are fine.
 *
 * Indices.  Sampling indices s run S, S-1, ..., 1, 0 (the paper's t, with S the
 * paper's T).  DDIM / DDPM: the network is fed the training timestep tau_s = (s-1) *
 * floor(train_steps / S) for s >= 1.  alpha-bar_s is the cumulative product of
 * (1 - beta) up to tau_s with linear betas; alpha-bar_0 = 1 (clean data).
 * Euler: the ODE time of index s is sigma_s = shift u / (1 + (shift - 1) u), u = s/S
 * (sigma_0 = 0 data, sigma_S = 1 noise), the network is a velocity predictor and is fed
 * the integer time floor(sigma_s train_steps + 1/2).
 * The block size k of the paper is `n` here.
 *
 * The noise predictor is a latent DiT whose internals the paper does not fix;
 * they are defined at drf_dit_config below.
 */
#ifndef DRF_H
#define DRF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct drf_denoiser drf_denoiser;

typedef enum {
    DRF_OK = 0,
    DRF_EINVAL = -1,        /* NULL pointer, count or index out of range */
    DRF_ESHAPE = -2,        /* configuration the kernels cannot take (divisibility) */
    DRF_ENOMEM = -3,        /* device or host allocation failed */
    DRF_EHIP = -4,          /* a HIP runtime call failed */
    DRF_EUNSUPPORTED = -5   /* valid in the paper, not built here */
} drf_status;

typedef enum { DRF_CONSERVATIVE = 0, DRF_AGGRESSIVE = 1 } drf_mode;
typedef enum { DRF_F32 = 0, DRF_BF16 = 1 } drf_dtype;
typedef enum { DRF_COND_VECTOR = 0, DRF_COND_CLASS = 1, DRF_COND_TEXT = 2 } drf_cond_kind;
/*
 * Which skip transition the sampler uses (section "Skip Transitions"):
 *   DRF_DDIM   Eq. ddim_skip_reverse with sigma_{t,k} = eta * (posterior std of the same jump);
 *   DRF_DDPM   Eq. ddpm_skip_reverse: a draw from the Bayes posterior q(x_{t-k} | x_t, x_0_hat)
 *              (mean mu', variance sigma_{t,k}^2 of Eq. ddpm_skip_reverse_detail); eta is ignored;
 *   DRF_EULER  x_{t-k} = x_t + (sigma_{t-k} - sigma_t) v(x_t, sigma_t), the network output read as
 *              the velocity v; no variance; beta_* and eta are ignored.
 */
typedef enum { DRF_DDIM = 0, DRF_DDPM = 1, DRF_EULER = 2 } drf_sampler;

/*
 * The DiT (this build's definition; D = hidden, P = in_ch*patch^2, R = mlp_ratio,
 * T = (lat_h/patch)*(lat_w/patch) tokens, d = D/heads):
 *   token (py,px) = x[ch][py*patch+dy][px*patch+dx] at position ch*patch^2 + dy*patch + dx
 *   h   = Linear(P->D)(token) + pos, pos = fixed 2-D sin-cos code: columns [0,D/2) from
 *         the grid row, [D/2,D) from the grid column, each half [sin | cos] over D/4
 *         frequencies 10000^(-i/(D/4))
 *   c   = Linear(D->D)(SiLU(Linear(256->D)(femb(tau)))) + cond_emb,
 *         femb = [cos(tau f_i) | sin(tau f_i)], f_i = 10000^(-i/128), i < 128;
 *         cond_emb = Linear(cond_dim->D)(vector) | table[class] (row cond_dim = null class)
 *         | 0 for text
 *   per block: (shift1, scale1, gate1, shift2, scale2, gate2) = Linear(D->6D)(SiLU(c))
 *     h += gate1 * Proj(SelfAttn(LN(h)(1+scale1)+shift1))      softmax(q k^T / sqrt(d)) v, no mask
 *     text only: h += XProj(CrossAttn(q = Linear(LN(h)), k|v = Linear(cond_dim->2D)(context)))
 *     h += gate2 * Fc2(GELU_tanh(Fc1(LN(h)(1+scale2)+shift2)))
 *   (shift, scale) = Linear(D->2D)(SiLU(c)); eps tokens = Linear(D->P)(LN(h)(1+scale)+shift),
 *   scattered back to [in_ch][lat_h][lat_w].  LN has no affine, eps 1e-6.
 * dtype DRF_BF16: every parameter is rounded to bf16 (round-to-nearest-even) once at
 * create; GEMM and attention operands are bf16 with fp32 accumulation; the gated branch
 * outputs (attention projection, MLP) are rounded to bf16 before they are added to the
 * residual stream; LayerNorm and softmax statistics, the residual stream itself, latents
 * and all sampler updates are fp32.
 * dtype DRF_F32: everything in fp32.
 * Requirements: hidden % heads == 0, hidden % 4 == 0, lat_h, lat_w % patch == 0;
 * DRF_BF16 also needs hidden % 64 == 0, d % 8 == 0, d <= 96, cond_dim % 64 == 0 for text.
 */
typedef struct {
    int depth, hidden, heads, mlp_ratio, patch, in_ch, lat_h, lat_w;
    drf_dtype dtype;
    drf_cond_kind cond;
    int cond_dim;   /* vector width | number of classes | context width */
    int ctx_len;    /* text: context tokens; else 0 */
} drf_dit_config;

typedef struct {
    int train_steps;            /* training timesteps of the beta schedule (1000) */
    double beta_start, beta_end;/* linear betas */
    int steps;                  /* S, 1 <= S <= train_steps */
    double eta;                 /* DRF_DDIM: 0 <= eta <= 1; 0 = deterministic, 1 = DDPM-induced variance */
    drf_sampler sampler;
    double shift;               /* DRF_EULER: time shift of the sigma grid, > 0 (1 = uniform) */
} drf_sched_config;

/*
 * Where the fresh standard-normal fields of a stochastic sampler come from (the draws
 * "sample z" of Algorithm 1 / 2).  A field is one fp32 array [batch][elems_per_sample].
 *   z != NULL: DEVICE fp32 [count][batch][elems_per_sample], explicit fields; the k-th field
 *              a call consumes is z[k]; seed and field0 are ignored.
 *   z == NULL: the k-th field is field number field0 + k of the library's counter-based
 *              stream for `seed` (see drf_normal_fill), generated inside the update kernel
 *              and never stored.
 */
typedef struct {
    const float* z;
    uint64_t seed;
    uint32_t field0;
} drf_noise;

/*
 * Number of fp32 scalars in the flat parameter array.  Linear weights are [out][in]:
 *   patch_w [D][P], patch_b [D], t_w1 [D][256], t_b1 [D], t_w2 [D][D], t_b2 [D],
 *   vector: c_w [D][cond_dim], c_b [D] | class: table [cond_dim+1][D] | text: nothing,
 *   per block: ada_w [6D][D], ada_b [6D], qkv_w [3D][D], qkv_b [3D], proj_w [D][D], proj_b [D],
 *     text only: xq_w [D][D], xq_b [D], xkv_w [2D][cond_dim], xkv_b [2D], xo_w [D][D], xo_b [D],
 *     fc1_w [RD][D], fc1_b [RD], fc2_w [D][RD], fc2_b [D],
 *   fin_ada_w [2D][D], fin_ada_b [2D], fin_w [P][D], fin_b [P].
 * Returns 0 for an invalid configuration.
 */
size_t drf_denoiser_weight_count(const drf_dit_config* cfg);

/*
 * Build a denoiser: validates cfg, copies (and for DRF_BF16 rounds) the parameters
 * to the GPU.  host_weights: HOST, `count` fp32 values in the order above, only read
 * during the call.  Synchronous.  *out owns its device memory until destroyed.
 */
drf_status drf_denoiser_create(const drf_dit_config* cfg, const float* host_weights, size_t count,
                               void* hip_stream, drf_denoiser** out);
void drf_denoiser_destroy(drf_denoiser* den);

/*
 * Pre-size the handle's activation workspace for `max_slots` samples per pass
 * (synchronous).  drf_eps_batched and drf_sample grow it on demand otherwise, which
 * costs a device allocation and a stream synchronisation at that call.
 */
drf_status drf_denoiser_reserve(drf_denoiser* den, int max_slots);

/*
 * How drf_sample / drf_sample_noise enqueue their launch sequence (the loop of Algorithm 1 / 2 is a fixed
 * sequence of kernel launches once the arguments are known):
 *   mode 1 (default): the first call with a given set of arguments (schedule, mode, n, batch, the
 *           buffers' addresses, guidance scale, noise source) launches kernel by kernel; the second
 *           captures the sequence into a HIP graph, and that and every later call with the same
 *           arguments replay it with one graph launch (up to 8 argument sets are kept per handle);
 *   mode 2: capture at the first call already;
 *   mode 0: always kernel by kernel; drops the captured graphs.
 * Results are the same bits in every mode.  Calls made while the caller's stream is itself being
 * captured, or while profiling is enabled, always launch kernel by kernel.
 */
drf_status drf_denoiser_use_graphs(drf_denoiser* den, int mode);

/*
 * eps_theta for `slots` samples in ONE pass, each with its own timestep: the batched
 * draft evaluation of Algorithm 1 / Algorithm 2 (the loop marked "concurrently").
 *   x        DEVICE fp32 [slots][in_ch][lat_h][lat_w]
 *   t        DEVICE int32 [slots]   training timesteps tau (not sampling indices), >= 0
 *   cond     DEVICE: vector fp32 [slots][cond_dim] | class int32 [slots] in [0, cond_dim]
 *                    | text fp32 [slots][ctx_len][cond_dim]
 *   eps_out  DEVICE fp32 [slots][in_ch][lat_h][lat_w]
 * slots == 0 is a no-op.  Out-of-range class ids are clamped to the null class.
 */
drf_status drf_eps_batched(drf_denoiser* den, const float* x, const int32_t* t, const void* cond,
                           int slots, float* eps_out, void* hip_stream);

/*
 * drf_eps_batched for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and the same results as drf_eps_batched, but the pass's scratch buffers
 * (activations, conditioning rows, modulation table, K/V of a text context, and for bf16
 * handles the 16 MiB of partial tiles of the split-K GEMM) are carved out
 * of a static device array of DRF_STATIC_SCRATCH_BYTES that the library holds on every GPU
 * it runs on until the process ends, instead of the handle's workspace; the call makes no
 * device allocation and frees nothing.  A pass that needs more scratch than the array holds
 * returns DRF_ESHAPE before any work is enqueued; DRF_EUNSUPPORTED while per-launch profiling
 * is enabled on the handle.
 * The array is shared by every handle and call on that GPU and keeps the last call's
 * contents (nothing in it has to start at zero): calls that overlap on one GPU race.
 */
#define DRF_STATIC_SCRATCH_BYTES (48u << 20)
drf_status drf_eps_batched_static(drf_denoiser* den, const float* x, const int32_t* t, const void* cond,
                                  int slots, float* eps_out, void* hip_stream);

/*
 * Skip transitions without a noise term.  DRF_DDIM with eta = 0 (Eq. ddim_skip_reverse,
 * zero variance; the draft line of Algorithm 1): for j < m,
 *   x_to[j] = sqrt(ab_to/ab_from) x_from + (sqrt(1-ab_to) - sqrt(ab_to/ab_from) sqrt(1-ab_from)) eps_from
 * with ab_* the cumulative alpha at sampling indices s_from and s_to[j]; algebraically
 * the paper's predicted-x_0 form.  Coefficients are formed in double, applied in fp32.
 * Other samplers: the same call applies their A x + B net form (see
 * drf_skip_transition_noise) as long as no requested transition has variance.
 *   x_from, eps_from  DEVICE fp32 [batch][elems_per_sample]
 *   s_to              HOST int [m], each 0 <= s_to[j] <= S (any direction is allowed)
 *   x_to              DEVICE fp32 [m][batch][elems_per_sample]; must not alias the inputs
 */
drf_status drf_skip_transition(const drf_sched_config* sched, const float* x_from, const float* eps_from,
                               int s_from, const int* s_to, int m, int batch, size_t elems_per_sample,
                               float* x_to, void* hip_stream);

/*
 * Skip transitions of the configured sampler, variance included: for j < m,
 *   x_to[j] = A_j x_from + B_j net_from + C_j z_j
 * DRF_DDIM:  A = sqrt(ab_to/ab_from), B = sqrt(1 - ab_to - sigma^2) - A sqrt(1 - ab_from), C = sigma,
 *            sigma = eta sqrt((1 - ab_from/ab_to)(1 - ab_to)/(1 - ab_from))   (Eq. ddim_skip_reverse);
 * DRF_DDPM:  A x + B eps = mu'(x, x_0_hat), C = sigma_{t,k}          (Eq. ddpm_skip_reverse_detail);
 * DRF_EULER: A = 1, B = sigma_to - sigma_from, C = 0.
 * z_j is field j of `noise`.  noise may be NULL when every C_j is 0 (DRF_EULER, eta == 0, or
 * all targets at index 0); otherwise that is DRF_EINVAL.  A transition with variance needs
 * 1 <= s_from and s_to[j] <= s_from.  Other arguments as in drf_skip_transition, which is this
 * call with noise == NULL.
 */
drf_status drf_skip_transition_noise(const drf_sched_config* sched, const float* x_from, const float* net_from,
                                     int s_from, const int* s_to, int m, int batch, size_t elems_per_sample,
                                     const drf_noise* noise, float* x_to, void* hip_stream);

/*
 * The library's noise stream, written out: elements 4q .. 4q+3 of field f are the four
 * normals of the Philox4x32-10 block with counter (q low, q high, f, 0) and key
 * (seed low, seed high); word pairs (r0, r1), (r2, r3) each give two normals by Box-Muller,
 * sqrt(-2 ln u_a) (cos, sin)(2 pi u_b), u = ((r >> 9) + 1/2) 2^-23.
 *   out  DEVICE fp32 [n_fields][field_elems], fields field0 .. field0 + n_fields - 1.
 * A stochastic call with drf_noise.z == NULL uses exactly these values.
 */
drf_status drf_normal_fill(uint64_t seed, uint32_t field0, size_t n_fields, size_t field_elems, float* out,
                           void* hip_stream);

/*
 * The standard denoising update s_from -> s_from - 1 (Algorithm 1, refinement loop).
 * It is the skip transition with a jump of one and runs the same kernel, so the two
 * agree bit for bit.  x_out may alias x.
 */
drf_status drf_refine_step(const drf_sched_config* sched, const float* x, const float* eps, int s_from,
                           int batch, size_t elems_per_sample, float* x_out, void* hip_stream);

/*
 * Draft-and-refine sampling, Algorithm 1 (DRF_AGGRESSIVE) or Algorithm 2
 * (DRF_CONSERVATIVE) with block size n; n = 1 is the sequential sampler in both modes.  The
 * last block is cut short at index 0 and a draft of x_0 is never fed to the network,
 * so exactly S predictor evaluations per sample are made.
 *   x_T        DEVICE fp32 [batch][in_ch][lat_h][lat_w]
 *   cond       DEVICE, per sample, layout as in drf_eps_batched with slots = batch
 *   null_cond  DEVICE, same layout, or NULL.  Non-NULL enables classifier-free guidance
 *              eps = eps_null + cfg_scale (eps_cond - eps_null) on every evaluation
 *              (this doubles the slots of every pass); cfg_scale is ignored when NULL.
 *   x_0_out    DEVICE fp32, same shape as x_T (may alias x_T)
 * No host synchronisation happens inside unless the workspace has to grow.
 */
drf_status drf_sample(drf_denoiser* den, const drf_sched_config* sched, drf_mode mode, int n, int batch,
                      const float* x_T, const void* cond, const void* null_cond, float cfg_scale,
                      float* x_0_out, void* hip_stream);

/*
 * drf_sample with the draws of the stochastic samplers (eta > 0, DRF_DDPM): one fresh field
 * per kind-1 row and per kind-2 row of the plan (see drf_plan_build), consumed in row order,
 * also by rows whose transition has no variance (a step onto index 0).  drf_noise_count gives
 * their number.  noise == NULL is allowed only when no transition has variance; drf_sample is
 * this call with noise == NULL.
 */
drf_status drf_sample_noise(drf_denoiser* den, const drf_sched_config* sched, drf_mode mode, int n, int batch,
                            const float* x_T, const void* cond, const void* null_cond, float cfg_scale,
                            const drf_noise* noise, float* x_0_out, void* hip_stream);
drf_status drf_noise_count(const drf_sched_config* sched, drf_mode mode, int n, size_t* count);

/*
 * The bookkeeping of drf_sample as a table (host only, no GPU needed).  Rows of
 * DRF_PLAN_ROW int32: {round, kind, s_from, s_to, tau}
 *   kind 0: stand-alone evaluation at anchor s_from = s_to, tau = tau(s_to)
 *   kind 1: draft s_from -> s_to by skip transition, evaluated at tau(s_to);
 *           a draft landing on index 0 is not evaluated and has tau = -1
 *   kind 2: standard update s_from -> s_to = s_from - 1, tau = -1
 * `round` numbers the batched predictor passes; kind-2 rows carry the round whose
 * noises they consume.  rows: HOST, capacity `cap` rows (may be NULL with cap 0);
 * *n_rows always receives the full row count.
 */
#define DRF_PLAN_ROW 5
drf_status drf_plan_build(const drf_sched_config* sched, drf_mode mode, int n, int32_t* rows, size_t cap,
                          size_t* n_rows);

/* HOST, thread-local, valid until the next failing call on this thread. */
const char* drf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DRF_H */
