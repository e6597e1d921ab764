/*
 * drf.h -- C ABI of libdrf: DRiffusion draft-and-refine sampling on one MI355X.
 *
 * The paper states the problem as: given sampled noise x_T, a number of sampling
 * steps T and a block size k, produce x_0 (Algorithm 1 / Algorithm 2, "Require /
 * Ensure").  Its three building blocks are the calls below:
 *   - the noise predictor eps_theta(x, t), evaluated on k drafts at once
 *     (Algorithm 1, the "concurrently" loop): drf_eps_batched;
 *   - the skip transition x_{t-k} = Skip(x_t, eps_t) (Eq. ddim_skip_reverse):
 *     drf_skip_transition;
 *   - the standard denoising update that refines the drafts (Algorithm 1, second
 *     loop): drf_refine_step;
 * and drf_sample runs the whole draft-and-refine loop in either mode.
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
 *   - One denoiser handle may be used by one stream at a time.
 *
 * Indices.  Sampling indices s run S, S-1, ..., 1, 0 (the paper's t, with S the
 * paper's T).  The network is fed the training timestep tau_s = (s-1) *
 * floor(train_steps / S) for s >= 1.  alpha-bar_s is the cumulative product of
 * (1 - beta) up to tau_s with linear betas; alpha-bar_0 = 1 (clean data).
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
    DRF_EUNSUPPORTED = -5   /* valid in the paper, not built here (eta > 0) */
} drf_status;

typedef enum { DRF_CONSERVATIVE = 0, DRF_AGGRESSIVE = 1 } drf_mode;
typedef enum { DRF_F32 = 0, DRF_BF16 = 1 } drf_dtype;
typedef enum { DRF_COND_VECTOR = 0, DRF_COND_CLASS = 1, DRF_COND_TEXT = 2 } drf_cond_kind;

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
 * create; GEMM and attention operands are bf16 with fp32 accumulation; LayerNorm and
 * softmax statistics, the residual stream, latents and all sampler updates are fp32.
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
    double eta;                 /* must be 0: deterministic DDIM (Eq. ddim_skip_reverse, sigma = 0) */
} drf_sched_config;

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
 * Introspection for parity tests: run only the first n_blocks blocks (0 = embedding
 * only) and write the fp32 residual stream, DEVICE [slots][T][D], to resid_out.
 */
drf_status drf_eps_trace(drf_denoiser* den, const float* x, const int32_t* t, const void* cond,
                         int slots, int n_blocks, float* resid_out, void* hip_stream);

/*
 * DDIM skip transitions with zero variance (Eq. ddim_skip_reverse; the draft line of
 * Algorithm 1): for j < m,
 *   x_to[j] = sqrt(ab_to/ab_from) x_from + (sqrt(1-ab_to) - sqrt(ab_to/ab_from) sqrt(1-ab_from)) eps_from
 * with ab_* the cumulative alpha at sampling indices s_from and s_to[j]; algebraically
 * the paper's predicted-x_0 form.  Coefficients are formed in double, applied in fp32.
 *   x_from, eps_from  DEVICE fp32 [batch][elems_per_sample]
 *   s_to              HOST int [m], each 0 <= s_to[j] <= S (any direction is allowed)
 *   x_to              DEVICE fp32 [m][batch][elems_per_sample]; must not alias the inputs
 */
drf_status drf_skip_transition(const drf_sched_config* sched, const float* x_from, const float* eps_from,
                               int s_from, const int* s_to, int m, int batch, size_t elems_per_sample,
                               float* x_to, void* hip_stream);

/*
 * The standard denoising update s_from -> s_from - 1 (Algorithm 1, refinement loop).
 * It is the skip transition with a jump of one and runs the same kernel, so the two
 * agree bit for bit.  x_out may alias x.
 */
drf_status drf_refine_step(const drf_sched_config* sched, const float* x, const float* eps, int s_from,
                           int batch, size_t elems_per_sample, float* x_out, void* hip_stream);

/*
 * Draft-and-refine sampling, Algorithm 1 (DRF_AGGRESSIVE) or Algorithm 2
 * (DRF_CONSERVATIVE) with block size n; n = 1 is sequential DDIM in both modes.  The
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

/*
 * Per-kernel-family timing with HIP events on the handle's stream, for roofline
 * reports.  While enabled, every launch of a family is bracketed by two events (this
 * adds a few microseconds per launch; leave it off when timing whole calls).
 * drf_profile_read synchronises the stream and returns, for family `which`
 * (DRF_PROF_*), the number of launches, their summed duration in milliseconds and
 * their summed algorithmic work (flops for GEMM/attention, bytes otherwise), then
 * clears the counters.
 */
enum { DRF_PROF_GEMM = 0, DRF_PROF_ATTN = 1, DRF_PROF_ELEMWISE = 2, DRF_PROF_UPDATE = 3, DRF_PROF_FAMILIES = 4 };
drf_status drf_profile_enable(drf_denoiser* den, int on);
drf_status drf_profile_read(drf_denoiser* den, int which, long long* launches, double* ms, double* work);

/*
 * Measurement hook: one launch of the library's bf16 GEMM on caller buffers,
 * out[M][N] (bf16) = A[M][K] (bf16) . W[N][K]^T (bf16) + bias[N] (fp32), all DEVICE.
 * variant 0 = the tile shape the forward pass would pick, > 0 forces one (for sweeps).
 * K % 64 == 0 and N % 4 == 0 are required.
 */
drf_status drf_probe_gemm_bf16(const void* A, const void* W, int M, int N, int K, void* out_bf16, const float* bias,
                               int variant, void* hip_stream);

/*
 * Measurement hook: one launch of the bf16 self-attention kernel.  qkv: DEVICE bf16
 * [slots * tokens][3 * heads * head_dim] (q | k | v), out: DEVICE bf16 [slots * tokens][heads * head_dim].
 */
drf_status drf_probe_attn_bf16(const void* qkv, void* out, int slots, int tokens, int heads, int head_dim,
                               void* hip_stream);

/* HOST, thread-local, valid until the next failing call on this thread. */
const char* drf_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* DRF_H */
