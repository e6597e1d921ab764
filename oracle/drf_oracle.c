/*
 * drf_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow CPU statement of what the DRiffusion hot path computes, used to
 * check the HIP library.  It shares no code with that library and must never be
 * linked, imported or called by it; only tests, the smoke check and the bench's
 * cpu_baseline leg use it.
 *
 * What is written out here, and the passage each part follows:
 *   - cumulative noise schedule and the forward marginal's coefficients
 *     (section "Skip Transitions / DDPM": x_t = sqrt(a_t) x_0 + sqrt(1-a_t) eps,
 *     a_t cumulative);
 *   - the DDIM skip transition with zero variance, in the literal
 *     predicted-x_0 form (Eq. ddim_skip_reverse; Algorithm 1, the draft line);
 *     the standard denoising update is the same operator with k = 1;
 *   - the aggressive scheduler (Algorithm 1) and the conservative scheduler
 *     (Algorithm 2, appendix), step by step in the paper's order;
 *   - the noise predictor: a latent DiT with adaLN modulation.  The paper treats
 *     the predictor as a black box, so its internals are this build's own
 *     definition (documented in include/drf.h); PARITY UNPINNED by the paper for
 *     the DiT forward -- it is pinned instead against library primitives
 *     (torch float64) and invariants in the tests;
 *   - classifier-free guidance eps = eps_u + w (eps_c - eps_u) (not in the paper;
 *     part of the workload definition).
 *
 * Arithmetic type: `real` = double by default; building with -DORC_F32 gives a
 * float build of the same text.  Schedule coefficients are always computed in
 * double.  No blocking, fusion or reordering: every Linear is a triple loop,
 * attention materialises one score row at a time.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef ORC_F32
typedef float real;
#define ORC_REAL_BYTES 4
#else
typedef double real;
#define ORC_REAL_BYTES 8
#endif

int orc_real_bytes(void) { return ORC_REAL_BYTES; }

#ifdef _OPENMP
#include <omp.h>
int orc_num_threads(void) { return omp_get_max_threads(); }
#else
int orc_num_threads(void) { return 1; }
#endif

/* ------------------------------------------------------------------ schedule */

typedef struct {
    int train_steps;      /* number of training timesteps (1000) */
    double beta_start;    /* linear betas */
    double beta_end;
    int steps;            /* S: number of sampling steps */
    double eta;           /* DDIM: sigma_{t,k} = eta * (DDPM posterior std of the same jump) */
    int sampler;          /* ORC_DDIM | ORC_DDPM | ORC_EULER */
    double shift;         /* Euler: time shift of the sigma grid (1 = uniform) */
} orc_sched;

enum { ORC_DDIM = 0, ORC_DDPM = 1, ORC_EULER = 2 };

/* Cumulative alpha (the paper's alpha_t) at training timestep j:
 * prod_{i<=j} (1 - beta_i), betas linear from beta_start to beta_end. */
void orc_alpha_bar(const orc_sched* sc, double* abar /* [train_steps] */)
{
    double prod = 1.0;
    for (int j = 0; j < sc->train_steps; ++j) {
        double beta = sc->beta_start +
                      (sc->beta_end - sc->beta_start) * (double)j / (double)(sc->train_steps - 1);
        prod *= 1.0 - beta;
        abar[j] = prod;
    }
}

/* Sampling index s (the paper's t, S..1) -> training timestep fed to the network.
 * Uniform stride floor(train_steps / S), starting at 0 for s = 1. */
int orc_tau(const orc_sched* sc, int s)
{
    return (s - 1) * (sc->train_steps / sc->steps);
}

/* Euler solvers: discretisation sigma_s, s = 0..S, of the ODE's time variable, from
 * sigma_0 = 0 (data) to sigma_S = 1 (noise): uniform u = s/S, optionally warped by the
 * usual time shift  sigma = shift u / (1 + (shift - 1) u). */
double orc_sigma_at(const orc_sched* sc, int s)
{
    double u = (double)s / (double)sc->steps;
    return sc->shift * u / (1.0 + (sc->shift - 1.0) * u);
}

/* Timestep fed to the network for sampling index s under the configured sampler.
 * Euler: the network's time input is sigma scaled to the training range, rounded to
 * the nearest integer timestep. */
int orc_net_time(const orc_sched* sc, int s)
{
    if (sc->sampler == ORC_EULER) return (int)floor(orc_sigma_at(sc, s) * (double)sc->train_steps + 0.5);
    return orc_tau(sc, s);
}

/* Cumulative alpha at sampling index s; index 0 is clean data (alpha = 1). */
double orc_abar_at(const orc_sched* sc, const double* abar, int s)
{
    return s == 0 ? 1.0 : abar[orc_tau(sc, s)];
}

/* ---------------------------------------------------- skip transition (DDIM) */

/* Eq. ddim_skip_reverse with sigma = 0, in the form Algorithm 1 prints:
 *   x0_hat = (x - sqrt(1 - a_from) eps) / sqrt(a_from)
 *   x_to   = sqrt(a_to) x0_hat + sqrt(1 - a_to) eps
 * Used both for drafts (any jump) and for the standard update (jump of 1). */
void orc_skip(const real* x, const real* eps, double a_from, double a_to, size_t n, real* out)
{
    const real sa_from = (real)sqrt(a_from), sn_from = (real)sqrt(1.0 - a_from);
    const real sa_to = (real)sqrt(a_to), sn_to = (real)sqrt(1.0 - a_to);
    for (size_t e = 0; e < n; ++e) {
        real x0_hat = (x[e] - sn_from * eps[e]) / sa_from;
        out[e] = sa_to * x0_hat + sn_to * eps[e];
    }
}

/* Variance of the Bayes posterior q(x_{t-k} | x_t, x_0) (Eq. ddpm_skip_reverse_detail),
 * with a_from = alpha_t and a_to = alpha_{t-k}. */
double orc_posterior_var(double a_from, double a_to)
{
    return (1.0 - a_from / a_to) * (1.0 - a_to) / (1.0 - a_from);
}

/* sigma_{t,k} of the stochastic DDIM skip: eta times the posterior standard deviation
 * of the same jump (eta = 0 deterministic, eta = 1 the DDPM-induced variance). */
double orc_sigma(double eta, double a_from, double a_to)
{
    return eta * sqrt(orc_posterior_var(a_from, a_to));
}

/* Eq. ddim_skip_reverse with sigma > 0, as the draft and refine lines of Algorithm 1
 * print it: predicted x_0, the noise direction shrunk to sqrt(1 - a_to - sigma^2), and
 * fresh noise z scaled by sigma.  z may be NULL when sigma == 0. */
void orc_skip_eta(const real* x, const real* eps, const real* z, double a_from, double a_to,
                  double sigma, size_t n, real* out)
{
    const real sa_from = (real)sqrt(a_from), sn_from = (real)sqrt(1.0 - a_from);
    const real sa_to = (real)sqrt(a_to), dir = (real)sqrt(1.0 - a_to - sigma * sigma);
    const real sg = (real)sigma;
    for (size_t e = 0; e < n; ++e) {
        real x0_hat = (x[e] - sn_from * eps[e]) / sa_from;
        real v = sa_to * x0_hat + dir * eps[e];
        if (z) v += sg * z[e];
        out[e] = v;
    }
}

/* DDPM skip transition (Eq. ddpm_skip_reverse, ddpm_skip_reverse_detail): a draw from the
 * Bayes posterior q(x_{t-k} | x_t, x_0) with x_0 replaced by the prediction from
 * (x_t, eps): mean mu', variance sigma_{t,k}^2.  z may be NULL when the variance is 0. */
void orc_ddpm_skip(const real* x, const real* eps, const real* z, double a_from, double a_to,
                   size_t n, real* out)
{
    const double ratio = a_from / a_to;                      /* alpha_t / alpha_{t-k} */
    const real sa_from = (real)sqrt(a_from), sn_from = (real)sqrt(1.0 - a_from);
    const real wx = (real)(sqrt(ratio) * (1.0 - a_to));      /* weight of x_t in mu' */
    const real w0 = (real)(sqrt(a_to) * (1.0 - ratio));      /* weight of x_0 in mu' */
    const real den = (real)(1.0 - a_from);
    const real sd = (real)sqrt(orc_posterior_var(a_from, a_to));
    for (size_t e = 0; e < n; ++e) {
        real x0_hat = (x[e] - sn_from * eps[e]) / sa_from;
        real v = (wx * x[e] + w0 * x0_hat) / den;
        if (z) v += sd * z[e];
        out[e] = v;
    }
}

/* First-order Euler skip of the ODE dx/dsigma = v: one integration step of any length,
 * x_to = x + (sigma_to - sigma_from) v. */
void orc_euler_skip(const real* x, const real* v, double sig_from, double sig_to, size_t n, real* out)
{
    const real h = (real)(sig_to - sig_from);
    for (size_t e = 0; e < n; ++e) out[e] = x[e] + h * v[e];
}

/* One transition s_from -> s_to of the configured sampler from the pair (x, net output);
 * z is this transition's fresh standard-normal field, or NULL for none. */
static void transition(const orc_sched* sc, const double* abar, const real* x, const real* net,
                       const real* z, int s_from, int s_to, size_t n, real* out)
{
    if (sc->sampler == ORC_EULER) {
        orc_euler_skip(x, net, orc_sigma_at(sc, s_from), orc_sigma_at(sc, s_to), n, out);
        return;
    }
    const double a_from = orc_abar_at(sc, abar, s_from), a_to = orc_abar_at(sc, abar, s_to);
    if (sc->sampler == ORC_DDPM)
        orc_ddpm_skip(x, net, z, a_from, a_to, n, out);
    else if (sc->eta == 0.0)
        orc_skip(x, net, a_from, a_to, n, out);
    else
        orc_skip_eta(x, net, z, a_from, a_to, orc_sigma(sc->eta, a_from, a_to), n, out);
}

/* ---------------------------------------------------------------- scheduler */

/* Noise predictor callback: eps for `batch` states that all sit at sampling
 * index s (training timestep tau).  x and eps_out are [batch * E]. */
typedef void (*orc_eps_fn)(void* user, const real* x, int s, int tau, real* eps_out);

/* Plan rows, 5 int32 each: {round, kind, s_from, s_to, tau}
 *   kind 0: stand-alone evaluation at an anchor   (s_from = s_to = anchor, tau = tau(s_to))
 *   kind 1: draft by skip s_from -> s_to, then evaluation at s_to (tau = tau(s_to));
 *           a draft that lands on index 0 is not evaluated: tau = -1
 *   kind 2: standard denoising update s_from -> s_to = s_from - 1 (tau = -1)
 * `round` counts batched predictor passes; kind-2 rows carry the round whose
 * noises they consume. */
enum { ORC_ROW = 5 };
enum { ORC_CONSERVATIVE = 0, ORC_AGGRESSIVE = 1 };

typedef struct {
    int32_t* rows;
    size_t cap, n;
} orc_plan;

static void plan_push(orc_plan* p, int round, int kind, int s_from, int s_to, int tau)
{
    if (p && p->rows && p->n < p->cap) {
        int32_t* r = p->rows + ORC_ROW * p->n;
        r[0] = round; r[1] = kind; r[2] = s_from; r[3] = s_to; r[4] = tau;
    }
    if (p) p->n++;
}

/* Draft-and-refine sampling.  Returns 0, or -1 on bad arguments.
 * fn may be NULL: then only the plan is produced (xT, x0 unused).
 * z: fresh standard-normal fields [n_noise][batch * E] for the stochastic samplers, one per
 * kind-1 row and one per kind-2 row of the plan, in plan order (the draws of the draft
 * loop and of the refine loop of Algorithm 1 / 2); NULL = no noise term is added.
 * plan_rows may be NULL.  *n_rows receives the number of rows the plan has
 * (even when it exceeds cap). */
int orc_sample(const orc_sched* sc, int mode, int n, int batch, size_t E, const real* xT,
               const real* z, orc_eps_fn fn, void* user, real* x0, int32_t* plan_rows, size_t cap,
               size_t* n_rows)
{
    if (!sc || n < 1 || sc->steps < 1 || sc->steps > sc->train_steps ||
        (mode != ORC_CONSERVATIVE && mode != ORC_AGGRESSIVE) || sc->sampler < ORC_DDIM ||
        sc->sampler > ORC_EULER)
        return -1;
    const int S = sc->steps;
    const size_t F = (size_t)batch * E;          /* one field: all samples at one index */
    double* abar = (double*)malloc(sizeof(double) * (size_t)sc->train_steps);
    orc_alpha_bar(sc, abar);
    orc_plan plan = { plan_rows, cap, 0 };
    size_t zi = 0;                               /* next unused noise field */
#define NEXT_Z() (z ? z + F * (zi++) : (zi++, (const real*)NULL))

    real *x = NULL, *eps = NULL, *drafts = NULL, *deps = NULL, *y = NULL;
    if (fn) {
        x = (real*)malloc(sizeof(real) * F);
        eps = (real*)malloc(sizeof(real) * F);
        y = (real*)malloc(sizeof(real) * F);
        drafts = (real*)malloc(sizeof(real) * F * (size_t)n);
        deps = (real*)malloc(sizeof(real) * F * (size_t)n);
        memcpy(x, xT, sizeof(real) * F);
    }

    int s = S, round = 0;
    if (mode == ORC_AGGRESSIVE) {
        /* Algorithm 1: one evaluation at the start gives the first anchor noise. */
        plan_push(&plan, round, 0, s, s, orc_net_time(sc, s));
        if (fn) fn(user, x, s, orc_net_time(sc, s), eps);
        ++round;
    }
    while (s > 0) {
        int m;
        if (mode == ORC_CONSERVATIVE) {
            /* Algorithm 2: stand-alone noise at every anchor. */
            plan_push(&plan, round, 0, s, s, orc_net_time(sc, s));
            if (fn) fn(user, x, s, orc_net_time(sc, s), eps);
            ++round;
            m = n < s - 1 ? n : s - 1;           /* last block is cut short at index 0 */
            if (m == 0) {                        /* one step left: plain update 1 -> 0 */
                plan_push(&plan, round - 1, 2, s, s - 1, -1);
                const real* zf = NEXT_Z();
                if (fn) {
                    transition(sc, abar, x, eps, zf, s, s - 1, F, y);
                    memcpy(x, y, sizeof(real) * F);
                }
                s = 0;
                break;
            }
        } else {
            m = n < s ? n : s;
        }
        /* Drafts x^d_{s-i} by skip transitions from the anchor pair (x_s, eps_s),
         * and their noises; a draft of x_0 itself is never fed to the network.
         * A block whose only draft is x_0 runs no predictor pass: its rows keep
         * the previous round's number. */
        const int has_eval = s >= 2;
        if (!has_eval) --round;
        for (int i = 1; i <= m; ++i) {
            int to = s - i;
            int tau = to >= 1 ? orc_net_time(sc, to) : -1;
            plan_push(&plan, round, 1, s, to, tau);
            const real* zf = NEXT_Z();
            if (fn) {
                real* d = drafts + F * (size_t)(i - 1);
                transition(sc, abar, x, eps, zf, s, to, F, d);
                if (to >= 1) fn(user, d, to, tau, deps + F * (size_t)(i - 1));
            }
        }
        /* Refinement: replay the standard update from the first draft onwards.
         * x_{s-1} is the first draft itself (a skip of one IS the standard update). */
        int last = (mode == ORC_CONSERVATIVE) ? m + 1 : m;
        if (fn) memcpy(y, drafts, sizeof(real) * F);
        for (int i = 2; i <= last; ++i) {
            plan_push(&plan, round, 2, s - i + 1, s - i, -1);
            const real* zf = NEXT_Z();
            if (fn) {
                transition(sc, abar, y, deps + F * (size_t)(i - 2), zf, s - i + 1, s - i, F, x);
                memcpy(y, x, sizeof(real) * F);
            }
        }
        if (fn) memcpy(x, y, sizeof(real) * F);
        s -= last;
        if (mode == ORC_AGGRESSIVE && s > 0 && fn)
            /* carry the noise of the draft that sat at the new anchor */
            memcpy(eps, deps + F * (size_t)(m - 1), sizeof(real) * F);
        ++round;
    }
#undef NEXT_Z
    if (fn) memcpy(x0, x, sizeof(real) * F);
    if (n_rows) *n_rows = plan.n;
    free(abar); free(x); free(eps); free(y); free(drafts); free(deps);
    return 0;
}

/* Number of noise fields orc_sample consumes: the kind-1 plus kind-2 rows of the plan. */
long orc_noise_count(const orc_sched* sc, int mode, int n)
{
    size_t rows = 0;
    if (orc_sample(sc, mode, n, 0, 0, NULL, NULL, NULL, NULL, NULL, NULL, 0, &rows) != 0) return -1;
    int32_t* tab = (int32_t*)malloc(sizeof(int32_t) * ORC_ROW * (rows ? rows : 1));
    orc_sample(sc, mode, n, 0, 0, NULL, NULL, NULL, NULL, NULL, tab, rows, &rows);
    long cnt = 0;
    for (size_t r = 0; r < rows; ++r) cnt += tab[ORC_ROW * r + 1] != 0;
    free(tab);
    return cnt;
}

/* ------------------------------------------------- counter-based normal draws */

/* Philox4x32 with 10 rounds (Salmon et al., "Parallel random numbers: as easy as 1, 2, 3",
 * SC'11): counter c[4], key k[2] -> four 32-bit words. */
void orc_philox4x32(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3], k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0, p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The library's noise stream: elements 4q .. 4q+3 of noise field f come from the Philox
 * block with counter (q low, q high, f, 0) and key = the 64-bit seed.  Words (r0, r1)
 * and (r2, r3) each give two normals by Box-Muller with u = ((r >> 9) + 1/2) 2^-23 in (0,1)
 * (24 significant bits: the same number in single and double precision):
 * sqrt(-2 ln u_a) * (cos, sin)(2 pi u_b). */
void orc_normal_fill(uint64_t seed, uint32_t field0, size_t n_fields, size_t F, real* out)
{
    const uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    const double two_pi = 6.283185307179586476925286766559;
    for (size_t f = 0; f < n_fields; ++f)
        for (size_t q = 0; 4 * q < F; ++q) {
            const uint32_t ctr[4] = { (uint32_t)q, (uint32_t)((uint64_t)q >> 32), field0 + (uint32_t)f, 0u };
            uint32_t r[4];
            orc_philox4x32(ctr, key, r);
            double u[4];
            for (int j = 0; j < 4; ++j) u[j] = ((double)(r[j] >> 9) + 0.5) / 8388608.0;
            const double nrm[4] = { sqrt(-2.0 * log(u[0])) * cos(two_pi * u[1]),
                                    sqrt(-2.0 * log(u[0])) * sin(two_pi * u[1]),
                                    sqrt(-2.0 * log(u[2])) * cos(two_pi * u[3]),
                                    sqrt(-2.0 * log(u[2])) * sin(two_pi * u[3]) };
            for (int j = 0; j < 4 && 4 * q + (size_t)j < F; ++j) out[f * F + 4 * q + (size_t)j] = (real)nrm[j];
        }
}

/* ------------------------------------------------------------- DiT denoiser */

enum { ORC_COND_VECTOR = 0, ORC_COND_CLASS = 1, ORC_COND_TEXT = 2 };

typedef struct {
    int depth, hidden, heads, mlp_ratio, patch, in_ch, lat_h, lat_w;
    int cond_kind;   /* vector | class | text */
    int cond_dim;    /* vector width | number of classes | context width */
    int ctx_len;     /* text: tokens of context, else 0 */
    int round_bf16;  /* 1: every parameter is rounded to bf16 (RNE) before use */
} orc_dit_config;

enum { ORC_TFREQ = 256 };   /* width of the sinusoidal timestep embedding */

/* Parameter layout: one flat array, Linear weights stored [out][in], in this
 * order (P = in_ch*patch^2, D = hidden, R = mlp_ratio):
 *   patch_w [D][P], patch_b [D]
 *   t_w1 [D][256], t_b1 [D], t_w2 [D][D], t_b2 [D]
 *   vector: c_w [D][cond_dim], c_b [D] | class: table [cond_dim+1][D] | text: none
 *   per block: ada_w [6D][D], ada_b [6D], qkv_w [3D][D], qkv_b [3D],
 *              proj_w [D][D], proj_b [D],
 *              text only: xq_w [D][D], xq_b [D], xkv_w [2D][cond_dim], xkv_b [2D],
 *                         xo_w [D][D], xo_b [D],
 *              fc1_w [RD][D], fc1_b [RD], fc2_w [D][RD], fc2_b [D]
 *   fin_ada_w [2D][D], fin_ada_b [2D], fin_w [P][D], fin_b [P]
 */
typedef struct {
    const real *patch_w, *patch_b, *t_w1, *t_b1, *t_w2, *t_b2, *c_w, *c_b, *table;
    const real *fin_ada_w, *fin_ada_b, *fin_w, *fin_b;
} orc_globals;
typedef struct {
    const real *ada_w, *ada_b, *qkv_w, *qkv_b, *proj_w, *proj_b;
    const real *xq_w, *xq_b, *xkv_w, *xkv_b, *xo_w, *xo_b;
    const real *fc1_w, *fc1_b, *fc2_w, *fc2_b;
} orc_block;

static size_t take(const real* base, size_t* off, size_t n, const real** out)
{
    if (out) *out = base ? base + *off : NULL;
    *off += n;
    return n;
}

static size_t layout(const orc_dit_config* c, const real* w, orc_globals* g, orc_block* blk)
{
    const size_t D = (size_t)c->hidden, P = (size_t)c->in_ch * c->patch * c->patch;
    const size_t R = (size_t)c->mlp_ratio;
    size_t off = 0;
    orc_globals gg; orc_block bb;
    if (!g) g = &gg;
    memset(g, 0, sizeof(*g));
    take(w, &off, D * P, &g->patch_w); take(w, &off, D, &g->patch_b);
    take(w, &off, D * ORC_TFREQ, &g->t_w1); take(w, &off, D, &g->t_b1);
    take(w, &off, D * D, &g->t_w2); take(w, &off, D, &g->t_b2);
    if (c->cond_kind == ORC_COND_VECTOR) {
        take(w, &off, D * (size_t)c->cond_dim, &g->c_w); take(w, &off, D, &g->c_b);
    } else if (c->cond_kind == ORC_COND_CLASS) {
        take(w, &off, ((size_t)c->cond_dim + 1) * D, &g->table);
    }
    for (int l = 0; l < c->depth; ++l) {
        orc_block* b = blk ? blk + l : &bb;
        memset(b, 0, sizeof(*b));
        take(w, &off, 6 * D * D, &b->ada_w); take(w, &off, 6 * D, &b->ada_b);
        take(w, &off, 3 * D * D, &b->qkv_w); take(w, &off, 3 * D, &b->qkv_b);
        take(w, &off, D * D, &b->proj_w); take(w, &off, D, &b->proj_b);
        if (c->cond_kind == ORC_COND_TEXT) {
            take(w, &off, D * D, &b->xq_w); take(w, &off, D, &b->xq_b);
            take(w, &off, 2 * D * (size_t)c->cond_dim, &b->xkv_w); take(w, &off, 2 * D, &b->xkv_b);
            take(w, &off, D * D, &b->xo_w); take(w, &off, D, &b->xo_b);
        }
        take(w, &off, R * D * D, &b->fc1_w); take(w, &off, R * D, &b->fc1_b);
        take(w, &off, D * R * D, &b->fc2_w); take(w, &off, D, &b->fc2_b);
    }
    take(w, &off, 2 * D * D, &g->fin_ada_w); take(w, &off, 2 * D, &g->fin_ada_b);
    take(w, &off, P * D, &g->fin_w); take(w, &off, P, &g->fin_b);
    return off;
}

size_t orc_weight_count(const orc_dit_config* c) { return layout(c, NULL, NULL, NULL); }

/* Round-to-nearest-even to bfloat16 (1-8-7), returned as a real. */
static real round_bf16(real v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) != 0x7f800000u)       /* finite */
        u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (real)f;
}

/* y[M][N] = x[M][K] . W[N][K]^T + b[N] */
static void linear(real* y, const real* x, const real* W, const real* b, size_t M, size_t K, size_t N)
{
#pragma omp parallel for schedule(static)
    for (size_t m = 0; m < M; ++m)
        for (size_t n = 0; n < N; ++n) {
            real acc = 0;
            const real *xr = x + m * K, *wr = W + n * K;
#pragma omp simd reduction(+ : acc)
            for (size_t k = 0; k < K; ++k) acc += xr[k] * wr[k];
            y[m * N + n] = acc + b[n];
        }
}

static real silu(real v) { return v / (1 + (real)exp(-(double)v)); }

static real gelu_tanh(real v)
{
    double x = (double)v;
    return (real)(0.5 * x * (1.0 + tanh(0.7978845608028654 * (x + 0.044715 * x * x * x))));
}

/* LayerNorm over the last axis, no affine, eps 1e-6 (biased variance), then
 * optional modulation out = ln * (1 + scale) + shift with per-row vectors. */
static void ln_modulate(real* out, const real* x, size_t rows, size_t D, const real* shift,
                        const real* scale)
{
    for (size_t r = 0; r < rows; ++r) {
        const real* xr = x + r * D;
        double mean = 0, var = 0;
        for (size_t j = 0; j < D; ++j) mean += xr[j];
        mean /= (double)D;
        for (size_t j = 0; j < D; ++j) var += (xr[j] - mean) * (xr[j] - mean);
        var /= (double)D;
        double rstd = 1.0 / sqrt(var + 1e-6);
        for (size_t j = 0; j < D; ++j) {
            real v = (real)((xr[j] - mean) * rstd);
            out[r * D + j] = shift ? v * (1 + scale[j]) + shift[j] : v;
        }
    }
}

/* Multi-head attention, no mask: q [Nq][ldq], k/v [Nk][ldk]; head h uses
 * columns [h*d, (h+1)*d).  out [Nq][D]. */
static void attention(real* out, const real* q, size_t ldq, const real* k, const real* v,
                      size_t ldk, size_t Nq, size_t Nk, int heads, size_t d)
{
    const size_t D = (size_t)heads * d;
    const double scale = 1.0 / sqrt((double)d);
#pragma omp parallel
    {
        double* p = (double*)malloc(sizeof(double) * Nk);
#pragma omp for collapse(2) schedule(static)
        for (int h = 0; h < heads; ++h)
            for (size_t i = 0; i < Nq; ++i) {
                const real* qi = q + i * ldq + (size_t)h * d;
                double mx = -INFINITY, sum = 0;
                for (size_t j = 0; j < Nk; ++j) {
                    const real* kj = k + j * ldk + (size_t)h * d;
                    double sc = 0;
                    for (size_t e = 0; e < d; ++e) sc += (double)qi[e] * (double)kj[e];
                    p[j] = sc * scale;
                    if (p[j] > mx) mx = p[j];
                }
                for (size_t j = 0; j < Nk; ++j) { p[j] = exp(p[j] - mx); sum += p[j]; }
                for (size_t e = 0; e < d; ++e) {
                    double acc = 0;
                    for (size_t j = 0; j < Nk; ++j)
                        acc += p[j] * (double)v[j * ldk + (size_t)h * d + e];
                    out[i * D + (size_t)h * d + e] = (real)(acc / sum);
                }
            }
        free(p);
    }
}

/* The two building blocks above, exported for kernel-level parity tests. */
void orc_linear(real* y, const real* x, const real* W, const real* b, size_t M, size_t K, size_t N)
{
    linear(y, x, W, b, M, K, N);
}
void orc_attention(real* out, const real* q, size_t ldq, const real* k, const real* v, size_t ldk, size_t Nq,
                   size_t Nk, int heads, size_t d)
{
    attention(out, q, ldq, k, v, ldk, Nq, Nk, heads, d);
}

/* eps_theta(x, tau, cond) for `slots` independent samples, each with its own
 * timestep.  x, eps_out: [slots][in_ch][lat_h][lat_w].
 * cond: vector real [slots][cond_dim] | class int32 [slots] (cond_dim = null class)
 *       | text real [slots][ctx_len][cond_dim].
 * stop_blocks >= 0 with resid_out != NULL: run only that many blocks, write the
 * residual stream [slots][tokens][D] to resid_out and leave eps_out untouched.
 * Returns 0, -1 on bad configuration. */
int orc_dit_eps(const orc_dit_config* c, const real* weights, const real* x, const int32_t* t,
                const void* cond, int slots, real* eps_out, int stop_blocks, real* resid_out)
{
    const size_t D = (size_t)c->hidden, p = (size_t)c->patch, C = (size_t)c->in_ch;
    const size_t H = (size_t)c->lat_h, W = (size_t)c->lat_w;
    if (c->hidden % c->heads || c->hidden % 4 || c->lat_h % c->patch || c->lat_w % c->patch) return -1;
    const size_t gh = H / p, gw = W / p, T = gh * gw, P = C * p * p, R = (size_t)c->mlp_ratio;
    const size_t d = D / (size_t)c->heads, E = C * H * W;

    /* parameters, rounded once when the configuration says bf16 */
    const size_t nw = orc_weight_count(c);
    real* wr = NULL;
    if (c->round_bf16) {
        wr = (real*)malloc(sizeof(real) * nw);
        for (size_t i = 0; i < nw; ++i) wr[i] = round_bf16(weights[i]);
        weights = wr;
    }
    orc_globals g;
    orc_block* blk = (orc_block*)malloc(sizeof(orc_block) * (size_t)c->depth);
    layout(c, weights, &g, blk);

    real* tok = (real*)malloc(sizeof(real) * T * P);
    real* xs = (real*)malloc(sizeof(real) * T * D);       /* residual stream */
    real* hbuf = (real*)malloc(sizeof(real) * T * D);
    real* qkv = (real*)malloc(sizeof(real) * T * 3 * D);
    real* att = (real*)malloc(sizeof(real) * T * D);
    real* prj = (real*)malloc(sizeof(real) * T * D);
    real* mid = (real*)malloc(sizeof(real) * T * R * D);
    real* mod = (real*)malloc(sizeof(real) * 6 * D);
    real* ckv = c->cond_kind == ORC_COND_TEXT ? (real*)malloc(sizeof(real) * (size_t)c->ctx_len * 2 * D) : NULL;
    real* outp = (real*)malloc(sizeof(real) * T * P);
    real *femb = (real*)malloc(sizeof(real) * ORC_TFREQ), *h1 = (real*)malloc(sizeof(real) * D);
    real *cvec = (real*)malloc(sizeof(real) * D), *cact = (real*)malloc(sizeof(real) * D);
    real* cemb = (real*)malloc(sizeof(real) * D);

    for (int sl = 0; sl < slots; ++sl) {
        /* conditioning vector c = MLP(sinusoid(tau)) + cond embedding */
        const int half = ORC_TFREQ / 2;
        for (int i = 0; i < half; ++i) {
            double f = exp(-log(10000.0) * (double)i / (double)half);
            femb[i] = (real)cos((double)t[sl] * f);
            femb[half + i] = (real)sin((double)t[sl] * f);
        }
        linear(h1, femb, g.t_w1, g.t_b1, 1, ORC_TFREQ, D);
        for (size_t j = 0; j < D; ++j) h1[j] = silu(h1[j]);
        linear(cvec, h1, g.t_w2, g.t_b2, 1, D, D);
        if (c->cond_kind == ORC_COND_VECTOR) {
            linear(cemb, (const real*)cond + (size_t)sl * c->cond_dim, g.c_w, g.c_b, 1, (size_t)c->cond_dim, D);
            for (size_t j = 0; j < D; ++j) cvec[j] += cemb[j];
        } else if (c->cond_kind == ORC_COND_CLASS) {
            int cls = ((const int32_t*)cond)[sl];
            for (size_t j = 0; j < D; ++j) cvec[j] += g.table[(size_t)cls * D + j];
        }
        for (size_t j = 0; j < D; ++j) cact[j] = silu(cvec[j]);

        /* patchify: token (py,px) holds x[ch][py*p+dy][px*p+dx] at ch*p*p + dy*p + dx */
        const real* xi = x + (size_t)sl * E;
        for (size_t py = 0; py < gh; ++py)
            for (size_t px = 0; px < gw; ++px)
                for (size_t ch = 0; ch < C; ++ch)
                    for (size_t dy = 0; dy < p; ++dy)
                        for (size_t dx = 0; dx < p; ++dx)
                            tok[(py * gw + px) * P + ch * p * p + dy * p + dx] =
                                xi[(ch * H + py * p + dy) * W + px * p + dx];
        linear(xs, tok, g.patch_w, g.patch_b, T, P, D);
        /* fixed 2-D sin-cos position code: first D/2 columns from the grid row,
         * last D/2 from the grid column; each half is [sin | cos] over D/4
         * frequencies 10000^(-i/(D/4)). */
        const size_t q4 = D / 4;
        for (size_t py = 0; py < gh; ++py)
            for (size_t px = 0; px < gw; ++px)
                for (size_t i = 0; i < q4; ++i) {
                    double om = exp(-log(10000.0) * (double)i / (double)q4);
                    real* row = xs + (py * gw + px) * D;
                    row[i] += (real)sin((double)py * om);
                    row[q4 + i] += (real)cos((double)py * om);
                    row[2 * q4 + i] += (real)sin((double)px * om);
                    row[3 * q4 + i] += (real)cos((double)px * om);
                }

        int nblk = (stop_blocks >= 0 && resid_out) ? stop_blocks : c->depth;
        for (int l = 0; l < nblk; ++l) {
            const orc_block* b = blk + l;
            linear(mod, cact, b->ada_w, b->ada_b, 1, D, 6 * D);
            const real *shift1 = mod, *scale1 = mod + D, *gate1 = mod + 2 * D;
            const real *shift2 = mod + 3 * D, *scale2 = mod + 4 * D, *gate2 = mod + 5 * D;
            /* self-attention branch */
            ln_modulate(hbuf, xs, T, D, shift1, scale1);
            linear(qkv, hbuf, b->qkv_w, b->qkv_b, T, D, 3 * D);
            attention(att, qkv, 3 * D, qkv + D, qkv + 2 * D, 3 * D, T, T, c->heads, d);
            linear(prj, att, b->proj_w, b->proj_b, T, D, D);
            for (size_t r = 0; r < T; ++r)
                for (size_t j = 0; j < D; ++j) xs[r * D + j] += gate1[j] * prj[r * D + j];
            /* cross-attention to the text context (ungated, plain LayerNorm) */
            if (c->cond_kind == ORC_COND_TEXT) {
                const real* ctx = (const real*)cond + (size_t)sl * c->ctx_len * c->cond_dim;
                ln_modulate(hbuf, xs, T, D, NULL, NULL);
                linear(qkv, hbuf, b->xq_w, b->xq_b, T, D, D);
                linear(ckv, ctx, b->xkv_w, b->xkv_b, (size_t)c->ctx_len, (size_t)c->cond_dim, 2 * D);
                attention(att, qkv, D, ckv, ckv + D, 2 * D, T, (size_t)c->ctx_len, c->heads, d);
                linear(prj, att, b->xo_w, b->xo_b, T, D, D);
                for (size_t i = 0; i < T * D; ++i) xs[i] += prj[i];
            }
            /* MLP branch */
            ln_modulate(hbuf, xs, T, D, shift2, scale2);
            linear(mid, hbuf, b->fc1_w, b->fc1_b, T, D, R * D);
            for (size_t i = 0; i < T * R * D; ++i) mid[i] = gelu_tanh(mid[i]);
            linear(prj, mid, b->fc2_w, b->fc2_b, T, R * D, D);
            for (size_t r = 0; r < T; ++r)
                for (size_t j = 0; j < D; ++j) xs[r * D + j] += gate2[j] * prj[r * D + j];
        }
        if (stop_blocks >= 0 && resid_out) {
            memcpy(resid_out + (size_t)sl * T * D, xs, sizeof(real) * T * D);
            continue;
        }
        /* final layer and unpatchify (predicts eps only: in_ch output channels) */
        linear(mod, cact, g.fin_ada_w, g.fin_ada_b, 1, D, 2 * D);
        ln_modulate(hbuf, xs, T, D, mod, mod + D);
        linear(outp, hbuf, g.fin_w, g.fin_b, T, D, P);
        real* eo = eps_out + (size_t)sl * E;
        for (size_t py = 0; py < gh; ++py)
            for (size_t px = 0; px < gw; ++px)
                for (size_t ch = 0; ch < C; ++ch)
                    for (size_t dy = 0; dy < p; ++dy)
                        for (size_t dx = 0; dx < p; ++dx)
                            eo[(ch * H + py * p + dy) * W + px * p + dx] =
                                outp[(py * gw + px) * P + ch * p * p + dy * p + dx];
    }
    free(tok); free(xs); free(hbuf); free(qkv); free(att); free(prj); free(mid); free(mod);
    free(ckv); free(outp); free(femb); free(h1); free(cvec); free(cact); free(cemb);
    free(blk); free(wr);
    return 0;
}

/* --------------------------------------- DiT + guidance as the noise predictor */

typedef struct {
    const orc_dit_config* cfg;
    const real* weights;
    const void* cond;        /* [batch] conditioning, layout as in orc_dit_eps */
    const void* null_cond;   /* same layout; NULL: no guidance */
    double guidance;         /* w */
    int batch;
} orc_dit_user;

static void dit_eps_fn(void* user, const real* x, int s, int tau, real* eps_out)
{
    (void)s;
    const orc_dit_user* u = (const orc_dit_user*)user;
    const orc_dit_config* c = u->cfg;
    const size_t E = (size_t)c->in_ch * c->lat_h * c->lat_w, F = E * (size_t)u->batch;
    int32_t* t = (int32_t*)malloc(sizeof(int32_t) * (size_t)u->batch);
    for (int b = 0; b < u->batch; ++b) t[b] = tau;
    orc_dit_eps(c, u->weights, x, t, u->cond, u->batch, eps_out, -1, NULL);
    if (u->null_cond) {
        /* guidance: eps = eps_u + w (eps_c - eps_u), same x and tau for both */
        real* eu = (real*)malloc(sizeof(real) * F);
        orc_dit_eps(c, u->weights, x, t, u->null_cond, u->batch, eu, -1, NULL);
        const real w = (real)u->guidance;
        for (size_t e = 0; e < F; ++e) eps_out[e] = eu[e] + w * (eps_out[e] - eu[e]);
        free(eu);
    }
    free(t);
}

/* Whole path with the DiT as predictor.  null_cond == NULL: no guidance.
 * z: noise fields as in orc_sample, or NULL. */
int orc_sample_dit(const orc_dit_config* c, const real* weights, const orc_sched* sc, int mode,
                   int n, int batch, const real* xT, const real* z, const void* cond,
                   const void* null_cond, double guidance, real* x0)
{
    orc_dit_user u = { c, weights, cond, null_cond, guidance, batch };
    const size_t E = (size_t)c->in_ch * c->lat_h * c->lat_w;
    return orc_sample(sc, mode, n, batch, E, xT, z, dit_eps_fn, &u, x0, NULL, 0, NULL);
}

/* One guided noise evaluation for a batch at a common training timestep. */
int orc_eps_guided(const orc_dit_config* c, const real* weights, const real* x, int tau,
                   const void* cond, const void* null_cond, double guidance, int batch,
                   real* eps_out)
{
    orc_dit_user u = { c, weights, cond, null_cond, guidance, batch };
    dit_eps_fn(&u, x, 0, tau, eps_out);
    return 0;
}
