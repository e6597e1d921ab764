// Host-side bookkeeping of draft-and-refine sampling: the noise schedule, the
// coefficients of the skip transition, and the list of batched predictor passes
// for Algorithm 1 (aggressive) and Algorithm 2 (conservative).
#include <cmath>
#include <cstdarg>
#include <cstdio>

#include "common.h"

namespace drf {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

drf_status make_schedule(const drf_sched_config* sc, Schedule* out)
{
    if (!sc) DRF_FAIL(DRF_EINVAL, "schedule config is NULL");
    if (sc->train_steps < 2 || sc->steps < 1 || sc->steps > sc->train_steps)
        DRF_FAIL(DRF_EINVAL, "need 1 <= steps (%d) <= train_steps (%d), train_steps >= 2", sc->steps, sc->train_steps);
    if (!(sc->beta_start > 0.0) || !(sc->beta_end < 1.0) || !(sc->beta_start <= sc->beta_end))
        DRF_FAIL(DRF_EINVAL, "need 0 < beta_start <= beta_end < 1");
    if (sc->sampler != DRF_DDIM && sc->sampler != DRF_DDPM && sc->sampler != DRF_EULER)
        DRF_FAIL(DRF_EINVAL, "unknown sampler %d", (int)sc->sampler);
    if (sc->sampler == DRF_DDIM && !(sc->eta >= 0.0 && sc->eta <= 1.0)) DRF_FAIL(DRF_EINVAL, "need 0 <= eta <= 1");
    if (sc->sampler == DRF_EULER && !(sc->shift > 0.0)) DRF_FAIL(DRF_EINVAL, "need shift > 0 for the Euler sigma grid");
    // The paper's alpha_t is cumulative (forward marginal x_t = sqrt(alpha_t) x_0 + sqrt(1 - alpha_t) eps).
    out->abar.resize((size_t)sc->train_steps);
    double run = 1.0;
    const double db = (sc->beta_end - sc->beta_start) / (double)(sc->train_steps - 1);
    for (int j = 0; j < sc->train_steps; ++j) {
        run *= 1.0 - (sc->beta_start + db * (double)j);
        out->abar[(size_t)j] = run;
    }
    out->steps = sc->steps;
    out->stride = sc->train_steps / sc->steps;
    out->train_steps = sc->train_steps;
    out->sampler = sc->sampler;
    out->eta = sc->sampler == DRF_DDIM ? sc->eta : 0.0;
    out->shift = sc->sampler == DRF_EULER ? sc->shift : 1.0;
    return DRF_OK;
}

// Discretisation of the ODE time (section "Euler ODE Solvers" leaves the grid open): uniform in
// u = s / S from 0 (data) to 1 (noise), warped by sigma = shift u / (1 + (shift - 1) u).
double Schedule::sigma_at(int s) const
{
    const double u = (double)s / (double)steps;
    return shift * u / (1.0 + (shift - 1.0) * u);
}

int Schedule::net_time(int s) const
{
    if (sampler == DRF_EULER) return (int)std::floor(sigma_at(s) * (double)train_steps + 0.5);
    return tau(s);
}

// Every skip transition is affine in (x, net output, fresh noise): x_to = A x + B net + C z.
//   DDIM (Eq. ddim_skip_reverse), predicted x_0 substituted:
//     x_to = sqrt(ab_to) (x - sqrt(1-ab_from) eps)/sqrt(ab_from) + sqrt(1-ab_to-sigma^2) eps + sigma z,
//     sigma = eta * sqrt(posterior variance of the same jump);
//   DDPM (Eq. ddpm_skip_reverse_detail): mu' = [sqrt(r)(1-ab_to) x + sqrt(ab_to)(1-r) x_0_hat]/(1-ab_from),
//     r = ab_from/ab_to, plus sqrt((1-r)(1-ab_to)/(1-ab_from)) z;
//   Euler: x_to = x + (sigma_to - sigma_from) v.
drf_status Schedule::coef(int s_from, int s_to, float* A, float* B, float* C) const
{
    if (sampler == DRF_EULER) {
        *A = 1.f;
        *B = (float)(sigma_at(s_to) - sigma_at(s_from));
        *C = 0.f;
        return DRF_OK;
    }
    const double af = abar_at(s_from), at = abar_at(s_to);
    double sd = 0.0;
    if (stochastic() && s_to != s_from && s_to != 0) {
        if (s_from < 1 || s_to > s_from)
            DRF_FAIL(DRF_EINVAL, "a transition with variance must move towards data from an index >= 1 (got %d -> %d)",
                     s_from, s_to);
        sd = std::sqrt((1.0 - af / at) * (1.0 - at) / (1.0 - af));
    }
    if (sampler == DRF_DDPM) {
        if (s_from < 1) DRF_FAIL(DRF_EINVAL, "the DDPM posterior needs s_from >= 1 (got %d)", s_from);
        const double r = af / at;
        const double w0 = std::sqrt(at) * (1.0 - r) / (1.0 - af);        // weight of the predicted x_0
        *A = (float)(std::sqrt(r) * (1.0 - at) / (1.0 - af) + w0 / std::sqrt(af));
        *B = (float)(-w0 * std::sqrt(1.0 - af) / std::sqrt(af));
        *C = (float)sd;
        return DRF_OK;
    }
    const double sigma = eta * sd;
    const double a = std::sqrt(at / af);
    *A = (float)a;
    *B = (float)(std::sqrt(1.0 - at - sigma * sigma) - a * std::sqrt(1.0 - af));
    *C = (float)sigma;
    return DRF_OK;
}

// Division by an invariant (round-up method): for d not a power of two let s = ceil(log2 d)
// and magic = floor(2^(31+s) / d) + 1 < 2^32.  Then magic * d - 2^(31+s) <= d <= 2^s, which
// makes floor(n / d) = (n * magic) >> (31 + s) exact for every 0 <= n < 2^31.
void make_fast_div(int d, uint32_t* magic, int* shift)
{
    int s = 0;
    while ((1ll << s) < d) ++s;
    if ((1ll << s) == d) { *magic = 0; *shift = s; return; }
    *magic = (uint32_t)(((1ull << (31 + s)) / (unsigned long long)d) + 1ull);
    *shift = s - 1;             // after the high half of the 32 x 32 product
}

void set_rows_per_slot(Epilogue* e, int d)
{
    e->rows_per_slot = d;
    make_fast_div(d, &e->rps_magic, &e->rps_shift);
}

namespace {
struct RowSink {
    std::vector<int32_t>* rows;
    int draws = 0;              // kind-1 and kind-2 rows so far: each draws one fresh-noise field
    // returns the ordinal of the row's draw (kind 1, 2), else -1
    int put(int round, int kind, int from, int to, int tau)
    {
        if (rows) {
            const int32_t r[DRF_PLAN_ROW] = { round, kind, from, to, tau };
            rows->insert(rows->end(), r, r + DRF_PLAN_ROW);
        }
        return kind == 0 ? -1 : draws++;
    }
};
}  // namespace

drf_status build_plan(const Schedule& sch, drf_mode mode, int n, std::vector<Pass>* passes, std::vector<int32_t>* rows,
                      size_t* n_noise)
{
    if (n < 1) DRF_FAIL(DRF_EINVAL, "block size n must be >= 1 (got %d)", n);
    if (mode != DRF_CONSERVATIVE && mode != DRF_AGGRESSIVE) DRF_FAIL(DRF_EINVAL, "unknown mode %d", (int)mode);
    RowSink sink{ rows };
    std::vector<Pass> local;
    std::vector<Pass>& P = passes ? *passes : local;
    P.clear();
    if (rows) rows->clear();

    // Fills the `draft_to` of a pass whose update leaves an anchor pair at index s:
    // drafts to s-1 .. s-m.  A draft landing on 0 is only kept when it is x_0 itself (m == 1).
    // The rows of these drafts are the next ones emitted, so draft i draws field sink.draws + i - 1
    // (a draft that is not kept still has its row and its draw).
    auto plan_drafts = [&](Pass& p, int s, int m) {
        for (int i = 1; i <= m; ++i)
            if (s - i >= 1 || i == 1) {
                p.draft_to.push_back(s - i);
                p.draft_z.push_back(sink.draws + i - 1);
            }
        if (m == 1 && s == 1) p.writes_x0 = true;
    };

    int s = sch.steps, round = 0;
    if (mode == DRF_AGGRESSIVE) {
        // Algorithm 1.  One stand-alone evaluation at s = S seeds the first anchor pair;
        // afterwards each block's last draft noise is carried as the next anchor noise.
        Pass first;
        first.round = round; first.solo = true; first.s_anchor = s; first.eval_s = { s };
        first.anchor_field = 0; first.s_after = s;
        sink.put(round, 0, s, s, sch.net_time(s));
        int m = n < s ? n : s;
        plan_drafts(first, s, m);
        P.push_back(first);
        ++round;
        while (s > 0) {
            m = n < s ? n : s;
            const bool evaluates = s >= 2;          // a block whose only draft is x_0 runs no pass
            const int r = evaluates ? round : round - 1;
            for (int i = 1; i <= m; ++i) sink.put(r, 1, s, s - i, s - i >= 1 ? sch.net_time(s - i) : -1);
            std::vector<int> zs;
            for (int i = 2; i <= m; ++i) zs.push_back(sink.put(r, 2, s - i + 1, s - i, -1));
            if (!evaluates) break;                  // x_0 was written by the previous pass's update
            Pass p;
            p.round = round; p.s_anchor = s; p.base_is_draft = true;
            for (int i = 1; i <= m && s - i >= 1; ++i) p.eval_s.push_back(s - i);
            for (int i = 2; i <= m; ++i) p.chain.push_back({ s - i + 1, s - i });
            p.chain_z = zs;
            s -= m;
            p.s_after = s;
            if (s > 0) {
                p.anchor_field = m - 1;
                plan_drafts(p, s, n < s ? n : s);
            } else {
                p.writes_x0 = true;
            }
            P.push_back(p);
            ++round;
        }
    } else {
        // Algorithm 2.  Every anchor gets its own evaluation; the block then runs one update
        // further than the aggressive one because its last noise need not be carried.
        while (s > 0) {
            Pass solo;
            solo.round = round; solo.solo = true; solo.s_anchor = s; solo.eval_s = { s };
            solo.anchor_field = 0; solo.s_after = s;
            sink.put(round, 0, s, s, sch.net_time(s));
            const int m = n < s - 1 ? n : s - 1;
            if (m == 0) {                           // a single step is left: plain update 1 -> 0
                solo.draft_z = { sink.put(round, 2, s, s - 1, -1) };
                solo.draft_to = { 0 };
                solo.writes_x0 = true;
                P.push_back(solo);
                break;
            }
            for (int i = 1; i <= m; ++i) {
                solo.draft_to.push_back(s - i);
                solo.draft_z.push_back(sink.draws + i - 1);     // the kind-1 rows below
            }
            P.push_back(solo);
            ++round;
            Pass p;
            p.round = round; p.s_anchor = s; p.base_is_draft = true;
            for (int i = 1; i <= m; ++i) {
                p.eval_s.push_back(s - i);
                sink.put(round, 1, s, s - i, sch.net_time(s - i));
            }
            for (int i = 2; i <= m + 1; ++i) {
                p.chain.push_back({ s - i + 1, s - i });
                p.chain_z.push_back(sink.put(round, 2, s - i + 1, s - i, -1));
            }
            s -= m + 1;
            p.s_after = s;
            p.writes_x0 = (s == 0);
            P.push_back(p);
            ++round;
        }
    }
    if (n_noise) *n_noise = (size_t)sink.draws;
    return DRF_OK;
}

drf_status set_noise_source(UpdateArgs* a, const drf_noise* noise)
{
    bool needed = false;
    for (int i = 0; i < a->n_chain; ++i) needed = needed || a->cC[i] != 0.f;
    for (int j = 0; j < a->n_draft; ++j) needed = needed || a->dC[j] != 0.f;
    a->noise_mode = NOISE_NONE; a->z = nullptr; a->seed = 0; a->z_field0 = 0;
    if (!needed) return DRF_OK;
    if (!noise) DRF_FAIL(DRF_EINVAL, "this sampler adds fresh noise: a noise source is required");
    if (noise->z) { a->noise_mode = NOISE_EXPLICIT; a->z = noise->z; }
    else { a->noise_mode = NOISE_PHILOX; a->seed = noise->seed; a->z_field0 = noise->field0; }
    return DRF_OK;
}

}  // namespace drf

extern "C" const char* drf_last_error(void) { return drf::g_err; }

extern "C" drf_status drf_plan_build(const drf_sched_config* sched, drf_mode mode, int n, int32_t* rows, size_t cap,
                                     size_t* n_rows)
{
    drf::Schedule sch;
    drf_status st = drf::make_schedule(sched, &sch);
    if (st != DRF_OK) return st;
    if (!n_rows) DRF_FAIL(DRF_EINVAL, "n_rows is NULL");
    std::vector<int32_t> table;
    st = drf::build_plan(sch, mode, n, nullptr, &table);
    if (st != DRF_OK) return st;
    *n_rows = table.size() / DRF_PLAN_ROW;
    if (rows) {
        const size_t take = (*n_rows < cap ? *n_rows : cap) * DRF_PLAN_ROW;
        for (size_t i = 0; i < take; ++i) rows[i] = table[i];
    }
    return DRF_OK;
}

extern "C" drf_status drf_noise_count(const drf_sched_config* sched, drf_mode mode, int n, size_t* count)
{
    drf::Schedule sch;
    drf_status st = drf::make_schedule(sched, &sch);
    if (st != DRF_OK) return st;
    if (!count) DRF_FAIL(DRF_EINVAL, "count is NULL");
    return drf::build_plan(sch, mode, n, nullptr, nullptr, count);
}
