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
    if (sc->eta != 0.0) DRF_FAIL(DRF_EUNSUPPORTED, "only eta = 0 (zero-variance DDIM skip transitions) is built");
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
    return DRF_OK;
}

// Eq. ddim_skip_reverse with sigma = 0, with the predicted x_0 substituted:
//   x_to = sqrt(ab_to) (x - sqrt(1-ab_from) eps)/sqrt(ab_from) + sqrt(1-ab_to) eps = A x + B eps.
void Schedule::coef(int s_from, int s_to, float* A, float* B) const
{
    const double af = abar_at(s_from), at = abar_at(s_to);
    const double a = std::sqrt(at / af);
    *A = (float)a;
    *B = (float)(std::sqrt(1.0 - at) - a * std::sqrt(1.0 - af));
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
    void put(int round, int kind, int from, int to, int tau)
    {
        if (!rows) return;
        const int32_t r[DRF_PLAN_ROW] = { round, kind, from, to, tau };
        rows->insert(rows->end(), r, r + DRF_PLAN_ROW);
    }
};
}  // namespace

drf_status build_plan(const Schedule& sch, drf_mode mode, int n, std::vector<Pass>* passes, std::vector<int32_t>* rows)
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
    auto plan_drafts = [&](Pass& p, int s, int m) {
        for (int i = 1; i <= m; ++i)
            if (s - i >= 1 || i == 1) p.draft_to.push_back(s - i);
        if (m == 1 && s == 1) p.writes_x0 = true;
    };

    int s = sch.steps, round = 0;
    if (mode == DRF_AGGRESSIVE) {
        // Algorithm 1.  One stand-alone evaluation at s = S seeds the first anchor pair;
        // afterwards each block's last draft noise is carried as the next anchor noise.
        Pass first;
        first.round = round; first.solo = true; first.s_anchor = s; first.eval_s = { s };
        first.anchor_field = 0; first.s_after = s;
        sink.put(round, 0, s, s, sch.tau(s));
        int m = n < s ? n : s;
        plan_drafts(first, s, m);
        P.push_back(first);
        ++round;
        while (s > 0) {
            m = n < s ? n : s;
            const bool evaluates = s >= 2;          // a block whose only draft is x_0 runs no pass
            const int r = evaluates ? round : round - 1;
            for (int i = 1; i <= m; ++i) sink.put(r, 1, s, s - i, s - i >= 1 ? sch.tau(s - i) : -1);
            for (int i = 2; i <= m; ++i) sink.put(r, 2, s - i + 1, s - i, -1);
            if (!evaluates) break;                  // x_0 was written by the previous pass's update
            Pass p;
            p.round = round; p.s_anchor = s; p.base_is_draft = true;
            for (int i = 1; i <= m && s - i >= 1; ++i) p.eval_s.push_back(s - i);
            for (int i = 2; i <= m; ++i) p.chain.push_back({ s - i + 1, s - i });
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
            sink.put(round, 0, s, s, sch.tau(s));
            const int m = n < s - 1 ? n : s - 1;
            if (m == 0) {                           // a single step is left: plain update 1 -> 0
                sink.put(round, 2, s, s - 1, -1);
                solo.draft_to = { 0 };
                solo.writes_x0 = true;
                P.push_back(solo);
                break;
            }
            for (int i = 1; i <= m; ++i) solo.draft_to.push_back(s - i);
            P.push_back(solo);
            ++round;
            Pass p;
            p.round = round; p.s_anchor = s; p.base_is_draft = true;
            for (int i = 1; i <= m; ++i) {
                p.eval_s.push_back(s - i);
                sink.put(round, 1, s, s - i, sch.tau(s - i));
            }
            for (int i = 2; i <= m + 1; ++i) {
                p.chain.push_back({ s - i + 1, s - i });
                sink.put(round, 2, s - i + 1, s - i, -1);
            }
            s -= m + 1;
            p.s_after = s;
            p.writes_x0 = (s == 0);
            P.push_back(p);
            ++round;
        }
    }
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
