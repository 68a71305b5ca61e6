// Host-side speculative-length policy (paper Sec. 4 and 5): time model, accepted-token model,
// SLO-aware efficiency estimator (Alg. 3), adaptive drafter (Alg. 1) and draft-token
// elimination (Alg. 2).  Pure host code in double precision; the estimates are kept as running
// sums so that one more draft step or one eliminated token costs O(B) or O(1), not a recount.
#include <math.h>
#include <stdint.h>

#include <limits>
#include <vector>

#include "adaspec.h"
#include "adaspec_policy.h"

namespace {

// sum over j = 1..n of (C + j - 1): context tokens of n consecutive passes / positions
inline double ctx_tokens(double C, double n) { return n * C + n * (n - 1.0) * 0.5; }
// context tokens the target pass is charged for a request with k drafts
inline double verify_ctx(const adaspec_time_model &m, double C, double k)
{
    return m.verify_ctx_once ? C + k + 1.0 : ctx_tokens(C, k + 1.0);
}

struct Sums {
    double sum_c = 0.0;      // sum of C_i
    int B = 0;
};

inline double draft_time(const adaspec_time_model &m, const Sums &s, int steps)
{
    // passes 1..steps, each over all B requests
    const double n_c = steps * s.sum_c + s.B * (double)steps * (steps - 1.0) * 0.5;
    return m.alpha_d * n_c + m.gamma_d * (double)steps * s.B + m.delta_d * steps;
}

inline double verify_time(const adaspec_time_model &m, double n_c, double n_b)
{
    return m.alpha_v * n_c + m.gamma_v * n_b + m.delta_v;
}

bool bad_model(const adaspec_time_model *m) { return m == nullptr; }

}  // namespace

extern "C" {

double adaspec_policy_estimate_time(const adaspec_time_model *m, int32_t B, const int32_t *C,
                                    int32_t draft_steps, const int32_t *spec_lens)
{
    if (bad_model(m) || B < 0 || draft_steps < 0 || (B > 0 && !C)) return NAN;
    Sums s;
    s.B = B;
    double n_c = 0.0, n_b = 0.0;
    for (int i = 0; i < B; ++i) {
        const int k = spec_lens ? spec_lens[i] : draft_steps;
        if (k < 0 || k > draft_steps) return NAN;
        s.sum_c += C[i];
        n_c += verify_ctx(*m, C[i], k);
        n_b += k + 1.0;
    }
    return draft_time(*m, s, draft_steps) + verify_time(*m, n_c, n_b);
}

double adaspec_policy_goodput(const adaspec_time_model *m, int32_t B, const int32_t *C,
                              int32_t draft_steps, const int32_t *spec_lens, const double *ar, double tpot)
{
    const double t = adaspec_policy_estimate_time(m, B, C, draft_steps, spec_lens);
    if (isnan(t) || (draft_steps > 0 && B > 0 && !ar)) return NAN;
    if (t > tpot) return -1.0;
    double nat = 0.0;
    for (int i = 0; i < B; ++i) {
        const int k = spec_lens ? spec_lens[i] : draft_steps;
        nat += 1.0;
        for (int s = 0; s < k; ++s) nat += ar[(int64_t)s * B + i];
    }
    return nat / t;
}

int adaspec_policy_adaptive_draft(const adaspec_time_model *m, int32_t B, const int32_t *C,
                                  const double *conf, int32_t max_steps, double prev_conf, double tpot,
                                  int32_t *steps_out, double *ar_out, double *goodput_out)
{
    if (bad_model(m) || !steps_out || !goodput_out) return ADASPEC_ERR_NULL;
    if (B < 0 || max_steps < 0) return ADASPEC_ERR_DIM;
    if (B > 0 && (!C || (max_steps > 0 && (!conf || !ar_out)))) return ADASPEC_ERR_NULL;
    Sums s;
    s.B = B;
    for (int i = 0; i < B; ++i) s.sum_c += C[i];
    // running state of the EXECUTED steps: every request carries `steps` drafts
    int steps = 0;
    double nat = B;                      // bonus tokens
    double best = -1.0;
    auto time_at = [&](int st) {         // all requests verified at st drafts each
        double n_c = m->verify_ctx_once ? s.sum_c + B * (st + 1.0)
                                        : (st + 1.0) * s.sum_c + B * (st + 1.0) * st * 0.5;
        return draft_time(*m, s, st) + verify_time(*m, n_c, (st + 1.0) * B);
    };
    for (;;) {
        // predict: one more step whose acceptance rates are all prev_conf
        const double t_pred = time_at(steps + 1);
        const double g_pred = t_pred > tpot ? -1.0 : (nat + prev_conf * B) / t_pred;
        if (!(g_pred > best) || steps >= max_steps) break;
        // execute: the draft model's confidences of this step; correct the running sums
        double add = 0.0;
        for (int i = 0; i < B; ++i) {
            const double before = steps == 0 ? 1.0 : ar_out[(int64_t)(steps - 1) * B + i];
            const double a = before * conf[(int64_t)steps * B + i];
            ar_out[(int64_t)steps * B + i] = a;
            add += a;
        }
        nat += add;
        ++steps;
        const double t_now = time_at(steps);
        best = t_now > tpot ? -1.0 : nat / t_now;
    }
    *steps_out = steps;
    *goodput_out = best;
    return ADASPEC_OK;
}

int adaspec_policy_eliminate(const adaspec_time_model *m, int32_t B, const int32_t *C,
                             int32_t draft_steps, const double *ar, double tpot,
                             int32_t *spec_lens_out, double *goodput_out)
{
    if (bad_model(m) || !goodput_out) return ADASPEC_ERR_NULL;
    if (B < 0 || draft_steps < 0) return ADASPEC_ERR_DIM;
    if (B > 0 && (!C || !spec_lens_out || (draft_steps > 0 && !ar))) return ADASPEC_ERR_NULL;
    Sums s;
    s.B = B;
    double n_c = 0.0, n_b = 0.0, nat = 0.0;
    for (int i = 0; i < B; ++i) {
        s.sum_c += C[i];
        spec_lens_out[i] = draft_steps;
        n_c += verify_ctx(*m, C[i], draft_steps);
        n_b += draft_steps + 1.0;
        nat += 1.0;
        for (int st = 0; st < draft_steps; ++st) nat += ar[(int64_t)st * B + i];
    }
    const double t_d = draft_time(*m, s, draft_steps);     // already spent: elimination cannot undo it
    auto gp = [&](double nat_, double n_c_, double n_b_) {
        const double t = t_d + verify_time(*m, n_c_, n_b_);
        return t > tpot ? -1.0 : nat_ / t;
    };
    double best = gp(nat, n_c, n_b);
    for (;;) {
        int cand = -1;
        double lo = std::numeric_limits<double>::infinity();
        for (int i = 0; i < B; ++i) {
            const int k = spec_lens_out[i];
            if (k > 0 && ar[(int64_t)(k - 1) * B + i] < lo) { lo = ar[(int64_t)(k - 1) * B + i]; cand = i; }
        }
        if (cand < 0) break;
        const int k = spec_lens_out[cand];
        // dropping the last draft of `cand` removes position k + 1 (its context: C + k tokens, or the one
        // token it added to the request's cache when contexts count once) and one batch token
        const double nat2 = nat - lo, n_b2 = n_b - 1.0;
        const double n_c2 = n_c - (m->verify_ctx_once ? 1.0 : C[cand] + (double)k);
        const double g = gp(nat2, n_c2, n_b2);
        if (!(g > best)) break;
        best = g; nat = nat2; n_c = n_c2; n_b = n_b2;
        spec_lens_out[cand] = k - 1;
    }
    *goodput_out = best;
    return ADASPEC_OK;
}

int adaspec_policy_count_tokens(int32_t B, const int32_t *C, const int32_t *spec_lens, int32_t verify_ctx_once,
                                double *n_c, double *n_b)
{
    if (!n_c || !n_b || (B > 0 && (!C || !spec_lens))) return ADASPEC_ERR_NULL;
    if (B < 0) return ADASPEC_ERR_DIM;
    adaspec_time_model m = {};
    m.verify_ctx_once = verify_ctx_once ? 1 : 0;
    double c = 0.0, b = 0.0;
    for (int i = 0; i < B; ++i) {
        if (spec_lens[i] < 0 || C[i] < 0) return ADASPEC_ERR_DIM;
        c += verify_ctx(m, C[i], spec_lens[i]);
        b += spec_lens[i] + 1.0;
    }
    *n_c = c;
    *n_b = b;
    return ADASPEC_OK;
}

int adaspec_policy_fit_time_model(int32_t n, const double *n_c, const double *n_b, const double *t,
                                  double *alpha, double *gamma, double *delta)
{
    if (!n_c || !n_b || !t || !alpha || !gamma || !delta) return ADASPEC_ERR_NULL;
    if (n < 3) return ADASPEC_ERR_DIM;
    // normal equations of [n_c n_b 1] x = t, columns scaled to unit maximum for conditioning
    double sc = 0.0, sb = 0.0;
    for (int i = 0; i < n; ++i) { sc = fmax(sc, fabs(n_c[i])); sb = fmax(sb, fabs(n_b[i])); }
    if (sc == 0.0 || sb == 0.0) return ADASPEC_ERR_DIM;
    long double A[3][4] = {{0}};
    for (int i = 0; i < n; ++i) {
        const long double r[3] = {n_c[i] / sc, n_b[i] / sb, 1.0L};
        for (int a = 0; a < 3; ++a) {
            for (int b = 0; b < 3; ++b) A[a][b] += r[a] * r[b];
            A[a][3] += r[a] * t[i];
        }
    }
    for (int c = 0; c < 3; ++c) {        // Gaussian elimination with partial pivoting
        int p = c;
        for (int r = c + 1; r < 3; ++r) if (fabsl(A[r][c]) > fabsl(A[p][c])) p = r;
        if (fabsl(A[p][c]) < 1e-12L * n) return ADASPEC_ERR_DIM;
        for (int b = 0; b < 4; ++b) { const long double tmp = A[c][b]; A[c][b] = A[p][b]; A[p][b] = tmp; }
        for (int r = 0; r < 3; ++r) {
            if (r == c) continue;
            const long double f = A[r][c] / A[c][c];
            for (int b = c; b < 4; ++b) A[r][b] -= f * A[c][b];
        }
    }
    *alpha = (double)(A[0][3] / A[0][0]) / sc;
    *gamma = (double)(A[1][3] / A[1][1]) / sb;
    *delta = (double)(A[2][3] / A[2][2]);
    return ADASPEC_OK;
}

}  // extern "C"
