/*
 * CPU oracle for one ragged speculative-decoding verification step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * verification step computes; it exists so that the GPU library can be checked
 * against something written independently of it.  It shares no code, header,
 * table or helper with the GPU library, and nothing in the product path may
 * call it: only the test-suite, the smoke check and the benchmark's
 * cpu-baseline leg do.
 *
 * All arithmetic is IEEE double.  Inputs stored in 32/16-bit formats are
 * widened exactly.  No blocking, fusion or reordering: every loop is the
 * definition written out.  OpenMP only spreads independent (request, head)
 * pairs / requests over cores; each unit is computed sequentially.
 *
 * What the step is (paper Sec. 2.2): a draft model proposes y_1..y_SL, the
 * target model scores all SL+1 positions in one pass, position t conditioned on
 * the committed tokens and y_1..y_{t-1}; drafts are accepted left to right until
 * the first rejection, and one further token always comes from the target (the
 * "bonus" token, Sec. 4.2: AR_{i,0} = 1).  The paper's per-request draft lengths
 * (Alg. 2, Sec. 5.2) make the batch ragged: request i carries k_i drafts and
 * n_i = k_i + 1 query rows.  The stochastic accept/resample rule is the
 * speculative-sampling rule of the works the paper builds on (its refs for
 * "speculative decoding" in Sec. 1): accept x with probability min(1, p_x/q_x),
 * otherwise resample from the normalised positive part of p - q.
 *
 * Parity pins: see tests/test_oracle_*.py.  Every function below is pinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };

/* ---- exact widening of stored values ---------------------------------- */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, m = h & 0x3FF;
    double v;
    if (e == 0)        v = ldexp((double)m, -24);              /* subnormal / zero */
    else if (e == 31)  v = m ? NAN : INFINITY;
    else               v = ldexp((double)(m | 0x400), e - 25);
    return sign ? -v : v;
}

static double bf16_to_double(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double load(const void *base, int64_t idx, int dt)
{
    switch (dt) {
    case DT_F32:  return (double)((const float *)base)[idx];
    case DT_F16:  return half_to_double(((const uint16_t *)base)[idx]);
    default:      return bf16_to_double(((const uint16_t *)base)[idx]);
    }
}

/* ---- one round-to-nearest-even of a double into a storage format ------- */
/* sig = significand bits incl. the hidden one, emin = exponent of the smallest
 * normal, emax_val = largest finite value.  Result returned as a double. */
static double round_to_format(double x, int sig, int emin, double max_val)
{
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    int e;
    (void)frexp(x, &e);               /* |x| = f * 2^e, f in [0.5, 1) */
    int lsb = e - sig;                /* exponent of the last kept bit */
    if (lsb < emin - (sig - 1)) lsb = emin - (sig - 1);   /* subnormal range: fixed quantum */
    double r = ldexp(nearbyint(ldexp(x, -lsb)), lsb);     /* default mode: ties to even */
    if (fabs(r) > max_val) r = (x < 0) ? -INFINITY : INFINITY;
    return r;
}

static double round_to_dtype(double x, int dt)
{
    switch (dt) {
    case DT_F32:  return (double)(float)x;
    case DT_F16:  return round_to_format(x, 11, -14, 65504.0);
    default:      return round_to_format(x, 8, -126, 0x1.FEp127);
    }
}

/* Exposed for the tests that pin the rounding helper itself. */
double oracle_round_to_dtype(double x, int dt) { return round_to_dtype(x, dt); }
double oracle_widen_u16(uint16_t bits, int dt) { return dt == DT_F16 ? half_to_double(bits) : bf16_to_double(bits); }

/* =========================================================================
 * Ragged multi-query causal attention over a paged KV cache.
 *
 * Request i has n_i = spec_lens[i]+1 query rows (row 0 = last committed token,
 * rows 1..k_i = the drafts) and L_i = ctx_lens[i] cached tokens, the n_i new
 * ones included (their K/V are already in the pages).  Row j sits at position
 * pos = L_i - n_i + j and sees tokens 0..pos: everything committed, and the new
 * tokens up to itself (Sec. 2.2: the distribution for z_t conditions on
 * x_{1:n}, y_{1:t-1}; Eq. 4: the context count N_c(i) grows by one per position).
 * Token t of request i lives in page block_table[i][t / P], slot t % P; q head h
 * reads kv head h / G, G = Hq / Hkv.
 *
 *   s_t  = scale * <q_row, K_t>
 *   w_t  = exp(s_t - max_t s_t) / sum_t exp(s_t - max_t s_t)
 *   out  = sum_t w_t V_t
 *
 * out_f64   : [TQ][Hq][d] the double result.
 * out_round : same shape, each value rounded once (nearest-even) to `dtype`,
 *             held as a double; may be NULL.
 * Returns 0, or a negative code if the ragged metadata is inconsistent.
 * ======================================================================= */
int oracle_verify_attn(const void *q, const void *k_pages, const void *v_pages,
                       const int32_t *block_table, const int32_t *ctx_lens,
                       const int32_t *spec_lens, double *out_f64, double *out_round,
                       int batch, int n_q_heads, int n_kv_heads, int head_dim,
                       int page_size, int num_pages, int max_pages_per_req,
                       int dtype, double scale)
{
    if (n_kv_heads <= 0 || n_q_heads % n_kv_heads) return -2;
    const int G = n_q_heads / n_kv_heads, d = head_dim, P = page_size;
    if (scale == 0.0) scale = 1.0 / sqrt((double)d);

    int64_t *cu_q = (int64_t *)malloc(sizeof(int64_t) * (size_t)(batch + 1));
    cu_q[0] = 0;
    for (int i = 0; i < batch; ++i) {
        int n = spec_lens[i] + 1;
        if (spec_lens[i] < 0 || ctx_lens[i] < n) { free(cu_q); return -2; }
        if ((ctx_lens[i] + P - 1) / P > max_pages_per_req) { free(cu_q); return -2; }
        for (int pg = 0; pg < (ctx_lens[i] + P - 1) / P; ++pg) {
            int id = block_table[(int64_t)i * max_pages_per_req + pg];
            if (id < 0 || id >= num_pages) { free(cu_q); return -3; }
        }
        cu_q[i + 1] = cu_q[i] + n;
    }

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int i = 0; i < batch; ++i) {
        for (int h = 0; h < n_q_heads; ++h) {
            const int n = spec_lens[i] + 1, L = ctx_lens[i], g = h / G;
            double *s = (double *)malloc(sizeof(double) * (size_t)L);
            for (int j = 0; j < n; ++j) {
                const int pos = L - n + j;
                const int64_t qoff = ((cu_q[i] + j) * n_q_heads + h) * (int64_t)d;
                double smax = -INFINITY;
                for (int t = 0; t <= pos; ++t) {
                    const int64_t page = block_table[(int64_t)i * max_pages_per_req + t / P];
                    const int64_t koff = ((page * n_kv_heads + g) * P + t % P) * (int64_t)d;
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c)
                        dot += load(q, qoff + c, dtype) * load(k_pages, koff + c, dtype);
                    s[t] = scale * dot;
                    if (s[t] > smax) smax = s[t];
                }
                double denom = 0.0;
                for (int t = 0; t <= pos; ++t) {
                    s[t] = exp(s[t] - smax);
                    denom += s[t];
                }
                double *o = out_f64 + qoff;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int t = 0; t <= pos; ++t) {
                    const int64_t page = block_table[(int64_t)i * max_pages_per_req + t / P];
                    const int64_t voff = ((page * n_kv_heads + g) * P + t % P) * (int64_t)d;
                    const double w = s[t] / denom;
                    for (int c = 0; c < d; ++c)
                        o[c] += w * load(v_pages, voff + c, dtype);
                }
                if (out_round)
                    for (int c = 0; c < d; ++c)
                        out_round[qoff + c] = round_to_dtype(o[c], dtype);
            }
            free(s);
        }
    }
    free(cu_q);
    return 0;
}

/* =========================================================================
 * Acceptance: one logits row.
 *
 * logits : the target's row (V values), q_row : the draft distribution the
 * draft token x was sampled from, or NULL for a bonus row (no draft to judge:
 * the row is sampled from p itself, i.e. the residual with q == 0).
 *
 *   T == 0 (greedy, Sec. 2.2 / Fig. 1): z = argmax logits (lowest index on
 *     ties); accept iff x == z; the candidate token is z.
 *   T > 0: p = softmax(logits / T).  accept iff u0 < p_x / q_x (q_x == 0 counts
 *     as accept).  r_v = max(0, p_v - q_v), R = sum r_v; the candidate is the
 *     smallest t whose inclusive prefix sum of r exceeds u1 * R.  If R == 0
 *     (p == q everywhere) the candidate is drawn from p the same way.  Should
 *     rounding leave no such t, the last token with positive mass is taken.
 *
 * res[0] = accept flag (1/0; 1 for a bonus row), res[1] = p_x/q_x (NaN if not
 * defined), res[2] = candidate token, res[3] = R (mass the candidate was drawn
 * from), res[4] = prefix sum just before the candidate, res[5] = prefix sum
 * including it.
 * ======================================================================= */
void oracle_accept_row(const void *logits, int ldt, const void *q_row, int qdt,
                       int V, double T, int x, double u0, double u1, double *res)
{
    res[1] = NAN; res[3] = NAN; res[4] = NAN; res[5] = NAN;
    if (T == 0.0) {
        int z = 0;
        double best = load(logits, 0, ldt);
        for (int v = 1; v < V; ++v) {
            double l = load(logits, v, ldt);
            if (l > best) { best = l; z = v; }
        }
        res[0] = (q_row == NULL) ? 1.0 : (double)(x == z);
        res[2] = (double)z;
        return;
    }
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double m = -INFINITY, Z = 0.0;
    for (int v = 0; v < V; ++v) { p[v] = load(logits, v, ldt); if (p[v] > m) m = p[v]; }
    for (int v = 0; v < V; ++v) { p[v] = exp((p[v] - m) / T); Z += p[v]; }
    for (int v = 0; v < V; ++v) p[v] /= Z;

    if (q_row) {
        double qx = load(q_row, x, qdt);
        double ratio = (qx > 0.0) ? p[x] / qx : INFINITY;
        res[0] = (double)(u0 < ratio);
        res[1] = ratio;
    } else {
        res[0] = 1.0;
    }

    /* residual mass; for a bonus row q == 0 so r == p */
    double R = 0.0;
    double *r = (double *)malloc(sizeof(double) * (size_t)V);
    for (int v = 0; v < V; ++v) {
        double qv = q_row ? load(q_row, v, qdt) : 0.0;
        r[v] = p[v] - qv;
        if (r[v] < 0.0) r[v] = 0.0;
        R += r[v];
    }
    if (!(R > 0.0)) {                 /* p == q: fall back to p */
        R = 0.0;
        for (int v = 0; v < V; ++v) { r[v] = p[v]; R += r[v]; }
    }
    const double thr = u1 * R;
    double c = 0.0, before = 0.0;
    int cand = -1, last_pos = 0;
    for (int v = 0; v < V; ++v) {
        before = c;
        c += r[v];
        if (r[v] > 0.0) last_pos = v;
        if (c > thr) { cand = v; break; }
    }
    if (cand < 0) {                   /* rounding left no crossing */
        cand = last_pos;
        c = 0.0;
        for (int v = 0; v < cand; ++v) c += r[v];
        before = c; c += r[cand];
    }
    res[2] = (double)cand; res[3] = R; res[4] = before; res[5] = c;
    free(r);
    free(p);
}

/* Inclusive-prefix interval [lo, hi) that token t owns in the row's sampling
 * mass (same r as above) and the total R: used by the tests to decide whether a
 * disagreement on a sampled token is a rounding near-tie. */
void oracle_cdf_interval(const void *logits, int ldt, const void *q_row, int qdt,
                         int V, double T, int t, double *lo, double *hi, double *R_out)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)V);
    double m = -INFINITY, Z = 0.0;
    for (int v = 0; v < V; ++v) { p[v] = load(logits, v, ldt); if (p[v] > m) m = p[v]; }
    for (int v = 0; v < V; ++v) { p[v] = exp((p[v] - m) / T); Z += p[v]; }
    double R = 0.0;
    for (int v = 0; v < V; ++v) {
        double qv = q_row ? load(q_row, v, qdt) : 0.0;
        double rv = p[v] / Z - qv;
        p[v] = rv > 0.0 ? rv : 0.0;
        R += p[v];
    }
    double c = 0.0;
    for (int v = 0; v < t; ++v) c += p[v];
    *lo = c; *hi = c + p[t]; *R_out = R;
    free(p);
}

/* =========================================================================
 * Acceptance over the ragged batch, in the order the method states it.
 *
 * target_logits [TQ][V] (row stride given): request i owns rows cu_q[i] ..
 *   cu_q[i]+k_i; row j judges draft j, row k_i is the bonus row.
 * draft_probs   [TD][V]: request i owns rows cu_q[i]-i ..; draft_tokens [TD].
 * uniforms      [TQ][2]: [r][0] accept test, [r][1] inverse-CDF draw.
 * out_tokens    [B][out_stride]: accepted drafts, then the recovered/bonus
 *   token, then -1 padding.  out_accept_len[i] = number of accepted drafts.
 * row_info      [TQ][6] or NULL: oracle_accept_row's res[] for every row the
 *   sequential procedure visited, NaN for rows after the first rejection.
 * ======================================================================= */
int oracle_accept(const void *target_logits, const void *draft_probs,
                  const int32_t *draft_tokens, const float *uniforms,
                  const int32_t *spec_lens, const float *temperature,
                  int32_t *out_tokens, int32_t *out_accept_len, double *row_info,
                  int batch, int vocab, int logits_dtype, int probs_dtype,
                  int64_t logits_row_stride, int64_t probs_row_stride, int out_stride)
{
    int64_t *cu_q = (int64_t *)malloc(sizeof(int64_t) * (size_t)(batch + 1));
    cu_q[0] = 0;
    int kmax = 0;
    for (int i = 0; i < batch; ++i) {
        if (spec_lens[i] < 0) { free(cu_q); return -2; }
        if (spec_lens[i] > kmax) kmax = spec_lens[i];
        cu_q[i + 1] = cu_q[i] + spec_lens[i] + 1;
    }
    if (out_stride < kmax + 1) { free(cu_q); return -2; }
    const int lsz = logits_dtype == DT_F32 ? 4 : 2, psz = probs_dtype == DT_F32 ? 4 : 2;
    if (row_info)
        for (int64_t r = 0; r < cu_q[batch] * 6; ++r) row_info[r] = NAN;

#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < batch; ++i) {
        const int k = spec_lens[i];
        const double T = (double)temperature[i];
        int32_t *out = out_tokens + (int64_t)i * out_stride;
        for (int s = 0; s < out_stride; ++s) out[s] = -1;
        int emitted = 0, done = 0;
        for (int j = 0; j < k && !done; ++j) {
            const int64_t r = cu_q[i] + j, dr = cu_q[i] - i + j;
            const int x = draft_tokens[dr];
            double res[6];
            oracle_accept_row((const char *)target_logits + r * logits_row_stride * lsz, logits_dtype,
                              (const char *)draft_probs + dr * probs_row_stride * psz, probs_dtype,
                              vocab, T, x, (double)uniforms[2 * r], (double)uniforms[2 * r + 1], res);
            if (row_info) memcpy(row_info + 6 * r, res, sizeof res);
            if (res[0] != 0.0) {
                out[emitted++] = x;                    /* draft accepted */
            } else {
                out[emitted++] = (int32_t)res[2];      /* first rejection: recovered token, stop */
                out_accept_len[i] = j;
                done = 1;
            }
        }
        if (!done) {                                   /* every draft accepted (or k == 0): bonus token */
            const int64_t r = cu_q[i] + k;
            double res[6];
            oracle_accept_row((const char *)target_logits + r * logits_row_stride * lsz, logits_dtype,
                              NULL, probs_dtype, vocab, T, -1,
                              (double)uniforms[2 * r], (double)uniforms[2 * r + 1], res);
            if (row_info) memcpy(row_info + 6 * r, res, sizeof res);
            out[emitted++] = (int32_t)res[2];
            out_accept_len[i] = k;
        }
    }
    free(cu_q);
    return 0;
}

/* =========================================================================
 * Draft-side sampling (paper Eq. 6: confidence scores c_{i,k}; Alg. 1: each run
 * of the draft model returns draft tokens and their confidences).
 *
 * One row of draft logits, temperature T, one uniform u:
 *   T > 0 : p = softmax(l / T); q_v = p_v rounded once to the storage type qdt;
 *           token = smallest t with sum_{v<=t} q_v > u * sum_v q_v (sums over the
 *           ROUNDED values, so a zero-probability token is never drawn; if
 *           rounding leaves no crossing, the last token with q > 0);
 *   T == 0: token = argmax l (lowest index on ties); q = softmax(l) at T = 1, rounded;
 *   confidence = q[token].
 * out_q [V]: the rounded row as doubles.
 * res[0] = token, res[1] = confidence, res[2] = Q = sum q, res[3] = prefix sum
 * before the token, res[4] = prefix sum including it (res[3..4] NaN if T == 0).
 * ======================================================================= */
void oracle_draft_sample_row(const void *logits, int ldt, int V, double T, double u, int qdt,
                             double *out_q, double *res)
{
    int z = 0;
    double m = load(logits, 0, ldt);
    for (int v = 1; v < V; ++v) {
        double l = load(logits, v, ldt);
        if (l > m) { m = l; z = v; }
    }
    const double temp = (T == 0.0) ? 1.0 : T;
    double Z = 0.0;
    for (int v = 0; v < V; ++v) { out_q[v] = exp((load(logits, v, ldt) - m) / temp); Z += out_q[v]; }
    double Q = 0.0;
    for (int v = 0; v < V; ++v) { out_q[v] = round_to_dtype(out_q[v] / Z, qdt); Q += out_q[v]; }
    res[2] = Q; res[3] = NAN; res[4] = NAN;
    if (T == 0.0) {
        res[0] = (double)z; res[1] = out_q[z];
        return;
    }
    const double thr = u * Q;
    double c = 0.0, before = 0.0;
    int cand = -1, last_pos = 0;
    for (int v = 0; v < V; ++v) {
        before = c;
        c += out_q[v];
        if (out_q[v] > 0.0) last_pos = v;
        if (c > thr) { cand = v; break; }
    }
    if (cand < 0) {
        cand = last_pos;
        c = 0.0;
        for (int v = 0; v < cand; ++v) c += out_q[v];
        before = c; c += out_q[cand];
    }
    res[0] = (double)cand; res[1] = out_q[cand]; res[3] = before; res[4] = c;
}

/* All rows: out_q [R][V] doubles, tokens [R], conf [R] doubles, info [R][5] = res of every row. */
int oracle_draft_sample(const void *logits, int ldt, int64_t lstride, int R, int V,
                        const float *temperature, const float *uniforms, int qdt,
                        double *out_q, int32_t *tokens, double *conf, double *info)
{
    const size_t esz = (ldt == DT_F32) ? 4 : 2;
#pragma omp parallel for schedule(dynamic)
    for (int r = 0; r < R; ++r) {
        double res[5];
        oracle_draft_sample_row((const char *)logits + (size_t)r * (size_t)lstride * esz, ldt, V,
                                (double)temperature[r], (double)uniforms[r], qdt,
                                out_q + (size_t)r * (size_t)V, res);
        tokens[r] = (int32_t)res[0];
        conf[r] = res[1];
        if (info) memcpy(info + (size_t)r * 5, res, sizeof(res));
    }
    return 0;
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    n = omp_get_max_threads();
#endif
    return n;
}

/* Limits the OpenMP team of later calls (n >= 1); used to time the single-thread baseline. */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    extern void omp_set_num_threads(int);
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
