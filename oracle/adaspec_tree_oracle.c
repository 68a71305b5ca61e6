/*
 * CPU oracle for verification of a draft-token TREE (width > 1).
 *
 * TEST INFRASTRUCTURE ONLY, like adaspec_oracle.c: the slow, plain statement of
 * what tree verification computes, in IEEE double, sharing nothing with the GPU
 * library.  Only the test-suite, the smoke check and the benchmark's
 * cpu-baseline leg may call it.
 *
 * Where this comes from.  The paper verifies one chain of drafts per request
 * and, in its evaluation (Sec. 7.1, baselines), runs the tree-based system it
 * compares with at tree width 1; its related work (Sec. 8) names tree-based
 * speculative decoding as the other family.  The paper therefore fixes the
 * chain case only.  The tree case below is the published token-tree
 * verification of that baseline system, restated: the target scores every node
 * of the tree in one pass, each node seeing the committed context and its own
 * ancestors; acceptance walks down from the root, trying the children of the
 * current node one after another with the speculative-sampling test, and after
 * every rejection replaces the target distribution by the normalised positive
 * part of (distribution - draft distribution).  Children of a node are taken to
 * be independent draws from that node's draft distribution.  With every node
 * having at most one child the procedure IS the chain procedure of
 * adaspec_oracle.c, step for step; the tests pin that, the exactness of the
 * emitted distribution, and the greedy form.
 *
 * Layout.  Request i has n_i = spec_lens[i] + 1 nodes, rows cu_q[i] .. of the
 * ragged row space: node 0 is the root (the last committed token), nodes
 * 1..k_i are drafts in an order in which every parent precedes its children.
 * parents[row] is the parent's index INSIDE the request (-1 for the root).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { DT_F32 = 0, DT_F16 = 1, DT_BF16 = 2 };

static double widen_half(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1F, m = h & 0x3FF;
    double v;
    if (e == 0)        v = ldexp((double)m, -24);
    else if (e == 31)  v = m ? NAN : INFINITY;
    else               v = ldexp((double)(m | 0x400), e - 25);
    return sign ? -v : v;
}

static double widen_bf16(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

static double value_at(const void *base, int64_t idx, int dt)
{
    switch (dt) {
    case DT_F32:  return (double)((const float *)base)[idx];
    case DT_F16:  return widen_half(((const uint16_t *)base)[idx]);
    default:      return widen_bf16(((const uint16_t *)base)[idx]);
    }
}

/* nearest-even rounding of a double into one of the storage formats (as a double) */
static double round_once(double x, int dt)
{
    if (dt == DT_F32) return (double)(float)x;
    if (x == 0.0 || isnan(x) || isinf(x)) return x;
    const int sig = dt == DT_F16 ? 11 : 8, emin = dt == DT_F16 ? -14 : -126;
    const double max_val = dt == DT_F16 ? 65504.0 : 0x1.FEp127;
    int e;
    (void)frexp(x, &e);
    int lsb = e - sig;
    if (lsb < emin - (sig - 1)) lsb = emin - (sig - 1);
    double r = ldexp(nearbyint(ldexp(x, -lsb)), lsb);
    if (fabs(r) > max_val) r = (x < 0) ? -INFINITY : INFINITY;
    return r;
}

/* 1 if the parent array of a request with n nodes is a tree in parent-first order */
static int tree_ok(const int32_t *par, int n)
{
    if (n < 1 || par[0] != -1) return 0;
    for (int j = 1; j < n; ++j)
        if (par[j] < 0 || par[j] >= j) return 0;
    return 1;
}

/* =========================================================================
 * Tree attention.  Node j of request i has its K/V at cache position
 * L_i - n_i + j (the nodes are appended in node order).  Its query row sees
 * the committed tokens 0 .. L_i - n_i - 1 and, of the n_i new positions, those
 * of its ancestors and its own:
 *     visible(j, t) = t < L_i - n_i  or  node (t - (L_i - n_i)) is j or an ancestor of j
 * Everything else is as in the chain case (softmax over the visible tokens of
 * scale * <q, K_t>, weighted sum of V_t; q head h reads kv head h / G).
 * out_f64 / out_round as in oracle_verify_attn.  Returns 0 or a negative code.
 * ======================================================================= */
int oracle_verify_attn_tree(const void *q, const void *k_pages, const void *v_pages,
                            const int32_t *block_table, const int32_t *ctx_lens,
                            const int32_t *spec_lens, const int32_t *parents,
                            double *out_f64, double *out_round,
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
        const int n = spec_lens[i] + 1;
        if (spec_lens[i] < 0 || ctx_lens[i] < n) { free(cu_q); return -2; }
        if ((ctx_lens[i] + P - 1) / P > max_pages_per_req) { free(cu_q); return -2; }
        for (int pg = 0; pg < (ctx_lens[i] + P - 1) / P; ++pg) {
            const int id = block_table[(int64_t)i * max_pages_per_req + pg];
            if (id < 0 || id >= num_pages) { free(cu_q); return -3; }
        }
        if (!tree_ok(parents + cu_q[i], n)) { free(cu_q); return -4; }
        cu_q[i + 1] = cu_q[i] + n;
    }

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int i = 0; i < batch; ++i) {
        for (int h = 0; h < n_q_heads; ++h) {
            const int n = spec_lens[i] + 1, L = ctx_lens[i], g = h / G, base = L - n;
            const int32_t *par = parents + cu_q[i];
            double *s = (double *)malloc(sizeof(double) * (size_t)L);
            char *vis = (char *)malloc((size_t)L);
            for (int j = 0; j < n; ++j) {
                for (int t = 0; t < L; ++t) vis[t] = t < base;
                for (int a = j; a >= 0; a = par[a]) vis[base + a] = 1;   /* j and its ancestors */
                const int64_t qoff = ((cu_q[i] + j) * n_q_heads + h) * (int64_t)d;
                double smax = -INFINITY;
                for (int t = 0; t < L; ++t) {
                    if (!vis[t]) continue;
                    const int64_t page = block_table[(int64_t)i * max_pages_per_req + t / P];
                    const int64_t koff = ((page * n_kv_heads + g) * P + t % P) * (int64_t)d;
                    double dot = 0.0;
                    for (int c = 0; c < d; ++c)
                        dot += value_at(q, qoff + c, dtype) * value_at(k_pages, koff + c, dtype);
                    s[t] = scale * dot;
                    if (s[t] > smax) smax = s[t];
                }
                double denom = 0.0;
                for (int t = 0; t < L; ++t) {
                    if (!vis[t]) continue;
                    s[t] = exp(s[t] - smax);
                    denom += s[t];
                }
                double *o = out_f64 + qoff;
                for (int c = 0; c < d; ++c) o[c] = 0.0;
                for (int t = 0; t < L; ++t) {
                    if (!vis[t]) continue;
                    const int64_t page = block_table[(int64_t)i * max_pages_per_req + t / P];
                    const int64_t voff = ((page * n_kv_heads + g) * P + t % P) * (int64_t)d;
                    const double w = s[t] / denom;
                    for (int c = 0; c < d; ++c)
                        o[c] += w * value_at(v_pages, voff + c, dtype);
                }
                if (out_round)
                    for (int c = 0; c < d; ++c)
                        out_round[qoff + c] = round_once(o[c], dtype);
            }
            free(vis);
            free(s);
        }
    }
    free(cu_q);
    return 0;
}

/* =========================================================================
 * The sampling state of one node: the current target-side distribution after
 * some number of rejected children.
 *
 *   stage 0:  P = softmax(logits / T)
 *   one more rejection:  r_v = max(0, P_v - q_v),  R = sum_v r_v;
 *                        if R == 0 (P == q everywhere) r = P and R = sum_v P_v;
 *                        then P = r / R
 * A token is DRAWN from the state's last unnormalised mass (r, R): the smallest
 * t whose inclusive prefix sum of r exceeds u * R (at stage 0: r = P, R = sum P).
 * ======================================================================= */
typedef struct {
    int V;
    double *P;      /* normalised distribution the next child is tested against */
    double *r;      /* unnormalised mass a token is drawn from                   */
    double R;       /* its total                                                 */
} node_state;

static void state_init(node_state *s, const void *logits, int ldt, int V, double T)
{
    s->V = V;
    s->P = (double *)malloc(sizeof(double) * (size_t)V);
    s->r = (double *)malloc(sizeof(double) * (size_t)V);
    double m = -INFINITY, Z = 0.0;
    for (int v = 0; v < V; ++v) { s->P[v] = value_at(logits, v, ldt); if (s->P[v] > m) m = s->P[v]; }
    for (int v = 0; v < V; ++v) { s->P[v] = exp((s->P[v] - m) / T); Z += s->P[v]; }
    s->R = 0.0;
    for (int v = 0; v < V; ++v) { s->P[v] /= Z; s->r[v] = s->P[v]; s->R += s->r[v]; }
}

static void state_reject(node_state *s, const void *q_row, int qdt)
{
    double R = 0.0;
    for (int v = 0; v < s->V; ++v) {
        double rv = s->P[v] - value_at(q_row, v, qdt);
        s->r[v] = rv > 0.0 ? rv : 0.0;
        R += s->r[v];
    }
    if (!(R > 0.0)) {
        R = 0.0;
        for (int v = 0; v < s->V; ++v) { s->r[v] = s->P[v]; R += s->r[v]; }
    }
    s->R = R;
    for (int v = 0; v < s->V; ++v) s->P[v] = s->r[v] / R;
}

/* draw: token, prefix sum before it, prefix sum including it */
static int state_draw(const node_state *s, double u, double *before_out, double *incl_out)
{
    const double thr = u * s->R;
    double c = 0.0, before = 0.0;
    int cand = -1, last_pos = 0;
    for (int v = 0; v < s->V; ++v) {
        before = c;
        c += s->r[v];
        if (s->r[v] > 0.0) last_pos = v;
        if (c > thr) { cand = v; break; }
    }
    if (cand < 0) {                   /* rounding left no crossing: last token with mass */
        cand = last_pos;
        c = 0.0;
        for (int v = 0; v < cand; ++v) c += s->r[v];
        before = c; c += s->r[cand];
    }
    *before_out = before; *incl_out = c;
    return cand;
}

static void state_free(node_state *s) { free(s->P); free(s->r); }

static int argmax_low(const void *logits, int ldt, int V)
{
    int z = 0;
    double best = value_at(logits, 0, ldt);
    for (int v = 1; v < V; ++v) {
        double l = value_at(logits, v, ldt);
        if (l > best) { best = l; z = v; }
    }
    return z;
}

/* Interval [lo, hi) that token t owns in the mass a node draws from after `rejections`
 * rejected children, and that mass's total: lets the tests tell a rounding near-tie from an
 * error when two implementations draw different tokens.  q_row may be NULL if rejections == 0. */
void oracle_tree_cdf_interval(const void *logits, int ldt, const void *q_row, int qdt, int V,
                              double T, int rejections, int t, double *lo, double *hi, double *R_out)
{
    node_state s;
    state_init(&s, logits, ldt, V, T);
    for (int m = 0; m < rejections; ++m) state_reject(&s, q_row, qdt);
    double c = 0.0;
    for (int v = 0; v < t; ++v) c += s.r[v];
    *lo = c; *hi = c + s.r[t]; *R_out = s.R;
    state_free(&s);
}

/* =========================================================================
 * Tree acceptance over the ragged batch.
 *
 * target_logits [TQ][V]: row of node j = the target's logits for the token that
 *   follows node j (given the path from the root to j).
 * draft_probs   [TD][V]: request i owns rows cu_q[i]-i ..; row j (j = 0..k_i-1)
 *   is the draft distribution AT node j, from which the tokens of node j's
 *   children were drawn.  The last node of a request cannot have children (a
 *   parent precedes its children), so it has no row.  Rows of other childless
 *   nodes are not read.
 * draft_tokens  [TD]: row j-1 of the request = token of node j (j >= 1).
 * uniforms      [TQ][2]: the accept test of node c (c >= 1) uses [cu_q[i]+c-1][0];
 *   the draw at the node where the walk stops uses [cu_q[i]+u][1].
 *
 * Walk of request i, temperature T, starting at u = 0:
 *   children of u in ascending node order, c_1 < c_2 < ...
 *   T == 0: z = argmax logits_u (lowest index on ties).  The first child whose
 *           token is z is accepted (u = that child, continue); if none, emit z, stop.
 *   T > 0 : state = stage 0 of node u.  For each child c with token x:
 *             ratio = P_x / q_u[x]  (q_u[x] == 0 counts as accept);
 *             accept iff u0 < ratio -> emit x, u = c, continue the walk;
 *             else the state takes one more rejection (q = q_u).
 *           No child accepted (or none exists): emit a token drawn from the
 *           state with this node's u1, stop.
 *
 * out_tokens [B][out_stride]: tokens of the accepted nodes in path order, then the
 *   token emitted at the stop, then -1.   out_accept_len[i] = accepted nodes a_i.
 * out_path   [B][out_stride]: node indices of the accepted nodes (path order), then -1.
 * test_info  [TQ][2] or NULL: for node c, row cu_q[i]+c: {ratio of its test, rejections
 *   before it}; NaN where the walk did not test the node (and for T == 0).
 * stop_info  [B][5] or NULL: {stop node, rejections at it, R, prefix before the emitted
 *   token, prefix including it} (last three NaN for T == 0).
 * ======================================================================= */
int oracle_accept_tree(const void *target_logits, const void *draft_probs,
                       const int32_t *draft_tokens, const int32_t *parents,
                       const float *uniforms, const int32_t *spec_lens, const float *temperature,
                       int32_t *out_tokens, int32_t *out_accept_len, int32_t *out_path,
                       double *test_info, double *stop_info,
                       int batch, int vocab, int logits_dtype, int probs_dtype,
                       int64_t logits_row_stride, int64_t probs_row_stride, int out_stride)
{
    int64_t *cu_q = (int64_t *)malloc(sizeof(int64_t) * (size_t)(batch + 1));
    cu_q[0] = 0;
    int kmax = 0;
    for (int i = 0; i < batch; ++i) {
        if (spec_lens[i] < 0) { free(cu_q); return -2; }
        if (!tree_ok(parents + cu_q[i], spec_lens[i] + 1)) { free(cu_q); return -4; }
        if (spec_lens[i] > kmax) kmax = spec_lens[i];
        cu_q[i + 1] = cu_q[i] + spec_lens[i] + 1;
    }
    if (out_stride < kmax + 1) { free(cu_q); return -2; }
    const int lsz = logits_dtype == DT_F32 ? 4 : 2, psz = probs_dtype == DT_F32 ? 4 : 2;
    if (test_info)
        for (int64_t r = 0; r < cu_q[batch] * 2; ++r) test_info[r] = NAN;

#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < batch; ++i) {
        const int k = spec_lens[i], n = k + 1;
        const double T = (double)temperature[i];
        const int32_t *par = parents + cu_q[i];
        int32_t *out = out_tokens + (int64_t)i * out_stride;
        int32_t *path = out_path + (int64_t)i * out_stride;
        for (int s = 0; s < out_stride; ++s) { out[s] = -1; path[s] = -1; }
        int u = 0, depth = 0;
        for (;;) {
            const char *lrow = (const char *)target_logits + (cu_q[i] + u) * logits_row_stride * lsz;
            const char *qrow = (const char *)draft_probs + (cu_q[i] - i + u) * probs_row_stride * psz;
            int next = -1, rejections = 0;
            if (T == 0.0) {
                const int z = argmax_low(lrow, logits_dtype, vocab);
                for (int c = u + 1; c < n && next < 0; ++c)
                    if (par[c] == u && draft_tokens[cu_q[i] - i + c - 1] == z) next = c;
                if (next < 0) {
                    out[depth] = z;
                    if (stop_info) {
                        double *si = stop_info + 5 * (int64_t)i;
                        si[0] = u; si[1] = 0; si[2] = NAN; si[3] = NAN; si[4] = NAN;
                    }
                }
            } else {
                node_state st;
                state_init(&st, lrow, logits_dtype, vocab, T);
                for (int c = u + 1; c < n && next < 0; ++c) {
                    if (par[c] != u) continue;
                    const int x = draft_tokens[cu_q[i] - i + c - 1];
                    const double qx = value_at(qrow, x, probs_dtype);
                    const double ratio = (qx > 0.0) ? st.P[x] / qx : INFINITY;
                    if (test_info) {
                        test_info[2 * (cu_q[i] + c)] = ratio;
                        test_info[2 * (cu_q[i] + c) + 1] = rejections;
                    }
                    if ((double)uniforms[2 * (cu_q[i] + c - 1)] < ratio) next = c;
                    else { state_reject(&st, qrow, probs_dtype); ++rejections; }
                }
                if (next < 0) {
                    double before, incl;
                    out[depth] = state_draw(&st, (double)uniforms[2 * (cu_q[i] + u) + 1], &before, &incl);
                    if (stop_info) {
                        double *si = stop_info + 5 * (int64_t)i;
                        si[0] = u; si[1] = rejections; si[2] = st.R; si[3] = before; si[4] = incl;
                    }
                }
                state_free(&st);
            }
            if (next < 0) break;
            out[depth] = draft_tokens[cu_q[i] - i + next - 1];
            path[depth] = next;
            ++depth;
            u = next;
        }
        out_accept_len[i] = depth;
    }
    free(cu_q);
    return 0;
}
