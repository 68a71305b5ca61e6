/* Driver for the sanitizer build of the host code (the CPU oracle's C files and the policy's
 * host C++): reads the inputs tests/test_host_sanitizers.py wrote into a directory, calls every
 * entry point once, writes the results back.  Built with -fsanitize=address,undefined; any report
 * of either sanitizer ends the process with a non-zero status. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "adaspec_policy.h"

int oracle_verify_attn(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                       const int32_t *ctx_lens, const int32_t *spec_lens, double *out_f64, double *out_round,
                       int batch, int n_q_heads, int n_kv_heads, int head_dim, int page_size, int num_pages,
                       int max_pages_per_req, int dtype, double scale);
int oracle_verify_attn_tree(const void *q, const void *k_pages, const void *v_pages, const int32_t *block_table,
                            const int32_t *ctx_lens, const int32_t *spec_lens, const int32_t *parents,
                            double *out_f64, double *out_round, int batch, int n_q_heads, int n_kv_heads,
                            int head_dim, int page_size, int num_pages, int max_pages_per_req, int dtype,
                            double scale);
int oracle_accept(const void *target_logits, const void *draft_probs, const int32_t *draft_tokens,
                  const float *uniforms, const int32_t *spec_lens, const float *temperature, int32_t *out_tokens,
                  int32_t *out_accept_len, double *row_info, int batch, int vocab, int logits_dtype,
                  int probs_dtype, int64_t logits_row_stride, int64_t probs_row_stride, int out_stride);
int oracle_accept_tree(const void *target_logits, const void *draft_probs, const int32_t *draft_tokens,
                       const int32_t *parents, const float *uniforms, const int32_t *spec_lens,
                       const float *temperature, int32_t *out_tokens, int32_t *out_accept_len, int32_t *out_path,
                       double *test_info, double *stop_info, int batch, int vocab, int logits_dtype,
                       int probs_dtype, int64_t logits_row_stride, int64_t probs_row_stride, int out_stride);
int oracle_draft_sample(const void *logits, int ldt, int64_t lstride, int R, int V, const float *temperature,
                        const float *uniforms, int qdt, double *out_q, int32_t *tokens, double *conf, double *info);

static char g_dir[4096];

static void *read_file(const char *name, size_t *bytes)
{
    char path[4400];
    snprintf(path, sizeof path, "%s/%s.bin", g_dir, name);
    FILE *f = fopen(path, "rb");
    if (!f) { fprintf(stderr, "cannot open %s\n", path); exit(3); }
    fseek(f, 0, SEEK_END);
    long n = ftell(f);
    fseek(f, 0, SEEK_SET);
    void *p = malloc(n > 0 ? (size_t)n : 1);           /* exact size: an over-read is an ASan report */
    if (n > 0 && fread(p, 1, (size_t)n, f) != (size_t)n) { fprintf(stderr, "short read %s\n", path); exit(3); }
    fclose(f);
    if (bytes) *bytes = (size_t)n;
    return p;
}

static void write_file(const char *name, const void *p, size_t bytes)
{
    char path[4400];
    snprintf(path, sizeof path, "%s/%s.bin", g_dir, name);
    FILE *f = fopen(path, "wb");
    if (!f || fwrite(p, 1, bytes, f) != bytes) { fprintf(stderr, "cannot write %s\n", path); exit(3); }
    fclose(f);
}

int main(int argc, char **argv)
{
    if (argc != 2) { fprintf(stderr, "usage: %s <dir>\n", argv[0]); return 2; }
    snprintf(g_dir, sizeof g_dir, "%s", argv[1]);
    /* dims: B TQ Hq Hkv d P num_pages max_pages dtype V ldt qdt out_stride max_steps */
    int32_t *dm = read_file("dims", NULL);
    const int B = dm[0], TQ = dm[1], Hq = dm[2], Hkv = dm[3], d = dm[4], P = dm[5], num_pages = dm[6],
              max_pages = dm[7], dtype = dm[8], V = dm[9], ldt = dm[10], qdt = dm[11], out_stride = dm[12],
              max_steps = dm[13];
    void *q = read_file("q", NULL), *kp = read_file("k_pages", NULL), *vp = read_file("v_pages", NULL);
    int32_t *bt = read_file("block_table", NULL), *ctx = read_file("ctx_lens", NULL), *spec = read_file("spec_lens", NULL);
    int32_t *parents = read_file("parents", NULL), *tree_tokens = read_file("tree_draft_tokens", NULL);
    void *logits = read_file("target_logits", NULL), *probs = read_file("draft_probs", NULL);
    int32_t *toks = read_file("draft_tokens", NULL);
    float *uni = read_file("uniforms", NULL), *temp = read_file("temperature", NULL);
    int rc;

    const size_t n_out = (size_t)TQ * Hq * d;
    double *o64 = malloc(n_out * 8), *ord = malloc(n_out * 8);
    rc = oracle_verify_attn(q, kp, vp, bt, ctx, spec, o64, ord, B, Hq, Hkv, d, P, num_pages, max_pages, dtype, 0.0);
    if (rc) { fprintf(stderr, "oracle_verify_attn %d\n", rc); return 4; }
    write_file("out_attn", o64, n_out * 8);
    write_file("out_attn_rounded", ord, n_out * 8);
    rc = oracle_verify_attn_tree(q, kp, vp, bt, ctx, spec, parents, o64, ord, B, Hq, Hkv, d, P, num_pages, max_pages,
                                 dtype, 0.0);
    if (rc) { fprintf(stderr, "oracle_verify_attn_tree %d\n", rc); return 4; }
    write_file("out_attn_tree", o64, n_out * 8);

    int32_t *otok = malloc((size_t)B * out_stride * 4), *olen = malloc((size_t)B * 4), *opath = malloc((size_t)B * out_stride * 4);
    double *info = malloc((size_t)TQ * 6 * 8);
    rc = oracle_accept(logits, probs, toks, uni, spec, temp, otok, olen, info, B, V, ldt, qdt, V, V, out_stride);
    if (rc) { fprintf(stderr, "oracle_accept %d\n", rc); return 4; }
    write_file("out_tokens", otok, (size_t)B * out_stride * 4);
    write_file("out_accept_len", olen, (size_t)B * 4);
    double *tinfo = malloc((size_t)TQ * 2 * 8), *sinfo = malloc((size_t)B * 5 * 8);
    rc = oracle_accept_tree(logits, probs, tree_tokens, parents, uni, spec, temp, otok, olen, opath, tinfo, sinfo, B, V,
                            ldt, qdt, V, V, out_stride);
    if (rc) { fprintf(stderr, "oracle_accept_tree %d\n", rc); return 4; }
    write_file("out_tree_tokens", otok, (size_t)B * out_stride * 4);
    write_file("out_tree_accept_len", olen, (size_t)B * 4);
    write_file("out_tree_path", opath, (size_t)B * out_stride * 4);

    /* draft sampling on the first B logits rows (one per request), the call's own uniforms */
    float *du = malloc((size_t)B * 4);
    for (int i = 0; i < B; ++i) du[i] = uni[2 * i + 1];
    double *dq = malloc((size_t)B * V * 8), *dconf = malloc((size_t)B * 8);
    int32_t *dtok = malloc((size_t)B * 4);
    rc = oracle_draft_sample(logits, ldt, V, B, V, temp, du, qdt, dq, dtok, dconf, NULL);
    if (rc) { fprintf(stderr, "oracle_draft_sample %d\n", rc); return 4; }
    write_file("out_draft_q", dq, (size_t)B * V * 8);
    write_file("out_draft_tokens", dtok, (size_t)B * 4);

    /* the policy's host code */
    adaspec_time_model *m = read_file("time_model", NULL);
    int32_t *C = read_file("ctx_committed", NULL);
    double *conf = read_file("conf", NULL);
    double res[8] = {0};
    int32_t steps = 0;
    double *ar = malloc((size_t)max_steps * B * 8);
    double g = 0.0;
    rc = adaspec_policy_adaptive_draft(m, B, C, conf, max_steps, 0.7, 1e30, &steps, ar, &g);
    if (rc) { fprintf(stderr, "adaptive_draft %d\n", rc); return 4; }
    int32_t *kout = malloc((size_t)B * 4);
    double g2 = 0.0;
    rc = adaspec_policy_eliminate(m, B, C, steps, ar, 1e30, kout, &g2);
    if (rc) { fprintf(stderr, "eliminate %d\n", rc); return 4; }
    res[0] = steps; res[1] = g; res[2] = g2;
    res[3] = adaspec_policy_estimate_time(m, B, C, steps, kout);
    res[4] = adaspec_policy_goodput(m, B, C, steps, kout, ar, 1e30);
    rc = adaspec_policy_count_tokens(B, C, kout, 0, &res[5], &res[6]);
    if (rc) { fprintf(stderr, "count_tokens %d\n", rc); return 4; }
    write_file("out_policy", res, sizeof res);
    write_file("out_policy_spec_lens", kout, (size_t)B * 4);
    double nc[6] = {10, 200, 3000, 47, 900, 12}, nb[6] = {1, 2, 4, 8, 16, 32}, tt[6], fit[3];
    for (int i = 0; i < 6; ++i) tt[i] = 3e-9 * nc[i] + 2e-6 * nb[i] + 1e-4;
    rc = adaspec_policy_fit_time_model(6, nc, nb, tt, &fit[0], &fit[1], &fit[2]);
    if (rc) { fprintf(stderr, "fit %d\n", rc); return 4; }
    write_file("out_policy_fit", fit, sizeof fit);

    free(dm); free(q); free(kp); free(vp); free(bt); free(ctx); free(spec); free(parents); free(tree_tokens);
    free(logits); free(probs); free(toks); free(uni); free(temp); free(o64); free(ord); free(otok); free(olen);
    free(opath); free(info); free(tinfo); free(sinfo); free(du); free(dq); free(dconf); free(dtok); free(m); free(C);
    free(conf); free(ar); free(kout);
    puts("sanitizer driver: done");
    return 0;
}
