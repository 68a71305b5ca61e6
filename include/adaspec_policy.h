/*
 * adaspec_policy.h - host-side speculative-length policy (C ABI, HOST pointers).
 *
 * The paper's policy runs on the CPU next to the scheduler (Sec. 6) and decides,
 * per step and per request, how many draft tokens go to verification; its
 * output spec_lens[] is the ragged shape that adaspec_verify_attn /
 * adaspec_accept consume.  Everything here is plain host code in double
 * precision: no device memory, no HIP call, no allocation visible to the
 * caller.  All pointers are HOST pointers owned by the caller.
 *
 * Conventions (they reproduce the closed form of Lemma 1, Sec. 4.1)
 *   C_i = ctx_committed[i]: cached tokens of request i before the step, i.e.
 *         the tokens that precede the first new token;
 *   the j-th forward pass / position (j = 1, 2, ...) counts C_i + j - 1 context
 *   tokens and one batch token per request;
 *   ar[s * B + i] = AR_{i,s+1} = c_{i,1} * ... * c_{i,s+1} (Eq. 6), s = 0..steps-1;
 *   the bonus token AR_{i,0} = 1 is added by the library (Eq. 5).
 * Return value: 0 or a negative adaspec_status (adaspec.h); functions that
 * return a double return NaN on invalid arguments.
 */
#ifndef ADASPEC_POLICY_H
#define ADASPEC_POLICY_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Performance coefficients of the forward-time model T = alpha*N_c + gamma*N_b + delta
 * (Eq. 2) for the draft (d) and the target (v) model. */
typedef struct {
    double alpha_d, gamma_d, delta_d;
    double alpha_v, gamma_v, delta_v;
    /* How the target pass counts context tokens.  0: as in Eq. 4, every verified position
     * counts its own context (request i contributes sum_{j=1..k_i+1} (C_i + j - 1)).
     * 1: every request's context counts ONCE, C_i + k_i + 1 tokens: the cost shape of a
     * verification kernel that reads the cached keys and values once for all k_i + 1 positions
     * of a request, as adaspec_verify_attn does (fit the coefficients with the same setting). */
    int32_t verify_ctx_once;
    int32_t reserved;
} adaspec_time_model;

/* T_sd = T_d + T_v (Eq. 1, 3, 4): `draft_steps` passes of the draft model over all B
 * requests, one target pass over spec_lens[i] + 1 positions of request i
 * (spec_lens == NULL means spec_lens[i] = draft_steps for every request). */
double adaspec_policy_estimate_time(const adaspec_time_model *m, int32_t batch,
                                    const int32_t *ctx_committed, int32_t draft_steps,
                                    const int32_t *spec_lens);

/* Alg. 3 (SLO-aware efficiency estimator): expected accepted tokens (Eq. 5) divided by the
 * estimated step time, or -1 when that time exceeds the TPOT constraint `tpot`
 * (same unit as the model's times; pass +inf for no constraint). */
double adaspec_policy_goodput(const adaspec_time_model *m, int32_t batch,
                              const int32_t *ctx_committed, int32_t draft_steps,
                              const int32_t *spec_lens, const double *ar, double tpot);

/* Alg. 1 (adaptive drafter, predict - execute - correct).  The draft model is outside this
 * library: conf[s * B + i] is the confidence it reports for request i at draft step s + 1,
 * read only when the loop decides to execute that step; at most max_steps steps.
 * prev_conf is the historical average confidence used for the prediction.
 * Outputs: *steps_out = draft steps executed (the step-level speculative length),
 * ar_out[max_steps * B] (first *steps_out rows filled), *goodput_out = the estimate after
 * the last executed step (-1 if none was executed). */
int adaspec_policy_adaptive_draft(const adaspec_time_model *m, int32_t batch,
                                  const int32_t *ctx_committed, const double *conf,
                                  int32_t max_steps, double prev_conf, double tpot,
                                  int32_t *steps_out, double *ar_out, double *goodput_out);

/* Alg. 2 (confidence prior verifier, draft-token elimination): starting from draft_steps
 * tokens per request, repeatedly drops the remaining draft token with the lowest acceptance
 * rate (always the last remaining draft of a request; lowest request index on ties) while
 * the goodput estimate strictly improves.  Outputs: spec_lens_out[B] (the request-level
 * speculative lengths), *goodput_out. */
int adaspec_policy_eliminate(const adaspec_time_model *m, int32_t batch,
                             const int32_t *ctx_committed, int32_t draft_steps,
                             const double *ar, double tpot,
                             int32_t *spec_lens_out, double *goodput_out);

/* The two counts of Eq. 4 for ONE target pass over a ragged batch: *n_b = sum (spec_lens[i] + 1), the
 * verified positions, and *n_c = the context tokens they are charged: every position its own context,
 * sum_i sum_{j=1..k_i+1} (C_i + j - 1), as printed (verify_ctx_once == 0), or every request's context
 * once, sum_i (C_i + k_i + 1) (verify_ctx_once != 0; see adaspec_time_model).  What the offline analyzer
 * regresses its measured times on.  ADASPEC_ERR_DIM for a negative length. */
int adaspec_policy_count_tokens(int32_t batch, const int32_t *ctx_committed, const int32_t *spec_lens,
                                int32_t verify_ctx_once, double *n_c, double *n_b);

/* Offline analyzer (Sec. 6): least-squares fit of (alpha, gamma, delta) of Eq. 2 to n measured
 * forward passes with n_c[i] context tokens, n_b[i] batch tokens and time t[i].
 * ADASPEC_ERR_DIM if n < 3 or the three columns are linearly dependent. */
int adaspec_policy_fit_time_model(int32_t n, const double *n_c, const double *n_b, const double *t,
                                  double *alpha, double *gamma, double *delta);

#ifdef __cplusplus
}
#endif
#endif /* ADASPEC_POLICY_H */
