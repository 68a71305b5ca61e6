/*
 * adaspec.h - C ABI of the MI355X (gfx950) ragged verification step.
 *
 * One speculative-decoding verification step over a batch whose requests carry
 * different numbers of draft tokens (the per-request speculative lengths that
 * the paper's Confidence Prior Verifier leaves after draft-token elimination:
 * Alg. 2, Sec. 5.2).  Request i has k_i = spec_lens[i] draft tokens and
 * n_i = k_i + 1 query rows: row 0 is the last committed token, rows 1..k_i are
 * the drafts.  TQ = sum n_i, TD = sum k_i.  Rows of request i start at
 * cu_q[i] = sum_{j<i} n_j; its draft rows start at cu_q[i] - i.
 *
 * Conventions for every call
 *   - Every pointer except the dims struct is a DEVICE pointer owned by the
 *     caller.  The library allocates nothing, frees nothing and never
 *     synchronises; work is enqueued on `stream` (a hipStream_t passed as
 *     void*, NULL = the default stream).
 *   - `workspace` is caller-provided device scratch of at least
 *     *_workspace_bytes(dims) bytes, 256-byte aligned; its contents are
 *     undefined before and after a call.  Calls that share a workspace must be
 *     ordered on one stream.
 *   - Return value: 0 (ADASPEC_OK) or a negative adaspec_status.  On error
 *     nothing has been enqueued.  Errors the host can see (null pointers, bad
 *     dims, unsupported dtype, misalignment, small workspace) are reported;
 *     inconsistent DEVICE data (ctx_lens[i] < n_i, page id out of range,
 *     sum(spec_lens)+batch != total_q, a draft token outside [0, V)) is
 *     undefined behaviour unless checked first with
 *     adaspec_check_ragged_inputs() / adaspec_check_accept_inputs().
 *   - Outputs are fully overwritten.  Results are deterministic: the same
 *     inputs give bit-identical outputs (no floating-point atomics).
 *   - Host threads: the library keeps no state between calls apart from
 *     one-time device queries.  Calls from several threads are safe as long
 *     as they do not share a workspace.  The calls enqueue kernels only (no allocation, no
 *     memset, no synchronisation), so they can be captured into a HIP graph.
 *     The first call of a kernel path on a device does its one-time set-up
 *     (occupancy and device queries; the streaming and two-pass acceptance
 *     paths also raise their kernel's LDS limit): make one call with the same
 *     dims outside the capture before capturing.
 */
#ifndef ADASPEC_H
#define ADASPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ADASPEC_OK = 0,
    ADASPEC_ERR_NULL = -1,        /* a required pointer is NULL                    */
    ADASPEC_ERR_DIM = -2,         /* a size is negative/zero/inconsistent          */
    ADASPEC_ERR_DTYPE = -3,       /* unknown or unsupported element type           */
    ADASPEC_ERR_ALIGN = -4,       /* pointer or row stride not 16-byte aligned     */
    ADASPEC_ERR_WORKSPACE = -5,   /* workspace smaller than *_workspace_bytes()    */
    ADASPEC_ERR_UNSUPPORTED = -6, /* shape outside what the kernels implement      */
    ADASPEC_ERR_HIP = -7          /* a HIP launch failed                           */
} adaspec_status;

typedef enum { ADASPEC_F32 = 0, ADASPEC_F16 = 1, ADASPEC_BF16 = 2 } adaspec_dtype;

/* Kernel selection for adaspec_verify_attn / adaspec_accept / adaspec_draft_sample.
 * AUTO picks the fastest kernel the shape allows (attention: matrix-core, else the
 * portable vector kernel; acceptance: see adaspec_accept); the other values force
 * one kernel (ADASPEC_ERR_UNSUPPORTED if the shape does not fit it). */
typedef enum {
    ADASPEC_PATH_AUTO = 0, ADASPEC_PATH_VECTOR = 1, ADASPEC_PATH_FAST = 2,
    ADASPEC_PATH_STREAM = 3,  /* adaspec_accept only: the streaming 16-bit kernel (V up to 524288), which AUTO
                                 picks for vocabularies too large for the register-resident kernel */
    ADASPEC_PATH_TWO_PASS = 4 /* adaspec_accept only, same shapes as ADASPEC_PATH_FAST: first the accept test
                                 of every draft row (one read of its logits row), then per request the
                                 sampling step on its first rejected row, or on its bonus row, alone.  Rows
                                 after a rejection are not read; the draft-probability row is read only
                                 where a token is recovered from the residual distribution. */
} adaspec_path;

/* ------------------------------------------------------------------------
 * Verification attention (paper Sec. 2.2: the target scores all SL+1 positions
 * in one pass, position t conditioned on the committed tokens and the drafts
 * before it; Eq. 4: the context count grows by one per position; Sec. 6: the
 * KV cache is paged).
 *
 * Row j of request i sits at position pos = ctx_lens[i] - n_i + j and attends
 * to cached tokens 0..pos of its request:
 *     out = softmax(scale * q . K[0..pos]) V[0..pos]
 * q head h reads kv head h / (n_q_heads / n_kv_heads).
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t batch;              /* B >= 0                                              */
    int32_t total_q;            /* TQ = sum(spec_lens[i] + 1); known to the host policy */
    int32_t max_spec_len;       /* upper bound on spec_lens[i]                          */
    int32_t n_q_heads;          /* Hq                                                   */
    int32_t n_kv_heads;         /* Hkv, divides Hq                                      */
    int32_t head_dim;           /* d: 64 or 128 (vector path: any multiple of 8 <= 256) */
    int32_t page_size;          /* P = 16 tokens                                        */
    int32_t num_pages;          /* pages in k_pages / v_pages                           */
    int32_t max_pages_per_req;  /* row stride of block_table                            */
    int32_t dtype;              /* adaspec_dtype of q, k_pages, v_pages                 */
    int32_t out_dtype;          /* adaspec_dtype of out: same as dtype, or ADASPEC_F32
                                   (the fp32 accumulator before the final rounding)     */
    int32_t path;               /* adaspec_path                                         */
    float   scale;              /* softmax scale; 0 means 1/sqrt(head_dim)              */
    int32_t plan_mode;          /* adaspec_plan_mode (below); 0 for a self-contained call */
    void   *timing_start;       /* optional pair of hipEvent_t (both or neither, NULL = none):      */
    void   *timing_stop;        /* recorded on `stream` right before / right after the call's main
                                   kernel (not the metadata kernel, not the split-KV combine), for
                                   callers that want the kernel's own duration.  Events belong to
                                   the caller, who must keep them alive until they have completed. */
} adaspec_attn_dims;

/* The ragged metadata of a verification pass (row offsets, KV-split work list, schedule)
 * depends only on ctx_lens and spec_lens, and every attention layer of the target model sees
 * the same ones (paper Sec. 4.1: ONE target pass over all SL+1 positions).  A caller that runs
 * many layers can therefore build it once:
 *   ADASPEC_PLAN_BUILD_AND_RUN  build the metadata in the workspace, then run (default);
 *   ADASPEC_PLAN_BUILD_ONLY     build it and return; q, k_pages, v_pages, out may be NULL;
 *   ADASPEC_PLAN_REUSE          run with the metadata a previous call left in THIS workspace:
 *                               same dims (except plan_mode and out_dtype), same block_table,
 *                               ctx_lens and spec_lens contents, workspace not used by
 *                               anything else in between.  Violations are undefined behaviour. */
typedef enum { ADASPEC_PLAN_BUILD_AND_RUN = 0, ADASPEC_PLAN_BUILD_ONLY = 1, ADASPEC_PLAN_REUSE = 2 } adaspec_plan_mode;

/* Device scratch needed by adaspec_verify_attn for these dims (0 on bad dims).
 * Dims whose work does not fit the kernels' 32-bit counters are rejected with
 * ADASPEC_ERR_UNSUPPORTED by every attention entry point: more than 2^24 (request, 256-token
 * split) pairs at batch * ceil(max_pages_per_req * 16 / 256), or 2^31 or more
 * (pair, kv head, row group) units. */
size_t adaspec_verify_attn_workspace_bytes(const adaspec_attn_dims *dims);

/*
 * q           [TQ][Hq][d]                       request-major rows (see cu_q above)
 * k_pages     [num_pages][Hkv][P][d]            one (page, kv head) block is contiguous
 * v_pages     same layout as k_pages
 * block_table [B][max_pages_per_req] int32      page id of tokens 16p..16p+15 of request i;
 *                                               entries past ceil(ctx_lens[i]/P) are ignored
 * ctx_lens    [B] int32   L_i: cached tokens of request i INCLUDING its n_i query tokens
 *                         (their K/V are already in the pages); L_i >= n_i
 * spec_lens   [B] int32   k_i in [0, max_spec_len]
 * out         [TQ][Hq][d] of out_dtype; one round-to-nearest-even from the fp32 accumulator
 * Slots of a request's last page beyond L_i, and pages no request uses, are never
 * allowed to influence the result (they may hold NaN).
 * q, k_pages, v_pages, out must be 16-byte aligned.
 */
int adaspec_verify_attn(const void *q, const void *k_pages, const void *v_pages,
                        const int32_t *block_table, const int32_t *ctx_lens,
                        const int32_t *spec_lens, void *out,
                        const adaspec_attn_dims *dims,
                        void *workspace, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------------------
 * Acceptance (paper Sec. 2.2 and Fig. 1 for the greedy form: accept a draft
 * while it equals the target's choice, stop at the first mismatch, emit the
 * target's token there; Sec. 4.2: one bonus token is always produced.  The
 * stochastic form is the speculative-sampling rule of the works the paper
 * cites for speculative decoding in Sec. 1.)
 *
 * Per request, left to right over its drafts x_0..x_{k-1}, temperature T:
 *   T > 0: p = softmax(logits_row / T), q = the draft row.
 *          accept x_j iff uniforms[row][0] < p[x_j] / q[x_j]  (q[x_j] == 0 accepts);
 *          on the first rejection emit the smallest t whose inclusive prefix sum
 *          of r = max(0, p - q) exceeds uniforms[row][1] * sum(r), and stop;
 *          (if sum(r) == 0 the token is drawn from p the same way);
 *          if every draft is accepted emit a token drawn from the bonus row's p
 *          with that row's uniforms[.][1].
 *   T == 0: accept x_j iff x_j == argmax(logits_row) (lowest index on ties);
 *          the emitted token at the stop / bonus row is that argmax.
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t batch;              /* B                                                   */
    int32_t total_q;            /* TQ: rows of target_logits                           */
    int32_t total_draft;        /* TD = TQ - B: rows of draft_probs                    */
    int32_t max_spec_len;       /* upper bound on spec_lens[i]                         */
    int32_t vocab;              /* V                                                   */
    int32_t logits_dtype;       /* adaspec_dtype of target_logits                      */
    int32_t probs_dtype;        /* adaspec_dtype of draft_probs                        */
    int32_t out_stride;         /* row stride of out_tokens, >= max_spec_len + 1       */
    int64_t logits_row_stride;  /* elements between logits rows, >= V                  */
    int64_t probs_row_stride;   /* elements between draft_probs rows, >= V             */
    int32_t path;               /* adaspec_path                                        */
    int32_t reserved;
    void   *timing_start;       /* optional pair of hipEvent_t (both or neither, NULL = none), recorded */
    void   *timing_stop;        /* on `stream` around the call's acceptance kernels (two-pass form: both
                                   passes; per-row forms: the row kernel, not the emit kernel)          */
} adaspec_accept_dims;

size_t adaspec_accept_workspace_bytes(const adaspec_accept_dims *dims);

/*
 * target_logits [TQ][V]   request i owns rows cu_q[i]..cu_q[i]+k_i; row j judges draft j,
 *                         row k_i is the bonus row
 * draft_probs   [TD][V]   request i owns rows cu_q[i]-i ..; the distribution x_j was drawn from
 *                         (final probabilities: the temperature is NOT applied to them)
 * draft_tokens  [TD] int32 in [0, V)
 * uniforms      [TQ][2] float32 in [0, 1): [r][0] accept test, [r][1] inverse-CDF draw
 * spec_lens     [B] int32
 * temperature   [B] float32 >= 0, per request
 * out_tokens    [B][out_stride] int32: a_i accepted drafts, one recovered/bonus token, then -1
 * out_accept_len[B] int32: a_i in [0, k_i]; request i emitted a_i + 1 tokens
 * The per-row paths (vector, register-resident, streaming) evaluate every row, also those after a
 * request's first rejection (the rows are independent), and apply the sequential rule to the
 * per-row results afterwards.  The two-pass path judges every draft row first and then runs the
 * sampling step only on the one row per request that decides its token.  All paths give the same
 * outputs.
 * The register-resident and two-pass paths need 16-bit logits/probs of one type, V % 8 == 0,
 * V <= 131072, strides % 8 == 0 and 16-byte aligned base pointers; the streaming path takes the
 * same up to V <= 524288 (it reads the logits row twice, the second time from the caches);
 * anything else runs on the vector path.  AUTO: two-pass when it fits (batches above 1024 requests:
 * only with more logits rows than compute units or V >= 65536), register-resident when it fits,
 * streaming for larger vocabularies, else vector.
 */
int adaspec_accept(const void *target_logits, const void *draft_probs,
                   const int32_t *draft_tokens, const float *uniforms,
                   const int32_t *spec_lens, const float *temperature,
                   int32_t *out_tokens, int32_t *out_accept_len,
                   const adaspec_accept_dims *dims,
                   void *workspace, size_t workspace_bytes, void *stream);

/*
 * adaspec_accept_noalloc - adaspec_accept for callers that cannot allocate device memory and have no
 * workspace to hand over: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments (without workspace / workspace_bytes), same kernels, same outputs bit for
 * bit.  What the workspace would hold lives in a device array of ADASPEC_NOALLOC_SCRATCH_BYTES that is
 * part of the library's code object: every GPU the library runs on holds it from the first use until
 * the process ends.  The call allocates and frees nothing and synchronises nothing.
 *   - dims whose adaspec_accept_workspace_bytes exceeds ADASPEC_NOALLOC_SCRATCH_BYTES are rejected
 *     with ADASPEC_ERR_WORKSPACE before anything is enqueued (use adaspec_accept for those).
 *   - All calls on one GPU share that GPU's array: calls that can overlap in time on one GPU (other
 *     streams, other threads) race on it; order them on one stream.  The array keeps the previous
 *     call's contents; the kernels initialise whatever they rely on.
 *   - The first call on a device looks the array's address up (no allocation); a caller that captures
 *     graphs makes one call outside a capture first.  More than 64 devices: ADASPEC_ERR_UNSUPPORTED.
 */
#define ADASPEC_NOALLOC_SCRATCH_BYTES ((size_t)8 << 20)
int adaspec_accept_noalloc(const void *target_logits, const void *draft_probs,
                           const int32_t *draft_tokens, const float *uniforms,
                           const int32_t *spec_lens, const float *temperature,
                           int32_t *out_tokens, int32_t *out_accept_len,
                           const adaspec_accept_dims *dims, void *stream);

/* The kernel path adaspec_accept takes for these dims and base pointers (the pointers are only
 * looked at for their alignment): ADASPEC_PATH_VECTOR, _FAST, _STREAM or _TWO_PASS; dims->path
 * itself unless it is ADASPEC_PATH_AUTO; a negative adaspec_status if dims are invalid or a
 * forced path does not fit.  Host-only, launches nothing.  For callers that account for the bytes
 * a call reads: the two-pass path skips rows (see above). */
int adaspec_accept_resolved_path(const void *target_logits, const void *draft_probs,
                                 const adaspec_accept_dims *dims);

/* ------------------------------------------------------------------------
 * Optional device-side check of the ragged metadata (for callers that cannot
 * vouch for it): enqueues one small kernel that writes a bit mask to
 * *err_flags (device int32): bit 0 spec_lens[i] outside [0, max_spec_len],
 * bit 1 ctx_lens[i] < n_i or more pages than max_pages_per_req, bit 2 a used
 * block_table entry outside [0, num_pages), bit 3 sum(n_i) != total_q.
 * 0 means consistent.
 * ---------------------------------------------------------------------- */
int adaspec_check_ragged_inputs(const int32_t *block_table, const int32_t *ctx_lens,
                                const int32_t *spec_lens, const adaspec_attn_dims *dims,
                                int32_t *err_flags, void *stream);

/* ------------------------------------------------------------------------
 * The two steps on either side of a verification step (paper Sec. 6: the
 * target model's KV cache is paged, and the results of one speculative step
 * are integrated into the input of the next).
 *
 * adaspec_kv_append - BEFORE verification: scatter the K and V rows of the n_i
 * new tokens of every request (the last committed token and its k_i drafts)
 * into the pages.  Row j of request i goes to position pos = ctx_lens[i] - n_i + j:
 * page block_table[i][pos / P], slot pos % P, every kv head.
 *   k_new, v_new [TQ][Hkv][d] of dims->dtype, request-major rows like q
 *   k_pages, v_pages are updated in place; nothing else in them is touched.
 * Uses of dims: batch, total_q, max_spec_len, n_kv_heads, head_dim (a multiple
 * of 8 for 16-bit types, of 4 for fp32), page_size, num_pages,
 * max_pages_per_req, dtype; the other fields are ignored.  All four tensors
 * must be 16-byte aligned.  Needs no workspace.
 * ---------------------------------------------------------------------- */
int adaspec_kv_append(const void *k_new, const void *v_new, void *k_pages, void *v_pages,
                      const int32_t *block_table, const int32_t *ctx_lens,
                      const int32_t *spec_lens, const adaspec_attn_dims *dims, void *stream);

/*
 * adaspec_commit - AFTER acceptance: keep what was accepted, drop the rest.
 * Request i had L_i = ctx_lens[i] cached tokens including its n_i = k_i + 1 new
 * ones and accepted a_i = out_accept_len[i] drafts.  The cache entries of the
 * last committed token and of the a_i accepted drafts stay; the k_i - a_i
 * rejected ones become dead slots (they are overwritten by later appends).
 * The recovered / bonus token out_tokens[i][a_i] has no cache entry yet: it is
 * row 0 of the next step.
 *   committed_lens [B]  = L_i - k_i + a_i                      (cache length kept)
 *   next_ctx_lens  [B]  = committed_lens[i] + next_spec_lens[i] + 1, i.e. the
 *                         ctx_lens of the next step; written only if both
 *                         next_spec_lens and next_ctx_lens are non-NULL
 *   last_token     [B]  = out_tokens[i][a_i]
 *   seq_tokens [B][seq_stride], seq_lens [B] (both NULL, or both non-NULL): the
 *                         a_i + 1 emitted tokens are appended at seq_lens[i] and
 *                         seq_lens[i] grows by a_i + 1; tokens that do not fit
 *                         in seq_stride are dropped and seq_lens[i] stops at
 *                         seq_stride.
 * committed_lens may alias ctx_lens (in-place update).
 */
typedef struct {
    int32_t batch;          /* B                                     */
    int32_t max_spec_len;   /* upper bound on spec_lens[i]           */
    int32_t out_stride;     /* row stride of out_tokens              */
    int32_t seq_stride;     /* row stride of seq_tokens (0 if unused) */
} adaspec_commit_dims;

int adaspec_commit(const int32_t *out_tokens, const int32_t *out_accept_len,
                   const int32_t *spec_lens, const int32_t *ctx_lens,
                   const int32_t *next_spec_lens,
                   int32_t *committed_lens, int32_t *next_ctx_lens, int32_t *last_token,
                   int32_t *seq_tokens, int32_t *seq_lens,
                   const adaspec_commit_dims *dims, void *stream);

/* ------------------------------------------------------------------------
 * Tree verification: the drafts of a request form a token TREE instead of a
 * chain.  The paper verifies chains and runs the tree-based system it compares
 * with at tree width 1 (Sec. 7.1, baselines; Sec. 8 names tree-based
 * speculative decoding as the other family), so these three calls lie beside
 * its method: they are the token-tree verification of that baseline, restated.
 * With parent = previous node they compute what the chain calls compute.
 *
 * Nodes.  Request i has n_i = k_i + 1 nodes = its query rows: node 0 is the
 * last committed token (the root), nodes 1..k_i are drafts, ordered so that a
 * parent comes before its children.  parents [TQ] int32 gives, for every row,
 * the parent's index INSIDE the request (anything for the root; values outside
 * [0, j) for node j are forced into that range).  At most 64 nodes per request:
 * max_spec_len <= 63, else ADASPEC_ERR_UNSUPPORTED.
 *
 * adaspec_verify_attn_tree - as adaspec_verify_attn, except for what a row sees.
 * Node j's K/V sit at cache position ctx_lens[i] - n_i + j (the nodes are
 * appended in node order, e.g. by adaspec_kv_append); its row attends to the
 * committed tokens 0 .. ctx_lens[i] - n_i - 1 and to the positions of node j's
 * ancestors and its own.  Same dims, workspace size, plan modes (the ancestor
 * masks belong to the reusable metadata: a PLAN_REUSE call must see the same
 * parents) and error rules as adaspec_verify_attn.
 * ---------------------------------------------------------------------- */
int adaspec_verify_attn_tree(const void *q, const void *k_pages, const void *v_pages,
                             const int32_t *block_table, const int32_t *ctx_lens,
                             const int32_t *spec_lens, const int32_t *parents, void *out,
                             const adaspec_attn_dims *dims,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * adaspec_check_accept_inputs - optional device-side check of what the acceptance calls (chain and
 * tree) index with: enqueues one small kernel that writes a bit mask to *err_flags (device int32):
 * bit 0 spec_lens[i] outside [0, max_spec_len], bit 3 sum(n_i) != total_q (both as in
 * adaspec_check_ragged_inputs), bit 5 (32) a draft token outside [0, vocab), bit 6 (64) a
 * temperature that is negative, infinite or NaN; 0 if all is well.  The acceptance kernels read
 * logits[x] and draft_probs[x] for every draft token x without a range check of their own.
 */
int adaspec_check_accept_inputs(const int32_t *draft_tokens, const int32_t *spec_lens, const float *temperature,
                                const adaspec_accept_dims *dims, int32_t *err_flags, void *stream);

/*
 * adaspec_check_tree_parents - optional device-side check of a parent array (the tree calls force
 * malformed entries into range silently): enqueues one small kernel that writes 16 (bit 4) to
 * *err_flags (device int32) if some node j >= 1 of some request names a parent outside [0, j), else 0.
 * The root's entry is not looked at.  spec_lens and total_q must be consistent
 * (adaspec_check_ragged_inputs).
 */
int adaspec_check_tree_parents(const int32_t *parents, const int32_t *spec_lens, int32_t batch,
                               int32_t total_q, int32_t max_spec_len, int32_t *err_flags, void *stream);

/*
 * adaspec_accept_tree - acceptance walk over the tree of every request.
 *   target_logits [TQ][V]  row of node j: the target's logits for the token after node j
 *   draft_probs   [TD][V]  request i owns rows cu_q[i]-i ..; row j (0 <= j < k_i) is the draft
 *                          distribution AT node j, which the tokens of j's children were drawn
 *                          from (independent draws).  The last node of a request cannot have
 *                          children and has no row; rows of other childless nodes are not read.
 *   draft_tokens  [TD]     row j-1 of the request: token of node j
 *   uniforms      [TQ][2]  the accept test of node c uses [cu_q[i]+c-1][0]; the draw at the node
 *                          where the walk stops uses [cu_q[i]+u][1]
 * Walk, from u = node 0, children of u in ascending node order:
 *   T > 0 : P = softmax(logits_u / T).  Child c with token x is accepted iff
 *           u0 < P[x] / q_u[x]  (q_u[x] == 0 accepts): emit x, go on from c.  After a
 *           rejection r = max(0, P - q_u) and P = r / sum(r) (if sum(r) == 0, P stays).
 *           No child accepted, or none exists: emit the smallest t whose inclusive prefix sum
 *           of the last r (of P at a childless node) exceeds u1 * its total, and stop.
 *   T == 0: z = argmax(logits_u) (lowest index on ties); the first child whose token is z is
 *           accepted; if none, emit z and stop.
 *   out_tokens     [B][out_stride]  tokens of the accepted nodes, the token emitted at the stop, then -1
 *   out_accept_len [B]              accepted nodes a_i
 *   out_path       [B][out_stride]  node indices of the accepted nodes in path order, then -1
 * Dims and workspace as for adaspec_accept.  dims->path:
 *   VECTOR  the portable form (any storage types and vocabulary size): every node of every tree is
 *           evaluated, one workgroup per node, then a small kernel walks the results;
 *   FAST    16-bit logits/probs of one type, V % 8 == 0, V <= 524288, strides % 8 == 0, 16-byte aligned
 *           base pointers: first the statistics of every node (one read of its logits row), then one
 *           workgroup per request walks its tree
 *           and reads, at the nodes it reaches only, the logits and draft-probability rows once per
 *           rejected child;
 *   AUTO    FAST when it fits, else VECTOR.
 */
int adaspec_accept_tree(const void *target_logits, const void *draft_probs,
                        const int32_t *draft_tokens, const int32_t *parents, const float *uniforms,
                        const int32_t *spec_lens, const float *temperature,
                        int32_t *out_tokens, int32_t *out_accept_len, int32_t *out_path,
                        const adaspec_accept_dims *dims,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * adaspec_kv_compact_path - AFTER tree acceptance, BEFORE adaspec_commit: move the K/V rows of
 * the accepted nodes to where a chain would have put them.  Node out_path[i][j] (j < a_i) moves
 * from position base + out_path[i][j] to base + 1 + j, base = ctx_lens[i] - n_i; the root stays.
 * Afterwards adaspec_commit (with the same out_accept_len) keeps exactly those rows.
 * ctx_lens / spec_lens are those of the verification step; path_stride = row stride of out_path.
 * Uses of dims as in adaspec_kv_append.  Needs no workspace.
 */
int adaspec_kv_compact_path(void *k_pages, void *v_pages, const int32_t *block_table,
                            const int32_t *ctx_lens, const int32_t *spec_lens,
                            const int32_t *out_path, const int32_t *out_accept_len,
                            const adaspec_attn_dims *dims, int32_t path_stride, void *stream);

/* ------------------------------------------------------------------------
 * Draft-side sampling: the producer of draft_probs, draft_tokens and of the
 * confidence scores the speculative-length policy consumes (paper Sec. 4.2,
 * Eq. 6: a draft token's acceptance rate is modelled by the product of the
 * confidence scores c_{i,k}; Alg. 1: every execution of the draft model
 * returns the draft tokens and their confidences).
 *
 * For each of `rows` rows of draft-model logits, with T = temperature[r]:
 *   T > 0 : q = softmax(logits / T), every entry rounded ONCE (nearest-even) to
 *           probs_dtype and stored; token = smallest t whose inclusive prefix
 *           sum of the ROUNDED row exceeds uniforms[r] * (sum of the rounded
 *           row), so a token of probability zero is never drawn;
 *   T == 0: greedy drafting: token = argmax(logits) (lowest index on ties) and
 *           q = softmax(logits) (temperature 1), rounded and stored.  The token
 *           is then NOT a draw from the stored row: such a draft must be
 *           verified at temperature 0 as well (adaspec_accept with
 *           temperature[i] == 0 never looks at q); verified at T > 0 the
 *           emitted tokens would no longer follow the target's distribution;
 *   confidence[r] = q[token] as stored, widened to float.
 * The row is written to draft_probs row out_rows[r] (row r if out_rows is
 * NULL), so a caller can place it directly into the ragged [TD][V] layout
 * that adaspec_accept reads.
 *
 * Needs V % 8 == 0, V <= 524288, row strides that are multiples of 8 elements
 * and 16-byte aligned logits / draft_probs (ADASPEC_ERR_UNSUPPORTED or
 * ADASPEC_ERR_ALIGN otherwise).
 * Workspace: only the split form uses one (adaspec_draft_sample_workspace_bytes;
 * 256-byte aligned device memory, contents need not be initialised).  With
 * workspace == NULL the call runs a single-kernel form.
 * ---------------------------------------------------------------------- */
typedef struct {
    int32_t rows;               /* R >= 0                                      */
    int32_t vocab;              /* V                                           */
    int32_t logits_dtype;       /* adaspec_dtype of draft_logits               */
    int32_t probs_dtype;        /* adaspec_dtype of draft_probs                */
    int64_t logits_row_stride;  /* elements between logits rows, >= V          */
    int64_t probs_row_stride;   /* elements between draft_probs rows, >= V     */
    int32_t path;               /* adaspec_path: FAST = register-resident kernel
                                   (16-bit logits, V <= 131072), VECTOR = the
                                   three-sweep kernel, TWO_PASS = the split form
                                   (same shapes as FAST, needs the workspace):
                                   every row cut into four parts over three small
                                   kernels, for steps with fewer rows than the
                                   device has compute units; AUTO = the split
                                   form when it fits, a workspace is given and
                                   V >= 32768, else FAST when it fits, else VECTOR */
    int32_t reserved;
    void   *timing_start;       /* optional pair of hipEvent_t (both or neither, NULL = none), recorded */
    void   *timing_stop;        /* on `stream` around the call's kernels                                */
} adaspec_draft_dims;

/* Bytes of workspace the split form needs for these dims (0 if it does not apply). */
size_t adaspec_draft_sample_workspace_bytes(const adaspec_draft_dims *dims);

int adaspec_draft_sample(const void *draft_logits,      /* [R][V]                               */
                         const float *temperature,      /* [R] >= 0                             */
                         const float *uniforms,         /* [R] in [0, 1)                        */
                         const int32_t *out_rows,       /* [R] destination rows, or NULL        */
                         void *draft_probs,             /* [max(out_rows)+1][V], written        */
                         int32_t *draft_tokens,         /* [R]                                  */
                         float *confidence,             /* [R]                                  */
                         const adaspec_draft_dims *dims,
                         void *workspace, size_t workspace_bytes, void *stream);

const char *adaspec_status_string(int status);
int adaspec_version(void);

#ifdef __cplusplus
}
#endif
#endif /* ADASPEC_H */
