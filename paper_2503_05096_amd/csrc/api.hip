// C ABI entry points of libadaspec.so: host-side validation, workspace layout
// and the launch sequence of each call.  The entry points that enqueue work make
// no HIP call before their arguments have been validated, so their error paths
// work on a machine with no GPU (adaspec_accept_resolved_path asks the device for
// its compute-unit count; without a device it assumes 256).
#include <math.h>
#include <string.h>

#include <mutex>

#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

// the optional event pair of a dims struct: recorded only if both are given
static bool record_event(void *start, void *stop, bool first, hipStream_t stream)
{
    if (!start || !stop) return true;
    return hipEventRecord(static_cast<hipEvent_t>(first ? start : stop), stream) == hipSuccess;
}

// ---- scratch memory of adaspec_accept_noalloc ------------------------------------------------------
// A file-scope device array stands in for the workspace argument: every GPU the library runs on holds
// its own copy, at its own address, until the process ends.  In host code the NAME of the array is
// only a handle for hipGetSymbolAddress; the device address it yields (looked up once per device,
// with that device current) is what kernels, and anything else that touches the memory, are given.
constexpr size_t kNoallocScratchBytes = ADASPEC_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kNoallocScratchBytes];
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices] = {};
static std::mutex g_scratch_mutex;

// device address of `scratch` on the current device (ADASPEC_OK), or a negative status
static int noalloc_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return ADASPEC_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return ADASPEC_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return ADASPEC_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ADASPEC_OK;
}

// compute units of the current device (asked once; 256 if the runtime cannot tell)
static int compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

static bool dtype_ok(int dt) { return dt == ADASPEC_F32 || dt == ADASPEC_F16 || dt == ADASPEC_BF16; }
static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static int validate_attn_dims(const adaspec_attn_dims *d)
{
    if (!d) return ADASPEC_ERR_NULL;
    if (d->batch < 0 || d->total_q < d->batch || d->max_spec_len < 0) return ADASPEC_ERR_DIM;
    if ((int64_t)d->total_q > (int64_t)d->batch * (d->max_spec_len + 1)) return ADASPEC_ERR_DIM;
    if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->n_q_heads % d->n_kv_heads) return ADASPEC_ERR_DIM;
    if (d->num_pages <= 0 || d->max_pages_per_req <= 0) return ADASPEC_ERR_DIM;
    if (d->head_dim <= 0) return ADASPEC_ERR_DIM;
    if (!dtype_ok(d->dtype) || !dtype_ok(d->out_dtype)) return ADASPEC_ERR_DTYPE;
    if (d->out_dtype != d->dtype && d->out_dtype != ADASPEC_F32) return ADASPEC_ERR_DTYPE;
    if (d->page_size != 16) return ADASPEC_ERR_UNSUPPORTED;
    if (d->head_dim % 8 || d->head_dim > 256) return ADASPEC_ERR_UNSUPPORTED;
    if (d->path < ADASPEC_PATH_AUTO || d->path > ADASPEC_PATH_FAST) return ADASPEC_ERR_DIM;
    if (!(d->scale >= 0.0f) || isinf(d->scale)) return ADASPEC_ERR_DIM;
    if (d->path == ADASPEC_PATH_FAST && !attn_fast_path_supported(*d)) return ADASPEC_ERR_UNSUPPORTED;
    if (d->plan_mode < ADASPEC_PLAN_BUILD_AND_RUN || d->plan_mode > ADASPEC_PLAN_REUSE) return ADASPEC_ERR_DIM;
    {   // the kernels count work items and units in 32 bits: bound them at the shortest split (256 tokens)
        const int64_t per_req = ((int64_t)d->max_pages_per_req * d->page_size + 255) / 256;
        const int64_t items = (int64_t)d->batch * per_req;
        const int64_t rows = (int64_t)(d->max_spec_len + 1) * (d->n_q_heads / d->n_kv_heads);
        if (rows > (1 << 20) || items > kMaxAttnItems ||
            items * d->n_kv_heads * attn_row_groups((int)rows) >= (int64_t)1 << 31)
            return ADASPEC_ERR_UNSUPPORTED;
    }
    return ADASPEC_OK;
}

static bool attn_use_fast(const adaspec_attn_dims &d)
{
    if (d.path == ADASPEC_PATH_VECTOR) return false;
    return attn_fast_path_supported(d);
}

AttnPlan make_attn_plan(const adaspec_attn_dims &d, bool fast_path)
{
    AttnPlan p;
    const int G = d.n_q_heads / d.n_kv_heads;
    // The matrix-core kernel runs 4 wavefronts per work item, each over up to 256
    // tokens, and merges them on chip; the vector kernel runs one wavefront per
    // item.  With few (request, kv head) pairs the splits are shortened so that
    // the chip still sees enough independent items.
    const int64_t pairs = (int64_t)d.batch * d.n_kv_heads;
    if (fast_path) {
        p.block_tokens = 32;
        p.split_tokens = pairs >= 512 ? 2048 : (pairs >= 256 ? 2048 : (pairs >= 128 ? 1024 : (pairs >= 32 ? 512 : 256)));
    } else {
        p.block_tokens = 64;
        p.split_tokens = 256;
    }
    const int64_t max_ctx = (int64_t)d.max_pages_per_req * d.page_size;
    const int64_t per_req = (max_ctx + p.split_tokens - 1) / p.split_tokens;
    p.max_items = (int)((int64_t)d.batch * per_req);
    p.max_rows = (d.max_spec_len + 1) * G;
    size_t off = 0;
    p.off_header = off;     off = align_up(off + 16 * sizeof(int32_t), 256);
    p.off_cu_q = off;       off = align_up(off + (size_t)(d.batch + 1) * 4, 256);
    p.off_split_base = off; off = align_up(off + (size_t)(d.batch + 1) * 4, 256);
    p.off_item_req = off;   off = align_up(off + (size_t)(p.max_items > 0 ? p.max_items : 1) * 4, 256);
    p.off_item_order = off; off = align_up(off + (size_t)(p.max_items > 0 ? p.max_items : 1) * 4, 256);
    p.off_unit_meta = off;  off = align_up(off + (size_t)(p.max_items > 0 ? p.max_items : 1) * 32, 256);
    p.off_row_rec = off;    off = align_up(off + (size_t)(d.total_q > 0 ? d.total_q : 1) * 16, 256);
    {   // schedule table: every unit appears once, every round is W <= kMaxSchedW wide
        const size_t units = (size_t)p.max_items * d.n_kv_heads * attn_row_groups(p.max_rows);
        p.off_sched = off;  off = align_up(off + (fast_path ? units + kMaxSchedW : 1) * 4, 256);
    }
    p.off_anc = off;        off = align_up(off + (size_t)(d.total_q > 0 ? d.total_q : 1) * 8, 256);
    p.off_part_ml = off;
    off = align_up(off + (size_t)p.max_items * d.n_kv_heads * p.max_rows * 2 * sizeof(float), 256);
    p.off_part_o = off;
    off = align_up(off + (size_t)p.max_items * d.n_kv_heads * p.max_rows * d.head_dim * sizeof(float), 256);
    p.total_bytes = off;
    return p;
}

static int validate_accept_dims(const adaspec_accept_dims *d)
{
    if (!d) return ADASPEC_ERR_NULL;
    if (d->batch < 0 || d->total_q < d->batch || d->max_spec_len < 0) return ADASPEC_ERR_DIM;
    if (d->total_draft != d->total_q - d->batch) return ADASPEC_ERR_DIM;
    if ((int64_t)d->total_q > (int64_t)d->batch * (d->max_spec_len + 1)) return ADASPEC_ERR_DIM;
    if (d->vocab <= 0) return ADASPEC_ERR_DIM;
    if (!dtype_ok(d->logits_dtype) || !dtype_ok(d->probs_dtype)) return ADASPEC_ERR_DTYPE;
    if (d->logits_row_stride < d->vocab || d->probs_row_stride < d->vocab) return ADASPEC_ERR_DIM;
    if (d->out_stride < d->max_spec_len + 1) return ADASPEC_ERR_DIM;
    if (d->path < ADASPEC_PATH_AUTO || d->path > ADASPEC_PATH_TWO_PASS) return ADASPEC_ERR_DIM;
    return ADASPEC_OK;
}

AcceptPlan make_accept_plan(const adaspec_accept_dims &d)
{
    AcceptPlan p;
    size_t off = 0;
    const size_t tq = (size_t)(d.total_q > 0 ? d.total_q : 1);
    p.off_cu_q = off;     off = align_up(off + (size_t)(d.batch + 1) * 4, 256);
    p.off_row_req = off;  off = align_up(off + tq * 4, 256);
    p.off_row_flag = off; off = align_up(off + tq * 4, 256);
    p.off_row_cand = off; off = align_up(off + tq * 4, 256);
    p.off_row_meta = off; off = align_up(off + tq * 32, 256);
    const size_t nb = (size_t)(d.batch > 0 ? d.batch : 1);
    p.off_row_stat = off;   off = align_up(off + tq * sizeof(RowStat), 256);
    p.off_req_ticket = off; off = align_up(off + nb * 4, 256);
    p.off_slot_rec = off;   off = align_up(off + accept_parts_slot_bytes(d), 256);
    p.off_part_stat = off;  off = align_up(off + accept_parts_stat_bytes(d), 256);
    p.off_half_stat = off;  off = align_up(off + accept_parts_sum_stat_bytes(d), 256);
    p.off_part = off;       off = align_up(off + accept_parts_sum_bytes(d), 256);
    p.off_tree_stat = off; off = align_up(off + tq * tree_node_stat_bytes(), 256);
    p.total_bytes = off;
    return p;
}

}  // namespace adaspec

using namespace adaspec;

extern "C" {

size_t adaspec_verify_attn_workspace_bytes(const adaspec_attn_dims *dims)
{
    if (validate_attn_dims(dims) != ADASPEC_OK) return 0;
    return make_attn_plan(*dims, attn_use_fast(*dims)).total_bytes;
}

// chain (parents == NULL, tree == false) and tree verification share everything but the mask
static int verify_attn_impl(const void *q, const void *k_pages, const void *v_pages,
                            const int32_t *block_table, const int32_t *ctx_lens,
                            const int32_t *spec_lens, const int32_t *parents, bool tree, void *out,
                            const adaspec_attn_dims *dims,
                            void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = validate_attn_dims(dims);
    if (rc != ADASPEC_OK) return rc;
    if (tree && dims->max_spec_len > 63) return ADASPEC_ERR_UNSUPPORTED;
    if (dims->batch == 0) return ADASPEC_OK;
    if (tree && !parents) return ADASPEC_ERR_NULL;
    const bool plan_only = dims->plan_mode == ADASPEC_PLAN_BUILD_ONLY;
    if (!block_table || !ctx_lens || !spec_lens || !workspace) return ADASPEC_ERR_NULL;
    if (!plan_only && (!q || !k_pages || !v_pages || !out)) return ADASPEC_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ADASPEC_ERR_ALIGN;
    if (!plan_only && (!aligned16(q) || !aligned16(k_pages) || !aligned16(v_pages) || !aligned16(out)))
        return ADASPEC_ERR_ALIGN;
    AttnArgs a;
    const bool fast = attn_use_fast(*dims);
    a.plan = make_attn_plan(*dims, fast);
    if (workspace_bytes < a.plan.total_bytes) return ADASPEC_ERR_WORKSPACE;
    a.q = q; a.k_pages = k_pages; a.v_pages = v_pages;
    a.block_table = block_table; a.ctx_lens = ctx_lens; a.spec_lens = spec_lens;
    a.parents = tree ? parents : nullptr;
    a.out = out; a.dims = *dims; a.ws = static_cast<char *>(workspace);
    a.stream = static_cast<hipStream_t>(stream);
    const float scale = dims->scale > 0.0f ? dims->scale : 1.0f / sqrtf((float)dims->head_dim);
    a.scale_log2 = scale * 1.4426950408889634f;

    if (fast) attn_mfma_shape(a);
    if (dims->plan_mode != ADASPEC_PLAN_REUSE) {
        if (launch_attn_plan(a) != hipSuccess) return ADASPEC_ERR_HIP;
        if (tree && launch_tree_masks(a) != hipSuccess) return ADASPEC_ERR_HIP;
    }
    if (plan_only) return ADASPEC_OK;
    if (!record_event(dims->timing_start, dims->timing_stop, true, a.stream)) return ADASPEC_ERR_HIP;
    hipError_t e = fast ? launch_attn_mfma(a) : launch_attn_vector(a);
    if (e != hipSuccess) return ADASPEC_ERR_HIP;
    if (!record_event(dims->timing_start, dims->timing_stop, false, a.stream)) return ADASPEC_ERR_HIP;
    if (launch_attn_combine(a) != hipSuccess) return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

int adaspec_verify_attn(const void *q, const void *k_pages, const void *v_pages,
                        const int32_t *block_table, const int32_t *ctx_lens,
                        const int32_t *spec_lens, void *out, const adaspec_attn_dims *dims,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    return verify_attn_impl(q, k_pages, v_pages, block_table, ctx_lens, spec_lens, nullptr, false, out, dims,
                            workspace, workspace_bytes, stream);
}

int adaspec_verify_attn_tree(const void *q, const void *k_pages, const void *v_pages,
                             const int32_t *block_table, const int32_t *ctx_lens,
                             const int32_t *spec_lens, const int32_t *parents, void *out,
                             const adaspec_attn_dims *dims,
                             void *workspace, size_t workspace_bytes, void *stream)
{
    return verify_attn_impl(q, k_pages, v_pages, block_table, ctx_lens, spec_lens, parents, true, out, dims,
                            workspace, workspace_bytes, stream);
}

size_t adaspec_accept_workspace_bytes(const adaspec_accept_dims *dims)
{
    if (validate_accept_dims(dims) != ADASPEC_OK) return 0;
    return make_accept_plan(*dims).total_bytes;
}

// The kernel path a call with these dims and pointers takes (an adaspec_path other than AUTO), or a
// negative status if a forced path does not fit the shape.
static int resolve_accept_path(const adaspec_accept_dims &d, const void *logits, const void *probs)
{
    const bool fast_ok = accept_fast_path_supported(d, logits, probs);
    const bool stream_ok = accept_stream_path_supported(d, logits, probs);
    const bool two_pass_ok = fast_ok && stream_ok;
    if (d.path == ADASPEC_PATH_FAST && !fast_ok) return ADASPEC_ERR_UNSUPPORTED;
    if (d.path == ADASPEC_PATH_STREAM && !stream_ok) return ADASPEC_ERR_UNSUPPORTED;
    if (d.path == ADASPEC_PATH_TWO_PASS && !two_pass_ok) return ADASPEC_ERR_UNSUPPORTED;
    if (d.path != ADASPEC_PATH_AUTO) return d.path;
    // AUTO.  The two-pass form in row parts does the least work (rows behind a rejection are never read, the
    // sampling step runs on one row per request) and spreads every row over many small workgroups; measured
    // on MI355X it is ahead of the per-row kernels (+ emit kernel) on every benchmark shape: V = 32000, 150
    // rows 16.5 against 21.4 us; V = 128256: 227 rows 28 against 38 us, 380 rows 39 against 63 us, 510 rows
    // 42 against 70 us; all greedy 17.1 against 16.9 us.  Batches it does not take (more than 1024 requests)
    // use the older two-pass pair when there are more rows than compute units or the vocabulary is large; a
    // row that does not fit the registers of one workgroup (V > 131072) goes to the streaming kernel, anything
    // else to the vector kernel.
    if (two_pass_ok && accept_parts_supported(d)) return ADASPEC_PATH_TWO_PASS;
    if (two_pass_ok && (d.total_q > compute_units() || d.vocab >= 65536)) return ADASPEC_PATH_TWO_PASS;
    if (fast_ok) return ADASPEC_PATH_FAST;
    if (stream_ok) return ADASPEC_PATH_STREAM;
    return ADASPEC_PATH_VECTOR;
}

int adaspec_accept_resolved_path(const void *target_logits, const void *draft_probs,
                                 const adaspec_accept_dims *dims)
{
    const int rc = validate_accept_dims(dims);
    if (rc != ADASPEC_OK) return rc;
    return resolve_accept_path(*dims, target_logits, draft_probs);
}

// workspace == NULL with use_static_scratch: the library's own device array takes its place
static int accept_impl(const void *target_logits, const void *draft_probs,
                       const int32_t *draft_tokens, const float *uniforms,
                       const int32_t *spec_lens, const float *temperature,
                       int32_t *out_tokens, int32_t *out_accept_len,
                       const adaspec_accept_dims *dims,
                       void *workspace, size_t workspace_bytes, bool use_static_scratch, void *stream)
{
    int rc = validate_accept_dims(dims);
    if (rc != ADASPEC_OK) return rc;
    if (use_static_scratch && make_accept_plan(*dims).total_bytes > kNoallocScratchBytes)
        return ADASPEC_ERR_WORKSPACE;           // larger than the built-in scratch: use adaspec_accept
    if (dims->batch == 0) return ADASPEC_OK;
    if (!target_logits || !uniforms || !spec_lens || !temperature || !out_tokens || !out_accept_len ||
        (!workspace && !use_static_scratch))
        return ADASPEC_ERR_NULL;
    if (dims->total_draft > 0 && (!draft_probs || !draft_tokens)) return ADASPEC_ERR_NULL;
    if (use_static_scratch) {
        rc = noalloc_scratch(&workspace);
        if (rc != ADASPEC_OK) return rc;
        workspace_bytes = kNoallocScratchBytes;
    }
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ADASPEC_ERR_ALIGN;
    const int path = resolve_accept_path(*dims, target_logits, draft_probs);
    if (path < 0) return path;
    const bool two_pass = path == ADASPEC_PATH_TWO_PASS, fast = path == ADASPEC_PATH_FAST,
               streaming = path == ADASPEC_PATH_STREAM;
    AcceptArgs a;
    a.plan = make_accept_plan(*dims);
    if (workspace_bytes < a.plan.total_bytes) return ADASPEC_ERR_WORKSPACE;
    a.logits = target_logits; a.probs = draft_probs; a.draft_tokens = draft_tokens;
    a.uniforms = uniforms; a.spec_lens = spec_lens; a.temperature = temperature;
    a.out_tokens = out_tokens; a.out_accept_len = out_accept_len;
    a.dims = *dims; a.ws = static_cast<char *>(workspace);
    a.stream = static_cast<hipStream_t>(stream);

    if (two_pass) {
        // the statistics of the draft rows, then per request the accept tests, the sampling on the one row
        // that decides its token, and the request's outputs (no emit kernel); both in row parts for up to
        // 1024 requests, larger batches with one workgroup per row and then per request
        if (!record_event(dims->timing_start, dims->timing_stop, true, a.stream)) return ADASPEC_ERR_HIP;
        if (accept_parts_supported(*dims)) {
            if (launch_accept_parts(a) != hipSuccess) return ADASPEC_ERR_HIP;
        } else {
            if (launch_accept_test(a) != hipSuccess) return ADASPEC_ERR_HIP;
            if (launch_accept_resolve(a) != hipSuccess) return ADASPEC_ERR_HIP;
        }
        if (!record_event(dims->timing_start, dims->timing_stop, false, a.stream)) return ADASPEC_ERR_HIP;
        return ADASPEC_OK;
    }
    // the register-resident kernel finds each row's request itself; only the vector kernel needs the plan
    if (!fast && !streaming && launch_accept_plan(a) != hipSuccess) return ADASPEC_ERR_HIP;
    if (!record_event(dims->timing_start, dims->timing_stop, true, a.stream)) return ADASPEC_ERR_HIP;
    hipError_t e = fast ? launch_accept_fast(a) : (streaming ? launch_accept_stream(a) : launch_accept_vector(a));
    if (e != hipSuccess) return ADASPEC_ERR_HIP;
    if (!record_event(dims->timing_start, dims->timing_stop, false, a.stream)) return ADASPEC_ERR_HIP;
    if (launch_accept_emit(a) != hipSuccess) return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

int adaspec_accept(const void *target_logits, const void *draft_probs,
                   const int32_t *draft_tokens, const float *uniforms,
                   const int32_t *spec_lens, const float *temperature,
                   int32_t *out_tokens, int32_t *out_accept_len,
                   const adaspec_accept_dims *dims,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    return accept_impl(target_logits, draft_probs, draft_tokens, uniforms, spec_lens, temperature, out_tokens,
                       out_accept_len, dims, workspace, workspace_bytes, false, stream);
}

int adaspec_accept_noalloc(const void *target_logits, const void *draft_probs,
                           const int32_t *draft_tokens, const float *uniforms,
                           const int32_t *spec_lens, const float *temperature,
                           int32_t *out_tokens, int32_t *out_accept_len,
                           const adaspec_accept_dims *dims, void *stream)
{
    return accept_impl(target_logits, draft_probs, draft_tokens, uniforms, spec_lens, temperature, out_tokens,
                       out_accept_len, dims, nullptr, 0, true, stream);
}

int adaspec_accept_tree(const void *target_logits, const void *draft_probs,
                        const int32_t *draft_tokens, const int32_t *parents, const float *uniforms,
                        const int32_t *spec_lens, const float *temperature,
                        int32_t *out_tokens, int32_t *out_accept_len, int32_t *out_path,
                        const adaspec_accept_dims *dims,
                        void *workspace, size_t workspace_bytes, void *stream)
{
    int rc = validate_accept_dims(dims);
    if (rc != ADASPEC_OK) return rc;
    if (dims->path != ADASPEC_PATH_AUTO && dims->path != ADASPEC_PATH_VECTOR && dims->path != ADASPEC_PATH_FAST)
        return ADASPEC_ERR_UNSUPPORTED;
    if (dims->max_spec_len > 63) return ADASPEC_ERR_UNSUPPORTED;
    // (the fast tree kernels take the shapes of the streaming chain kernel: 16-bit rows of one type, V % 8 == 0,
    // V <= 524288, strides % 8 == 0, 16-byte aligned)
    const bool fast_ok = accept_stream_path_supported(*dims, target_logits, draft_probs);
    if (dims->path == ADASPEC_PATH_FAST && !fast_ok) return ADASPEC_ERR_UNSUPPORTED;
    const bool fast = fast_ok && dims->path != ADASPEC_PATH_VECTOR;
    if (dims->batch == 0) return ADASPEC_OK;
    if (!target_logits || !parents || !uniforms || !spec_lens || !temperature || !out_tokens ||
        !out_accept_len || !out_path || !workspace)
        return ADASPEC_ERR_NULL;
    if (dims->total_draft > 0 && (!draft_probs || !draft_tokens)) return ADASPEC_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ADASPEC_ERR_ALIGN;
    AcceptArgs a;
    a.plan = make_accept_plan(*dims);
    if (workspace_bytes < a.plan.total_bytes) return ADASPEC_ERR_WORKSPACE;
    a.logits = target_logits; a.probs = draft_probs; a.draft_tokens = draft_tokens;
    a.uniforms = uniforms; a.spec_lens = spec_lens; a.temperature = temperature;
    a.out_tokens = out_tokens; a.out_accept_len = out_accept_len;
    a.dims = *dims; a.ws = static_cast<char *>(workspace);
    a.stream = static_cast<hipStream_t>(stream);
    // (the fast kernels find their rows and requests themselves, up to a few thousand requests)
    if ((!fast || tree_fast_needs_plan(*dims)) && launch_accept_plan(a) != hipSuccess) return ADASPEC_ERR_HIP;
    if (!record_event(dims->timing_start, dims->timing_stop, true, a.stream)) return ADASPEC_ERR_HIP;
    if (fast) {
        if (launch_accept_tree_fast(a, parents, out_path) != hipSuccess) return ADASPEC_ERR_HIP;
    } else {
        if (launch_accept_tree_nodes(a, parents) != hipSuccess) return ADASPEC_ERR_HIP;
        if (launch_accept_tree_walk(a, out_path) != hipSuccess) return ADASPEC_ERR_HIP;
    }
    if (!record_event(dims->timing_start, dims->timing_stop, false, a.stream)) return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

int adaspec_kv_compact_path(void *k_pages, void *v_pages, const int32_t *block_table,
                            const int32_t *ctx_lens, const int32_t *spec_lens,
                            const int32_t *out_path, const int32_t *out_accept_len,
                            const adaspec_attn_dims *d, int32_t path_stride, void *stream)
{
    if (!d) return ADASPEC_ERR_NULL;
    if (d->batch < 0 || d->max_spec_len < 0 || path_stride < d->max_spec_len + 1) return ADASPEC_ERR_DIM;
    if (d->n_kv_heads <= 0 || d->head_dim <= 0 || d->page_size <= 0) return ADASPEC_ERR_DIM;
    if (d->num_pages <= 0 || d->max_pages_per_req <= 0) return ADASPEC_ERR_DIM;
    if (!dtype_ok(d->dtype)) return ADASPEC_ERR_DTYPE;
    if ((d->head_dim * (d->dtype == ADASPEC_F32 ? 4 : 2)) % 16) return ADASPEC_ERR_UNSUPPORTED;
    if (d->batch > 65535) return ADASPEC_ERR_UNSUPPORTED;
    if (d->batch == 0) return ADASPEC_OK;
    if (!k_pages || !v_pages || !block_table || !ctx_lens || !spec_lens || !out_path || !out_accept_len)
        return ADASPEC_ERR_NULL;
    if (!aligned16(k_pages) || !aligned16(v_pages)) return ADASPEC_ERR_ALIGN;
    if (launch_kv_compact_path(k_pages, v_pages, block_table, ctx_lens, spec_lens, out_path, out_accept_len, *d,
                               path_stride, static_cast<hipStream_t>(stream)) != hipSuccess)
        return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

int adaspec_check_ragged_inputs(const int32_t *block_table, const int32_t *ctx_lens,
                                const int32_t *spec_lens, const adaspec_attn_dims *dims,
                                int32_t *err_flags, void *stream)
{
    int rc = validate_attn_dims(dims);
    if (rc != ADASPEC_OK) return rc;
    if (!block_table || !ctx_lens || !spec_lens || !err_flags) return ADASPEC_ERR_NULL;
    if (launch_check_ragged(block_table, ctx_lens, spec_lens, *dims, err_flags,
                            static_cast<hipStream_t>(stream)) != hipSuccess)
        return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

int adaspec_check_accept_inputs(const int32_t *draft_tokens, const int32_t *spec_lens, const float *temperature,
                                const adaspec_accept_dims *dims, int32_t *err_flags, void *stream)
{
    int rc = validate_accept_dims(dims);
    if (rc != ADASPEC_OK) return rc;
    if (!spec_lens || !temperature || !err_flags) return ADASPEC_ERR_NULL;
    if (dims->total_draft > 0 && !draft_tokens) return ADASPEC_ERR_NULL;
    if (launch_check_accept_inputs(draft_tokens, spec_lens, temperature, *dims, err_flags,
                                   static_cast<hipStream_t>(stream)) != hipSuccess)
        return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

int adaspec_check_tree_parents(const int32_t *parents, const int32_t *spec_lens, int32_t batch, int32_t total_q,
                               int32_t max_spec_len, int32_t *err_flags, void *stream)
{
    if (batch < 0 || total_q < batch || max_spec_len < 0) return ADASPEC_ERR_DIM;
    if ((int64_t)total_q > (int64_t)batch * (max_spec_len + 1)) return ADASPEC_ERR_DIM;
    if (max_spec_len > 63) return ADASPEC_ERR_UNSUPPORTED;
    if (!parents || !spec_lens || !err_flags) return ADASPEC_ERR_NULL;
    if (launch_check_tree_parents(parents, spec_lens, batch, total_q, max_spec_len, err_flags,
                                  static_cast<hipStream_t>(stream)) != hipSuccess)
        return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

int adaspec_kv_append(const void *k_new, const void *v_new, void *k_pages, void *v_pages,
                      const int32_t *block_table, const int32_t *ctx_lens,
                      const int32_t *spec_lens, const adaspec_attn_dims *d, void *stream)
{
    if (!d) return ADASPEC_ERR_NULL;
    if (d->batch < 0 || d->total_q < d->batch || d->max_spec_len < 0) return ADASPEC_ERR_DIM;
    if ((int64_t)d->total_q > (int64_t)d->batch * (d->max_spec_len + 1)) return ADASPEC_ERR_DIM;
    if (d->n_kv_heads <= 0 || d->head_dim <= 0 || d->page_size <= 0) return ADASPEC_ERR_DIM;
    if (d->num_pages <= 0 || d->max_pages_per_req <= 0) return ADASPEC_ERR_DIM;
    if (!dtype_ok(d->dtype)) return ADASPEC_ERR_DTYPE;
    if ((d->head_dim * (d->dtype == ADASPEC_F32 ? 4 : 2)) % 16) return ADASPEC_ERR_UNSUPPORTED;
    if (d->batch == 0) return ADASPEC_OK;
    if (!k_new || !v_new || !k_pages || !v_pages || !block_table || !ctx_lens || !spec_lens)
        return ADASPEC_ERR_NULL;
    if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(k_pages) || !aligned16(v_pages))
        return ADASPEC_ERR_ALIGN;
    if (launch_kv_append(k_new, v_new, k_pages, v_pages, block_table, ctx_lens, spec_lens, *d,
                         static_cast<hipStream_t>(stream)) != hipSuccess)
        return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

int adaspec_commit(const int32_t *out_tokens, const int32_t *out_accept_len,
                   const int32_t *spec_lens, const int32_t *ctx_lens,
                   const int32_t *next_spec_lens,
                   int32_t *committed_lens, int32_t *next_ctx_lens, int32_t *last_token,
                   int32_t *seq_tokens, int32_t *seq_lens,
                   const adaspec_commit_dims *d, void *stream)
{
    if (!d) return ADASPEC_ERR_NULL;
    if (d->batch < 0 || d->max_spec_len < 0 || d->seq_stride < 0) return ADASPEC_ERR_DIM;
    if (d->out_stride < d->max_spec_len + 1) return ADASPEC_ERR_DIM;
    if ((seq_tokens == nullptr) != (seq_lens == nullptr)) return ADASPEC_ERR_NULL;
    if (seq_tokens && d->seq_stride <= 0) return ADASPEC_ERR_DIM;
    if (d->batch == 0) return ADASPEC_OK;
    if (!out_tokens || !out_accept_len || !spec_lens || !ctx_lens || !committed_lens || !last_token)
        return ADASPEC_ERR_NULL;
    if (launch_commit(out_tokens, out_accept_len, spec_lens, ctx_lens, next_spec_lens, committed_lens,
                      next_ctx_lens, last_token, seq_tokens, seq_lens, *d,
                      static_cast<hipStream_t>(stream)) != hipSuccess)
        return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

static int validate_draft_dims(const adaspec_draft_dims *d)
{
    if (!d) return ADASPEC_ERR_NULL;
    if (d->rows < 0 || d->vocab <= 0) return ADASPEC_ERR_DIM;
    if (d->logits_row_stride < d->vocab || d->probs_row_stride < d->vocab) return ADASPEC_ERR_DIM;
    if (!dtype_ok(d->logits_dtype) || !dtype_ok(d->probs_dtype)) return ADASPEC_ERR_DTYPE;
    if (d->path < ADASPEC_PATH_AUTO || d->path > ADASPEC_PATH_TWO_PASS || d->path == ADASPEC_PATH_STREAM)
        return ADASPEC_ERR_DIM;
    return ADASPEC_OK;
}

size_t adaspec_draft_sample_workspace_bytes(const adaspec_draft_dims *d)
{
    if (validate_draft_dims(d) != ADASPEC_OK || d->rows == 0) return 0;
    if (d->vocab % 8 || d->logits_row_stride % 8 || d->probs_row_stride % 8 || !draft_split_supported(*d)) return 0;
    if (d->path == ADASPEC_PATH_VECTOR || d->path == ADASPEC_PATH_FAST) return 0;
    return draft_split_workspace_bytes(d->rows);
}

int adaspec_draft_sample(const void *draft_logits, const float *temperature, const float *uniforms,
                         const int32_t *out_rows, void *draft_probs, int32_t *draft_tokens,
                         float *confidence, const adaspec_draft_dims *d, void *workspace, size_t workspace_bytes,
                         void *stream)
{
    const int rc = validate_draft_dims(d);
    if (rc != ADASPEC_OK) return rc;
    if (d->rows == 0) return ADASPEC_OK;
    if (!draft_logits || !temperature || !uniforms || !draft_probs || !draft_tokens || !confidence)
        return ADASPEC_ERR_NULL;
    if (!aligned16(draft_logits) || !aligned16(draft_probs)) return ADASPEC_ERR_ALIGN;
    if (!draft_sample_supported(*d, draft_logits, draft_probs)) return ADASPEC_ERR_UNSUPPORTED;
    const bool fast_ok = draft_fast_supported(*d);
    const bool split_ok = draft_split_supported(*d);
    if (d->path == ADASPEC_PATH_FAST && !fast_ok) return ADASPEC_ERR_UNSUPPORTED;
    bool split = false;
    if (d->path == ADASPEC_PATH_TWO_PASS) {
        if (!split_ok) return ADASPEC_ERR_UNSUPPORTED;
        if (!workspace) return ADASPEC_ERR_NULL;
        if (reinterpret_cast<uintptr_t>(workspace) & 255u) return ADASPEC_ERR_ALIGN;
        if (workspace_bytes < draft_split_workspace_bytes(d->rows)) return ADASPEC_ERR_WORKSPACE;
        split = true;
    } else if (d->path == ADASPEC_PATH_AUTO) {
        // three small kernels against one long one: worth it once a row is long (measured on MI355X, 128 rows:
        // V = 128256 24 against 36 us)
        split = split_ok && d->vocab >= 32768 && workspace && !(reinterpret_cast<uintptr_t>(workspace) & 255u) &&
                workspace_bytes >= draft_split_workspace_bytes(d->rows);
    }
    const bool fast = !split && fast_ok && d->path != ADASPEC_PATH_VECTOR;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (!record_event(d->timing_start, d->timing_stop, true, st)) return ADASPEC_ERR_HIP;
    hipError_t e;
    if (split)
        e = launch_draft_split(draft_logits, temperature, uniforms, out_rows, draft_probs, draft_tokens, confidence, *d,
                               static_cast<char *>(workspace), st);
    else if (fast)
        e = launch_draft_fast(draft_logits, temperature, uniforms, out_rows, draft_probs, draft_tokens, confidence, *d, st);
    else
        e = launch_draft_sample(draft_logits, temperature, uniforms, out_rows, draft_probs, draft_tokens, confidence, *d, st);
    if (e != hipSuccess) return ADASPEC_ERR_HIP;
    if (!record_event(d->timing_start, d->timing_stop, false, st)) return ADASPEC_ERR_HIP;
    return ADASPEC_OK;
}

const char *adaspec_status_string(int status)
{
    switch (status) {
    case ADASPEC_OK: return "ok";
    case ADASPEC_ERR_NULL: return "a required pointer is NULL";
    case ADASPEC_ERR_DIM: return "a dimension is out of range or inconsistent";
    case ADASPEC_ERR_DTYPE: return "unknown or unsupported element type";
    case ADASPEC_ERR_ALIGN: return "pointer or stride is not aligned as required";
    case ADASPEC_ERR_WORKSPACE: return "workspace too small";
    case ADASPEC_ERR_UNSUPPORTED: return "shape not supported by the requested kernel path";
    case ADASPEC_ERR_HIP: return "a HIP call failed";
    default: return "unknown status";
    }
}

int adaspec_version(void) { return 100; }

}  // extern "C"
