// Ragged metadata for the attention call (row offsets, KV-split work list),
// the split-KV combine, and the optional device-side input check.
#include "adaspec_internal.h"
#include "device_utils.h"
#include "tree_masks.h"

namespace adaspec {

constexpr int kPlanThreads = 1024;
constexpr int kSchedItems = 8192;        // work items whose request and length the kernel keeps on chip
constexpr int kUnitFixedBlocks = 2;      // fixed cost of a unit (Q load, merge, output), in token blocks
constexpr int kBalancedRounds = 1;       // last rounds of the schedule that are assigned by accumulated work
static_assert(kMaxSchedW <= kPlanThreads, "one plan thread per workgroup of the schedule");

__host__ __device__ inline int log2_exact(int v)          // v is a power of two
{
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

// One workgroup.  cu_q = exclusive scan of n_i = spec_lens[i] + 1; split_base = exclusive scan of
// the per-request split counts ceil(L_i / S); a work item is one (request, split).  Values are
// clamped to the host-declared bounds so that inconsistent device data cannot make the library
// write outside its workspace.
//
// W > 0 (matrix-core kernel): writes row_rec, unit_meta, the schedule table and the header
// (cu_q and split_base only when asked for, or when the requests do not fit on chip).
// W = 0 (vector kernel): writes cu_q, split_base, item_req, item_order, row_rec and the header.
//
// The kernel is a chain of short dependent phases, so what it costs is latency: the barriers
// between phases wait for LDS traffic only (a full barrier would also wait until every global
// store of the phase before has been acknowledged, about a microsecond each time), and whatever a
// later phase needs again stays in LDS.  Only shapes too large for that (more than kPlanThreads
// requests, more than kSchedItems items) read their own global stores back, behind a full barrier.
__global__ __launch_bounds__(kPlanThreads) void attn_plan_kernel(
    const int32_t *__restrict__ ctx_lens, const int32_t *__restrict__ spec_lens, int B, int total_q,
    int max_spec_len, int split_log2, int block_log2, int max_items, int G, int32_t *__restrict__ header,
    int32_t *__restrict__ cu_q, int32_t *__restrict__ split_base, int32_t *__restrict__ item_req,
    int32_t *__restrict__ item_order, int32_t *__restrict__ unit_meta, int32_t *__restrict__ row_rec,
    int W, int Hkv, int n_row_groups, int rows_per_group, int32_t *__restrict__ sched, int cus,
    int want_cu_q, const int32_t *__restrict__ parents, unsigned long long *__restrict__ anc)
{
    if (blockIdx.x > 0) {
        // Tree calls (batches up to kFusedMaskMaxBatch): workgroups 1.. build the ancestor masks beside the
        // plan, one wavefront per request.  They share nothing with workgroup 0: each wavefront adds up the
        // rows of the requests before its own.
        const int i = (blockIdx.x - 1) * (kPlanThreads / kWave) + (threadIdx.x >> 6), lane = threadIdx.x & 63;
        if (i >= B) return;
        int part = 0;
        for (int j = lane; j < i; j += kWave) part += min(max(spec_lens[j], 0), max_spec_len) + 1;
        const int r0 = wave_sum(part);
        const int n = min(max(spec_lens[i], 0), max_spec_len) + 1;
        if (r0 + n > total_q) return;                   // inconsistent metadata: leave the rows alone
        tree_masks_of_request(parents, r0, n, lane, anc);
        return;
    }
    __shared__ int tot_n[kPlanThreads / kWave], tot_s[kPlanThreads / kWave];
    __shared__ int carry[2];
    __shared__ int hist[64];
    __shared__ int4 req[kPlanThreads];         // (L, n, cu_q, split_base) of the first kPlanThreads requests
    __shared__ uint16_t item_req_l[kSchedItems];                        // request of each item
    __shared__ uint8_t item_blocks[kSchedItems], item_groups[kSchedItems];   // per SORTED item: token blocks, row groups
    __shared__ int bins[kPlanThreads], wg_work[kPlanThreads], wave_tot[kPlanThreads / kWave];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int split_tokens = 1 << split_log2, block_tokens = 1 << block_log2;
    const bool fast = W > 0;
    const bool items_on_chip = max_items <= kSchedItems && B <= 65535;  // host-side bounds: uniform
    const bool reqs_on_chip = B <= kPlanThreads;
    if (tid == 0) { carry[0] = 0; carry[1] = 0; }
    lds_barrier();
    for (int base = 0; base < B; base += kPlanThreads) {
        const int i = base + tid;
        int n = 0, ns = 0, L = 1;
        if (i < B) {
            n = min(max(spec_lens[i], 0), max_spec_len) + 1;
            L = max(ctx_lens[i], 1);
            ns = (L + split_tokens - 1) >> split_log2;
        }
        const int inc_n = wave_scan_incl_dpp(n), inc_s = wave_scan_incl_dpp(ns);
        if (lane == 63) { tot_n[wv] = inc_n; tot_s[wv] = inc_s; }
        lds_barrier();
        int pre_n = carry[0], pre_s = carry[1];
#pragma unroll
        for (int w = 0; w < kPlanThreads / kWave; ++w) {   // fixed trip count: the reads go out together
            pre_n += w < wv ? tot_n[w] : 0;
            pre_s += w < wv ? tot_s[w] : 0;
        }
        const int my_q = pre_n + inc_n - n, my_s = pre_s + inc_s - ns;
        if (i < B) {
            // (want_cu_q: a later kernel of the call reads cu_q from the workspace, e.g. the tree masks)
            if (!fast || !reqs_on_chip || want_cu_q) { cu_q[i] = my_q; split_base[i] = my_s; }
            if (base == 0) req[tid] = make_int4(L, n, my_q, my_s);
            // record for the combine kernel: (request, number of splits, first split, first row index of
            // this query row inside its (item, kv head) partial block)
            for (int j = 0; j < n; ++j)
                if (my_q + j < total_q)
                    *reinterpret_cast<int4 *>(row_rec + 4 * (int64_t)(my_q + j)) = make_int4(i, ns, my_s, j * G);
            for (int s = 0; s < ns; ++s)
                if (my_s + s < max_items) {
                    if (items_on_chip) item_req_l[my_s + s] = (uint16_t)i;
                    if (!fast || !items_on_chip) item_req[my_s + s] = i;
                }
        }
        lds_barrier();
        if (tid == kPlanThreads - 1) { carry[0] = pre_n + inc_n; carry[1] = pre_s + inc_s; }
        lds_barrier();
    }
    if (tid == 0) {
        if (!fast) { cu_q[B] = carry[0]; split_base[B] = carry[1]; }
        header[0] = min(carry[1], max_items);   // number of work items
        header[1] = 0;                          // (unused)
    }
    // Schedule order: longest items first (counting sort on the length in token blocks), so that
    // the workgroups that take units last get the short items and the tail of the launch is short.
    const int n_items = min(carry[1], max_items);
    const int per_split = split_tokens >> block_log2;          // token blocks of a full split
    const int nbins = min(64, max(1, per_split));
    if (tid < 64) hist[tid] = 0;
    if (items_on_chip && reqs_on_chip) lds_barrier();
    else __syncthreads();                      // the phases below read global stores of the one above
    struct Item { int4 rq; int i, s, blocks, bin; };
    auto item_info = [&](int item) -> Item {
        Item it;
        it.i = items_on_chip ? (int)item_req_l[item] : item_req[item];
        if (it.i < kPlanThreads) it.rq = req[it.i];
        else
            it.rq = make_int4(max(ctx_lens[it.i], 1), min(max(spec_lens[it.i], 0), max_spec_len) + 1, cu_q[it.i],
                              split_base[it.i]);
        const int L = it.rq.x, ns = (L + split_tokens - 1) >> split_log2;
        it.s = item - it.rq.w;
        const int slen = split_len_of(L, ns, block_tokens);
        const int len = min(L, (it.s + 1) * slen) - it.s * slen;
        it.blocks = (max(len, 1) + block_tokens - 1) >> block_log2;
        // bin 0 = longest; with more than 64 blocks per split the length is scaled down to 64 bins
        const int scaled = per_split <= 64 ? it.blocks
                                           : (int)(((int64_t)max(len, 1) * nbins + split_tokens - 1) >> split_log2);
        it.bin = nbins - min(max(scaled, 1), nbins);
        return it;
    };
    Item mine;                                  // this thread's first item, kept for the second pass
    mine.i = -1;
    for (int item = tid; item < n_items; item += kPlanThreads) {
        const Item it = item_info(item);
        if (item == tid) mine = it;
        atomicAdd(&hist[it.bin], 1);
    }
    lds_barrier();
    if (tid < 64) {                            // exclusive prefix over the bins (one wavefront)
        const int c = tid < nbins ? hist[tid] : 0;
        const int inc = wave_scan_incl_dpp(c);
        hist[tid] = inc - c;
    }
    lds_barrier();
    for (int item = tid; item < n_items; item += kPlanThreads) {
        const Item it = item == tid ? mine : item_info(item);
        const int pos = atomicAdd(&hist[it.bin], 1);
        if (!fast) { item_order[pos] = item; continue; }
        int32_t *m = unit_meta + 8 * (int64_t)pos;
        *reinterpret_cast<int4 *>(m) =
            make_int4(it.i, it.s, (it.rq.x + split_tokens - 1) >> split_log2, it.rq.x);
        *reinterpret_cast<int4 *>(m + 4) = make_int4(it.rq.y, it.rq.z, item, 0);
        if (items_on_chip) {
            item_blocks[pos] = (uint8_t)min(it.blocks, 255);
            item_groups[pos] = (uint8_t)min(ceil_div(it.rq.y * G, rows_per_group), 255);
        }
    }
    if (!fast) return;

    // ---- static schedule of the matrix-core kernel ---------------------------------------------
    // Units (item, kv head, row group) in the sorted item order are handed out in rounds of W, one
    // per workgroup and round; thread w plays workgroup w.  Rounds alternate direction (round 0 is
    // the identity, round 1 the reverse, ...), which evens out the work when every workgroup takes
    // the same number of units.  The last kBalancedRounds rounds are assigned by accumulated work
    // instead.  What has to be even there is the work per COMPUTE UNIT, not per workgroup: the
    // workgroups resident on one compute unit share its load pipeline (the older one is served
    // first), and a compute unit finishes when its total is done.  Workgroups w, w + cus,
    // w + 2 cus, ... land on the same compute unit (the dispatcher fills the compute units in
    // order, one workgroup each, then starts over), so such a round is cut into sub-rounds of
    // `cus` units: in each the j-th longest unit goes to the compute unit with the j-th least
    // work, found by a counting sort.  The table only decides who computes what; results do not
    // depend on it, nor on the assumed placement.
    const int units_per_item = Hkv * n_row_groups;
    const int upi_log2 = (units_per_item & (units_per_item - 1)) == 0 ? log2_exact(units_per_item) : -1;
    const int total_units = n_items * units_per_item;
    const int rounds = ceil_div(total_units, W);
    if (tid == 0) header[2] = rounds;
    wg_work[tid] = 0;
    int shift = 0;                              // compute-unit work >> shift fits the bins
    {
        const int64_t most = (int64_t)rounds * ceil_div(W, cus) * (255 + kUnitFixedBlocks);
        while ((most >> shift) >= kPlanThreads) ++shift;
    }
    lds_barrier();                             // item_blocks / item_groups are complete
    auto take = [&](int r, int idx) {          // workgroup tid takes unit idx (if it exists) in round r
        int v = -1;
        if (idx < total_units) {
            v = idx;
            if (items_on_chip) {
                const int pos = upi_log2 >= 0 ? idx >> upi_log2 : idx / units_per_item;
                const int rg = n_row_groups == 1 ? 0 : idx % n_row_groups;
                if (rg < item_groups[pos]) wg_work[tid] += item_blocks[pos] + kUnitFixedBlocks;
            }
        }
        sched[(int64_t)r * W + tid] = v;
    };
    for (int r = 0; r < rounds; ++r) {
        if (!(r >= 1 && items_on_chip && rounds - r <= kBalancedRounds)) {
            if (tid < W) take(r, r * W + ((r & 1) ? (W - 1 - tid) : tid));
            continue;
        }
        for (int base = 0; base < W; base += cus) {
            const int c = tid - base;
            const bool active = c >= 0 && c < min(cus, W - base);
            if (r * W + base >= total_units) {  // nothing left for this sub-round
                if (active) take(r, total_units);
                continue;
            }
            lds_barrier();                      // wg_work of everything assigned so far
            bins[tid] = 0;
            int cu_work = 0;
            if (active)
                for (int w = c; w < W; w += cus) cu_work += wg_work[w];
            const int key = min(cu_work >> shift, kPlanThreads - 1);
            lds_barrier();
            if (active) atomicAdd(&bins[key], 1);
            lds_barrier();
            const int cnt = bins[tid], inc = wave_scan_incl_dpp(cnt);
            if (lane == 63) wave_tot[wv] = inc;
            lds_barrier();
            int pre = 0;
#pragma unroll
            for (int w = 0; w < kPlanThreads / kWave; ++w) pre += w < wv ? wave_tot[w] : 0;
            bins[tid] = pre + inc - cnt;
            lds_barrier();
            if (active) take(r, r * W + base + atomicAdd(&bins[key], 1));
        }
    }
}

hipError_t launch_attn_plan(const AttnArgs &a)
{
    const AttnPlan &p = a.plan;
    // tree calls: one more workgroup per 16 requests for the ancestor masks (see the kernel)
    const bool fused_masks = a.parents != nullptr && a.dims.batch <= kFusedMaskMaxBatch;
    const int mask_wgs = fused_masks ? ceil_div(a.dims.batch, kPlanThreads / kWave) : 0;
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1 + mask_wgs), dim3(kPlanThreads), 0, a.stream, a.ctx_lens,
                       a.spec_lens, a.dims.batch, a.dims.total_q, a.dims.max_spec_len,
                       log2_exact(p.split_tokens), log2_exact(p.block_tokens), p.max_items,
                       a.dims.n_q_heads / a.dims.n_kv_heads, (int32_t *)(a.ws + p.off_header),
                       (int32_t *)(a.ws + p.off_cu_q), (int32_t *)(a.ws + p.off_split_base),
                       (int32_t *)(a.ws + p.off_item_req), (int32_t *)(a.ws + p.off_item_order),
                       (int32_t *)(a.ws + p.off_unit_meta), (int32_t *)(a.ws + p.off_row_rec), a.sched_w,
                       a.dims.n_kv_heads, a.n_row_groups, a.rows_per_group, (int32_t *)(a.ws + p.off_sched),
                       a.sched_cus, (a.parents != nullptr && !fused_masks) ? 1 : 0, a.parents,
                       (unsigned long long *)(a.ws + p.off_anc));
    return hipGetLastError();
}

// Merge the per-split softmax states of one (query row, q head):
//   m* = max_s m_s,  out = sum_s 2^(m_s - m*) O_s / sum_s 2^(m_s - m*) l_s.
// One wavefront per (row, head); rows whose request has a single split were
// already finalised by the main kernel and are skipped.
__global__ __launch_bounds__(256) void attn_combine_kernel(
    const int32_t *__restrict__ row_rec, const float *__restrict__ part_ml,
    const float *__restrict__ part_o, void *__restrict__ out, int total_q, int Hq, int Hkv, int d,
    int max_rows, int out_dtype)
{
    const int unit = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (unit >= total_q * Hq) return;
    const int r = unit / Hq, h = unit % Hq;
    const int4 rec = *reinterpret_cast<const int4 *>(row_rec + 4 * (int64_t)r);   // (request, ns, first split, row base)
    const int ns = rec.y, s0 = rec.z;
    if (ns <= 1) return;
    const int G = Hq / Hkv, g = h / G, rr = rec.w + (h % G);
    const int64_t idx0 = ((int64_t)s0 * Hkv + g) * max_rows + rr;
    const int64_t step = (int64_t)Hkv * max_rows;                   // from one split's record to the next
    const int c0 = lane * 2;                                         // two adjacent channels per lane and pass
    // Four splits at a time: their (m, l) pairs and partial rows are all requested before any of them is
    // looked at (one memory round trip per group instead of two per split); groups are merged on line.
    float mrun = -INFINITY, den = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int sg = 0; sg < ns; sg += 4) {
        float2 ml[4], o[4][2];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            ml[u] = make_float2(-INFINITY, 0.f);
            o[u][0] = o[u][1] = make_float2(0.f, 0.f);
            if (sg + u < ns) {
                const int64_t idx = idx0 + (sg + u) * step;
                ml[u] = *reinterpret_cast<const float2 *>(part_ml + idx * 2);
#pragma unroll
                for (int e = 0; e < 2; ++e)
                    if (c0 + 128 * e < d) o[u][e] = *reinterpret_cast<const float2 *>(part_o + idx * d + c0 + 128 * e);
            }
        }
        float gm = mrun;
#pragma unroll
        for (int u = 0; u < 4; ++u) gm = fmaxf(gm, ml[u].x);
        const float keep = __builtin_amdgcn_exp2f(mrun - gm);       // 0 for the first group (mrun = -inf)
        den *= keep;
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[e] *= keep;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = __builtin_amdgcn_exp2f(ml[u].x - gm);   // 0 for a slot past the last split
            den += w * ml[u].y;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                acc[2 * e] += w * o[u][e].x;
                acc[2 * e + 1] += w * o[u][e].y;
            }
        }
        mrun = gm;
    }
    const float inv = 1.0f / den;
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int c = c0 + 128 * e;
        if (c < d) {
            store_out(out, ((int64_t)r * Hq + h) * d + c, acc[2 * e] * inv, out_dtype);
            store_out(out, ((int64_t)r * Hq + h) * d + c + 1, acc[2 * e + 1] * inv, out_dtype);
        }
    }
}

hipError_t launch_attn_combine(const AttnArgs &a)
{
    const AttnPlan &p = a.plan;
    const int units = a.dims.total_q * a.dims.n_q_heads;
    if (units == 0) return hipSuccess;
    // no request can have more than one split: every row was finalised by the main kernel
    if ((int64_t)a.dims.max_pages_per_req * a.dims.page_size <= p.split_tokens) return hipSuccess;
    hipLaunchKernelGGL(attn_combine_kernel, dim3(ceil_div(units, 4)), dim3(256), 0, a.stream,
                       (const int32_t *)(a.ws + p.off_row_rec), (const float *)(a.ws + p.off_part_ml),
                       (const float *)(a.ws + p.off_part_o), a.out, a.dims.total_q, a.dims.n_q_heads,
                       a.dims.n_kv_heads, a.dims.head_dim, p.max_rows, a.dims.out_dtype);
    return hipGetLastError();
}

// Device-side consistency check of the ragged metadata (see adaspec.h).
__global__ __launch_bounds__(256) void check_ragged_kernel(
    const int32_t *__restrict__ block_table, const int32_t *__restrict__ ctx_lens,
    const int32_t *__restrict__ spec_lens, int B, int total_q, int max_spec_len, int page_size,
    int num_pages, int max_pages_per_req, int32_t *__restrict__ err_flags)
{
    __shared__ int s_flags, s_rows;
    if (threadIdx.x == 0) { s_flags = 0; s_rows = 0; }
    __syncthreads();
    int flags = 0, rows = 0;
    for (int i = threadIdx.x; i < B; i += blockDim.x) {
        const int k = spec_lens[i], L = ctx_lens[i];
        if (k < 0 || k > max_spec_len) flags |= 1;
        const int n = k + 1;
        rows += n;
        const int pages = L > 0 ? ceil_div(L, page_size) : 0;
        if (L < n || pages > max_pages_per_req) { flags |= 2; continue; }
        for (int pg = 0; pg < pages; ++pg) {
            const int id = block_table[(int64_t)i * max_pages_per_req + pg];
            if (id < 0 || id >= num_pages) flags |= 4;
        }
    }
    atomicOr(&s_flags, flags);
    atomicAdd(&s_rows, rows);
    __syncthreads();
    if (threadIdx.x == 0) *err_flags = s_flags | (s_rows != total_q ? 8 : 0);
}

hipError_t launch_check_ragged(const int32_t *block_table, const int32_t *ctx_lens,
                               const int32_t *spec_lens, const adaspec_attn_dims &d,
                               int32_t *err_flags, hipStream_t stream)
{
    hipLaunchKernelGGL(check_ragged_kernel, dim3(1), dim3(256), 0, stream, block_table, ctx_lens,
                       spec_lens, d.batch, d.total_q, d.max_spec_len, d.page_size, d.num_pages,
                       d.max_pages_per_req, err_flags);
    return hipGetLastError();
}

}  // namespace adaspec
