// Ragged metadata for the attention call (row offsets, KV-split work list),
// the split-KV combine, and the optional device-side input check.
#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

constexpr int kPlanThreads = 1024;

// One workgroup.  cu_q = exclusive scan of n_i = spec_lens[i] + 1; split_base =
// exclusive scan of the per-request split counts ceil(L_i / S); row_req / item_req
// map a query row / a work item back to its request.  Values are clamped to the
// host-declared bounds so that inconsistent device data cannot make the library
// write outside its workspace.
__global__ __launch_bounds__(kPlanThreads) void attn_plan_kernel(
    const int32_t *__restrict__ ctx_lens, const int32_t *__restrict__ spec_lens, int B, int total_q,
    int max_spec_len, int split_tokens, int block_tokens, int max_items, int G, int32_t *__restrict__ header,
    int32_t *__restrict__ cu_q, int32_t *__restrict__ row_req, int32_t *__restrict__ split_base,
    int32_t *__restrict__ item_req, int32_t *__restrict__ item_order, int32_t *__restrict__ unit_meta,
    int32_t *__restrict__ row_rec)
{
    __shared__ int tot_n[kPlanThreads / kWave], tot_s[kPlanThreads / kWave];
    __shared__ int carry[2];
    __shared__ int hist[64];
    // per-request values of the first kPlanThreads requests stay in LDS: the item phase below then
    // needs no global round trip for them (later requests, if any, are read back from memory)
    __shared__ int4 req[kPlanThreads];         // (L, n, cu_q, split_base)
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) { carry[0] = 0; carry[1] = 0; }
    __syncthreads();
    for (int base = 0; base < B; base += kPlanThreads) {
        const int i = base + tid;
        int n = 0, ns = 0, L = 1;
        if (i < B) {
            n = min(max(spec_lens[i], 0), max_spec_len) + 1;
            L = max(ctx_lens[i], 1);
            ns = ceil_div(L, split_tokens);
        }
        const int inc_n = wave_scan_incl(n, lane), inc_s = wave_scan_incl(ns, lane);
        if (lane == 63) { tot_n[wv] = inc_n; tot_s[wv] = inc_s; }
        __syncthreads();
        int pre_n = carry[0], pre_s = carry[1];
        for (int w = 0; w < wv; ++w) { pre_n += tot_n[w]; pre_s += tot_s[w]; }
        const int my_q = pre_n + inc_n - n, my_s = pre_s + inc_s - ns;
        if (i < B) {
            cu_q[i] = my_q;
            split_base[i] = my_s;
            if (base == 0) req[tid] = make_int4(L, n, my_q, my_s);
            for (int j = 0; j < n; ++j)
                if (my_q + j < total_q) {
                    row_req[my_q + j] = i;
                    // record for the combine kernel: (request, number of splits, first split, first row index of
                    // this query row inside its (item, kv head) partial block)
                    *reinterpret_cast<int4 *>(row_rec + 4 * (int64_t)(my_q + j)) = make_int4(i, ns, my_s, j * G);
                }
            for (int s = 0; s < ns; ++s)
                if (my_s + s < max_items) item_req[my_s + s] = i;
        }
        __syncthreads();
        if (tid == kPlanThreads - 1) { carry[0] = pre_n + inc_n; carry[1] = pre_s + inc_s; }
        __syncthreads();
    }
    if (tid == 0) {
        cu_q[B] = carry[0];
        split_base[B] = carry[1];
        header[0] = min(carry[1], max_items);   // number of work items
        header[1] = 0;                          // ticket counter of the vector kernel
    }
    // Schedule order: longest items first (counting sort on the length in token blocks), so that
    // the workgroups that take units last get the short items and the tail of the launch is short.
    const int n_items = min(carry[1], max_items);
    const int nbins = min(64, max(1, split_tokens / block_tokens));
    if (tid < 64) hist[tid] = 0;
    __syncthreads();
    auto request_of = [&](int i) -> int4 {
        if (i < kPlanThreads) return req[i];
        return make_int4(max(ctx_lens[i], 1), min(max(spec_lens[i], 0), max_spec_len) + 1, cu_q[i], split_base[i]);
    };
    auto bin_of = [&](int item, const int4 &rq) {
        const int L = rq.x;
        const int ns = ceil_div(L, split_tokens), s = item - rq.w;
        const int slen = split_len_of(L, ns, block_tokens);
        const int len = min(L, (s + 1) * slen) - s * slen;
        const int scaled = (int)(((int64_t)max(len, 1) * nbins + split_tokens - 1) / split_tokens);
        return nbins - min(max(scaled, 1), nbins);   // bin 0 = longest
    };
    for (int item = tid; item < n_items; item += kPlanThreads) {
        const int4 rq = request_of(item_req[item]);
        atomicAdd(&hist[bin_of(item, rq)], 1);
    }
    __syncthreads();
    if (tid < 64) {                            // exclusive prefix over the bins (one wavefront)
        const int c = tid < nbins ? hist[tid] : 0;
        const int inc = wave_scan_incl(c, lane);
        hist[tid] = inc - c;
    }
    __syncthreads();
    for (int item = tid; item < n_items; item += kPlanThreads) {
        const int i = item_req[item];
        const int4 rq = request_of(i);
        const int pos = atomicAdd(&hist[bin_of(item, rq)], 1);
        item_order[pos] = item;
        int32_t *m = unit_meta + 8 * (int64_t)pos;
        *reinterpret_cast<int4 *>(m) = make_int4(i, item - rq.w, ceil_div(rq.x, split_tokens), rq.x);
        *reinterpret_cast<int4 *>(m + 4) = make_int4(rq.y, rq.z, item, 0);
    }
}

hipError_t launch_attn_plan(const AttnArgs &a)
{
    const AttnPlan &p = a.plan;
    hipLaunchKernelGGL(attn_plan_kernel, dim3(1), dim3(kPlanThreads), 0, a.stream, a.ctx_lens,
                       a.spec_lens, a.dims.batch, a.dims.total_q, a.dims.max_spec_len, p.split_tokens,
                       p.block_tokens, p.max_items, a.dims.n_q_heads / a.dims.n_kv_heads,
                       (int32_t *)(a.ws + p.off_header),
                       (int32_t *)(a.ws + p.off_cu_q), (int32_t *)(a.ws + p.off_row_req),
                       (int32_t *)(a.ws + p.off_split_base), (int32_t *)(a.ws + p.off_item_req),
                       (int32_t *)(a.ws + p.off_item_order), (int32_t *)(a.ws + p.off_unit_meta),
                       (int32_t *)(a.ws + p.off_row_rec));
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
    float mstar = -INFINITY;
    for (int s = 0; s < ns; ++s) mstar = fmaxf(mstar, part_ml[(idx0 + s * step) * 2]);
    float acc[4] = {0.f, 0.f, 0.f, 0.f}, den = 0.f;
    for (int s = 0; s < ns; ++s) {
        const int64_t idx = idx0 + s * step;
        const float2 ml = *reinterpret_cast<const float2 *>(part_ml + idx * 2);
        const float w = __builtin_amdgcn_exp2f(ml.x - mstar);
        den += w * ml.y;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
            const int c = c0 + 128 * e;
            if (c < d) {
                const float2 o = *reinterpret_cast<const float2 *>(part_o + idx * d + c);
                acc[2 * e] += w * o.x;
                acc[2 * e + 1] += w * o.y;
            }
        }
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
