// Ragged metadata for the acceptance call and the final per-request scan that
// turns independent per-row results into the emitted token sequence.
#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

constexpr int kPlanThreads = 1024;

// cu_q = exclusive scan of spec_lens[i] + 1, row_req = request of each logits row.
__global__ __launch_bounds__(kPlanThreads) void accept_plan_kernel(
    const int32_t *__restrict__ spec_lens, const float *__restrict__ temperature,
    const int32_t *__restrict__ draft_tokens, int B, int total_q, int max_spec_len,
    int32_t *__restrict__ cu_q, int32_t *__restrict__ row_req, int32_t *__restrict__ row_meta)
{
    __shared__ int tot[kPlanThreads / kWave];
    __shared__ int carry;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < B; base += kPlanThreads) {
        const int i = base + tid;
        const int n = i < B ? min(max(spec_lens[i], 0), max_spec_len) + 1 : 0;
        const int inc = wave_scan_incl(n, lane);
        if (lane == 63) tot[wv] = inc;
        __syncthreads();
        int pre = carry;
        for (int w = 0; w < wv; ++w) pre += tot[w];
        const int mine = pre + inc - n;
        if (i < B) {
            cu_q[i] = mine;
            const int tbits = __float_as_int(temperature[i]);
            for (int j = 0; j < n; ++j) {
                const int r = mine + j;
                if (r >= total_q) break;
                row_req[r] = i;
                int32_t *m = row_meta + 8 * (int64_t)r;
                m[0] = i; m[1] = j; m[2] = n - 1;
                m[3] = j < n - 1 ? draft_tokens[r - i] : -1;
                m[4] = tbits; m[5] = j < n - 1 ? r - i : 0; m[6] = 0; m[7] = 0;
            }
        }
        __syncthreads();
        if (tid == kPlanThreads - 1) carry = pre + inc;
        __syncthreads();
    }
    if (tid == 0) cu_q[B] = carry;
}

hipError_t launch_accept_plan(const AcceptArgs &a)
{
    hipLaunchKernelGGL(accept_plan_kernel, dim3(1), dim3(kPlanThreads), 0, a.stream, a.spec_lens,
                       a.temperature, a.draft_tokens, a.dims.batch, a.dims.total_q, a.dims.max_spec_len,
                       (int32_t *)(a.ws + a.plan.off_cu_q), (int32_t *)(a.ws + a.plan.off_row_req),
                       (int32_t *)(a.ws + a.plan.off_row_meta));
    return hipGetLastError();
}

// Sequential rule applied to the per-row results: accepted drafts up to the
// first rejected row, then that row's candidate; if no row rejects, the bonus
// row's candidate.  One workgroup; it scans spec_lens itself (cu_q), so it does
// not depend on the plan kernel; one thread per request, 1024 requests at a time.
__global__ __launch_bounds__(kPlanThreads) void accept_emit_kernel(
    const int32_t *__restrict__ spec_lens, const int32_t *__restrict__ draft_tokens,
    const int32_t *__restrict__ row_flag, const int32_t *__restrict__ row_cand, int B, int total_q,
    int max_spec_len, int out_stride, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ out_accept_len)
{
    __shared__ int tot[kPlanThreads / kWave];
    __shared__ int carry;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < B; base += kPlanThreads) {
        const int i = base + tid;
        const int k = i < B ? min(max(spec_lens[i], 0), max_spec_len) : -1;
        const int n = k + 1;
        const int inc = wave_scan_incl(n, lane);
        if (lane == 63) tot[wv] = inc;
        __syncthreads();
        int pre = carry;
        for (int w = 0; w < wv; ++w) pre += tot[w];
        const int r0 = pre + inc - n;
        if (i < B && r0 + n <= total_q) {
            const int d0 = r0 - i;
            int32_t *o = out_tokens + (int64_t)i * out_stride;
            // flags and draft tokens of the request are requested eight at a time BEFORE any of them is
            // looked at (a loop that stops at the first rejection would pay one memory round trip per draft);
            // the drafts are copied provisionally and everything from the stop position on is overwritten
            int a = k;
            int cand = row_cand[r0 + k];          // the bonus row's token, replaced below if a draft is rejected
            for (int j0 = 0; j0 < k; j0 += 8) {
                int f[8], t[8], c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const bool in = j0 + u < k;
                    f[u] = in ? row_flag[r0 + j0 + u] : 1;
                    t[u] = in ? draft_tokens[d0 + j0 + u] : -1;
                    c[u] = in ? row_cand[r0 + j0 + u] : -1;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    if (j0 + u < k) {
                        if (a == k && f[u] == 0) { a = j0 + u; cand = c[u]; }
                        o[j0 + u] = t[u];
                    }
                }
            }
            o[a] = cand;
            for (int j = a + 1; j < out_stride; ++j) o[j] = -1;
            out_accept_len[i] = a;
        }
        __syncthreads();
        if (tid == kPlanThreads - 1) carry = pre + inc;
        __syncthreads();
    }
}

hipError_t launch_accept_emit(const AcceptArgs &a)
{
    hipLaunchKernelGGL(accept_emit_kernel, dim3(1), dim3(kPlanThreads), 0, a.stream, a.spec_lens,
                       a.draft_tokens, (const int32_t *)(a.ws + a.plan.off_row_flag),
                       (const int32_t *)(a.ws + a.plan.off_row_cand), a.dims.batch, a.dims.total_q,
                       a.dims.max_spec_len, a.dims.out_stride, a.out_tokens, a.out_accept_len);
    return hipGetLastError();
}

// Device-side consistency check of the acceptance inputs (see adaspec.h).
__global__ __launch_bounds__(256) void check_accept_inputs_kernel(
    const int32_t *__restrict__ draft_tokens, const int32_t *__restrict__ spec_lens,
    const float *__restrict__ temperature, int B, int total_q, int total_draft, int max_spec_len, int V,
    int32_t *__restrict__ err_flags)
{
    __shared__ int s_flags, s_rows;
    if (threadIdx.x == 0) { s_flags = 0; s_rows = 0; }
    __syncthreads();
    int flags = 0, rows = 0;
    for (int i = threadIdx.x; i < B; i += blockDim.x) {
        const int k = spec_lens[i];
        if (k < 0 || k > max_spec_len) flags |= 1;
        rows += k + 1;
        const float T = temperature[i];
        if (!(T >= 0.0f) || isinf(T)) flags |= 64;
    }
    for (int j = threadIdx.x; j < total_draft; j += blockDim.x) {
        const int x = draft_tokens[j];
        if (x < 0 || x >= V) flags |= 32;
    }
    atomicOr(&s_flags, flags);
    atomicAdd(&s_rows, rows);
    __syncthreads();
    if (threadIdx.x == 0) *err_flags = s_flags | (s_rows != total_q ? 8 : 0);
}

hipError_t launch_check_accept_inputs(const int32_t *draft_tokens, const int32_t *spec_lens, const float *temperature,
                                      const adaspec_accept_dims &d, int32_t *err_flags, hipStream_t stream)
{
    hipLaunchKernelGGL(check_accept_inputs_kernel, dim3(1), dim3(256), 0, stream, draft_tokens, spec_lens, temperature,
                       d.batch, d.total_q, d.total_draft, d.max_spec_len, d.vocab, err_flags);
    return hipGetLastError();
}

}  // namespace adaspec
