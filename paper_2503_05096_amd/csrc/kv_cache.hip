// The two small steps on either side of a verification step (paper Sec. 6: paged KV cache of the
// target model; the results of one step become the input of the next):
//   kv_append_kernel - scatter the new tokens' K/V rows into their pages before verification,
//   commit_kernel    - after acceptance, keep the accepted entries and hand over the next input.
// Both move a few megabytes at most; they are written for low latency, not for bandwidth.
#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

constexpr int kKvThreads = 256;

// One workgroup per request.  It first adds up n_j = k_j + 1 over the requests before it (its first
// row in k_new / v_new), then copies its n_i rows, 16 bytes per thread and access:
// row j, kv head h  ->  page block_table[i][pos / P], head h, slot pos % P  with  pos = L_i - n_i + j.
__global__ __launch_bounds__(kKvThreads) void kv_append_kernel(
    const uint4 *__restrict__ k_new, const uint4 *__restrict__ v_new, uint4 *__restrict__ k_pages,
    uint4 *__restrict__ v_pages, const int32_t *__restrict__ block_table,
    const int32_t *__restrict__ ctx_lens, const int32_t *__restrict__ spec_lens, int total_q,
    int max_spec_len, int Hkv, int vec_per_row /* d * sizeof / 16 */, int P, int num_pages,
    int max_pages_per_req)
{
    __shared__ int wsum[kKvThreads / kWave];
    const int i = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int part = 0;
    for (int jj = tid; jj < i; jj += kKvThreads) part += min(max(spec_lens[jj], 0), max_spec_len) + 1;
    part = wave_sum(part);
    if (lane == 0) wsum[wv] = part;
    __syncthreads();
    int row0 = 0;
#pragma unroll
    for (int w = 0; w < kKvThreads / kWave; ++w) row0 += wsum[w];

    const int n = min(max(spec_lens[i], 0), max_spec_len) + 1;
    const int L = ctx_lens[i];
    if (L < n || row0 + n > total_q) return;            // inconsistent metadata: touch nothing
    const int per_token = Hkv * vec_per_row;            // 16-byte units of one token in one tensor
    for (int idx = tid; idx < n * per_token; idx += kKvThreads) {
        const int j = idx / per_token, rem = idx - j * per_token;
        const int h = rem / vec_per_row, c = rem - h * vec_per_row;
        const int pos = L - n + j;
        const int pg = pos / P;
        if (pg >= max_pages_per_req) continue;
        const int page = block_table[(int64_t)i * max_pages_per_req + pg];
        if (page < 0 || page >= num_pages) continue;
        const int64_t src = (int64_t)(row0 + j) * per_token + rem;
        const int64_t dst = (((int64_t)page * Hkv + h) * P + pos % P) * vec_per_row + c;
        k_pages[dst] = k_new[src];
        v_pages[dst] = v_new[src];
    }
}

hipError_t launch_kv_append(const void *k_new, const void *v_new, void *k_pages, void *v_pages,
                            const int32_t *block_table, const int32_t *ctx_lens,
                            const int32_t *spec_lens, const adaspec_attn_dims &d, hipStream_t stream)
{
    const int esize = d.dtype == ADASPEC_F32 ? 4 : 2;
    hipLaunchKernelGGL(kv_append_kernel, dim3(d.batch), dim3(kKvThreads), 0, stream,
                       (const uint4 *)k_new, (const uint4 *)v_new, (uint4 *)k_pages, (uint4 *)v_pages,
                       block_table, ctx_lens, spec_lens, d.total_q, d.max_spec_len, d.n_kv_heads,
                       d.head_dim * esize / 16, d.page_size, d.num_pages, d.max_pages_per_req);
    return hipGetLastError();
}

// One thread per request.
__global__ __launch_bounds__(kKvThreads) void commit_kernel(
    const int32_t *__restrict__ out_tokens, const int32_t *__restrict__ out_accept_len,
    const int32_t *__restrict__ spec_lens, const int32_t *ctx_lens,
    const int32_t *__restrict__ next_spec_lens, int32_t *committed_lens, int32_t *next_ctx_lens,
    int32_t *__restrict__ last_token, int32_t *__restrict__ seq_tokens, int32_t *__restrict__ seq_lens,
    int B, int max_spec_len, int out_stride, int seq_stride)
{
    const int i = blockIdx.x * kKvThreads + threadIdx.x;
    if (i >= B) return;
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const int a = min(max(out_accept_len[i], 0), k);
    const int kept = ctx_lens[i] - k + a;
    const int32_t *o = out_tokens + (int64_t)i * out_stride;
    committed_lens[i] = kept;
    if (next_ctx_lens && next_spec_lens) next_ctx_lens[i] = kept + next_spec_lens[i] + 1;
    last_token[i] = o[a];
    if (seq_tokens && seq_lens) {
        const int have = min(max(seq_lens[i], 0), seq_stride);
        const int room = seq_stride - have;
        const int put = min(a + 1, room);
        int32_t *sq = seq_tokens + (int64_t)i * seq_stride + have;
        for (int t = 0; t < put; ++t) sq[t] = o[t];
        seq_lens[i] = have + put;
    }
}

hipError_t launch_commit(const int32_t *out_tokens, const int32_t *out_accept_len,
                         const int32_t *spec_lens, const int32_t *ctx_lens,
                         const int32_t *next_spec_lens, int32_t *committed_lens,
                         int32_t *next_ctx_lens, int32_t *last_token, int32_t *seq_tokens,
                         int32_t *seq_lens, const adaspec_commit_dims &d, hipStream_t stream)
{
    hipLaunchKernelGGL(commit_kernel, dim3(ceil_div(d.batch, kKvThreads)), dim3(kKvThreads), 0, stream,
                       out_tokens, out_accept_len, spec_lens, ctx_lens, next_spec_lens, committed_lens,
                       next_ctx_lens, last_token, seq_tokens, seq_lens, d.batch, d.max_spec_len,
                       d.out_stride, d.seq_stride);
    return hipGetLastError();
}

}  // namespace adaspec
