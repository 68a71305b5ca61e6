// Portable vector-ALU verification attention: any of the three storage types,
// any head_dim that is a multiple of 8 up to 256.  One wavefront per
// (work item, kv head, chunk of 8 query rows).  It is the path for fp32 inputs
// and for shapes the matrix-core kernel does not take; speed is secondary here,
// clarity and generality come first.
//
// Per 64-token block:  lane <-> token for the scores (each lane walks its key
// row, the query rows are broadcast from LDS), wavefront reductions for the
// online-softmax statistics, then lane <-> channel for P.V (the 64 weights of a
// row are broadcast from LDS while the lanes read a value row coalesced).
#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

constexpr int kRC = 8;      // query rows per unit
constexpr int kMaxD = 256;

template <class T>
__global__ __launch_bounds__(64) void attn_vector_kernel(
    const void *__restrict__ q, const void *__restrict__ k_pages, const void *__restrict__ v_pages,
    const int32_t *__restrict__ block_table, const int32_t *__restrict__ ctx_lens,
    const int32_t *__restrict__ spec_lens, void *__restrict__ out, const int32_t *__restrict__ header,
    const int32_t *__restrict__ cu_q, const int32_t *__restrict__ split_base,
    const int32_t *__restrict__ item_req, const int32_t *__restrict__ item_order,
    const unsigned long long *__restrict__ anc, float *__restrict__ part_ml, float *__restrict__ part_o,
    int Hq, int Hkv, int d, int P, int max_pages_per_req, int max_rows, int n_row_chunks,
    int split_tokens, int block_tokens, float scale_log2, int out_dtype)
{
    __shared__ float qs[kRC][kMaxD];
    __shared__ float ps[kRC][64];
    const int lane = threadIdx.x;
    const int G = Hq / Hkv;
    const int n_items = header[0];
    const int total_units = n_items * Hkv * n_row_chunks;

    // Units are handed out statically (longest items first, strided over the grid): the metadata holds
    // no counter that a launch would use up, so a caller may reuse it for any number of layers.
    for (int ticket = blockIdx.x; ticket < total_units; ticket += gridDim.x) {
        const int rc = ticket % n_row_chunks;
        const int g = (ticket / n_row_chunks) % Hkv;
        const int item = item_order[ticket / (n_row_chunks * Hkv)];
        const int i = item_req[item];
        const int s0 = split_base[i], ns = split_base[i + 1] - s0, s = item - s0;
        const int L = ctx_lens[i], n = spec_lens[i] + 1;
        const int rows = n * G, r0 = rc * kRC;
        if (r0 >= rows) continue;
        const int slen = split_len_of(L, ns, block_tokens);
        const int t0 = s * slen, t1 = min(L, t0 + slen);
        const int64_t qbase = (int64_t)cu_q[i];

        // stage the query rows of this chunk: row r = j*G + hh  ->  token row j, q head g*G + hh
        __syncthreads();
        for (int idx = lane; idx < kRC * d; idx += 64) {
            const int r = r0 + idx / d, c = idx % d;
            float v = 0.f;
            if (r < rows) v = load_as_float<T>(q, ((qbase + r / G) * Hq + g * G + r % G) * d + c);
            qs[idx / d][c] = v;
        }
        __syncthreads();

        // tree verification (anc != NULL): bit a of a row's mask = the request's node a is the row's
        // node or one of its ancestors; of the new positions L - n + a a row sees exactly those
        unsigned long long am[kRC];
#pragma unroll
        for (int r = 0; r < kRC; ++r)
            am[r] = (anc && r0 + r < rows) ? anc[qbase + (r0 + r) / G] : 0ull;

        float m[kRC], l[kRC], acc[kRC][4];
#pragma unroll
        for (int r = 0; r < kRC; ++r) {
            m[r] = -INFINITY; l[r] = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[r][e] = 0.f;
        }

        for (int tb = t0; tb < t1; tb += 64) {
            const int t = tb + lane;
            const bool valid = t < t1;
            float sc[kRC];
#pragma unroll
            for (int r = 0; r < kRC; ++r) sc[r] = 0.f;
            if (valid) {
                const int64_t page = block_table[(int64_t)i * max_pages_per_req + t / P];
                const int64_t koff = ((page * Hkv + g) * P + t % P) * (int64_t)d;
                for (int c = 0; c < d; c += 8) {
                    float kv[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) kv[e] = load_as_float<T>(k_pages, koff + c + e);
#pragma unroll
                    for (int r = 0; r < kRC; ++r)
#pragma unroll
                        for (int e = 0; e < 8; ++e) sc[r] = fmaf(qs[r][c + e], kv[e], sc[r]);
                }
            }
            __syncthreads();   // previous block's ps[] fully consumed
#pragma unroll
            for (int r = 0; r < kRC; ++r) {
                const int row = r0 + r;
                const int pos = L - n + row / G;            // last token this row may see
                bool vis = valid && row < rows && t <= pos;
                if (anc && t >= L - n) vis = vis && ((am[r] >> ((t - (L - n)) & 63)) & 1ull) != 0;
                const float sv = vis ? sc[r] * scale_log2 : -INFINITY;
                const float bm = wave_max(sv);
                const float mn = fmaxf(m[r], bm);
                float p = 0.f, alpha = 1.f;
                if (mn > -INFINITY) {
                    alpha = __builtin_amdgcn_exp2f(m[r] - mn);   // m = -inf -> 0
                    p = vis ? __builtin_amdgcn_exp2f(sv - mn) : 0.f;
                }
                l[r] = l[r] * alpha + wave_sum(p);
                m[r] = mn;
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[r][e] *= alpha;
                ps[r][lane] = p;
            }
            __syncthreads();
            const int cnt = min(64, t1 - tb);
            for (int tt = 0; tt < cnt; ++tt) {
                const int tk = tb + tt;
                const int64_t page = block_table[(int64_t)i * max_pages_per_req + tk / P];
                const int64_t voff = ((page * Hkv + g) * P + tk % P) * (int64_t)d;
                float vv[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int c = lane + 64 * e;
                    vv[e] = c < d ? load_as_float<T>(v_pages, voff + c) : 0.f;
                }
#pragma unroll
                for (int r = 0; r < kRC; ++r) {
                    const float p = ps[r][tt];
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[r][e] = fmaf(p, vv[e], acc[r][e]);
                }
            }
        }

        // finish: a request with one split is final here; otherwise leave (m, l, O) for the combine
#pragma unroll
        for (int r = 0; r < kRC; ++r) {
            const int row = r0 + r;
            if (row >= rows) continue;
            if (ns == 1) {
                const float inv = 1.0f / l[r];
                const int64_t obase = ((qbase + row / G) * Hq + g * G + row % G) * (int64_t)d;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int c = lane + 64 * e;
                    if (c < d) store_out(out, obase + c, acc[r][e] * inv, out_dtype);
                }
            } else {
                const int64_t idx = ((int64_t)item * Hkv + g) * max_rows + row;
                if (lane == 0) { part_ml[idx * 2] = m[r]; part_ml[idx * 2 + 1] = l[r]; }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int c = lane + 64 * e;
                    if (c < d) part_o[idx * d + c] = acc[r][e];
                }
            }
        }
    }
}

hipError_t launch_attn_vector(const AttnArgs &a)
{
    const AttnPlan &p = a.plan;
    const adaspec_attn_dims &d = a.dims;
    const int n_row_chunks = ceil_div(p.max_rows, kRC);
    const int64_t max_units = (int64_t)p.max_items * d.n_kv_heads * n_row_chunks;
    if (max_units == 0) return hipSuccess;
    const int grid = (int)(max_units < 256 * 16 ? max_units : 256 * 16);
    auto launch = [&](auto tag) {
        using T = decltype(tag);
        hipLaunchKernelGGL(attn_vector_kernel<T>, dim3(grid), dim3(64), 0, a.stream, a.q, a.k_pages,
                           a.v_pages, a.block_table, a.ctx_lens, a.spec_lens, a.out,
                           (const int32_t *)(a.ws + p.off_header), (const int32_t *)(a.ws + p.off_cu_q),
                           (const int32_t *)(a.ws + p.off_split_base),
                           (const int32_t *)(a.ws + p.off_item_req),
                           (const int32_t *)(a.ws + p.off_item_order),
                           a.parents ? (const unsigned long long *)(a.ws + p.off_anc) : nullptr,
                           (float *)(a.ws + p.off_part_ml),
                           (float *)(a.ws + p.off_part_o), d.n_q_heads, d.n_kv_heads, d.head_dim,
                           d.page_size, d.max_pages_per_req, p.max_rows, n_row_chunks, p.split_tokens,
                           p.block_tokens, a.scale_log2, d.out_dtype);
    };
    if (d.dtype == ADASPEC_F32) launch(F32{});
    else if (d.dtype == ADASPEC_F16) launch(F16{});
    else launch(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec
