// Verification of a draft-token TREE (several children per node) instead of a chain.
//
// The nodes of request i are its n_i query rows: node 0 = the last committed token, nodes 1..k_i
// the drafts, every parent before its children.  Three pieces live here:
//   * the ancestor masks the attention kernels read (one 64-bit mask per query row),
//   * the acceptance of every node (which child, if any, the walk would move to from this node,
//     and the token it would emit if it stopped here) and the walk that strings them together,
//   * the compaction of the accepted path's K/V rows after acceptance.
// A chain is the special case parent = previous node; on a chain the acceptance below performs
// the same float operations in the same order as the portable chain kernel.
#include "adaspec_internal.h"
#include "device_utils.h"
#include "tree_masks.h"

namespace adaspec {

// ---- ancestor masks ----------------------------------------------------------------------
// One wavefront per request, lane j = node j (tree_masks.h).  This kernel serves batches too large
// for the metadata kernel's own mask workgroups; it reads the row offsets that kernel wrote.
__global__ __launch_bounds__(256) void tree_mask_kernel(
    const int32_t *__restrict__ parents, const int32_t *__restrict__ spec_lens,
    const int32_t *__restrict__ cu_q, int B, int total_q, int max_spec_len,
    unsigned long long *__restrict__ anc)
{
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6), j = threadIdx.x & 63;
    if (i >= B) return;
    const int n = min(max(spec_lens[i], 0), max_spec_len) + 1;
    const int r0 = cu_q[i];
    if (r0 < 0 || r0 + n > total_q) return;             // inconsistent metadata: leave the rows alone
    tree_masks_of_request(parents, r0, n, j, anc);
}

hipError_t launch_tree_masks(const AttnArgs &a)
{
    const AttnPlan &p = a.plan;
    if (a.dims.batch == 0 || a.dims.batch <= kFusedMaskMaxBatch) return hipSuccess;   // none, or built by the metadata kernel
    hipLaunchKernelGGL(tree_mask_kernel, dim3(ceil_div(a.dims.batch, 4)), dim3(256), 0, a.stream, a.parents,
                       a.spec_lens, (const int32_t *)(a.ws + p.off_cu_q), a.dims.batch, a.dims.total_q,
                       a.dims.max_spec_len, (unsigned long long *)(a.ws + p.off_anc));
    return hipGetLastError();
}

// Device-side check of a parent array (see adaspec.h): bit 4 of *err_flags is set if some node j >= 1 of some
// request names a parent outside [0, j).  One thread per request; cu_q by a block scan, 256 requests at a time.
__global__ __launch_bounds__(256) void check_tree_parents_kernel(
    const int32_t *__restrict__ parents, const int32_t *__restrict__ spec_lens, int B, int total_q,
    int max_spec_len, int32_t *__restrict__ err_flags)
{
    __shared__ int wtot[4];
    __shared__ int bad;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    if (tid == 0) bad = 0;
    int carry = 0, mine_bad = 0;
    for (int base = 0; base < B; base += 256) {
        const int i = base + tid;
        const int n = i < B ? min(max(spec_lens[i], 0), max_spec_len) + 1 : 0;
        const int inc = wave_scan_incl(n, lane);
        __syncthreads();
        if (lane == 63) wtot[wv] = inc;
        __syncthreads();
        int pre = carry, tot = carry;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wv) pre += wtot[w];
            tot += wtot[w];
        }
        const int r0 = pre + inc - n;
        if (i < B && r0 + n <= total_q)
            for (int j = 1; j < n; ++j) {
                const int p = parents[r0 + j];
                if (p < 0 || p >= j) mine_bad = 1;
            }
        carry = tot;
    }
    if (mine_bad) atomicOr(&bad, 1);
    __syncthreads();
    if (tid == 0) *err_flags = bad ? 16 : 0;
}

hipError_t launch_check_tree_parents(const int32_t *parents, const int32_t *spec_lens, int B, int total_q,
                                     int max_spec_len, int32_t *err_flags, hipStream_t stream)
{
    hipLaunchKernelGGL(check_tree_parents_kernel, dim3(1), dim3(256), 0, stream, parents, spec_lens, B, total_q,
                       max_spec_len, err_flags);
    return hipGetLastError();
}

// ---- acceptance of one node --------------------------------------------------------------
// One workgroup of 256 threads per node (= logits row), any storage types, any vocabulary size.
//
// State of a node after s rejected children ("stage s"):
//   P_0 = softmax(logits / T);  r_s = max(0, P_{s-1} - q),  R_s = sum r_s  (r_s = P_{s-1} if that
//   sum is 0),  P_s = r_s / R_s.   Child number s+1 is tested against P_s; a token is drawn from
//   (r_s, R_s), at stage 0 from (P_0, sum P_0).
// A thread evaluates r_s at one vocabulary entry by running this recurrence from the logit: the
// 1/R_j of the earlier stages are scalars in LDS.  Every stage costs one sweep over the row for
// its total; the draw costs one more up to the tile where the prefix crosses.  Per-element
// arithmetic is fp32, every sum across threads and tiles fp64.
constexpr int kTT = 256;
constexpr int kTW = kTT / kWave;
constexpr int kTE = 4;                  // contiguous elements per thread per tile
constexpr int kTTile = kTT * kTE;
constexpr int kMaxNodes = 64;

struct TreeScratch {
    float  av[kTW];
    int    ai[kTW];
    double d[kTW];
    float  inv_r[kMaxNodes];            // 1 / R_s of the stages taken so far (index s, 1-based)
    unsigned long long kept;            // bit s: stage s found no positive part and kept P_{s-1}
    unsigned long long kids;            // children of this node
    int    verdict;                     // accept flag of the child under test
    int    hit;
};

template <class LT, class PT>
__global__ __launch_bounds__(kTT) void accept_tree_node_kernel(
    const void *__restrict__ logits, const void *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const int32_t *__restrict__ parents,
    const float *__restrict__ uniforms, const int32_t *__restrict__ spec_lens,
    const float *__restrict__ temperature, const int32_t *__restrict__ cu_q,
    const int32_t *__restrict__ row_req, int V, int max_spec_len, int64_t lstride, int64_t pstride,
    int32_t *__restrict__ node_next, int32_t *__restrict__ row_cand)
{
    __shared__ TreeScratch sm;
    const int tid = threadIdx.x, lane = tid & 63;
    const int r = blockIdx.x;
    const int i = row_req[r];
    const int r0 = cu_q[i];
    const int u = r - r0;                                       // this node
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const float T = temperature[i];
    const int64_t lrow = (int64_t)r * lstride;
    const int64_t prow = (int64_t)(r - i) * pstride;            // read only if the node has children (u < k)

    // children of u: lane c of the first wavefront looks at node c
    if (tid < kWave) {
        const bool child = lane > u && lane <= k && sane_parent(parents[r0 + lane], lane) == u;
        const unsigned long long kids = __builtin_amdgcn_ballot_w64(child);
        if (lane == 0) { sm.kids = kids; sm.kept = 0ull; sm.hit = 0; }
    }

    // sweep 1: maximum and its lowest index
    ArgMax best{-INFINITY, V};
    for (int v = tid; v < V; v += kTT) {
        const float l = load_as_float<LT>(logits, lrow + v);
        if (l > best.v) best = ArgMax{l, v};
    }
    best = wave_argmax(best);
    if (lane == 0) { sm.av[tid >> 6] = best.v; sm.ai[tid >> 6] = best.i; }
    __syncthreads();
    best = ArgMax{sm.av[0], sm.ai[0]};
#pragma unroll
    for (int w = 1; w < kTW; ++w) best = argmax_merge(best, ArgMax{sm.av[w], sm.ai[w]});
    if (best.i >= V) best.i = 0;
    unsigned long long kids = sm.kids;

    if (T == 0.0f) {
        // greedy: the first child that carries the target's arg-max, else stop with the arg-max
        if (tid == 0) {
            int next = -1;
            while (kids != 0ull && next < 0) {
                const int c = __builtin_ctzll(kids);
                kids &= kids - 1;
                if (draft_tokens[r0 - i + c - 1] == best.i) next = c;
            }
            node_next[r] = next;
            row_cand[r] = best.i;
        }
        return;
    }
    const float m = best.v;
    const float cexp = 1.4426950408889634f / T;

    auto block_sum = [&](double v) -> double {
        v = wave_sum(v);
        __syncthreads();
        if (lane == 0) sm.d[tid >> 6] = v;
        __syncthreads();
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kTW; ++w) s += sm.d[w];
        return s;
    };
    // exclusive / inclusive prefix over the 256 threads and the block total; excl of thread t+1 is
    // bit-identical to incl of thread t
    auto block_scan = [&](double v, double &excl, double &incl, double &total) {
        const double wi = wave_scan_incl(v, lane);
        double we = __shfl_up(wi, 1, kWave);
        if (lane == 0) we = 0.0;
        __syncthreads();
        if (lane == 63) sm.d[tid >> 6] = wi;
        __syncthreads();
        double wp = 0.0, run = 0.0;
#pragma unroll
        for (int w = 0; w < kTW; ++w) {
            if (w == (tid >> 6)) wp = run;
            run = run + sm.d[w];
        }
        excl = wp + we; incl = wp + wi; total = run;
    };

    // sweep 2: normaliser
    float zt = 0.f;
    for (int v = tid; v < V; v += kTT)
        zt += __builtin_amdgcn_exp2f((load_as_float<LT>(logits, lrow + v) - m) * cexp);
    const double Z = block_sum((double)zt);
    const float invZ = (float)(1.0 / Z);

    // P_s (the distribution child s+1 is tested against) and the stage's unnormalised mass r_s at
    // one entry.  `keep_last`: stage s itself keeps P_{s-1} (only known once its sum came out 0).
    int stage = 0;
    auto dist_at = [&](int v, int s) -> float {                 // P_s(v)
        float P = __builtin_amdgcn_exp2f((load_as_float<LT>(logits, lrow + v) - m) * cexp) * invZ;
        if (s > 0) {
            const float qv = load_as_float<PT>(probs, prow + v);
            const unsigned long long kept = sm.kept;
            for (int j = 1; j <= s; ++j) {
                const float rj = ((kept >> j) & 1ull) ? P : fmaxf(0.f, P - qv);
                P = rj * sm.inv_r[j];
            }
        }
        return P;
    };
    auto mass_at = [&](int v, int s, bool keep_last) -> float { // r_s(v); s == 0: P_0(v)
        if (s == 0) return dist_at(v, 0);
        const float P = dist_at(v, s - 1);
        return keep_last ? P : fmaxf(0.f, P - load_as_float<PT>(probs, prow + v));
    };
    auto total_mass = [&](int s, bool keep_last) -> double {    // tile by tile, as the draw sums it
        double running = 0.0;
        for (int tb = 0; tb < V; tb += kTTile) {
            const int v0 = tb + tid * kTE;
            float seg = 0.f;
#pragma unroll
            for (int e = 0; e < kTE; ++e)
                if (v0 + e < V) seg += mass_at(v0 + e, s, keep_last);
            double ex, in, tot;
            block_scan((double)seg, ex, in, tot);
            running = running + tot;
        }
        return running;
    };

    // the children, one after another
    int next = -1;
    double R = 0.0;                                             // total of the current stage's mass (stage > 0)
    bool keep_last = false;
    while (kids != 0ull) {
        const int c = __builtin_ctzll(kids);
        kids &= kids - 1;
        __syncthreads();                                        // sm.verdict of the previous child was read
        if (tid == 0) {
            const int x = draft_tokens[r0 - i + c - 1];
            const float px = dist_at(x, stage);
            const float qx = load_as_float<PT>(probs, prow + x);
            sm.verdict = (qx > 0.f) ? (uniforms[2 * (int64_t)(r0 + c - 1)] < px / qx) : 1;
        }
        __syncthreads();
        if (sm.verdict) { next = c; break; }
        // one more rejection
        ++stage;
        keep_last = false;
        R = total_mass(stage, false);
        if (!(R > 0.0)) {                                       // P == q everywhere: the state stays
            keep_last = true;
            R = total_mass(stage, true);
        }
        __syncthreads();
        if (tid == 0) {
            sm.inv_r[stage] = (float)(1.0 / R);
            if (keep_last) sm.kept |= 1ull << stage;
        }
        __syncthreads();
    }
    if (next >= 0) {
        if (tid == 0) { node_next[r] = next; row_cand[r] = best.i; }   // the token is never used
        return;
    }
    if (stage == 0) R = total_mass(0, false);                   // childless node: draw from P_0
    const double tau = (double)uniforms[2 * (int64_t)r + 1] * R;

    // the draw: first tile, thread and element where the inclusive prefix exceeds tau
    int cand = best.i;
    double running = 0.0;
    for (int tb = 0; tb < V; tb += kTTile) {
        const int v0 = tb + tid * kTE;
        float rv[kTE];
        float seg = 0.f;
#pragma unroll
        for (int e = 0; e < kTE; ++e) {
            rv[e] = (v0 + e < V) ? mass_at(v0 + e, stage, keep_last) : 0.f;
            seg += rv[e];
        }
        double ex, in, tot;
        block_scan((double)seg, ex, in, tot);
        if (running + tot > tau) {
            if (running + in > tau && !(running + ex > tau)) {
                double cum = running + ex;
                int pick = -1, lastpos = -1;
#pragma unroll
                for (int e = 0; e < kTE; ++e) {
                    cum += (double)rv[e];
                    if (rv[e] > 0.f) lastpos = v0 + e;
                    if (pick < 0 && cum > tau && rv[e] > 0.f) pick = v0 + e;
                }
                sm.hit = pick >= 0 ? pick : lastpos;
            }
            __syncthreads();
            cand = sm.hit;
            break;
        }
        running = running + tot;
    }
    if (tid == 0) { node_next[r] = -1; row_cand[r] = cand; }
}

// The walk: from the root along node_next until a node that stops; one thread per request.
__global__ __launch_bounds__(256) void accept_tree_walk_kernel(
    const int32_t *__restrict__ spec_lens, const int32_t *__restrict__ draft_tokens,
    const int32_t *__restrict__ cu_q, const int32_t *__restrict__ node_next,
    const int32_t *__restrict__ row_cand, int B, int total_q, int max_spec_len, int out_stride,
    int32_t *__restrict__ out_tokens, int32_t *__restrict__ out_accept_len, int32_t *__restrict__ out_path)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= B) return;
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const int r0 = cu_q[i];
    if (r0 < 0 || r0 + k + 1 > total_q) return;
    int32_t *o = out_tokens + (int64_t)i * out_stride;
    int32_t *pth = out_path + (int64_t)i * out_stride;
    int u = 0, depth = 0;
    for (;;) {
        const int nx = node_next[r0 + u];
        if (nx <= u || nx > k || depth >= k) break;             // -1, or anything that is not a later node
        o[depth] = draft_tokens[r0 - i + nx - 1];
        pth[depth] = nx;
        ++depth;
        u = nx;
    }
    o[depth] = row_cand[r0 + u];
    pth[depth] = -1;
    for (int j = depth + 1; j < out_stride; ++j) { o[j] = -1; pth[j] = -1; }
    out_accept_len[i] = depth;
}

hipError_t launch_accept_tree_walk(const AcceptArgs &a, int32_t *out_path)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.batch == 0) return hipSuccess;
    hipLaunchKernelGGL(accept_tree_walk_kernel, dim3(ceil_div(d.batch, 256)), dim3(256), 0, a.stream,
                       a.spec_lens, a.draft_tokens, (const int32_t *)(a.ws + a.plan.off_cu_q),
                       (const int32_t *)(a.ws + a.plan.off_row_flag), (const int32_t *)(a.ws + a.plan.off_row_cand),
                       d.batch, d.total_q, d.max_spec_len, d.out_stride, a.out_tokens, a.out_accept_len, out_path);
    return hipGetLastError();
}

hipError_t launch_accept_tree_nodes(const AcceptArgs &a, const int32_t *parents)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.total_q == 0) return hipSuccess;
    int32_t *node_next = (int32_t *)(a.ws + a.plan.off_row_flag);
    int32_t *row_cand = (int32_t *)(a.ws + a.plan.off_row_cand);
    const int32_t *cu_q = (const int32_t *)(a.ws + a.plan.off_cu_q);
    auto launch = [&](auto lt, auto pt) {
        using LT = decltype(lt);
        using PT = decltype(pt);
        hipLaunchKernelGGL((accept_tree_node_kernel<LT, PT>), dim3(d.total_q), dim3(kTT), 0, a.stream,
                           a.logits, a.probs, a.draft_tokens, parents, a.uniforms, a.spec_lens, a.temperature,
                           cu_q, (const int32_t *)(a.ws + a.plan.off_row_req), d.vocab, d.max_spec_len,
                           d.logits_row_stride, d.probs_row_stride, node_next, row_cand);
    };
    auto with_l = [&](auto lt) {
        if (d.probs_dtype == ADASPEC_F32) launch(lt, F32{});
        else if (d.probs_dtype == ADASPEC_F16) launch(lt, F16{});
        else launch(lt, BF16{});
    };
    if (d.logits_dtype == ADASPEC_F32) with_l(F32{});
    else if (d.logits_dtype == ADASPEC_F16) with_l(F16{});
    else with_l(BF16{});
    return hipGetLastError();
}

// ---- compaction of the accepted path ------------------------------------------------------
// The nodes' K/V rows were appended in node order at positions base + j, base = L - n.  The
// accepted nodes path[0] < path[1] < ... move to base + 1, base + 2, ...  One thread owns one
// 16-byte piece of a (kv head) row for one request and moves it for j = 0, 1, ... in turn:
// path[j] >= j + 1, so a destination is never a source that is still to be read.
__global__ __launch_bounds__(256) void kv_compact_path_kernel(
    char *__restrict__ k_pages, char *__restrict__ v_pages, const int32_t *__restrict__ block_table,
    const int32_t *__restrict__ ctx_lens, const int32_t *__restrict__ spec_lens,
    const int32_t *__restrict__ out_path, const int32_t *__restrict__ out_accept_len,
    int max_spec_len, int Hkv, int row_bytes, int P, int max_pages_per_req, int path_stride)
{
    const int i = blockIdx.y;
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const int a = min(max(out_accept_len[i], 0), k);
    const int base = ctx_lens[i] - (k + 1);
    const int pieces = row_bytes / 16;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;      // (kv head, piece)
    if (idx >= Hkv * pieces || base < 0) return;
    const int h = idx / pieces, off = (idx % pieces) * 16;
    const int32_t *bt = block_table + (int64_t)i * max_pages_per_req;
    int prev = 0;
    for (int j = 0; j < a; ++j) {
        const int node = out_path[(int64_t)i * path_stride + j];
        if (node <= prev || node > k) break;                    // not a path: stop
        prev = node;
        const int src = base + node, dst = base + 1 + j;
        if (src == dst) continue;
        const int64_t so = (((int64_t)bt[src / P] * Hkv + h) * P + src % P) * row_bytes + off;
        const int64_t dn = (((int64_t)bt[dst / P] * Hkv + h) * P + dst % P) * row_bytes + off;
        *reinterpret_cast<uint4 *>(k_pages + dn) = *reinterpret_cast<const uint4 *>(k_pages + so);
        *reinterpret_cast<uint4 *>(v_pages + dn) = *reinterpret_cast<const uint4 *>(v_pages + so);
    }
}

hipError_t launch_kv_compact_path(void *k_pages, void *v_pages, const int32_t *block_table,
                                  const int32_t *ctx_lens, const int32_t *spec_lens,
                                  const int32_t *out_path, const int32_t *out_accept_len,
                                  const adaspec_attn_dims &d, int path_stride, hipStream_t stream)
{
    const int row_bytes = d.head_dim * (d.dtype == ADASPEC_F32 ? 4 : 2);
    const int work = d.n_kv_heads * (row_bytes / 16);
    hipLaunchKernelGGL(kv_compact_path_kernel, dim3(ceil_div(work, 256), d.batch), dim3(256), 0, stream,
                       (char *)k_pages, (char *)v_pages, block_table, ctx_lens, spec_lens, out_path,
                       out_accept_len, d.max_spec_len, d.n_kv_heads, row_bytes, d.page_size,
                       d.max_pages_per_req, path_stride);
    return hipGetLastError();
}

}  // namespace adaspec
