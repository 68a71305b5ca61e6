// Two-pass acceptance, second pass for batches of up to 256 requests: the sampling step on the one row
// per request that decides its token, with the row cut into four parts.
//
// A row of V = 128 K elements costs one compute unit about 12 us of vector-ALU time per sweep, and a
// pass with one workgroup per request is as slow as that one row.  So four workgroups share the row
// (accept_partial_kernel: each adds up the residual mass of its part per (step, wavefront)), and a
// small kernel per request (accept_pick_kernel) finds the (part, step, wavefront) that holds
// tau = u1 * R from those sums, recomputes that one wavefront's 64 chunks and picks the element.
//
//   first pass (accept_stream.hip, test-only form): flag of every draft row, (m, Z) of the sampled
//       draft rows, arg-max of the greedy ones
//   accept_partial_kernel, workgroup (request i, part h): first row of i (block sum of n), first
//       rejected draft a (ballot over the flags) -> deciding row r; h = 0 also writes the accepted
//       drafts, the padding and the length.  Rejected draft: (m, Z) from the first pass; bonus row:
//       maximum and normaliser of its own part from registers.  Then per step of 8192 elements
//       r_v = max(0, 2^((l_v - m) c) / Z - q_v) and p_v, summed over 16-lane rows (fp32) and written
//       as they are: four row sums per (step, wavefront) and kind.
//   accept_pick_kernel, one workgroup per request: thread (part, step, wavefront) adds its four row
//       sums in fp64 and puts the parts on one scale (a bonus row's parts have their own (m, Z));
//       one wavefront scans the steps, then the wavefronts of the step, then the 64 lanes of the
//       wavefront (same expressions and order as the partial kernel), and the owning lane walks its
//       8 elements.  R == 0 on a rejected draft (p == q everywhere): the same search on p.
// Outputs equal those of the other acceptance paths up to the rounding of the partial sums.
#include "adaspec_internal.h"
#include "device_utils.h"
#include "row_registers.h"

namespace adaspec {

constexpr int kPT = 1024;                // threads of a partial-sum workgroup
constexpr int kPW = kPT / kWave;         // its 16 wavefronts
constexpr int kRowSteps = 16;            // steps of 8192 elements in the longest row (V <= 131072)
constexpr int kPickT = kRowSteps * kPW;  // pick kernel: one thread per (part, step, wavefront)

// A row is cut into PARTS parts (2 or 4) of kRowSteps / PARTS steps at most.
// part: float[B][PARTS][kRowSteps / PARTS][kPW][2 kinds (residual, p)][4 rows of 16 lanes]
template <int PARTS>
__device__ __forceinline__ size_t part_index(int i, int h, int it, int w, int kind)
{
    return ((((size_t)(i * PARTS + h) * (kRowSteps / PARTS) + it) * kPW + w) * 2 + kind) * 4;
}

struct PartGeometry {
    int part_steps;     // steps of kPT chunks per part
    int chunk0;         // first 16-byte chunk of the part inside the row
    int nchunks;        // chunks of the part (0: the row ends before it)
};
template <int PARTS>
__device__ __forceinline__ PartGeometry part_geometry(int V, int h)
{
    PartGeometry g;
    const int row_chunks = V >> 3, steps = ceil_div(row_chunks, kPT);
    g.part_steps = ceil_div(steps, PARTS);
    g.chunk0 = h * g.part_steps * kPT;
    g.nchunks = min(max(row_chunks - g.chunk0, 0), g.part_steps * kPT);
    return g;
}

// One 16-byte chunk (8 elements): residual r_v = max(0, e_v / Z - q_v) and p_v = e_v / Z with
// e_v = 2^(l_v c - m c).  Both kernels call this, so that the sums of the first and the search of
// the second see the same numbers.
template <class P>
__device__ __forceinline__ void chunk_masses(const uint4 &lv, const uint4 &qv, float c, float mc, float invZ,
                                             float (&rv)[8], float (&pv)[8])
{
    const uint32_t w[4] = {lv.x, lv.y, lv.z, lv.w}, qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float ea = __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mc));
        const float eb = __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mc));
        rv[2 * e] = fmaxf(0.f, fmaf(ea, invZ, -P::lo(qw[e])));
        rv[2 * e + 1] = fmaxf(0.f, fmaf(eb, invZ, -P::hi(qw[e])));
        pv[2 * e] = ea * invZ;
        pv[2 * e + 1] = eb * invZ;
    }
}

template <class DT, int PARTS>
__global__ __launch_bounds__(kPT, PARTS == 4 ? 8 : 4) void accept_partial_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const int32_t *__restrict__ spec_lens,
    const float *__restrict__ temperature, int V, int max_spec_len, int64_t lstride, int64_t pstride,
    const int32_t *__restrict__ row_flag, const RowStat *__restrict__ row_stat, int out_stride,
    int32_t *__restrict__ out_tokens, int32_t *__restrict__ out_accept_len, int2 *__restrict__ req_pick,
    float *__restrict__ part, HalfStat *__restrict__ half_stat)
{
    using P = Pair16<DT>;
    constexpr int kPSteps = kRowSteps / PARTS;
    __shared__ int s_ahead[kPW];
    __shared__ float s_m[kPW], s_z[kPW];
    __shared__ int s_ai[kPW];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i = blockIdx.x / PARTS, h = blockIdx.x % PARTS;

    // ---- the request's deciding row (as in the resolve form of accept_fast_kernel) ----------------
    int ahead = 0;
    for (int base = 0; base < i; base += kPT) {
        const int idx = base + tid;
        if (idx < i) ahead += min(max(spec_lens[idx], 0), max_spec_len) + 1;
    }
    const int k = min(max(spec_lens[i], 0), max_spec_len);       // uniform: scalar loads
    const float T = temperature[i];
    ahead = wave_sum(ahead);
    if (lane == 0) s_ahead[wv] = ahead;
    lds_barrier();
    int start = 0;
#pragma unroll
    for (int w = 0; w < kPW; ++w) start += s_ahead[w];
    start = __builtin_amdgcn_readfirstlane(start);
    int a = k;
    for (int j0 = 0; j0 < k; j0 += kWave) {
        const int f = j0 + lane < k ? row_flag[start + j0 + lane] : 1;
        const unsigned long long rej = __ballot(f == 0);
        if (rej) { a = j0 + (int)__builtin_ctzll(rej); break; }
    }
    a = __builtin_amdgcn_readfirstlane(a);
    const int r = start + a;
    const bool bonus = a >= k;
    if (h == 0 && wv == 0) {                  // everything but the sampled token
        int32_t *o = out_tokens + (int64_t)i * out_stride;
        for (int jj = lane; jj < out_stride; jj += kWave)
            if (jj != a) o[jj] = jj < a ? draft_tokens[start - i + jj] : -1;
        if (lane == 0) { out_accept_len[i] = a; req_pick[i] = make_int2(r, a); }
    }
    if (T == 0.0f && !bonus) return;          // greedy and rejected: the first pass left the row's arg-max

    const PartGeometry g = part_geometry<PARTS>(V, h);
    float *my_part = part + part_index<PARTS>(i, h, 0, 0, 0);
    HalfStat *my_stat = half_stat + i * PARTS + h;
    auto nothing_here = [&]() {               // the row ends before this half, or the half holds no finite logit
        for (int t = tid; t < kPSteps * kPW * 8; t += kPT) my_part[t] = 0.f;
        if (tid == 0) { HalfStat st; st.m = -INFINITY; st.arg = -1; st.Z = 1.0; *my_stat = st; }
    };
    if (g.nchunks == 0) { nothing_here(); return; }

    // ---- the half row (and its draft probabilities) into registers --------------------------------
    const char *lrow = logits + (int64_t)r * lstride * 2 + (int64_t)g.chunk0 * 16;
    const char *prow = probs + (int64_t)(r - i) * pstride * 2 + (int64_t)g.chunk0 * 16;
    const bool sampled = T != 0.0f, has_q = sampled && !bonus;
    const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(lrow), 0, g.nchunks * 16, 0x00020000);
    // (a bonus row has no draft probabilities: descriptor of size zero, the loads return zeros)
    const __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(prow), 0, has_q ? g.nchunks * 16 : 0, 0x00020000);
    const uint32_t tid16 = (uint32_t)tid * 16u;
    auto load_chunk = [&](const __amdgpu_buffer_rsrc_t &rs, int it) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)tid16, it * (kPT * 16), 0);
        return make_uint4(v.x, v.y, v.z, v.w);
    };
    uint4 lg[kPSteps], qg[kPSteps];
#pragma unroll
    for (int it = 0; it < kPSteps; ++it) lg[it] = load_chunk(rl, it);
#pragma unroll
    for (int it = 0; it < kPSteps; ++it) qg[it] = load_chunk(rq, it);
    float m = 0.f;
    double Zd = 1.0;
    if (has_q) { m = row_stat[r].m; Zd = row_stat[r].Z; }         // scalar loads
#pragma unroll
    for (int it = 0; it < kPSteps; ++it) {                        // chunks past the end arrive as zeros: -inf
        const uint32_t ninf = (it * kPT + tid >= g.nchunks) ? P::kNegInf2 : 0u;
        lg[it].x |= ninf; lg[it].y |= ninf; lg[it].z |= ninf; lg[it].w |= ninf;
    }

    if (!sampled) {
        // greedy bonus row: arg-max of the half (lowest index on ties); the pick kernel merges the halves
        ArgMax best{-INFINITY, V};
#pragma unroll
        for (int it = 0; it < kPSteps; ++it) {
            keep_packed(lg[it]);
            const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
            const int base = (g.chunk0 + it * kPT + tid) * 8;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float x0 = P::lo(w[e]), x1 = P::hi(w[e]);
                if (x0 > best.v) best = ArgMax{x0, base + 2 * e};
                if (x1 > best.v) best = ArgMax{x1, base + 2 * e + 1};
            }
        }
        best = wave_argmax(best);
        if (lane == 0) { s_m[wv] = best.v; s_ai[wv] = best.i; }
        __syncthreads();
        if (tid == 0) {
            ArgMax b{s_m[0], s_ai[0]};
            for (int w = 1; w < kPW; ++w) b = argmax_merge(b, ArgMax{s_m[w], s_ai[w]});
            HalfStat st; st.m = b.v; st.arg = b.i < V ? b.i : -1; st.Z = 0.0; *my_stat = st;
        }
        return;
    }

    const float c = 1.4426950408889634f / T;
    if (bonus) {
        // maximum and normaliser of this half alone (the pick kernel puts the two halves on one scale)
        float mx = -INFINITY;
#pragma unroll
        for (int it = 0; it < kPSteps; ++it) {
            keep_packed(lg[it]);                                  // (the row stays packed between the sweeps)
            const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) mx = fmaxf(mx, fmaxf(P::lo(w[e]), P::hi(w[e])));
        }
        mx = wave_max(mx);
        if (lane == 0) s_m[wv] = mx;
        lds_barrier();
        m = s_m[0];
#pragma unroll
        for (int w = 1; w < kPW; ++w) m = fmaxf(m, s_m[w]);
        if (!(m > -INFINITY)) { nothing_here(); return; }
        const float mc0 = m * c;
        float z = 0.f;
#pragma unroll
        for (int it = 0; it < kPSteps; ++it) {
            keep_packed(lg[it]);
            const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                z += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mc0));
                z += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mc0));
            }
        }
        z = wave_sum(z);
        if (lane == 0) s_z[wv] = z;
        lds_barrier();
        Zd = 0.0;
#pragma unroll
        for (int w = 0; w < kPW; ++w) Zd += (double)s_z[w];
    }
    const float mc = m * c;
    const float invZ = (float)(1.0 / Zd);

    // ---- residual and probability mass per (step, wavefront, row of 16 lanes) ----------------------
#pragma unroll
    for (int it = 0; it < kPSteps; ++it) {
        float rv[8], pv[8], acc_r = 0.f, acc_p = 0.f;
        keep_packed(lg[it]);
        keep_packed(qg[it]);
        chunk_masses<P>(lg[it], qg[it], c, mc, invZ, rv, pv);
#pragma unroll
        for (int e = 0; e < 8; ++e) { acc_r += rv[e]; acc_p += pv[e]; }
        acc_r = row16_sum(acc_r);
        acc_p = row16_sum(acc_p);
        if ((lane & 15) == 0) {
            part[part_index<PARTS>(i, h, it, wv, 0) + (lane >> 4)] = acc_r;
            part[part_index<PARTS>(i, h, it, wv, 1) + (lane >> 4)] = acc_p;
        }
    }
    if (tid == 0) { HalfStat st; st.m = m; st.arg = 0; st.Z = Zd; *my_stat = st; }
}

template <class DT, int PARTS>
__global__ __launch_bounds__(kPickT) void accept_pick_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs, const float *__restrict__ uniforms,
    const int32_t *__restrict__ spec_lens, const float *__restrict__ temperature, int V, int max_spec_len,
    int64_t lstride, int64_t pstride, const int32_t *__restrict__ row_cand, int out_stride,
    int32_t *__restrict__ out_tokens, const int2 *__restrict__ req_pick, const float *__restrict__ part,
    const HalfStat *__restrict__ half_stat)
{
    using P = Pair16<DT>;
    constexpr int kPSteps = kRowSteps / PARTS;
    __shared__ double mass[PARTS][kPSteps][kPW];
    __shared__ double s_tau, s_before;
    __shared__ int s_step, s_retry;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i = blockIdx.x;
    const int2 pk = req_pick[i];              // (deciding row, accepted drafts): scalar loads from here on
    const int r = pk.x, a = pk.y;
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const float T = temperature[i];
    const bool bonus = a >= k;
    int32_t *o = out_tokens + (int64_t)i * out_stride + a;
    HalfStat st[PARTS];
#pragma unroll
    for (int p = 0; p < PARTS; ++p) st[p] = half_stat[i * PARTS + p];
    if (T == 0.0f) {
        if (tid == 0) {
            int tok = 0;
            if (!bonus) tok = row_cand[r];
            else {
                ArgMax b{-INFINITY, V};
#pragma unroll
                for (int p = 0; p < PARTS; ++p)
                    if (st[p].arg >= 0) b = argmax_merge(b, ArgMax{st[p].m, st[p].arg});
                tok = b.i < V ? b.i : 0;
            }
            *o = tok;
        }
        return;
    }

    // thread (part, step, wavefront): its residual and probability mass, all parts on one scale
    const int h = tid / (kPSteps * kPW), it = (tid / kPW) % kPSteps, w = tid % kPW;
    const float4 pr = *reinterpret_cast<const float4 *>(part + part_index<PARTS>(i, h, it, w, 0));
    const float4 pp = *reinterpret_cast<const float4 *>(part + part_index<PARTS>(i, h, it, w, 1));
    const float c = 1.4426950408889634f / T;
    float M = st[0].m;
#pragma unroll
    for (int p = 1; p < PARTS; ++p) M = fmaxf(M, st[p].m);
    // p_v of part h was computed as 2^((l_v - m_h) c) / Z_h: times Z_h 2^((m_h - M) c) it is relative to M in
    // every part (a rejected draft row has the same (m, Z) in all: a common factor, which tau absorbs)
    double sc[PARTS];
#pragma unroll
    for (int p = 0; p < PARTS; ++p)
        sc[p] = st[p].m > -INFINITY ? st[p].Z * (double)__builtin_amdgcn_exp2f((st[p].m - M) * c) : 0.0;
    double my_sc = sc[0];
#pragma unroll
    for (int p = 1; p < PARTS; ++p)
        if (h == p) my_sc = sc[p];
    const double res = (((double)pr.x + (double)pr.y) + ((double)pr.z + (double)pr.w)) * my_sc;
    const double pm = (((double)pp.x + (double)pp.y) + ((double)pp.z + (double)pp.w)) * my_sc;
    const int steps = ceil_div(V >> 3, kPT), part_steps = part_geometry<PARTS>(V, 0).part_steps;
    const float u_draw = uniforms[2 * (int64_t)r + 1];
    bool use_p = bonus;                       // (for a bonus row the two sums are the same numbers)
    for (int attempt = 0; attempt < 2; ++attempt) {
        mass[h][it][w] = use_p ? pm : res;
        __syncthreads();
        if (wv == 0) {
            // lane L owns step L of the row: total over its wavefronts, running totals over the steps, R,
            // and the step whose running total first exceeds tau
            const int hh = lane / part_steps, ii = lane % part_steps;
            double t = 0.0;
            if (lane < steps) {
#pragma unroll
                for (int ww = 0; ww < kPW; ++ww) t = t + mass[hh][ii][ww];
            }
            const double incl = wave_scan_incl(t, lane);
            const double R = __shfl(incl, steps - 1, kWave);
            const double tq = (double)u_draw * R;
            const unsigned long long hits = __ballot(lane < steps && incl > tq);
            const int pick = hits ? (int)__builtin_ctzll(hits) : steps - 1;
            const double bef = __shfl(incl - t, pick, kWave);
            if (lane == 0) { s_tau = tq; s_before = bef; s_step = pick; s_retry = !(R > 0.0) && !use_p; }
        }
        __syncthreads();
        if (!s_retry) break;
        use_p = true;                         // p == q everywhere (R == 0): draw from p instead
        __syncthreads();
    }
    if (wv != 0) return;

    // ---- inside the step: the wavefront, then the lane, then the element (one wavefront works) -----
    const double tau = s_tau;
    const int sstep = s_step;
    const int hh = sstep / part_steps, ii = sstep % part_steps;
    const double ws = lane < kPW ? mass[hh][ii][lane] : 0.0;
    const double wincl = s_before + wave_scan_incl(ws, lane);
    const unsigned long long whit = __ballot(lane < kPW && ws > 0.0 && wincl > tau);
    const unsigned long long wpos = __ballot(lane < kPW && ws > 0.0);
    if (!wpos) {                              // no mass anywhere (non-finite input): stay defined
        if (lane == 0) *o = 0;
        return;
    }
    const int wstar = whit ? (int)__builtin_ctzll(whit) : 63 - (int)__builtin_clzll(wpos);
    const double base = __shfl(wincl - ws, wstar, kWave);
    HalfStat sth = st[0];
    double sch = sc[0];
#pragma unroll
    for (int p = 1; p < PARTS; ++p)
        if (hh == p) { sth = st[p]; sch = sc[p]; }
    const int chunk = hh * part_steps * kPT + ii * kPT + wstar * kWave + lane;   // this lane's 16 bytes of the row
    const bool has_q = !bonus && !use_p;
    uint4 lv = make_uint4(P::kNegInf2, P::kNegInf2, P::kNegInf2, P::kNegInf2), qv = make_uint4(0, 0, 0, 0);
    if (chunk < (V >> 3)) {
        lv = *reinterpret_cast<const uint4 *>(logits + (int64_t)r * lstride * 2 + (int64_t)chunk * 16);
        if (has_q) qv = *reinterpret_cast<const uint4 *>(probs + (int64_t)(r - i) * pstride * 2 + (int64_t)chunk * 16);
    }
    float rv[8], pv[8], sstar = 0.f;
    chunk_masses<P>(lv, qv, c, sth.m * c, (float)(1.0 / sth.Z), rv, pv);   // same expressions as the partial kernel
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (use_p) rv[e] = pv[e];
        sstar += rv[e];
    }
    const double mine = (double)sstar * sch;
    const double li = base + wave_scan_incl(mine, lane);
    const unsigned long long lhit = __ballot(sstar > 0.f && li > tau);
    const unsigned long long lpos = __ballot(sstar > 0.f);
    if (!lpos) {                              // the sums said there was mass here, the recomputation finds none
        if (lane == 0) *o = 0;
        return;
    }
    const int owner = lhit ? (int)__builtin_ctzll(lhit) : 63 - (int)__builtin_clzll(lpos);
    if (lane == owner) {
        double cum = li - mine;
        int pick = -1, lastpos = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            cum += (double)rv[e] * sch;
            if (rv[e] > 0.f) lastpos = e;
            if (pick < 0 && rv[e] > 0.f && cum > tau) pick = e;
        }
        if (pick < 0) pick = lastpos < 0 ? 0 : lastpos;
        *o = chunk * 8 + pick;
    }
}

// The split second pass keeps 8 KB of partial sums per request: it is set up for batches up to kSplitMaxBatch,
// larger ones take the pass with one workgroup per request.
bool accept_split_supported(const adaspec_accept_dims &d) { return d.batch <= kSplitMaxBatch; }

size_t accept_split_part_bytes(int batch) { return (size_t)batch * kRowSteps * kPW * 8 * sizeof(float); }

hipError_t launch_accept_split(const AcceptArgs &a)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.batch == 0) return hipSuccess;
    // Four parts per row: the partial kernel then stays within 64 registers, two workgroups share a compute
    // unit, and the four of a request run at once for batches up to half the number of compute units
    // (measured on MI355X, config 3: 16.7 us against 18.5 us with two parts of 8 steps).
    constexpr int PARTS = 4;
    auto launch = [&](auto tag) {
        using DT = decltype(tag);
        int32_t *row_flag = (int32_t *)(a.ws + a.plan.off_row_flag), *row_cand = (int32_t *)(a.ws + a.plan.off_row_cand);
        RowStat *row_stat = (RowStat *)(a.ws + a.plan.off_row_stat);
        int2 *req_pick = (int2 *)(a.ws + a.plan.off_req_pick);
        float *part = (float *)(a.ws + a.plan.off_part);
        HalfStat *half_stat = (HalfStat *)(a.ws + a.plan.off_half_stat);
        hipLaunchKernelGGL((accept_partial_kernel<DT, PARTS>), dim3(PARTS * d.batch), dim3(kPT), 0, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.draft_tokens, a.spec_lens, a.temperature,
                           d.vocab, d.max_spec_len, d.logits_row_stride, d.probs_row_stride, row_flag, row_stat,
                           d.out_stride, a.out_tokens, a.out_accept_len, req_pick, part, half_stat);
        hipLaunchKernelGGL((accept_pick_kernel<DT, PARTS>), dim3(d.batch), dim3(kPickT), 0, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.uniforms, a.spec_lens, a.temperature,
                           d.vocab, d.max_spec_len, d.logits_row_stride, d.probs_row_stride, row_cand, d.out_stride,
                           a.out_tokens, req_pick, part, half_stat);
    };
    if (d.logits_dtype == ADASPEC_F16) launch(F16{});
    else launch(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec
