// Streaming acceptance kernel for gfx950: 16-bit logits and draft probabilities, V % 8 == 0,
// V <= 524288.  Same rule and same per-row results (flag, candidate) as the other two acceptance
// kernels.  It serves vocabularies too large for the register-resident kernel and the two-pass form
// (V > 131072): it needs at most 64 registers per thread and 73 KB of LDS, so TWO workgroups (rows)
// share a compute unit and one row's compute and latency phases overlap the other's memory phases.
//
// One workgroup of 1024 threads per logits row, 16 bytes = 8 elements per thread per step of 8192:
//   stash    steps 0..3 of the row go from memory straight into LDS (no registers), requested before
//            anything else; steps 4..7 are kept in registers during sweep 1: half of a 256 KB row
//            stays on chip
//   sweep 1  maximum and normaliser on line (running per-thread reference, (m, z) pairs merged);
//            greedy rows: arg-max (lowest index on ties) and done
//   sweep 2  the logits again (resident half from LDS / registers, the rest from the caches) with the
//            draft-probability row: residual mass r = max(0, p - q) per (step, wavefront) in fp64
//   search   the step holding tau = u1 * R by a lane-parallel scan, then that step's two chunks once
//            more: wavefront, lane, element
// Per-element arithmetic is fp32, sums across threads fp64 in a fixed order.
#include "adaspec_internal.h"
#include "device_utils.h"
#include "row_registers.h"

namespace adaspec {

constexpr int kST = 1024;
constexpr int kSW = kST / kWave;
constexpr int kSMaxSteps = 64;
constexpr int kStash = 4;                 // steps of the logits row kept in LDS between the sweeps (64 KB, dynamic)
constexpr int kKeep = 4;                  // further steps kept in registers (the kernel must stay at <= 64 VGPRs:
                                          // two workgroups per compute unit is what makes this kernel fast)

struct StreamScratch {
    double sw[kSMaxSteps][kSW];
    float  wm[kSW], wz[kSW];
    float  av[kSW];
    int    ai[kSW];
    double tau, before;
    int    sstar, retry;
    int    row_i, row_j, row_k;
    float  row_T;
    int    first_hit, last_pos;
};

// 16 bytes per lane through a buffer descriptor (past the end of the buffer: zeros)
__device__ __forceinline__ uint4 stream_load16(__amdgpu_buffer_rsrc_t rs, uint32_t lane_offset, int step)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)lane_offset, step * (kST * 16), 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// one of the four steps kept in registers (s is uniform over the workgroup)
__device__ __forceinline__ uint4 kept_step(int s, const uint4 &k0, const uint4 &k1, const uint4 &k2, const uint4 &k3)
{
    uint4 v = k0;
    if (s == kStash + 1) v = k1;
    if (s == kStash + 2) v = k2;
    if (s == kStash + 3) v = k3;
    return v;
}

// kTestOnly: the first pass of the two-pass form for batches above 1024 requests (second pass: accept_fast.hip,
// resolve mode; smaller batches take accept_parts.hip).  Only draft rows
// are judged: sweep 1, the accept test, the flag (greedy rows also leave their arg-max as candidate),
// and the workgroup is done; bonus rows leave at once.  Nothing of sweep 2 is compiled in.
template <class DT, bool kTestOnly>
__global__ __launch_bounds__(kST, 8) void accept_stream_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const float *__restrict__ uniforms,
    const int32_t *__restrict__ spec_lens, const float *__restrict__ temperature, int B, int V,
    int max_spec_len, int64_t lstride, int64_t pstride, int32_t *__restrict__ row_flag,
    int32_t *__restrict__ row_cand, RowStat *__restrict__ row_stat)
{
    using P = Pair16<DT>;
    __shared__ StreamScratch sm;
    // The first kStash steps of the row live in LDS, so sweep 2 and the search re-read only the rest from
    // the caches.  (Two workgroups share a compute unit: 2 x 73 KB of its 160 KB.)
    extern __shared__ __attribute__((aligned(16))) uint4 stash_mem[];
    uint4 (*stash)[kST] = reinterpret_cast<uint4 (*)[kST]>(stash_mem);
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x;
    const int nchunks = V >> 3;
    const int steps = ceil_div(nchunks, kST);
    const char *lrow = logits + (int64_t)r * lstride * 2;
    const uint32_t tid16 = (uint32_t)tid * 16u;
    const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(lrow), 0, V * 2, 0x00020000);
    // (lambdas capture by VALUE: anything captured by reference would be given a home in scratch memory)
    auto logits_chunk = [=](int s) {                                       // zeros past the end must count as -inf
        uint4 v = stream_load16(rl, tid16, s);
        const uint32_t ninf = (s * kST + tid >= nchunks) ? P::kNegInf2 : 0u;
        v.x |= ninf; v.y |= ninf; v.z |= ninf; v.w |= ninf;
        return v;
    };

    // (the first 1024 draft lengths and temperatures are requested ahead of the row: the memory counter
    // retires in order, so a value asked for after the row's loads would only be seen once those have landed)
    int n_first = 0;
    float t_first = 0.f;
    if (tid < B) {
        n_first = min(max(spec_lens[tid], 0), max_spec_len) + 1;
        t_first = temperature[tid];
    }
    // The first kStash steps of the row go straight from memory into the LDS stash (loads that write LDS
    // need no registers): requested before the row's request is worked out, they travel meanwhile.  Lane i of a wavefront lands at the wavefront's slot + 16 i, i.e. at stash[step][tid].
    {
        const int wvu = __builtin_amdgcn_readfirstlane(wv);
#pragma unroll
        for (int u = 0; u < kStash; ++u)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rl, (__attribute__((address_space(3))) void *)((char *)stash_mem + (u * kSW + wvu) * 1024), 16,
                (int)tid16, u * (kST * 16), 0, 0);
    }
    auto stash_chunk = [=](int s) {                                        // zeros past the end must count as -inf
        uint4 v = stash[s][tid];
        const uint32_t ninf = (s * kST + tid >= nchunks) ? P::kNegInf2 : 0u;
        v.x |= ninf; v.y |= ninf; v.z |= ninf; v.w |= ninf;
        return v;
    };

    // ---- which request owns row r: block scan of n_i = k_i + 1, 1024 requests at a time -----------
    {
        int carry = 0;
        for (int base = 0; base < B; base += kST) {
            const int i = base + tid;
            int n = n_first;
            float tt = t_first;
            if (base > 0) {
                n = i < B ? min(max(spec_lens[i], 0), max_spec_len) + 1 : 0;
                tt = i < B ? temperature[i] : 0.f;
            }
            const int inc = wave_scan_incl_dpp(n);
            if (lane == 63) sm.ai[wv] = inc;
            lds_barrier();           // LDS only: the requested steps stay in flight
            int pre = carry, tot = carry;
#pragma unroll
            for (int w = 0; w < kSW; ++w) {
                if (w < wv) pre += sm.ai[w];
                tot += sm.ai[w];
            }
            const int start = pre + inc - n;
            if (r >= start && r < start + n) { sm.row_i = i; sm.row_j = r - start; sm.row_k = n - 1; sm.row_T = tt; }
            lds_barrier();
            carry = tot;
            if (r < carry) break;
        }
    }
    const int ri = __builtin_amdgcn_readfirstlane(sm.row_i), j = __builtin_amdgcn_readfirstlane(sm.row_j),
              k = __builtin_amdgcn_readfirstlane(sm.row_k);
    const float T = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sm.row_T)));
    const bool bonus = j >= k;
    if constexpr (kTestOnly) {
        if (bonus) {                          // not judged here; the stash loads must have landed before the
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // workgroup gives its LDS back
            return;
        }
    }
    const int x = bonus ? -1 : draft_tokens[r - ri];
    const char *prow = probs + (int64_t)(r - ri) * pstride * 2;
    if (tid == 0) { sm.first_hit = kST; sm.last_pos = -1; }
    // test-only form: everything the accept test needs is requested here (scalar loads, the same for the
    // whole workgroup), one sweep ahead of its use
    uint32_t lw_t = 0, qw_t = 0;
    float u_t = 0.f;
    if constexpr (kTestOnly) {
        if (T != 0.0f) {
            lw_t = reinterpret_cast<const uint32_t *>(lrow)[x >> 1];
            qw_t = reinterpret_cast<const uint32_t *>(prow)[x >> 1];
            u_t = uniforms[2 * (int64_t)r];
        }
    }

    if (T == 0.0f) {
        ArgMax best{-INFINITY, V};
        for (int s = 0; s < steps; ++s) {
            if (s == 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            const uint4 v = s < kStash ? stash_chunk(s) : logits_chunk(s);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
            const int base = (s * kST + tid) * 8;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a = P::lo(w[e]), b = P::hi(w[e]);
                if (a > best.v) best = ArgMax{a, base + 2 * e};
                if (b > best.v) best = ArgMax{b, base + 2 * e + 1};
            }
        }
        best = wave_argmax(best);
        if (lane == 0) { sm.av[wv] = best.v; sm.ai[wv] = best.i; }
        __syncthreads();
        if (tid == 0) {
            ArgMax a{sm.av[0], sm.ai[0]};
            for (int w = 1; w < kSW; ++w) a = argmax_merge(a, ArgMax{sm.av[w], sm.ai[w]});
            if (a.i >= V) a.i = 0;
            row_flag[r] = bonus ? 1 : (x == a.i);
            row_cand[r] = a.i;
        }
        return;
    }

    // ---- sweep 1: maximum and normaliser on line ----------------------------------------------
    const float c = 1.4426950408889634f / T;
    float m_run = -INFINITY, zt = 0.f;
    static_assert(kStash % 4 == 0 && (kKeep == 4 || kKeep == 0), "the kept steps are exactly one load group of sweep 1, or none");
    uint4 keep0 = make_uint4(0, 0, 0, 0), keep1 = keep0, keep2 = keep0, keep3 = keep0;   // (named, not an array:
                                                                                         // an array would live in scratch memory)
    for (int s0 = 0; s0 < steps; s0 += 4) {
        uint4 v[4];
        if (s0 < kStash) {
            // a wavefront reads back only what it requested itself: waiting for its own loads is enough
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = stash_chunk(s0 + u);
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = logits_chunk(min(s0 + u, steps - 1));   // four requests in flight
        }
        if (kKeep > 0 && s0 == kStash) { keep0 = v[0]; keep1 = v[1]; keep2 = v[2]; keep3 = v[3]; }   // steps kStash .. kStash + 3
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (s0 + u >= steps) break;

            const uint32_t w[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
            float mn = m_run;
#pragma unroll
            for (int e = 0; e < 4; ++e) mn = fmaxf(mn, fmaxf(P::lo(w[e]), P::hi(w[e])));
            if (mn > -INFINITY) {
                zt *= __builtin_amdgcn_exp2f((m_run - mn) * c);                     // (-inf - finite) -> 0
                const float mnc = mn * c;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    zt += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mnc));
                    zt += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mnc));
                }
                m_run = mn;
            }
        }
    }
    {
        const float mw = wave_max(m_run);
        const float zw = wave_sum(m_run > -INFINITY ? zt * __builtin_amdgcn_exp2f((m_run - mw) * c) : 0.f);
        if (lane == 0) { sm.wm[wv] = mw; sm.wz[wv] = zw; }
    }
    __syncthreads();
    float m = sm.wm[0];
#pragma unroll
    for (int w = 1; w < kSW; ++w) m = fmaxf(m, sm.wm[w]);
    double Zd = 0.0;
#pragma unroll
    for (int w = 0; w < kSW; ++w)
        Zd += sm.wm[w] > -INFINITY ? (double)(sm.wz[w] * __builtin_amdgcn_exp2f((sm.wm[w] - m) * c)) : 0.0;
    const float mc = m * c;
    const float invZ = (float)(1.0 / Zd);

    // accept test (scalar loads: x is the same for the whole workgroup)
    if constexpr (kTestOnly) {
        if (tid == 0) {
            const float lx = (x & 1) ? P::hi(lw_t) : P::lo(lw_t);
            const float qx = (x & 1) ? P::hi(qw_t) : P::lo(qw_t);
            const float px = __builtin_amdgcn_exp2f(fmaf(lx, c, -mc)) * invZ;
            row_flag[r] = (qx > 0.f) ? (u_t < px / qx) : 1;
            RowStat st;                       // a rejected row is sampled by the second pass with these
            st.m = m; st.pad = 0.f; st.Z = Zd;
            row_stat[r] = st;
        }
        return;
    }
    if (tid == 0) {
        int flag = 1;
        if (!bonus) {
            const uint32_t lw = reinterpret_cast<const uint32_t *>(lrow)[x >> 1];
            const uint32_t qw = reinterpret_cast<const uint32_t *>(prow)[x >> 1];
            const float lx = (x & 1) ? P::hi(lw) : P::lo(lw);
            const float qx = (x & 1) ? P::hi(qw) : P::lo(qw);
            const float px = __builtin_amdgcn_exp2f(fmaf(lx, c, -mc)) * invZ;
            flag = (qx > 0.f) ? (uniforms[2 * (int64_t)r] < px / qx) : 1;
        }
        row_flag[r] = flag;
    }

    // ---- sweep 2: residual mass per (step, wavefront); a bonus row has q == 0 (descriptor of size 0)
    bool use_q = !bonus;
    __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(prow), 0, use_q ? V * 2 : 0, 0x00020000);
    auto residuals = [=](const uint4 &lv, const uint4 &qv, float (&rv)[8]) {
        const uint32_t w[4] = {lv.x, lv.y, lv.z, lv.w}, qw[4] = {qv.x, qv.y, qv.z, qv.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float ea = __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mc));
            const float eb = __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mc));
            rv[2 * e] = fmaxf(0.f, fmaf(ea, invZ, -P::lo(qw[e])));
            rv[2 * e + 1] = fmaxf(0.f, fmaf(eb, invZ, -P::hi(qw[e])));
        }
    };
    for (int attempt = 0; attempt < 2; ++attempt) {
        for (int s0 = 0; s0 < steps; s0 += 2) {
            uint4 lv[2], qv[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int s = min(s0 + u, steps - 1);
                if (s < kStash) lv[u] = stash_chunk(s);
                else if (s < kStash + kKeep) lv[u] = kept_step(s, keep0, keep1, keep2, keep3);
                else lv[u] = logits_chunk(s);
                qv[u] = stream_load16(rq, tid16, s);
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if (s0 + u >= steps) break;
                float rv[8], acc = 0.f;
                residuals(lv[u], qv[u], rv);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc += rv[e];
                const double wsum = wave_sum((double)acc);
                if (lane == 0) sm.sw[s0 + u][wv] = wsum;
            }
        }
        __syncthreads();
        if (wv == 0) {                        // lane s owns step s: running totals, R, the step holding tau
            double t = 0.0;
            if (lane < steps) {
#pragma unroll
                for (int w = 0; w < kSW; ++w) t = t + sm.sw[lane][w];
            }
            const double incl = wave_scan_incl(t, lane);
            const double R = __shfl(incl, steps - 1, kWave);
            const double tq = (double)uniforms[2 * (int64_t)r + 1] * R;
            const unsigned long long hits = __ballot(lane < steps && incl > tq);
            const int pick = hits ? (int)__builtin_ctzll(hits) : steps - 1;
            const double bef = __shfl(incl - t, pick, kWave);
            if (lane == 0) { sm.tau = tq; sm.before = bef; sm.sstar = pick; sm.retry = !(R > 0.0) && use_q; }
        }
        __syncthreads();
        if (!sm.retry) break;
        use_q = false;                        // p == q everywhere (R == 0): draw from p instead
        rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(prow), 0, 0, 0x00020000);
        __syncthreads();
    }
    const double tau = sm.tau;
    const int sstar = __builtin_amdgcn_readfirstlane(sm.sstar);

    // ---- inside step s*: wavefront prefix, lane prefix, element ---------------------------------
    double base = sm.before;
    {
        const double ws = lane < kSW ? sm.sw[sstar][lane] : 0.0;
        const double wincl = wave_scan_incl(ws, lane);
        const double ahead = __shfl(wincl, max(wv - 1, 0), kWave);
        if (wv > 0) base = base + ahead;
    }
    float rv[8], sstar_sum = 0.f;
    {
        uint4 lv;
        if (sstar < kStash) lv = stash_chunk(sstar);
        else if (sstar < kStash + kKeep) lv = kept_step(sstar, keep0, keep1, keep2, keep3);
        else lv = logits_chunk(sstar);
        residuals(lv, stream_load16(rq, tid16, sstar), rv);            // same expressions, same order as in sweep 2
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) sstar_sum += rv[e];
    const double wi = wave_scan_incl((double)sstar_sum, lane);
    double we = __shfl_up(wi, 1, kWave);
    if (lane == 0) we = 0.0;
    const double incl = base + wi, excl = base + we;
    if (incl > tau && sstar_sum > 0.f) atomicMin(&sm.first_hit, tid);
    if (sstar_sum > 0.f) atomicMax(&sm.last_pos, tid);
    __syncthreads();
    const int owner = sm.first_hit < kST ? sm.first_hit : sm.last_pos;
    if (tid == owner) {
        double cum = excl;
        int pick = -1, lastpos = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            cum += (double)rv[e];
            if (rv[e] > 0.f) lastpos = e;
            if (pick < 0 && rv[e] > 0.f && cum > tau) pick = e;
        }
        if (pick < 0) pick = lastpos < 0 ? 0 : lastpos;
        row_cand[r] = (sstar * kST + tid) * 8 + pick;
    }
    if (owner < 0 && tid == 0) row_cand[r] = 0;     // no mass anywhere (non-finite input): stay defined
}

bool accept_stream_path_supported(const adaspec_accept_dims &d, const void *logits, const void *probs)
{
    if (d.logits_dtype == ADASPEC_F32 || d.logits_dtype != d.probs_dtype) return false;
    if (d.vocab % 8 || d.vocab > kSMaxSteps * kST * 8) return false;
    if (d.logits_row_stride % 8 || d.probs_row_stride % 8) return false;
    if ((reinterpret_cast<uintptr_t>(logits) & 15u) || (reinterpret_cast<uintptr_t>(probs) & 15u)) return false;
    return true;
}

template <bool kTestOnly>
static hipError_t launch_stream_kernel(const AcceptArgs &a)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.total_q == 0) return hipSuccess;
    constexpr int kStashBytes = kStash * kST * 16;
    auto launch = [&](auto tag) {
        using DT = decltype(tag);
        static bool configured = false;        // more than 64 KB of LDS per workgroup has to be asked for once
        if (!configured) {
            if (hipFuncSetAttribute((const void *)accept_stream_kernel<DT, kTestOnly>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, kStashBytes) != hipSuccess)
                return;
            configured = true;
        }
        hipLaunchKernelGGL((accept_stream_kernel<DT, kTestOnly>), dim3(d.total_q), dim3(kST), kStashBytes, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.draft_tokens, a.uniforms,
                           a.spec_lens, a.temperature, d.batch, d.vocab, d.max_spec_len,
                           d.logits_row_stride, d.probs_row_stride,
                           (int32_t *)(a.ws + a.plan.off_row_flag), (int32_t *)(a.ws + a.plan.off_row_cand),
                           (RowStat *)(a.ws + a.plan.off_row_stat));
    };
    if (d.logits_dtype == ADASPEC_F16) launch(F16{});
    else launch(BF16{});
    return hipGetLastError();
}

hipError_t launch_accept_stream(const AcceptArgs &a) { return launch_stream_kernel<false>(a); }

// First pass of the two-pass form: flags of the draft rows (and arg-max candidates of greedy ones).
hipError_t launch_accept_test(const AcceptArgs &a)
{
    if (a.dims.total_draft == 0) return hipSuccess;
    return launch_stream_kernel<true>(a);
}

}  // namespace adaspec
