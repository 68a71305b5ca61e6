// Register-resident acceptance kernel for gfx950: 16-bit logits and draft
// probabilities, V % 8 == 0, V <= 131072.
//
// One workgroup of 1024 threads per logits row.  The whole logits row is loaded
// ONCE into registers (16 bytes = 8 elements per thread per step, V/8192 steps),
// the draft-probability row is streamed ONCE, nothing is re-read from memory
// except one 16-byte chunk per thread for the final token search:
//
//   1. load the row; greedy rows: argmax (lowest index on ties) and done
//   2. m = max, Z = sum 2^((l - m) c), c = log2(e) / T  (thread-local maxima first,
//      then one exchange through LDS)
//   3. stream q: chunk sums s[it] of r = max(0, 2^((l - m) c) / Z - q) kept in registers
//   4. per-step block totals (fp64) -> R, tau = u1 * R, the step it* whose running
//      total first exceeds tau
//   5. inside step it*: fp64 scan over wavefronts and lanes -> the owning thread,
//      which walks its 8 elements
// Per-element arithmetic is fp32; every sum across threads is fp64.
#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

constexpr int kFT = 1024;                // threads per row
constexpr int kFW = kFT / kWave;         // 16 wavefronts
constexpr int kQPre = 4;                 // draft-prob chunks in flight per thread

template <class T> struct Pair16;
template <> struct Pair16<BF16> {
    static constexpr uint32_t kNegInf2 = 0xFF80FF80u;
    static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
};
template <> struct Pair16<F16> {
    static constexpr uint32_t kNegInf2 = 0xFC00FC00u;
    static __device__ __forceinline__ float lo(uint32_t w) { return f16_bits_to_float((uint16_t)(w & 0xffffu)); }
    static __device__ __forceinline__ float hi(uint32_t w) { return f16_bits_to_float((uint16_t)(w >> 16)); }
};

// Opaque to the optimiser: forces later code to unpack the 16-bit pairs again instead of
// keeping 128 unpacked floats alive across the phases (the row must stay packed to fit).
__device__ __forceinline__ void keep_packed(uint4 &v)
{
    asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
}

struct FastScratch {
    double sw[kFW][16];      // per-wavefront totals of every step
    double st[16];           // block totals of every step
    float  wm[kFW], wz[kFW];
    float  av[kFW];
    int    ai[kFW];
    double tau, before;
    int    itstar, retry;
    int    first_hit, last_pos;
};

template <class DT, int ITER>
__global__ __launch_bounds__(kFT) void accept_fast_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const float *__restrict__ uniforms,
    const int32_t *__restrict__ spec_lens, const float *__restrict__ temperature,
    const int32_t *__restrict__ cu_q, const int32_t *__restrict__ row_req, int V, int max_spec_len,
    int64_t lstride, int64_t pstride, int32_t *__restrict__ row_flag, int32_t *__restrict__ row_cand)
{
    using P = Pair16<DT>;
    __shared__ FastScratch sm;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x;
    const int i = row_req[r];
    const int j = r - cu_q[i];
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const bool bonus = j >= k;
    const float T = temperature[i];
    const int nchunks = V >> 3;
    const char *lrow = logits + (int64_t)r * lstride * 2;
    const char *prow = probs + (int64_t)(r - i) * pstride * 2;
    const int x = bonus ? -1 : draft_tokens[r - i];
    const uint32_t tid16 = (uint32_t)tid * 16u;

    // ---- 1. the logits row, once ---------------------------------------------------------
    // Loads are unconditional (the lane offset is clamped into the row) so that all of them are
    // in flight together; chunks past the end of the row are blanked afterwards, which only the
    // last step(s) need (wave-uniform test).
    const uint32_t last16 = (uint32_t)(nchunks - 1) * 16u;
    auto chunk_ptr = [&](const char *row, int it) {
        const uint32_t base = min((uint32_t)it * (kFT * 16u), last16);      // wave-uniform
        return row + base + min(tid16, last16 - base);
    };
    uint4 lg[ITER];
#pragma unroll
    for (int it = 0; it < ITER; ++it) lg[it] = *reinterpret_cast<const uint4 *>(chunk_ptr(lrow, it));
    const bool sampled = T != 0.0f;
    const bool has_q = sampled && !bonus;
    uint4 qb[kQPre];
    if (has_q) {
#pragma unroll
        for (int it = 0; it < kQPre && it < ITER; ++it)
            qb[it] = *reinterpret_cast<const uint4 *>(chunk_ptr(prow, it));
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it)
        if ((it + 1) * kFT > nchunks && it * kFT + tid >= nchunks)
            lg[it] = make_uint4(P::kNegInf2, P::kNegInf2, P::kNegInf2, P::kNegInf2);

    if (!sampled) {
        // greedy: argmax with the lowest index on ties (elements are visited in index order per thread)
        ArgMax best{-INFINITY, V};
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            keep_packed(lg[it]);
            const uint32_t *w = &lg[it].x;
            const int base = (it * kFT + tid) * 8;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float a = P::lo(w[e]), b = P::hi(w[e]);
                if (a > best.v) best = ArgMax{a, base + 2 * e};
                if (b > best.v) best = ArgMax{b, base + 2 * e + 1};
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        best = wave_argmax(best);
        if (lane == 0) { sm.av[wv] = best.v; sm.ai[wv] = best.i; }
        __syncthreads();
        if (tid == 0) {
            ArgMax a{sm.av[0], sm.ai[0]};
            for (int w = 1; w < kFW; ++w) a = argmax_merge(a, ArgMax{sm.av[w], sm.ai[w]});
            if (a.i >= V) a.i = 0;
            row_flag[r] = bonus ? 1 : (x == a.i);
            row_cand[r] = a.i;
        }
        return;
    }

    // ---- 2. maximum and normaliser ---------------------------------------------------------
    const float c = 1.4426950408889634f / T;
    float mt = -1.0e30f;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        keep_packed(lg[it]);
        const uint32_t *w = &lg[it].x;
#pragma unroll
        for (int e = 0; e < 4; ++e) mt = fmaxf(mt, fmaxf(P::lo(w[e]), P::hi(w[e])));
        __builtin_amdgcn_sched_barrier(0);
    }
    float zt = 0.f;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        keep_packed(lg[it]);
        const uint32_t *w = &lg[it].x;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            zt += __builtin_amdgcn_exp2f((P::lo(w[e]) - mt) * c);
            zt += __builtin_amdgcn_exp2f((P::hi(w[e]) - mt) * c);
            if (e == 1) __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    {
        const float mw = wave_max(mt);
        const float zw = wave_sum(zt * __builtin_amdgcn_exp2f((mt - mw) * c));
        if (lane == 0) { sm.wm[wv] = mw; sm.wz[wv] = zw; }
        if (tid == 0) { sm.first_hit = kFT; sm.last_pos = -1; }
    }
    __syncthreads();
    float m = sm.wm[0];
#pragma unroll
    for (int w = 1; w < kFW; ++w) m = fmaxf(m, sm.wm[w]);
    double Zd = 0.0;
#pragma unroll
    for (int w = 0; w < kFW; ++w) Zd += (double)(sm.wz[w] * __builtin_amdgcn_exp2f((sm.wm[w] - m) * c));
    const float invZ = (float)(1.0 / Zd);

    if (tid == 0) {
        int flag = 1;
        if (!bonus) {
            const uint16_t lb = *reinterpret_cast<const uint16_t *>(lrow + (int64_t)x * 2);
            const uint16_t qx16 = *reinterpret_cast<const uint16_t *>(prow + (int64_t)x * 2);
            const float lx = P::lo(lb), qx = P::lo(qx16);
            const float px = __builtin_amdgcn_exp2f((lx - m) * c) * invZ;
            flag = (qx > 0.f) ? (uniforms[2 * (int64_t)r] < px / qx) : 1;
        }
        row_flag[r] = flag;
    }

    // ---- 3./4. residual mass per step, block totals, the step that holds tau ------------------
    bool use_q = has_q;
    for (int attempt = 0; attempt < 2; ++attempt) {
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            uint4 qv = make_uint4(0, 0, 0, 0);
            if (use_q) {
                qv = qb[it % kQPre];
                if (it + kQPre < ITER)
                    qb[it % kQPre] = *reinterpret_cast<const uint4 *>(chunk_ptr(prow, it + kQPre));
                if ((it + 1) * kFT > nchunks && it * kFT + tid >= nchunks) qv = make_uint4(0, 0, 0, 0);
            }
            keep_packed(lg[it]);
            const uint32_t *w = &lg[it].x, *qw = &qv.x;
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float ea = __builtin_amdgcn_exp2f((P::lo(w[e]) - m) * c);
                const float eb = __builtin_amdgcn_exp2f((P::hi(w[e]) - m) * c);
                acc += fmaxf(0.f, fmaf(ea, invZ, -P::lo(qw[e])));
                acc += fmaxf(0.f, fmaf(eb, invZ, -P::hi(qw[e])));
                if (e == 1) __builtin_amdgcn_sched_barrier(0);
            }
            const double t = wave_sum((double)acc);
            if (lane == 0) sm.sw[wv][it] = t;
            __builtin_amdgcn_sched_barrier(0);
        }
        __syncthreads();
        if (tid < ITER) {
            double t = 0.0;
#pragma unroll 1
            for (int w = 0; w < kFW; ++w) t = t + sm.sw[w][tid];
            sm.st[tid] = t;
        }
        __syncthreads();
        if (tid == 0) {                       // running totals over the steps: R, tau and the step holding tau
            double R = 0.0;
#pragma unroll 1
            for (int it = 0; it < ITER; ++it) R = R + sm.st[it];
            const double tq = (double)uniforms[2 * (int64_t)r + 1] * R;
            double run = 0.0, bef = 0.0;
            int pick = -1;
#pragma unroll 1
            for (int it = 0; it < ITER; ++it) {
                const double nxt = run + sm.st[it];
                if (pick < 0 && nxt > tq) { pick = it; bef = run; }
                run = nxt;
            }
            if (pick < 0) {                   // cannot happen for u1 < 1; keep the result defined
                pick = ITER - 1;
                bef = 0.0;
#pragma unroll 1
                for (int it = 0; it < ITER - 1; ++it) bef = bef + sm.st[it];
            }
            sm.tau = tq; sm.before = bef; sm.itstar = pick;
            sm.retry = !(R > 0.0) && use_q;
        }
        __syncthreads();
        if (!sm.retry) break;
        // p == q everywhere (R == 0): draw from p instead; the q row is not read on the second pass
        use_q = false;
        __syncthreads();
    }
    const double tau = sm.tau, before = sm.before;

    // ---- 5. inside step it*: the owning thread, then the element --------------------------------
    const int itstar = __builtin_amdgcn_readfirstlane(sm.itstar);
    uint4 lstar = lg[0];
#pragma unroll
    for (int it = 1; it < ITER; ++it)
        if (it == itstar) lstar = lg[it];
    const int cstar = itstar * kFT + tid;
    uint4 qstar = make_uint4(0, 0, 0, 0);
    if (use_q && cstar < nchunks) qstar = *reinterpret_cast<const uint4 *>(chunk_ptr(prow, itstar));
    float rv[8], sstar = 0.f;
    {
        const uint32_t *w = &lstar.x, *qw = &qstar.x;
#pragma unroll
        for (int e = 0; e < 4; ++e) {          // same expressions, same order as in the streaming pass
            const float ea = __builtin_amdgcn_exp2f((P::lo(w[e]) - m) * c);
            const float eb = __builtin_amdgcn_exp2f((P::hi(w[e]) - m) * c);
            rv[2 * e] = fmaxf(0.f, fmaf(ea, invZ, -P::lo(qw[e])));
            rv[2 * e + 1] = fmaxf(0.f, fmaf(eb, invZ, -P::hi(qw[e])));
            sstar += rv[2 * e];
            sstar += rv[2 * e + 1];
        }
    }
    double base = before;
#pragma unroll 1
    for (int w = 0; w < wv; ++w) base = base + sm.sw[w][itstar];
    const double wi = wave_scan_incl((double)sstar, lane);
    double we = __shfl_up(wi, 1, kWave);
    if (lane == 0) we = 0.0;
    const double incl = base + wi, excl = base + we;
    if (incl > tau && sstar > 0.f) atomicMin(&sm.first_hit, tid);
    if (sstar > 0.f) atomicMax(&sm.last_pos, tid);
    __syncthreads();
    const int owner = sm.first_hit < kFT ? sm.first_hit : sm.last_pos;
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
        row_cand[r] = cstar * 8 + pick;
    }
    if (owner < 0 && tid == 0) row_cand[r] = 0;     // no mass anywhere (non-finite input): stay defined
}

bool accept_fast_path_supported(const adaspec_accept_dims &d, const void *logits, const void *probs)
{
    if (d.logits_dtype == ADASPEC_F32 || d.logits_dtype != d.probs_dtype) return false;
    if (d.vocab % 8 || d.vocab > kFT * 8 * 16) return false;
    if (d.logits_row_stride % 8 || d.probs_row_stride % 8) return false;
    if ((reinterpret_cast<uintptr_t>(logits) & 15u) || (reinterpret_cast<uintptr_t>(probs) & 15u)) return false;
    return true;
}

hipError_t launch_accept_fast(const AcceptArgs &a)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.total_q == 0) return hipSuccess;
    const int steps = ceil_div(d.vocab / 8, kFT);
    auto launch = [&](auto tag, auto it_tag) {
        using DT = decltype(tag);
        constexpr int ITER = decltype(it_tag)::value;
        hipLaunchKernelGGL((accept_fast_kernel<DT, ITER>), dim3(d.total_q), dim3(kFT), 0, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.draft_tokens, a.uniforms,
                           a.spec_lens, a.temperature, (const int32_t *)(a.ws + a.plan.off_cu_q),
                           (const int32_t *)(a.ws + a.plan.off_row_req), d.vocab, d.max_spec_len,
                           d.logits_row_stride, d.probs_row_stride,
                           (int32_t *)(a.ws + a.plan.off_row_flag), (int32_t *)(a.ws + a.plan.off_row_cand));
    };
    auto with_it = [&](auto tag) {
        if (steps <= 4) launch(tag, std::integral_constant<int, 4>{});
        else if (steps <= 8) launch(tag, std::integral_constant<int, 8>{});
        else launch(tag, std::integral_constant<int, 16>{});
    };
    if (d.logits_dtype == ADASPEC_F16) with_it(F16{});
    else with_it(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec
