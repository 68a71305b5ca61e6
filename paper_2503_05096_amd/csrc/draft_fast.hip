// Register-resident draft-side sampling for gfx950: 16-bit draft logits, V % 8 == 0, V <= 131072.
// (What the step computes is stated in draft_sample.hip; this is its single-pass form.)
//
// One workgroup of 1024 threads per row.  The logits row is read from memory ONCE and stays packed
// in registers; the probability row is written ONCE; nothing is read back:
//   1. request the row step by step; maximum and normaliser in one sweep that follows the loads
//      (running per-thread reference, (m, z) pairs merged across the workgroup)
//   2. q_v = 2^(l_v c - m c) / Z, rounded once to the storage type, stored; the rounded mass of every
//      (step, wavefront) in fp64
//   3. the step holding tau = u * sum(q), then wavefront, lane and element, recomputing the few q_v
//      involved from the registers with the same expression (same bits as the stored row)
// Greedy rows (T == 0): arg-max with the lowest index on ties from the registers, q at temperature 1.
#include <type_traits>
#include <utility>

#include "adaspec_internal.h"
#include "device_utils.h"
#include "row_registers.h"
#include "draft_common.h"

namespace adaspec {

constexpr int kGT = 1024;                // threads per row
constexpr int kGW = kGT / kWave;

struct DraftFastScratch {
    double sw[16][kGW];                  // rounded probability mass of every (step, wavefront)
    float  wm[kGW], wz[kGW];
    float  av[kGW];
    int    ai[kGW];
    double tau, before;
    int    sstar;
    int    first_hit, last_pos;
};

template <class DT, class PT, int ITER>
__global__ __launch_bounds__(kGT) void draft_fast_kernel(
    const char *__restrict__ logits, const float *__restrict__ temperature,
    const float *__restrict__ uniforms, const int32_t *__restrict__ out_rows, char *__restrict__ probs,
    int32_t *__restrict__ tokens, float *__restrict__ confidence, int V, int64_t lstride_bytes,
    int64_t pstride_bytes)
{
    using P = Pair16<DT>;
    constexpr int kPsz = std::is_same<PT, F32>::value ? 4 : 2;
    __shared__ DraftFastScratch sm;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x;
    const int nchunks = V >> 3;
    const char *lrow = logits + (int64_t)r * lstride_bytes;
    char *prow = probs + (int64_t)(out_rows ? out_rows[r] : r) * pstride_bytes;
    const uint32_t tid16 = (uint32_t)tid * 16u;
    const float T = temperature[r];
    const float u = uniforms[r];
    const bool greedy = T == 0.0f;

    // Buffer descriptors: a lane supplies a 32-bit offset, accesses past the end of the row are
    // dropped by the range check (loads return zero, stores do nothing).
    const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(lrow), 0, V * 2, 0x00020000);
    const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(prow, 0, V * kPsz, 0x00020000);
    auto load_chunk = [&](int it) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rl, (int)tid16, it * (kGT * 16), 0);
        return make_uint4(v.x, v.y, v.z, v.w);
    };
    auto blank_tail = [&](uint4 &v, int it) {             // zeros past the end of the row must count as -inf
        const uint32_t ninf = (it * kGT + tid >= nchunks) ? P::kNegInf2 : 0u;
        asm volatile("v_or_b32 %0, %0, %4\n\tv_or_b32 %1, %1, %4\n\tv_or_b32 %2, %2, %4\n\tv_or_b32 %3, %3, %4"
                     : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w) : "v"(ninf));
    };
    // A wavefront executes in order and a load is held back while the memory pipeline of the compute
    // unit is full: only the first steps are requested up front, the rest inside the sweep.
    constexpr int kLPre = ITER < 8 ? ITER : 8;
    uint4 lg[ITER];
#pragma unroll
    for (int it = 0; it < kLPre; ++it) {
        lg[it] = load_chunk(it);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (tid == 0) { sm.first_hit = kGT; sm.last_pos = -1; }

    // ---- 1. maximum and normaliser in one sweep ----------------------------------------------
    // Packed signed 16-bit integer max (both formats are sign-magnitude) tracks max(0, largest logit
    // so far); the partial sum is rescaled when it grows.  A row without a positive logit (block
    // maximum 0) is redone with the exact float maximum.
    const float c2 = greedy ? 1.4426950408889634f : 1.4426950408889634f / T;
    short2v pm = {0, 0};
    float m_run = 0.f, zt = 0.f;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        if (it + kLPre < ITER) lg[it + kLPre] = load_chunk(it + kLPre);
        blank_tail(lg[it], it);
        keep_packed(lg[it]);
        const uint32_t *w = &lg[it].x;
#pragma unroll
        for (int e = 0; e < 4; ++e) pm = __builtin_elementwise_max(pm, __builtin_bit_cast(short2v, w[e]));
        const float mn = P::lo((uint32_t)(uint16_t)max(pm.x, pm.y));
        zt *= __builtin_amdgcn_exp2f((m_run - mn) * c2);
        m_run = mn;
        const float mnc = mn * c2;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            zt += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c2, -mnc));
            zt += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c2, -mnc));
            if (e == 1) __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    {
        const float mw = wave_max(m_run);
        const float zw = wave_sum(zt * __builtin_amdgcn_exp2f((m_run - mw) * c2));
        if (lane == 0) { sm.wm[wv] = mw; sm.wz[wv] = zw; }
    }
    __syncthreads();
    float m = sm.wm[0];
#pragma unroll
    for (int w = 1; w < kGW; ++w) m = fmaxf(m, sm.wm[w]);
    double Zd = 0.0;
#pragma unroll
    for (int w = 0; w < kGW; ++w) Zd += (double)(sm.wz[w] * __builtin_amdgcn_exp2f((sm.wm[w] - m) * c2));
    if (m == 0.f) {                           // rare: no positive logit in the row -> exact two-sweep form
        float mt = -INFINITY;
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            keep_packed(lg[it]);
            const uint32_t *w = &lg[it].x;
#pragma unroll
            for (int e = 0; e < 4; ++e) mt = fmaxf(mt, fmaxf(P::lo(w[e]), P::hi(w[e])));
            __builtin_amdgcn_sched_barrier(0);
        }
        mt = wave_max(mt);
        __syncthreads();
        if (lane == 0) sm.wm[wv] = mt;
        __syncthreads();
        m = sm.wm[0];
#pragma unroll
        for (int w = 1; w < kGW; ++w) m = fmaxf(m, sm.wm[w]);
        const float mc0 = m * c2;
        float z2 = 0.f;
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            keep_packed(lg[it]);
            const uint32_t *w = &lg[it].x;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                z2 += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c2, -mc0));
                z2 += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c2, -mc0));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        z2 = wave_sum(z2);
        if (lane == 0) sm.wz[wv] = z2;
        __syncthreads();
        Zd = 0.0;
#pragma unroll
        for (int w = 0; w < kGW; ++w) Zd += (double)sm.wz[w];
    }
    const float mc = m * c2;
    const float invZ = (float)(1.0 / Zd);

    // ---- 2. the probability row: rounded once, stored once; its mass per (step, wavefront) ------
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        keep_packed(lg[it]);
        float q[8];
        uint4 packed;
        chunk_probs<DT, PT>(lg[it], c2, mc, invZ, q, packed);
        // (The step's offset goes into the lane offset, not into the scalar-offset operand: with a scalar
        // register there the compiler leaves no wait state between a 16-byte buffer store and a vector
        // instruction that overwrites its data registers, and on gfx950 the store was seen to pick up the
        // new value of its first data register.)
        if constexpr (kPsz == 2) {
            __builtin_amdgcn_raw_buffer_store_b128(u32x4{packed.x, packed.y, packed.z, packed.w}, rp,
                                                   (int)tid16 + it * (kGT * 16), 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(
                u32x4{__float_as_uint(q[0]), __float_as_uint(q[1]), __float_as_uint(q[2]), __float_as_uint(q[3])}, rp,
                (int)(tid16 * 2) + it * (kGT * 32), 0, 0);
            __builtin_amdgcn_raw_buffer_store_b128(
                u32x4{__float_as_uint(q[4]), __float_as_uint(q[5]), __float_as_uint(q[6]), __float_as_uint(q[7])}, rp,
                (int)(tid16 * 2 + 16) + it * (kGT * 32), 0, 0);
        }
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += q[e];
        const double wsum = wave_sum((double)acc);
        if (lane == 0) sm.sw[it][wv] = wsum;
        __builtin_amdgcn_sched_barrier(0);
    }

    if (greedy) {
        // arg-max with the lowest index on ties (a thread visits its elements in index order)
        ArgMax best{-INFINITY, V};
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            keep_packed(lg[it]);
            const uint32_t *w = &lg[it].x;
            const int base = (it * kGT + tid) * 8;
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
            for (int w = 1; w < kGW; ++w) a = argmax_merge(a, ArgMax{sm.av[w], sm.ai[w]});
            if (a.i >= V) a.i = 0;
            // its probability, with the expression and the rounding of the stored row
            uint4 one = make_uint4(0, 0, 0, 0);
            uint16_t bits;
            if constexpr (std::is_same<DT, BF16>::value) bits = float_to_bf16_bits(a.v); else bits = float_to_f16_bits(a.v);
            one.x = bits;                      // the maximum is a stored logit: converting it back is exact
            float q[8];
            uint4 packed;
            chunk_probs<DT, PT>(one, c2, mc, invZ, q, packed);
            tokens[r] = a.i;
            confidence[r] = q[0];
        }
        return;
    }
    __syncthreads();

    // ---- 3. the step that holds tau = u * Q: one wavefront, lane s owns step s -------------------
    if (wv == 0) {
        double t = 0.0;
        if (lane < ITER) {
#pragma unroll
            for (int w = 0; w < kGW; ++w) t = t + sm.sw[lane][w];
        }
        const double incl = wave_scan_incl(t, lane);
        const double Q = __shfl(incl, ITER - 1, kWave);
        const double tq = (double)u * Q;
        const unsigned long long hits = __ballot(lane < ITER && incl > tq);
        const int pick = hits ? (int)__builtin_ctzll(hits) : ITER - 1;
        const double bef = __shfl(incl - t, pick, kWave);
        if (lane == 0) { sm.tau = tq; sm.before = bef; sm.sstar = pick; }
    }
    __syncthreads();
    const double tau = sm.tau;
    const int sstar = __builtin_amdgcn_readfirstlane(sm.sstar);

    // ---- inside that step: wavefront prefix, lane prefix, element --------------------------------
    double base = sm.before;
    {
        const double ws = lane < kGW ? sm.sw[sstar][lane] : 0.0;
        const double wincl = wave_scan_incl(ws, lane);
        const double ahead = __shfl(wincl, max(wv - 1, 0), kWave);
        if (wv > 0) base = base + ahead;
    }
    uint4 lstar = lg[0];
#pragma unroll
    for (int it = 1; it < ITER; ++it)
        if (it == sstar) lstar = lg[it];
    const int cstar = sstar * kGT + tid;
    float qv[8], mine = 0.f;
    {
        uint4 packed;
        chunk_probs<DT, PT>(lstar, c2, mc, invZ, qv, packed);      // same expression, same rounding as the stored row
#pragma unroll
        for (int e = 0; e < 8; ++e) mine += qv[e];
    }
    const double wi = wave_scan_incl((double)mine, lane);
    double we = __shfl_up(wi, 1, kWave);
    if (lane == 0) we = 0.0;
    const double incl = base + wi, excl = base + we;
    if (incl > tau && mine > 0.f) atomicMin(&sm.first_hit, tid);
    if (mine > 0.f) atomicMax(&sm.last_pos, tid);
    __syncthreads();
    const int owner = sm.first_hit < kGT ? sm.first_hit : sm.last_pos;
    if (tid == owner) {
        double cum = excl;
        int pick = -1, lastpos = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            cum += (double)qv[e];
            if (qv[e] > 0.f) lastpos = e;
            if (pick < 0 && qv[e] > 0.f && cum > tau) pick = e;
        }
        if (pick < 0) pick = lastpos < 0 ? 0 : lastpos;
        tokens[r] = cstar * 8 + pick;
        confidence[r] = qv[pick];
    }
    if (owner < 0 && tid == 0) { tokens[r] = 0; confidence[r] = 0.f; }   // no mass (non-finite input)
}

bool draft_fast_supported(const adaspec_draft_dims &d)
{
    if (d.logits_dtype == ADASPEC_F32) return false;
    return d.vocab % 8 == 0 && d.vocab <= kGT * 8 * 16;
}

hipError_t launch_draft_fast(const void *logits, const float *temperature, const float *uniforms,
                             const int32_t *out_rows, void *probs, int32_t *tokens, float *confidence,
                             const adaspec_draft_dims &d, hipStream_t stream)
{
    if (d.rows == 0) return hipSuccess;
    const int steps = ceil_div(d.vocab / 8, kGT);
    const int psz = d.probs_dtype == ADASPEC_F32 ? 4 : 2;
    auto launch = [&](auto lt, auto pt, auto it_tag) {
        using DT = decltype(lt);
        using PT = decltype(pt);
        constexpr int ITER = decltype(it_tag)::value;
        hipLaunchKernelGGL((draft_fast_kernel<DT, PT, ITER>), dim3(d.rows), dim3(kGT), 0, stream,
                           (const char *)logits, temperature, uniforms, out_rows, (char *)probs, tokens, confidence,
                           d.vocab, d.logits_row_stride * 2, d.probs_row_stride * psz);
    };
    auto with_it = [&](auto lt, auto pt) {
        if (steps <= 4) launch(lt, pt, std::integral_constant<int, 4>{});
        else if (steps <= 8) launch(lt, pt, std::integral_constant<int, 8>{});
        else launch(lt, pt, std::integral_constant<int, 16>{});
    };
    auto with_p = [&](auto lt) {
        if (d.probs_dtype == ADASPEC_F32) with_it(lt, F32{});
        else if (d.probs_dtype == ADASPEC_F16) with_it(lt, F16{});
        else with_it(lt, BF16{});
    };
    if (d.logits_dtype == ADASPEC_F16) with_p(F16{});
    else with_p(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec
