// Draft-side sampling: from one row of draft-model logits produce, in one kernel,
//   the draft-probability row q = softmax(l / T), rounded once to its storage type (this rounded
//     row is what the acceptance step later reads and divides by),
//   the draft token, drawn from the ROUNDED row by inverse CDF (so q[token] > 0 always), or the
//     arg-max for greedy drafting (T == 0, lowest index on ties; q is then softmax(l) at T = 1),
//   the token's confidence score c = q[token] (paper Eq. 6: the acceptance rate of a draft is
//     approximated by the product of the confidence scores; Alg. 1: "dts, confs <- M_d").
//
// One workgroup of 1024 threads per row; each thread owns 8 consecutive vocabulary entries per
// step of 8192.  Three sweeps over the logits (maximum, normaliser, probabilities): the first
// comes from HBM, the others from the caches (a row is at most 512 KB).  The probabilities are
// written once.  Sums across threads are fp64 in a fixed order: results do not depend on timing.
#include <type_traits>

#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

constexpr int kDT = 1024;
constexpr int kDW = kDT / kWave;
constexpr int kDMaxSteps = 64;            // V <= 64 * 8192

struct DraftScratch {
    double sw[kDMaxSteps][kDW];           // per step: residual... probability mass of every wavefront
    double wz[kDW];
    float  av[kDW];
    int    ai[kDW];
    double tau, before;
    int    sstar;
    int    first_hit, last_pos;
};

// 8 consecutive values of a row as floats (chunk index c covers elements 8c .. 8c+7)
template <class T> __device__ __forceinline__ void load8(const char *row, int c, float (&v)[8])
{
    if constexpr (std::is_same<T, F32>::value) {
        const float4 a = *reinterpret_cast<const float4 *>(row + (int64_t)c * 32);
        const float4 b = *reinterpret_cast<const float4 *>(row + (int64_t)c * 32 + 16);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    } else {
        const uint4 u = *reinterpret_cast<const uint4 *>(row + (int64_t)c * 16);
        const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if constexpr (std::is_same<T, BF16>::value) {
                v[2 * e] = bf16_bits_to_float(w[e] & 0xffffu);
                v[2 * e + 1] = bf16_bits_to_float(w[e] >> 16);
            } else {
                v[2 * e] = f16_bits_to_float((uint16_t)(w[e] & 0xffffu));
                v[2 * e + 1] = f16_bits_to_float((uint16_t)(w[e] >> 16));
            }
        }
    }
}

// round 8 floats to the storage type, store them, and return the rounded values as floats
template <class T> __device__ __forceinline__ void round_store8(char *row, int c, float (&v)[8])
{
    if constexpr (std::is_same<T, F32>::value) {
        *reinterpret_cast<float4 *>(row + (int64_t)c * 32) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4 *>(row + (int64_t)c * 32 + 16) = make_float4(v[4], v[5], v[6], v[7]);
    } else {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            uint16_t lo, hi;
            if constexpr (std::is_same<T, BF16>::value) {
                lo = float_to_bf16_bits(v[2 * e]); hi = float_to_bf16_bits(v[2 * e + 1]);
                v[2 * e] = bf16_bits_to_float(lo); v[2 * e + 1] = bf16_bits_to_float(hi);
            } else {
                lo = float_to_f16_bits(v[2 * e]); hi = float_to_f16_bits(v[2 * e + 1]);
                v[2 * e] = f16_bits_to_float(lo); v[2 * e + 1] = f16_bits_to_float(hi);
            }
            w[e] = (uint32_t)lo | ((uint32_t)hi << 16);
        }
        *reinterpret_cast<uint4 *>(row + (int64_t)c * 16) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

template <class LT, class PT>
__global__ __launch_bounds__(kDT) void draft_sample_kernel(
    const char *__restrict__ logits, const float *__restrict__ temperature,
    const float *__restrict__ uniforms, const int32_t *__restrict__ out_rows, char *__restrict__ probs,
    int32_t *__restrict__ tokens, float *__restrict__ confidence, int V, int64_t lstride_bytes,
    int64_t pstride_bytes)
{
    __shared__ DraftScratch sm;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x;
    const int nchunks = V >> 3;
    const int steps = ceil_div(nchunks, kDT);
    const char *lrow = logits + (int64_t)r * lstride_bytes;
    char *prow = probs + (int64_t)(out_rows ? out_rows[r] : r) * pstride_bytes;
    const float T = temperature[r];
    const bool greedy = T == 0.0f;
    if (tid == 0) { sm.first_hit = kDT; sm.last_pos = -1; }

    // ---- sweep 1: maximum and its lowest index --------------------------------------------
    ArgMax best{-INFINITY, V};
    for (int s = 0; s < steps; ++s) {
        const int c = s * kDT + tid;
        if (c >= nchunks) break;
        float v[8];
        load8<LT>(lrow, c, v);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (v[e] > best.v) best = ArgMax{v[e], c * 8 + e};
    }
    best = wave_argmax(best);
    if (lane == 0) { sm.av[wv] = best.v; sm.ai[wv] = best.i; }
    __syncthreads();
    best = ArgMax{sm.av[0], sm.ai[0]};
#pragma unroll
    for (int w = 1; w < kDW; ++w) best = argmax_merge(best, ArgMax{sm.av[w], sm.ai[w]});
    if (best.i >= V) best.i = 0;
    const float m = best.v;
    const float c2 = greedy ? 1.4426950408889634f : 1.4426950408889634f / T;
    const float mc = m * c2;

    // ---- sweep 2: normaliser ----------------------------------------------------------------
    float zt = 0.f;
    for (int s = 0; s < steps; ++s) {
        const int c = s * kDT + tid;
        if (c >= nchunks) break;
        float v[8];
        load8<LT>(lrow, c, v);
#pragma unroll
        for (int e = 0; e < 8; ++e) zt += __builtin_amdgcn_exp2f(fmaf(v[e], c2, -mc));
    }
    {
        const double zw = wave_sum((double)zt);
        if (lane == 0) sm.wz[wv] = zw;
    }
    __syncthreads();
    double Zd = 0.0;
#pragma unroll
    for (int w = 0; w < kDW; ++w) Zd += sm.wz[w];
    const float invZ = (float)(1.0 / Zd);

    // ---- sweep 3: probabilities, rounded once and stored; their mass per step and wavefront ----
    for (int s = 0; s < steps; ++s) {
        const int c = s * kDT + tid;
        float acc = 0.f;
        if (c < nchunks) {
            float v[8];
            load8<LT>(lrow, c, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = __builtin_amdgcn_exp2f(fmaf(v[e], c2, -mc)) * invZ;
            round_store8<PT>(prow, c, v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += v[e];
        }
        const double wsum = wave_sum((double)acc);
        if (lane == 0) sm.sw[s][wv] = wsum;
    }
    __syncthreads();                          // (also makes this workgroup's stores visible to itself)

    if (greedy) {
        if (tid == 0) {
            float q;
            if constexpr (std::is_same<PT, F32>::value) q = reinterpret_cast<const float *>(prow)[best.i];
            else if constexpr (std::is_same<PT, BF16>::value) q = bf16_bits_to_float(reinterpret_cast<const uint16_t *>(prow)[best.i]);
            else q = f16_bits_to_float(reinterpret_cast<const uint16_t *>(prow)[best.i]);
            tokens[r] = best.i;
            confidence[r] = q;
        }
        return;
    }

    // ---- the step that holds tau = u * Q: one wavefront, lane s owns step s -----------------------
    if (wv == 0) {
        double t = 0.0;
        if (lane < steps) {
#pragma unroll
            for (int w = 0; w < kDW; ++w) t = t + sm.sw[lane][w];
        }
        const double incl = wave_scan_incl(t, lane);
        const double Q = __shfl(incl, steps - 1, kWave);
        const double tq = (double)uniforms[r] * Q;
        const unsigned long long hits = __ballot(lane < steps && incl > tq);
        const int pick = hits ? (int)__builtin_ctzll(hits) : steps - 1;
        const double bef = __shfl(incl - t, pick, kWave);
        if (lane == 0) { sm.tau = tq; sm.before = bef; sm.sstar = pick; }
    }
    __syncthreads();
    const double tau = sm.tau;
    const int sstar = sm.sstar;

    // ---- inside that step: wavefront prefix, lane prefix, element --------------------------------
    double base = sm.before;
    {
        const double ws = lane < kDW ? sm.sw[sstar][lane] : 0.0;
        const double wincl = wave_scan_incl(ws, lane);
        const double ahead = __shfl(wincl, max(wv - 1, 0), kWave);
        if (wv > 0) base = base + ahead;
    }
    const int cstar = sstar * kDT + tid;
    float qv[8], mine = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) qv[e] = 0.f;
    if (cstar < nchunks) {
        load8<PT>(prow, cstar, qv);           // the rounded values this workgroup just wrote
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
    const int owner = sm.first_hit < kDT ? sm.first_hit : sm.last_pos;
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

bool draft_sample_supported(const adaspec_draft_dims &d, const void *logits, const void *probs)
{
    if (d.vocab % 8 || d.vocab > kDMaxSteps * kDT * 8) return false;
    if (d.logits_row_stride % 8 || d.probs_row_stride % 8) return false;
    if ((reinterpret_cast<uintptr_t>(logits) & 15u) || (reinterpret_cast<uintptr_t>(probs) & 15u)) return false;
    return true;
}

hipError_t launch_draft_sample(const void *logits, const float *temperature, const float *uniforms,
                               const int32_t *out_rows, void *probs, int32_t *tokens, float *confidence,
                               const adaspec_draft_dims &d, hipStream_t stream)
{
    if (d.rows == 0) return hipSuccess;
    auto launch = [&](auto lt, auto pt) {
        using LT = decltype(lt);
        using PT = decltype(pt);
        const int lsz = std::is_same<LT, F32>::value ? 4 : 2, psz = std::is_same<PT, F32>::value ? 4 : 2;
        hipLaunchKernelGGL((draft_sample_kernel<LT, PT>), dim3(d.rows), dim3(kDT), 0, stream,
                           (const char *)logits, temperature, uniforms, out_rows, (char *)probs, tokens,
                           confidence, d.vocab, d.logits_row_stride * lsz, d.probs_row_stride * psz);
    };
    auto with_p = [&](auto lt) {
        if (d.probs_dtype == ADASPEC_F32) launch(lt, F32{});
        else if (d.probs_dtype == ADASPEC_F16) launch(lt, F16{});
        else launch(lt, BF16{});
    };
    if (d.logits_dtype == ADASPEC_F32) with_p(F32{});
    else if (d.logits_dtype == ADASPEC_F16) with_p(F16{});
    else with_p(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec
