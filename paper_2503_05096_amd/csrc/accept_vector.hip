// Portable acceptance kernel: any vocabulary size, any of the three storage
// types for logits and draft probabilities, arbitrary row strides.  One
// workgroup of 256 threads per logits row, several sweeps over the row (the
// later ones served by the caches).  It is the path for fp32 inputs and for
// shapes the register-resident kernel does not take.
//
// Per row:  sweep 1  max / argmax (lowest index wins ties)      -> greedy rows end here
//           sweep 2  Z = sum 2^((l - m) * log2(e)/T)
//           sweep 3  R = sum max(0, p - q)  (tile by tile, double prefix)
//           sweep 4  the same tiles again up to the one where the prefix crosses u1 * R
// Per-element arithmetic is fp32; every sum across threads and tiles is fp64.
#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

constexpr int kNT = 256;
constexpr int kNW = kNT / kWave;
constexpr int kE = 4;                 // contiguous elements per thread per tile
constexpr int kTile = kNT * kE;

struct BlockScratch {
    float  av[kNW];
    int    ai[kNW];
    double d[kNW];
    double total;
    int    hit;
};

__device__ __forceinline__ ArgMax block_argmax(ArgMax a, BlockScratch &s, int tid)
{
    a = wave_argmax(a);
    __syncthreads();
    if ((tid & 63) == 0) { s.av[tid >> 6] = a.v; s.ai[tid >> 6] = a.i; }
    __syncthreads();
    ArgMax r{s.av[0], s.ai[0]};
#pragma unroll
    for (int w = 1; w < kNW; ++w) r = argmax_merge(r, ArgMax{s.av[w], s.ai[w]});
    return r;
}

__device__ __forceinline__ double block_sum(double v, BlockScratch &s, int tid)
{
    v = wave_sum(v);
    __syncthreads();
    if ((tid & 63) == 0) s.d[tid >> 6] = v;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int w = 0; w < kNW; ++w) r += s.d[w];
    return r;
}

// exclusive and inclusive prefix over the 256 threads, and the block total;
// excl of thread t+1 is bit-identical to incl of thread t
__device__ __forceinline__ void block_scan(double v, BlockScratch &s, int tid, double &excl,
                                           double &incl, double &total)
{
    const int lane = tid & 63, wv = tid >> 6;
    const double wi = wave_scan_incl(v, lane);
    double we = __shfl_up(wi, 1, kWave);
    if (lane == 0) we = 0.0;
    __syncthreads();
    if (lane == 63) s.d[wv] = wi;
    __syncthreads();
    double wp = 0.0, run = 0.0;
#pragma unroll
    for (int w = 0; w < kNW; ++w) {
        if (w == wv) wp = run;
        run = run + s.d[w];
    }
    excl = wp + we;
    incl = wp + wi;
    total = run;
}

template <class LT, class PT>
__global__ __launch_bounds__(kNT) void accept_vector_kernel(
    const void *__restrict__ logits, const void *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const float *__restrict__ uniforms,
    const int32_t *__restrict__ spec_lens, const float *__restrict__ temperature,
    const int32_t *__restrict__ cu_q, const int32_t *__restrict__ row_req, int V, int max_spec_len,
    int64_t lstride, int64_t pstride, int32_t *__restrict__ row_flag, int32_t *__restrict__ row_cand)
{
    __shared__ BlockScratch sm;
    const int tid = threadIdx.x;
    const int r = blockIdx.x;
    const int i = row_req[r];
    const int j = r - cu_q[i];
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const bool bonus = j >= k;
    const float T = temperature[i];
    const int64_t lrow = (int64_t)r * lstride;
    const int64_t prow = (int64_t)(r - i) * pstride;
    const int x = bonus ? -1 : draft_tokens[r - i];
    if (tid == 0) sm.hit = 0;

    // sweep 1: maximum and its lowest index
    ArgMax best{-INFINITY, V};
    for (int v = tid; v < V; v += kNT) {
        const float l = load_as_float<LT>(logits, lrow + v);
        if (l > best.v) best = ArgMax{l, v};
    }
    best = block_argmax(best, sm, tid);
    if (best.i >= V) best.i = 0;
    if (T == 0.0f) {
        if (tid == 0) {
            row_flag[r] = bonus ? 1 : (x == best.i);
            row_cand[r] = best.i;
        }
        return;
    }
    const float m = best.v;
    const float c = 1.4426950408889634f / T;

    // sweep 2: normaliser
    float zt = 0.f;
    for (int v = tid; v < V; v += kNT)
        zt += __builtin_amdgcn_exp2f((load_as_float<LT>(logits, lrow + v) - m) * c);
    const double Z = block_sum((double)zt, sm, tid);
    const float invZ = (float)(1.0 / Z);

    if (tid == 0) {
        int flag = 1;
        if (!bonus) {
            const float px = __builtin_amdgcn_exp2f((load_as_float<LT>(logits, lrow + x) - m) * c) * invZ;
            const float qx = load_as_float<PT>(probs, prow + x);
            flag = (qx > 0.f) ? (uniforms[2 * (int64_t)r] < px / qx) : 1;
        }
        row_flag[r] = flag;
    }

    bool use_p = bonus;
    auto resid = [&](int v) -> float {
        const float p = __builtin_amdgcn_exp2f((load_as_float<LT>(logits, lrow + v) - m) * c) * invZ;
        if (use_p) return p;
        return fmaxf(0.f, p - load_as_float<PT>(probs, prow + v));
    };

    // sweep 3: total sampling mass, tile by tile
    double R = 0.0;
    for (int attempt = 0; attempt < 2; ++attempt) {
        double running = 0.0;
        for (int tb = 0; tb < V; tb += kTile) {
            const int v0 = tb + tid * kE;
            float seg = 0.f;
#pragma unroll
            for (int e = 0; e < kE; ++e)
                if (v0 + e < V) seg += resid(v0 + e);
            double ex, in, tot;
            block_scan((double)seg, sm, tid, ex, in, tot);
            running = running + tot;
        }
        R = running;
        if (R > 0.0 || use_p) break;
        use_p = true;                       // p == q everywhere: draw from p instead
    }
    const double tau = (double)uniforms[2 * (int64_t)r + 1] * R;

    // sweep 4: first tile, thread and element where the inclusive prefix exceeds tau
    int cand = best.i;
    double running = 0.0;
    for (int tb = 0; tb < V; tb += kTile) {
        const int v0 = tb + tid * kE;
        float rv[kE];
        float seg = 0.f;
#pragma unroll
        for (int e = 0; e < kE; ++e) {
            rv[e] = (v0 + e < V) ? resid(v0 + e) : 0.f;
            seg += rv[e];
        }
        double ex, in, tot;
        block_scan((double)seg, sm, tid, ex, in, tot);
        if (running + tot > tau) {
            if (running + in > tau && !(running + ex > tau)) {
                double cum = running + ex;
                int pick = -1, lastpos = -1;
#pragma unroll
                for (int e = 0; e < kE; ++e) {
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
    if (tid == 0) row_cand[r] = cand;
}

hipError_t launch_accept_vector(const AcceptArgs &a)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.total_q == 0) return hipSuccess;
    auto launch = [&](auto lt, auto pt) {
        using LT = decltype(lt);
        using PT = decltype(pt);
        hipLaunchKernelGGL((accept_vector_kernel<LT, PT>), dim3(d.total_q), dim3(kNT), 0, a.stream,
                           a.logits, a.probs, a.draft_tokens, a.uniforms, a.spec_lens, a.temperature,
                           (const int32_t *)(a.ws + a.plan.off_cu_q),
                           (const int32_t *)(a.ws + a.plan.off_row_req), d.vocab, d.max_spec_len,
                           d.logits_row_stride, d.probs_row_stride,
                           (int32_t *)(a.ws + a.plan.off_row_flag), (int32_t *)(a.ws + a.plan.off_row_cand));
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

}  // namespace adaspec
