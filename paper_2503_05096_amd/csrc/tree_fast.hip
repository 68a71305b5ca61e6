// Tree acceptance of one node per workgroup, for 16-bit logits and draft probabilities of one
// type, V % 8 == 0, V <= 131072 (the shapes of the register-resident chain kernel).
//
// Same procedure and same per-element arithmetic as the portable node kernel (tree.hip):
//   stage 0: P = softmax(logits / T); after each rejected child r = max(0, P - q), P = r / sum(r).
// What differs is how the row is walked: 1024 threads, 16-byte loads, element (s * 1024 + t) * 8 + e
// belongs to step s, thread t.  A "sweep" reads the logits row (and from stage 1 on the
// draft-probability row) once and leaves, per thread, the fp32 sum of its 8 elements in every step
// (seg[s]) and, per step, the fp64 total over the threads (S[s]); R = sum of the S[s].  A node
// costs: one sweep for the maximum, one for the normaliser (= the stage-0 mass, unnormalised), one
// per rejected child.  The draw needs no sweep of its own: the step where the prefix crosses comes
// from S[], the thread from a scan over that step's seg values, and that thread alone loads its
// 8 elements again.  The row is not kept in registers: later sweeps hit the caches.
#include "adaspec_internal.h"
#include "device_utils.h"
#include "row_registers.h"

namespace adaspec {

constexpr int kNT = 1024;
constexpr int kNW = kNT / kWave;
constexpr int kNSteps = 16;             // V <= kNT * 8 * kNSteps
constexpr int kHoist = 3;               // stages whose 1/R is kept in registers during a sweep

__device__ __forceinline__ int sane_parent_f(int p, int j) { return j == 0 ? -1 : min(max(p, 0), j - 1); }

struct NodeScratch {
    float  wmax[kNW];
    int    warg[kNW];
    double wsum[kNW];
    double step_tot[kNW][kNSteps];
    double S[kNSteps];
    float  inv_r[64];                   // 1 / R_s, s = 1 ..
    unsigned long long kept;            // bit s: stage s kept P_{s-1} (no positive part)
    unsigned long long kids;
    int verdict, hit, last_thread;
};

template <class DT>
__global__ __launch_bounds__(kNT) void accept_tree_node_fast_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const int32_t *__restrict__ parents,
    const float *__restrict__ uniforms, const int32_t *__restrict__ spec_lens,
    const float *__restrict__ temperature, const int32_t *__restrict__ cu_q,
    const int32_t *__restrict__ row_req, int V, int max_spec_len, int64_t lstride, int64_t pstride,
    int32_t *__restrict__ node_next, int32_t *__restrict__ row_cand)
{
    __shared__ NodeScratch sm;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x;
    const int i = row_req[r];
    const int r0 = cu_q[i];
    const int u = r - r0;
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const float T = temperature[i];
    const char *lrow = logits + (int64_t)r * lstride * 2;
    const char *prow = probs + (int64_t)(r - i) * pstride * 2;   // read only if the node has children
    const int nsteps = ceil_div(V / 8, kNT);

    if (tid < kWave) {
        const bool child = lane > u && lane <= k && sane_parent_f(parents[r0 + lane], lane) == u;
        const unsigned long long kids = __builtin_amdgcn_ballot_w64(child);
        if (lane == 0) { sm.kids = kids; sm.kept = 0ull; sm.hit = -1; sm.last_thread = -1; }
    }

    auto unpack = [](const uint4 &w, float (&x)[8]) {
        x[0] = Pair16<DT>::lo(w.x); x[1] = Pair16<DT>::hi(w.x);
        x[2] = Pair16<DT>::lo(w.y); x[3] = Pair16<DT>::hi(w.y);
        x[4] = Pair16<DT>::lo(w.z); x[5] = Pair16<DT>::hi(w.z);
        x[6] = Pair16<DT>::lo(w.w); x[7] = Pair16<DT>::hi(w.w);
    };
    auto elem16 = [](const char *row, int v) -> float {
        const uint16_t b = reinterpret_cast<const uint16_t *>(row)[v];
        return Pair16<DT>::lo((uint32_t)b);
    };

    // ---- sweep 1: maximum and its lowest index ------------------------------------------------
    ArgMax best{-INFINITY, V};
    for (int s = 0; s < nsteps; ++s) {
        const int v0 = (s * kNT + tid) * 8;
        if (v0 >= V) break;
        float x[8];
        unpack(*reinterpret_cast<const uint4 *>(lrow + (int64_t)v0 * 2), x);
#pragma unroll
        for (int e = 0; e < 8; ++e)
            if (x[e] > best.v) best = ArgMax{x[e], v0 + e};
    }
    best = wave_argmax(best);
    if (lane == 0) { sm.wmax[wv] = best.v; sm.warg[wv] = best.i; }
    __syncthreads();
    best = ArgMax{sm.wmax[0], sm.warg[0]};
#pragma unroll
    for (int w = 1; w < kNW; ++w) best = argmax_merge(best, ArgMax{sm.wmax[w], sm.warg[w]});
    if (best.i >= V) best.i = 0;
    unsigned long long kids = sm.kids;

    if (T == 0.0f) {
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
    float invZ = 1.0f;

    // P_s at one entry from its logit and draft probability (s >= 0); inv[] = hoisted 1/R_1..
    auto dist = [&](float l, float q, int s, const float (&inv)[kHoist], unsigned long long kept) -> float {
        float P = __builtin_amdgcn_exp2f((l - m) * cexp) * invZ;
#pragma unroll
        for (int j = 1; j <= kHoist; ++j)
            if (j <= s) P = (((kept >> j) & 1ull) ? P : fmaxf(0.f, P - q)) * inv[j - 1];
        for (int j = kHoist + 1; j <= s; ++j)
            P = (((kept >> j) & 1ull) ? P : fmaxf(0.f, P - q)) * sm.inv_r[j];
        return P;
    };
    // r_s at one entry (s >= 1); keep_last: stage s keeps P_{s-1}
    auto mass = [&](float l, float q, int s, bool keep_last, const float (&inv)[kHoist],
                    unsigned long long kept) -> float {
        const float P = dist(l, q, s - 1, inv, kept);
        return keep_last ? P : fmaxf(0.f, P - q);
    };

    float seg[kNSteps];
    // One sweep: seg[] of every thread, S[] and the total.  stage 0: unnormalised 2^((l - m) c).
    auto sweep = [&](int s_stage, bool keep_last) -> double {
        float inv[kHoist];
#pragma unroll
        for (int j = 0; j < kHoist; ++j) inv[j] = (j + 1 < s_stage) ? sm.inv_r[j + 1] : 1.0f;
        const unsigned long long kept = sm.kept;
#pragma unroll
        for (int s = 0; s < kNSteps; ++s) {
            seg[s] = 0.f;
            const int v0 = (s * kNT + tid) * 8;
            if (s < nsteps && v0 < V) {
                float x[8];
                unpack(*reinterpret_cast<const uint4 *>(lrow + (int64_t)v0 * 2), x);
                float acc = 0.f;
                if (s_stage == 0) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc += __builtin_amdgcn_exp2f((x[e] - m) * cexp);
                } else {
                    float q[8];
                    unpack(*reinterpret_cast<const uint4 *>(prow + (int64_t)v0 * 2), q);
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc += mass(x[e], q[e], s_stage, keep_last, inv, kept);
                }
                seg[s] = acc;
            }
            if (s < nsteps) {
                const double ws = wave_sum((double)seg[s]);
                if (lane == 0) sm.step_tot[wv][s] = ws;
            }
        }
        __syncthreads();
        if (tid < kNSteps) {
            double t = 0.0;
            if (tid < nsteps)
                for (int w = 0; w < kNW; ++w) t += sm.step_tot[w][tid];
            sm.S[tid] = t;
        }
        __syncthreads();
        double R = 0.0;
#pragma unroll
        for (int s = 0; s < kNSteps; ++s) R += sm.S[s];
        return R;
    };

    // ---- sweep 2: the normaliser (= total of the stage-0 mass) ---------------------------------
    double R = sweep(0, false);
    invZ = (float)(1.0 / R);

    // ---- the children, one after another -------------------------------------------------------
    int next = -1, stage = 0;
    bool keep_last = false;
    while (kids != 0ull) {
        const int c = __builtin_ctzll(kids);
        kids &= kids - 1;
        __syncthreads();                                        // the previous verdict has been read
        if (tid == 0) {
            const int x = draft_tokens[r0 - i + c - 1];
            float inv[kHoist];
#pragma unroll
            for (int j = 0; j < kHoist; ++j) inv[j] = (j + 1 <= stage) ? sm.inv_r[j + 1] : 1.0f;
            const float qx = elem16(prow, x);
            const float px = dist(elem16(lrow, x), qx, stage, inv, sm.kept);
            sm.verdict = (qx > 0.f) ? (uniforms[2 * (int64_t)(r0 + c - 1)] < px / qx) : 1;
        }
        __syncthreads();
        if (sm.verdict) { next = c; break; }
        ++stage;
        keep_last = false;
        R = sweep(stage, false);
        if (!(R > 0.0)) {                                       // P == q everywhere: the state stays
            keep_last = true;
            R = sweep(stage, true);
        }
        if (tid == 0) {                                         // (sweep ended on a barrier; the next reader
            sm.inv_r[stage] = (float)(1.0 / R);                 //  is behind the barrier at the loop's top or below)
            if (keep_last) sm.kept |= 1ull << stage;
        }
    }
    if (next >= 0) {
        if (tid == 0) { node_next[r] = next; row_cand[r] = best.i; }
        return;
    }
    __syncthreads();

    // ---- the draw from (seg, S, R) of the last sweep ------------------------------------------
    const double tau = (double)uniforms[2 * (int64_t)r + 1] * R;
    int sstar = -1, last_pos_step = 0;
    double before = 0.0, run = 0.0, before_last = 0.0;
#pragma unroll
    for (int s = 0; s < kNSteps; ++s) {
        const double Ss = sm.S[s];
        if (Ss > 0.0) { last_pos_step = s; before_last = run; }
        if (sstar < 0 && run + Ss > tau) { sstar = s; before = run; }
        run += Ss;
    }
    if (sstar < 0) { sstar = last_pos_step; before = before_last; }   // rounding left no crossing
    float mine = 0.f;
#pragma unroll
    for (int s = 0; s < kNSteps; ++s) mine = (s == sstar) ? seg[s] : mine;
    // scan over the threads of that step
    const double wi = wave_scan_incl((double)mine, lane);
    double we = __shfl_up(wi, 1, kWave);
    if (lane == 0) we = 0.0;
    if (lane == 63) sm.wsum[wv] = wi;
    if (mine > 0.f) atomicMax(&sm.last_thread, tid);
    __syncthreads();
    double wp = 0.0;
#pragma unroll
    for (int w = 0; w < kNW; ++w) wp += (w < wv) ? sm.wsum[w] : 0.0;
    const double excl = before + wp + we, incl = before + wp + wi;
    const bool crossing = incl > tau && !(excl > tau);
    const int last_thread = sm.last_thread;
    // the crossing thread, and (in case rounding leaves none) the last thread with mass, look at their 8 elements
    if (crossing || tid == last_thread) {
        const int v0 = (sstar * kNT + tid) * 8;
        float x[8], q[8], inv[kHoist];
#pragma unroll
        for (int j = 0; j < kHoist; ++j) inv[j] = (j + 1 < stage) ? sm.inv_r[j + 1] : 1.0f;
        unpack(*reinterpret_cast<const uint4 *>(lrow + (int64_t)v0 * 2), x);
        if (stage > 0) unpack(*reinterpret_cast<const uint4 *>(prow + (int64_t)v0 * 2), q);
        double cum = excl;
        int pick = -1, lastpos = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float rv = stage == 0 ? __builtin_amdgcn_exp2f((x[e] - m) * cexp)
                                        : mass(x[e], q[e], stage, keep_last, inv, sm.kept);
            cum += (double)rv;
            if (rv > 0.f) lastpos = v0 + e;
            if (pick < 0 && cum > tau && rv > 0.f) pick = v0 + e;
        }
        if (crossing) sm.hit = pick >= 0 ? pick : lastpos;
        else if (tid == last_thread) sm.verdict = lastpos;       // fallback candidate
    }
    __syncthreads();
    if (tid == 0) {
        int cand = sm.hit;
        if (cand < 0) cand = last_thread >= 0 ? sm.verdict : best.i;
        node_next[r] = -1;
        row_cand[r] = cand;
    }
}

hipError_t launch_accept_tree_nodes_fast(const AcceptArgs &a, const int32_t *parents)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.total_q == 0) return hipSuccess;
    auto launch = [&](auto tag) {
        using DT = decltype(tag);
        hipLaunchKernelGGL((accept_tree_node_fast_kernel<DT>), dim3(d.total_q), dim3(kNT), 0, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.draft_tokens, parents, a.uniforms,
                           a.spec_lens, a.temperature, (const int32_t *)(a.ws + a.plan.off_cu_q),
                           (const int32_t *)(a.ws + a.plan.off_row_req), d.vocab, d.max_spec_len,
                           d.logits_row_stride, d.probs_row_stride, (int32_t *)(a.ws + a.plan.off_row_flag),
                           (int32_t *)(a.ws + a.plan.off_row_cand));
    };
    if (d.logits_dtype == ADASPEC_F16) launch(F16{});
    else launch(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec
