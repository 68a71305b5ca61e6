// Tree acceptance of one node per workgroup, for 16-bit logits and draft probabilities of one
// type, V % 8 == 0, V <= 131072 (the shapes of the register-resident chain kernel).
//
// Same procedure and same per-element arithmetic as the portable node kernel (tree.hip):
//   stage 0: P = softmax(logits / T); after each rejected child r = max(0, P - q), P = r / sum(r).
// What differs is how the row is walked: 1024 threads, 16-byte loads, element (s * 1024 + t) * 8 + e
// belongs to step s, thread t.  A "sweep" reads the logits row (and from stage 1 on the
// draft-probability row) once and leaves, per step, the total mass S[s] (fp32 sums over the 128
// elements of 16 neighbouring lanes, fp64 above that); R = sum of the S[s].  A node costs: one sweep
// for the maximum, one for the normaliser (= the stage-0 mass, unnormalised), one per rejected
// child.  The draw needs no sweep of its own: the step where the prefix crosses comes from S[];
// the threads then load their 8 elements of that one step again, a scan over the threads finds
// the one where the prefix crosses, and it picks the element.  The row is not kept in registers:
// later sweeps hit the caches.  What a child's test needs (its token's logit, draft probability
// and uniform) is fetched when the kernel starts, so a test is arithmetic on values already on chip.
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
    float  part[kNSteps][kWave];        // per step: fp32 sums of the 64 groups of 16 lanes (wave * 4 + lane / 16)
    double S[kNSteps];
    float  ch_l[64], ch_q[64], ch_u[64];   // per child node: logit and draft probability of its token, its uniform
    float  inv_r[64];                   // 1 / R_s, s = 1 ..
    unsigned long long kept;            // bit s: stage s kept P_{s-1} (no positive part)
    unsigned long long kids;
    int verdict, hit, last_thread;
};

template <class DT>
__global__ __launch_bounds__(kNT, 8) void accept_tree_node_fast_kernel(
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

    auto elem16 = [](const char *row, int v) -> float {
        const uint16_t b = reinterpret_cast<const uint16_t *>(row)[v];
        return Pair16<DT>::lo((uint32_t)b);
    };
    // children of this node (lane c of the first wavefront looks at node c) and what their tests need
    float pre_l = 0.f, pre_q = 0.f, pre_u = 0.f;
    bool is_child = false;
    if (tid < kWave) {
        is_child = lane > u && lane <= k && sane_parent_f(parents[r0 + lane], lane) == u;
        const unsigned long long kids = __builtin_amdgcn_ballot_w64(is_child);
        if (lane == 0) { sm.kids = kids; sm.kept = 0ull; sm.hit = -1; sm.last_thread = -1; }
        if (is_child) {
            const int x = draft_tokens[r0 - i + lane - 1];
            pre_l = elem16(lrow, x);
            pre_q = elem16(prow, x);
            pre_u = uniforms[2 * (int64_t)(r0 + lane - 1)];
        }
    }

    auto unpack = [](const uint4 &w, float (&x)[8]) {
        x[0] = Pair16<DT>::lo(w.x); x[1] = Pair16<DT>::hi(w.x);
        x[2] = Pair16<DT>::lo(w.y); x[3] = Pair16<DT>::hi(w.y);
        x[4] = Pair16<DT>::lo(w.z); x[5] = Pair16<DT>::hi(w.z);
        x[6] = Pair16<DT>::lo(w.w); x[7] = Pair16<DT>::hi(w.w);
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
    if (is_child) { sm.ch_l[lane] = pre_l; sm.ch_q[lane] = pre_q; sm.ch_u[lane] = pre_u; }
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

    // the mass of this thread's 8 elements of step s at the given stage (0: unnormalised 2^((l - m) c))
    auto step_mass = [&](int s, int s_stage, bool keep_last, const float (&inv)[kHoist],
                         unsigned long long kept, float (&rv)[8]) -> float {
        const int v0 = (s * kNT + tid) * 8;
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) rv[e] = 0.f;
        if (v0 < V) {
            float x[8];
            unpack(*reinterpret_cast<const uint4 *>(lrow + (int64_t)v0 * 2), x);
            if (s_stage == 0) {
#pragma unroll
                for (int e = 0; e < 8; ++e) rv[e] = __builtin_amdgcn_exp2f((x[e] - m) * cexp);
            } else {
                float q[8];
                unpack(*reinterpret_cast<const uint4 *>(prow + (int64_t)v0 * 2), q);
#pragma unroll
                for (int e = 0; e < 8; ++e) rv[e] = mass(x[e], q[e], s_stage, keep_last, inv, kept);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += rv[e];
        }
        return acc;
    };
    // One sweep: S[] and the total.
    auto sweep = [&](int s_stage, bool keep_last) -> double {
        float inv[kHoist];
#pragma unroll
        for (int j = 0; j < kHoist; ++j) inv[j] = (j + 1 < s_stage) ? sm.inv_r[j + 1] : 1.0f;
        const unsigned long long kept = sm.kept;
#pragma unroll 1
        for (int s = 0; s < nsteps; ++s) {
            float rv[8];
            const float acc = row16_sum(step_mass(s, s_stage, keep_last, inv, kept, rv));
            if ((lane & 15) == 0) sm.part[s][wv * 4 + (lane >> 4)] = acc;
        }
        __syncthreads();
        // wavefront s adds up the 64 partial sums of step s
        {
            const double t = wave_sum(wv < nsteps ? (double)sm.part[wv][lane] : 0.0);
            if (lane == 0) sm.S[wv] = t;
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
        // every thread evaluates the test from the values fetched at the start: no exchange needed
        {
            float inv[kHoist];
#pragma unroll
            for (int j = 0; j < kHoist; ++j) inv[j] = (j + 1 <= stage) ? sm.inv_r[j + 1] : 1.0f;
            const float qx = sm.ch_q[c];
            const float px = dist(sm.ch_l[c], qx, stage, inv, sm.kept);
            const bool accepted = (qx > 0.f) ? (sm.ch_u[c] < px / qx) : true;
            if (accepted) { next = c; break; }
        }
        ++stage;
        keep_last = false;
        R = sweep(stage, false);
        if (!(R > 0.0)) {                                       // P == q everywhere: the state stays
            keep_last = true;
            R = sweep(stage, true);
        }
        if (tid == 0) {
            sm.inv_r[stage] = (float)(1.0 / R);
            if (keep_last) sm.kept |= 1ull << stage;
        }
        __syncthreads();
    }
    if (next >= 0) {
        if (tid == 0) { node_next[r] = next; row_cand[r] = best.i; }
        return;
    }

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
    // this thread's 8 elements of that step, once more
    float rv[8];
    float mine;
    {
        float inv[kHoist];
#pragma unroll
        for (int j = 0; j < kHoist; ++j) inv[j] = (j + 1 < stage) ? sm.inv_r[j + 1] : 1.0f;
        mine = step_mass(sstar, stage, keep_last, inv, sm.kept, rv);
    }
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
        double cum = excl;
        int pick = -1, lastpos = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            cum += (double)rv[e];
            if (rv[e] > 0.f) lastpos = v0 + e;
            if (pick < 0 && cum > tau && rv[e] > 0.f) pick = v0 + e;
        }
        if (crossing) sm.hit = pick >= 0 ? pick : lastpos;
        else sm.verdict = lastpos;                               // fallback candidate
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
