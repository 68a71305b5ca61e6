// Tree acceptance for 16-bit logits and draft probabilities of one type, V % 8 == 0,
// V <= 524288 (the shapes of the streaming chain kernel), in two kernels:
//
//   1. node statistics, one workgroup per node (= logits row), one read of the row: the maximum
//      and its index, and for a sampled request the normaliser Z with its per-step parts S0[];
//   2. the walk, one workgroup per request: from the root, at every node it reaches it tests
//      the children in turn and, after each rejection, sweeps the node's logits and
//      draft-probability rows once for the next residual mass; where the walk stops it draws
//      the token.  It writes the request's outputs itself.
// Nodes the walk does not reach cost their statistics only, and a node where the first child
// is accepted never reads its draft-probability row.
//
// Same procedure as the portable node kernel (tree.hip):
//   stage 0: P = softmax(logits / T); after each rejected child r = max(0, P - q), P = r / sum(r),
// evaluated in its closed form (see kernel 2).
// The row is walked by 1024 threads with 16-byte loads: element (s * 1024 + t) * 8 + e belongs
// to step s, thread t.  A "sweep" leaves, per step, the total mass S[s] (fp32 sums over the 128
// elements of 16 neighbouring lanes, fp64 above that); R = sum of the S[s].  The draw needs no
// sweep of its own: the step where the prefix crosses comes from S[]; the threads then load
// their 8 elements of that one step again, a scan over the threads finds the one where the
// prefix crosses, and it picks the element.  What a child's test needs (its token, the token's
// logit and draft probability, its uniform) is fetched when the walk arrives at the parent, so a
// test is arithmetic on values already on chip.
#include "adaspec_internal.h"
#include "device_utils.h"
#include "row_registers.h"
#include "row_stream.h"

namespace adaspec {

__device__ __forceinline__ int sane_parent_f(int p, int j) { return j == 0 ? -1 : min(max(p, 0), j - 1); }

// what kernel 1 leaves per node
struct TreeNodeStat {
    float  m;               // maximum logit
    int    arg;             // its lowest index (greedy requests; 0 for sampled ones, which never emit it)
    double Z;               // sum_v 2^((l_v - m) c) = sum of S0[]      (sampled requests only)
    double S0[kNSteps];     // the same sum step by step
};
size_t tree_node_stat_bytes() { return sizeof(TreeNodeStat); }

// ---- kernel 1: statistics of every node ---------------------------------------------------------
// ONE read of the row.  The sums of a step are taken relative to the maximum of the 128 elements of
// each 16-lane group (known as soon as the group's loads are there) and put on the row's maximum at
// the end: S0[s] = sum_g part[s][g] * 2^((gmax[s][g] - m) c).  A sampled row costs one exponential
// per element, as a second sweep would, but the row is not fetched a second time.
template <class DT>
__global__ __launch_bounds__(kNT, 8) void tree_node_stats_kernel(
    const char *__restrict__ logits, const int32_t *__restrict__ spec_lens,
    const float *__restrict__ temperature, int B, int V, int max_spec_len, int64_t lstride,
    TreeNodeStat *__restrict__ stats)
{
    __shared__ float wmax[kNW];
    __shared__ int warg[kNW];
    __shared__ float part[kNSteps][kWave], gmax[kNSteps][kWave];
    __shared__ double S[kNSteps];
    __shared__ int wtot[kNW], owner;
    __shared__ float owner_T;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x;
    const char *lrow = logits + (int64_t)r * lstride * 2;
    const int nsteps = ceil_div(V / 8, kNT);

    // The first 1024 draft lengths and temperatures, then the first steps of the row: all requested before
    // anything is waited for.  Which request owns row r (only its temperature is needed) is found by a block
    // scan of n_i = k_i + 1, 1024 requests at a time, while the row's data travels.
    int n_first = 0;
    float t_first = 0.f;
    if (tid < B) {
        n_first = min(max(spec_lens[tid], 0), max_spec_len) + 1;
        t_first = temperature[tid];
    }
    RowPipe<false> pipe;
    pipe.start(lrow, lrow, nsteps, V, tid);
    if (tid == 0) owner = -1;
    {
        int carry = 0;
        for (int base = 0; base < B; base += kNT) {
            const int i = base + tid;
            int n = n_first;
            float tt = t_first;
            if (base > 0) {
                n = i < B ? min(max(spec_lens[i], 0), max_spec_len) + 1 : 0;
                tt = i < B ? temperature[i] : 0.f;
            }
            const int inc = wave_scan_incl_dpp(n);
            lds_barrier();                                      // (later trips: wtot of the trip before has been read)
            if (lane == 63) wtot[wv] = inc;
            lds_barrier();                                      // LDS only: the row's loads stay in flight
            int pre = carry, tot = carry;
#pragma unroll
            for (int w = 0; w < kNW; ++w) {
                if (w < wv) pre += wtot[w];
                tot += wtot[w];
            }
            const int start = pre + inc - n;
            if (i < B && r >= start && r < start + n) { owner = i; owner_T = tt; }
            carry = tot;
            if (r < carry) break;                               // uniform: found
        }
    }
    lds_barrier();
    if (owner < 0) {                                            // no request owns this row (inconsistent metadata)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        return;
    }
    const float T = owner_T;
    const bool sampled = T != 0.0f;
    const float cexp = sampled ? 1.4426950408889634f / T : 0.f;
    constexpr float kLowest = -3.0e38f;                          // stands in for -inf: differences stay defined

    TreeNodeStat *st = stats + r;
    if (!sampled) {
        // greedy: the arg-max (lowest index on ties) is all the walk needs
        ArgMax best{-INFINITY, V};
        pipe.run([&](int s, bool in_range, const uint4 &lw, const uint4 &) {
            if (!in_range) return;
            const int v0 = (s * kNT + tid) * 8;
            float x[8];
            unpack8<DT>(lw, x);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (x[e] > best.v) best = ArgMax{x[e], v0 + e};
        });
        best = wave_argmax(best);
        if (lane == 0) { wmax[wv] = best.v; warg[wv] = best.i; }
        __syncthreads();
        best = ArgMax{wmax[0], warg[0]};
#pragma unroll
        for (int w = 1; w < kNW; ++w) best = argmax_merge(best, ArgMax{wmax[w], warg[w]});
        if (best.i >= V) best.i = 0;
        if (tid == 0) { st->m = best.v; st->arg = best.i; st->Z = 1.0; }
        return;
    }
    // sampled: maximum and normaliser; the index of the maximum is not needed (a sampled walk never emits it)
    float tmax = kLowest;
    pipe.run([&](int s, bool in_range, const uint4 &lw, const uint4 &) {
        float x[8];
        float mx = kLowest;
        if (in_range) {
            unpack8<DT>(lw, x);
#pragma unroll
            for (int e = 0; e < 8; ++e) mx = fmaxf(mx, x[e]);
        }
        const float gm = row16_max(mx);
        tmax = fmaxf(tmax, gm);
        float acc = 0.f;
        if (in_range) {
            const float off = fminf(-gm * cexp, 3.0e38f);        // stays finite when the whole group is -inf
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += __builtin_amdgcn_exp2f(fmaf(x[e], cexp, off));
        }
        acc = row16_sum(acc);
        if ((lane & 15) == 0) { part[s][wv * 4 + (lane >> 4)] = acc; gmax[s][wv * 4 + (lane >> 4)] = gm; }
    });
    tmax = wave_max(tmax);
    if (lane == 0) wmax[wv] = tmax;
    __syncthreads();
    float m = wmax[0];
#pragma unroll
    for (int w = 1; w < kNW; ++w) m = fmaxf(m, wmax[w]);
    // wavefront w puts the 64 group sums of steps w, w + 16, ... on the row's maximum and adds them up
    for (int s = wv; s < nsteps; s += kNW) {
        const double t = wave_sum((double)(part[s][lane] * __builtin_amdgcn_exp2f((gmax[s][lane] - m) * cexp)));
        if (lane == 0) S[s] = t;
    }
    __syncthreads();
    double Z = 0.0;
    for (int s = 0; s < nsteps; ++s) Z += S[s];
    if (tid == 0) { st->m = m; st->arg = 0; st->Z = Z; }
    if (tid < kNSteps) st->S0[tid] = tid < nsteps ? S[tid] : 0.0;
}

// ---- kernel 2: the walk of every request ---------------------------------------------------------
// After s rejected children the distribution at a node is
//     P_s = max(0, p - c_s q) / G_s,   G_s = sum_v max(0, p_v - c_s q_v),   c_0 = 0, c_{s+1} = c_s + G_s
// (substitute P_s into r = max(0, P_s - q) and pull the positive factor 1 / G_s out of the maximum).
// So the walk keeps two numbers per node, (c, G), and every sweep costs the same few operations per
// element whatever the stage.  A stage whose residual has no mass leaves (c, G) as they are, and so does
// every later stage at that node.
struct WalkScratch {
    float  part[kNSteps][kWave];        // per step: fp32 sums of the 64 groups of 16 lanes (wave * 4 + lane / 16)
    double S[kNSteps];
    double wsum[kNW];
    float  ch_l[64], ch_q[64], ch_u[64];   // per child node: logit and draft probability of its token, its uniform
    int    ch_x[64];                    // its token
    unsigned long long kids;
    int fallback, hit, last_thread;
    int fallback_tot[kNW];              // (start-up only) per-wavefront row counts of the requests before this one
};

template <class DT>
__global__ __launch_bounds__(kNT, 4) void accept_tree_walk_fast_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const int32_t *__restrict__ parents,
    const float *__restrict__ uniforms, const int32_t *__restrict__ spec_lens,
    const float *__restrict__ temperature, const int32_t *__restrict__ cu_q,
    const TreeNodeStat *__restrict__ stats, int V, int total_q, int max_spec_len, int64_t lstride,
    int64_t pstride, int out_stride, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ out_accept_len, int32_t *__restrict__ out_path)
{
    __shared__ WalkScratch sm;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i = blockIdx.x;
    const int k = min(max(spec_lens[i], 0), max_spec_len);
    const float T = temperature[i];
    // first row of the request: from the metadata kernel if the caller ran it (large batches), else the rows
    // of the requests before it, added up by the workgroup
    int r0;
    if (cu_q != nullptr) {
        r0 = cu_q[i];
    } else {
        int part = 0;
        for (int j = tid; j < i; j += kNT) part += min(max(spec_lens[j], 0), max_spec_len) + 1;
        part = wave_sum(part);
        if (lane == 0) sm.fallback_tot[wv] = part;
        __syncthreads();
        r0 = 0;
#pragma unroll
        for (int w = 0; w < kNW; ++w) r0 += sm.fallback_tot[w];
    }
    if (r0 < 0 || r0 + k + 1 > total_q) return;                 // inconsistent metadata: leave the request alone
    const float cexp = T == 0.0f ? 0.f : 1.4426950408889634f / T;
    const int nsteps = ceil_div(V / 8, kNT);
    int32_t *o = out_tokens + (int64_t)i * out_stride;
    int32_t *pth = out_path + (int64_t)i * out_stride;

    // state of the node the walk stands on
    const char *lrow = logits, *prow = probs;
    float m = 0.f, invZ = 1.f;

    // max(0, p - c q) at one entry from its logit and draft probability (c = 0: p itself)
    auto residual = [&](float l, float q, float c) -> float {
        return fmaxf(0.f, fmaf(-c, q, __builtin_amdgcn_exp2f((l - m) * cexp) * invZ));
    };
    // this thread's 8 masses of one step: before any sweep the unnormalised 2^((l - m) cexp) the node's
    // statistics were summed from, afterwards max(0, p - c q)
    auto mass8 = [&](bool in_range, const uint4 &lw, const uint4 &qw, bool swept, float c, float (&rv)[8]) -> float {
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) rv[e] = 0.f;
        if (in_range) {
            float x[8];
            unpack8<DT>(lw, x);
            if (!swept) {
#pragma unroll
                for (int e = 0; e < 8; ++e) rv[e] = __builtin_amdgcn_exp2f((x[e] - m) * cexp);
            } else {
                float q[8];
                unpack8<DT>(qw, q);
#pragma unroll
                for (int e = 0; e < 8; ++e) rv[e] = residual(x[e], q[e], c);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc += rv[e];
        }
        return acc;
    };
    // one sweep over both rows: S[] and the total of max(0, p - c q)
    auto sweep = [&](float c) -> double {
        for_each_step<true>(lrow, prow, nsteps, V, tid, [&](int s, bool in_range, const uint4 &lw, const uint4 &qw) {
            float acc = 0.f;
            if (in_range) {
                float x[8], q[8];
                unpack8<DT>(lw, x);
                unpack8<DT>(qw, q);
#pragma unroll
                for (int e = 0; e < 8; ++e) acc += residual(x[e], q[e], c);
            }
            acc = row16_sum(acc);
            if ((lane & 15) == 0) sm.part[s][wv * 4 + (lane >> 4)] = acc;
        });
        return finish_sweep(sm.part, sm.S, nsteps, wv, lane);
    };

    int u = 0, depth = 0;
    for (;;) {
        const int r = r0 + u;
        lrow = logits + (int64_t)r * lstride * 2;
        prow = probs + (int64_t)(r - i) * pstride * 2;          // read only if the node has children
        const TreeNodeStat *st = stats + r;
        __syncthreads();                                        // everything of the previous node has been read
        // children of u (lane c of the first wavefront looks at node c) and what their tests need
        if (tid < kWave) {
            const bool is_child = lane > u && lane <= k && sane_parent_f(parents[r0 + lane], lane) == u;
            const unsigned long long kmask = __builtin_amdgcn_ballot_w64(is_child);
            if (lane == 0) { sm.kids = kmask; sm.hit = -1; sm.last_thread = -1; sm.fallback = -1; }
            if (is_child) {
                const int x = draft_tokens[r0 - i + lane - 1];
                sm.ch_x[lane] = x;
                sm.ch_l[lane] = elem16<DT>(lrow, x);
                sm.ch_q[lane] = elem16<DT>(prow, x);
                sm.ch_u[lane] = uniforms[2 * (int64_t)(r0 + lane - 1)];
            }
        } else if (tid < kWave + kNSteps) {
            sm.S[tid - kWave] = st->S0[tid - kWave];
        }
        m = st->m;
        const int arg = st->arg;
        double R = st->Z;                                       // total of S[]
        invZ = (float)(1.0 / R);
        __syncthreads();
        unsigned long long kids = sm.kids;

        int next = -1, cand = arg;
        if (T == 0.0f) {
            // greedy: the first child that carries the target's arg-max, else stop with the arg-max
            while (kids != 0ull && next < 0) {
                const int c = __builtin_ctzll(kids);
                kids &= kids - 1;
                if (sm.ch_x[c] == arg) next = c;
            }
        } else {
            double cd = 0.0, Gd = 1.0;                          // (c, G) of the current distribution
            float cf = 0.f, invG = 1.f;
            bool swept = false, frozen = false;
            while (kids != 0ull) {
                const int c = __builtin_ctzll(kids);
                kids &= kids - 1;
                {   // every thread evaluates the test from the values fetched on arrival: no exchange needed
                    const float qx = sm.ch_q[c];
                    const float px = residual(sm.ch_l[c], qx, cf) * invG;
                    const bool accepted = (qx > 0.f) ? (sm.ch_u[c] < px / qx) : true;
                    if (accepted) { next = c; break; }
                }
                if (frozen) continue;                           // the residual had no mass before: it has none now
                const double ct = cd + Gd;
                const double Gt = sweep((float)ct);
                if (Gt > 0.0) {
                    cd = ct; Gd = Gt;
                    cf = (float)ct; invG = (float)(1.0 / Gt);
                    R = Gt;
                } else {                                        // P == q everywhere: the state stays; S[] again
                    frozen = true;
                    R = sweep(cf);
                }
                swept = true;
            }
            if (next < 0) {
                // ---- the draw from (S, R): of the last sweep, or of the node's statistics ----------------
                const double tau = (double)uniforms[2 * (int64_t)r + 1] * R;
                int sstar = -1, last_pos_step = 0;
                double before = 0.0, run = 0.0, before_last = 0.0;
                for (int s = 0; s < nsteps; ++s) {
                    const double Ss = sm.S[s];
                    if (Ss > 0.0) { last_pos_step = s; before_last = run; }
                    if (sstar < 0 && run + Ss > tau) { sstar = s; before = run; }
                    run += Ss;
                }
                if (sstar < 0) { sstar = last_pos_step; before = before_last; }   // rounding left no crossing
                float rv[8];
                float mine;
                {
                    const int v0 = (sstar * kNT + tid) * 8;
                    uint4 lw = make_uint4(0, 0, 0, 0), qw = make_uint4(0, 0, 0, 0);
                    if (v0 < V) {
                        lw = *reinterpret_cast<const uint4 *>(lrow + (int64_t)v0 * 2);
                        if (swept) qw = *reinterpret_cast<const uint4 *>(prow + (int64_t)v0 * 2);
                    }
                    mine = mass8(v0 < V, lw, qw, swept, cf, rv);
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
                // the crossing thread, and (in case rounding leaves none) the last thread with mass
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
                    else sm.fallback = lastpos;
                }
                __syncthreads();
                cand = sm.hit;
                if (cand < 0) cand = sm.fallback;
                if (cand < 0) cand = arg;
            }
        }
        if (next < 0) {                                         // the walk stops here
            if (tid == 0) {
                o[depth] = cand;
                pth[depth] = -1;
                out_accept_len[i] = depth;
            }
            for (int j = depth + 1 + tid; j < out_stride; j += kNT) { o[j] = -1; pth[j] = -1; }
            return;
        }
        if (tid == 0) { o[depth] = sm.ch_x[next]; pth[depth] = next; }
        ++depth;
        u = next;
    }
}

// Every walk workgroup adds up the rows of the requests before its own: fine for a few thousand requests,
// quadratic beyond; larger batches take the row offsets from the metadata kernel.
bool tree_fast_needs_plan(const adaspec_accept_dims &d) { return d.batch > 2048; }

hipError_t launch_accept_tree_fast(const AcceptArgs &a, const int32_t *parents, int32_t *out_path)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.total_q == 0) return hipSuccess;
    TreeNodeStat *stats = (TreeNodeStat *)(a.ws + a.plan.off_tree_stat);
    auto launch = [&](auto tag) {
        using DT = decltype(tag);
        hipLaunchKernelGGL((tree_node_stats_kernel<DT>), dim3(d.total_q), dim3(kNT), 0, a.stream,
                           (const char *)a.logits, a.spec_lens, a.temperature, d.batch, d.vocab, d.max_spec_len,
                           d.logits_row_stride, stats);
        hipLaunchKernelGGL((accept_tree_walk_fast_kernel<DT>), dim3(d.batch), dim3(kNT), 0, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.draft_tokens, parents, a.uniforms,
                           a.spec_lens, a.temperature,
                           tree_fast_needs_plan(d) ? (const int32_t *)(a.ws + a.plan.off_cu_q) : nullptr, stats, d.vocab,
                           d.total_q, d.max_spec_len, d.logits_row_stride, d.probs_row_stride, d.out_stride,
                           a.out_tokens, a.out_accept_len, out_path);
    };
    if (d.logits_dtype == ADASPEC_F16) launch(F16{});
    else launch(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec
