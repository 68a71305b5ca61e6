// Register-resident acceptance kernel for gfx950: 16-bit logits and draft
// probabilities, V % 8 == 0, V <= 131072.
//
// One workgroup of 1024 threads per logits row.  The whole logits row is loaded
// ONCE into registers (16 bytes = 8 elements per thread per step, V/8192 steps),
// the draft-probability row is streamed ONCE, nothing is re-read from memory
// except one 16-byte chunk per thread for the final token search:
//
//   0. which request owns the row: block scan of spec_lens (its loads are requested
//      before the row's, LDS-only barriers), no plan kernel in front
//   1. the row is requested step by step while ONE sweep follows the loads:
//      m = max and Z = sum 2^((l - m) c), c = log2(e) / T, against a running
//      per-thread reference, (m, z) pairs merged through LDS;
//      greedy rows: argmax (lowest index on ties) and done
//   2. stream q (zero-size descriptor for bonus rows): per-step sums of
//      r = max(0, 2^((l - m) c) / Z - q), 16-lane DPP sums in fp32, fp64 above
//   3. one wavefront: per-step block totals -> R, tau = u1 * R, the step it* whose
//      running total first exceeds tau (lane-parallel fp64 scan)
//   4. inside step it*: fp64 scan over wavefronts and lanes -> the owning thread,
//      which walks its 8 elements
// Per-element arithmetic is fp32; every sum across threads is fp64.
// A per-row form: every logits row is evaluated completely, the emit kernel applies the sequential rule
// afterwards.  AUTO prefers the two-pass form in row parts (accept_parts.hip), which reads less and spreads
// every row over many workgroups; this kernel remains as a forced path, and in resolve mode as the second
// pass of batches above 1024 requests: the streaming kernel (accept_stream.hip) in test-only mode judges
// every draft row, then this kernel runs steps 1-4 once per REQUEST, on the row that decides its token, and
// writes the request's outputs.
#include "adaspec_internal.h"
#include "device_utils.h"
#include "row_registers.h"

namespace adaspec {

constexpr int kFT = 1024;                // threads per row
constexpr int kFW = kFT / kWave;         // 16 wavefronts
constexpr int kQPre = 4;                 // draft-prob chunks in flight per thread

struct FastScratch {
    alignas(16) float sw[kFW][16][4];   // per step: the four 16-lane row sums of every wavefront
    float  wm[kFW], wz[kFW];
    float  av[kFW];
    int    ai[kFW];
    double tau, before;
    int    itstar, retry;
    int    row_i, row_j, row_k;
    float  row_T;
    int    first_hit, last_pos;
    int    ahead[kFW];                  // resolve mode: rows of the requests in front, per wavefront
};

// kResolve = false: one workgroup per logits row; writes the row's flag and candidate, the emit kernel
// applies the sequential rule afterwards.
// kResolve = true: second pass of the two-pass form, one workgroup per REQUEST.  The first pass
// (accept_stream_kernel in test-only mode) has left the flag of every draft row; this pass finds the
// request's first rejected draft (or its bonus row), runs the sampling part of the rule on that one
// row only, and writes the request's outputs itself.  Rows after a rejection are never read, accepted
// rows are read once (by the first pass), and no emit kernel is needed.
template <class DT, int ITER, bool kResolve>
__global__ __launch_bounds__(kFT) void accept_fast_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const float *__restrict__ uniforms,
    const int32_t *__restrict__ spec_lens, const float *__restrict__ temperature, int B, int V,
    int max_spec_len, int64_t lstride, int64_t pstride, int32_t *__restrict__ row_flag,
    int32_t *__restrict__ row_cand, int out_stride, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ out_accept_len)
{
    using P = Pair16<DT>;
    __shared__ FastScratch sm;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    int r = blockIdx.x;
    int ri = 0, j = 0, k = 0;
    float T = 0.f;
    if constexpr (kResolve) {
        // request i = blockIdx.x: its first row (sum of n over the requests in front), k and T
        const int i = blockIdx.x;
        int ahead = 0;
        for (int base = 0; base < i; base += kFT) {
            const int idx = base + tid;
            if (idx < i) ahead += min(max(spec_lens[idx], 0), max_spec_len) + 1;
        }
        k = min(max(spec_lens[i], 0), max_spec_len);          // uniform: scalar loads
        T = temperature[i];
        ahead = wave_sum(ahead);
        if (lane == 0) sm.ahead[wv] = ahead;
        lds_barrier();
        int start = 0;
#pragma unroll
        for (int w = 0; w < kFW; ++w) start += sm.ahead[w];
        start = __builtin_amdgcn_readfirstlane(start);
        // the first rejected draft (every wavefront looks for itself: no second barrier)
        int a = k;
        for (int j0 = 0; j0 < k; j0 += kWave) {
            const int f = j0 + lane < k ? row_flag[start + j0 + lane] : 1;
            const unsigned long long rej = __ballot(f == 0);
            if (rej) { a = j0 + (int)__builtin_ctzll(rej); break; }
        }
        a = __builtin_amdgcn_readfirstlane(a);
        ri = i; j = a; r = start + a;
        if (wv == 0) {                        // everything but the sampled token: accepted drafts, padding, length
            int32_t *o = out_tokens + (int64_t)i * out_stride;
            for (int jj = lane; jj < out_stride; jj += kWave)
                if (jj != a) o[jj] = jj < a ? draft_tokens[start - i + jj] : -1;
            if (lane == 0) out_accept_len[i] = a;
        }
        if (T == 0.0f && a < k) {             // greedy and rejected: the first pass left the row's arg-max
            if (tid == 0) out_tokens[(int64_t)i * out_stride + a] = row_cand[r];
            return;
        }
    }
    // the row's result: its candidate token (per-row form) or the request's token at position j
    auto put_cand = [&](int cand) {
        if constexpr (kResolve) out_tokens[(int64_t)ri * out_stride + j] = cand;
        else row_cand[r] = cand;
    };
    const int nchunks = V >> 3;
    const char *lrow = logits + (int64_t)r * lstride * 2;
    const uint32_t tid16 = (uint32_t)tid * 16u;

    // ---- 1. the logits row, once ---------------------------------------------------------
    // Buffer loads: the row's base and size sit in a scalar descriptor, the lane supplies a 32-bit
    // offset (no 64-bit address registers), and chunks past the end of the row read as zero.  All
    // loads of the row are in flight together; they only need the row index, so they are requested
    // before the row's request is even known.
    const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(lrow), 0, V * 2, 0x00020000);
    auto load_chunk = [&](const __amdgpu_buffer_rsrc_t &rs, int it) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)tid16, it * (kFT * 16), 0);
        return make_uint4(v.x, v.y, v.z, v.w);
    };
    // Chunks past the end of the row arrive as zeros (buffer range check) and must count as -inf:
    // OR-ing the -inf pattern into them is branch-free and in place, one chunk at a time right before
    // its first use, so that no step waits for data it does not need yet.
    auto blank_tail = [&](uint4 &v, int it) {
        const uint32_t ninf = (it * kFT + tid >= nchunks) ? P::kNegInf2 : 0u;
        // (in assembly so that the result stays in the registers the load wrote: as plain C the
        // compiler keeps blanked copies next to the originals and runs out of registers)
        asm volatile("v_or_b32 %0, %0, %4\n\tv_or_b32 %1, %1, %4\n\tv_or_b32 %2, %2, %4\n\tv_or_b32 %3, %3, %4"
                     : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w) : "v"(ninf));
    };
    // (the first 1024 draft lengths are requested ahead of the row: the memory counter is in order,
    // so anything asked for after the row would only be seen once the whole row has arrived)
    int n_first = 0;
    float t_first = 0.f;
    if constexpr (!kResolve) {
        if (tid < B) {
            n_first = min(max(spec_lens[tid], 0), max_spec_len) + 1;
            t_first = temperature[tid];       // the owner of the row's request publishes it with (i, j, k)
        }
    }
    // Only the first kLPre steps of the row are requested here.  A wavefront executes in order and a
    // load instruction is held back while the memory pipeline of the compute unit is full, so a
    // wavefront that asks for its whole share at once does nothing else until most of it has
    // arrived; the rest is requested step by step inside the sweep below.
    constexpr int kLPre = ITER < 8 ? ITER : 8;
    uint4 lg[ITER];
#pragma unroll
    for (int it = 0; it < kLPre; ++it) {
        lg[it] = load_chunk(rl, it);
        __builtin_amdgcn_sched_barrier(0);    // issue in step order: the sweep consumes them in that order
    }

    // ---- which request owns row r?  (while the loads travel)  Block scan of n_i = k_i + 1 over the
    // requests, 1024 at a time; the thread whose request covers r publishes (i, j, k).
    if constexpr (!kResolve) {
        int carry = 0;
        for (int base = 0; base < B; base += kFT) {
            const int i = base + tid;
            int n = n_first;
            float tt = t_first;
            if (base > 0) {
                n = i < B ? min(max(spec_lens[i], 0), max_spec_len) + 1 : 0;
                tt = i < B ? temperature[i] : 0.f;
            }
            const int inc = wave_scan_incl(n, lane);
            if (lane == 63) sm.ai[wv] = inc;
            lds_barrier();           // LDS only: the row's loads stay in flight
            int pre = carry, tot = carry;
#pragma unroll
            for (int w = 0; w < kFW; ++w) {
                if (w < wv) pre += sm.ai[w];
                tot += sm.ai[w];
            }
            const int start = pre + inc - n;
            if (r >= start && r < start + n) { sm.row_i = i; sm.row_j = r - start; sm.row_k = n - 1; sm.row_T = tt; }
            lds_barrier();           // LDS only: the row's loads stay in flight
            carry = tot;
            if (r < carry) break;
        }
        ri = __builtin_amdgcn_readfirstlane(sm.row_i);       // wave-uniform: the loads below are scalar
        j = __builtin_amdgcn_readfirstlane(sm.row_j);
        k = __builtin_amdgcn_readfirstlane(sm.row_k);
        T = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sm.row_T)));
    }
    const bool bonus = j >= k;
    const char *prow = probs + (int64_t)(r - ri) * pstride * 2;
    const bool sampled = T != 0.0f;
    const bool has_q = sampled && !bonus;
    // A row without draft probabilities (bonus row, q == 0) gets a descriptor of size zero: its loads
    // return zeros without touching memory.  So the stream below is unconditional and the number of
    // loads in flight is the same on every path, which lets each wait name exactly the chunk it needs.
    __amdgpu_buffer_rsrc_t rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(prow), 0, has_q ? V * 2 : 0, 0x00020000);
    uint4 qb[kQPre];
    if (!sampled) {
        // greedy: argmax with the lowest index on ties (elements are visited in index order per thread)
        ArgMax best{-INFINITY, V};
#pragma unroll
        for (int it = kLPre; it < ITER; ++it) lg[it] = load_chunk(rl, it);
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            blank_tail(lg[it], it);
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
            if constexpr (!kResolve) row_flag[r] = bonus ? 1 : (draft_tokens[r - ri] == a.i);
            put_cand(a.i);
        }
        return;
    }

    // ---- 2. maximum and normaliser, in ONE sweep, step by step as the loads land ----------------
    // The vector ALUs would idle while the row travels, so the normaliser is accumulated on line
    // against a running per-thread reference m_run = max(0, largest logit seen so far).  Both 16-bit
    // formats are sign-magnitude, so a packed SIGNED 16-bit integer maximum started at +0 tracks it
    // with one instruction per two elements; when it grows, the partial sum is rescaled (one extra
    // exponential per 8-element chunk).  Thread, wavefront and block results are combined as (m, z)
    // pairs.  A row without any positive logit (block maximum 0) is redone with the exact maximum.
    const float c = 1.4426950408889634f / T;
    short2v pm = {0, 0};
    float m_run = 0.f, zt = 0.f;
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        // keep the memory pipeline fed: the row's step it + kLPre, then the first steps of the
        // draft-probability row (they are consumed by the streaming pass further down)
        if (it + kLPre < ITER) lg[it + kLPre] = load_chunk(rl, it + kLPre);
        else if (it + kLPre - ITER < kQPre) qb[it + kLPre - ITER] = load_chunk(rq, it + kLPre - ITER);
        blank_tail(lg[it], it);
        keep_packed(lg[it]);
        const uint32_t *w = &lg[it].x;
#pragma unroll
        for (int e = 0; e < 4; ++e) pm = __builtin_elementwise_max(pm, __builtin_bit_cast(short2v, w[e]));
        const float mn = P::lo((uint32_t)(uint16_t)max(pm.x, pm.y));
        zt *= __builtin_amdgcn_exp2f((m_run - mn) * c);
        m_run = mn;
        const float mnc = mn * c;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            zt += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mnc));
            zt += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mnc));
            if (e == 1) __builtin_amdgcn_sched_barrier(0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    // The draft token is asked for only now (scalar load): scalar loads and LDS reads share one
    // counter that cannot tell them apart, so an earlier request would have made the temperature
    // above wait for this load as well.  It arrives while the block result is being exchanged.
    __builtin_amdgcn_sched_barrier(0);
    int x = -1;
    if constexpr (!kResolve) x = bonus ? -1 : draft_tokens[r - ri];
    {
        const float mw = wave_max(m_run);
        const float zw = wave_sum(zt * __builtin_amdgcn_exp2f((m_run - mw) * c));
        if (lane == 0) { sm.wm[wv] = mw; sm.wz[wv] = zw; }
        if (tid == 0) { sm.first_hit = kFT; sm.last_pos = -1; }
    }
    lds_barrier();
    float m = sm.wm[0];
#pragma unroll
    for (int w = 1; w < kFW; ++w) m = fmaxf(m, sm.wm[w]);
    double Zd = 0.0;
#pragma unroll
    for (int w = 0; w < kFW; ++w) Zd += (double)(sm.wz[w] * __builtin_amdgcn_exp2f((sm.wm[w] - m) * c));
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
        lds_barrier();                        // everyone has read wm / wz
        if (lane == 0) sm.wm[wv] = mt;
        lds_barrier();
        m = sm.wm[0];
#pragma unroll
        for (int w = 1; w < kFW; ++w) m = fmaxf(m, sm.wm[w]);
        const float mc0 = m * c;
        float z2 = 0.f;
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            keep_packed(lg[it]);
            const uint32_t *w = &lg[it].x;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                z2 += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mc0));
                z2 += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mc0));
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        z2 = wave_sum(z2);
        if (lane == 0) sm.wz[wv] = z2;
        lds_barrier();
        Zd = 0.0;
#pragma unroll
        for (int w = 0; w < kFW; ++w) Zd += (double)sm.wz[w];
    }
    // e_v = 2^(l_v * c - m * c) from here on: one fused expression for the accept test, the residual
    // sums and the final search, so that all of them see the same p_v = e_v / Z
    const float mc = m * c;
    const float invZ = (float)(1.0 / Zd);

    // accept test, first half.  x is the same for the whole workgroup, so l_x and q_x come by scalar
    // loads (aligned 32-bit words holding the 16-bit values): they do not queue behind the vector
    // loads of the draft-probability stream.  They are requested here and used after the streaming
    // pass, so nobody waits for them.
    uint32_t lw_x = 0, qw_x = 0;
    const float u_acc = uniforms[2 * (int64_t)r], u_draw = uniforms[2 * (int64_t)r + 1];
    if constexpr (!kResolve) {
        if (!bonus) {
            lw_x = reinterpret_cast<const uint32_t *>(lrow)[x >> 1];
            qw_x = reinterpret_cast<const uint32_t *>(prow)[x >> 1];
        }
    }

    // ---- 3./4. residual mass per step, block totals, the step that holds tau ------------------
    bool use_q = has_q;
    for (int attempt = 0; attempt < 2; ++attempt) {
#pragma unroll
        for (int it = 0; it < ITER; ++it) {
            const uint4 qv = qb[it % kQPre];
            if (it + kQPre < ITER) qb[it % kQPre] = load_chunk(rq, it + kQPre);
            keep_packed(lg[it]);
            const uint32_t *w = &lg[it].x, *qw = &qv.x;
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float ea = __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mc));
                const float eb = __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mc));
                acc += fmaxf(0.f, fmaf(ea, invZ, -P::lo(qw[e])));
                acc += fmaxf(0.f, fmaf(eb, invZ, -P::hi(qw[e])));
                if (e == 1) __builtin_amdgcn_sched_barrier(0);
            }
            acc = row16_sum(acc);             // fp32 over 16 lanes; the 64 row sums per step are added in fp64
            if ((lane & 15) == 0) sm.sw[wv][it][lane >> 4] = acc;
            __builtin_amdgcn_sched_barrier(0);
        }
        lds_barrier();
        if (wv == 0) {
            // One wavefront finishes the reduction: lane L owns step L (16 wavefronts x 4 row sums each,
            // added in fp64), an inclusive scan over the lanes gives the running totals, R is the
            // last of them, and the step that holds tau = u1 * R is the first lane whose running
            // total exceeds it.
            double t = 0.0;
            if (lane < ITER) {
#pragma unroll
                for (int w = 0; w < kFW; ++w) {
                    const float4 v = *reinterpret_cast<const float4 *>(sm.sw[w][lane]);
                    t = t + (((double)v.x + (double)v.y) + ((double)v.z + (double)v.w));
                }
            }
            const double incl = wave_scan_incl(t, lane);
            const double R = __shfl(incl, ITER - 1, kWave);
            const double tq = (double)u_draw * R;
            const unsigned long long hits = __ballot(lane < ITER && incl > tq);
            // (no lane can only happen through rounding at u1 -> 1: take the last step)
            const int pick = hits ? (int)__builtin_ctzll(hits) : ITER - 1;
            const double bef = __shfl(incl - t, pick, kWave);
            if (lane == 0) {
                sm.tau = tq; sm.before = bef; sm.itstar = pick;
                sm.retry = !(R > 0.0) && use_q;
            }
        }
        lds_barrier();
        if (!sm.retry) break;
        // p == q everywhere (R == 0): draw from p instead; the q row is not read on the second pass
        use_q = false;
        rq = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(prow), 0, 0, 0x00020000);
#pragma unroll
        for (int it = 0; it < kQPre; ++it) qb[it] = make_uint4(0, 0, 0, 0);
        __syncthreads();
    }
    const double tau = sm.tau, before = sm.before;

    if (!kResolve && tid == 0) {              // accept test, second half
        int flag = 1;
        if (!bonus) {
            const float lx = (x & 1) ? P::hi(lw_x) : P::lo(lw_x);
            const float qx = (x & 1) ? P::hi(qw_x) : P::lo(qw_x);
            const float px = __builtin_amdgcn_exp2f(fmaf(lx, c, -mc)) * invZ;
            flag = (qx > 0.f) ? (u_acc < px / qx) : 1;
        }
        row_flag[r] = flag;
    }

    // ---- 5. inside step it*: the owning thread, then the element --------------------------------
    const int itstar = __builtin_amdgcn_readfirstlane(sm.itstar);
    uint4 lstar = lg[0];
#pragma unroll
    for (int it = 1; it < ITER; ++it)
        if (it == itstar) lstar = lg[it];
    const int cstar = itstar * kFT + tid;
    const uint4 qstar = load_chunk(rq, itstar);
    // residual mass ahead of this wavefront inside step it*: lane L adds up wavefront L's four row
    // sums, a scan over the lanes gives the prefixes (done while the chunk above travels)
    double base = before;
    {
        double ws = 0.0;
        if (lane < kFW) {
            const float4 v = *reinterpret_cast<const float4 *>(sm.sw[lane][itstar]);
            ws = ((double)v.x + (double)v.y) + ((double)v.z + (double)v.w);
        }
        const double wincl = wave_scan_incl(ws, lane);
        const double ahead = __shfl(wincl, max(wv - 1, 0), kWave);
        if (wv > 0) base = base + ahead;
    }
    __builtin_amdgcn_sched_barrier(0);
    float rv[8], sstar = 0.f;
    {
        const uint32_t *w = &lstar.x, *qw = &qstar.x;
#pragma unroll
        for (int e = 0; e < 4; ++e) {          // same expressions, same order as in the streaming pass
            const float ea = __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mc));
            const float eb = __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mc));
            rv[2 * e] = fmaxf(0.f, fmaf(ea, invZ, -P::lo(qw[e])));
            rv[2 * e + 1] = fmaxf(0.f, fmaf(eb, invZ, -P::hi(qw[e])));
            sstar += rv[2 * e];
            sstar += rv[2 * e + 1];
        }
    }
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
        put_cand(cstar * 8 + pick);
    }
    if (owner < 0 && tid == 0) put_cand(0);         // no mass anywhere (non-finite input): stay defined
}

bool accept_fast_path_supported(const adaspec_accept_dims &d, const void *logits, const void *probs)
{
    if (d.logits_dtype == ADASPEC_F32 || d.logits_dtype != d.probs_dtype) return false;
    if (d.vocab % 8 || d.vocab > kFT * 8 * 16) return false;
    if (d.logits_row_stride % 8 || d.probs_row_stride % 8) return false;
    if ((reinterpret_cast<uintptr_t>(logits) & 15u) || (reinterpret_cast<uintptr_t>(probs) & 15u)) return false;
    return true;
}

template <bool kResolve>
static hipError_t launch_fast_kernel(const AcceptArgs &a)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.total_q == 0) return hipSuccess;
    const int steps = ceil_div(d.vocab / 8, kFT);
    auto launch = [&](auto tag, auto it_tag) {
        using DT = decltype(tag);
        constexpr int ITER = decltype(it_tag)::value;
        hipLaunchKernelGGL((accept_fast_kernel<DT, ITER, kResolve>), dim3(kResolve ? d.batch : d.total_q),
                           dim3(kFT), 0, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.draft_tokens, a.uniforms,
                           a.spec_lens, a.temperature, d.batch, d.vocab, d.max_spec_len,
                           d.logits_row_stride, d.probs_row_stride,
                           (int32_t *)(a.ws + a.plan.off_row_flag), (int32_t *)(a.ws + a.plan.off_row_cand),
                           d.out_stride, a.out_tokens, a.out_accept_len);
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

hipError_t launch_accept_fast(const AcceptArgs &a) { return launch_fast_kernel<false>(a); }

// Second pass of the two-pass form (after launch_accept_test): one workgroup per request.
hipError_t launch_accept_resolve(const AcceptArgs &a) { return launch_fast_kernel<true>(a); }

}  // namespace adaspec
