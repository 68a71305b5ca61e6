// Two-pass acceptance in row PARTS for gfx950: 16-bit logits and draft probabilities of one type,
// V % 8 == 0, V <= 131072, up to 1024 requests.
//
// The sequential rule (accept drafts in order, recover one token at the first rejection, else take the
// bonus token) needs two things: the accept test on draft rows, for which the row's softmax statistics
// (m, Z) suffice, and the residual distribution with a draw from it on ONE row per request.  Both are
// sweeps over vocabulary rows of 256 KB that a single compute unit takes 7-12 us for; handing whole rows
// to workgroups leaves the chip unevenly loaded (382 rows on 256 compute units) and every row a serial
// chain.  Here every row is cut into parts, one small workgroup (256 threads) each, a few per compute
// unit, all resident at once.
//
//   accept_rowparts_kernel   workgroup = (draft row, part).  Finds the row's request from spec_lens itself
//       (block scan, up to 1024 requests), streams its part of the logits row once (part h = steps h,
//       h + n_parts, ... of 4 KB; 8 steps in flight, maximum and normaliser on line) and leaves the part's
//       (maximum, normaliser) or, for a greedy request, (maximum, arg-max); part 0 also leaves what the
//       accept test needs besides: the draft token, its logit, its draft probability and the uniform.
//       Records are stored per SLOT (request, draft position), so the second pass reads them without
//       knowing where the request's rows start.  Workgroup 0 also writes cu_q and clears the tickets of
//       the second pass.
//   accept_decide_kernel     workgroup = (request, part of <= 1024 chunks of 16 bytes).  Merges the part
//       statistics of the request's draft rows, applies the accept test to each (one lane per draft), finds
//       the first rejection -> the deciding row; part 0 writes the accepted drafts, the padding and the
//       length.  A greedy rejection is decided by the merged arg-max.  Otherwise the workgroup loads its
//       part of the deciding row (and of its draft-probability row) and publishes the residual and
//       probability mass per (step, wavefront, 16-lane row); the workgroup that finishes LAST for its
//       request (an integer ticket per request, one atomic add at the exit, no waiting) puts the parts on
//       one scale, finds the (part, step, wavefront) that holds tau = u1 * R, recomputes that wavefront's
//       64 chunks with the same expressions and picks the element.
// Per-element arithmetic is fp32, sums across lanes and workgroups fp64, in a fixed order: outputs do
// not depend on which workgroup arrives last.
//
// What the time goes to (MI355X, 510 rows of V = 128256, time stamps): a dependent memory access costs
// 1.2-1.7 us and the chain has six of them (first pass: lengths -> row; second pass: slot records -> row,
// then stores acknowledged -> ticket -> partial sums -> the 64 chunks of the draw), the two launches add
// 1.7 us each, and the rows themselves stream at 5.0-5.5 TB/s.
#include "adaspec_internal.h"
#include "device_utils.h"
#include "row_registers.h"

namespace adaspec {

constexpr int kQT = 256;                    // threads per workgroup
constexpr int kQW = kQT / kWave;            // 4 wavefronts
constexpr int kStatSteps = 8;               // first pass: steps of kQT chunks per part (32 KB of logits)
constexpr int kStatWgsPerCu = 6;           // first pass: workgroups that fit a compute unit (80 registers each)
constexpr int kStatTargetWgsPerCu = 3;     // ... and how many the launch aims for: few long streams read faster than many short ones
constexpr int kStatParts = 8;               // parts per row at most: V <= 8 * 8 * 256 * 8 = 131072
constexpr int kSumSteps = 4;                // second pass: steps per part (16 KB of logits + 16 KB of probabilities)
constexpr int kSumParts = 16;               // parts per row at most
constexpr int kPartsMaxBatch = 1024;        // requests the in-kernel scan covers (4 per thread)
constexpr int kPartsMaxSlots = 32768;       // batch * max_spec_len slots the workspace is laid out for
static_assert(kSumParts * kSumSteps == 64, "one lane per step of the row in the final search");
static_assert(kSumParts * kSumSteps * kQW == kQT, "one thread per (part, step, wavefront) in the final search");

// Phase time stamps for tuning builds (-DADASPEC_STAMPS): thread 0 of every workgroup leaves the 100 MHz
// wall clock at up to 8 points of each kernel; adaspec_debug_read_stamps copies them out.  Product builds
// compile none of it.
#ifdef ADASPEC_STAMPS
constexpr int kStampGroups = 8192;
static __device__ long long g_stamps[2][kStampGroups][8];
#define ADASPEC_STAMP(which, k)                                                                        \
    do {                                                                                               \
        if (threadIdx.x == 0 && blockIdx.x < kStampGroups) g_stamps[which][blockIdx.x][k] = wall_clock64(); \
    } while (0)
#else
#define ADASPEC_STAMP(which, k) do { } while (0)
#endif

// what part 0 of a draft row leaves for the accept test
struct SlotRec { int x; uint32_t lx_bits, qx_bits, u0_bits; };

// ---- memory that crosses workgroups inside one launch ---------------------------------------------
// The partial sums of the second pass are written by one workgroup and read by another one of the same
// launch, possibly on another XCD (each XCD has its own L2).  They travel as relaxed agent-scope atomic
// stores and loads (write-through / read-through to the level all XCDs share); the writer waits until its
// stores have been acknowledged before it takes its ticket, and the reader's loads depend on the ticket's
// return value.  No cache-wide write-back or invalidate is needed, and nobody waits for anybody.
__device__ __forceinline__ void publish_f32(float *p, float v)
{
    __hip_atomic_store(reinterpret_cast<uint32_t *>(p), __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_u64(void *p, unsigned long long v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long fetch_u64(const void *p)
{
    return __hip_atomic_load(reinterpret_cast<const unsigned long long *>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void publish_stat(HalfStat *p, float m, int arg, double Z)
{
    publish_u64(p, (unsigned long long)__float_as_uint(m) | ((unsigned long long)(uint32_t)arg << 32));
    publish_u64(reinterpret_cast<char *>(p) + 8, (unsigned long long)__double_as_longlong(Z));
}
__device__ __forceinline__ HalfStat fetch_stat(const HalfStat *p)
{
    const unsigned long long a = fetch_u64(p), b = fetch_u64(reinterpret_cast<const char *>(p) + 8);
    HalfStat s;
    s.m = __uint_as_float((uint32_t)a);
    s.arg = (int)(uint32_t)(a >> 32);
    s.Z = __longlong_as_double((long long)b);
    return s;
}

// sums of the second pass: float[B][kSumParts][kSumSteps][kQW][2 kinds (residual, p)][4 rows of 16 lanes]
__device__ __forceinline__ size_t sum_index(int i, int h, int it, int w, int kind)
{
    return ((((size_t)(i * kSumParts + h) * kSumSteps + it) * kQW + w) * 2 + kind) * 4;
}

// One 16-byte chunk (8 elements): residual r_v = max(0, e_v / Z - q_v) and p_v = e_v / Z with
// e_v = 2^(l_v c - m c).  The sums and the final search both call this, so they see the same numbers.
template <class P>
__device__ __forceinline__ void part_chunk_masses(const uint4 &lv, const uint4 &qv, float c, float mc, float invZ,
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

// 16 bytes per lane through a buffer descriptor (past the end of the buffer: zeros); AUX = cache policy bits
// of the instruction (0 = default, 2 = non-temporal: data that is read once)
constexpr int kAuxDefault = 0, kAuxStream = 2;
template <int AUX>
__device__ __forceinline__ uint4 part_load16(__amdgpu_buffer_rsrc_t rs, uint32_t lane_offset, int step)
{
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, (int)lane_offset, step * (kQT * 16), AUX);
    return make_uint4(v.x, v.y, v.z, v.w);
}

// exact maximum of the 8 values of a chunk
template <class P>
__device__ __forceinline__ float chunk_max(const uint4 &v, float m)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) m = fmaxf(m, fmaxf(P::lo(w[e]), P::hi(w[e])));
    return m;
}

// Exact maximum of a thread's STEPS chunks, on the bit patterns.  Both 16-bit formats are sign-magnitude:
// among non-negative values the order of the patterns as SIGNED 16-bit integers is the order of the
// values, and every negative value is a negative integer, so a packed signed maximum (one instruction per
// two elements) is exact as soon as one value is >= +0.  A thread that holds nothing but negative values
// (masked vocabularies) wants the smallest magnitude instead: the packed UNSIGNED minimum.
typedef unsigned short ushort2v __attribute__((ext_vector_type(2)));
template <class P, int STEPS>
__device__ __forceinline__ float thread_max(const uint4 (&lg)[STEPS])
{
    short2v pm = {(short)0x8000, (short)0x8000};
#pragma unroll
    for (int it = 0; it < STEPS; ++it) {
        const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) pm = __builtin_elementwise_max(pm, __builtin_bit_cast(short2v, w[e]));
    }
    int top = max((int)pm.x, (int)pm.y);
    if (top < 0) {
        ushort2v pn = {(unsigned short)0xffff, (unsigned short)0xffff};
#pragma unroll
        for (int it = 0; it < STEPS; ++it) {
            const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) pn = __builtin_elementwise_min(pn, __builtin_bit_cast(ushort2v, w[e]));
        }
        top = min((int)pn.x, (int)pn.y);
    }
    return P::lo((uint32_t)top & 0xffffu);
}

// (maximum, normaliser) of STEPS chunks per thread over the whole workgroup, relative to the workgroup's
// maximum: every thread sums against its own maximum (no barrier between the two sweeps), the pairs are
// merged over the wavefront and, through LDS, over the workgroup.  Returns false if no finite value exists.
template <class P, int STEPS>
__device__ __forceinline__ bool part_max_and_norm(uint4 (&lg)[STEPS], float c, float *s_m, double *s_z,
                                                  int lane, int wv, float &m_out, double &z_out)
{
    const float mt = thread_max<P, STEPS>(lg);
    float zt = 0.f;
    if (mt > -INFINITY) {
        const float mtc = mt * c;
#pragma unroll
        for (int it = 0; it < STEPS; ++it) {
            keep_packed(lg[it]);
            const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                zt += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mtc));
                zt += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mtc));
            }
        }
    }
    const float mw = wave_max(mt);
    const double zw = wave_sum(mt > -INFINITY ? (double)(zt * __builtin_amdgcn_exp2f((mt - mw) * c)) : 0.0);
    if (lane == 0) { s_m[wv] = mw; s_z[wv] = zw; }
    lds_barrier();
    float m = s_m[0];
#pragma unroll
    for (int w = 1; w < kQW; ++w) m = fmaxf(m, s_m[w]);
    double z = 0.0;
#pragma unroll
    for (int w = 0; w < kQW; ++w)
        z += s_m[w] > -INFINITY ? s_z[w] * (double)__builtin_amdgcn_exp2f((s_m[w] - m) * c) : 0.0;
    m_out = m; z_out = z;
    return m > -INFINITY;
}

// arg-max (lowest index on ties) of STEPS chunks per thread over the workgroup; chunk0 = first chunk of the part
template <class P, int STEPS>
__device__ __forceinline__ ArgMax part_argmax(uint4 (&lg)[STEPS], int chunk0, int V, float *s_m, int *s_i,
                                              int tid, int lane, int wv)
{
    ArgMax best{-INFINITY, V};
#pragma unroll
    for (int it = 0; it < STEPS; ++it) {
        keep_packed(lg[it]);
        const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
        const int base = (chunk0 + it * kQT + tid) * 8;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x0 = P::lo(w[e]), x1 = P::hi(w[e]);
            if (x0 > best.v) best = ArgMax{x0, base + 2 * e};
            if (x1 > best.v) best = ArgMax{x1, base + 2 * e + 1};
        }
    }
    best = wave_argmax(best);
    if (lane == 0) { s_m[wv] = best.v; s_i[wv] = best.i; }
    lds_barrier();
    ArgMax b{s_m[0], s_i[0]};
#pragma unroll
    for (int w = 1; w < kQW; ++w) b = argmax_merge(b, ArgMax{s_m[w], s_i[w]});
    return b;
}

// ---------------------------------------------------------------------------------------------------
// First pass: statistics of every draft row, in parts.
template <class DT>
__global__ __launch_bounds__(kQT, kStatWgsPerCu) void accept_rowparts_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const float *__restrict__ uniforms,
    const int32_t *__restrict__ spec_lens, const float *__restrict__ temperature, int B, int V, int total_q,
    int total_draft, int max_spec_len, int n_parts, int64_t lstride, int64_t pstride,
    int32_t *__restrict__ cu_q, int32_t *__restrict__ req_ticket, SlotRec *__restrict__ slot_rec,
    HalfStat *__restrict__ part_stat)
{
    using P = Pair16<DT>;
    __shared__ int s_tot[kQW];
    __shared__ int s_row[5];                 // request, position, k, temperature bits, logits row
    __shared__ float s_m[kQW];
    __shared__ double s_z[kQW];
    __shared__ int s_i[kQW];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int dr = blockIdx.x / n_parts, h = blockIdx.x % n_parts;      // draft row, part
    ADASPEC_STAMP(0, 0);

    // ---- which request owns draft row dr: scan of n_i = k_i + 1, four requests per thread --------------
    int kk[4];
    float tt[4];
    int n_thread = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int i = tid * 4 + u;
        kk[u] = -1;
        tt[u] = 0.f;
        if (i < B) {
            kk[u] = min(max(spec_lens[i], 0), max_spec_len);
            tt[u] = temperature[i];
            n_thread += kk[u] + 1;
        }
    }
    const int inc = wave_scan_incl_dpp(n_thread);
    if (lane == 63) s_tot[wv] = inc;
    if (tid == 0) s_row[0] = -1;
    lds_barrier();
    int first = inc - n_thread;              // cu_q of this thread's first request
#pragma unroll
    for (int w = 0; w < kQW; ++w) first += w < wv ? s_tot[w] : 0;
    {
        int q0 = first;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int i = tid * 4 + u;
            if (kk[u] >= 0) {
                const int d0 = q0 - i;       // first draft row of request i
                if (dr >= d0 && dr < d0 + kk[u]) {
                    s_row[0] = i; s_row[1] = dr - d0; s_row[2] = kk[u];
                    s_row[3] = __float_as_int(tt[u]); s_row[4] = q0 + (dr - d0);
                }
                if (blockIdx.x == 0) {       // one workgroup leaves cu_q and clears the second pass's tickets
                    cu_q[i] = q0;
                    req_ticket[i] = 0;
                    if (i == B - 1) cu_q[B] = q0 + kk[u] + 1;
                }
                q0 += kk[u] + 1;
            }
        }
    }
    lds_barrier();
    const int ri = __builtin_amdgcn_readfirstlane(s_row[0]);
    if (ri < 0 || dr >= total_draft) return;             // no such draft row (also: inconsistent lengths)
    const int j = __builtin_amdgcn_readfirstlane(s_row[1]);
    const float T = __int_as_float(__builtin_amdgcn_readfirstlane(s_row[3]));
    const int r = __builtin_amdgcn_readfirstlane(s_row[4]);
    if (r >= total_q) return;
    ADASPEC_STAMP(0, 1);

    // ---- the part of the row, streamed once: kStatSteps steps in flight, each consumed as it lands -------
    // (a compute unit needs about as long for the exponentials of a row as the memory system needs to
    // deliver it: only a stream whose arithmetic runs under its own loads gets both done in the time of one)
    const int row_chunks = V >> 3;
    const char *lrow = logits + (int64_t)r * lstride * 2;
    // Part h takes the steps h, h + n_parts, h + 2 n_parts, ... of the row, so that the workgroups of a row
    // sweep it together (neighbouring addresses are in flight at the same time), and reads them past the
    // caches: a draft row is read once, here.
    const int row_steps = ceil_div(row_chunks, kQT);
    const int steps = (row_steps - h + n_parts - 1) / n_parts;
    const __amdgpu_buffer_rsrc_t rl = __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(lrow), 0, row_chunks * 16, 0x00020000);
#define ADASPEC_ROW_STEP(s) ((s) * n_parts + h)
#define ADASPEC_STEP_CHUNK(s) (ADASPEC_ROW_STEP(s) * kQT + tid)
#define ADASPEC_STEP_PAST_END(s) (ADASPEC_STEP_CHUNK(s) >= row_chunks)
    const uint32_t tid16 = (uint32_t)tid * 16u;
    uint4 lg[kStatSteps];
#pragma unroll
    for (int u = 0; u < kStatSteps; ++u) lg[u] = part_load16<kAuxStream>(rl, tid16, ADASPEC_ROW_STEP(u));

    const int64_t slot = (int64_t)ri * max_spec_len + j;
    if (h == 0 && tid == 0) {
        // what the accept test needs besides (m, Z): scalar loads, they travel with the row
        const int x = draft_tokens[dr];
        const int xa = min(max(x, 0), V - 1);            // (address only: an out-of-range token must not fault)
        const char *prow = probs + (int64_t)dr * pstride * 2;
        const uint32_t lw = reinterpret_cast<const uint32_t *>(lrow)[xa >> 1];
        const uint32_t qw = reinterpret_cast<const uint32_t *>(prow)[xa >> 1];
        SlotRec rec;
        rec.x = x;
        rec.lx_bits = __float_as_uint((xa & 1) ? P::hi(lw) : P::lo(lw));
        rec.qx_bits = __float_as_uint((xa & 1) ? P::hi(qw) : P::lo(qw));
        rec.u0_bits = __float_as_uint(uniforms[2 * (int64_t)r]);
        slot_rec[slot] = rec;
    }
    HalfStat *my_stat = part_stat + slot * kStatParts + h;
    ADASPEC_STAMP(0, 2);
    // One step of the stream: the chunk of step s (past the end of the part: -inf), used in place, and once
    // it has been consumed the request for the step that takes its place in the window (past the part:
    // zeros, no traffic) into the same registers.  Macros, not lambdas: an array captured by reference
    // would be given a home in scratch memory.
#define ADASPEC_STEP_WORDS(w, s, u)                                                                   \
    const uint32_t ninf_##w = ADASPEC_STEP_PAST_END(s) ? P::kNegInf2 : 0u;                             \
    const uint32_t w[4] = {lg[u].x | ninf_##w, lg[u].y | ninf_##w, lg[u].z | ninf_##w, lg[u].w | ninf_##w};
#define ADASPEC_STEP_REFILL(s, u)                                                                     \
    lg[u] = part_load16<kAuxStream>(rl, tid16, ADASPEC_ROW_STEP((s) + kStatSteps));        \
    __builtin_amdgcn_sched_barrier(0);       /* one step at a time: nothing unpacked ahead of its turn */
    if (T == 0.0f) {
        // greedy: arg-max, lowest index on ties (a thread meets its elements in index order)
        ArgMax best{-INFINITY, V};
        for (int s0 = 0; s0 < steps; s0 += kStatSteps) {
#pragma unroll
            for (int u = 0; u < kStatSteps; ++u) {
                ADASPEC_STEP_WORDS(w, s0 + u, u)
                const int base = ADASPEC_STEP_CHUNK(s0 + u) * 8;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x0 = P::lo(w[e]), x1 = P::hi(w[e]);
                    if (x0 > best.v) best = ArgMax{x0, base + 2 * e};
                    if (x1 > best.v) best = ArgMax{x1, base + 2 * e + 1};
                }
                ADASPEC_STEP_REFILL(s0 + u, u)
            }
        }
        best = wave_argmax(best);
        if (lane == 0) { s_m[wv] = best.v; s_i[wv] = best.i; }
        lds_barrier();
        if (tid == 0) {
            ArgMax b{s_m[0], s_i[0]};
#pragma unroll
            for (int w = 1; w < kQW; ++w) b = argmax_merge(b, ArgMax{s_m[w], s_i[w]});
            HalfStat st; st.m = b.v; st.arg = b.i < V ? b.i : -1; st.Z = 0.0; *my_stat = st;
        }
        return;
    }
    // Maximum and normaliser on line, against a running per-thread reference m_run.  Both 16-bit formats are
    // sign-magnitude: among non-negative values the order of the bit patterns as SIGNED 16-bit integers is
    // the order of the values and every negative value is a negative integer, so a running packed signed
    // maximum (one instruction per two elements) is the exact maximum as soon as the thread has seen one
    // value >= +0; until then (masked vocabularies) the chunk's float maximum is taken the slow way.
    const float c = 1.4426950408889634f / T;
    short2v pm = {(short)0x8000, (short)0x8000};
    float m_run = -INFINITY, zt = 0.f;
    for (int s0 = 0; s0 < steps; s0 += kStatSteps) {
#pragma unroll
        for (int u = 0; u < kStatSteps; ++u) {
            ADASPEC_STEP_WORDS(w, s0 + u, u)
#pragma unroll
            for (int e = 0; e < 4; ++e) pm = __builtin_elementwise_max(pm, __builtin_bit_cast(short2v, w[e]));
            const int top = max((int)pm.x, (int)pm.y);
            const float mn = top >= 0 ? P::lo((uint32_t)top & 0xffffu) : chunk_max<P>(make_uint4(w[0], w[1], w[2], w[3]), m_run);
            if (mn > m_run) {
                zt *= __builtin_amdgcn_exp2f((m_run - mn) * c);          // (-inf - finite) -> 0
                m_run = mn;
            }
            if (m_run > -INFINITY) {
                const float mnc = m_run * c;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    zt += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c, -mnc));
                    zt += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c, -mnc));
                }
            }
            ADASPEC_STEP_REFILL(s0 + u, u)
        }
    }
#undef ADASPEC_STEP_WORDS
#undef ADASPEC_STEP_REFILL
#undef ADASPEC_ROW_STEP
#undef ADASPEC_STEP_CHUNK
#undef ADASPEC_STEP_PAST_END
    const float mw = wave_max(m_run);
    const double zw = wave_sum(m_run > -INFINITY ? (double)(zt * __builtin_amdgcn_exp2f((m_run - mw) * c)) : 0.0);
    if (lane == 0) { s_m[wv] = mw; s_z[wv] = zw; }
    lds_barrier();
    if (tid == 0) {
        float m = s_m[0];
#pragma unroll
        for (int w = 1; w < kQW; ++w) m = fmaxf(m, s_m[w]);
        double z = 0.0;
#pragma unroll
        for (int w = 0; w < kQW; ++w)
            z += s_m[w] > -INFINITY ? s_z[w] * (double)__builtin_amdgcn_exp2f((s_m[w] - m) * c) : 0.0;
        HalfStat st; st.m = m; st.arg = 0; st.Z = z; *my_stat = st;
    }
    ADASPEC_STAMP(0, 3);
}

// (m, Z) of a whole row from its parts' records, or for a greedy request (maximum, arg-max)
struct RowMerge { float m; double Z; int arg; };
__device__ __forceinline__ void load_row_parts(const HalfStat *__restrict__ st, int n_parts, HalfStat (&s)[kStatParts])
{
#pragma unroll
    for (int p = 0; p < kStatParts; ++p) {
        s[p].m = -INFINITY; s[p].arg = -1; s[p].Z = 0.0;
        if (p < n_parts) s[p] = st[p];
    }
}
__device__ __forceinline__ RowMerge merge_row_parts(const HalfStat (&s)[kStatParts], float c, bool greedy)
{
    RowMerge out;
    out.Z = 0.0; out.arg = 0;
    if (greedy) {
        ArgMax b{-INFINITY, 0x7fffffff};
#pragma unroll
        for (int p = 0; p < kStatParts; ++p)
            if (s[p].arg >= 0) b = argmax_merge(b, ArgMax{s[p].m, s[p].arg});
        out.m = b.v;
        out.arg = b.i == 0x7fffffff ? 0 : b.i;
        return out;
    }
    float m = s[0].m;
#pragma unroll
    for (int p = 1; p < kStatParts; ++p) m = fmaxf(m, s[p].m);
#pragma unroll
    for (int p = 0; p < kStatParts; ++p)
        out.Z += s[p].m > -INFINITY ? s[p].Z * (double)__builtin_amdgcn_exp2f((s[p].m - m) * c) : 0.0;
    out.m = m;
    return out;
}

// ---------------------------------------------------------------------------------------------------
// Second pass: the deciding row of every request, in parts, and the draw.
template <class DT>
__global__ __launch_bounds__(kQT, 8) void accept_decide_kernel(
    const char *__restrict__ logits, const char *__restrict__ probs,
    const int32_t *__restrict__ draft_tokens, const float *__restrict__ uniforms,
    const int32_t *__restrict__ spec_lens, const float *__restrict__ temperature, int V, int total_q,
    int total_draft, int max_spec_len, int n_stat_parts, int n_parts, int64_t lstride, int64_t pstride,
    const int32_t *__restrict__ cu_q, int32_t *__restrict__ req_ticket, const SlotRec *__restrict__ slot_rec,
    const HalfStat *__restrict__ part_stat, int out_stride, int32_t *__restrict__ out_tokens,
    int32_t *__restrict__ out_accept_len, float *__restrict__ sums, HalfStat *__restrict__ sum_stat)
{
    using P = Pair16<DT>;
    __shared__ float s_m[kSumParts > kQW ? kSumParts : kQW];
    __shared__ double s_z[kSumParts > kQW ? kSumParts : kQW];
    __shared__ int s_i[kQW];
    __shared__ int s_last;
    __shared__ double mass[kSumParts][kSumSteps][kQW];
    __shared__ double s_tau, s_before;
    __shared__ int s_step, s_retry;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int i = blockIdx.x / n_parts, h = blockIdx.x % n_parts;
    ADASPEC_STAMP(1, 0);

    // ---- the request's first rejected draft: wavefront 0 decides, one lane per draft --------------------
    // The records of the request's first 64 slots are requested before anything else: they need neither
    // the draft count nor the row offset (slots beyond the count hold leftovers, which are not looked at).
    // Requested this early they are back before the first workgroups of the launch start streaming rows;
    // later they would queue behind that traffic.
    __shared__ int s_dec[3];
    __shared__ double s_dec_z;
    SlotRec rec;
    HalfStat parts[kStatParts];
    rec.x = 0; rec.lx_bits = rec.qx_bits = rec.u0_bits = 0;
    if (wv == 0 && lane < max_spec_len) {
        const int64_t slot = (int64_t)i * max_spec_len + lane;
        rec = slot_rec[slot];
        load_row_parts(part_stat + slot * kStatParts, n_stat_parts, parts);
    }
    const int start = cu_q[i];
    const int k = min(max(spec_lens[i], 0), max_spec_len);          // uniform: scalar loads
    const float T = temperature[i];
    const bool sampled = T != 0.0f;
    const float c = sampled ? 1.4426950408889634f / T : 0.f;
    if (wv == 0) {
        int a0 = k;
        RowMerge row0;                                               // statistics of the deciding row, if a draft
        row0.m = 0.f; row0.Z = 1.0; row0.arg = 0;
        for (int j0 = 0; j0 < k; j0 += kWave) {
            const int jj = j0 + lane;
            int flag = 1;
            RowMerge mine;
            mine.m = 0.f; mine.Z = 1.0; mine.arg = 0;
            if (jj < k) {
                if (j0 > 0) {                                        // more drafts than lanes: the next 64 slots
                    const int64_t slot = (int64_t)i * max_spec_len + jj;
                    rec = slot_rec[slot];
                    load_row_parts(part_stat + slot * kStatParts, n_stat_parts, parts);
                }
                mine = merge_row_parts(parts, c, !sampled);
                if (sampled) {
                    const float lx = __uint_as_float(rec.lx_bits), qx = __uint_as_float(rec.qx_bits);
                    const float px = __builtin_amdgcn_exp2f(fmaf(lx, c, -(mine.m * c))) * (float)(1.0 / mine.Z);
                    flag = (qx > 0.f) ? (__uint_as_float(rec.u0_bits) < px / qx) : 1;
                } else {
                    flag = rec.x == mine.arg;
                }
            }
            const unsigned long long rej = __ballot(flag == 0);
            if (rej) {
                const int src = (int)__builtin_ctzll(rej);
                a0 = j0 + src;
                row0.m = __shfl(mine.m, src, kWave);
                row0.Z = __shfl(mine.Z, src, kWave);
                row0.arg = __shfl(mine.arg, src, kWave);
                break;
            }
        }
        if (lane == 0) { s_dec[0] = a0; s_dec[1] = __float_as_int(row0.m); s_dec[2] = row0.arg; s_dec_z = row0.Z; }
    }
    lds_barrier();
    RowMerge row;
    row.m = __int_as_float(s_dec[1]); row.arg = s_dec[2]; row.Z = s_dec_z;
    const int a = __builtin_amdgcn_readfirstlane(s_dec[0]);
    const int r = start + a;
    const bool bonus = a >= k;
    int32_t *o = out_tokens + (int64_t)i * out_stride;
    if (h == 0 && wv == 0) {                  // everything but the sampled token
        for (int jj = lane; jj < out_stride; jj += kWave)
            if (jj != a) o[jj] = (jj < a && start - i + jj < total_draft) ? draft_tokens[start - i + jj] : -1;
        if (lane == 0) out_accept_len[i] = a;
    }
    if (r >= total_q) {                       // inconsistent lengths: stay inside the tensors
        if (h == 0 && tid == 0) o[a] = 0;
        return;
    }
    if (!sampled && !bonus) {                 // greedy and rejected: the row's arg-max, already merged
        if (h == 0 && tid == 0) o[a] = row.arg;
        return;
    }

    ADASPEC_STAMP(1, 1);
    // ---- this workgroup's part of the deciding row (and of its draft probabilities) -------------------
    const int row_chunks = V >> 3;
    const int chunk0 = h * (kSumSteps * kQT);
    const int nchunks = min(row_chunks - chunk0, kSumSteps * kQT);   // >= 1 by the choice of n_parts
    const char *lrow = logits + (int64_t)r * lstride * 2;
    const char *prow = probs + (int64_t)(r - i) * pstride * 2;
    const bool has_q = sampled && !bonus;
    const __amdgpu_buffer_rsrc_t rl =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(lrow) + (int64_t)chunk0 * 16, 0, nchunks * 16, 0x00020000);
    // (a bonus row has no draft probabilities: descriptor of size zero, the loads return zeros)
    const __amdgpu_buffer_rsrc_t rq =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(prow) + (int64_t)chunk0 * 16, 0, has_q ? nchunks * 16 : 0, 0x00020000);
    const uint32_t tid16 = (uint32_t)tid * 16u;
    uint4 lg[kSumSteps], qg[kSumSteps];
#pragma unroll
    for (int it = 0; it < kSumSteps; ++it) lg[it] = part_load16<kAuxDefault>(rl, tid16, it);
#pragma unroll
    for (int it = 0; it < kSumSteps; ++it) qg[it] = part_load16<kAuxDefault>(rq, tid16, it);
    const float u_draw = uniforms[2 * (int64_t)r + 1];
#pragma unroll
    for (int it = 0; it < kSumSteps; ++it) {
        const uint32_t ninf = (it * kQT + tid >= nchunks) ? P::kNegInf2 : 0u;
        lg[it].x |= ninf; lg[it].y |= ninf; lg[it].z |= ninf; lg[it].w |= ninf;
    }
    HalfStat *my_stat = sum_stat + i * kSumParts + h;
    float *my_sums = sums + sum_index(i, h, 0, 0, 0);
    ADASPEC_STAMP(1, 2);
    if (!sampled) {
        // greedy bonus row: arg-max of the part; the last workgroup merges the parts
        const ArgMax b = part_argmax<P, kSumSteps>(lg, chunk0, V, s_m, s_i, tid, lane, wv);
        if (tid == 0) publish_stat(my_stat, b.v, b.i < V ? b.i : -1, 0.0);
    } else {
        float m = row.m;
        double Zd = row.Z;
        bool any = true;
        // a bonus row was not seen by the first pass: maximum and normaliser of this part alone (the last
        // workgroup puts the parts on one scale)
        if (bonus) any = part_max_and_norm<P, kSumSteps>(lg, c, s_m, s_z, lane, wv, m, Zd);
        if (!any) {
            for (int t = tid; t < kSumSteps * kQW * 8; t += kQT) publish_f32(my_sums + t, 0.f);
            if (tid == 0) publish_stat(my_stat, -INFINITY, -1, 1.0);
        } else {
            const float mc = m * c, invZ = (float)(1.0 / Zd);
#pragma unroll
            for (int it = 0; it < kSumSteps; ++it) {
                float rv[8], pv[8], acc_r = 0.f, acc_p = 0.f;
                keep_packed(lg[it]);
                keep_packed(qg[it]);
                part_chunk_masses<P>(lg[it], qg[it], c, mc, invZ, rv, pv);
#pragma unroll
                for (int e = 0; e < 8; ++e) { acc_r += rv[e]; acc_p += pv[e]; }
                acc_r = row16_sum(acc_r);
                acc_p = row16_sum(acc_p);
                if ((lane & 15) == 0) {
                    publish_f32(sums + sum_index(i, h, it, wv, 0) + (lane >> 4), acc_r);
                    publish_f32(sums + sum_index(i, h, it, wv, 1) + (lane >> 4), acc_p);
                }
            }
            if (tid == 0) publish_stat(my_stat, m, 0, Zd);
        }
    }

    // ---- ticket: the workgroup that finishes last for this request does the draw ----------------------
    ADASPEC_STAMP(1, 3);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");     // this wavefront's stores have been acknowledged
    __syncthreads();
    ADASPEC_STAMP(1, 4);
    if (tid == 0) s_last = __hip_atomic_fetch_add(req_ticket + i, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == n_parts - 1;
    __syncthreads();
    ADASPEC_STAMP(1, 5);
    if (!s_last) return;

    if (!sampled) {
        if (wv == 0) {
            ArgMax b{-INFINITY, V};
            if (lane < n_parts) {
                const HalfStat st = fetch_stat(sum_stat + i * kSumParts + lane);
                if (st.arg >= 0) b = ArgMax{st.m, st.arg};
            }
            b = wave_argmax(b);
            if (lane == 0) o[a] = b.i < V ? b.i : 0;
        }
        return;
    }
    // thread (part, step, wavefront): its residual and probability mass, all parts on one scale
    const int ph = tid >> 4, pit = (tid >> 2) & 3, pw = tid & 3;
    HalfStat st;
    st.m = -INFINITY; st.arg = -1; st.Z = 1.0;
    float4 pr = make_float4(0.f, 0.f, 0.f, 0.f), pp = pr;
    if (ph < n_parts) {
        st = fetch_stat(sum_stat + i * kSumParts + ph);
        const float *src = sums + sum_index(i, ph, pit, pw, 0);
        const unsigned long long r0 = fetch_u64(src), r1 = fetch_u64(src + 2), p0 = fetch_u64(src + 4), p1 = fetch_u64(src + 6);
        pr = make_float4(__uint_as_float((uint32_t)r0), __uint_as_float((uint32_t)(r0 >> 32)),
                         __uint_as_float((uint32_t)r1), __uint_as_float((uint32_t)(r1 >> 32)));
        pp = make_float4(__uint_as_float((uint32_t)p0), __uint_as_float((uint32_t)(p0 >> 32)),
                         __uint_as_float((uint32_t)p1), __uint_as_float((uint32_t)(p1 >> 32)));
    }
    if ((tid & 15) == 0) { s_m[ph] = st.m; s_z[ph] = st.Z; }
    __syncthreads();
    float M = s_m[0];
#pragma unroll
    for (int p = 1; p < kSumParts; ++p) M = fmaxf(M, s_m[p]);
    // p_v of part h was computed as 2^((l_v - m_h) c) / Z_h: times Z_h 2^((m_h - M) c) it is relative to M in
    // every part (a rejected draft row has the same (m, Z) in all parts: a common factor, which tau absorbs)
    const double my_sc = st.m > -INFINITY ? st.Z * (double)__builtin_amdgcn_exp2f((st.m - M) * c) : 0.0;
    const double res = (((double)pr.x + (double)pr.y) + ((double)pr.z + (double)pr.w)) * my_sc;
    const double pm = (((double)pp.x + (double)pp.y) + ((double)pp.z + (double)pp.w)) * my_sc;
    const int steps = ceil_div(row_chunks, kQT);             // steps of kQT chunks in the row (<= 64)
    bool use_p = bonus;                                       // (for a bonus row the two sums are the same numbers)
    for (int attempt = 0; attempt < 2; ++attempt) {
        mass[ph][pit][pw] = use_p ? pm : res;
        __syncthreads();
        if (wv == 0) {
            // lane L owns step L of the row: total over its wavefronts, running totals over the steps, R,
            // and the step whose running total first exceeds tau
            double t = 0.0;
            if (lane < steps) {
#pragma unroll
                for (int ww = 0; ww < kQW; ++ww) t = t + mass[lane >> 2][lane & 3][ww];
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
    ADASPEC_STAMP(1, 6);

    // ---- inside the step: the wavefront, then the lane, then the element (one wavefront works) -----
    const double tau = s_tau;
    const int sstep = s_step;
    const int hh = sstep >> 2, ii = sstep & 3;
    const double ws = lane < kQW ? mass[hh][ii][lane] : 0.0;
    const double wincl = s_before + wave_scan_incl(ws, lane);
    const unsigned long long whit = __ballot(lane < kQW && ws > 0.0 && wincl > tau);
    const unsigned long long wpos = __ballot(lane < kQW && ws > 0.0);
    if (!wpos) {                              // no mass anywhere (non-finite input): stay defined
        if (lane == 0) o[a] = 0;
        return;
    }
    const int wstar = whit ? (int)__builtin_ctzll(whit) : 63 - (int)__builtin_clzll(wpos);
    const double base = __shfl(wincl - ws, wstar, kWave);
    // statistics and scale of the part that holds the step
    HalfStat sth;
    sth.m = s_m[hh]; sth.arg = 0; sth.Z = s_z[hh];
    const double sch = sth.m > -INFINITY ? sth.Z * (double)__builtin_amdgcn_exp2f((sth.m - M) * c) : 0.0;
    const int chunk = hh * (kSumSteps * kQT) + ii * kQT + wstar * kWave + lane;   // this lane's 16 bytes of the row
    const bool with_q = has_q && !use_p;
    uint4 lv = make_uint4(P::kNegInf2, P::kNegInf2, P::kNegInf2, P::kNegInf2), qv = make_uint4(0, 0, 0, 0);
    if (chunk < row_chunks) {
        lv = *reinterpret_cast<const uint4 *>(lrow + (int64_t)chunk * 16);
        if (with_q) qv = *reinterpret_cast<const uint4 *>(prow + (int64_t)chunk * 16);
    }
    float rv[8], pv[8], sstar = 0.f;
    part_chunk_masses<P>(lv, qv, c, sth.m * c, (float)(1.0 / sth.Z), rv, pv);   // same expressions as the sums
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
        if (lane == 0) o[a] = 0;
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
        o[a] = chunk * 8 + pick;
    }
    ADASPEC_STAMP(1, 7);
}

static int parts_compute_units()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        cus = (hipGetDevice(&dev) == hipSuccess &&
               hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0) ? n : 256;
    }
    return cus;
}

bool accept_parts_supported(const adaspec_accept_dims &d)
{
    return d.batch <= kPartsMaxBatch && (int64_t)d.batch * d.max_spec_len <= kPartsMaxSlots &&
           d.vocab <= kStatParts * kStatSteps * kQT * 8;
}

size_t accept_parts_slot_bytes(const adaspec_accept_dims &d)
{
    if (!accept_parts_supported(d)) return 0;
    return (size_t)d.batch * (d.max_spec_len > 0 ? d.max_spec_len : 1) * sizeof(SlotRec);
}
size_t accept_parts_stat_bytes(const adaspec_accept_dims &d)
{
    if (!accept_parts_supported(d)) return 0;
    return (size_t)d.batch * (d.max_spec_len > 0 ? d.max_spec_len : 1) * kStatParts * sizeof(HalfStat);
}
size_t accept_parts_sum_bytes(const adaspec_accept_dims &d)
{
    if (!accept_parts_supported(d)) return 0;
    return (size_t)(d.batch > 0 ? d.batch : 1) * kSumParts * kSumSteps * kQW * 8 * sizeof(float);
}
size_t accept_parts_sum_stat_bytes(const adaspec_accept_dims &d)
{
    if (!accept_parts_supported(d)) return 0;
    return (size_t)(d.batch > 0 ? d.batch : 1) * kSumParts * sizeof(HalfStat);
}

hipError_t launch_accept_parts(const AcceptArgs &a)
{
    const adaspec_accept_dims &d = a.dims;
    if (d.batch == 0) return hipSuccess;
    const int row_chunks = d.vocab >> 3, row_steps = ceil_div(row_chunks, kQT);
    // First pass: a part is a stream of 8, 16, 32 or 64 steps.  Short streams spread a row over more compute
    // units; long ones read faster (measured on MI355X, config 3: 8 steps 48 us for the whole call, 16 steps
    // 44 us, 32 steps 42 us).  Aim: about three workgroups per compute unit, all resident at once.
    int stat_steps = kStatSteps;
    while (stat_steps < 64 && (int64_t)d.total_draft * ceil_div(row_steps, stat_steps) > (int64_t)kStatTargetWgsPerCu * parts_compute_units())
        stat_steps *= 2;
    const int n_stat_parts = ceil_div(row_steps, stat_steps);
    const int n_sum_parts = ceil_div(row_chunks, kSumSteps * kQT);
    auto launch = [&](auto tag) {
        using DT = decltype(tag);
        int32_t *cu_q = (int32_t *)(a.ws + a.plan.off_cu_q);
        int32_t *ticket = (int32_t *)(a.ws + a.plan.off_req_ticket);
        SlotRec *slot_rec = (SlotRec *)(a.ws + a.plan.off_slot_rec);
        HalfStat *part_stat = (HalfStat *)(a.ws + a.plan.off_part_stat);
        // (the first pass always runs, at least with one workgroup: it also clears the tickets)
        const int grid1 = d.total_draft > 0 ? d.total_draft * n_stat_parts : 1;
        hipLaunchKernelGGL((accept_rowparts_kernel<DT>), dim3(grid1), dim3(kQT), 0, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.draft_tokens, a.uniforms, a.spec_lens,
                           a.temperature, d.batch, d.vocab, d.total_q, d.total_draft, d.max_spec_len, n_stat_parts,
                           d.logits_row_stride, d.probs_row_stride, cu_q, ticket, slot_rec, part_stat);
        hipLaunchKernelGGL((accept_decide_kernel<DT>), dim3(d.batch * n_sum_parts), dim3(kQT), 0, a.stream,
                           (const char *)a.logits, (const char *)a.probs, a.draft_tokens, a.uniforms, a.spec_lens,
                           a.temperature, d.vocab, d.total_q, d.total_draft, d.max_spec_len, n_stat_parts, n_sum_parts,
                           d.logits_row_stride, d.probs_row_stride, cu_q, ticket, slot_rec, part_stat, d.out_stride,
                           a.out_tokens, a.out_accept_len, (float *)(a.ws + a.plan.off_part),
                           (HalfStat *)(a.ws + a.plan.off_half_stat));
    };
    if (d.logits_dtype == ADASPEC_F16) launch(F16{});
    else launch(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec

#ifdef ADASPEC_STAMPS
extern "C" int adaspec_debug_read_stamps(int which, long long *host, size_t groups)
{
    if (which < 0 || which > 1 || groups > (size_t)adaspec::kStampGroups) return -2;
    return hipMemcpyFromSymbol(host, HIP_SYMBOL(adaspec::g_stamps), groups * 8 * sizeof(long long),
                               (size_t)which * adaspec::kStampGroups * 8 * sizeof(long long), hipMemcpyDeviceToHost) == hipSuccess ? 0 : -7;
}
#endif
