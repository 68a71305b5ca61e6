// Draft-side sampling with every row cut into four parts (16-bit draft logits, V % 8 == 0,
// V <= 131072).  What the step computes is stated in draft_sample.hip.
//
// One row of V = 128 K elements keeps a compute unit busy for about 30 us (two sweeps of exponentials
// and the store of the probability row), and a draft step has one row per request: with fewer rows
// than compute units the single-workgroup kernels leave most of the chip idle for that long.  Here
// four workgroups share a row, at the price of three kernels:
//   draft_part_stats   (row, part): maximum, arg-max (lowest index) and sum 2^((l - m) c) of the part
//   draft_part_probs   (row, part): the row's (m, Z) from the four parts, q_v = 2^(l_v c - m c) / Z rounded
//                      once and stored, the rounded mass per (step, wavefront, row of 16 lanes)
//   draft_pick         one workgroup per row: the (part, step, wavefront) holding tau = u * sum(q) from
//                      those sums, that wavefront's 64 chunks recomputed (same expression, same bits as
//                      the stored row), the lane, the element; greedy rows: the arg-max of the parts
// The second kernel re-reads the logits (they come from the caches: the first one has just read them).
#include "adaspec_internal.h"
#include "device_utils.h"
#include "row_registers.h"
#include "draft_common.h"

namespace adaspec {

constexpr int kDT = 1024;                // threads per (row, part)
constexpr int kDW = kDT / kWave;
constexpr int kDParts = 4;
constexpr int kDRowSteps = 16;           // steps of 8192 elements in the longest row
constexpr int kDPSteps = kDRowSteps / kDParts;
constexpr int kDPickT = kDRowSteps * kDW;

struct DraftPartStat { float m; int arg; double z; };   // 16 bytes

// workspace: DraftPartStat[R][4], then float[R][4 parts][4 steps][16 wavefronts][4 rows of 16 lanes]
static size_t draft_split_stats_bytes(int rows) { return align_up((size_t)rows * kDParts * sizeof(DraftPartStat), 256); }
size_t draft_split_workspace_bytes(int rows)
{
    return draft_split_stats_bytes(rows) + (size_t)rows * kDRowSteps * kDW * 4 * sizeof(float);
}

struct DraftPartGeometry { int part_steps, chunk0, nchunks; };
__device__ __forceinline__ DraftPartGeometry draft_part_geometry(int V, int h)
{
    DraftPartGeometry g;
    const int row_chunks = V >> 3, steps = ceil_div(row_chunks, kDT);
    g.part_steps = ceil_div(steps, kDParts);
    g.chunk0 = h * g.part_steps * kDT;
    g.nchunks = min(max(row_chunks - g.chunk0, 0), g.part_steps * kDT);
    return g;
}

__device__ __forceinline__ size_t draft_mass_index(int r, int h, int it, int w)
{
    return ((((size_t)r * kDParts + h) * kDPSteps + it) * kDW + w) * 4;
}

// the part's chunks into registers; chunks past its end count as -inf
template <class P>
__device__ __forceinline__ void load_part(const char *lrow, const DraftPartGeometry &g, int tid, uint4 (&lg)[kDPSteps])
{
    const __amdgpu_buffer_rsrc_t rl =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<char *>(lrow + (int64_t)g.chunk0 * 16), 0, g.nchunks * 16, 0x00020000);
#pragma unroll
    for (int it = 0; it < kDPSteps; ++it) {
        const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rl, tid * 16, it * (kDT * 16), 0);
        lg[it] = make_uint4(v.x, v.y, v.z, v.w);
    }
#pragma unroll
    for (int it = 0; it < kDPSteps; ++it) {
        const uint32_t ninf = (it * kDT + tid >= g.nchunks) ? P::kNegInf2 : 0u;
        lg[it].x |= ninf; lg[it].y |= ninf; lg[it].z |= ninf; lg[it].w |= ninf;
    }
}

template <class DT>
__global__ __launch_bounds__(kDT, 8) void draft_part_stats_kernel(
    const char *__restrict__ logits, const float *__restrict__ temperature, int V, int64_t lstride_bytes,
    DraftPartStat *__restrict__ stats)
{
    using P = Pair16<DT>;
    __shared__ float s_v[kDW], s_z[kDW];
    __shared__ int s_i[kDW];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x / kDParts, h = blockIdx.x % kDParts;
    const float T = temperature[r];
    const float c2 = T == 0.0f ? 1.4426950408889634f : 1.4426950408889634f / T;
    const DraftPartGeometry g = draft_part_geometry(V, h);
    DraftPartStat *my = stats + (size_t)r * kDParts + h;
    if (g.nchunks == 0) {
        if (tid == 0) { DraftPartStat st; st.m = -INFINITY; st.arg = -1; st.z = 0.0; *my = st; }
        return;
    }
    uint4 lg[kDPSteps];
    load_part<P>(logits + (int64_t)r * lstride_bytes, g, tid, lg);
    // maximum with the lowest index on ties (a thread visits its elements in index order)
    ArgMax best{-INFINITY, V};
#pragma unroll
    for (int it = 0; it < kDPSteps; ++it) {
        const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
        const int base = (g.chunk0 + it * kDT + tid) * 8;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float a = P::lo(w[e]), b = P::hi(w[e]);
            if (a > best.v) best = ArgMax{a, base + 2 * e};
            if (b > best.v) best = ArgMax{b, base + 2 * e + 1};
        }
    }
    best = wave_argmax(best);
    if (lane == 0) { s_v[wv] = best.v; s_i[wv] = best.i; }
    lds_barrier();
    ArgMax top{s_v[0], s_i[0]};
#pragma unroll
    for (int w = 1; w < kDW; ++w) top = argmax_merge(top, ArgMax{s_v[w], s_i[w]});
    if (!(top.v > -INFINITY)) {               // no finite logit in this part
        if (tid == 0) { DraftPartStat st; st.m = -INFINITY; st.arg = -1; st.z = 0.0; *my = st; }
        return;
    }
    const float mc = top.v * c2;
    float z = 0.f;
#pragma unroll
    for (int it = 0; it < kDPSteps; ++it) {
        keep_packed(lg[it]);
        const uint32_t w[4] = {lg[it].x, lg[it].y, lg[it].z, lg[it].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            z += __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c2, -mc));
            z += __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c2, -mc));
        }
    }
    z = wave_sum(z);
    if (lane == 0) s_z[wv] = z;
    lds_barrier();
    if (tid == 0) {
        double zd = 0.0;
        for (int w = 0; w < kDW; ++w) zd += (double)s_z[w];
        DraftPartStat st; st.m = top.v; st.arg = top.i; st.z = zd; *my = st;
    }
}

// (m, Z) of the whole row from its parts; returns the arg-max (lowest index: the parts are in index order)
__device__ __forceinline__ int merge_parts(const DraftPartStat *st, float c2, float &m, double &Z)
{
    m = -INFINITY;
    int arg = -1;
#pragma unroll
    for (int p = 0; p < kDParts; ++p)
        if (st[p].arg >= 0 && st[p].m > m) { m = st[p].m; arg = st[p].arg; }
    Z = 0.0;
#pragma unroll
    for (int p = 0; p < kDParts; ++p)
        if (st[p].arg >= 0) Z += st[p].z * (double)__builtin_amdgcn_exp2f((st[p].m - m) * c2);
    return arg;
}

template <class DT, class PT>
__global__ __launch_bounds__(kDT, 8) void draft_part_probs_kernel(
    const char *__restrict__ logits, const float *__restrict__ temperature, const int32_t *__restrict__ out_rows,
    char *__restrict__ probs, int V, int64_t lstride_bytes, int64_t pstride_bytes,
    const DraftPartStat *__restrict__ stats, float *__restrict__ mass)
{
    using P = Pair16<DT>;
    constexpr int kPsz = std::is_same<PT, F32>::value ? 4 : 2;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x / kDParts, h = blockIdx.x % kDParts;
    const float T = temperature[r];
    const float c2 = T == 0.0f ? 1.4426950408889634f : 1.4426950408889634f / T;
    const DraftPartGeometry g = draft_part_geometry(V, h);
    DraftPartStat st[kDParts];
#pragma unroll
    for (int p = 0; p < kDParts; ++p) st[p] = stats[(size_t)r * kDParts + p];   // scalar loads
    if (g.nchunks == 0) {
        for (int t = tid; t < kDPSteps * kDW * 4; t += kDT) mass[draft_mass_index(r, h, 0, 0) + t] = 0.f;
        return;
    }
    uint4 lg[kDPSteps];
    load_part<P>(logits + (int64_t)r * lstride_bytes, g, tid, lg);
    float m;
    double Zd;
    merge_parts(st, c2, m, Zd);
    const float mc = m * c2, invZ = (float)(1.0 / Zd);     // (a row without any finite logit: q = NaN, as in the other kernels)
    char *prow = probs + (int64_t)(out_rows ? out_rows[r] : r) * pstride_bytes + (int64_t)g.chunk0 * 8 * kPsz;
    const __amdgpu_buffer_rsrc_t rp = __builtin_amdgcn_make_buffer_rsrc(prow, 0, g.nchunks * 8 * kPsz, 0x00020000);
#pragma unroll
    for (int it = 0; it < kDPSteps; ++it) {
        keep_packed(lg[it]);
        float q[8];
        uint4 packed;
        chunk_probs<DT, PT>(lg[it], c2, mc, invZ, q, packed);
        // (the step's offset in the lane offset, scalar offset 0: see the store in draft_fast.hip)
        if constexpr (kPsz == 2) {
            __builtin_amdgcn_raw_buffer_store_b128(u32x4{packed.x, packed.y, packed.z, packed.w}, rp,
                                                   tid * 16 + it * (kDT * 16), 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(
                u32x4{__float_as_uint(q[0]), __float_as_uint(q[1]), __float_as_uint(q[2]), __float_as_uint(q[3])}, rp,
                tid * 32 + it * (kDT * 32), 0, 0);
            __builtin_amdgcn_raw_buffer_store_b128(
                u32x4{__float_as_uint(q[4]), __float_as_uint(q[5]), __float_as_uint(q[6]), __float_as_uint(q[7])}, rp,
                tid * 32 + 16 + it * (kDT * 32), 0, 0);
        }
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc += q[e];
        acc = row16_sum(acc);
        if ((lane & 15) == 0) mass[draft_mass_index(r, h, it, wv) + (lane >> 4)] = acc;
    }
}

template <class DT, class PT>
__global__ __launch_bounds__(kDPickT) void draft_pick_kernel(
    const char *__restrict__ logits, const float *__restrict__ temperature, const float *__restrict__ uniforms,
    int32_t *__restrict__ tokens, float *__restrict__ confidence, int V, int64_t lstride_bytes,
    const DraftPartStat *__restrict__ stats, const float *__restrict__ mass)
{
    using P = Pair16<DT>;
    __shared__ double sm[kDParts][kDPSteps][kDW];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int r = blockIdx.x;
    const float T = temperature[r], u = uniforms[r];
    const float c2 = T == 0.0f ? 1.4426950408889634f : 1.4426950408889634f / T;
    DraftPartStat st[kDParts];
#pragma unroll
    for (int p = 0; p < kDParts; ++p) st[p] = stats[(size_t)r * kDParts + p];
    float m;
    double Zd;
    const int amax = merge_parts(st, c2, m, Zd);
    const float mc = m * c2, invZ = (float)(1.0 / Zd);
    if (T == 0.0f) {
        if (tid == 0) {
            // the arg-max and its probability, with the expression and the rounding of the stored row
            uint4 one = make_uint4(0, 0, 0, 0);
            uint16_t bits;
            if constexpr (std::is_same<DT, BF16>::value) bits = float_to_bf16_bits(m); else bits = float_to_f16_bits(m);
            one.x = bits;                      // the maximum is a stored logit: converting it back is exact
            float q[8];
            uint4 packed;
            chunk_probs<DT, PT>(one, c2, mc, invZ, q, packed);
            tokens[r] = amax >= 0 ? amax : 0;
            confidence[r] = amax >= 0 ? q[0] : 0.f;
        }
        return;
    }
    const int h = tid / (kDPSteps * kDW), it = (tid / kDW) % kDPSteps, w = tid % kDW;
    const float4 v = *reinterpret_cast<const float4 *>(mass + draft_mass_index(r, h, it, w));
    sm[h][it][w] = ((double)v.x + (double)v.y) + ((double)v.z + (double)v.w);
    __syncthreads();
    const int steps = ceil_div(V >> 3, kDT), part_steps = draft_part_geometry(V, 0).part_steps;
    if (wv != 0) return;
    // One wavefront from here on.  Lane L owns step L of the row: its total, running totals over the
    // steps, Q, and the step holding tau (all of them the same in every lane).
    double tau, before;
    int sstep;
    {
        const int hl = lane / part_steps, il = lane % part_steps;
        double t = 0.0;
        if (lane < steps) {
#pragma unroll
            for (int ww = 0; ww < kDW; ++ww) t = t + sm[hl][il][ww];
        }
        const double incl = wave_scan_incl(t, lane);
        const double Q = __shfl(incl, steps - 1, kWave);
        tau = (double)u * Q;
        const unsigned long long hits = __ballot(lane < steps && incl > tau);
        sstep = hits ? (int)__builtin_ctzll(hits) : steps - 1;
        before = __shfl(incl - t, sstep, kWave);
    }
    const int hh = sstep / part_steps, ii = sstep % part_steps;
    const double ws = lane < kDW ? sm[hh][ii][lane] : 0.0;
    const double wincl = before + wave_scan_incl(ws, lane);
    const unsigned long long whit = __ballot(lane < kDW && ws > 0.0 && wincl > tau);
    const unsigned long long wpos = __ballot(lane < kDW && ws > 0.0);
    if (!wpos) {                              // no mass (non-finite input): stay defined
        if (lane == 0) { tokens[r] = 0; confidence[r] = 0.f; }
        return;
    }
    const int wstar = whit ? (int)__builtin_ctzll(whit) : 63 - (int)__builtin_clzll(wpos);
    const double base = __shfl(wincl - ws, wstar, kWave);
    const int chunk = hh * part_steps * kDT + ii * kDT + wstar * kWave + lane;
    uint4 lv = make_uint4(P::kNegInf2, P::kNegInf2, P::kNegInf2, P::kNegInf2);
    if (chunk < (V >> 3)) lv = *reinterpret_cast<const uint4 *>(logits + (int64_t)r * lstride_bytes + (int64_t)chunk * 16);
    float qv[8], mine = 0.f;
    uint4 packed;
    chunk_probs<DT, PT>(lv, c2, mc, invZ, qv, packed);     // same expression, same rounding as the stored row
#pragma unroll
    for (int e = 0; e < 8; ++e) mine += qv[e];
    const double li = base + wave_scan_incl((double)mine, lane);
    const unsigned long long lhit = __ballot(mine > 0.f && li > tau);
    const unsigned long long lpos = __ballot(mine > 0.f);
    if (!lpos) {
        if (lane == 0) { tokens[r] = 0; confidence[r] = 0.f; }
        return;
    }
    const int owner = lhit ? (int)__builtin_ctzll(lhit) : 63 - (int)__builtin_clzll(lpos);
    if (lane == owner) {
        double cum = li - (double)mine;
        int pick = -1, lastpos = -1;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            cum += (double)qv[e];
            if (qv[e] > 0.f) lastpos = e;
            if (pick < 0 && qv[e] > 0.f && cum > tau) pick = e;
        }
        if (pick < 0) pick = lastpos < 0 ? 0 : lastpos;
        tokens[r] = chunk * 8 + pick;
        confidence[r] = qv[pick];
    }
}

bool draft_split_supported(const adaspec_draft_dims &d)
{
    if (d.logits_dtype == ADASPEC_F32) return false;
    return d.vocab % 8 == 0 && d.vocab <= kDT * 8 * kDRowSteps;
}

hipError_t launch_draft_split(const void *logits, const float *temperature, const float *uniforms,
                              const int32_t *out_rows, void *probs, int32_t *tokens, float *confidence,
                              const adaspec_draft_dims &d, char *ws, hipStream_t stream)
{
    if (d.rows == 0) return hipSuccess;
    const int psz = d.probs_dtype == ADASPEC_F32 ? 4 : 2;
    DraftPartStat *stats = reinterpret_cast<DraftPartStat *>(ws);
    float *mass = reinterpret_cast<float *>(ws + draft_split_stats_bytes(d.rows));
    auto launch = [&](auto lt, auto pt) {
        using DT = decltype(lt);
        using PT = decltype(pt);
        hipLaunchKernelGGL((draft_part_stats_kernel<DT>), dim3(d.rows * kDParts), dim3(kDT), 0, stream,
                           (const char *)logits, temperature, d.vocab, d.logits_row_stride * 2, stats);
        hipLaunchKernelGGL((draft_part_probs_kernel<DT, PT>), dim3(d.rows * kDParts), dim3(kDT), 0, stream,
                           (const char *)logits, temperature, out_rows, (char *)probs, d.vocab, d.logits_row_stride * 2,
                           d.probs_row_stride * psz, stats, mass);
        hipLaunchKernelGGL((draft_pick_kernel<DT, PT>), dim3(d.rows), dim3(kDPickT), 0, stream,
                           (const char *)logits, temperature, uniforms, tokens, confidence, d.vocab,
                           d.logits_row_stride * 2, stats, mass);
    };
    auto with_p = [&](auto lt) {
        if (d.probs_dtype == ADASPEC_F32) launch(lt, F32{});
        else if (d.probs_dtype == ADASPEC_F16) launch(lt, F16{});
        else launch(lt, BF16{});
    };
    if (d.logits_dtype == ADASPEC_F16) with_p(F16{});
    else with_p(BF16{});
    return hipGetLastError();
}

}  // namespace adaspec
