// Matrix-core verification attention for gfx950: 16-bit K/V/Q, head_dim 128.
//
// Work unit = (work item = request x KV split, kv head, group of up to 16*RT
// query rows).  A workgroup of 4 wavefronts takes one unit; wavefront w streams
// the 32-token blocks w, w+4, ... of the split, keeping the online-softmax state
// of ALL rows of the unit (the n_i*G rows that share this kv head) in registers,
// so every K and V byte is fetched from HBM once per unit.  The four partial
// states are merged through LDS at the end.
//
// Everything is computed transposed so that no operand ever needs a shuffle:
//   S^T[token][row] = K[token][:] . Q[row][:]      A = K (straight from global), B = Q^T
//   O^T[d][row]    += V^T[d][token] P^T[token][row]  A = V^T (through LDS),       B = P^T
// With v_mfma_f32_16x16x32 the accumulator lane (g = lane/16, n = lane%16) holds
// S^T[4g..4g+3][n]; those 2x4 values per lane (two 16-token tiles) are exactly the
// 8 k-slots lane (g, n) must supply as B operand of the second product, so P never
// leaves the registers.  The k-slot order (g, e) <-> token 16*(e/4) + 4g + e%4 is
// then imposed on V^T: V rows are loaded coalesced (each lane: 4 tokens x 8
// channels per page), transposed 4x8 in registers with byte permutes and written
// to a wavefront-private 8 KB LDS tile laid out so that both the 16-byte writes
// and the 16-byte operand reads are bank-conflict free.
//
// kTree: the drafts of a request form a tree instead of a chain.  A row then sees the committed
// tokens and, of the request's new positions, those of its own ancestors: a 64-bit mask per query
// row (bit a = node a is the row's node or an ancestor of it), prepared once per verification pass.
// Only the blocks that hold new positions look at it; the instantiations for chains are untouched.
#include "adaspec_internal.h"
#include "attn_mfma_common.h"
#include "device_utils.h"

namespace adaspec {

template <class T, int RT, bool kTree>
__global__ __launch_bounds__(256, (RT <= 2 ? 2 : 1)) void attn_mfma_kernel(
    const char *__restrict__ q, const char *__restrict__ k_pages, const char *__restrict__ v_pages,
    const int32_t *__restrict__ block_table, void *__restrict__ out, int32_t *__restrict__ header,
    const int32_t *__restrict__ unit_meta, const int32_t *__restrict__ sched,
    const unsigned long long *__restrict__ anc, float *__restrict__ part_ml, float *__restrict__ part_o,
    int Hq, int Hkv, int max_pages_per_req, int max_rows, int n_row_groups, float scale_log2,
    int out_dtype)
{
    constexpr int kRows = 16 * RT;
    constexpr int kMerge = kRows * kORowStride * 4;                 // the [rows][d] fp32 merge buffer
    constexpr int kSmem = kWaves * kVtBytes > kMerge ? kWaves * kVtBytes : kMerge;
    __shared__ __attribute__((aligned(16))) char smem[kSmem];
    __shared__ __attribute__((aligned(16))) uint4 q_lds[RT * 4 * 64];   // Q^T operands, MFMA lane order
    __shared__ float s_m[kWaves][kRows], s_l[kWaves][kRows], s_mstar[kRows];
    __shared__ unsigned long long s_anc[kTree ? kRows : 1];         // ancestor mask of each row of the unit

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);        // wave-uniform by construction
    const int g = lane >> 4, n16 = lane & 15;
    const int G = Hq / Hkv;
    const int total_units = header[0] * Hkv * n_row_groups;
    const int64_t head_bytes = (int64_t)16 * kD * 2;                // one (page, head) block
    char *my_lds = smem + wv * kVtBytes;
    char *vt_wr = my_lds + 16 * (16 * g + n16);
    const char *vt_rd = my_lds + 16 * (66 * (n16 & 7) + 16 * g + (n16 >> 3));
    float *obuf = reinterpret_cast<float *>(smem);

    // K operand: lane (g, m) <- token 16 mt + m, channels 32 s + 8 g .. +7
    // V raw:     lane (tq = g, c = n16) <- token 16 pg + 4 tq + i, channels 8 c .. 8 c + 7
    uint4 kreg[2][4], vreg[2][4];
    const uint32_t k_lane_off = n16 * (kD * 2) + 16 * g;
    const uint32_t v_lane_off = (4 * g) * (kD * 2) + 16 * n16;

    // ---- work-unit bookkeeping ----------------------------------------------------------------
    // Units are listed longest first and handed out in rounds of W (one unit per workgroup and
    // round).  Which unit a workgroup takes in a round is a table the plan kernel wrote: it gives
    // the longest unit of the round to the workgroup with the least work so far.  No atomic is
    // needed and the next unit is known ahead of time, so its data can be requested early.
    const int W = gridDim.x, wg = blockIdx.x;
    const int n_rounds = header[2];
    int round = 0;
    int idx_ahead = wg;                                             // round 0 is the identity
    auto next_unit = [&](Unit &u) -> bool {
        for (; round < n_rounds; ++round) {
            const int idx = idx_ahead;
            // the entry of the following round is requested together with this unit's record, one
            // unit before it is needed
            idx_ahead = round + 1 < n_rounds ? sched[(int64_t)(round + 1) * W + wg] : -1;
            if (idx < 0 || idx >= total_units) continue;
            const int rg = idx % n_row_groups;
            u.gkv = (idx / n_row_groups) % Hkv;
            const int32_t *mt = unit_meta + 8 * (int64_t)(idx / (n_row_groups * Hkv));
            u.i = mt[0];
            const int sp = mt[1];
            u.ns = mt[2]; u.L = mt[3]; u.n = mt[4]; u.qrow0 = mt[5]; u.item = mt[6];
            u.rows = u.n * G; u.r0 = rg * kRows;
            if (u.r0 >= u.rows) continue;
            const int slen = split_len_of(u.L, u.ns, kBlk);
            u.t0 = sp * slen; u.t1 = min(u.L, u.t0 + slen);
            u.nblk = (u.t1 - u.t0 + kBlk - 1) / kBlk;
            u.bt_off = (int64_t)u.i * max_pages_per_req;
            ++round;
            return true;
        }
        return false;
    };

    // Page ids are wave-uniform (scalar loads: they never wait on the vector-memory counter).
    // Loads are issued unconditionally so that the counter waits stay exact: a block's second
    // page may lie past the split's end, then the first page is fetched again and the tail
    // code below blanks what must not be used.
    auto page_bases = [&](const Unit &u, int bi, int64_t &b0, int64_t &b1) {
        const int tb = u.t0 + bi * kBlk;
        const int64_t p0 = block_table[u.bt_off + (tb >> 4)];
        const int64_t p1 = (tb + 16 < u.t1) ? block_table[u.bt_off + (tb >> 4) + 1] : p0;
        b0 = (p0 * Hkv + u.gkv) * head_bytes;
        b1 = (p1 * Hkv + u.gkv) * head_bytes;
    };
    auto load_k = [&](int64_t b0, int64_t b1) {
        const char *kp0 = k_pages + b0 + k_lane_off, *kp1 = k_pages + b1 + k_lane_off;
#pragma unroll
        for (int s = 0; s < 4; ++s) kreg[0][s] = ld16_stream(kp0 + 64 * s);
#pragma unroll
        for (int s = 0; s < 4; ++s) kreg[1][s] = ld16_stream(kp1 + 64 * s);
    };
    auto load_v = [&](int64_t b0, int64_t b1) {
        const char *vp0 = v_pages + b0 + v_lane_off, *vp1 = v_pages + b1 + v_lane_off;
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) vreg[0][ii] = ld16_stream(vp0 + ii * (kD * 2));
#pragma unroll
        for (int ii = 0; ii < 4; ++ii) vreg[1][ii] = ld16_stream(vp1 + ii * (kD * 2));
    };
    // request the first block of this wavefront for unit u (if it has one)
    auto first_loads = [&](const Unit &u) {
        if (wv < u.nblk) {
            int64_t b0, b1;
            page_bases(u, wv, b0, b1);
            load_k(b0, b1);
            load_v(b0, b1);
        }
    };
    // this thread's share of the unit's Q^T operands: entry (nt = k, s = tid / 64, lane = tid % 64)
    auto load_q = [&](const Unit &u, uint4 (&qv)[RT]) {
#pragma unroll
        for (int k = 0; k < RT; ++k) {
            const int row = u.r0 + 16 * k + n16;
            qv[k] = make_uint4(0, 0, 0, 0);
            if (row < u.rows)
                qv[k] = ld16(q + (((u.qrow0 + row / G) * Hq + u.gkv * G + row % G) * kD) * 2 + 64 * wv + 16 * g);
        }
    };

    // tree: the ancestor mask of row tid of the unit (threads 0 .. kRows-1), requested with the Q rows
    auto load_anc = [&](const Unit &u) -> unsigned long long {
        const int row = u.r0 + tid;
        return (tid < kRows && row < u.rows) ? anc[u.qrow0 + row / G] : 0ull;
    };

    Unit cur, nxt;
    bool have = next_unit(cur);
    uint4 qv[RT];
    unsigned long long av = 0ull;
    if (have) {
        load_q(cur, qv);
        if constexpr (kTree) av = load_anc(cur);
        first_loads(cur);
    }

    while (have) {
        const Unit u = cur;
        const bool have_next = next_unit(nxt);
        const int first_masked = u.L - u.n + 1;                    // tokens >= this are hidden from some row
#pragma unroll
        for (int k = 0; k < RT; ++k) q_lds[tid + 256 * k] = qv[k];
        if constexpr (kTree) { if (tid < kRows) s_anc[tid] = av; }
        int pos[RT];
#pragma unroll
        for (int nt = 0; nt < RT; ++nt) {
            const int row = u.r0 + 16 * nt + n16;
            pos[nt] = row < u.rows ? (u.L - u.n + row / G) : -1;
        }
        __syncthreads();

        float m[RT], lsum[RT];
        f32x4 o[RT][8];
#pragma unroll
        for (int nt = 0; nt < RT; ++nt) {
            m[nt] = kNegBig; lsum[nt] = 0.f;
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) o[nt][dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }

        // One 32-token block; kNext: the following block's K and V are requested while this one
        // is being processed (K right after the first product, V right after the LDS hand-over).
        auto block = [&](int bi, auto next_tag) {
            constexpr bool kNext = decltype(next_tag)::value;
            const int tb = u.t0 + bi * kBlk;
            int64_t nb0 = 0, nb1 = 0;
            if constexpr (kNext) page_bases(u, bi + kWaves, nb0, nb1);

            // ---- S^T = K Q^T ------------------------------------------------------------
            f32x4 sacc[RT][2];
#pragma unroll
            for (int nt = 0; nt < RT; ++nt) {
                uint4 qop[4];
#pragma unroll
                for (int s = 0; s < 4; ++s) qop[s] = q_lds[(nt * 4 + s) * 64 + lane];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < 4; ++s) acc = Mma<T>::run(kreg[mt][s], qop[s], acc);
                    sacc[nt][mt] = acc;
                }
            }
            if constexpr (kNext) load_k(nb0, nb1);

            // ---- online softmax (per lane: row n16 of each row tile, 8 of the 32 tokens) ----
            const bool need_mask = (tb + kBlk > first_masked) || (tb + kBlk > u.t1);
            uint4 pop[RT], pop_lo[RT];
#pragma unroll
            for (int nt = 0; nt < RT; ++nt) {
                float sv[8];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) sv[4 * mt + r] = sacc[nt][mt][r];
                if (need_mask) {
                    if constexpr (kTree) {
                        // committed tokens are visible to every real row; new position base + a only
                        // if bit a of the row's mask is set (padding rows: pos < 0, mask 0)
                        const unsigned long long am = s_anc[16 * nt + n16];
                        const int base = u.L - u.n;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int t = tb + 16 * (e >> 2) + 4 * g + (e & 3);
                            const int rel = t - base;
                            const bool vis = t < u.t1 && (rel < 0 ? pos[nt] >= 0 : ((am >> (rel & 63)) & 1ull) != 0);
                            sv[e] = vis ? sv[e] : -INFINITY;
                        }
                    } else {
                        const int lim = min(pos[nt], u.t1 - 1);
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int t = tb + 16 * (e >> 2) + 4 * g + (e & 3);
                            sv[e] = (t <= lim) ? sv[e] : -INFINITY;
                        }
                    }
                }
                float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])),
                                 fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
                mx = max_over_row_groups(mx);
                // Lazy reference: the running reference m of a row moves only when the block's maximum exceeds it
                // by more than kLazyLog2 (weights then stay below 2^kLazyLog2, harmless in fp32 and in the
                // 16-bit operand formats), so the accumulators are rescaled in a handful of blocks per unit
                // instead of in almost every one, and the rescaling sits on a cold path.
                const float mxs = mx * scale_log2;
                const bool grow = mxs > m[nt] + kLazyLog2;
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0, 0)) {
                    const float m_new = grow ? mxs : m[nt];
                    const float alpha = __builtin_amdgcn_exp2f(m[nt] - m_new);
                    m[nt] = m_new;
                    lsum[nt] *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) o[nt][dt] *= alpha;
                }
                const float m_ref = m[nt];
                float p[8], psum = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = __builtin_amdgcn_exp2f(fmaf(sv[e], scale_log2, -m_ref));
                    psum += p[e];
                }
                lsum[nt] += psum;
                pop[nt] = make_uint4(Mma<T>::pack2(p[0], p[1]), Mma<T>::pack2(p[2], p[3]),
                                     Mma<T>::pack2(p[4], p[5]), Mma<T>::pack2(p[6], p[7]));
                if constexpr (Mma<T>::kSplitP) {
                    const uint32_t *hi = &pop[nt].x;
                    uint32_t lo[4];
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        lo[w] = Mma<T>::pack2(p[2 * w] - __uint_as_float(hi[w] << 16),
                                              p[2 * w + 1] - __uint_as_float(hi[w] & 0xffff0000u));
                    pop_lo[nt] = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                }
            }

            // ---- V^T tile: blank the tail, transpose 4x8 in registers, write to LDS --------
            if (tb + kBlk > u.L) {                     // the request's last, partial block
#pragma unroll
                for (int pg = 0; pg < 2; ++pg)
#pragma unroll
                    for (int ii = 0; ii < 4; ++ii)
                        if (tb + 16 * pg + 4 * g + ii >= u.L) vreg[pg][ii] = make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t a0 = (&vreg[0][0].x)[w], a1 = (&vreg[0][1].x)[w];
                const uint32_t a2 = (&vreg[0][2].x)[w], a3 = (&vreg[0][3].x)[w];
                const uint32_t b0 = (&vreg[1][0].x)[w], b1 = (&vreg[1][1].x)[w];
                const uint32_t b2 = (&vreg[1][2].x)[w], b3 = (&vreg[1][3].x)[w];
                uint4 even = make_uint4(__builtin_amdgcn_perm(a1, a0, 0x05040100u),
                                        __builtin_amdgcn_perm(a3, a2, 0x05040100u),
                                        __builtin_amdgcn_perm(b1, b0, 0x05040100u),
                                        __builtin_amdgcn_perm(b3, b2, 0x05040100u));
                uint4 odd = make_uint4(__builtin_amdgcn_perm(a1, a0, 0x07060302u),
                                       __builtin_amdgcn_perm(a3, a2, 0x07060302u),
                                       __builtin_amdgcn_perm(b1, b0, 0x07060302u),
                                       __builtin_amdgcn_perm(b3, b2, 0x07060302u));
                *reinterpret_cast<uint4 *>(vt_wr + 66 * 16 * (2 * w)) = even;
                *reinterpret_cast<uint4 *>(vt_wr + 66 * 16 * (2 * w + 1)) = odd;
            }
            if constexpr (kNext) load_v(nb0, nb1);

            // ---- O^T += V^T P^T -------------------------------------------------------------
            uint4 vt = *reinterpret_cast<const uint4 *>(vt_rd);
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) {
                uint4 vt_next = vt;
                if (dt < 7) vt_next = *reinterpret_cast<const uint4 *>(vt_rd + 32 * (dt + 1));
#pragma unroll
                for (int nt = 0; nt < RT; ++nt) {
                    o[nt][dt] = Mma<T>::run(vt, pop[nt], o[nt][dt]);
                    if constexpr (Mma<T>::kSplitP) o[nt][dt] = Mma<T>::run(vt, pop_lo[nt], o[nt][dt]);
                }
                vt = vt_next;
            }
        };

        if (wv < u.nblk) {
            int bi = wv;
            for (; bi + kWaves < u.nblk; bi += kWaves) block(bi, std::true_type{});
            block(bi, std::false_type{});
        }

        // ---- next unit: request its first K/V block and its Q rows now, so that they travel while
        // this unit's states are merged and written out.
#pragma unroll
        for (int nt = 0; nt < RT; ++nt) {
            lsum[nt] += __shfl_xor(lsum[nt], 16, kWave);
            lsum[nt] += __shfl_xor(lsum[nt], 32, kWave);
            if (g == 0) s_m[wv][16 * nt + n16] = m[nt];
        }
        if (have_next) {
            load_q(nxt, qv);
            if constexpr (kTree) av = load_anc(nxt);
            first_loads(nxt);
        }
        __syncthreads();            // s_m complete; every wavefront is done with its V^T tile and q_lds

        // ---- merge the four wavefronts' states through LDS --------------------------------
        // m* = max over wavefronts, each state rescaled by 2^(m - m*); the O tiles are summed
        // into one [rows][d] fp32 buffer (aliasing the V^T tiles) one wavefront after another.
        float fsc[RT];
#pragma unroll
        for (int nt = 0; nt < RT; ++nt) {
            const int rl = 16 * nt + n16;
            float ms = s_m[0][rl];
#pragma unroll
            for (int w = 1; w < kWaves; ++w) ms = fmaxf(ms, s_m[w][rl]);
            fsc[nt] = __builtin_amdgcn_exp2f(m[nt] - ms);
            if (g == 0) {
                s_l[wv][rl] = lsum[nt] * fsc[nt];
                if (wv == 0) s_mstar[rl] = ms;
            }
        }
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            if (wv == w) {
#pragma unroll
                for (int nt = 0; nt < RT; ++nt)
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) {
                        f32x4 *dst = reinterpret_cast<f32x4 *>(obuf + (16 * nt + n16) * kORowStride +
                                                               16 * dt + 4 * g);
                        f32x4 v = o[nt][dt] * fsc[nt];
                        if (w > 0) v += *dst;
                        *dst = v;
                    }
            }
            __syncthreads();
        }
        // 256 threads: 16*RT rows x 32 float4 columns
#pragma unroll
        for (int it = 0; it < 2 * RT; ++it) {
            const int idx = tid + 256 * it;
            const int rl = idx >> 5, c4 = idx & 31;
            const int row = u.r0 + rl;
            if (row >= u.rows) continue;
            const f32x4 acc = *reinterpret_cast<const f32x4 *>(obuf + rl * kORowStride + 4 * c4);
            const float ltot = (s_l[0][rl] + s_l[1][rl]) + (s_l[2][rl] + s_l[3][rl]);
            if (u.ns == 1) {
                const float inv = 1.0f / ltot;
                const int64_t obase = ((u.qrow0 + row / G) * Hq + u.gkv * G + row % G) * (int64_t)kD + 4 * c4;
                if (out_dtype == ADASPEC_F32) {
                    *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(out) + obase) = acc * inv;
                } else {
                    uint2 pk = make_uint2(Mma<T>::pack2(acc[0] * inv, acc[1] * inv),
                                          Mma<T>::pack2(acc[2] * inv, acc[3] * inv));
                    *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + obase) = pk;
                }
            } else {
                const int64_t idx_row = ((int64_t)u.item * Hkv + u.gkv) * max_rows + row;
                *reinterpret_cast<f32x4 *>(part_o + idx_row * kD + 4 * c4) = acc;
                if (c4 == 0) {
                    part_ml[idx_row * 2] = s_mstar[rl];
                    part_ml[idx_row * 2 + 1] = ltot;
                }
            }
        }
        // the next loop iteration overwrites q_lds and the V^T tiles: everyone must be done reading obuf
        __syncthreads();
        cur = nxt;
        have = have_next;
    }
}

bool attn_fast_path_supported(const adaspec_attn_dims &d)
{
    return d.head_dim == kD && (d.dtype == ADASPEC_F16 || d.dtype == ADASPEC_BF16) && d.page_size == 16;
}

// Resident workgroups of attn_mfma_kernel<T, RT> on the current device: the schedule balances
// over exactly these.  Queried once per instantiation.
static int device_cus()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 256;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1)
            n = 256;
        cus = n;
    }
    return cus;
}

template <typename T, int RT, bool kTree>
static int attn_mfma_slots()
{
    static int slots = 0;
    if (slots == 0) {
        int per_cu = 1;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, attn_mfma_kernel<T, RT, kTree>, 256, 0) != hipSuccess)
            per_cu = 1;
        const int n = device_cus() * (per_cu > 0 ? per_cu : 1);
        slots = n < kMaxSchedW ? n : kMaxSchedW;
    }
    return slots;
}

template <typename F>
static void with_instance(int dtype, int rt, bool tree, F &&f)
{
    auto with_rt = [&](auto tag, auto tree_tag) {
        if (rt == 1) f(tag, std::integral_constant<int, 1>{}, tree_tag);
        else f(tag, std::integral_constant<int, 2>{}, tree_tag);
    };
    auto with_tree = [&](auto tag) {
        if (tree) with_rt(tag, std::true_type{});
        else with_rt(tag, std::false_type{});
    };
    if (dtype == ADASPEC_F16) with_tree(F16{});
    else with_tree(BF16{});
}

void attn_mfma_shape(AttnArgs &a)
{
    const AttnPlan &p = a.plan;
    const int rt = attn_row_tiles(p.max_rows);
    a.n_row_groups = attn_row_groups(p.max_rows);
    a.rows_per_group = 16 * rt;
    const int64_t max_units = (int64_t)p.max_items * a.dims.n_kv_heads * a.n_row_groups;
    int slots = 1;
    if (rt > 2) {
        slots = attn_rows_grid_slots(a, device_cus());               // more than 32 rows: the row-split kernel
        if (slots <= 0) slots = device_cus();
    } else {
        with_instance(a.dims.dtype, rt, a.parents != nullptr, [&](auto tag, auto rt_tag, auto tree_tag) {
            slots = attn_mfma_slots<decltype(tag), decltype(rt_tag)::value, decltype(tree_tag)::value>();
        });
    }
    a.sched_w = (int)(max_units < slots ? max_units : slots);
    a.sched_cus = device_cus();
}

hipError_t launch_attn_mfma(const AttnArgs &a)
{
    const AttnPlan &p = a.plan;
    const adaspec_attn_dims &d = a.dims;
    if (a.sched_w <= 0) return hipSuccess;                          // no work item can exist
    if (attn_row_tiles(p.max_rows) > 2) return launch_attn_rows(a);
    with_instance(d.dtype, attn_row_tiles(p.max_rows), a.parents != nullptr, [&](auto tag, auto rt_tag, auto tree_tag) {
        using T = decltype(tag);
        constexpr int RT = decltype(rt_tag)::value;
        constexpr bool kTree = decltype(tree_tag)::value;
        hipLaunchKernelGGL((attn_mfma_kernel<T, RT, kTree>), dim3(a.sched_w), dim3(256), 0, a.stream,
                           (const char *)a.q, (const char *)a.k_pages, (const char *)a.v_pages,
                           a.block_table, a.out, (int32_t *)(a.ws + p.off_header),
                           (const int32_t *)(a.ws + p.off_unit_meta), (const int32_t *)(a.ws + p.off_sched),
                           (const unsigned long long *)(a.ws + p.off_anc), (float *)(a.ws + p.off_part_ml), (float *)(a.ws + p.off_part_o), d.n_q_heads,
                           d.n_kv_heads, d.max_pages_per_req, p.max_rows, a.n_row_groups, a.scale_log2,
                           d.out_dtype);
    });
    return hipGetLastError();
}

}  // namespace adaspec
