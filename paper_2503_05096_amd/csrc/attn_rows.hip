// Matrix-core verification attention for units with MANY query rows (more than 32 rows share a kv
// head: long drafts times a wide GQA group), gfx950, 16-bit K/V/Q, head_dim 128.
//
// attn_mfma.hip lets the four wavefronts of a workgroup split a unit's TOKENS, every wavefront holding the
// softmax state of all rows.  Past two 16-row tiles that state (32 accumulator registers per tile) no
// longer fits beside the K/V registers: the three-tile form runs one wavefront per SIMD with a third of
// its instructions copying between register files.  Here the wavefronts split the ROWS instead:
//
//   * wavefront w owns row tile w (rows 16w .. 16w+15 of the unit's group of up to 64 rows) for ALL
//     tokens of the unit: 32 accumulator registers, no merge between wavefronts at the end;
//   * K and V of a 32-token block travel from memory straight into LDS (buffer loads with an LDS
//     destination: no registers, so two blocks ahead of the one being processed are in flight per
//     workgroup), shared by the four wavefronts: every byte is still fetched once per unit;
//   * S^T = K Q^T with A = K from LDS (a swizzle makes the 16-byte operand reads conflict free while
//     the loader still fetches whole 256-byte rows), B = Q^T held in registers for the whole unit;
//     softmax per row tile as in attn_mfma.hip (lazy reference, P stays in registers in B layout);
//     the V^T tile is built ONCE per block, each wavefront transposing a quarter of it, and read by
//     all four for O^T += V^T P^T.
// One LDS-only barrier per block: behind it a wavefront multiplies the PREVIOUS block's weights with its V^T
// tile and scores the current block (two independent matrix products), then builds the current V^T tile.
// 64.5 KB of LDS and ~130 registers: two workgroups per compute unit.
// Work units, schedule table and split-KV partials are those of attn_mfma.hip (row groups of 64 rows).
//
// Measured on MI355X, 64 requests x 8..48 rows per kv head, contexts 2048-8192: 280 us against 294 us for the
// three-tile token-split kernel it replaces (0.64 against 0.60 of the HBM peak); a batch whose requests all carry
// 24-36 rows gains 14 %.  What holds it back: with loads alone (no arithmetic) the ring sustains 5.7 TB/s, the
// arithmetic adds 12 %, and a unit with few rows leaves wavefronts 1-3 waiting at the barrier for wavefront 0.
#include "adaspec_internal.h"
#include "attn_mfma_common.h"
#include "device_utils.h"

namespace adaspec {

constexpr int kRowsPerGroup = 64;           // four row tiles, one per wavefront
constexpr int kAhead = 2;                   // blocks requested ahead of the one being processed
constexpr int kSlots = kAhead + 1;          // ring of raw K/V blocks in LDS
constexpr int kSlotBytes = 2 * kBlk * kD * 2;           // K (8 KB) then V (8 KB)
constexpr int kRowsSmem = kSlots * kSlotBytes + 2 * kVtBytes;   // + two V^T tiles (the one being read, the one being built)
constexpr int kLoadsPerBlock = 4;           // LDS-destination loads one wavefront issues per block (2 K + 2 V)

typedef int v4i32 __attribute__((ext_vector_type(4)));

// buffer descriptor of one (page, kv head) block of 4 KB (raw buffer: offsets in bytes, reads past the end give 0)
__device__ __forceinline__ v4i32 page_rsrc(const char *p)
{
    const unsigned long long a = reinterpret_cast<unsigned long long>(p);
    v4i32 r;
    r.x = (int)(uint32_t)a;
    r.y = (int)(uint32_t)(a >> 32);
    r.z = 16 * kD * 2;
    r.w = 0x00020000;
    return r;
}

// 16 bytes per lane from memory straight into LDS: lane i lands at lds_addr + 16 i (M0 carries the LDS address;
// the data never passes through registers).  Written in assembly on purpose: the compiler, not knowing which
// LDS bytes such a load will write, would make every later LDS read wait until ALL loads in flight have landed,
// and the point of the ring is that several blocks stay in flight.  The kernel waits for the block it needs itself
// (s_waitcnt vmcnt with the number of younger loads) before the barrier that publishes it.
// Two such loads behind one M0: the second lands 1024 bytes further in LDS; the instruction's offset field
// moves the memory address by the same 1024 bytes, which lane_offset1 has been reduced by.
__device__ __forceinline__ void load_pair_to_lds(const v4i32 &rsrc, uint32_t lane_offset0, uint32_t lane_offset1_minus_1024,
                                                 uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %3, 0 offen nt lds\n\t"
                 "buffer_load_dwordx4 %2, %3, 0 offen offset:1024 nt lds"
                 :: "s"(lds_addr), "v"(lane_offset0), "v"(lane_offset1_minus_1024), "s"(rsrc) : "memory", "m0");
}

template <class T, bool kTree>
__global__ __launch_bounds__(256, 2) void attn_rows_kernel(
    const char *__restrict__ q, const char *__restrict__ k_pages, const char *__restrict__ v_pages,
    const int32_t *__restrict__ block_table, void *__restrict__ out, const int32_t *__restrict__ header,
    const int32_t *__restrict__ unit_meta, const int32_t *__restrict__ sched,
    const unsigned long long *__restrict__ anc, float *__restrict__ part_ml, float *__restrict__ part_o,
    int Hq, int Hkv, int max_pages_per_req, int max_rows, int n_row_groups, float scale_log2, int out_dtype)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char *vt_tile = smem + kSlots * kSlotBytes;
    const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char *)smem;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, n16 = lane & 15;
    const int G = Hq / Hkv;
    const int total_units = header[0] * Hkv * n_row_groups;
    const int n_rounds = header[2];
    const int W = gridDim.x, wg = blockIdx.x;

    // ---- work units of this workgroup, in schedule order; two cursors walk them: the loader runs kAhead
    // blocks ahead of the arithmetic, across unit boundaries
    auto next_unit = [&](int &round, Unit &u) -> bool {
        for (; round < n_rounds; ++round) {
            const int idx = sched[(int64_t)round * W + wg];
            if (idx < 0 || idx >= total_units) continue;
            const int rg = idx % n_row_groups;
            u.gkv = (idx / n_row_groups) % Hkv;
            const int32_t *mt = unit_meta + 8 * (int64_t)(idx / (n_row_groups * Hkv));
            u.i = mt[0];
            const int sp = mt[1];
            u.ns = mt[2]; u.L = mt[3]; u.n = mt[4]; u.qrow0 = mt[5]; u.item = mt[6];
            u.rows = u.n * G; u.r0 = rg * kRowsPerGroup;
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

    // ---- loader: this wavefront's share of a block = LDS units [128 wv, 128 wv + 128) of K and of V --------
    // LDS unit p (16 bytes) of a raw block holds token p / 16; K keeps chunk (p % 16) ^ (token % 16) of that
    // token's 256-byte row there (XOR swizzle: operand reads below are conflict free), V keeps chunk p % 16.
    // A load instruction fills 64 consecutive units = four whole token rows; tokens 0..15 are the block's first
    // page, 16..31 its second.
    uint32_t k_voff[2], v_voff[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int tok = (4 * (2 * wv + j) + (lane >> 4)) & 15;          // token inside its page
        // (j = 1: tokens 4..7 of the wavefront's eight, tok >= 4; its instruction adds 1024 to the address itself)
        k_voff[j] = (uint32_t)(tok * 256 + ((n16 ^ tok) * 16) - 1024 * j);
        v_voff[j] = (uint32_t)(tok * 256 + n16 * 16 - 1024 * j);
    }
    // page ids of a block (scalar loads): requested one block before the block's own loads are issued, so
    // that their latency is not part of the loader's turn
    auto page_ids = [&](const Unit &u, int bi, int &p0, int &p1) {
        const int tb = u.t0 + bi * kBlk;
        p0 = block_table[u.bt_off + (tb >> 4)];
        // (a block's second page may lie past the split's end: the first is fetched again, masks blank it)
        p1 = (tb + 16 < u.t1) ? block_table[u.bt_off + (tb >> 4) + 1] : p0;
    };
    auto issue_block = [&](const Unit &u, int p0, int p1, int slot) {
        const int64_t base = ((int64_t)(wv >= 2 ? p1 : p0) * Hkv + u.gkv) * (int64_t)(16 * kD * 2);
        const v4i32 rk = page_rsrc(k_pages + base), rv = page_rsrc(v_pages + base);
        const uint32_t dst = lds_base + (uint32_t)(slot * kSlotBytes + (2 * wv) * 1024);
        load_pair_to_lds(rk, k_voff[0], k_voff[1], dst);
        load_pair_to_lds(rv, v_voff[0], v_voff[1], dst + kBlk * kD * 2);
    };

    // ---- operand addresses inside a raw block / the V^T tile -------------------------------------------
    // K as A operand of (mt, s): lane (g, m) <- token 16 mt + m, chunk 4 s + g
    uint32_t k_rd[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) k_rd[s] = (uint32_t)((n16 * 16 + ((4 * s + g) ^ n16)) * 16);
    // raw V for the transposition: lane (tq = g, c = n16) <- token 16 pg + 4 tq + ii, chunk c
    const uint32_t v_rd = (uint32_t)(kBlk * kD * 2 + g * 1024 + n16 * 16);
    char *vt_wr = vt_tile + 16 * (16 * g + n16);
    const char *vt_rd = vt_tile + 16 * (66 * (n16 & 7) + 16 * g + (n16 >> 3));

    Unit cu, pu;                               // consumer's unit, producer's unit
    int c_round = 0, p_round = 0;
    bool c_have = next_unit(c_round, cu);
    bool p_have = next_unit(p_round, pu);
    int p_blk = 0;                             // next block of pu to request
    int issued = 0, consumed = 0;              // stream positions (blocks over all units of this workgroup)
    int p_p0 = 0, p_p1 = 0;                    // page ids of that block
    if (p_have) page_ids(pu, 0, p_p0, p_p1);
    auto produce = [&]() {                     // request the next block of the stream, if there is one
        if (!p_have) return;
        issue_block(pu, p_p0, p_p1, issued % kSlots);
        ++issued;
        if (++p_blk == pu.nblk) { p_blk = 0; p_have = next_unit(p_round, pu); }
        if (p_have) page_ids(pu, p_blk, p_p0, p_p1);
    };
#pragma unroll 1
    for (int a = 0; a < kAhead; ++a) produce();

    while (c_have) {
        const Unit u = cu;
        // ---- this wavefront's row tile: Q^T operands (and ancestor masks) for the whole unit -------------
        const int row = u.r0 + 16 * wv + n16;
        const bool has_rows = u.r0 + 16 * wv < u.rows;              // wave-uniform
        uint4 qop[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) qop[s] = make_uint4(0, 0, 0, 0);
        unsigned long long am = 0ull;
        if (row < u.rows) {
            const char *qp = q + (((u.qrow0 + row / G) * Hq + u.gkv * G + row % G) * kD) * 2 + 16 * g;
#pragma unroll
            for (int s = 0; s < 4; ++s) qop[s] = ld16(qp + 64 * s);
            if constexpr (kTree) am = anc[u.qrow0 + row / G];
        }
        const int pos = row < u.rows ? (u.L - u.n + row / G) : -1;  // last token this row may see
        const int first_masked = u.L - u.n + 1;                     // tokens >= this are hidden from some row
        float m = kNegBig, lsum = 0.f;
        f32x4 o[8];
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
        // (the Q loads share the memory counter with the block loads in flight: rather than count them into
        // every wait below, the unit starts with everything landed; one memory latency per unit)
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        // (the compiler must see the loaded registers consumed HERE: it would otherwise put its own wait for
        // them at their first use inside the block loop, where it would also wait for every block in flight)
#pragma unroll
        for (int s = 0; s < 4; ++s) asm volatile("" : "+v"(qop[s].x), "+v"(qop[s].y), "+v"(qop[s].z), "+v"(qop[s].w));
        if constexpr (kTree) {
            uint32_t lo = (uint32_t)am, hi = (uint32_t)(am >> 32);
            asm volatile("" : "+v"(lo), "+v"(hi));
            am = ((unsigned long long)hi << 32) | lo;
        }

        // One barrier per block: behind it the wavefront multiplies the PREVIOUS block's weights with its V^T
        // tile, computes this block's scores and weights, and builds this block's V^T tile (the other of the two
        // tiles).  The two matrix products are independent, so one runs under the other's latencies.  A last
        // turn without a new block finishes the unit.
        uint4 pop = make_uint4(0, 0, 0, 0), pop_lo = make_uint4(0, 0, 0, 0);      // weights of the previous block
        for (int bi = 0; bi <= u.nblk; ++bi) {
            const bool fresh = bi < u.nblk;                             // a new block to score
            const int tb = u.t0 + bi * kBlk;
            const char *slot = smem + (consumed % kSlots) * kSlotBytes;
            if (fresh) {
                // ---- block `consumed` has landed (this wavefront's loads; the barrier covers the others') ---
                const int ahead = issued - consumed - 1;            // blocks requested after it
                if (ahead >= 2) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * kLoadsPerBlock) : "memory");
                else if (ahead == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoadsPerBlock) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
            // also: the previous block's V^T tile is complete, and everyone is done with the tile this turn
            // rebuilds and with the raw slot the next request overwrites
            lds_barrier();
            if (fresh) {
                produce();
                ++consumed;
            }

            // this block's K operands are requested first: they travel under the product below
            uint4 ka[2][4];
            if (has_rows && fresh) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int s = 0; s < 4; ++s) ka[mt][s] = *reinterpret_cast<const uint4 *>(slot + mt * 4096 + k_rd[s]);
            }
            // ---- O^T += V^T P^T of the previous block ----------------------------------------------------
            if (has_rows && bi > 0) {
                const char *vt_prev = vt_rd + ((bi - 1) & 1) * kVtBytes;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) {
                    const uint4 vt = *reinterpret_cast<const uint4 *>(vt_prev + 32 * dt);
                    o[dt] = Mma<T>::run(vt, pop, o[dt]);
                    if constexpr (Mma<T>::kSplitP) o[dt] = Mma<T>::run(vt, pop_lo, o[dt]);
                }
            }
            if (!fresh) break;

            if (has_rows) {
                // ---- S^T = K Q^T for this wavefront's 16 rows, 32 tokens ---------------------------------
                f32x4 sacc[2];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int s = 0; s < 4; ++s) acc = Mma<T>::run(ka[mt][s], qop[s], acc);
                    sacc[mt] = acc;
                }
                // ---- online softmax (per lane: row n16 of the tile, 8 of the 32 tokens) --------------------
                float sv[8];
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) sv[4 * mt + r] = sacc[mt][r];
                if ((tb + kBlk > first_masked) || (tb + kBlk > u.t1)) {
                    if constexpr (kTree) {
                        const int base = u.L - u.n;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int t = tb + 16 * (e >> 2) + 4 * g + (e & 3);
                            const int rel = t - base;
                            const bool vis = t < u.t1 && (rel < 0 ? pos >= 0 : ((am >> (rel & 63)) & 1ull) != 0);
                            sv[e] = vis ? sv[e] : -INFINITY;
                        }
                    } else {
                        const int lim = min(pos, u.t1 - 1);
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
                const float mxs = mx * scale_log2;
                const bool grow = mxs > m + kLazyLog2;               // lazy reference, as in attn_mfma.hip
                if (__builtin_expect(__builtin_amdgcn_ballot_w64(grow) != 0, 0)) {
                    const float m_new = grow ? mxs : m;
                    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
                    m = m_new;
                    lsum *= alpha;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) o[dt] *= alpha;
                }
                float p[8], psum = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    p[e] = __builtin_amdgcn_exp2f(fmaf(sv[e], scale_log2, -m));
                    psum += p[e];
                }
                lsum += psum;
                pop = make_uint4(Mma<T>::pack2(p[0], p[1]), Mma<T>::pack2(p[2], p[3]),
                                 Mma<T>::pack2(p[4], p[5]), Mma<T>::pack2(p[6], p[7]));
                if constexpr (Mma<T>::kSplitP) {
                    const uint32_t *hi = &pop.x;
                    uint32_t lo[4];
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        lo[w] = Mma<T>::pack2(p[2 * w] - __uint_as_float(hi[w] << 16),
                                              p[2 * w + 1] - __uint_as_float(hi[w] & 0xffff0000u));
                    pop_lo = make_uint4(lo[0], lo[1], lo[2], lo[3]);
                }
            }
            // ---- V^T tile, a quarter per wavefront: word wv of every raw chunk = channels 8c + 2wv, + 1 ----
            {
                uint32_t a[4], b[4];                                 // tokens 4 tq + ii of page 0 / page 1
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    a[ii] = *reinterpret_cast<const uint32_t *>(slot + v_rd + 4 * wv + ii * 256);
                    b[ii] = *reinterpret_cast<const uint32_t *>(slot + v_rd + 4 * wv + 4096 + ii * 256);
                }
                if (tb + kBlk > u.L) {                               // the request's last, partial block
#pragma unroll
                    for (int ii = 0; ii < 4; ++ii) {
                        if (tb + 4 * g + ii >= u.L) a[ii] = 0u;
                        if (tb + 16 + 4 * g + ii >= u.L) b[ii] = 0u;
                    }
                }
                const uint4 even = make_uint4(__builtin_amdgcn_perm(a[1], a[0], 0x05040100u),
                                              __builtin_amdgcn_perm(a[3], a[2], 0x05040100u),
                                              __builtin_amdgcn_perm(b[1], b[0], 0x05040100u),
                                              __builtin_amdgcn_perm(b[3], b[2], 0x05040100u));
                const uint4 odd = make_uint4(__builtin_amdgcn_perm(a[1], a[0], 0x07060302u),
                                             __builtin_amdgcn_perm(a[3], a[2], 0x07060302u),
                                             __builtin_amdgcn_perm(b[1], b[0], 0x07060302u),
                                             __builtin_amdgcn_perm(b[3], b[2], 0x07060302u));
                char *vt_cur = vt_wr + (bi & 1) * kVtBytes;
                *reinterpret_cast<uint4 *>(vt_cur + 66 * 16 * (2 * wv)) = even;
                *reinterpret_cast<uint4 *>(vt_cur + 66 * 16 * (2 * wv + 1)) = odd;
            }
        }

        // ---- the unit's rows are complete in their wavefronts: normalise and store, or leave the split's state
        if (has_rows) {
            lsum += __shfl_xor(lsum, 16, kWave);
            lsum += __shfl_xor(lsum, 32, kWave);
            if (row < u.rows) {
                // lane (g, n16) holds O^T[16 dt + 4 g .. + 3][row]: four consecutive channels per dt
                if (u.ns == 1) {
                    const float inv = 1.0f / lsum;
                    const int64_t obase = ((u.qrow0 + row / G) * Hq + u.gkv * G + row % G) * (int64_t)kD + 4 * g;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt) {
                        const f32x4 val = o[dt] * inv;
                        if (out_dtype == ADASPEC_F32) {
                            *reinterpret_cast<f32x4 *>(reinterpret_cast<float *>(out) + obase + 16 * dt) = val;
                        } else {
                            const uint2 pk = make_uint2(Mma<T>::pack2(val[0], val[1]), Mma<T>::pack2(val[2], val[3]));
                            *reinterpret_cast<uint2 *>(reinterpret_cast<uint16_t *>(out) + obase + 16 * dt) = pk;
                        }
                    }
                } else {
                    const int64_t idx_row = ((int64_t)u.item * Hkv + u.gkv) * max_rows + row;
#pragma unroll
                    for (int dt = 0; dt < 8; ++dt)
                        *reinterpret_cast<f32x4 *>(part_o + idx_row * kD + 16 * dt + 4 * g) = o[dt];
                    if (g == 0) {
                        part_ml[idx_row * 2] = m;
                        part_ml[idx_row * 2 + 1] = lsum;
                    }
                }
            }
        }
        c_have = next_unit(c_round, cu);
    }
    // (every block requested has been consumed: the loader stops with the last unit, so nothing is in flight)
}

// ---- host side -----------------------------------------------------------------------------------------------
template <typename T, bool kTree>
static int attn_rows_slots(int cus)
{
    static int slots = 0;
    if (slots == 0) {
        if (hipFuncSetAttribute((const void *)attn_rows_kernel<T, kTree>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                kRowsSmem) != hipSuccess)
            return 0;
        int per_cu = 1;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, attn_rows_kernel<T, kTree>, 256, kRowsSmem) != hipSuccess)
            per_cu = 1;
        const int n = cus * (per_cu > 0 ? per_cu : 1);
        slots = n < kMaxSchedW ? n : kMaxSchedW;
    }
    return slots;
}

template <typename F>
static void with_rows_instance(int dtype, bool tree, F &&f)
{
    auto with_tree = [&](auto tag) {
        if (tree) f(tag, std::true_type{});
        else f(tag, std::false_type{});
    };
    if (dtype == ADASPEC_F16) with_tree(F16{});
    else with_tree(BF16{});
}

int attn_rows_grid_slots(const AttnArgs &a, int cus)
{
    int slots = 0;
    with_rows_instance(a.dims.dtype, a.parents != nullptr, [&](auto tag, auto tree_tag) {
        slots = attn_rows_slots<decltype(tag), decltype(tree_tag)::value>(cus);
    });
    return slots;
}

hipError_t launch_attn_rows(const AttnArgs &a)
{
    const AttnPlan &p = a.plan;
    const adaspec_attn_dims &d = a.dims;
    if (a.sched_w <= 0) return hipSuccess;                          // no work item can exist
    with_rows_instance(d.dtype, a.parents != nullptr, [&](auto tag, auto tree_tag) {
        using T = decltype(tag);
        constexpr bool kTree = decltype(tree_tag)::value;
        hipLaunchKernelGGL((attn_rows_kernel<T, kTree>), dim3(a.sched_w), dim3(256), kRowsSmem, a.stream,
                           (const char *)a.q, (const char *)a.k_pages, (const char *)a.v_pages, a.block_table, a.out,
                           (const int32_t *)(a.ws + p.off_header), (const int32_t *)(a.ws + p.off_unit_meta),
                           (const int32_t *)(a.ws + p.off_sched), (const unsigned long long *)(a.ws + p.off_anc),
                           (float *)(a.ws + p.off_part_ml), (float *)(a.ws + p.off_part_o), d.n_q_heads, d.n_kv_heads,
                           d.max_pages_per_req, p.max_rows, a.n_row_groups, a.scale_log2, d.out_dtype);
    });
    return hipGetLastError();
}

}  // namespace adaspec
