// Pieces shared by the two matrix-core attention kernels (attn_mfma.hip: the wavefronts of a workgroup
// split a unit's TOKENS; attn_rows.hip: they split its query ROWS): MFMA wrappers, the V^T tile layout,
// the work-unit record.
#pragma once
#include "adaspec_internal.h"
#include "device_utils.h"

namespace adaspec {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kD = 128;                 // head_dim
constexpr int kBlk = 32;                // tokens per block (two pages)
constexpr int kWaves = 4;
constexpr int kORowStride = 132;        // floats per row of the merge buffer (padded: conflict-free b128)
constexpr float kNegBig = -1.0e30f;     // "no token seen yet": finite, so differences never give NaN
constexpr float kLazyLog2 = 8.0f;       // a row's softmax reference trails its running maximum by at most this (log2 units)

template <class T> struct Mma;
template <> struct Mma<BF16> {
    // bf16 keeps 8 significant bits: a softmax weight rounded to it is off by up to 2^-9 relative,
    // which with a handful of dominant tokens reaches the 2e-3 output tolerance.  The weights are
    // therefore fed to the matrix core as hi + lo (two bf16 values, 16 significant bits).
    static constexpr bool kSplitP = true;
    static __device__ __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                       __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        f32x2 x = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, bf16x2));   // v_cvt_pk_bf16_f32, RNE
    }
};
template <> struct Mma<F16> {
    static constexpr bool kSplitP = false;       // fp16 keeps 11 bits: 2^-12 relative is enough
    static __device__ __forceinline__ f32x4 run(uint4 a, uint4 b, f32x4 c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                      __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    }
    static __device__ __forceinline__ uint32_t pack2(float lo, float hi)
    {
        f32x2 x = {lo, hi};
        return __builtin_bit_cast(uint32_t, __builtin_convertvector(x, f16x2));    // v_cvt_pk_f16_f32, RNE
    }
};

__device__ __forceinline__ uint4 ld16(const char *p) { return *reinterpret_cast<const uint4 *>(p); }

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// K and V are read exactly once per work unit: stream them past the caches.
__device__ __forceinline__ uint4 ld16_stream(const char *p)
{
    const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

// Maximum over the four lanes n, n + 16, n + 32, n + 48 (the lanes that hold the same query row in the
// accumulator layout), left in all four.  gfx950's row-swap instructions do it in the vector ALU: swapping
// a value with itself puts row pairs (then wavefront halves) side by side in the two results, and their
// maximum is the exchange-and-reduce step; a shuffle through LDS costs a round trip of ~100 cycles each.
typedef unsigned int u32x2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float max_over_row_groups(float v)
{
    u32x2v r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
    r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r.x), __uint_as_float(r.y));
}

// V^T tile in LDS, in units of 16 bytes (= the 8 k-slots of one channel for one lane group):
//   unit(d = 8c + dd, grp) = 66 dd + 16 grp + c
// The writer lane (grp = tq, c) stores channel 8c + dd at its base + 66*16*dd bytes; the reader
// lane (grp, m = 8h + dd') loads channel 16 dt + m = 8 (2dt + h) + dd' from its base + 32 dt bytes.
// Within a 16-lane group both patterns hit 16 distinct 16-byte bank groups: conflict free.
constexpr int kVtUnits = 66 * 7 + 64;
constexpr int kVtBytes = ((kVtUnits * 16 + 255) / 256) * 256;

// Everything a workgroup needs to know about one work unit; all wave-uniform.
struct Unit {
    int item, gkv, i, ns, L, n, rows, r0, t0, t1, nblk;
    int64_t qrow0, bt_off;      // first query row; offset of the request's row in block_table
};

}  // namespace adaspec
