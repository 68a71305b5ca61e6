// Device helpers shared by the kernels that keep one vocabulary row of 16-bit values packed in
// registers (1024 threads x 16 bytes per step): the acceptance kernel and the draft-sampling kernel.
#pragma once
#include "device_utils.h"

namespace adaspec {

template <class T> struct Pair16;
template <> struct Pair16<BF16> {
    static constexpr uint32_t kNegInf2 = 0xFF80FF80u;
    static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
    static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
};
template <> struct Pair16<F16> {
    static constexpr uint32_t kNegInf2 = 0xFC00FC00u;
    static __device__ __forceinline__ float lo(uint32_t w) { return f16_bits_to_float((uint16_t)(w & 0xffffu)); }
    static __device__ __forceinline__ float hi(uint32_t w) { return f16_bits_to_float((uint16_t)(w >> 16)); }
};

// Opaque to the optimiser: forces later code to unpack the 16-bit pairs again instead of
// keeping 128 unpacked floats alive across the phases (the row must stay packed to fit).
__device__ __forceinline__ void keep_packed(uint4 &v)
{
    asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
}

typedef short short2v __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// sum over the 16 lanes of a DPP row (every lane of the row ends up with the row's total)
__device__ __forceinline__ float row16_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xF, 0xF, true));  // row_ror 4
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xF, 0xF, true));  // row_ror 8
    return v;
}

// maximum over the 16 lanes of a DPP row (every lane of the row ends up with it)
__device__ __forceinline__ float row16_max(float v)
{
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x124, 0xF, 0xF, true)));
    v = fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x128, 0xF, 0xF, true)));
    return v;
}

}  // namespace adaspec
