// Shared by the draft-sampling kernels that work on packed 16-bit logits (draft_fast.hip,
// draft_split.hip): the probabilities of one 16-byte chunk.
#pragma once
#include <type_traits>

#include "device_utils.h"
#include "row_registers.h"

namespace adaspec {

// the 8 probabilities of one chunk: computed in fp32, rounded once to the storage type PT;
// returns them as floats (the rounded values) and, for 16-bit storage, packed for the store
template <class DT, class PT>
__device__ __forceinline__ void chunk_probs(const uint4 &lg, float c2, float mc, float invZ, float (&q)[8], uint4 &packed)
{
    using P = Pair16<DT>;
    const uint32_t w[4] = {lg.x, lg.y, lg.z, lg.w};
    uint32_t o[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float a = __builtin_amdgcn_exp2f(fmaf(P::lo(w[e]), c2, -mc)) * invZ;
        float b = __builtin_amdgcn_exp2f(fmaf(P::hi(w[e]), c2, -mc)) * invZ;
        if constexpr (std::is_same<PT, BF16>::value) {
            const uint16_t ba = float_to_bf16_bits(a), bb = float_to_bf16_bits(b);
            a = bf16_bits_to_float(ba); b = bf16_bits_to_float(bb);
            o[e] = (uint32_t)ba | ((uint32_t)bb << 16);
        } else if constexpr (std::is_same<PT, F16>::value) {
            const uint16_t ba = float_to_f16_bits(a), bb = float_to_f16_bits(b);
            a = f16_bits_to_float(ba); b = f16_bits_to_float(bb);
            o[e] = (uint32_t)ba | ((uint32_t)bb << 16);
        } else {
            o[e] = 0;
        }
        q[2 * e] = a; q[2 * e + 1] = b;
    }
    packed = make_uint4(o[0], o[1], o[2], o[3]);
}

}  // namespace adaspec
