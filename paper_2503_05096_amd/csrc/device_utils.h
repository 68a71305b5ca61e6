// Small device helpers shared by the gfx950 kernels: storage-type conversion,
// 64-lane wavefront reductions and scans.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adaspec {

constexpr int kWave = 64;

// ---- storage types -------------------------------------------------------
struct F32 { using storage = float;    static constexpr int id = 0; };
struct F16 { using storage = uint16_t; static constexpr int id = 1; };
struct BF16 { using storage = uint16_t; static constexpr int id = 2; };

__device__ __forceinline__ float bf16_bits_to_float(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float f16_bits_to_float(uint16_t b)
{
    _Float16 h;
    __builtin_memcpy(&h, &b, 2);
    return (float)h;
}

// round-to-nearest-even from fp32
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // NaN stays NaN
    return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ uint16_t float_to_f16_bits(float f)
{
    _Float16 h = (_Float16)f;   // v_cvt_f16_f32, RNE
    uint16_t b;
    __builtin_memcpy(&b, &h, 2);
    return b;
}

template <class T> __device__ __forceinline__ float load_as_float(const void *base, int64_t idx);
template <> __device__ __forceinline__ float load_as_float<F32>(const void *base, int64_t idx)
{ return ((const float *)base)[idx]; }
template <> __device__ __forceinline__ float load_as_float<F16>(const void *base, int64_t idx)
{ return f16_bits_to_float(((const uint16_t *)base)[idx]); }
template <> __device__ __forceinline__ float load_as_float<BF16>(const void *base, int64_t idx)
{ return bf16_bits_to_float(((const uint16_t *)base)[idx]); }

// store one accumulator value in the requested output type
__device__ __forceinline__ void store_out(void *base, int64_t idx, float v, int out_dtype)
{
    if (out_dtype == 0)      ((float *)base)[idx] = v;
    else if (out_dtype == 1) ((uint16_t *)base)[idx] = float_to_f16_bits(v);
    else                     ((uint16_t *)base)[idx] = float_to_bf16_bits(v);
}

// ---- wavefront collectives ---------------------------------------------
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ int wave_sum(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ int wave_max(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = max(v, __shfl_xor(v, o, kWave));
    return v;
}
// inclusive scans over the 64 lanes
__device__ __forceinline__ double wave_scan_incl(double v, int lane)
{
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        double t = __shfl_up(v, o, kWave);
        if (lane >= o) v += t;
    }
    return v;
}
__device__ __forceinline__ int wave_scan_incl(int v, int lane)
{
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        int t = __shfl_up(v, o, kWave);
        if (lane >= o) v += t;
    }
    return v;
}

// The same inclusive scan with data-parallel-primitive moves instead of LDS permutes: no LDS round
// trip per step, which is what a latency-bound kernel pays for.  Lanes that a shift leaves without a
// source, and rows that a broadcast does not address, add 0.
__device__ __forceinline__ int wave_scan_incl_dpp(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8 -> scan inside each row of 16
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
    return v;
}

// (value, index) max with the LOWEST index winning ties
struct ArgMax { float v; int i; };
__device__ __forceinline__ ArgMax argmax_merge(ArgMax a, ArgMax b)
{
    return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}
__device__ __forceinline__ ArgMax wave_argmax(ArgMax a)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        ArgMax b{__shfl_xor(a.v, o, kWave), __shfl_xor(a.i, o, kWave)};
        a = argmax_merge(a, b);
    }
    return a;
}

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also drains the
// vector-memory counter (its fences cover global memory), which would stall on every global load
// that was deliberately left in flight across the barrier; this one waits for LDS traffic alone.
__device__ __forceinline__ void lds_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__host__ __device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }
__host__ __device__ __forceinline__ size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

}  // namespace adaspec
