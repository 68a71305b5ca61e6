// Helpers for kernels that walk one vocabulary row of 16-bit values with 1024 threads and 16-byte
// loads WITHOUT keeping it in registers: element (s * 1024 + t) * 8 + e belongs to step s, thread t.
#pragma once
#include "device_utils.h"
#include "row_registers.h"

namespace adaspec {

constexpr int kNT = 1024;
constexpr int kNW = kNT / kWave;
constexpr int kNSteps = 64;             // V <= kNT * 8 * kNSteps = 524288


template <class DT>
__device__ __forceinline__ void unpack8(const uint4 &w, float (&x)[8])
{
    x[0] = Pair16<DT>::lo(w.x); x[1] = Pair16<DT>::hi(w.x);
    x[2] = Pair16<DT>::lo(w.y); x[3] = Pair16<DT>::hi(w.y);
    x[4] = Pair16<DT>::lo(w.z); x[5] = Pair16<DT>::hi(w.z);
    x[6] = Pair16<DT>::lo(w.w); x[7] = Pair16<DT>::hi(w.w);
}
template <class DT>
__device__ __forceinline__ float elem16(const char *row, int v)
{
    return Pair16<DT>::lo((uint32_t) reinterpret_cast<const uint16_t *>(row)[v]);
}

// Per-step totals from the 64 partial sums each step left in `part`: wavefront w adds up steps w, w + 16, ...
// Every thread returns R = sum of S[0 .. nsteps); ends on a barrier.
__device__ __forceinline__ double finish_sweep(const float (&part)[kNSteps][kWave], double (&S)[kNSteps],
                                               int nsteps, int wv, int lane)
{
    __syncthreads();
    for (int s = wv; s < nsteps; s += kNW) {
        const double t = wave_sum((double)part[s][lane]);
        if (lane == 0) S[s] = t;
    }
    __syncthreads();
    double R = 0.0;
    for (int s = 0; s < nsteps; ++s) R += S[s];
    return R;
}

// Walks the steps of a row with the loads of the next kDepth steps in flight: f(step, in_range, logits
// word, draft-probability word).  A wavefront that waited for every step's data before asking for the next
// would pay one memory round trip per step.  start() may be called well before run(): the first loads
// then travel while the kernel does something else.
constexpr int kDepth = 4;
template <bool kWithProbs>
struct RowPipe {
    uint4 lw[kDepth], qw[kDepth];
    const char *lrow, *prow;
    int nsteps, V, tid;

    __device__ __forceinline__ void issue(int j, int s)
    {
        const int v0 = (s * kNT + tid) * 8;
        if (s < nsteps && v0 < V) {
            lw[j] = *reinterpret_cast<const uint4 *>(lrow + (int64_t)v0 * 2);
            if (kWithProbs) qw[j] = *reinterpret_cast<const uint4 *>(prow + (int64_t)v0 * 2);
        }
    }
    __device__ __forceinline__ void start(const char *lrow_, const char *prow_, int nsteps_, int V_, int tid_)
    {
        lrow = lrow_; prow = prow_; nsteps = nsteps_; V = V_; tid = tid_;
#pragma unroll
        for (int j = 0; j < kDepth; ++j) { lw[j] = make_uint4(0, 0, 0, 0); qw[j] = make_uint4(0, 0, 0, 0); issue(j, j); }
    }
    template <class F>
    __device__ __forceinline__ void run(F f)
    {
        for (int s0 = 0; s0 < nsteps; s0 += kDepth) {
#pragma unroll
            for (int j = 0; j < kDepth; ++j) {
                const int s = s0 + j;
                if (s < nsteps) {
                    f(s, (s * kNT + tid) * 8 < V, lw[j], qw[j]);
                    issue(j, s + kDepth);
                }
            }
        }
    }
};

template <bool kWithProbs, class F>
__device__ __forceinline__ void for_each_step(const char *lrow, const char *prow, int nsteps, int V, int tid, F f)
{
    RowPipe<kWithProbs> pipe;
    pipe.start(lrow, prow, nsteps, V, tid);
    pipe.run(f);
}

}  // namespace adaspec
