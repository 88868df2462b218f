// Sums of exp(x) kept as (m, s) pairs meaning s * e^m: the wide-range arithmetic of the ordered-subset
// log-probability (Eq. 2) and its gradient.
//
// The ordinary path of those kernels works with e_t = exp(s_t - max s) in fp32.  That is exact enough and
// cheap, but e_t underflows to 0 once s_t lies ~100 below the maximum; a sequence that picks such entries after
// everything larger is gone (K = n rounds over heavy-tailed logits) then has R_j = 0 and log R_j = -inf where
// the true term is finite.  Segments whose finite logits span more than NGC_WIDE_SPREAD take the route below
// instead: every running sum carries its own exponent, so nothing underflows whatever the span; each term
// costs up to two exponentials instead of one.  The exponents are logits as they came (no shift by the
// segment's maximum, which would round at the size of the span): differences are only ever taken between an
// entry and the largest entry still in its sum.  Values are positive sums; (-inf, 0) is the empty sum.
#pragma once

#include <hip/hip_runtime.h>
#include <math.h>

#include "ngc_device.h"

namespace ngc {

constexpr float NGC_WIDE_SPREAD = 80.0f;   // e^-80 ~ 1.8e-35: still a normal fp32 number, with room for sums

struct LogSum {
    float m, s;
};

__device__ __forceinline__ LogSum ls_empty() { return LogSum{-INFINITY, 0.f}; }

__device__ __forceinline__ LogSum ls_add(LogSum a, LogSum b)
{
    const float M = fmaxf(a.m, b.m);
    if (M == -INFINITY) return ls_empty();
    // the operand that holds the maximum keeps its sum as is; exp(-inf - M) = 0 drops an empty operand
    return LogSum{M, a.s * expf(a.m - M) + b.s * expf(b.m - M)};
}

// one more term e^x (x = -inf adds nothing)
__device__ __forceinline__ LogSum ls_add_term(LogSum a, float x)
{
    if (x == -INFINITY) return a;
    if (x <= a.m) return LogSum{a.m, a.s + expf(x - a.m)};
    return LogSum{x, a.s * expf(a.m - x) + 1.0f};   // a.m = -inf: a.s = 0
}

// log of the sum; -inf for the empty sum
__device__ __forceinline__ float ls_log(LogSum a) { return a.s > 0.f ? a.m + logf(a.s) : -INFINITY; }

__device__ __forceinline__ LogSum ls_shfl_up(LogSum a, int o)
{
    return LogSum{__shfl_up(a.m, o, NGC_WAVE), __shfl_up(a.s, o, NGC_WAVE)};
}
__device__ __forceinline__ LogSum ls_shfl_xor(LogSum a, int o)
{
    return LogSum{__shfl_xor(a.m, o, NGC_WAVE), __shfl_xor(a.s, o, NGC_WAVE)};
}

// Block-wide sum.  `tmp` holds two floats per wave.  Two barriers; every thread calls it.
template <int THREADS>
__device__ __forceinline__ LogSum block_sum_ls(LogSum v, float *tmp)
{
    constexpr int NW = THREADS / NGC_WAVE;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = ls_add(v, ls_shfl_xor(v, o));
    if (lane_id() == 0) { tmp[2 * wave_id()] = v.m; tmp[2 * wave_id() + 1] = v.s; }
    __syncthreads();
    LogSum all = ls_empty();
#pragma unroll
    for (int w = 0; w < NW; ++w) all = ls_add(all, LogSum{tmp[2 * w], tmp[2 * w + 1]});
    __syncthreads();
    return all;
}

// Block-wide exclusive scan (thread order).  `tmp` holds two floats per wave.  Returns the sum of the
// values of the threads below; *total receives the block sum.  Two barriers; every thread calls it.
template <int THREADS>
__device__ __forceinline__ LogSum block_excl_scan_ls(LogSum v, float *tmp, LogSum *total)
{
    constexpr int NW = THREADS / NGC_WAVE;
    const int lane = lane_id();
    LogSum incl = v;
#pragma unroll
    for (int o = 1; o < NGC_WAVE; o <<= 1) {
        const LogSum t = ls_shfl_up(incl, o);
        if (lane >= o) incl = ls_add(t, incl);
    }
    if (lane == NGC_WAVE - 1) { tmp[2 * wave_id()] = incl.m; tmp[2 * wave_id() + 1] = incl.s; }
    __syncthreads();
    LogSum base = ls_empty(), all = ls_empty();
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const LogSum t = LogSum{tmp[2 * w], tmp[2 * w + 1]};
        if (w < wave_id()) base = ls_add(base, t);
        all = ls_add(all, t);
    }
    __syncthreads();
    *total = all;
    LogSum prev = ls_shfl_up(incl, 1);
    if (lane == 0) prev = ls_empty();
    return ls_add(base, prev);
}

// Eq. 2 for the picks in sampled order, wide-range route.  term(j) = logit of the j-th pick as it came
// (-inf for a masked pick), U = the sum of e^logit over everything never picked.  Thread 0 owns the last
// chunk of picks, so an exclusive scan over threads yields what was picked after a thread's chunk.  Whole
// workgroup; returns log p in every thread.  `tmp` holds two floats per wave.
template <int THREADS, class Term>
__device__ __forceinline__ float sigma_logprob_wide(Term term, int K, LogSum U, float *tmp)
{
    const int tid = threadIdx.x;
    const int chunk = (K + THREADS - 1) / THREADS;
    const int nchunks = (K + chunk - 1) / chunk;
    const int cidx = nchunks - 1 - tid;
    const int j_lo = cidx * chunk;
    const int j_hi = (cidx >= 0) ? ((j_lo + chunk < K) ? j_lo + chunk : K) : 0;
    LogSum mass = ls_empty();
    if (cidx >= 0)
        for (int j = j_lo; j < j_hi; ++j) mass = ls_add_term(mass, term(j));
    LogSum total;
    const LogSum after = block_excl_scan_ls<THREADS>(mass, tmp, &total);
    float acc = 0.f;
    if (cidx >= 0) {
        LogSum R = ls_add(U, after);
        for (int j = j_hi - 1; j >= j_lo; --j) {
            const float x = term(j);
            R = ls_add_term(R, x);
            // a masked pick (logit -inf) has probability 0: log p = -inf.  Otherwise x - log R, with the
            // difference to the largest entry left taken first (exact when the two are close)
            acc += (x == -INFINITY) ? -INFINITY : (x - R.m) - logf(R.s);
        }
    }
    return block_sum_f<THREADS>(acc, tmp);
}

}  // namespace ngc
