// Shared device helpers for the gfx950 kernels: wave64 primitives, block
// scans and reductions.  Everything assumes 64-wide wavefronts.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define NGC_WAVE 64

#define NGC_HIP_CHECK(expr)                         \
    do {                                            \
        hipError_t _e = (expr);                     \
        if (_e != hipSuccess) return NGC_EHIP;      \
    } while (0)

namespace ngc {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// 2^x by the hardware instruction (-inf -> 0); for exponents <= 0 or small.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (NGC_WAVE - 1); }
__device__ __forceinline__ int wave_id() { return threadIdx.x >> 6; }

// Number of set bits of `mask` below this lane.
__device__ __forceinline__ int popc_below(uint64_t mask)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Reductions over the four lanes {l, l ^ 16, l ^ 32, l ^ 48} (the lane groups that share lane % 16 in the
// attention kernels), result in all four.  gfx950's lane-swap instructions exchange the halves / the odd and even
// rows of two registers inside the vector ALU: with both operands holding x, one comes back as [lo, lo] and the
// other as [hi, hi] (rows [r0, r0, r2, r2] and [r1, r1, r3, r3]), so combining the pair is the xor-32 (xor-16)
// step of a butterfly -- without the trip through LDS that a shuffle takes.
// max of two numbers that are known not to be NaN: the median of (a, b, +inf), one instruction, where fmaxf()
// first spends one more on each operand whose origin the compiler cannot see (a matrix-core result, a lane swap)
// to quiet a signalling NaN.
__device__ __forceinline__ float max_no_nan(float a, float b)
{
    return __builtin_amdgcn_fmed3f(a, b, __builtin_inff());
}
__device__ __forceinline__ float quad_rows_max(float v)
{
    uint32_t u = __float_as_uint(v);
    auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    u = __float_as_uint(max_no_nan(__uint_as_float(a[0]), __uint_as_float(a[1])));
    auto b = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return max_no_nan(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float quad_rows_sum(float v)
{
    uint32_t u = __float_as_uint(v);
    auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    u = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane16_swap(u, u, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

__device__ __forceinline__ int wave_sum_i(int v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, NGC_WAVE);
    return v;
}
__device__ __forceinline__ float wave_sum_f(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, NGC_WAVE);
    return v;
}
__device__ __forceinline__ float wave_max_f(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, NGC_WAVE));
    return v;
}
__device__ __forceinline__ int wave_incl_scan_i(int v)
{
    const int lane = lane_id();
#pragma unroll
    for (int o = 1; o < NGC_WAVE; o <<= 1) {
        int t = __shfl_up(v, o, NGC_WAVE);
        if (lane >= o) v += t;
    }
    return v;
}
__device__ __forceinline__ float wave_incl_scan_f(float v)
{
    const int lane = lane_id();
#pragma unroll
    for (int o = 1; o < NGC_WAVE; o <<= 1) {
        float t = __shfl_up(v, o, NGC_WAVE);
        if (lane >= o) v += t;
    }
    return v;
}

// Block-wide exclusive scan of one int per thread.  `tmp` holds one int per
// wave (+1).  Returns the exclusive prefix; *total receives the block sum.
// Contains two barriers; every thread of the block must call it.
template <int THREADS>
__device__ __forceinline__ int block_excl_scan_i(int v, int *tmp, int *total)
{
    constexpr int NW = THREADS / NGC_WAVE;
    const int incl = wave_incl_scan_i(v);
    if (lane_id() == NGC_WAVE - 1) tmp[wave_id()] = incl;
    __syncthreads();
    int base = 0, all = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        int t = tmp[w];
        if (w < wave_id()) base += t;
        all += t;
    }
    __syncthreads();
    *total = all;
    return base + incl - v;
}

template <int THREADS>
__device__ __forceinline__ float block_excl_scan_f(float v, float *tmp, float *total)
{
    constexpr int NW = THREADS / NGC_WAVE;
    const float incl = wave_incl_scan_f(v);
    if (lane_id() == NGC_WAVE - 1) tmp[wave_id()] = incl;
    __syncthreads();
    float base = 0.f, all = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        float t = tmp[w];
        if (w < wave_id()) base += t;
        all += t;
    }
    __syncthreads();
    *total = all;
    float prev = __shfl_up(incl, 1, NGC_WAVE);   // sum of the lanes below, no subtraction
    if (lane_id() == 0) prev = 0.f;
    return base + prev;
}

template <int THREADS>
__device__ __forceinline__ float block_sum_f(float v, float *tmp)
{
    constexpr int NW = THREADS / NGC_WAVE;
    v = wave_sum_f(v);
    if (lane_id() == 0) tmp[wave_id()] = v;
    __syncthreads();
    float all = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) all += tmp[w];
    __syncthreads();
    return all;
}

template <int THREADS>
__device__ __forceinline__ float block_max_f(float v, float *tmp)
{
    constexpr int NW = THREADS / NGC_WAVE;
    v = wave_max_f(v);
    if (lane_id() == 0) tmp[wave_id()] = v;
    __syncthreads();
    float all = tmp[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) all = fmaxf(all, tmp[w]);
    __syncthreads();
    return all;
}

// Two maxima in one pass (same barriers as one).  `tmp` holds two floats per wave.
template <int THREADS>
__device__ __forceinline__ void block_max2_f(float &a, float &b, float *tmp)
{
    constexpr int NW = THREADS / NGC_WAVE;
    a = wave_max_f(a);
    b = wave_max_f(b);
    if (lane_id() == 0) { tmp[2 * wave_id()] = a; tmp[2 * wave_id() + 1] = b; }
    __syncthreads();
    a = tmp[0];
    b = tmp[1];
#pragma unroll
    for (int w = 1; w < NW; ++w) {
        a = fmaxf(a, tmp[2 * w]);
        b = fmaxf(b, tmp[2 * w + 1]);
    }
    __syncthreads();
}

template <int THREADS>
__device__ __forceinline__ uint32_t block_max_u(uint32_t v, uint32_t *tmp)
{
    constexpr int NW = THREADS / NGC_WAVE;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const uint32_t t = (uint32_t)__shfl_xor((int)v, o, NGC_WAVE);
        v = t > v ? t : v;
    }
    if (lane_id() == 0) tmp[wave_id()] = v;
    __syncthreads();
    uint32_t all = tmp[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) all = tmp[w] > all ? tmp[w] : all;
    __syncthreads();
    return all;
}

}  // namespace ngc
