// Wavefront-level helpers shared by the DAMP kernels (gfx950, 64-wide wavefronts).
#pragma once

#include <hip/hip_runtime.h>

namespace dol {

constexpr int kWave = 64;

// Workgroups are dealt round-robin to the 8 XCDs of the chip (one L2 each).  This maps workgroup `id` of a
// grid of `n` to a work index such that each XCD walks one contiguous range of indices (a bijection on 0..n-1),
// so that memory lines shared by neighbouring indices are fetched into one L2 only.
__device__ __forceinline__ int xcd_contiguous(unsigned id, unsigned n)
{
    const unsigned x = id & 7u, k = id >> 3, q = n >> 3, r = n & 7u;
    return static_cast<int>(x * q + (x < r ? x : r) + k);
}

template <int CTRL>
__device__ __forceinline__ float dpp(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

template <int CTRL>
__device__ __forceinline__ int dpp_i(int x)
{
    return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xF, 0xF, false);
}

// All-reduce over the 32 lanes that share a sample (lanes 0-31 or 32-63 of a wavefront): quad butterflies,
// mirrored halves of 8 and 16 lanes (every lane of a group already holds the group's value), then the
// other row of 16.  Every lane of the wavefront must be active.
struct AddOp { __device__ static float f(float a, float b) { return a + b; } };
struct MaxOp { __device__ static float f(float a, float b) { return fmaxf(a, b); } };
template <typename Op>
__device__ __forceinline__ float reduce32(float x)
{
    x = Op::f(x, dpp<0xB1>(x));          // quad_perm [1,0,3,2]
    x = Op::f(x, dpp<0x4E>(x));          // quad_perm [2,3,0,1]
    x = Op::f(x, dpp<0x141>(x));         // row_half_mirror
    x = Op::f(x, dpp<0x140>(x));         // row_mirror
    x = Op::f(x, __shfl_xor(x, 16, kWave));
    return x;
}

// The same over the 16 lanes of one DPP row.
template <typename Op>
__device__ __forceinline__ float reduce16(float x)
{
    x = Op::f(x, dpp<0xB1>(x));
    x = Op::f(x, dpp<0x4E>(x));
    x = Op::f(x, dpp<0x141>(x));
    x = Op::f(x, dpp<0x140>(x));
    return x;
}

__device__ __forceinline__ int reduce16_or(int x)
{
    x |= dpp_i<0xB1>(x);
    x |= dpp_i<0x4E>(x);
    x |= dpp_i<0x141>(x);
    x |= dpp_i<0x140>(x);
    return x;
}

__device__ __forceinline__ int reduce32_or(int x)
{
    x |= dpp_i<0xB1>(x);
    x |= dpp_i<0x4E>(x);
    x |= dpp_i<0x141>(x);
    x |= dpp_i<0x140>(x);
    x |= __shfl_xor(x, 16, kWave);
    return x;
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x = fmaxf(x, __shfl_xor(x, d, kWave));
    return x;
}

// LDS rows that are written and read by the lanes of one wavefront only need nothing but program order
// within the wavefront: this keeps the compiler from moving LDS accesses across the point and costs no
// instruction.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Workgroup barrier that orders LDS accesses only.  __syncthreads() also waits until every global store issued
// before it has been acknowledged; kernels whose threads exchange data through LDS alone, and stream results to
// memory that nobody reads back, need not pay that round trip at every barrier.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

}  // namespace dol
