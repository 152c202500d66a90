// Cross-lane reductions for the matrix-core kernels' operand layout (gfx950).
#pragma once
#include <hip/hip_runtime.h>

// Lanes n, n+16, n+32, n+48 of a wave (n = lane % 16) hold parts of one column of a
// 16-wide MFMA result.  Two swap instructions give every one of them the maximum (or
// the sum) over the four: the first exchanges odd rows of 16 lanes with even ones, the
// second the upper 32 lanes with the lower.  No LDS traffic, unlike a lane permute.
__device__ __forceinline__ float quad_rows_max(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ __forceinline__ float quad_rows_sum(float x)
{
    auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

