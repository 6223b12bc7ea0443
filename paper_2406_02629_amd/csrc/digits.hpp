// Balanced radix-2^8 digits of field elements and their byte transposition, shared by the kernels that
// write int8 limb tiles or limb planes.
#pragma once
#include "field.hpp"

// balanced digits of x as 8 signed bytes: x = sum d_i 2^(8i), d_i in [-128, 127]
__device__ __forceinline__ u64 balanced_digits(u64 x) { return (x + 0x8080808080808080ULL) ^ 0x8080808080808080ULL; }

// one dword per limb from the digit words of four consecutive contraction indices (byte c of the result is
// digit `limb` of y[c]); limb may differ from lane to lane
__device__ __forceinline__ u32 limb_dword(const u64 (&y)[4], int limb)
{
    const int i = limb & 3;
    const u32 a = limb < 4 ? (u32)y[0] : (u32)(y[0] >> 32), b = limb < 4 ? (u32)y[1] : (u32)(y[1] >> 32);
    const u32 c = limb < 4 ? (u32)y[2] : (u32)(y[2] >> 32), d = limb < 4 ? (u32)y[3] : (u32)(y[3] >> 32);
    // v_perm_b32: selector byte k picks byte k of {second operand (0..3), first operand (4..7)}; 0x0c = zero
    const u32 sel = (u32)i | ((u32)(4 + i) << 8) | 0x0c0c0000u;
    return __builtin_amdgcn_perm(__builtin_amdgcn_perm(d, c, sel), __builtin_amdgcn_perm(b, a, sel), 0x05040100u);
}
