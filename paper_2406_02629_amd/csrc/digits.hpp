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

// Limb dwords of a block of 16 pixels x 16 channels, staged in LDS as [party][limb][pixel][group of four
// channels], to channel-innermost limb planes (per party [limb][pixel][C channels], int8): thread t of the 256
// takes limb t/16 % SS_NLIMB of pixel t%16 for the parties t/(16 SS_NLIMB), that + 2, ... and writes the 16
// channels c0..c0+15 as one 16-byte store (a dword per wave would be a 4-byte store at a stride of C bytes).
template <int MAXP>
__device__ __forceinline__ void store_staged_planes(const u32 (&stage)[MAXP][SS_NLIMB][16][4],
                                                    signed char *__restrict__ planes, size_t party_bytes, size_t plane,
                                                    int pix0, int npix, int C, int c0, int n)
{
    constexpr int PSTEP = 256 / (16 * SS_NLIMB);   // parties in flight: 2
    const int t = threadIdx.x, px = t & 15, limb = (t >> 4) % SS_NLIMB, p0 = t / (16 * SS_NLIMB);
    if (pix0 + px >= npix || p0 >= PSTEP) return;
    for (int p = p0; p < n; p += PSTEP) {
        const int4 val = *reinterpret_cast<const int4 *>(&stage[p][limb][px][0]);
        *reinterpret_cast<int4 *>(planes + p * party_bytes + (size_t)limb * plane + (size_t)(pix0 + px) * C + c0) = val;
    }
}
