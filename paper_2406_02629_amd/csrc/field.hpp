// Field arithmetic and the counter-based generator, for device and host code
// of the GPU library.  The field is fixed when the library is compiled:
//   default           p = 2^61 - 1: 2^61 = 1 (mod p), a value is reduced by
//                     adding its bits above 61 to its low 61 bits ("fold");
//   -DSS_FIELD_P45    p = 2^45 - 55, the prime of Sec. VII-A: 2^45 = 55 (mod p),
//                     the bits above 45 are folded in with weight 55.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint64_t u64;
typedef uint32_t u32;

#define SS_GAMMA 0x9E3779B97F4A7C15ULL
#define SS_MAXN 8
#define SS_MAXT 3
#define SS_MAXK (SS_MAXT + 1)

#define SS_HD __host__ __device__ __forceinline__

SS_HD u64 ss_mulhi(u64 a, u64 b)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __umul64hi(a, b);
#else
    return (u64)(((unsigned __int128)a * b) >> 64);
#endif
}

#if defined(SS_FIELD_P45)

#define SS_P 0x1FFFFFFFFFC9ULL   // 2^45 - 55 = 35184372088777, the prime of Sec. VII-A
#define SS_PBITS 45
#define SS_NLIMB 6             // balanced 8-bit digits of a field element
#define SS_NS ss45             // namespace of this build's kernels and launchers
#define SS_PC 55ULL            // 2^45 = 55 (mod p)
#define SS_PMASK ((1ULL << 45) - 1)

// x < 2^64  ->  result < 2^45 + 2^25 < 2p, same residue
SS_HD u64 ss_fold(u64 x) { return (x & SS_PMASK) + SS_PC * (x >> 45); }

// x < 2p  ->  canonical
SS_HD u64 ss_canon(u64 x) { return x >= SS_P ? x - SS_P : x; }

// any x < 2^64  ->  canonical
SS_HD u64 ss_reduce(u64 x) { return ss_canon(ss_fold(x)); }

SS_HD u64 ss_add(u64 a, u64 b) { return ss_canon(a + b); }          // a, b canonical
SS_HD u64 ss_sub(u64 a, u64 b) { return ss_canon(a + SS_P - b); }   // a, b canonical
SS_HD u64 ss_neg(u64 a) { return a ? SS_P - a : 0; }

// 128-bit value hi:lo with hi < 2^38 -> canonical: cut at bit 45, the upper part weighs 55
SS_HD u64 ss_reduce128(u64 hi, u64 lo)
{
    const u64 upper = (hi << 19) | (lo >> 45);            // < 2^57
    return ss_reduce((lo & SS_PMASK) + SS_PC * upper);    // < 2^45 + 2^63
}

// a, b < 2^45: product < 2^90, hi < 2^26
SS_HD u64 ss_mul(u64 a, u64 b) { return ss_reduce128(ss_mulhi(a, b), a * b); }

// 128-bit accumulator for sums of a few products of canonical values
struct ss_acc {
    u64 hi, lo;
    SS_HD void clear() { hi = 0; lo = 0; }
    SS_HD void mac(u64 a, u64 b)
    {
        u64 l = a * b, h = ss_mulhi(a, b);
        lo += l;
        hi += h + (lo < l);
    }
    // up to 2^6 products of values below 2^45: sum < 2^96, hi < 2^32
    SS_HD u64 value() const { return ss_reduce128(hi, lo); }
};

// Accumulator for sums of v * c with v canonical and c a small signed integer
// (|c| < 2^26), at most 8 terms; the two 32-bit halves of v are multiplied
// separately.  A negative c multiplies p - v instead.
struct ss_sacc {
    u64 lo, hi;
    SS_HD void clear() { lo = 0; hi = 0; }
    SS_HD void mac(u64 v, int c)
    {
        const u64 w = c < 0 ? SS_P - v : v;
        const u32 m = (u32)(c < 0 ? -c : c);
        lo += (w & 0xFFFFFFFFull) * (u64)m;   // each < 2^58
        hi += (w >> 32) * (u64)m;             // each < 2^39
    }
    // lo + hi 2^32; hi = a 2^13 + b gives hi 2^32 = a 2^45 + b 2^32 = 55 a + b 2^32
    SS_HD u64 value() const
    {
        return ss_reduce(ss_fold(lo) + SS_PC * (hi >> 13) + ((hi & 0x1FFFull) << 32));
    }
};

// x canonical, c a small constant (c <= 8): x*c < 2^48
SS_HD u64 ss_mul_small(u64 x, u32 c) { return ss_reduce(x * (u64)c); }

#else

#define SS_P 0x1FFFFFFFFFFFFFFFULL
#define SS_PBITS 61
#define SS_NLIMB 8   // balanced 8-bit digits of a field element
#define SS_NS ss61   // namespace of this build's kernels and launchers

// x < 2^64  ->  result < 2^61 + 8, same residue
SS_HD u64 ss_fold(u64 x) { return (x & SS_P) + (x >> 61); }

// x < 2p  ->  canonical
SS_HD u64 ss_canon(u64 x) { return x >= SS_P ? x - SS_P : x; }

// any x < 2^64  ->  canonical
SS_HD u64 ss_reduce(u64 x) { return ss_canon(ss_fold(x)); }

SS_HD u64 ss_add(u64 a, u64 b) { return ss_canon(a + b); }          // a, b canonical
SS_HD u64 ss_sub(u64 a, u64 b) { return ss_canon(a + SS_P - b); }   // a, b canonical
SS_HD u64 ss_neg(u64 a) { return a ? SS_P - a : 0; }

// any 128-bit value hi:lo -> canonical.  2^64 = 2^3 (mod p), so
// hi * 2^64 = ((hi mod 2^58) << 3) + (hi >> 58) * 2^61 = ((hi mod 2^58) << 3) + (hi >> 58)
SS_HD u64 ss_reduce128(u64 hi, u64 lo)
{
    u64 r = (lo & SS_P) + (lo >> 61) + ((hi << 3) & SS_P) + (hi >> 58);   // < 2^62 + 2^7
    return ss_reduce(r);
}

// a, b < 2^61: product < 2^122, hi < 2^58
SS_HD u64 ss_mul(u64 a, u64 b) { return ss_reduce128(ss_mulhi(a, b), a * b); }

// 128-bit accumulator for sums of a few products of canonical values
struct ss_acc {
    u64 hi, lo;
    SS_HD void clear() { hi = 0; lo = 0; }
    SS_HD void mac(u64 a, u64 b)
    {
        u64 l = a * b, h = ss_mulhi(a, b);
        lo += l;
        hi += h + (lo < l);
    }
    // exact while the sum stays below 2^128: up to 2^6 products of values below 2^61
    SS_HD u64 value() const { return ss_reduce128(hi, lo); }
};

// Accumulator for sums of v * c with v canonical and c a small signed integer
// (|c| < 2^26), at most 8 terms: the two 32-bit halves of v are multiplied
// separately, so a term costs two 32 x 32 -> 64 multiply-adds instead of a
// 64 x 64 -> 128 product.  A negative c multiplies p - v instead.
struct ss_sacc {
    u64 lo, hi;
    SS_HD void clear() { lo = 0; hi = 0; }
    SS_HD void mac(u64 v, int c)
    {
        const u64 w = c < 0 ? SS_P - v : v;
        const u32 m = (u32)(c < 0 ? -c : c);
        lo += (w & 0xFFFFFFFFull) * (u64)m;   // each < 2^58
        hi += (w >> 32) * (u64)m;             // each < 2^55
    }
    // lo + hi 2^32 with 2^61 = 1
    SS_HD u64 value() const
    {
        return ss_reduce(ss_fold(lo) + ((hi & ((1ULL << 29) - 1)) << 32) + (hi >> 29));
    }
};

// x canonical, c a small constant (c <= 8): x*c < 2^64
SS_HD u64 ss_mul_small(u64 x, u32 c) { return ss_reduce(x * (u64)c); }

#endif

// ---- generator ----
SS_HD u64 ss_mix64(u64 z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

SS_HD u64 ss_key(u64 seed, u64 domain, u64 stream_id, u64 party, u64 j)
{
    u64 h = 0;
    h = ss_mix64((h ^ seed) + SS_GAMMA);
    h = ss_mix64((h ^ domain) + SS_GAMMA);
    h = ss_mix64((h ^ stream_id) + SS_GAMMA);
    h = ss_mix64((h ^ party) + SS_GAMMA);
    h = ss_mix64((h ^ j) + SS_GAMMA);
    return h;
}

SS_HD u64 ss_draw(u64 key, u64 e) { return ss_mix64(key + (e + 1) * SS_GAMMA); }

// field element from the top 61 bits of a draw: (draw >> 3) mod p
SS_HD u64 ss_field_of(u64 draw)
{
    const u64 r = draw >> 3;
#if defined(SS_FIELD_P45)
    return ss_reduce(r);
#else
    return r == SS_P ? 0 : r;
#endif
}

SS_HD u64 ss_draw_field(u64 key, u64 e) { return ss_field_of(ss_draw(key, e)); }

// the same draws from the element's counter word (e+1)*GAMMA, which all keys of an element share
SS_HD u64 ss_counter(u64 e) { return (e + 1) * SS_GAMMA; }
SS_HD u64 ss_draw_at(u64 key, u64 counter) { return ss_mix64(key + counter); }
SS_HD u64 ss_draw_field_at(u64 key, u64 counter) { return ss_field_of(ss_draw_at(key, counter)); }

// polynomial a0 + c[0] x + ... + c[d-1] x^d at the small point x (1..8), by
// Horner.  MAXD bounds d at compile time so that c[] stays in registers.
template <int MAXD>
SS_HD u64 ss_poly_eval(u64 a0, const u64 *c, int d, u32 x)
{
    u64 acc = 0;
#pragma unroll
    for (int j = MAXD; j >= 1; j--) {
        if (j <= d) {
            acc = ss_add(acc, c[j - 1]);
            acc = ss_mul_small(acc, x);
        }
    }
    return ss_add(acc, a0);
}
