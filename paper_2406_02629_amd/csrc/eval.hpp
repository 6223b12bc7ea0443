// Device-side evaluation of a sharing polynomial at the party IDs 1, 2, ...
#pragma once
#include "field.hpp"

// values a0 + a[0] x + ... at x = 1..M, canonical, handed to emit(x - 1, value); a0, a[] canonical
template <int T, int M, typename F>
__device__ __forceinline__ void eval_points(u64 a0, const u64 (&a)[T], F &&emit)
{
    static_assert(T == 1 || T == 2, "degrees 1 and 2");
    u64 s = a0;
    if constexpr (T == 1) {
#pragma unroll
        for (int x = 1; x <= M; x++) {
            s = ss_add(s, a[0]);
            emit(x - 1, s);
        }
    } else {
        // first difference d_x = s(x) - s(x-1) = a1 + (2x - 1) a2, second difference 2 a2
        u64 d = a[0] + a[1];       // < 2^62
        const u64 dd = 2 * a[1];   // < 2^62
#pragma unroll
        for (int x = 1; x <= M; x++) {
            if (x > 1) {
                if (x >= 4 && (x - 4) % 3 == 0) d = ss_fold(d);   // keeps d below 7 * 2^61 + 8
                d += dd;
            }
            s = ss_reduce(s + d);   // s < 2^61, so the sum stays below 2^64
            emit(x - 1, s);
        }
    }
}
