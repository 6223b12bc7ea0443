// Element-wise kernels: GEN (Eq. 1), REC (Eq. 2), reshare degree reduction with
// RERAND (Sec. IV-B, IV-C) and masked truncation (Sec. VI-B).
//
// One thread owns VEC consecutive elements and walks over all parties, so every
// plane is read and written with unit stride across a wave and the random
// coefficients of an element are drawn once, not once per party.
#include "kernels.hpp"
#include "eval.hpp"
#include "digits.hpp"

namespace SS_NS {

namespace {

constexpr int BLOCK = 256;

template <int VEC>
struct pack_t;
template <>
struct pack_t<1> {
    u64 v[1];
    __device__ __forceinline__ void load(const u64 *p) { v[0] = *p; }
    __device__ __forceinline__ void store(u64 *p) const { *p = v[0]; }
    __device__ __forceinline__ void store_streaming(u64 *p) const { __builtin_nontemporal_store(v[0], p); }
};
template <>
struct pack_t<2> {
    u64 v[2];
    __device__ __forceinline__ void load(const u64 *p)
    {
        const ulonglong2 q = *reinterpret_cast<const ulonglong2 *>(p);
        v[0] = q.x;
        v[1] = q.y;
    }
    __device__ __forceinline__ void store(u64 *p) const
    {
        ulonglong2 q;
        q.x = v[0];
        q.y = v[1];
        *reinterpret_cast<ulonglong2 *>(p) = q;
    }
    // for output that nothing in the same launch reads again
    __device__ __forceinline__ void store_streaming(u64 *p) const
    {
        typedef unsigned long long v2u __attribute__((ext_vector_type(2)));
        v2u q = {v[0], v[1]};
        __builtin_nontemporal_store(q, reinterpret_cast<v2u *>(p));
    }
};

// share i of element e of the incoming product, which may be given as a sum of planes (the partial-sum form
// of the product kernels): canonical sum of the planes' values
__device__ __forceinline__ u64 load_product(const u64 *c, size_t idx, const ss_part_src &ps)
{
    u64 v = c[idx];
    for (int s = 1; s < ps.planes; s++) v = ss_add(v, c[idx + (size_t)s * ps.stride]);
    return v;
}

template <int MAXD>
__device__ __forceinline__ void draw_coeffs(u64 (&c)[MAXD], const u64 *keys, int d, u64 e)
{
    const u64 counter = ss_counter(e);
#pragma unroll
    for (int j = 0; j < MAXD; j++) c[j] = (j < d) ? ss_draw_field_at(keys[j], counter) : 0;
}

// ------------------------------------------------------------------ GEN
// NC, DC > 0 fix the party count and the degree at compile time (the schemes
// the paper evaluates: (k,n) = (2,3) and (3,5)), so that the evaluation points
// become immediates; 0 means "take the run-time value".
template <int VEC, int NC, int DC>
__global__ __launch_bounds__(BLOCK) void share_kernel(const u64 *__restrict__ secret, u64 *__restrict__ shares,
                                                      size_t count, int n_rt, int degree_rt, ss_keys keys)
{
    constexpr int MAXD = DC ? DC : SS_MAXDEG;
    constexpr int MAXP = NC ? NC : SS_MAXN;
    const int n = NC ? NC : n_rt, degree = DC ? DC : degree_rt;
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    pack_t<VEC> a0;
    a0.load(secret + e0);
    u64 c[VEC][MAXD];
#pragma unroll
    for (int u = 0; u < VEC; u++) draw_coeffs<MAXD>(c[u], keys.k, degree, e0 + u);
    if constexpr (NC != 0 && (DC == 1 || DC == 2)) {
        // consecutive party IDs: forward differences, two additions per point instead of Horner's multiplications
        pack_t<VEC> s[NC];
#pragma unroll
        for (int u = 0; u < VEC; u++) eval_points<DC, NC>(a0.v[u], c[u], [&](int p, u64 v) { s[p].v[u] = v; });
#pragma unroll
        for (int p = 0; p < NC; p++) s[p].store_streaming(shares + (size_t)p * count + e0);   // written, not read again
    } else {
#pragma unroll
        for (int i = 1; i <= MAXP; i++) {
            if (i <= n) {
                pack_t<VEC> s;
#pragma unroll
                for (int u = 0; u < VEC; u++) s.v[u] = ss_poly_eval<MAXD>(a0.v[u], c[u], degree, i);
                s.store_streaming(shares + (size_t)(i - 1) * count + e0);
            }
        }
    }
}

// ------------------------------------------------------------------ REC
template <int VEC>
__global__ __launch_bounds__(BLOCK) void reconstruct_kernel(const u64 *__restrict__ shares,
                                                            u64 *__restrict__ secret, size_t count,
                                                            ss_rec_params rp)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    pack_t<VEC> out;
    ss_sacc acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; u++) acc[u].clear();
#pragma unroll
    for (int i = 0; i < SS_MAXN; i++) {
        if (i < rp.m) {
            pack_t<VEC> s;
            s.load(shares + (size_t)rp.plane[i] * count + e0);
#pragma unroll
            for (int u = 0; u < VEC; u++) acc[u].mac(s.v[u], rp.ilambda[i]);
        }
    }
#pragma unroll
    for (int u = 0; u < VEC; u++) out.v[u] = rp.dinv == 1 ? acc[u].value() : ss_mul(acc[u].value(), rp.dinv);
    out.store(secret + e0);
}

// e of the truncation mask alpha = e * 2^f: uniform in [1, 2^(32-f)]
__device__ __forceinline__ u64 mask_e(u64 key, u64 e, int f)
{
    return 1 + ((ss_draw(key, e) >> 3) & ((1ULL << (32 - f)) - 1));
}

// the same before a division by kh*kw: the sample space of e shrinks to [1, floor(2^(32-f) / kdiv)], which keeps
// alpha = e * 2^f * kdiv within (0, 2^32] (Sec. VII-B); range = 2^(32-f) gives mask_e
__device__ __forceinline__ u64 mask_e_below(u64 key, u64 e, unsigned range)
{
    return 1 + (ss_draw(key, e) >> 3) % range;
}

// what the elite party does with the reconstructed x + alpha: floor division of the signed value by 2^f
__device__ __forceinline__ u64 shift_signed(u64 v, int f)
{
    const int64_t sv = (v <= (SS_P - 1) / 2) ? (int64_t)v : (int64_t)v - (int64_t)SS_P;
    const int64_t qv = sv >> f;
    return qv >= 0 ? (u64)qv : SS_P - (u64)(-qv);
}

// The same followed by the rounding division that average pooling moves into the truncation (Sec. VI-C):
// [q / kdiv] = floor((q + floor(kdiv/2)) / kdiv) on the signed quotient q, so that a remainder of
// ceil(kdiv/2) or more goes up (the worst case of App. C) and [(q + e*kdiv) / kdiv] = [q / kdiv] + e.
__device__ __forceinline__ u64 shift_round_div(u64 v, int f, int kdiv)
{
    const int64_t sv = (v <= (SS_P - 1) / 2) ? (int64_t)v : (int64_t)v - (int64_t)SS_P;
    const int64_t a = (sv >> f) + kdiv / 2;
    const u64 d = (u64)kdiv;
    return a >= 0 ? (u64)a / d : SS_P - ((u64)(-a) + d - 1) / d;
}

// The three steps of masked truncation for the elements a thread owns, with
// the same send-to-workspace / receive-from-registers convention as above:
//   1. parties q = 1..k add their share of alpha = e * 2^f          -> umsg[q]
//      (alpha = e * 2^f * kdiv with the rounding division)
//   2. the elite party reconstructs x + alpha, divides by 2^f with floor on
//      the signed value (then by kdiv with rounding) and shares the quotient -> wsh[m]
//   3. every party m adds its share of alpha~ = -e                   -> out[m]
// x[q] holds the shares of parties q+1 = 1..k.  With rec != nullptr the new
// shares are also reconstructed (REC, Eq. 2) with the multipliers rf   -> rec
template <int VEC>
__device__ __forceinline__ void truncate_steps(const pack_t<VEC> *x, u64 *__restrict__ umsg, u64 *__restrict__ wsh,
                                               u64 *out, size_t count, size_t e0, const ss_tr_params &tp,
                                               u64 *__restrict__ rec, const ss_recf_params &rf)
{
    const int k = tp.t + 1;
    u64 ev[VEC], ca[VEC][SS_MAXT];
    ss_sacc acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        ev[u] = tp.kdiv > 1 ? mask_e_below(tp.e_key, e0 + u, tp.e_range) : mask_e(tp.e_key, e0 + u, tp.f);
        draw_coeffs<SS_MAXT>(ca[u], tp.alpha_key, tp.t, e0 + u);
        acc[u].clear();
    }
#pragma unroll
    for (int q = 0; q < SS_MAXK; q++) {
        if (q < k) {
            pack_t<VEC> s;
#pragma unroll
            for (int u = 0; u < VEC; u++) {
                const u64 alpha = tp.kdiv > 1 ? (ev[u] * (u64)tp.kdiv) << tp.f : ev[u] << tp.f;   // <= 2^32
                s.v[u] = ss_add(x[q].v[u], ss_poly_eval<SS_MAXT>(alpha, ca[u], tp.t, q + 1));
                acc[u].mac(s.v[u], tp.ilambda[q]);
            }
            s.store(umsg + (size_t)q * count + e0);
        }
    }
    u64 w[VEC], at[VEC], cw[VEC][SS_MAXT], cat[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        w[u] = tp.kdiv > 1 ? shift_round_div(acc[u].value(), tp.f, tp.kdiv) : shift_signed(acc[u].value(), tp.f);
        at[u] = SS_P - ev[u];
        draw_coeffs<SS_MAXT>(cw[u], tp.gen_key, tp.t, e0 + u);
        draw_coeffs<SS_MAXT>(cat[u], tp.alphat_key, tp.t, e0 + u);
    }
    ss_sacc racc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; u++) racc[u].clear();
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (m < tp.n) {
            pack_t<VEC> ws, s;
#pragma unroll
            for (int u = 0; u < VEC; u++) {
                ws.v[u] = ss_poly_eval<SS_MAXT>(w[u], cw[u], tp.t, m + 1);
                s.v[u] = ss_add(ws.v[u], ss_poly_eval<SS_MAXT>(at[u], cat[u], tp.t, m + 1));
                if (rec && rf.coef[m] != 0) racc[u].mac(s.v[u], rf.coef[m]);
            }
            ws.store(wsh + (size_t)m * count + e0);
            s.store(out + (size_t)m * count + e0);
        }
    }
    if (rec) {
        pack_t<VEC> r;
#pragma unroll
        for (int u = 0; u < VEC; u++) r.v[u] = rf.dinv == 1 ? racc[u].value() : ss_mul(racc[u].value(), rf.dinv);
        r.store(rec + e0);
    }
}

template <int VEC>
__global__ __launch_bounds__(BLOCK) void truncate_kernel(const u64 *x, u64 *__restrict__ umsg,
                                                         u64 *__restrict__ wsh, u64 *out, size_t count,
                                                         ss_tr_params tp)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    pack_t<VEC> xs[SS_MAXK];
#pragma unroll
    for (int q = 0; q < SS_MAXK; q++)
        if (q <= tp.t) xs[q].load(x + (size_t)q * count + e0);
    const ss_recf_params none = {};
    truncate_steps<VEC>(xs, umsg, wsh, out, count, e0, tp, nullptr, none);
}

// ------------------------------------------------------------------ RED + RERAND
// The three protocol steps for the elements a thread owns.  All parties are
// simulated by that one thread, so a message is written to the workspace (the
// "send") and consumed from registers (the "receive"); arithmetic and message
// contents are exactly those of the per-party steps:
//   1. party i = 1..2t+1: sub-shares of c_i for parties q = 1..k     -> msg1[i][q]
//   2. party q: received row vector times R, applied in factored form
//      R = B^-1[:, :k] * V (V[j][m] = m^j): first the k low coefficients of the
//      polynomial through the received values, then its value at every party
//      ID -- same residues as the (2t+1) x n product                 -> msg2[q][m]
//   3. party m: REC of the k received values, plus its share of zero  -> out[m]
//
// With TRUNC the reduced, re-randomised shares do not go to `out` but straight
// into the three truncation steps (truncate_kernel below), whose messages go to
// umsg / wsh: SSS-Linear followed by SSS-Truncation in one launch.
template <int VEC, bool TRUNC>
__global__ __launch_bounds__(BLOCK) void degree_reduce_kernel(const u64 *c, u64 *__restrict__ msg1,
                                                              u64 *__restrict__ msg2, u64 *__restrict__ umsg,
                                                              u64 *__restrict__ wsh, u64 *out, u64 *__restrict__ rec,
                                                              size_t count, ss_dr_params dp, ss_tr_params tp,
                                                              ss_recf_params rf, ss_part_src ps)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    const int k = dp.t + 1, nr = 2 * dp.t + 1;

    // step 1 fused with the accumulation of step 2: coef[q][j] = sum_i msg1[i][q] * binv[i][j]
    ss_sacc coef[VEC][SS_MAXK][SS_MAXK];
#pragma unroll
    for (int u = 0; u < VEC; u++)
#pragma unroll
        for (int q = 0; q < SS_MAXK; q++)
#pragma unroll
            for (int j = 0; j < SS_MAXK; j++) coef[u][q][j].clear();
#pragma unroll
    for (int i = 0; i < 2 * SS_MAXT + 1; i++) {
        if (i < nr) {
            pack_t<VEC> ci;
            ci.load(c + (size_t)i * count + e0);
            for (int s = 1; s < ps.planes; s++) {
                pack_t<VEC> more;
                more.load(c + (size_t)s * ps.stride + (size_t)i * count + e0);
#pragma unroll
                for (int u = 0; u < VEC; u++) ci.v[u] = ss_add(ci.v[u], more.v[u]);
            }
            u64 r[VEC][SS_MAXT];
#pragma unroll
            for (int u = 0; u < VEC; u++) draw_coeffs<SS_MAXT>(r[u], dp.reshare_key[i], dp.t, e0 + u);
#pragma unroll
            for (int q = 0; q < SS_MAXK; q++) {
                if (q < k) {
                    pack_t<VEC> s;
#pragma unroll
                    for (int u = 0; u < VEC; u++) {
                        s.v[u] = ss_poly_eval<SS_MAXT>(ci.v[u], r[u], dp.t, q + 1);
#pragma unroll
                        for (int j = 0; j < SS_MAXK; j++)
                            if (j < k) coef[u][q][j].mac(s.v[u], dp.ibinv[i][j]);
                    }
                    s.store(msg1 + ((size_t)i * k + q) * count + e0);
                }
            }
        }
    }

    // rest of step 2, fused with the accumulation of step 3: red[m] = sum_q lambda_q msg2[q][m]
    ss_sacc red[VEC][SS_MAXN];
#pragma unroll
    for (int u = 0; u < VEC; u++)
#pragma unroll
        for (int m = 0; m < SS_MAXN; m++) red[u][m].clear();
#pragma unroll
    for (int q = 0; q < SS_MAXK; q++) {
        if (q < k) {
            u64 a0[VEC], cf[VEC][SS_MAXT];
#pragma unroll
            for (int u = 0; u < VEC; u++) {
                a0[u] = ss_mul(coef[u][q][0].value(), dp.dinv);
#pragma unroll
                for (int j = 1; j < SS_MAXK; j++) cf[u][j - 1] = (j < k) ? ss_mul(coef[u][q][j].value(), dp.dinv) : 0;
            }
#pragma unroll
            for (int m = 0; m < SS_MAXN; m++) {
                if (m < dp.n) {
                    pack_t<VEC> s;
#pragma unroll
                    for (int u = 0; u < VEC; u++) {
                        s.v[u] = ss_poly_eval<SS_MAXT>(a0[u], cf[u], dp.t, m + 1);
                        red[u][m].mac(s.v[u], dp.ilambda[q]);
                    }
                    s.store(msg2 + ((size_t)q * dp.n + m) * count + e0);
                }
            }
        }
    }

    // rest of step 3 and RERAND
    u64 z[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) draw_coeffs<SS_MAXT>(z[u], dp.zero_key, dp.t, e0 + u);
    pack_t<VEC> y[TRUNC ? SS_MAXK : 1];   // with TRUNC: the new shares of parties 1..k
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (m < dp.n) {
            pack_t<VEC> s;
#pragma unroll
            for (int u = 0; u < VEC; u++)
                s.v[u] = ss_add(red[u][m].value(), ss_poly_eval<SS_MAXT>(0, z[u], dp.t, m + 1));
            if (!TRUNC)
                s.store(out + (size_t)m * count + e0);
            else if (m < SS_MAXK)
                y[m] = s;
        }
    }
    if (TRUNC) truncate_steps<VEC>(y, umsg, wsh, out, count, e0, tp, rec, rf);
}

// ---- the same steps with n and t fixed at compile time ((k,n) = (2,3), (3,5)) ----
// Same messages, same outputs, fewer instructions:
//  * a party evaluates its polynomial at the consecutive points 1, 2, ... by
//    forward differences (one or two additions per point) instead of Horner
//    with a modular multiplication per coefficient;
//  * sums of value * small signed constant keep the value in two pieces of 31
//    and 30 bits and accumulate in signed 64-bit words (one multiply-add per
//    piece), with no case split on the sign of the constant;
//  * sums stay unreduced ("lazy", any 64-bit word of the right residue) until
//    a value is stored or multiplied.

// sum of v * c over at most 8 terms, v canonical given as v = w0 + w1 2^31 (w0 < 2^31), |c| < 2^26
struct ss_sacc2 {
    long long lo, hi;
    __device__ __forceinline__ void clear() { lo = 0; hi = 0; }
    __device__ __forceinline__ void mac(u32 w0, u32 w1, int c)
    {
        lo += (long long)(int)w0 * c;   // |sum| < 8 * 2^31 * 2^26 = 2^60
        hi += (long long)(int)w1 * c;
    }
    __device__ __forceinline__ u64 value() const
    {
#if defined(SS_FIELD_P45)
        // here |hi| < 2^43 (w1 < 2^14).  Offsets that are multiples of p make both words positive;
        // h 2^31 with h = a 2^14 + b: a 2^45 + b 2^31 = 55 a + b 2^31
        const u64 l = (u64)(lo + (long long)(SS_P << 16)), h = (u64)(hi + (long long)SS_P);   // < 2^62, < 2^46
        return ss_reduce(l + SS_PC * (h >> 14) + ((h & 0x3FFFull) << 31));
#else
        const u64 l = (u64)(lo + (long long)SS_P), h = (u64)(hi + (long long)SS_P);   // in (2^60, 2^62)
        // h 2^31 with 2^61 = 1: low 30 bits of h shifted, the rest wraps to weight 1
        return ss_reduce(l + ((h & 0x3FFFFFFFull) << 31) + (h >> 30));
#endif
    }
};
#define SS_SPLIT31(v, w0, w1) const u32 w0 = (u32)(v)&0x7FFFFFFFu, w1 = (u32)((v) >> 31)

// all steps for element e; the messages go to the workspace, the new shares (reduced and re-randomised, with
// TRUNC also truncated) come back in o[]
// (em, mcount: position and plane size of this element in the message buffers, which need not be e, count)
template <int N, int T, bool TRUNC>
__device__ __forceinline__ void reduce_truncate_fixed(size_t e, size_t count, size_t em, size_t mcount, const u64 *c,
                                                      u64 *__restrict__ msg1, u64 *__restrict__ msg2,
                                                      u64 *__restrict__ umsg, u64 *__restrict__ wsh,
                                                      const ss_dr_params &dp, const ss_tr_params &tp,
                                                      const ss_part_src &ps, u64 (&o)[N])
{
    constexpr int K = T + 1, NR = 2 * T + 1;
    const u64 counter = ss_counter(e);
    auto draw = [&](const u64 *keys, u64 (&r)[T]) {
#pragma unroll
        for (int j = 0; j < T; j++) r[j] = ss_draw_field_at(keys[j], counter);
    };

    // all incoming shares are requested at once
    u64 cin[NR];
#pragma unroll
    for (int i = 0; i < NR; i++) cin[i] = c[(size_t)i * count + e];
    for (int s = 1; s < ps.planes; s++) {   // the product as a sum of planes: one more round of loads per plane
        u64 more[NR];
#pragma unroll
        for (int i = 0; i < NR; i++) more[i] = c[(size_t)s * ps.stride + (size_t)i * count + e];
#pragma unroll
        for (int i = 0; i < NR; i++) cin[i] = ss_add(cin[i], more[i]);
    }

    // step 1, and of step 2 the sums coef[q][j] = sum_i msg1[i][q] * D binv[i][j]
    ss_sacc2 coef[K][K];
#pragma unroll
    for (int q = 0; q < K; q++)
#pragma unroll
        for (int j = 0; j < K; j++) coef[q][j].clear();
#pragma unroll
    for (int i = 0; i < NR; i++) {
        const u64 ci = cin[i];
        u64 r[T];
        draw(dp.reshare_key[i], r);
        eval_points<T, K>(ci, r, [&](int q, u64 v) {
            msg1[((size_t)i * K + q) * mcount + em] = v;
            SS_SPLIT31(v, w0, w1);
#pragma unroll
            for (int j = 0; j < K; j++) coef[q][j].mac(w0, w1, dp.ibinv[i][j]);
        });
    }

    // rest of step 2 (party q evaluates its polynomial at every party ID), and of step 3 the sums
    // red[m] = sum_q lambda_q msg2[q][m]
    ss_sacc2 red[N];
#pragma unroll
    for (int m = 0; m < N; m++) red[m].clear();
#pragma unroll
    for (int q = 0; q < K; q++) {
        const u64 a0 = ss_mul(coef[q][0].value(), dp.dinv);
        u64 cf[T];
#pragma unroll
        for (int j = 1; j < K; j++) cf[j - 1] = ss_mul(coef[q][j].value(), dp.dinv);
        eval_points<T, N>(a0, cf, [&](int m, u64 v) {
            msg2[((size_t)q * N + m) * mcount + em] = v;
            SS_SPLIT31(v, w0, w1);
            red[m].mac(w0, w1, dp.ilambda[q]);
        });
    }

    // rest of step 3 and RERAND
    u64 z[T], y[N];
    draw(dp.zero_key, z);
    eval_points<T, N>(0, z, [&](int m, u64 v) { y[m] = ss_add(red[m].value(), v); });
    if (!TRUNC) {
#pragma unroll
        for (int m = 0; m < N; m++) o[m] = y[m];
        return;
    }

    // truncation step 1 (parties 1..k mask their share) and the elite party's REC of x + alpha
    const u64 ev = mask_e(tp.e_key, e, tp.f);
    u64 ca[T], cw[T], cat[T];
    draw(tp.alpha_key, ca);
    ss_sacc2 acc;
    acc.clear();
    eval_points<T, K>(ev << tp.f, ca, [&](int q, u64 v) {
        const u64 um = ss_add(y[q], v);
        umsg[(size_t)q * mcount + em] = um;
        SS_SPLIT31(um, w0, w1);
        acc.mac(w0, w1, tp.ilambda[q]);
    });
    // step 2: shift and re-share; step 3: unmask
    const u64 w = shift_signed(acc.value(), tp.f);
    draw(tp.gen_key, cw);
    draw(tp.alphat_key, cat);
    u64 ws[N];
    eval_points<T, N>(w, cw, [&](int m, u64 v) {
        wsh[(size_t)m * mcount + em] = v;
        ws[m] = v;
    });
    eval_points<T, N>(SS_P - ev, cat, [&](int m, u64 v) { o[m] = ss_add(ws[m], v); });
}

template <int N, int T, bool TRUNC>
__global__ __launch_bounds__(BLOCK) void degree_reduce_fixed_kernel(const u64 *c, u64 *__restrict__ msg1,
                                                                    u64 *__restrict__ msg2, u64 *__restrict__ umsg,
                                                                    u64 *__restrict__ wsh, u64 *out,
                                                                    u64 *__restrict__ rec, size_t count,
                                                                    ss_dr_params dp, ss_tr_params tp, ss_recf_params rf,
                                                                    ss_part_src ps)
{
    const size_t e = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    if (e >= count) return;
    u64 o[N];
    reduce_truncate_fixed<N, T, TRUNC>(e, count, e, count, c, msg1, msg2, umsg, wsh, dp, tp, ps, o);
    ss_sacc2 racc;   // if asked for, REC of the result
    racc.clear();
#pragma unroll
    for (int m = 0; m < N; m++) {
        out[(size_t)m * count + e] = o[m];
        if (TRUNC && rec) {
            SS_SPLIT31(o[m], w0, w1);
            racc.mac(w0, w1, rf.coef[m]);
        }
    }
    if (TRUNC && rec) rec[e] = rf.dinv == 1 ? racc.value() : ss_mul(racc.value(), rf.dinv);
}

// ReLU under the multiplicative mask for one element (the three steps of relu_kernel below), n and t
// fixed: x[] the n shares, r[] the n output shares
template <int N, int T>
__device__ __forceinline__ void relu_fixed(const u64 (&x)[N], size_t em, size_t mcount, const u64 (&b)[2 * T + 1],
                                           const u64 (&bi)[N], u64 *__restrict__ msg, u64 *__restrict__ yplain,
                                           const ss_nl_params &np, u64 (&r)[N])
{
    constexpr int NR = 2 * T + 1;
    ss_sacc acc;
    acc.clear();
#pragma unroll
    for (int i = 0; i < NR; i++) {
        const u64 m = ss_mul(x[i], b[i]);
        msg[(size_t)i * mcount + em] = m;
        acc.mac(m, np.ilambda[i]);
    }
    const u64 v = np.dinv == 1 ? acc.value() : ss_mul(acc.value(), np.dinv);
    const u64 y = v <= (SS_P - 1) / 2 ? v : 0;
    yplain[em] = y;
#pragma unroll
    for (int m = 0; m < N; m++) r[m] = ss_mul(y, bi[m]);
}

// Linear - Truncation - NonLinear tail of a convolution layer in one launch (the order of Sec. VII-A):
// reduction + RERAND + truncation of the product shares c [n][B][C][HW], then ReLU under the mask, the
// result stored as shares and, if planes != nullptr, as channel-innermost limb planes for the next
// convolution.  One element per thread, lanes arranged as in the share + planes kernel (lane l: pixel l%16,
// channel 4 g + l/16 of the wave's group g).  The messages hold the values of the separate kernels, in the
// order of this kernel's threads (so that a wave writes 512 consecutive bytes of every message plane): the
// element of thread t of block (x, y) is at position (y gridDim.x + x) 256 + t of a plane of gridDim.x
// gridDim.y 256 positions.
template <int N, int T>
__global__ __launch_bounds__(BLOCK) void layer_tail_kernel(const u64 *c, u64 *__restrict__ msg1, u64 *__restrict__ msg2,
                                                           u64 *__restrict__ umsg, u64 *__restrict__ wsh,
                                                           u64 *__restrict__ rmsg, u64 *__restrict__ yplain,
                                                           const u64 *__restrict__ sh_b, const u64 *__restrict__ sh_bi,
                                                           u64 *out, signed char *__restrict__ planes, int B, int C, int HW,
                                                           size_t party_bytes, ss_dr_params dp, ss_tr_params tp,
                                                           ss_nl_params np, ss_part_src ps)
{
    const int lane = threadIdx.x & 63, r16 = lane & 15, j = lane >> 4;
    const int pix = blockIdx.x * 16 + r16, c0 = blockIdx.y * 16 + 4 * (threadIdx.x >> 6);
    const size_t count = (size_t)B * HW * C;
    if (planes && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < N)
        *reinterpret_cast<int4 *>(planes + threadIdx.x * party_bytes + SS_NLIMB * count) = make_int4(0, 0, 0, 0);
    u64 dig[N];
#pragma unroll
    for (int p = 0; p < N; p++) dig[p] = 0;
    // A lane past the last pixel repeats the last pixel of its channel: it loads, computes and stores the very
    // values of that element's own lane, which sits in the same wave (so also in place nothing is read after
    // it was overwritten), and its messages go to its own, otherwise unused position.  Without this a block
    // of one or two pixels leaves its waves with four or eight active lanes, and waves with so few lanes run
    // their 64-bit integer arithmetic almost twice as slowly as full ones (measured on MI355X).
    if (c0 + j < C) {
        const int px = min(pix, B * HW - 1);
        const int b = px / HW, hw = px - b * HW;
        const size_t e = ((size_t)b * C + (c0 + j)) * HW + hw;
        const size_t mcount = (size_t)gridDim.x * gridDim.y * BLOCK;
        const size_t em = ((size_t)blockIdx.y * gridDim.x + blockIdx.x) * BLOCK + threadIdx.x;
        u64 o[N], r[N];
        // the mask shares are requested before the reduction starts, so that they arrive while it computes
        u64 mb[2 * T + 1], mbi[N];
#pragma unroll
        for (int i = 0; i < 2 * T + 1; i++) mb[i] = sh_b[(size_t)i * count + e];
#pragma unroll
        for (int m = 0; m < N; m++) mbi[m] = sh_bi[(size_t)m * count + e];
        reduce_truncate_fixed<N, T, true>(e, count, em, mcount, c, msg1, msg2, umsg, wsh, dp, tp, ps, o);
        relu_fixed<N, T>(o, em, mcount, mb, mbi, rmsg, yplain, np, r);
#pragma unroll
        for (int p = 0; p < N; p++) {
            out[(size_t)p * count + e] = r[p];
            dig[p] = balanced_digits(r[p]);
        }
    }
    if (!planes) return;   // uniform
    // the four lanes of a pixel swap their digit words; the limb dwords go through LDS and leave as 16-byte
    // stores of the block's 16 channels (see store_staged_planes)
    __shared__ __align__(16) u32 stage[N][SS_NLIMB][16][4];   // [party][limb][pixel][wave]
    const int w = threadIdx.x >> 6;
#pragma unroll
    for (int p = 0; p < N; p++) {
        u64 y[4];
#pragma unroll
        for (int q = 0; q < 4; q++) y[q] = __shfl(dig[p], r16 + 16 * q);
        if (2 * j < SS_NLIMB) {
            stage[p][2 * j][r16][w] = limb_dword(y, 2 * j);
            stage[p][2 * j + 1][r16][w] = limb_dword(y, 2 * j + 1);
        }
    }
    __syncthreads();
    store_staged_planes<N>(stage, planes, party_bytes, count, blockIdx.x * 16, B * HW, C, blockIdx.y * 16, N);
}

// The outputs of the layer tail without the protocol (all parties on one device): as for
// reduce_truncate_direct_kernel, what the parties end up with follows from the secret of the incoming
// degree-2t sharing.  x = REC of the 2t+1 product shares; the truncated value is floor(x / 2^f) on the signed
// value whatever the mask was; the elite party of the ReLU sees floor(x / 2^f) * beta, beta = REC of its k
// shares; every party's output is max(., 0) times its share of beta^-1.  Same residues in `out` and in the limb
// planes as layer_tail_kernel; no message is formed.  Lanes as in that kernel (pixel l%16, channel 4 g + l/16),
// so that the planes leave through the same staged 16-byte stores.
__global__ __launch_bounds__(BLOCK) void tail_direct_kernel(const u64 *c, const u64 *__restrict__ sh_b,
                                                            const u64 *__restrict__ sh_bi, u64 *out,
                                                            signed char *__restrict__ planes, int B, int C, int HW,
                                                            size_t party_bytes, ss_nl_params open_all, ss_tr_params tp,
                                                            ss_part_src ps)
{
    const int lane = threadIdx.x & 63, r16 = lane & 15, j = lane >> 4;
    const int pix = blockIdx.x * 16 + r16, c0 = blockIdx.y * 16 + 4 * (threadIdx.x >> 6);
    const size_t count = (size_t)B * HW * C;
    const int n = tp.n, k = tp.t + 1, nr = 2 * tp.t + 1;
    if (planes && blockIdx.x == 0 && blockIdx.y == 0 && (int)threadIdx.x < n)
        *reinterpret_cast<int4 *>(planes + threadIdx.x * party_bytes + SS_NLIMB * count) = make_int4(0, 0, 0, 0);
    u64 dig[SS_MAXN];
#pragma unroll
    for (int p = 0; p < SS_MAXN; p++) dig[p] = 0;
    if (pix < B * HW && c0 + j < C) {
        const int b = pix / HW, hw = pix - b * HW;
        const size_t e = ((size_t)b * C + (c0 + j)) * HW + hw;
        ss_sacc acc, bacc;
        acc.clear();
        bacc.clear();
#pragma unroll
        for (int i = 0; i < 2 * SS_MAXT + 1; i++)
            if (i < nr) acc.mac(load_product(c, (size_t)i * count + e, ps), open_all.ilambda[i]);
#pragma unroll
        for (int q = 0; q < SS_MAXK; q++)
            if (q < k) bacc.mac(sh_b[(size_t)q * count + e], tp.ilambda[q]);
        const u64 x = open_all.dinv == 1 ? acc.value() : ss_mul(acc.value(), open_all.dinv);
        const u64 v = ss_mul(shift_signed(x, tp.f), bacc.value());   // the multipliers of IDs 1..k are integers
        const u64 y = v <= (SS_P - 1) / 2 ? v : 0;
#pragma unroll
        for (int m = 0; m < SS_MAXN; m++) {
            if (m < n) {
                const u64 r = ss_mul(y, sh_bi[(size_t)m * count + e]);
                out[(size_t)m * count + e] = r;
                dig[m] = balanced_digits(r);
            }
        }
    }
    if (!planes) return;   // uniform
    __shared__ __align__(16) u32 stage[SS_MAXN][SS_NLIMB][16][4];   // [party][limb][pixel][wave]
    const int w = threadIdx.x >> 6;
#pragma unroll
    for (int p = 0; p < SS_MAXN; p++) {
        if (p < n) {
            u64 y4[4];
#pragma unroll
            for (int q = 0; q < 4; q++) y4[q] = __shfl(dig[p], r16 + 16 * q);
            if (2 * j < SS_NLIMB) {
                stage[p][2 * j][r16][w] = limb_dword(y4, 2 * j);
                stage[p][2 * j + 1][r16][w] = limb_dword(y4, 2 * j + 1);
            }
        }
    }
    __syncthreads();
    store_staged_planes<SS_MAXN>(stage, planes, party_bytes, count, blockIdx.x * 16, B * HW, C, blockIdx.y * 16, n);
}

// Same computation for small tensors, where the serial work of one thread per
// element leaves most of the chip idle: a workgroup takes 32 elements and eight
// party lanes per element.  Lane p first plays reducing party p+1 (step 1),
// while the lanes that do not reduce (2t+1 <= 7, so lane 7 at least) draw the
// coefficients every party needs later; then, after these went through LDS, lane
// p plays receiving party p+1: it forms the k values that parties 1..k would
// send it (step 2, with the full matrix R instead of its factors, so that the
// lanes do not wait on each other) and reconstructs from them (step 3, RERAND).
// With TRUNC the lanes go on with the truncation steps (mask, reconstruct and
// shift at the elite party, unmask), exchanging the k masked shares through LDS.
// Messages and outputs are the same residues as in the kernels above.
template <bool TRUNC>
__global__ __launch_bounds__(BLOCK) void degree_reduce_lanes_kernel(const u64 *c, u64 *__restrict__ msg1,
                                                                    u64 *__restrict__ msg2, u64 *__restrict__ umsg,
                                                                    u64 *__restrict__ wsh, u64 *out,
                                                                    u64 *__restrict__ rec, size_t count,
                                                                    ss_dr_params dp, ss_tr_params tp, ss_recf_params rf,
                                                                    ss_part_src ps)
{
    __shared__ u64 sub[2 * SS_MAXT + 1][SS_MAXK][32];
    // drawn once per element by the spare lanes: 0 zero sharing, 1 alpha, 2 elite re-sharing, 3 alpha~
    __shared__ u64 coef[4][SS_MAXT][32];
    __shared__ u64 mask[32];             // e of the truncation mask
    __shared__ u64 masked[SS_MAXK][32];  // x_q + alpha_q
    __shared__ u64 fin[SS_MAXN][32];     // truncated shares, for the fused REC
    const int el = threadIdx.x & 31, p = threadIdx.x >> 5;
    const size_t e = (size_t)blockIdx.x * 32 + el;
    const bool live = e < count;
    const int k = dp.t + 1, nr = 2 * dp.t + 1;
    if (live && p < nr) {
        const u64 ci = load_product(c, (size_t)p * count + e, ps);
        u64 r[SS_MAXT];
        draw_coeffs<SS_MAXT>(r, dp.reshare_key[p], dp.t, e);
#pragma unroll
        for (int q = 0; q < SS_MAXK; q++) {
            if (q < k) {
                const u64 v = ss_poly_eval<SS_MAXT>(ci, r, dp.t, q + 1);
                sub[p][q][el] = v;
                msg1[((size_t)p * k + q) * count + e] = v;
            }
        }
    } else if (live) {   // spare lanes nr..7 share the drawing jobs round-robin
        const int spare = 8 - nr, me = p - nr;
#pragma unroll
        for (int job = 0; job < (TRUNC ? 4 : 1); job++) {
            if (job % spare == me) {
                const u64 *keys = job == 0 ? dp.zero_key : job == 1 ? tp.alpha_key : job == 2 ? tp.gen_key : tp.alphat_key;
                u64 z[SS_MAXT];
                draw_coeffs<SS_MAXT>(z, keys, dp.t, e);
#pragma unroll
                for (int j = 0; j < SS_MAXT; j++) coef[job][j][el] = z[j];
                if (job == 1) mask[el] = mask_e(tp.e_key, e, tp.f);
            }
        }
    }
    __syncthreads();
    const bool party = live && p < dp.n;
    u64 y = 0;   // this party's reduced, re-randomised share
    if (party) {
        ss_sacc red;
        red.clear();
#pragma unroll
        for (int q = 0; q < SS_MAXK; q++) {
            if (q < k) {
                ss_sacc acc;
                acc.clear();
#pragma unroll
                for (int i = 0; i < 2 * SS_MAXT + 1; i++)
                    if (i < nr) acc.mac(sub[i][q][el], dp.irmat[i][p]);
                const u64 v = ss_mul(acc.value(), dp.dinv);
                msg2[((size_t)q * dp.n + p) * count + e] = v;
                red.mac(v, dp.ilambda[q]);
            }
        }
        u64 z[SS_MAXT];
#pragma unroll
        for (int j = 0; j < SS_MAXT; j++) z[j] = coef[0][j][el];
        y = ss_add(red.value(), ss_poly_eval<SS_MAXT>(0, z, dp.t, p + 1));
        if (!TRUNC) out[(size_t)p * count + e] = y;
    }
    if (!TRUNC) return;

    if (party && p < k) {   // truncation step 1 on parties 1..k
        u64 ca[SS_MAXT];
#pragma unroll
        for (int j = 0; j < SS_MAXT; j++) ca[j] = coef[1][j][el];
        const u64 um = ss_add(y, ss_poly_eval<SS_MAXT>(mask[el] << tp.f, ca, tp.t, p + 1));
        masked[p][el] = um;
        umsg[(size_t)p * count + e] = um;
    }
    __syncthreads();
    if (party) {   // step 2 (the elite party's result, recomputed by every lane) and step 3
        ss_sacc acc;
        acc.clear();
#pragma unroll
        for (int q = 0; q < SS_MAXK; q++)
            if (q < k) acc.mac(masked[q][el], tp.ilambda[q]);
        const u64 w = shift_signed(acc.value(), tp.f);
        u64 cw[SS_MAXT], cat[SS_MAXT];
#pragma unroll
        for (int j = 0; j < SS_MAXT; j++) {
            cw[j] = coef[2][j][el];
            cat[j] = coef[3][j][el];
        }
        const u64 ws = ss_poly_eval<SS_MAXT>(w, cw, tp.t, p + 1);
        wsh[(size_t)p * count + e] = ws;
        const u64 o = ss_add(ws, ss_poly_eval<SS_MAXT>(SS_P - mask[el], cat, tp.t, p + 1));
        out[(size_t)p * count + e] = o;
        fin[p][el] = o;
    }
    if (!rec) return;   // uniform over the grid
    __syncthreads();
    if (live && p == 0) {
        ss_sacc acc;
        acc.clear();
#pragma unroll
        for (int m = 0; m < SS_MAXN; m++)
            if (m < dp.n && rf.coef[m] != 0) acc.mac(fin[m][el], rf.coef[m]);
        rec[e] = rf.dinv == 1 ? acc.value() : ss_mul(acc.value(), rf.dinv);
    }
}

// ------------------------------------------------------------------ reduction + truncation, all parties at once
// The outputs of RED + RERAND + truncation do not depend on the reshare or zero
// randomness: the elite party of the truncation reconstructs x + alpha, where x
// is the secret of the incoming degree-2t sharing, whatever the reduced shares
// look like.  With every party's share in one thread that secret can be taken
// directly (REC from the 2t+1 incoming shares), and the output shares follow from
// it as in truncation steps 2 and 3.  Same residues in `out` (and `rec`) as the
// protocol kernels; no message is formed, so this is not what the parties of the
// protocol compute, only what they end up with.
template <int VEC>
__global__ __launch_bounds__(BLOCK) void reduce_truncate_direct_kernel(const u64 *c, u64 *out, u64 *__restrict__ rec,
                                                                       size_t count, ss_nl_params open_all,
                                                                       ss_tr_params tp, ss_recf_params rf)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    const int nr = 2 * tp.t + 1;
    ss_sacc acc[VEC], racc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        acc[u].clear();
        racc[u].clear();
    }
#pragma unroll
    for (int i = 0; i < 2 * SS_MAXT + 1; i++) {
        if (i < nr) {
            pack_t<VEC> ci;
            ci.load(c + (size_t)i * count + e0);
#pragma unroll
            for (int u = 0; u < VEC; u++) acc[u].mac(ci.v[u], open_all.ilambda[i]);
        }
    }
    u64 w[VEC], at[VEC], cw[VEC][SS_MAXT], cat[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        const u64 x = open_all.dinv == 1 ? acc[u].value() : ss_mul(acc[u].value(), open_all.dinv);
        const u64 ev = mask_e(tp.e_key, e0 + u, tp.f);
        w[u] = shift_signed(ss_add(x, ev << tp.f), tp.f);
        at[u] = SS_P - ev;
        draw_coeffs<SS_MAXT>(cw[u], tp.gen_key, tp.t, e0 + u);
        draw_coeffs<SS_MAXT>(cat[u], tp.alphat_key, tp.t, e0 + u);
    }
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (m < tp.n) {
            pack_t<VEC> s;
#pragma unroll
            for (int u = 0; u < VEC; u++) {
                s.v[u] = ss_add(ss_poly_eval<SS_MAXT>(w[u], cw[u], tp.t, m + 1),
                                ss_poly_eval<SS_MAXT>(at[u], cat[u], tp.t, m + 1));
                if (rec && rf.coef[m] != 0) racc[u].mac(s.v[u], rf.coef[m]);
            }
            s.store(out + (size_t)m * count + e0);
        }
    }
    if (rec) {
        pack_t<VEC> r;
#pragma unroll
        for (int u = 0; u < VEC; u++) r.v[u] = rf.dinv == 1 ? racc[u].value() : ss_mul(racc[u].value(), rf.dinv);
        r.store(rec + e0);
    }
}

// ------------------------------------------------------------------ SSS-NonLinear (Sec. VI-C)
// What the trusted source prepares ahead of the inference (Sec. VII-B): a positive
// mask beta per element, its inverse in F_p (Fermat: beta^(p-2), p - 2 = 2^61 - 3)
// and a degree-t sharing of each.  One thread per element.
__device__ __forceinline__ u64 mask_beta(const ss_nl_params &np, u64 counter)
{
    return 1 + ((ss_draw(np.beta_key, counter) >> 3) & ((1ULL << np.bbits) - 1));
}

__device__ __forceinline__ u64 field_inverse(u64 beta)
{
#if defined(SS_FIELD_P45)
    // beta^(p - 2), p - 2 = 2^45 - 57: square and multiply from the top bit down
    u64 inv = beta;
    for (int bit = SS_PBITS - 2; bit >= 0; bit--) {
        inv = ss_mul(inv, inv);
        if (((SS_P - 2) >> bit) & 1) inv = ss_mul(inv, beta);
    }
    return inv;
#else
    // beta^(2^61 - 3): the exponent is 59 one bits, then 0, then 1
    u64 inv = beta;
    for (int i = 0; i < 58; i++) inv = ss_mul(ss_mul(inv, inv), beta);   // beta^(2^59 - 1)
    inv = ss_mul(inv, inv);                                              // bit 1 of the exponent is 0
    return ss_mul(ss_mul(inv, inv), beta);                               // bit 0 is 1
#endif
}

__global__ __launch_bounds__(BLOCK) void nonlinear_masks_kernel(u64 *__restrict__ sh_b, u64 *__restrict__ sh_bi,
                                                                size_t count, ss_nl_params np)
{
    const size_t e = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    if (e >= count) return;
    const u64 beta = mask_beta(np, e);
    const u64 inv = field_inverse(beta);
    u64 cb[SS_MAXT], cbi[SS_MAXT];
    draw_coeffs<SS_MAXT>(cb, np.bgen_key, np.t, e);
    draw_coeffs<SS_MAXT>(cbi, np.bigen_key, np.t, e);
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (m < np.n) {
            sh_b[(size_t)m * count + e] = ss_poly_eval<SS_MAXT>(beta, cb, np.t, m + 1);
            sh_bi[(size_t)m * count + e] = ss_poly_eval<SS_MAXT>(inv, cbi, np.t, m + 1);
        }
    }
}

// ReLU on shares, the three steps for the elements a thread owns (send = store
// to the workspace, receive = from registers, as in the kernels above):
//   1. parties 1..2t+1: m_i = x_i * beta_i                          -> msg[i]
//   2. elite party: REC of the 2t+1 products = x * beta; ReLU on the
//      signed value, in the clear                                   -> yplain
//   3. every party: out_i = y * betainv_i                            -> out[i]
// MASKOFF = false stops after step 2 (the pooled form continues from yplain in another kernel).
template <int VEC, bool MASKOFF = true>
__global__ __launch_bounds__(BLOCK) void relu_kernel(const u64 *x, const u64 *__restrict__ sh_b,
                                                     const u64 *__restrict__ sh_bi, u64 *__restrict__ msg,
                                                     u64 *__restrict__ yplain, u64 *out, size_t count,
                                                     ss_nl_params np)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    const int nr = 2 * np.t + 1;
    // all operands are requested up front, so that the three steps wait for memory once
    pack_t<VEC> xi[2 * SS_MAXT + 1], bi[2 * SS_MAXT + 1], binv[SS_MAXN];
#pragma unroll
    for (int i = 0; i < 2 * SS_MAXT + 1; i++) {
        if (i < nr) {
            xi[i].load(x + (size_t)i * count + e0);
            bi[i].load(sh_b + (size_t)i * count + e0);
        }
    }
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++)
        if (MASKOFF && m < np.n) binv[m].load(sh_bi + (size_t)m * count + e0);
    ss_sacc acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; u++) acc[u].clear();
#pragma unroll
    for (int i = 0; i < 2 * SS_MAXT + 1; i++) {
        if (i < nr) {
            pack_t<VEC> m;
#pragma unroll
            for (int u = 0; u < VEC; u++) {
                m.v[u] = ss_mul(xi[i].v[u], bi[i].v[u]);
                acc[u].mac(m.v[u], np.ilambda[i]);
            }
            m.store(msg + (size_t)i * count + e0);
        }
    }
    pack_t<VEC> y;
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        const u64 v = np.dinv == 1 ? acc[u].value() : ss_mul(acc[u].value(), np.dinv);
        y.v[u] = v <= (SS_P - 1) / 2 ? v : 0;   // negative values are the upper half of the field
    }
    y.store(yplain + e0);
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (MASKOFF && m < np.n) {
            pack_t<VEC> o;
#pragma unroll
            for (int u = 0; u < VEC; u++) o.v[u] = ss_mul(y.v[u], binv[m].v[u]);
            o.store(out + (size_t)m * count + e0);
        }
    }
}

// Masks for ReLU followed by pooling: beta has to be equal inside one pooling kernel.  Where the kernels
// partition the plane a group is a kernel position (elements beyond the last full kernel join the last
// one), otherwise the whole plane; beta is drawn at counter = group index.  The sharing coefficients are
// drawn per element.  INV = false: one thread per input element, shares of beta; INV = true: one thread per
// pooled element, shares of beta^-1 of its kernel's group.
template <bool INV>
__global__ __launch_bounds__(BLOCK) void pool_masks_kernel(u64 *__restrict__ sh, size_t count, ss_pool_geom g,
                                                           ss_nl_params np)
{
    const size_t e = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    if (e >= count) return;
    const int w = INV ? g.Wo : g.W, h = INV ? g.Ho : g.H;
    const size_t plane = e / ((size_t)h * w);
    const int r = (int)(e - plane * (size_t)h * w), row = r / w, col = r - row * w;
    u64 group = plane;
    if (g.tiled) {
        const int oh = INV ? row : min(row / g.kh, g.Ho - 1), ow = INV ? col : min(col / g.kw, g.Wo - 1);
        group = (plane * g.Ho + oh) * g.Wo + ow;
    }
    u64 secret = mask_beta(np, group);
    if (INV) secret = field_inverse(secret);
    u64 cf[SS_MAXT];
    draw_coeffs<SS_MAXT>(cf, INV ? np.bigen_key : np.bgen_key, np.t, e);
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++)
        if (m < np.n) sh[(size_t)m * count + e] = ss_poly_eval<SS_MAXT>(secret, cf, np.t, m + 1);
}

// Pooling in the elite party's plain part of SSS-NonLinear and the mask-off (step 3), one thread per
// pooled element: the maximum or the sum of the opened, rectified products r = max(x*beta, 0) over the
// kernel's elements inside the plane (padding adds nothing to a sum and cannot win a maximum of
// non-negative values), then y * betainv_m for every party.
__global__ __launch_bounds__(BLOCK) void pool_maskoff_kernel(const u64 *__restrict__ rplain,
                                                             const u64 *__restrict__ sh_bi, u64 *__restrict__ yplain,
                                                             u64 *__restrict__ out, size_t count, ss_pool_geom g, int n)
{
    const size_t o = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    if (o >= count) return;
    const size_t plane = o / ((size_t)g.Ho * g.Wo);
    const int r = (int)(o - plane * (size_t)g.Ho * g.Wo), oh = r / g.Wo, ow = r - oh * g.Wo;
    const u64 *src = rplain + plane * (size_t)g.H * g.W;
    const int h0 = oh * g.sh - g.ph, w0 = ow * g.sw - g.pw;
    u64 acc = 0;
    for (int i = max(0, -h0); i < min(g.kh, g.H - h0); i++)
        for (int j = max(0, -w0); j < min(g.kw, g.W - w0); j++) {
            const u64 v = src[(size_t)(h0 + i) * g.W + (w0 + j)];
            acc = g.mode == 0 ? (v > acc ? v : acc) : ss_add(acc, v);
        }
    yplain[o] = acc;
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++)
        if (m < n) out[(size_t)m * count + o] = ss_mul(acc, sh_bi[(size_t)m * count + o]);
}

// below this many elements one element per thread gives more waves to hide latency
constexpr size_t VEC2_MIN_COUNT = (size_t)1 << 20;
// below this many elements degree reduction spreads an element over party lanes
constexpr size_t LANES_MAX_COUNT = 160 * 1024;   // measured cross-over on MI355X (n = 5, t = 2)
// the same cross-over against the kernels with n and t fixed at compile time
constexpr size_t LANES_MAX_COUNT_FIXED = 8 * 1024;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

inline unsigned blocks_for(size_t count, int vec)
{
    const size_t per_block = (size_t)BLOCK * vec;
    return (unsigned)((count + per_block - 1) / per_block);
}

}  // namespace

// The two-element path needs every plane start 16-byte aligned: aligned bases
// and an even element count.
#define SS_DISPATCH_VEC(cond, KERNEL, grid, ...)                                          \
    do {                                                                                  \
        if (cond)                                                                         \
            hipLaunchKernelGGL(KERNEL<2>, grid(2), dim3(BLOCK), 0, stream, __VA_ARGS__);  \
        else                                                                              \
            hipLaunchKernelGGL(KERNEL<1>, grid(1), dim3(BLOCK), 0, stream, __VA_ARGS__);  \
    } while (0)

hipError_t ss_launch_share(const u64 *secret, u64 *shares, size_t count, int n, int degree, const ss_keys &keys,
                           hipStream_t stream)
{
    const bool v2 = (count % 2 == 0) && aligned16(secret) && aligned16(shares);
    const dim3 grid(blocks_for(count, v2 ? 2 : 1)), block(BLOCK);
#define SS_SHARE(VEC, NC, DC) \
    hipLaunchKernelGGL((share_kernel<VEC, NC, DC>), grid, block, 0, stream, secret, shares, count, n, degree, keys)
    if (v2 && n == 5 && degree == 2)
        SS_SHARE(2, 5, 2);
    else if (v2 && n == 3 && degree == 1)
        SS_SHARE(2, 3, 1);
    else if (v2)
        SS_SHARE(2, 0, 0);
    else
        SS_SHARE(1, 0, 0);
#undef SS_SHARE
    return hipGetLastError();
}

hipError_t ss_launch_reconstruct(const u64 *shares, u64 *secret, size_t count, const ss_rec_params &rp,
                                 hipStream_t stream)
{
    const bool v2 = (count % 2 == 0) && aligned16(secret) && aligned16(shares);
    auto grid = [&](int vec) { return dim3(blocks_for(count, vec)); };
    SS_DISPATCH_VEC(v2, reconstruct_kernel, grid, shares, secret, count, rp);
    return hipGetLastError();
}

// sum of the product's planes, written to dst (which may be the first plane: each thread reads its element
// of every plane before it writes)
__global__ __launch_bounds__(BLOCK) void sum_planes_kernel(u64 *dst, const u64 *c, size_t total, ss_part_src ps)
{
    const size_t i = (size_t)blockIdx.x * BLOCK + threadIdx.x;
    if (i < total) dst[i] = load_product(c, i, ps);
}

hipError_t ss_launch_sum_planes(u64 *dst, const u64 *c, size_t total, const ss_part_src &ps, hipStream_t stream)
{
    if (ps.planes > 1 || dst != c)
        hipLaunchKernelGGL(sum_planes_kernel, dim3(blocks_for(total, 1)), dim3(BLOCK), 0, stream, dst, c, total, ps);
    return hipGetLastError();
}

hipError_t ss_launch_degree_reduce(const u64 *c, u64 *msg1, u64 *msg2, u64 *out, size_t count,
                                   const ss_dr_params &dp, const ss_part_src &ps, hipStream_t stream)
{
    const ss_tr_params none = {};
    const ss_recf_params norec = {};
    const bool fixed = (dp.n == 5 && dp.t == 2) || (dp.n == 3 && dp.t == 1);
    if (count < (fixed ? LANES_MAX_COUNT_FIXED : LANES_MAX_COUNT))
        hipLaunchKernelGGL(degree_reduce_lanes_kernel<false>, dim3((unsigned)((count + 31) / 32)), dim3(BLOCK), 0, stream,
                           c, msg1, msg2, (u64 *)nullptr, (u64 *)nullptr, out, (u64 *)nullptr, count, dp, none, norec, ps);
    else if (dp.n == 5 && dp.t == 2)
        hipLaunchKernelGGL((degree_reduce_fixed_kernel<5, 2, false>), dim3(blocks_for(count, 1)), dim3(BLOCK), 0, stream, c,
                           msg1, msg2, (u64 *)nullptr, (u64 *)nullptr, out, (u64 *)nullptr, count, dp, none, norec, ps);
    else if (dp.n == 3 && dp.t == 1)
        hipLaunchKernelGGL((degree_reduce_fixed_kernel<3, 1, false>), dim3(blocks_for(count, 1)), dim3(BLOCK), 0, stream, c,
                           msg1, msg2, (u64 *)nullptr, (u64 *)nullptr, out, (u64 *)nullptr, count, dp, none, norec, ps);
    else   // one element per thread: the k*k + n wide accumulators of two elements would not fit the register file
        hipLaunchKernelGGL((degree_reduce_kernel<1, false>), dim3(blocks_for(count, 1)), dim3(BLOCK), 0, stream, c, msg1,
                           msg2, (u64 *)nullptr, (u64 *)nullptr, out, (u64 *)nullptr, count, dp, none, norec, ps);
    return hipGetLastError();
}

hipError_t ss_launch_degree_reduce_truncate(const u64 *c, u64 *msg1, u64 *msg2, u64 *u, u64 *wsh, u64 *out,
                                            u64 *rec, size_t count, const ss_dr_params &dp, const ss_tr_params &tp,
                                            const ss_recf_params &rf, const ss_part_src &ps, hipStream_t stream)
{
    const bool fixed = (dp.n == 5 && dp.t == 2) || (dp.n == 3 && dp.t == 1);
    if (tp.kdiv > 1)   // the rounding division exists in the general kernel only
        hipLaunchKernelGGL((degree_reduce_kernel<1, true>), dim3(blocks_for(count, 1)), dim3(BLOCK), 0, stream, c, msg1,
                           msg2, u, wsh, out, rec, count, dp, tp, rf, ps);
    else if (count < (fixed ? LANES_MAX_COUNT_FIXED : LANES_MAX_COUNT))
        hipLaunchKernelGGL(degree_reduce_lanes_kernel<true>, dim3((unsigned)((count + 31) / 32)), dim3(BLOCK), 0, stream,
                           c, msg1, msg2, u, wsh, out, rec, count, dp, tp, rf, ps);
    else if (dp.n == 5 && dp.t == 2)
        hipLaunchKernelGGL((degree_reduce_fixed_kernel<5, 2, true>), dim3(blocks_for(count, 1)), dim3(BLOCK), 0, stream, c,
                           msg1, msg2, u, wsh, out, rec, count, dp, tp, rf, ps);
    else if (dp.n == 3 && dp.t == 1)
        hipLaunchKernelGGL((degree_reduce_fixed_kernel<3, 1, true>), dim3(blocks_for(count, 1)), dim3(BLOCK), 0, stream, c,
                           msg1, msg2, u, wsh, out, rec, count, dp, tp, rf, ps);
    else
        hipLaunchKernelGGL((degree_reduce_kernel<1, true>), dim3(blocks_for(count, 1)), dim3(BLOCK), 0, stream, c, msg1,
                           msg2, u, wsh, out, rec, count, dp, tp, rf, ps);
    return hipGetLastError();
}

hipError_t ss_launch_truncate(const u64 *x, u64 *u, u64 *wsh, u64 *out, size_t count, const ss_tr_params &tp,
                              hipStream_t stream)
{
    const bool v2 = (count % 2 == 0) && aligned16(x) && aligned16(u) && aligned16(wsh) && aligned16(out) &&
                    count >= VEC2_MIN_COUNT;
    auto grid = [&](int vec) { return dim3(blocks_for(count, vec)); };
    SS_DISPATCH_VEC(v2, truncate_kernel, grid, x, u, wsh, out, count, tp);
    return hipGetLastError();
}

hipError_t ss_launch_nonlinear_masks(u64 *sh_b, u64 *sh_bi, size_t count, const ss_nl_params &np, hipStream_t stream)
{
    hipLaunchKernelGGL(nonlinear_masks_kernel, dim3(blocks_for(count, 1)), dim3(BLOCK), 0, stream, sh_b, sh_bi, count,
                       np);
    return hipGetLastError();
}

hipError_t ss_launch_relu(const u64 *x, const u64 *sh_b, const u64 *sh_bi, u64 *msg, u64 *yplain, u64 *out,
                          size_t count, const ss_nl_params &np, hipStream_t stream)
{
    const bool v2 = (count % 2 == 0) && aligned16(x) && aligned16(sh_b) && aligned16(sh_bi) && aligned16(msg) &&
                    aligned16(yplain) && aligned16(out) && count >= VEC2_MIN_COUNT;
    auto grid = [&](int vec) { return dim3(blocks_for(count, vec)); };
    SS_DISPATCH_VEC(v2, relu_kernel, grid, x, sh_b, sh_bi, msg, yplain, out, count, np);
    return hipGetLastError();
}

hipError_t ss_launch_pool_masks(u64 *sh_b, u64 *sh_bi, size_t planes, const ss_pool_geom &g, const ss_nl_params &np,
                                hipStream_t stream)
{
    const size_t cin = planes * g.H * g.W, cout = planes * g.Ho * g.Wo;
    hipLaunchKernelGGL(pool_masks_kernel<false>, dim3(blocks_for(cin, 1)), dim3(BLOCK), 0, stream, sh_b, cin, g, np);
    hipLaunchKernelGGL(pool_masks_kernel<true>, dim3(blocks_for(cout, 1)), dim3(BLOCK), 0, stream, sh_bi, cout, g, np);
    return hipGetLastError();
}

hipError_t ss_launch_relu_pool(const u64 *x, const u64 *sh_b, const u64 *sh_bi, u64 *msg, u64 *rplain, u64 *yplain,
                               u64 *out, size_t planes, const ss_pool_geom &g, const ss_nl_params &np,
                               hipStream_t stream)
{
    const size_t cin = planes * g.H * g.W, cout = planes * g.Ho * g.Wo;
    hipLaunchKernelGGL((relu_kernel<1, false>), dim3(blocks_for(cin, 1)), dim3(BLOCK), 0, stream, x, sh_b,
                       (const u64 *)nullptr, msg, rplain, (u64 *)nullptr, cin, np);
    hipLaunchKernelGGL(pool_maskoff_kernel, dim3(blocks_for(cout, 1)), dim3(BLOCK), 0, stream, rplain, sh_bi, yplain, out,
                       cout, g, np.n);
    return hipGetLastError();
}

hipError_t ss_launch_reduce_truncate_direct(const u64 *c, u64 *out, u64 *rec, size_t count, const ss_nl_params &open_all,
                                            const ss_tr_params &tp, const ss_recf_params &rf, hipStream_t stream)
{
    if (tp.kdiv != 1) return hipErrorInvalidValue;   // no rounding division in this kernel
    const bool v2 = (count % 2 == 0) && aligned16(c) && aligned16(out) && (!rec || aligned16(rec)) &&
                    count >= VEC2_MIN_COUNT;
    auto grid = [&](int vec) { return dim3(blocks_for(count, vec)); };
    SS_DISPATCH_VEC(v2, reduce_truncate_direct_kernel, grid, c, out, rec, count, open_all, tp, rf);
    return hipGetLastError();
}

hipError_t ss_launch_tail_direct(const u64 *c, const u64 *sh_b, const u64 *sh_bi, u64 *out, void *planes, int B, int C,
                                 int HW, const ss_nl_params &open_all, const ss_tr_params &tp, const ss_part_src &ps,
                                 hipStream_t stream)
{
    if (tp.kdiv != 1) return hipErrorInvalidValue;   // no rounding division in this kernel
    const dim3 grid((B * HW + 15) / 16, (C + 15) / 16), block(BLOCK);
    hipLaunchKernelGGL(tail_direct_kernel, grid, block, 0, stream, c, sh_b, sh_bi, out, (signed char *)planes, B, C, HW,
                       ss_planes_bytes(B, C, HW, 1), open_all, tp, ps);
    return hipGetLastError();
}

hipError_t ss_launch_layer_tail(const u64 *c, u64 *msg1, u64 *msg2, u64 *umsg, u64 *wsh, u64 *rmsg, u64 *yplain,
                                const u64 *sh_b, const u64 *sh_bi, u64 *out, void *planes, int B, int C, int HW,
                                const ss_dr_params &dp, const ss_tr_params &tp, const ss_nl_params &np,
                                const ss_part_src &ps, hipStream_t stream)
{
    if (tp.kdiv != 1) return hipErrorInvalidValue;   // no rounding division in this kernel
    const dim3 grid((B * HW + 15) / 16, (C + 15) / 16), block(BLOCK);
    const size_t party_bytes = ss_planes_bytes(B, C, HW, 1);
    if (dp.n == 5 && dp.t == 2)
        hipLaunchKernelGGL((layer_tail_kernel<5, 2>), grid, block, 0, stream, c, msg1, msg2, umsg, wsh, rmsg, yplain, sh_b,
                           sh_bi, out, (signed char *)planes, B, C, HW, party_bytes, dp, tp, np, ps);
    else if (dp.n == 3 && dp.t == 1)
        hipLaunchKernelGGL((layer_tail_kernel<3, 1>), grid, block, 0, stream, c, msg1, msg2, umsg, wsh, rmsg, yplain, sh_b,
                           sh_bi, out, (signed char *)planes, B, C, HW, party_bytes, dp, tp, np, ps);
    else
        return hipErrorInvalidValue;   // the caller runs the separate kernels for other schemes
    return hipGetLastError();
}

}  // namespace SS_NS
