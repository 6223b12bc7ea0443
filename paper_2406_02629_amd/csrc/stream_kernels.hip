// Bandwidth-bound element-wise kernels: GEN (Eq. 1), REC (Eq. 2), the three
// steps of reshare degree reduction with RERAND (Sec. IV-B, IV-C) and the
// three steps of masked truncation (Sec. VI-B).
//
// One thread owns VEC consecutive elements and walks over all parties of its
// step, so every plane is read and written with unit stride across a wave and
// the random coefficients of an element are drawn once, not once per party.
#include "kernels.hpp"

namespace {

constexpr int BLOCK = 256;

template <int VEC>
struct pack_t;
template <>
struct pack_t<1> {
    u64 v[1];
    __device__ __forceinline__ void load(const u64 *p) { v[0] = *p; }
    __device__ __forceinline__ void store(u64 *p) const { *p = v[0]; }
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
};

template <int MAXD>
__device__ __forceinline__ void draw_coeffs(u64 (&c)[MAXD], const u64 *keys, int d, u64 e)
{
#pragma unroll
    for (int j = 0; j < MAXD; j++) c[j] = (j < d) ? ss_draw_field(keys[j], e) : 0;
}

// ------------------------------------------------------------------ GEN
template <int VEC>
__global__ __launch_bounds__(BLOCK) void share_kernel(const u64 *__restrict__ secret, u64 *__restrict__ shares,
                                                      size_t count, int n, int degree, ss_keys keys)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    pack_t<VEC> a0;
    a0.load(secret + e0);
    u64 c[VEC][SS_MAXDEG];
#pragma unroll
    for (int u = 0; u < VEC; u++) draw_coeffs<SS_MAXDEG>(c[u], keys.k, degree, e0 + u);
#pragma unroll
    for (int i = 1; i <= SS_MAXN; i++) {
        if (i <= n) {
            pack_t<VEC> s;
#pragma unroll
            for (int u = 0; u < VEC; u++) s.v[u] = ss_poly_eval<SS_MAXDEG>(a0.v[u], c[u], degree, i);
            s.store(shares + (size_t)(i - 1) * count + e0);
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
    ss_acc acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; u++) acc[u].clear();
#pragma unroll
    for (int i = 0; i < SS_MAXN; i++) {
        if (i < rp.m) {
            pack_t<VEC> s;
            s.load(shares + (size_t)rp.plane[i] * count + e0);
#pragma unroll
            for (int u = 0; u < VEC; u++) acc[u].mac(s.v[u], rp.lambda[i]);
        }
    }
    pack_t<VEC> out;
#pragma unroll
    for (int u = 0; u < VEC; u++) out.v[u] = acc[u].value();
    out.store(secret + e0);
}

// ------------------------------------------------------------------ RED step 1
// party i = blockIdx.y + 1 re-shares its value towards parties 1..k
template <int VEC>
__global__ __launch_bounds__(BLOCK) void dr1_kernel(const u64 *__restrict__ c, u64 *__restrict__ msg1,
                                                    size_t count, ss_dr_params dp)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    const int i = blockIdx.y, k = dp.t + 1;
    pack_t<VEC> ci;
    ci.load(c + (size_t)i * count + e0);
    u64 r[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) draw_coeffs<SS_MAXT>(r[u], dp.reshare_key[i], dp.t, e0 + u);
#pragma unroll
    for (int q = 0; q < SS_MAXK; q++) {
        if (q < k) {
            pack_t<VEC> s;
#pragma unroll
            for (int u = 0; u < VEC; u++) s.v[u] = ss_poly_eval<SS_MAXT>(ci.v[u], r[u], dp.t, q + 1);
            s.store(msg1 + ((size_t)i * k + q) * count + e0);
        }
    }
}

// ------------------------------------------------------------------ RED step 2
// party q = blockIdx.y + 1 multiplies the row vector it received by R.  R is
// applied in factored form R = B^-1[:, :k] * V (V[j][m] = (m+1)^j): first the k
// low coefficients of the polynomial through the received values, then its
// value at every party ID.  Same residues as the n x n product, k*(2t+1) wide
// multiplications instead of n*(2t+1).
template <int VEC>
__global__ __launch_bounds__(BLOCK) void dr2_kernel(const u64 *__restrict__ msg1, u64 *__restrict__ msg2,
                                                    size_t count, ss_dr_params dp)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    const int q = blockIdx.y, k = dp.t + 1, nr = 2 * dp.t + 1;
    ss_acc acc[VEC][SS_MAXK];
#pragma unroll
    for (int u = 0; u < VEC; u++)
#pragma unroll
        for (int j = 0; j < SS_MAXK; j++) acc[u][j].clear();
#pragma unroll
    for (int i = 0; i < 2 * SS_MAXT + 1; i++) {
        if (i < nr) {
            pack_t<VEC> v;
            v.load(msg1 + ((size_t)i * k + q) * count + e0);
#pragma unroll
            for (int j = 0; j < SS_MAXK; j++)
                if (j < k)
#pragma unroll
                    for (int u = 0; u < VEC; u++) acc[u][j].mac(v.v[u], dp.binv[i][j]);
        }
    }
    u64 a0[VEC], cf[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        a0[u] = acc[u][0].value();
#pragma unroll
        for (int j = 1; j < SS_MAXK; j++) cf[u][j - 1] = (j < k) ? acc[u][j].value() : 0;
    }
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (m < dp.n) {
            pack_t<VEC> s;
#pragma unroll
            for (int u = 0; u < VEC; u++) s.v[u] = ss_poly_eval<SS_MAXT>(a0[u], cf[u], dp.t, m + 1);
            s.store(msg2 + ((size_t)q * dp.n + m) * count + e0);
        }
    }
}

// ------------------------------------------------------------------ RED step 3 + RERAND
template <int VEC>
__global__ __launch_bounds__(BLOCK) void dr3_kernel(const u64 *__restrict__ msg2, u64 *__restrict__ out,
                                                    size_t count, ss_dr_params dp)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    const int k = dp.t + 1;
    u64 z[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) draw_coeffs<SS_MAXT>(z[u], dp.zero_key, dp.t, e0 + u);
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (m < dp.n) {
            ss_acc acc[VEC];
#pragma unroll
            for (int u = 0; u < VEC; u++) acc[u].clear();
#pragma unroll
            for (int q = 0; q < SS_MAXK; q++) {
                if (q < k) {
                    pack_t<VEC> v;
                    v.load(msg2 + ((size_t)q * dp.n + m) * count + e0);
#pragma unroll
                    for (int u = 0; u < VEC; u++) acc[u].mac(v.v[u], dp.lambda[q]);
                }
            }
            pack_t<VEC> s;
#pragma unroll
            for (int u = 0; u < VEC; u++)
                s.v[u] = ss_add(acc[u].value(), ss_poly_eval<SS_MAXT>(0, z[u], dp.t, m + 1));
            s.store(out + (size_t)m * count + e0);
        }
    }
}

// ------------------------------------------------------------------ truncation
__device__ __forceinline__ u64 mask_e(u64 key, u64 e, int f)
{
    return 1 + ((ss_draw(key, e) >> 3) & ((1ULL << (32 - f)) - 1));
}

// step 1: parties 1..k add their share of alpha = e * 2^f
template <int VEC>
__global__ __launch_bounds__(BLOCK) void tr1_kernel(const u64 *__restrict__ x, u64 *__restrict__ umsg,
                                                    size_t count, ss_tr_params tp)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    const int k = tp.t + 1;
    u64 alpha[VEC], ca[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        alpha[u] = mask_e(tp.e_key, e0 + u, tp.f) << tp.f;
        draw_coeffs<SS_MAXT>(ca[u], tp.alpha_key, tp.t, e0 + u);
    }
#pragma unroll
    for (int q = 0; q < SS_MAXK; q++) {
        if (q < k) {
            pack_t<VEC> xv, s;
            xv.load(x + (size_t)q * count + e0);
#pragma unroll
            for (int u = 0; u < VEC; u++)
                s.v[u] = ss_add(xv.v[u], ss_poly_eval<SS_MAXT>(alpha[u], ca[u], tp.t, q + 1));
            s.store(umsg + (size_t)q * count + e0);
        }
    }
}

// step 2: the elite party reconstructs x + alpha, divides by 2^f with floor on
// the signed value, and shares the quotient
template <int VEC>
__global__ __launch_bounds__(BLOCK) void tr2_kernel(const u64 *__restrict__ umsg, u64 *__restrict__ wsh,
                                                    size_t count, ss_tr_params tp)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    const int k = tp.t + 1;
    ss_acc acc[VEC];
#pragma unroll
    for (int u = 0; u < VEC; u++) acc[u].clear();
#pragma unroll
    for (int q = 0; q < SS_MAXK; q++) {
        if (q < k) {
            pack_t<VEC> v;
            v.load(umsg + (size_t)q * count + e0);
#pragma unroll
            for (int u = 0; u < VEC; u++) acc[u].mac(v.v[u], tp.lambda[q]);
        }
    }
    u64 w[VEC], cw[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        const u64 v = acc[u].value();
        const int64_t s = (v <= (SS_P - 1) / 2) ? (int64_t)v : (int64_t)v - (int64_t)SS_P;
        const int64_t qv = s >> tp.f;
        w[u] = qv >= 0 ? (u64)qv : SS_P - (u64)(-qv);
        draw_coeffs<SS_MAXT>(cw[u], tp.gen_key, tp.t, e0 + u);
    }
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (m < tp.n) {
            pack_t<VEC> s;
#pragma unroll
            for (int u = 0; u < VEC; u++) s.v[u] = ss_poly_eval<SS_MAXT>(w[u], cw[u], tp.t, m + 1);
            s.store(wsh + (size_t)m * count + e0);
        }
    }
}

// step 3: every party adds its share of alpha~ = -e
template <int VEC>
__global__ __launch_bounds__(BLOCK) void tr3_kernel(const u64 *__restrict__ wsh, u64 *__restrict__ out,
                                                    size_t count, ss_tr_params tp)
{
    const size_t e0 = ((size_t)blockIdx.x * BLOCK + threadIdx.x) * VEC;
    if (e0 >= count) return;
    u64 at[VEC], cat[VEC][SS_MAXT];
#pragma unroll
    for (int u = 0; u < VEC; u++) {
        at[u] = SS_P - mask_e(tp.e_key, e0 + u, tp.f);
        draw_coeffs<SS_MAXT>(cat[u], tp.alphat_key, tp.t, e0 + u);
    }
#pragma unroll
    for (int m = 0; m < SS_MAXN; m++) {
        if (m < tp.n) {
            pack_t<VEC> wv, s;
            wv.load(wsh + (size_t)m * count + e0);
#pragma unroll
            for (int u = 0; u < VEC; u++)
                s.v[u] = ss_add(wv.v[u], ss_poly_eval<SS_MAXT>(at[u], cat[u], tp.t, m + 1));
            s.store(out + (size_t)m * count + e0);
        }
    }
}

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
    auto grid = [&](int vec) { return dim3(blocks_for(count, vec)); };
    SS_DISPATCH_VEC(v2, share_kernel, grid, secret, shares, count, n, degree, keys);
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

hipError_t ss_launch_degree_reduce(const u64 *c, u64 *msg1, u64 *msg2, u64 *out, size_t count,
                                   const ss_dr_params &dp, hipStream_t stream)
{
    const bool v2 = (count % 2 == 0) && aligned16(c) && aligned16(msg1) && aligned16(msg2) && aligned16(out);
    const int k = dp.t + 1, nr = 2 * dp.t + 1;
    auto g1 = [&](int vec) { return dim3(blocks_for(count, vec), nr); };
    auto g2 = [&](int vec) { return dim3(blocks_for(count, vec), k); };
    auto g3 = [&](int vec) { return dim3(blocks_for(count, vec)); };
    SS_DISPATCH_VEC(v2, dr1_kernel, g1, c, msg1, count, dp);
    SS_DISPATCH_VEC(v2, dr2_kernel, g2, (const u64 *)msg1, msg2, count, dp);
    SS_DISPATCH_VEC(v2, dr3_kernel, g3, (const u64 *)msg2, out, count, dp);
    return hipGetLastError();
}

hipError_t ss_launch_truncate(const u64 *x, u64 *u, u64 *wsh, u64 *out, size_t count, const ss_tr_params &tp,
                              hipStream_t stream)
{
    const bool v2 = (count % 2 == 0) && aligned16(x) && aligned16(u) && aligned16(wsh) && aligned16(out);
    auto grid = [&](int vec) { return dim3(blocks_for(count, vec)); };
    SS_DISPATCH_VEC(v2, tr1_kernel, grid, x, u, count, tp);
    SS_DISPATCH_VEC(v2, tr2_kernel, grid, (const u64 *)u, wsh, count, tp);
    SS_DISPATCH_VEC(v2, tr3_kernel, grid, (const u64 *)wsh, out, count, tp);
    return hipGetLastError();
}
