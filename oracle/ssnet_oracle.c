/*
 * CPU oracle for the per-party arithmetic of Shamir-secret-sharing inference.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain statement of what the
 * GPU library must compute; only tests, the smoke check and the benchmark's
 * CPU-baseline leg may call it.  It shares no code with the GPU library.
 *
 * Every routine works over F_p for any prime p < 2^63 and reduces with the
 * `%` operator on unsigned __int128, so the small worked examples of the
 * paper (p = 11) run through the same code as p = 2^61 - 1.
 *
 * Layout conventions: a "share tensor" is party-major, shares[i*count + e]
 * is the share of element e held by the party with ID i+1 (Sec. IV-A: IDs are
 * 1..n).  Random polynomial coefficients are passed in explicitly to the
 * *_explicit routines; the seeded routines draw them from the counter-based
 * generator below and then call the explicit ones.
 *
 * Pins (tests/test_oracle_*.py): the F_11 worked example of Fig. 2 (product
 * shares (2,6,7) -> 6, after reduction and re-randomisation (2,9) -> 6), the
 * F_11 truncation case of App. B, 5 * 2^-1 = 8 in F_11 (Sec. IV-A), closed
 * forms for Lagrange multipliers, R^2 = R and rank k for the reduction
 * matrix, brute force over every polynomial of F_11 / F_13, integer GEMM and
 * convolution against numpy / torch int64 on small magnitudes, the
 * published SplitMix64 output sequence for the generator core, and for
 * SSS-NonLinear (ReLU under a multiplicative mask, Sec. VI-C) brute force over
 * every input and mask of a range in F_251 plus mask invariants at 2^61 - 1;
 * for the pooled form torch's max_pool2d / avg_pool2d on the plain values and
 * the constancy of beta inside a pooling kernel; for the truncation with the
 * rounding division of App. C the printed worst case (error 2 for a 2x2
 * kernel), its bound by brute force, and independence of the mask; over the
 * paper's prime 2^45 - 55 the split product of App. D restated with integers,
 * the 16-bit + 13-bit budget of Sec. VII-A, and a tiny layer end to end.
 * The choice of generator itself is not fixed by the paper ("randomly
 * generated", Sec. IV-A): parity unpinned for *which* random bits are drawn.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef uint64_t u64;
typedef int64_t i64;
typedef unsigned __int128 u128;

#define ORC_MAXN 16

/* ------------------------------------------------------------------ */
/* Field arithmetic in F_p (Sec. IV-A, last paragraph of REC).         */
/* Operands are canonical, i.e. in [0, p-1]; so are results.           */
/* ------------------------------------------------------------------ */

u64 orc_add(u64 a, u64 b, u64 p) { return (u64)(((u128)a + b) % p); }

u64 orc_sub(u64 a, u64 b, u64 p) { return (u64)(((u128)a + p - b) % p); }

u64 orc_mul(u64 a, u64 b, u64 p) { return (u64)(((u128)a * b) % p); }

u64 orc_pow(u64 a, u64 e, u64 p)
{
    u64 r = 1 % p;
    while (e) {
        if (e & 1) r = orc_mul(r, a, p);
        a = orc_mul(a, a, p);
        e >>= 1;
    }
    return r;
}

/* multiplicative inverse: b * b^-1 = 1 (mod p); Fermat, p prime */
u64 orc_inv(u64 a, u64 p) { return orc_pow(a, p - 2, p); }

/* ------------------------------------------------------------------ */
/* Signed <-> field and fixed point (Sec. II-B: F_p stands for the     */
/* signed range [-(p-1)/2, (p-1)/2]).                                   */
/* ------------------------------------------------------------------ */

/* centred lift: u if u <= (p-1)/2, else u - p */
i64 orc_lift1(u64 u, u64 p) { return (u <= (p - 1) / 2) ? (i64)u : (i64)u - (i64)p; }

void orc_lift(const u64 *u, size_t count, u64 p, i64 *out)
{
    for (size_t e = 0; e < count; e++) out[e] = orc_lift1(u[e], p);
}

/* signed integer -> field element */
u64 orc_from_signed(i64 v, u64 p)
{
    if (v >= 0) return (u64)v % p;
    u64 a = (u64)(-v) % p;
    return a ? p - a : 0;
}

/* x -> round-half-even(x * 2^f) as a field element.  Returns the number of
 * inputs whose scaled magnitude is 2^40 or more (those are still written). */
size_t orc_encode(const double *x, size_t count, int f, u64 p, u64 *out)
{
    size_t bad = 0;
    for (size_t e = 0; e < count; e++) {
        double s = rint(ldexp(x[e], f)); /* default rounding mode: nearest-even */
        if (!(fabs(s) < 1099511627776.0)) bad++;
        out[e] = orc_from_signed((i64)s, p);
    }
    return bad;
}

/* field element -> lift / 2^s as float64 */
void orc_decode(const u64 *u, size_t count, int s, u64 p, double *out)
{
    for (size_t e = 0; e < count; e++) out[e] = ldexp((double)orc_lift1(u[e], p), -s);
}

/* ------------------------------------------------------------------ */
/* Counter-based generator.  Core: the SplitMix64 output function      */
/* (Steele, Lea, Flood 2014; constants of Stafford's "mix13").          */
/* ------------------------------------------------------------------ */

#define ORC_GAMMA 0x9E3779B97F4A7C15ULL

u64 orc_mix64(u64 z)
{
    z ^= z >> 30;
    z *= 0xBF58476D1CE4E5B9ULL;
    z ^= z >> 27;
    z *= 0x94D049BB133111EBULL;
    z ^= z >> 31;
    return z;
}

/* one key per (seed, domain, stream_id, party, coefficient index j):
 * absorb the five words one after another */
u64 orc_key(u64 seed, u64 domain, u64 stream_id, u64 party, u64 j)
{
    u64 w[5] = {seed, domain, stream_id, party, j};
    u64 h = 0;
    for (int i = 0; i < 5; i++) h = orc_mix64((h ^ w[i]) + ORC_GAMMA);
    return h;
}

/* e-th 64-bit output of the stream with that key (random access) */
u64 orc_draw(u64 key, u64 e) { return orc_mix64(key + (e + 1) * ORC_GAMMA); }

/* field element from the top 61 bits */
u64 orc_draw_field(u64 key, u64 e, u64 p) { return (orc_draw(key, e) >> 3) % p; }

enum {
    ORC_DOM_SHARE = 1,
    ORC_DOM_RESHARE = 2,
    ORC_DOM_ZERO = 3,
    ORC_DOM_MASK_E = 4,
    ORC_DOM_MASK_ALPHA = 5,
    ORC_DOM_MASK_ALPHAT = 6,
    ORC_DOM_TRUNC_GEN = 7,
    ORC_DOM_MASK_BETA = 8,
    ORC_DOM_BETA_GEN = 9,
    ORC_DOM_BETAINV_GEN = 10
};

/* coef[(j-1)*count + e] = a_j of element e, j = 1..degree.  eidx gives the
 * global element index used as the counter (NULL: eidx[e] = e). */
void orc_draw_coeffs(u64 seed, u64 domain, u64 stream_id, u64 party, int degree, size_t count,
                     const u64 *eidx, u64 p, u64 *coef)
{
    for (int j = 1; j <= degree; j++) {
        u64 key = orc_key(seed, domain, stream_id, party, (u64)j);
#pragma omp parallel for schedule(static)
        for (size_t e = 0; e < count; e++)
            coef[(size_t)(j - 1) * count + e] = orc_draw_field(key, eidx ? eidx[e] : (u64)e, p);
    }
}

/* ------------------------------------------------------------------ */
/* GEN: share generation (Eq. 1).                                       */
/* share_i = a0 + a1*ID + ... + a_d*ID^d (mod p), ID = i for i = 1..n.  */
/* ------------------------------------------------------------------ */

/* polynomial with constant term a0 and higher coefficients coef[j-1][e],
 * evaluated at x (Horner) */
static u64 poly_eval(u64 a0, const u64 *coef, size_t count, size_t e, int degree, u64 x, u64 p)
{
    u64 acc = 0;
    for (int j = degree; j >= 1; j--) {
        acc = orc_add(acc, coef[(size_t)(j - 1) * count + e], p);
        acc = orc_mul(acc, x % p, p);
    }
    return orc_add(acc, a0, p);
}

void orc_share_explicit(const u64 *secret, const u64 *coef, size_t count, int n, int degree, u64 p,
                        u64 *shares)
{
    for (int i = 1; i <= n; i++) {
#pragma omp parallel for schedule(static)
        for (size_t e = 0; e < count; e++)
            shares[(size_t)(i - 1) * count + e] = poly_eval(secret[e], coef, count, e, degree, (u64)i, p);
    }
}

void orc_share(const u64 *secret, size_t count, const u64 *eidx, int n, int degree, u64 p, u64 seed,
               u64 stream_id, u64 *shares)
{
    u64 *coef = (u64 *)malloc(sizeof(u64) * count * (size_t)(degree > 0 ? degree : 1));
    orc_draw_coeffs(seed, ORC_DOM_SHARE, stream_id, 0, degree, count, eidx, p, coef);
    orc_share_explicit(secret, coef, count, n, degree, p, shares);
    free(coef);
}

/* ------------------------------------------------------------------ */
/* REC: reconstruction (Eq. 2).                                         */
/* lambda_i = prod_{j != i} ID_j / (ID_j - ID_i); a0 = sum lambda_i s_i */
/* ------------------------------------------------------------------ */

void orc_lagrange(const int *ids, int m, u64 p, u64 *lambda)
{
    for (int i = 0; i < m; i++) {
        u64 l = 1 % p;
        for (int j = 0; j < m; j++) {
            if (j == i) continue;
            u64 idj = (u64)ids[j] % p, idi = (u64)ids[i] % p;
            l = orc_mul(l, orc_mul(idj, orc_inv(orc_sub(idj, idi, p), p), p), p);
        }
        lambda[i] = l;
    }
}

/* shares is [n][count] party-major; ids[0..m-1] are the party IDs used */
void orc_reconstruct(const u64 *shares, size_t count, const int *ids, int m, u64 p, u64 *secret)
{
    u64 lambda[ORC_MAXN];
    orc_lagrange(ids, m, p, lambda);
#pragma omp parallel for schedule(static)
    for (size_t e = 0; e < count; e++) {
        u64 acc = 0;
        for (int i = 0; i < m; i++)
            acc = orc_add(acc, orc_mul(lambda[i], shares[(size_t)(ids[i] - 1) * count + e], p), p);
        secret[e] = acc;
    }
}

/* ------------------------------------------------------------------ */
/* Local linear layers on shares (Sec. VI-A step 1): each party         */
/* multiplies ITS share of x with ITS share of w, all arithmetic mod p. */
/* ------------------------------------------------------------------ */

/* acc + a*b with a, b < p < 2^63: a*b < 2^126, and acc is kept below 2^126 by
 * reducing it whenever bit 126 is set, so the sum never reaches 2^128. */
static inline u128 mac_lazy(u128 acc, u64 a, u64 b, u64 p)
{
    acc += (u128)a * b;
    if (acc >> 126) acc %= p;
    return acc;
}

/* x [n][M][K], w [n][K][N] -> y [n][M][N] */
void orc_linear(const u64 *x, const u64 *w, int n, int M, int K, int N, u64 p, u64 *y)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < n; i++)
        for (int m = 0; m < M; m++) {
            const u64 *xi = x + ((size_t)i * M + m) * K;
            const u64 *wi = w + (size_t)i * K * N;
            for (int c = 0; c < N; c++) {
                u128 acc = 0;
                for (int k = 0; k < K; k++) acc = mac_lazy(acc, xi[k], wi[(size_t)k * N + c], p);
                y[((size_t)i * M + m) * N + c] = (u64)(acc % p);
            }
        }
}

/* same product with a reduction after every multiply-add: the definition,
 * used to check the lazily reduced loops above and below */
void orc_linear_strict(const u64 *x, const u64 *w, int n, int M, int K, int N, u64 p, u64 *y)
{
    for (int i = 0; i < n; i++)
        for (int m = 0; m < M; m++)
            for (int c = 0; c < N; c++) {
                u64 acc = 0;
                for (int k = 0; k < K; k++)
                    acc = orc_add(acc, orc_mul(x[((size_t)i * M + m) * K + k],
                                               w[((size_t)i * K + k) * N + c], p), p);
                y[((size_t)i * M + m) * N + c] = acc;
            }
}

static int conv_out(int H, int k, int stride, int pad) { return (H + 2 * pad - k) / stride + 1; }

/* one output element of the cross-correlation (no kernel flip), zero padding:
 * x [n][B][C][H][W], w [n][Co][C][kh][kw] */
static u64 conv_point(const u64 *x, const u64 *w, int B, int C, int H, int W, int Co, int kh, int kw,
                      int stride, int pad, int i, int b, int co, int ho, int wo, u64 p)
{
    u128 acc = 0;
    for (int c = 0; c < C; c++)
        for (int r = 0; r < kh; r++)
            for (int s = 0; s < kw; s++) {
                int hi = ho * stride - pad + r, wi = wo * stride - pad + s;
                if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue; /* padded zero */
                u64 xv = x[((((size_t)i * B + b) * C + c) * H + hi) * W + wi];
                u64 wv = w[((((size_t)i * Co + co) * C + c) * kh + r) * kw + s];
                acc = mac_lazy(acc, xv, wv, p);
            }
    return (u64)(acc % p);
}

/* y [n][B][Co][Ho][Wo] */
void orc_conv(const u64 *x, const u64 *w, int n, int B, int C, int H, int W, int Co, int kh, int kw,
              int stride, int pad, u64 p, u64 *y)
{
    int Ho = conv_out(H, kh, stride, pad), Wo = conv_out(W, kw, stride, pad);
    int rows = n * B * Co;
#pragma omp parallel for schedule(dynamic, 1)
    for (int row = 0; row < rows; row++) {
        int co = row % Co, b = (row / Co) % B, i = row / (Co * B);
        for (int ho = 0; ho < Ho; ho++)
            for (int wo = 0; wo < Wo; wo++)
                y[(((size_t)row) * Ho + ho) * Wo + wo] =
                    conv_point(x, w, B, C, H, W, Co, kh, kw, stride, pad, i, b, co, ho, wo, p);
    }
}

/* sampled outputs: flat[q] indexes y as [n][B][Co][Ho][Wo] */
void orc_conv_points(const u64 *x, const u64 *w, int n, int B, int C, int H, int W, int Co, int kh,
                     int kw, int stride, int pad, u64 p, const u64 *flat, size_t npoints, u64 *out)
{
    int Ho = conv_out(H, kh, stride, pad), Wo = conv_out(W, kw, stride, pad);
    (void)n;
    for (size_t q = 0; q < npoints; q++) {
        u64 r = flat[q];
        int wo = (int)(r % Wo); r /= Wo;
        int ho = (int)(r % Ho); r /= Ho;
        int co = (int)(r % Co); r /= Co;
        int b = (int)(r % B); r /= B;
        out[q] = conv_point(x, w, B, C, H, W, Co, kh, kw, stride, pad, (int)r, b, co, ho, wo, p);
    }
}

/* ------------------------------------------------------------------ */
/* Degree-reduction matrix R = B^-1 P B (Eq. 3).                        */
/* B is the Vandermonde matrix b[i][j] = ID_j^(i-1) on the nr = 2t+1    */
/* reducing parties, P keeps the first k = t+1 coefficients.  Shares    */
/* are a row vector: c' = c * R.  With n > nr parties the last factor   */
/* has n columns (the truncated polynomial is evaluated at all n IDs),  */
/* so R is nr x n, row-major.                                           */
/* ------------------------------------------------------------------ */

/* inverse of the nr x nr matrix a (row-major) by Gauss-Jordan in F_p;
 * returns 0 on success */
static int mat_inv(const u64 *a, int nr, u64 p, u64 *inv)
{
    u64 m[ORC_MAXN][2 * ORC_MAXN];
    for (int i = 0; i < nr; i++)
        for (int j = 0; j < nr; j++) {
            m[i][j] = a[i * nr + j] % p;
            m[i][nr + j] = (i == j) ? 1 % p : 0;
        }
    for (int col = 0; col < nr; col++) {
        int piv = -1;
        for (int r = col; r < nr; r++)
            if (m[r][col]) { piv = r; break; }
        if (piv < 0) return -1;
        if (piv != col)
            for (int j = 0; j < 2 * nr; j++) { u64 tmp = m[col][j]; m[col][j] = m[piv][j]; m[piv][j] = tmp; }
        u64 s = orc_inv(m[col][col], p);
        for (int j = 0; j < 2 * nr; j++) m[col][j] = orc_mul(m[col][j], s, p);
        for (int r = 0; r < nr; r++) {
            if (r == col || !m[r][col]) continue;
            u64 fct = m[r][col];
            for (int j = 0; j < 2 * nr; j++) m[r][j] = orc_sub(m[r][j], orc_mul(fct, m[col][j], p), p);
        }
    }
    for (int i = 0; i < nr; i++)
        for (int j = 0; j < nr; j++) inv[i * nr + j] = m[i][nr + j];
    return 0;
}

int orc_red_matrix(int n, int t, u64 p, u64 *R /* [2t+1][n] */)
{
    int nr = 2 * t + 1, k = t + 1;
    if (nr > ORC_MAXN || n > ORC_MAXN || n < nr) return -1;
    u64 Bsq[ORC_MAXN * ORC_MAXN], Binv[ORC_MAXN * ORC_MAXN], Bext[ORC_MAXN * ORC_MAXN];
    for (int i = 0; i < nr; i++) {
        for (int j = 0; j < nr; j++) Bsq[i * nr + j] = orc_pow((u64)(j + 1) % p, (u64)i, p);
        for (int j = 0; j < n; j++) Bext[i * n + j] = orc_pow((u64)(j + 1) % p, (u64)i, p);
    }
    if (mat_inv(Bsq, nr, p, Binv)) return -2;
    /* R = Binv * P * Bext : sum over the first k coefficient indices only */
    for (int i = 0; i < nr; i++)
        for (int m = 0; m < n; m++) {
            u64 acc = 0;
            for (int c = 0; c < k; c++) acc = orc_add(acc, orc_mul(Binv[i * nr + c], Bext[c * n + m], p), p);
            R[i * n + m] = acc;
        }
    return 0;
}

/* ------------------------------------------------------------------ */
/* RED by resharing (Sec. IV-B, the three protocol steps) followed by   */
/* RERAND (Sec. IV-C).                                                  */
/*   c      [n][count]   degree-2t shares (parties 1..2t+1 are read)    */
/*   rcoef  [2t+1][t][count]  reshare coefficients of party i           */
/*   zcoef  [t][count]        coefficients of the zero sharing          */
/*   msg1   [2t+1][k][count]  step 1: party i -> party q (may be NULL)  */
/*   msg2   [k][n][count]     step 2: party q -> party m (may be NULL)  */
/*   red    [n][count]        step 3 result before RERAND (may be NULL) */
/*   out    [n][count]        after RERAND                              */
/* ------------------------------------------------------------------ */

int orc_degree_reduce_explicit(const u64 *c, const u64 *rcoef, const u64 *zcoef, size_t count, int n,
                               int t, u64 p, u64 *msg1, u64 *msg2, u64 *red, u64 *out)
{
    int nr = 2 * t + 1, k = t + 1;
    u64 R[ORC_MAXN * ORC_MAXN], lambda[ORC_MAXN];
    int ids[ORC_MAXN];
    if (orc_red_matrix(n, t, p, R)) return -1;
    for (int q = 0; q < k; q++) ids[q] = q + 1;
    orc_lagrange(ids, k, p, lambda);

    u64 *m1 = msg1 ? msg1 : (u64 *)malloc(sizeof(u64) * (size_t)nr * k * count);
    u64 *m2 = msg2 ? msg2 : (u64 *)malloc(sizeof(u64) * (size_t)k * n * count);
    u64 *rd = red ? red : (u64 *)malloc(sizeof(u64) * (size_t)n * count);

    /* step 1, on each reducing party i: GEN(c_i, k, k) towards parties 1..k */
    for (int i = 0; i < nr; i++)
        orc_share_explicit(c + (size_t)i * count, rcoef + (size_t)i * t * count, count, k, t, p,
                           m1 + (size_t)i * k * count);

    /* step 2, on party q = 1..k: row vector of received sub-shares times R */
    for (int q = 0; q < k; q++)
        for (int m = 0; m < n; m++) {
#pragma omp parallel for schedule(static)
            for (size_t e = 0; e < count; e++) {
                u64 acc = 0;
                for (int i = 0; i < nr; i++)
                    acc = orc_add(acc, orc_mul(m1[((size_t)i * k + q) * count + e], R[i * n + m], p), p);
                m2[((size_t)q * n + m) * count + e] = acc;
            }
        }

    /* step 3, on each party m: REC of the k sub-shares it received */
    for (int m = 0; m < n; m++) {
#pragma omp parallel for schedule(static)
        for (size_t e = 0; e < count; e++) {
            u64 acc = 0;
            for (int q = 0; q < k; q++)
                acc = orc_add(acc, orc_mul(lambda[q], m2[((size_t)q * n + m) * count + e], p), p);
            rd[(size_t)m * count + e] = acc;
        }
    }

    /* RERAND on all n parties: add the party's share of zero */
    for (int m = 0; m < n; m++) {
#pragma omp parallel for schedule(static)
        for (size_t e = 0; e < count; e++)
            out[(size_t)m * count + e] =
                orc_add(rd[(size_t)m * count + e], poly_eval(0, zcoef, count, e, t, (u64)(m + 1), p), p);
    }

    if (!msg1) free(m1);
    if (!msg2) free(m2);
    if (!red) free(rd);
    return 0;
}

int orc_degree_reduce(const u64 *c, size_t count, const u64 *eidx, int n, int t, u64 p, u64 seed,
                      u64 stream_id, u64 *msg1, u64 *msg2, u64 *red, u64 *out)
{
    int nr = 2 * t + 1;
    u64 *rcoef = (u64 *)malloc(sizeof(u64) * (size_t)nr * t * count);
    u64 *zcoef = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    for (int i = 0; i < nr; i++)
        orc_draw_coeffs(seed, ORC_DOM_RESHARE, stream_id, (u64)(i + 1), t, count, eidx, p,
                        rcoef + (size_t)i * t * count);
    orc_draw_coeffs(seed, ORC_DOM_ZERO, stream_id, 0, t, count, eidx, p, zcoef);
    int rc = orc_degree_reduce_explicit(c, rcoef, zcoef, count, n, t, p, msg1, msg2, red, out);
    free(rcoef);
    free(zcoef);
    return rc;
}

/* ------------------------------------------------------------------ */
/* Masked truncation (Sec. VI-B): y = floor(x / 2^f) on shares.         */
/*   x      [n][count]  degree-t shares (parties 1..k are read)         */
/*   eval   [count]     e >= 1; alpha = e * 2^f, alpha~ = -e            */
/*   ca, cat, cw  [t][count] coefficients for [[alpha]], [[alpha~]] and */
/*                the elite party's re-sharing of the truncated value   */
/*   u      [k][count]  step 1 messages x_q + alpha_q (may be NULL)     */
/*   wsh    [n][count]  step 2 shares of floor((x+alpha)/2^f) (or NULL) */
/*   out    [n][count]                                                  */
/* ------------------------------------------------------------------ */

void orc_truncate_explicit(const u64 *x, const u64 *eval, const u64 *ca, const u64 *cat, const u64 *cw,
                           size_t count, int n, int t, int f, u64 p, u64 *u, u64 *wsh, u64 *out)
{
    int k = t + 1;
    int ids[ORC_MAXN];
    for (int q = 0; q < k; q++) ids[q] = q + 1;

    u64 *alpha = (u64 *)malloc(sizeof(u64) * count);
    u64 *alphat = (u64 *)malloc(sizeof(u64) * count);
    u64 *sh_a = (u64 *)malloc(sizeof(u64) * (size_t)n * count);
    u64 *sh_at = (u64 *)malloc(sizeof(u64) * (size_t)n * count);
    u64 *v = (u64 *)malloc(sizeof(u64) * count);
    u64 *ww = wsh ? wsh : (u64 *)malloc(sizeof(u64) * (size_t)n * count);

    /* trusted source: masks alpha = e*r, alpha~ = -e, and their sharings */
    for (size_t e = 0; e < count; e++) {
        alpha[e] = orc_mul(eval[e] % p, orc_pow(2 % p, (u64)f, p), p);
        alphat[e] = orc_sub(0, eval[e] % p, p);
    }
    orc_share_explicit(alpha, ca, count, n, t, p, sh_a);
    orc_share_explicit(alphat, cat, count, n, t, p, sh_at);

    /* step 1 on parties 1..k: mask */
    u64 *ufull = (u64 *)calloc((size_t)n * count, sizeof(u64));
    for (int q = 0; q < k; q++)
        for (size_t e = 0; e < count; e++) {
            ufull[(size_t)q * count + e] = orc_add(x[(size_t)q * count + e], sh_a[(size_t)q * count + e], p);
            if (u) u[(size_t)q * count + e] = ufull[(size_t)q * count + e];
        }

    /* step 2 on the elite party: REC, floor division by r = 2^f on the signed
     * value, GEN of the result */
    orc_reconstruct(ufull, count, ids, k, p, v);
    for (size_t e = 0; e < count; e++) {
        i64 s = orc_lift1(v[e], p);
        i64 q = s >> f; /* arithmetic shift = floor(s / 2^f): s = q*2^f + b, 0 <= b < 2^f */
        v[e] = orc_from_signed(q, p);
    }
    orc_share_explicit(v, cw, count, n, t, p, ww);

    /* step 3 on all n parties: unmask */
    for (int m = 0; m < n; m++)
        for (size_t e = 0; e < count; e++)
            out[(size_t)m * count + e] = orc_add(ww[(size_t)m * count + e], sh_at[(size_t)m * count + e], p);

    free(alpha); free(alphat); free(sh_a); free(sh_at); free(v); free(ufull);
    if (!wsh) free(ww);
}

void orc_truncate(const u64 *x, size_t count, const u64 *eidx, int n, int t, int f, u64 p, u64 seed,
                  u64 stream_id, u64 *u, u64 *wsh, u64 *out)
{
    u64 *eval = (u64 *)malloc(sizeof(u64) * count);
    u64 *ca = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    u64 *cat = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    u64 *cw = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    /* alpha in (0, 2^32], a multiple of r = 2^f  =>  e uniform in [1, 2^(32-f)] */
    u64 key = orc_key(seed, ORC_DOM_MASK_E, stream_id, 0, 0);
    for (size_t e = 0; e < count; e++)
        eval[e] = 1 + (orc_draw(key, eidx ? eidx[e] : (u64)e) >> 3) % ((u64)1 << (32 - f));
    orc_draw_coeffs(seed, ORC_DOM_MASK_ALPHA, stream_id, 0, t, count, eidx, p, ca);
    orc_draw_coeffs(seed, ORC_DOM_MASK_ALPHAT, stream_id, 0, t, count, eidx, p, cat);
    orc_draw_coeffs(seed, ORC_DOM_TRUNC_GEN, stream_id, 0, t, count, eidx, p, cw);
    orc_truncate_explicit(x, eval, ca, cat, cw, count, n, t, f, p, u, wsh, out);
    free(eval); free(ca); free(cat); free(cw);
}

/* ------------------------------------------------------------------ */
/* SSS-NonLinear with ReLU (Sec. VI-C; masks: Sec. VII-B).              */
/*                                                                      */
/* Trusted source, ahead of the inference: a positive mask beta per      */
/* element, its field inverse, and a degree-t sharing of each.           */
/*   beta   [count]     1 <= beta (the paper draws it from (0, 2^28])    */
/*   cb, cbi [t][count] coefficients of [[beta]] and [[beta^-1]]         */
/*   sh_b, sh_bi [n][count]                                              */
/* ------------------------------------------------------------------ */

void orc_nonlinear_masks_explicit(const u64 *beta, const u64 *cb, const u64 *cbi, size_t count, int n, int t,
                                  u64 p, u64 *sh_b, u64 *sh_bi)
{
    u64 *b = (u64 *)malloc(sizeof(u64) * count);
    u64 *bi = (u64 *)malloc(sizeof(u64) * count);
    for (size_t e = 0; e < count; e++) {
        b[e] = beta[e] % p;
        bi[e] = orc_inv(b[e], p); /* beta * beta^-1 = 1 in F_p */
    }
    orc_share_explicit(b, cb, count, n, t, p, sh_b);
    orc_share_explicit(bi, cbi, count, n, t, p, sh_bi);
    free(b); free(bi);
}

/* beta uniform in [1, 2^bbits] from the generator (domain MASK_BETA); the paper's choice is bbits = 28 */
void orc_nonlinear_masks(size_t count, const u64 *eidx, int n, int t, int bbits, u64 p, u64 seed, u64 stream_id,
                         u64 *sh_b, u64 *sh_bi)
{
    u64 *beta = (u64 *)malloc(sizeof(u64) * count);
    u64 *cb = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    u64 *cbi = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    u64 key = orc_key(seed, ORC_DOM_MASK_BETA, stream_id, 0, 0);
    for (size_t e = 0; e < count; e++)
        beta[e] = 1 + (orc_draw(key, eidx ? eidx[e] : (u64)e) >> 3) % ((u64)1 << bbits);
    orc_draw_coeffs(seed, ORC_DOM_BETA_GEN, stream_id, 0, t, count, eidx, p, cb);
    orc_draw_coeffs(seed, ORC_DOM_BETAINV_GEN, stream_id, 0, t, count, eidx, p, cbi);
    orc_nonlinear_masks_explicit(beta, cb, cbi, count, n, t, p, sh_b, sh_bi);
    free(beta); free(cb); free(cbi);
}

/* The three steps of the protocol:                                      */
/*   1. parties 1..2t+1: Hadamard product m_i = x_i * beta_i (a sharing   */
/*      of x*beta of degree 2t)                       -> msg [2t+1][count] */
/*   2. elite party: v = REC(m; IDs 1..2t+1) = x*beta; the non-linear     */
/*      function in the clear on the signed value, y = max(v, 0)          */
/*                                                    -> yplain [count]   */
/*   3. every party: out_i = y * betainv_i (plain value times share: the  */
/*      degree stays t)                               -> out [n][count]   */
/* x, sh_b, sh_bi are [n][count]; msg and yplain may be NULL.            */
/* Requires |x| * beta < p/2, so that the sign of x*beta is that of x.   */
void orc_relu(const u64 *x, const u64 *sh_b, const u64 *sh_bi, size_t count, int n, int t, u64 p, u64 *msg,
              u64 *yplain, u64 *out)
{
    int nr = 2 * t + 1;
    int ids[ORC_MAXN];
    for (int i = 0; i < nr; i++) ids[i] = i + 1;
    u64 *m = (u64 *)calloc((size_t)n * count, sizeof(u64));
    u64 *v = (u64 *)malloc(sizeof(u64) * count);
    for (int i = 0; i < nr; i++)
        for (size_t e = 0; e < count; e++) {
            m[(size_t)i * count + e] = orc_mul(x[(size_t)i * count + e], sh_b[(size_t)i * count + e], p);
            if (msg) msg[(size_t)i * count + e] = m[(size_t)i * count + e];
        }
    orc_reconstruct(m, count, ids, nr, p, v);
    for (size_t e = 0; e < count; e++) {
        i64 s = orc_lift1(v[e], p);
        v[e] = s > 0 ? (u64)s : 0;
        if (yplain) yplain[e] = v[e];
    }
    for (int i = 0; i < n; i++)
        for (size_t e = 0; e < count; e++)
            out[(size_t)i * count + e] = orc_mul(v[e], sh_bi[(size_t)i * count + e], p);
    free(m); free(v);
}

/* ------------------------------------------------------------------ */
/* Truncation followed by a rounding division (Sec. VI-C, the extra     */
/* step for average pooling; App. C): y = [ floor(x / 2^f) / kdiv ],    */
/* kdiv = kh*kw of the pooling kernel that follows.  The mask becomes   */
/* alpha = e * 2^f * kdiv, alpha~ = -e stays; the sample space of e     */
/* shrinks to [1, floor(2^(32-f) / kdiv)] so that alpha stays in        */
/* (0, 2^32] (Sec. VII-B).  [.] rounds to the                           */
/* nearest integer, a remainder of ceil(kdiv/2) or more going up (the   */
/* worst case of App. C), i.e. [v/kdiv] = floor((v + floor(kdiv/2)) /   */
/* kdiv) on the signed value, so that [(v + e*kdiv)/kdiv] = [v/kdiv]+e. */
/* Arguments as orc_truncate_explicit.                                  */
/* ------------------------------------------------------------------ */

static i64 floor_div(i64 a, i64 b) /* b > 0 */
{
    i64 q = a / b;
    return (a % b < 0) ? q - 1 : q;
}

void orc_truncate_div_explicit(const u64 *x, const u64 *eval, const u64 *ca, const u64 *cat, const u64 *cw,
                               size_t count, int n, int t, int f, int kdiv, u64 p, u64 *u, u64 *wsh, u64 *out)
{
    int k = t + 1;
    int ids[ORC_MAXN];
    for (int q = 0; q < k; q++) ids[q] = q + 1;
    u64 *alpha = (u64 *)malloc(sizeof(u64) * count);
    u64 *alphat = (u64 *)malloc(sizeof(u64) * count);
    u64 *sh_a = (u64 *)malloc(sizeof(u64) * (size_t)n * count);
    u64 *sh_at = (u64 *)malloc(sizeof(u64) * (size_t)n * count);
    u64 *v = (u64 *)malloc(sizeof(u64) * count);
    u64 *ww = wsh ? wsh : (u64 *)malloc(sizeof(u64) * (size_t)n * count);
    u64 *ufull = (u64 *)calloc((size_t)n * count, sizeof(u64));

    /* trusted source: alpha = e * r * kh*kw, alpha~ = -e */
    u64 rk = orc_mul(orc_pow(2 % p, (u64)f, p), (u64)kdiv % p, p);
    for (size_t e = 0; e < count; e++) {
        alpha[e] = orc_mul(eval[e] % p, rk, p);
        alphat[e] = orc_sub(0, eval[e] % p, p);
    }
    orc_share_explicit(alpha, ca, count, n, t, p, sh_a);
    orc_share_explicit(alphat, cat, count, n, t, p, sh_at);

    for (int q = 0; q < k; q++)
        for (size_t e = 0; e < count; e++) {
            ufull[(size_t)q * count + e] = orc_add(x[(size_t)q * count + e], sh_a[(size_t)q * count + e], p);
            if (u) u[(size_t)q * count + e] = ufull[(size_t)q * count + e];
        }

    /* elite party: REC, floor by 2^f, then the rounding division */
    orc_reconstruct(ufull, count, ids, k, p, v);
    for (size_t e = 0; e < count; e++) {
        i64 s = orc_lift1(v[e], p) >> f;
        v[e] = orc_from_signed(floor_div(s + kdiv / 2, kdiv), p);
    }
    orc_share_explicit(v, cw, count, n, t, p, ww);

    for (int m = 0; m < n; m++)
        for (size_t e = 0; e < count; e++)
            out[(size_t)m * count + e] = orc_add(ww[(size_t)m * count + e], sh_at[(size_t)m * count + e], p);

    free(alpha); free(alphat); free(sh_a); free(sh_at); free(v); free(ufull);
    if (!wsh) free(ww);
}

/* same draws as orc_truncate; e uniform in [1, floor(2^(32-f) / kdiv)] (Sec. VII-B: the cardinality of the mask */
/* generation before a pooling kernel of kh*kw elements), the three coefficient domains                          */
void orc_truncate_div(const u64 *x, size_t count, const u64 *eidx, int n, int t, int f, int kdiv, u64 p, u64 seed,
                      u64 stream_id, u64 *u, u64 *wsh, u64 *out)
{
    u64 *eval = (u64 *)malloc(sizeof(u64) * count);
    u64 *ca = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    u64 *cat = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    u64 *cw = (u64 *)malloc(sizeof(u64) * (size_t)t * count);
    u64 key = orc_key(seed, ORC_DOM_MASK_E, stream_id, 0, 0);
    for (size_t e = 0; e < count; e++)
        eval[e] = 1 + (orc_draw(key, eidx ? eidx[e] : (u64)e) >> 3) % (((u64)1 << (32 - f)) / (u64)kdiv);
    orc_draw_coeffs(seed, ORC_DOM_MASK_ALPHA, stream_id, 0, t, count, eidx, p, ca);
    orc_draw_coeffs(seed, ORC_DOM_MASK_ALPHAT, stream_id, 0, t, count, eidx, p, cat);
    orc_draw_coeffs(seed, ORC_DOM_TRUNC_GEN, stream_id, 0, t, count, eidx, p, cw);
    orc_truncate_div_explicit(x, eval, ca, cat, cw, count, n, t, f, kdiv, p, u, wsh, out);
    free(eval); free(ca); free(cat); free(cw);
}

/* ------------------------------------------------------------------ */
/* SSS-NonLinear with ReLU followed by pooling (Sec. VI-C).             */
/*                                                                      */
/* A tensor is `planes` images of H x W (planes = batch * channels).    */
/* The pooling kernel is kh x kw, moved by (sh, sw) over the image      */
/* padded with ph / pw zeros on each side:                              */
/*   Ho = (H + 2 ph - kh) / sh + 1,  Wo likewise.                       */
/* The mask beta must be equal inside one pooling kernel.  Where the    */
/* kernels tile the image (stride = kernel, no padding) that is one     */
/* beta per kernel position (elements right of / below the last full    */
/* kernel join the last one); where kernels overlap, every element of   */
/* a plane is linked to every other through shared kernels, so it is    */
/* one beta per plane.  The group index is the counter of the beta      */
/* draw.                                                                */
/* ------------------------------------------------------------------ */

typedef struct { int H, W, kh, kw, sh, sw, ph, pw, Ho, Wo, tiled; } orc_pool_geom;

static orc_pool_geom pool_geom(int H, int W, int kh, int kw, int sh, int sw, int ph, int pw)
{
    orc_pool_geom g = {H, W, kh, kw, sh, sw, ph, pw, 0, 0, 0};
    g.Ho = (H + 2 * ph - kh) / sh + 1;
    g.Wo = (W + 2 * pw - kw) / sw + 1;
    g.tiled = (sh == kh && sw == kw && ph == 0 && pw == 0);
    return g;
}

static u64 pool_group_in(const orc_pool_geom *g, size_t plane, int h, int w)
{
    if (!g->tiled) return plane;
    int oh = h / g->kh < g->Ho - 1 ? h / g->kh : g->Ho - 1;
    int ow = w / g->kw < g->Wo - 1 ? w / g->kw : g->Wo - 1;
    return ((u64)plane * g->Ho + oh) * g->Wo + ow;
}

static u64 pool_group_out(const orc_pool_geom *g, size_t plane, int oh, int ow)
{
    return g->tiled ? ((u64)plane * g->Ho + oh) * g->Wo + ow : (u64)plane;
}

int orc_pool_out_size(int H, int k, int s, int pad) { return (H + 2 * pad - k) / s + 1; }

/* Trusted source: shares of beta for every input element [n][planes*H*W]
 * and of beta^-1 for every pooled element [n][planes*Ho*Wo].  beta of a
 * group is drawn at counter = group index (domain MASK_BETA), uniform in
 * [1, 2^bbits]; the sharing coefficients are drawn per element (domains
 * BETA_GEN at the input element's index, BETAINV_GEN at the pooled one's). */
void orc_pool_masks(size_t planes, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw, int n, int t,
                    int bbits, u64 p, u64 seed, u64 stream_id, u64 *sh_b, u64 *sh_bi)
{
    orc_pool_geom g = pool_geom(H, W, kh, kw, sh, sw, ph, pw);
    size_t cin = planes * (size_t)H * W, cout = planes * (size_t)g.Ho * g.Wo;
    u64 *b = (u64 *)malloc(sizeof(u64) * cin);
    u64 *bi = (u64 *)malloc(sizeof(u64) * cout);
    u64 *cb = (u64 *)malloc(sizeof(u64) * (size_t)t * cin);
    u64 *cbi = (u64 *)malloc(sizeof(u64) * (size_t)t * cout);
    u64 key = orc_key(seed, ORC_DOM_MASK_BETA, stream_id, 0, 0);
    for (size_t pl = 0; pl < planes; pl++) {
        for (int h = 0; h < H; h++)
            for (int w = 0; w < W; w++)
                b[(pl * H + h) * W + w] = (1 + (orc_draw(key, pool_group_in(&g, pl, h, w)) >> 3) % ((u64)1 << bbits)) % p;
        for (int oh = 0; oh < g.Ho; oh++)
            for (int ow = 0; ow < g.Wo; ow++) {
                u64 beta = (1 + (orc_draw(key, pool_group_out(&g, pl, oh, ow)) >> 3) % ((u64)1 << bbits)) % p;
                bi[(pl * g.Ho + oh) * g.Wo + ow] = orc_inv(beta, p);
            }
    }
    orc_draw_coeffs(seed, ORC_DOM_BETA_GEN, stream_id, 0, t, cin, NULL, p, cb);
    orc_draw_coeffs(seed, ORC_DOM_BETAINV_GEN, stream_id, 0, t, cout, NULL, p, cbi);
    orc_share_explicit(b, cb, cin, n, t, p, sh_b);
    orc_share_explicit(bi, cbi, cout, n, t, p, sh_bi);
    free(b); free(bi); free(cb); free(cbi);
}

/* The three steps, with pooling in the elite party's plain part:
 *   1. parties 1..2t+1: m_i = x_i * beta_i                 -> msg [2t+1][planes*H*W]
 *   2. elite party: v = REC(m) = x*beta elementwise; r = max(v, 0) on the
 *      signed value; per kernel position the maximum (mode 0) or the sum
 *      (mode 1; the division of an average has been done by the truncation
 *      before) of r over the kernel's elements inside the image.  Padding
 *      adds nothing to a sum and cannot win a maximum of non-negative values.
 *                                                          -> yplain [planes*Ho*Wo]
 *   3. every party: out_i = y * betainv_i                  -> out [n][planes*Ho*Wo]
 * Requires kh*kw * |x| * beta < p/2. */
void orc_relu_pool(const u64 *x, const u64 *sh_b, const u64 *sh_bi, size_t planes, int H, int W, int kh, int kw,
                   int sh, int sw, int ph, int pw, int mode, int n, int t, u64 p, u64 *msg, u64 *yplain, u64 *out)
{
    orc_pool_geom g = pool_geom(H, W, kh, kw, sh, sw, ph, pw);
    size_t cin = planes * (size_t)H * W, cout = planes * (size_t)g.Ho * g.Wo;
    int nr = 2 * t + 1;
    int ids[ORC_MAXN];
    for (int i = 0; i < nr; i++) ids[i] = i + 1;
    u64 *m = (u64 *)calloc((size_t)n * cin, sizeof(u64));
    u64 *v = (u64 *)malloc(sizeof(u64) * cin);
    u64 *y = (u64 *)malloc(sizeof(u64) * cout);
    for (int i = 0; i < nr; i++)
        for (size_t e = 0; e < cin; e++) {
            m[(size_t)i * cin + e] = orc_mul(x[(size_t)i * cin + e], sh_b[(size_t)i * cin + e], p);
            if (msg) msg[(size_t)i * cin + e] = m[(size_t)i * cin + e];
        }
    orc_reconstruct(m, cin, ids, nr, p, v);
    for (size_t e = 0; e < cin; e++) {
        i64 s = orc_lift1(v[e], p);
        v[e] = s > 0 ? (u64)s : 0;
    }
    for (size_t pl = 0; pl < planes; pl++)
        for (int oh = 0; oh < g.Ho; oh++)
            for (int ow = 0; ow < g.Wo; ow++) {
                u64 acc = 0;
                for (int i = 0; i < kh; i++)
                    for (int j = 0; j < kw; j++) {
                        int h = oh * sh - ph + i, w = ow * sw - pw + j;
                        if (h < 0 || h >= H || w < 0 || w >= W) continue;
                        u64 r = v[(pl * H + h) * W + w];
                        if (mode == 0) acc = r > acc ? r : acc;
                        else acc += r;
                    }
                y[(pl * g.Ho + oh) * g.Wo + ow] = acc % p;
            }
    if (yplain) memcpy(yplain, y, sizeof(u64) * cout);
    for (int i = 0; i < n; i++)
        for (size_t e = 0; e < cout; e++)
            out[(size_t)i * cout + e] = orc_mul(y[e], sh_bi[(size_t)i * cout + e], p);
    free(m); free(v); free(y);
}
