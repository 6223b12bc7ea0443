// C ABI of the library (include/ssnet.h): argument checks, host-side constant
// tables, workspace partitioning, kernel launches.  No arithmetic on share data
// happens on the host.
#include "../../include/ssnet.h"

#include <limits.h>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.hpp"

using namespace SS_NS;

// Message buffer of ssnet_degree_reduce_static, the entry point that allocates nothing: a fixed array in
// the library's device image.  Every GPU the library runs on holds its own copy at its own address until
// the process ends; host code reaches it only through the per-device address taken below.
static __device__ __align__(256) unsigned char scratch[SSNET_STATIC_SCRATCH_BYTES];

struct ssnet_ctx {
    int n, t, f;
    u64 seed;
    hipStream_t stream;
    void *ws;                             // caller's workspace: [reserved header][scratch ... pending product]
    size_t ws_bytes;
    // product shares that a ssnet_*_product_* call left at the end of the workspace as a sum of planes
    struct {
        bool on;
        size_t count;                     // per party
        u64 *base;                        // [planes][n][count]
        int planes;
    } pending;
    int last_hip;
    u64 binv[2 * SS_MAXT + 1][SS_MAXK];   // first k columns of the inverse Vandermonde matrix (Eq. 3)
    u64 lambda_k[SS_MAXK];                // Lagrange multipliers of IDs 1..k (Eq. 2)
    // the same tables as exact small integers over the common denominator D
    int ibinv[2 * SS_MAXT + 1][SS_MAXK];
    int irmat[2 * SS_MAXT + 1][SS_MAXN];
    int ilambda_k[SS_MAXK];
    u64 dinv;
    // optional per-kernel-class timing with HIP events on the context's stream
    bool prof;
    struct span { hipEvent_t a, b; int cls; };
    bool prof_kernels = false;            // also take the product kernels' own start and end (ssnet_profile_begin_kernels)
    std::vector<span> spans;              // recorded since ssnet_profile_begin
    std::vector<span> pool;               // events kept for reuse
};

namespace {

u64 h_pow(u64 a, u64 e)
{
    u64 r = 1;
    while (e) {
        if (e & 1) r = ss_mul(r, a);
        a = ss_mul(a, a);
        e >>= 1;
    }
    return r;
}

u64 h_inv(u64 a) { return h_pow(a, SS_P - 2); }

// Eq. 2 multipliers for an ID set
void h_lagrange(const int *ids, int m, u64 *lambda)
{
    for (int i = 0; i < m; i++) {
        u64 num = 1, den = 1;
        for (int j = 0; j < m; j++) {
            if (j == i) continue;
            num = ss_mul(num, (u64)ids[j]);
            den = ss_mul(den, ss_sub((u64)ids[j], (u64)ids[i]));
        }
        lambda[i] = ss_mul(num, h_inv(den));
    }
}

// Row i of B^-1 holds the coefficients of the Lagrange basis polynomial
// l_i(x) = prod_{l != i} (x - ID_l) / (ID_i - ID_l) over IDs 1..nr, because the
// coefficient vector of the polynomial through the shares c is sum_i c_i l_i.
// Only the k lowest coefficients survive the projection P.
void h_inverse_vandermonde(int nr, int k, u64 (*binv)[SS_MAXK])
{
    for (int i = 0; i < nr; i++) {
        u64 poly[2 * SS_MAXT + 2] = {1};   // running product, ascending powers
        int deg = 0;
        u64 den = 1;
        for (int l = 0; l < nr; l++) {
            if (l == i) continue;
            const u64 root = (u64)(l + 1);
            // poly *= (x - root)
            for (int d = deg + 1; d >= 0; d--) {
                const u64 up = d > 0 ? poly[d - 1] : 0;
                const u64 keep = d <= deg ? ss_mul(poly[d], ss_neg(root)) : 0;
                poly[d] = ss_add(up, keep);
            }
            deg++;
            den = ss_mul(den, ss_sub((u64)(i + 1), root));
        }
        const u64 s = h_inv(den);
        for (int j = 0; j < k; j++) binv[i][j] = ss_mul(poly[j], s);
    }
}

long h_gcd(long a, long b)
{
    a = a < 0 ? -a : a;
    b = b < 0 ? -b : b;
    while (b) {
        const long r = a % b;
        a = b;
        b = r;
    }
    return a;
}

u64 h_from_signed(long v) { return v >= 0 ? (u64)v % SS_P : ss_neg((u64)(-v) % SS_P); }

constexpr long SMALL_LIMIT = 1L << 26;   // magnitude bound of the integer tables (ss_sacc)

// Eq. 2 multipliers as exact integers over a common denominator:
// lambda_i = c[i] / D.  False if a c[i] is too large for the narrow multiply.
bool h_lagrange_int(const int *ids, int m, int *c, u64 *dinv)
{
    long num[SS_MAXN], den[SS_MAXN], D = 1;
    for (int i = 0; i < m; i++) {
        long nu = 1, de = 1;
        for (int j = 0; j < m; j++) {
            if (j == i) continue;
            nu *= ids[j];
            de *= ids[j] - ids[i];
        }
        const long g = h_gcd(nu, de);
        nu /= g;
        de /= g;
        if (de < 0) {
            nu = -nu;
            de = -de;
        }
        num[i] = nu;
        den[i] = de;
        D = D / h_gcd(D, de) * de;
    }
    for (int i = 0; i < m; i++) {
        const long v = num[i] * (D / den[i]);
        if (v >= SMALL_LIMIT || v <= -SMALL_LIMIT) return false;
        c[i] = (int)v;
    }
    *dinv = h_inv((u64)D % SS_P);
    return true;
}

// Integer form of the tables of Eq. 3 for IDs 1..nr: the Lagrange basis
// polynomial of party i is prod_{l != i} (x - l) / prod_{l != i} (i - l), an
// integer polynomial over an integer; D is the least common multiple of the
// denominators.  irmat[i][m] = D * R[i][m] = sum_j ibinv[i][j] (m+1)^j.
bool h_reduction_tables_int(int nr, int k, int n, int (*ibinv)[SS_MAXK], int (*irmat)[SS_MAXN], u64 *dinv)
{
    long poly[2 * SS_MAXT + 1][2 * SS_MAXT + 2], den[2 * SS_MAXT + 1], D = 1;
    for (int i = 0; i < nr; i++) {
        long *pl = poly[i];
        for (int d = 0; d < 2 * SS_MAXT + 2; d++) pl[d] = 0;
        pl[0] = 1;
        int deg = 0;
        den[i] = 1;
        for (int l = 0; l < nr; l++) {
            if (l == i) continue;
            for (int d = deg + 1; d >= 0; d--) pl[d] = (d > 0 ? pl[d - 1] : 0) - (long)(l + 1) * (d <= deg ? pl[d] : 0);
            deg++;
            den[i] *= (i - l);
        }
        const long a = den[i] < 0 ? -den[i] : den[i];
        D = D / h_gcd(D, a) * a;
    }
    for (int i = 0; i < nr; i++) {
        const long scale = D / den[i];   // exact, carries the sign of den[i]
        for (int j = 0; j < k; j++) {
            const long v = poly[i][j] * scale;
            if (v >= SMALL_LIMIT || v <= -SMALL_LIMIT) return false;
            ibinv[i][j] = (int)v;
        }
        for (int m = 0; m < n; m++) {
            long acc = 0;
            for (int j = k - 1; j >= 0; j--) acc = acc * (m + 1) + ibinv[i][j];
            if (acc >= SMALL_LIMIT || acc <= -SMALL_LIMIT) return false;
            irmat[i][m] = (int)acc;
        }
    }
    *dinv = h_inv((u64)D % SS_P);
    return true;
}

int fail_hip(ssnet_ctx *ctx, hipError_t e)
{
    ctx->last_hip = (int)e;
    return SSNET_EHIP;
}

// Brackets the launches of one kernel class with a pair of events while
// profiling is on; costs nothing otherwise.
struct timed {
    ssnet_ctx *ctx;
    ssnet_ctx::span sp;
    bool on;
    timed(ssnet_ctx *c, int cls) : ctx(c), on(c->prof)
    {
        if (!on) return;
        if (!c->pool.empty()) {
            sp = c->pool.back();
            c->pool.pop_back();
        } else if (hipEventCreate(&sp.a) != hipSuccess || hipEventCreate(&sp.b) != hipSuccess) {
            on = false;
            return;
        }
        sp.cls = cls;
        (void)hipEventRecord(sp.a, c->stream);
    }
    ~timed()
    {
        if (!on) return;
        (void)hipEventRecord(sp.b, ctx->stream);
        ctx->spans.push_back(sp);
    }
};

// While profiling is on: an event pair for the product kernel's own start and end (class
// SSNET_PROF_GEMM_KERNEL), handed to the launcher; a, b stay null otherwise.
struct kernel_span {
    ssnet_ctx *ctx;
    ssnet_ctx::span sp;
    bool on;
    kernel_span(ssnet_ctx *c) : ctx(c), on(c->prof && c->prof_kernels)
    {
        sp.a = sp.b = nullptr;
        if (!on) return;
        if (!c->pool.empty()) {
            sp = c->pool.back();
            c->pool.pop_back();
        } else if (hipEventCreate(&sp.a) != hipSuccess || hipEventCreate(&sp.b) != hipSuccess) {
            on = false;
            sp.a = sp.b = nullptr;
            return;
        }
        sp.cls = SSNET_PROF_GEMM_KERNEL;
    }
    hipEvent_t started() const { return on ? sp.a : nullptr; }
    hipEvent_t stopped() const { return on ? sp.b : nullptr; }
    // after the launch: the pair counts only if the launch took it
    void done(hipError_t e)
    {
        if (!on) return;
        if (e == hipSuccess)
            ctx->spans.push_back(sp);
        else
            ctx->pool.push_back(sp);
        on = false;
    }
};

int conv_out(int H, int k, int stride, int pad) { return (H + 2 * pad - k) / stride + 1; }

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

// The first bytes of the workspace are a reserved header (SSNET_WS_HEADER_BYTES); everything else lives
// behind it.
constexpr size_t WS_HEADER_BYTES = SSNET_WS_HEADER_BYTES;

char *ws_scratch(const ssnet_ctx *c) { return (char *)c->ws + WS_HEADER_BYTES; }
bool ws_fits(const ssnet_ctx *c, size_t scratch) { return c->ws && c->ws_bytes >= WS_HEADER_BYTES + scratch; }

// largest element count whose 1-D grid fits
constexpr size_t MAX_COUNT = (size_t)1 << 38;

bool gemm_shape_ok(long rows, long cols, long K)
{
    return rows >= 1 && cols >= 1 && K >= 1 && K <= SSNET_MAX_K && rows <= 16L * 65535 * 2 && cols <= (1L << 30);
}

// A product for a caller that wants the tensor itself: the kernel's planes go to the start of the scratch
// area and one more launch adds them up into d_y; with a single plane the kernel writes d_y directly.
// launch(out, part_stride) enqueues the product kernel.
template <typename F>
int run_product(ssnet_ctx *ctx, u64 *d_y, int rows, int cols, int K, bool planes_operand, F &&launch)
{
    const size_t total = (size_t)ctx->n * rows * cols;
    const int planes = ss_gemm_planes(ctx->n, rows, cols, K, planes_operand);
    timed tm(ctx, SSNET_PROF_GEMM);
    kernel_span ks(ctx);
    hipError_t e = launch(planes > 1 ? (u64 *)ws_scratch(ctx) : d_y, total, ks.started(), ks.stopped());
    ks.done(e);
    if (e == hipSuccess && planes > 1) e = ss_launch_sum_planes(d_y, (const u64 *)ws_scratch(ctx), total, {planes, total}, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int run_gemm(ssnet_ctx *ctx, const void *pa, const void *pb, u64 *out, int rows, int cols, int K,
             size_t out_party_stride, size_t stride_row, int cdiv, size_t stride_cb)
{
    return run_product(ctx, out, rows, cols, K, false, [&](u64 *o, size_t part_stride, hipEvent_t ea, hipEvent_t eb) {
        return ss_launch_gemm(pa, pb, o, part_stride, ctx->n, rows, cols, K, out_party_stride, stride_row, cdiv, stride_cb,
                              ctx->stream, ea, eb);
    });
}

size_t product_bytes(const ssnet_ctx *ctx, int rows, int cols, int K, bool planes_operand)
{
    return align256((size_t)ss_gemm_planes(ctx->n, rows, cols, K, planes_operand) * ctx->n * rows * cols * 8);
}

// Room for a product of `planes` planes at the very end of the workspace; the messages of the call that
// consumes it grow from the front.  nullptr if the workspace is too small.
u64 *reserve_pending(ssnet_ctx *ctx, int rows, int cols, int K, bool planes_operand)
{
    ctx->pending.on = false;
    const size_t bytes = product_bytes(ctx, rows, cols, K, planes_operand);
    if (!ctx->ws || ctx->ws_bytes < WS_HEADER_BYTES + bytes + 256) return nullptr;
    const uintptr_t end = ((uintptr_t)ctx->ws + ctx->ws_bytes) & ~(uintptr_t)255;
    if (end - bytes < (uintptr_t)ws_scratch(ctx)) return nullptr;
    ctx->pending.base = (u64 *)(end - bytes);
    ctx->pending.count = (size_t)rows * cols;
    ctx->pending.planes = ss_gemm_planes(ctx->n, rows, cols, K, planes_operand);
    return ctx->pending.base;
}

// The product shares a reduction reads: the caller's tensor, or (d_c == nullptr) the pending product, which
// must have `count` elements per party and leave `msg_bytes` of the workspace free in front of it.
int incoming_product(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, size_t msg_bytes, const u64 **c, ss_part_src *ps)
{
    if (d_c) {
        if (!ws_fits(ctx, msg_bytes)) return SSNET_EWORKSPACE;
        // a tensor of the caller's may be the pending product's consumer's output: it stays valid
        *c = d_c;
        *ps = {1, 0};
        return SSNET_OK;
    }
    if (!ctx->pending.on || ctx->pending.count != count) return SSNET_EINVAL;
    if ((uintptr_t)ws_scratch(ctx) + msg_bytes > (uintptr_t)ctx->pending.base) return SSNET_EWORKSPACE;
    *c = ctx->pending.base;
    *ps = {ctx->pending.planes, (size_t)ctx->n * count};
    return SSNET_OK;
}

}  // namespace

extern "C" {

int ssnet_create(ssnet_ctx **out, int n, int t, uint64_t p, int f, uint64_t seed, void *hip_stream)
{
    if (!out) return SSNET_EINVAL;
    *out = nullptr;
    if (p != SS_P) return SSNET_EPRIME;
    if (t < 1 || t > SSNET_MAX_T || n < 2 * t + 1 || n > SSNET_MAX_PARTIES || f < 1 || f > 31) return SSNET_EINVAL;
    ssnet_ctx *c = new (std::nothrow) ssnet_ctx();
    if (!c) return SSNET_EINVAL;
    c->n = n;
    c->t = t;
    c->f = f;
    c->seed = seed;
    c->stream = (hipStream_t)hip_stream;
    c->ws = nullptr;
    c->ws_bytes = 0;
    c->pending = {false, 0, nullptr, 0};
    c->last_hip = 0;
    c->prof = false;
    int ids[SS_MAXK];
    for (int q = 0; q <= t; q++) ids[q] = q + 1;
    h_lagrange(ids, t + 1, c->lambda_k);
    h_inverse_vandermonde(2 * t + 1, t + 1, c->binv);
    // integer forms, cross-checked against the field-valued tables computed above by other means
    u64 one = 0;
    bool ok = h_lagrange_int(ids, t + 1, c->ilambda_k, &one) && one == 1 &&
              h_reduction_tables_int(2 * t + 1, t + 1, n, c->ibinv, c->irmat, &c->dinv);
    for (int q = 0; ok && q <= t; q++) ok = h_from_signed(c->ilambda_k[q]) == c->lambda_k[q];
    for (int i = 0; ok && i < 2 * t + 1; i++)
        for (int j = 0; ok && j <= t; j++) ok = ss_mul(h_from_signed(c->ibinv[i][j]), c->dinv) == c->binv[i][j];
    if (!ok) {
        delete c;
        return SSNET_EINVAL;
    }
    *out = c;
    return SSNET_OK;
}

int ssnet_destroy(ssnet_ctx *ctx)
{
    if (!ctx) return SSNET_OK;
    for (auto &v : {&ctx->spans, &ctx->pool})
        for (auto &sp : *v) {
            (void)hipEventDestroy(sp.a);
            (void)hipEventDestroy(sp.b);
        }
    delete ctx;
    return SSNET_OK;
}

int ssnet_profile_begin(ssnet_ctx *ctx)
{
    if (!ctx) return SSNET_EINVAL;
    for (auto &sp : ctx->spans) ctx->pool.push_back(sp);
    ctx->spans.clear();
    ctx->prof = true;
    ctx->prof_kernels = false;
    return SSNET_OK;
}

int ssnet_profile_begin_kernels(ssnet_ctx *ctx)
{
    const int rc = ssnet_profile_begin(ctx);
    if (rc == SSNET_OK) ctx->prof_kernels = true;
    return rc;
}

int ssnet_profile_end(ssnet_ctx *ctx, double *ms_by_class, uint64_t *spans_by_class)
{
    if (!ctx || !ms_by_class || !spans_by_class) return SSNET_EINVAL;
    ctx->prof = false;
    ctx->prof_kernels = false;
    for (int c = 0; c < SSNET_PROF_CLASSES; c++) {
        ms_by_class[c] = 0.0;
        spans_by_class[c] = 0;
    }
    int rc = SSNET_OK;
    for (auto &sp : ctx->spans) {
        float ms = 0.f;
        hipError_t e = hipEventSynchronize(sp.b);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, sp.a, sp.b);
        if (e != hipSuccess) {
            rc = fail_hip(ctx, e);
        } else {
            ms_by_class[sp.cls] += ms;
            spans_by_class[sp.cls] += 1;
        }
        ctx->pool.push_back(sp);
    }
    ctx->spans.clear();
    return rc;
}

size_t ssnet_workspace_bytes_stream(const ssnet_ctx *ctx, size_t count)
{
    if (!ctx) return 0;
    const size_t k = ctx->t + 1, nr = 2 * ctx->t + 1, n = ctx->n;
    // the fused call keeps the messages of both protocols at once
    return WS_HEADER_BYTES + align256((nr * k + k * n + k + n) * count * 8);
}

size_t ssnet_workspace_bytes_linear(const ssnet_ctx *ctx, int M, int K, int N)
{
    if (!ctx || M < 1 || K < 1 || N < 1) return 0;
    return WS_HEADER_BYTES + align256(ss_gemm_scratch_bytes(ctx->n, M, N, K)) +
           (size_t)ctx->n * (ss_packed_bytes(M, K) + ss_packed_bytes(N, K));
}

size_t ssnet_workspace_bytes_conv(const ssnet_ctx *ctx, int B, int C, int H, int W, int Co, int kh, int kw, int stride,
                                  int pad)
{
    if (!ctx || B < 1 || C < 1 || Co < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0) return 0;
    const int Ho = conv_out(H, kh, stride, pad), Wo = conv_out(W, kw, stride, pad);
    if (Ho < 1 || Wo < 1) return 0;
    const long M = (long)B * Ho * Wo, K = (long)C * kh * kw;
    if (M > INT_MAX || K > INT_MAX) return 0;
    return WS_HEADER_BYTES + align256(ss_gemm_scratch_bytes(ctx->n, Co, (int)M, (int)K)) +
           (size_t)ctx->n * (ss_packed_bytes((int)M, (int)K) + ss_packed_bytes(Co, (int)K));
}

int ssnet_set_workspace(ssnet_ctx *ctx, void *d_workspace, size_t bytes)
{
    if (!ctx || (!d_workspace && bytes) || ((uintptr_t)d_workspace & 15)) return SSNET_EINVAL;
    ctx->ws = d_workspace;
    ctx->ws_bytes = bytes;
    ctx->pending.on = false;
    return SSNET_OK;
}

int ssnet_share(ssnet_ctx *ctx, const uint64_t *d_secret, size_t count, int degree, uint64_t stream_id,
                uint64_t *d_shares)
{
    if (!ctx || !d_secret || !d_shares || count == 0 || count > MAX_COUNT) return SSNET_EINVAL;
    if (degree < 0 || degree > 2 * ctx->t || degree > ctx->n - 1) return SSNET_EINVAL;
    ss_keys keys = {};
    for (int j = 1; j <= degree; j++) keys.k[j - 1] = ss_key(ctx->seed, SSNET_DOM_SHARE, stream_id, 0, (u64)j);
    timed tm(ctx, SSNET_PROF_SHARE);
    hipError_t e = ss_launch_share(d_secret, d_shares, count, ctx->n, degree, keys, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_share_packed(ssnet_ctx *ctx, const uint64_t *d_secret, int B, int K, int HW, uint64_t stream_id,
                       uint64_t *d_shares, void *d_packed)
{
    if (!ctx || !d_secret || !d_shares || !d_packed || ((uintptr_t)d_packed & 15)) return SSNET_EINVAL;
    if (B < 1 || HW < 1 || (long)B * HW > (1L << 30) || !gemm_shape_ok((long)B * HW, 1, K)) return SSNET_EINVAL;
    if ((size_t)B * K * HW > MAX_COUNT) return SSNET_EINVAL;
    ss_keys keys = {};
    for (int j = 1; j <= ctx->t; j++) keys.k[j - 1] = ss_key(ctx->seed, SSNET_DOM_SHARE, stream_id, 0, (u64)j);
    timed tm(ctx, SSNET_PROF_SHARE);
    hipError_t e = ss_launch_share_pack(d_secret, d_shares, d_packed, ctx->n, ctx->t, B, K, HW, keys, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_reconstruct(ssnet_ctx *ctx, const uint64_t *d_shares, size_t count, const int *party_ids, int m, int degree,
                      uint64_t *d_secret)
{
    if (!ctx || !d_shares || !d_secret || !party_ids || count == 0 || count > MAX_COUNT) return SSNET_EINVAL;
    if (degree < 0 || degree > 2 * ctx->t || m < 1 || m > ctx->n) return SSNET_EINVAL;
    for (int i = 0; i < m; i++) {
        if (party_ids[i] < 1 || party_ids[i] > ctx->n) return SSNET_EID;
        for (int j = 0; j < i; j++)
            if (party_ids[j] == party_ids[i]) return SSNET_EID;
    }
    if (m < degree + 1) return SSNET_ESHARES;
    ss_rec_params rp = {};
    rp.m = m;
    for (int i = 0; i < m; i++) rp.plane[i] = party_ids[i] - 1;
    if (!h_lagrange_int(party_ids, m, rp.ilambda, &rp.dinv)) return SSNET_EINVAL;
    timed tm(ctx, SSNET_PROF_RECONSTRUCT);
    hipError_t e = ss_launch_reconstruct(d_shares, d_secret, count, rp, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

size_t ssnet_packed_weight_bytes(int rows, int K)
{
    if (rows < 1 || K < 1) return 0;
    return ss_packed_bytes(rows, K);
}

int ssnet_pack_weights_linear(ssnet_ctx *ctx, const uint64_t *d_w, int K, int N, void *d_packed)
{
    if (!ctx || !d_w || !d_packed || !gemm_shape_ok(N, 1, K) || ((uintptr_t)d_packed & 15)) return SSNET_EINVAL;
    // row = output column c of w [K][N], contraction index strides by N
    timed tm(ctx, SSNET_PROF_PACK_W);
    hipError_t e = ss_launch_pack_matrix(d_w, d_packed, ctx->n, N, K, (size_t)K * N, 1, (size_t)N, 0, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_pack_weights_conv(ssnet_ctx *ctx, const uint64_t *d_w, int Co, int CKK, void *d_packed)
{
    if (!ctx || !d_w || !d_packed || !gemm_shape_ok(Co, 1, CKK) || ((uintptr_t)d_packed & 15)) return SSNET_EINVAL;
    timed tm(ctx, SSNET_PROF_PACK_W);
    hipError_t e = ss_launch_pack_matrix(d_w, d_packed, ctx->n, Co, CKK, (size_t)Co * CKK, (size_t)CKK, 1, 0, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_linear_mod_packed(ssnet_ctx *ctx, const uint64_t *d_x, const void *d_w_packed, int M, int K, int N,
                            uint64_t *d_y)
{
    if (!ctx || !d_x || !d_w_packed || !d_y || !gemm_shape_ok(M, N, K)) return SSNET_EINVAL;
    const size_t part = align256(ss_gemm_scratch_bytes(ctx->n, M, N, K));
    if (!ws_fits(ctx, part + (size_t)ctx->n * ss_packed_bytes(M, K))) return SSNET_EWORKSPACE;
    void *px = ws_scratch(ctx) + part;
    {
        timed tm(ctx, SSNET_PROF_PACK_X);
        hipError_t e = ss_launch_pack_matrix(d_x, px, ctx->n, M, K, (size_t)M * K, (size_t)K, 1, 0, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e);
    }
    return run_gemm(ctx, px, d_w_packed, d_y, M, N, K, (size_t)M * N, (size_t)N, INT_MAX, 0);
}

int ssnet_linear_mod_prepacked(ssnet_ctx *ctx, const void *d_x_packed, const void *d_w_packed, int M, int K, int N,
                               uint64_t *d_y)
{
    if (!ctx || !d_x_packed || !d_w_packed || !d_y || !gemm_shape_ok(M, N, K)) return SSNET_EINVAL;
    if (!ws_fits(ctx, align256(ss_gemm_scratch_bytes(ctx->n, M, N, K)))) return SSNET_EWORKSPACE;
    return run_gemm(ctx, d_x_packed, d_w_packed, d_y, M, N, K, (size_t)M * N, (size_t)N, INT_MAX, 0);
}

int ssnet_conv1x1_mod_prepacked(ssnet_ctx *ctx, const void *d_x_packed, const void *d_w_packed, int B, int C, int HW,
                                int Co, uint64_t *d_y)
{
    if (!ctx || !d_x_packed || !d_w_packed || !d_y || B < 1 || HW < 1 || (long)B * HW > (1L << 30) ||
        !gemm_shape_ok(Co, (long)B * HW, C))
        return SSNET_EINVAL;
    const int M = B * HW;
    if (!ws_fits(ctx, align256(ss_gemm_scratch_bytes(ctx->n, Co, M, C)))) return SSNET_EWORKSPACE;
    // rows = output channel, cols = (b, hw): y[b][co][hw]
    return run_gemm(ctx, d_w_packed, d_x_packed, d_y, Co, M, C, (size_t)B * Co * HW, (size_t)HW, HW, (size_t)Co * HW);
}

namespace {

static bool planes_shape_ok(long B, long C, long H, long W)
{
    return B >= 1 && C >= 64 && C % 64 == 0 && H >= 1 && W >= 1 && H < 32768 && W < 32768 && B * H * W < (1L << 30) &&
           B * H * W * C < (1L << 35);
}

}  // namespace

size_t ssnet_conv_planes_bytes(int B, int C, int H, int W)
{
    return planes_shape_ok(B, C, H, W) ? ss_planes_bytes(B, C, H, W) : 0;
}

int ssnet_share_planes(ssnet_ctx *ctx, const uint64_t *d_secret, int B, int C, int H, int W, uint64_t stream_id,
                       uint64_t *d_shares, void *d_planes)
{
    if (!ctx || !d_secret || !d_shares || !d_planes || ((uintptr_t)d_planes & 15) || !planes_shape_ok(B, C, H, W))
        return SSNET_EINVAL;
    if ((size_t)B * C * H * W > MAX_COUNT) return SSNET_EINVAL;
    ss_keys keys = {};
    for (int j = 1; j <= ctx->t; j++) keys.k[j - 1] = ss_key(ctx->seed, SSNET_DOM_SHARE, stream_id, 0, (u64)j);
    timed tm(ctx, SSNET_PROF_SHARE);
    hipError_t e = ss_launch_planes(d_secret, d_shares, d_planes, ctx->n, ctx->t, B, C, H * W, true, keys, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_split_planes(ssnet_ctx *ctx, const uint64_t *d_x, int B, int C, int H, int W, void *d_planes)
{
    if (!ctx || !d_x || !d_planes || ((uintptr_t)d_planes & 15) || !planes_shape_ok(B, C, H, W)) return SSNET_EINVAL;
    const ss_keys none = {};
    timed tm(ctx, SSNET_PROF_PACK_X);
    hipError_t e = ss_launch_planes(d_x, nullptr, d_planes, ctx->n, ctx->t, B, C, H * W, false, none, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_pack_weights_conv_taps(ssnet_ctx *ctx, const uint64_t *d_w, int Co, int C, int kh, int kw, void *d_packed)
{
    if (!ctx || !d_w || !d_packed || ((uintptr_t)d_packed & 15) || C < 1 || kh < 1 || kw < 1 ||
        !gemm_shape_ok(Co, 1, (long)C * kh * kw))
        return SSNET_EINVAL;
    const int K = C * kh * kw;
    timed tm(ctx, SSNET_PROF_PACK_W);
    hipError_t e = ss_launch_pack_matrix(d_w, d_packed, ctx->n, Co, K, (size_t)Co * K, (size_t)K, 1, kh * kw, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_conv_mod_planes(ssnet_ctx *ctx, const void *d_planes, const void *d_w_packed, int B, int C, int H, int W, int Co,
                          int kh, int kw, int stride, int pad, uint64_t *d_y)
{
    if (!ctx || !d_planes || !d_w_packed || !d_y || !planes_shape_ok(B, C, H, W) || Co < 1 || kh < 1 || kw < 1 ||
        stride < 1 || pad < 0 || pad >= 32768)
        return SSNET_EINVAL;
    const int Ho = conv_out(H, kh, stride, pad), Wo = conv_out(W, kw, stride, pad);
    if (Ho < 1 || Wo < 1) return SSNET_EINVAL;
    const long M = (long)B * Ho * Wo, K = (long)C * kh * kw;
    if (!gemm_shape_ok(Co, M, K)) return SSNET_EINVAL;
    if (!ws_fits(ctx, align256(ss_gemm_scratch_bytes(ctx->n, Co, (int)M, (int)K)))) return SSNET_EWORKSPACE;
    return run_product(ctx, d_y, Co, (int)M, (int)K, true, [&](u64 *o, size_t part_stride, hipEvent_t ea, hipEvent_t eb) {
        return ss_launch_gemm_conv(d_w_packed, d_planes, o, part_stride, ctx->n, B, C, H, W, Co, kh, kw, stride, pad, Ho, Wo,
                                   ctx->stream, ea, eb);
    });
}

size_t ssnet_product_bytes_linear(const ssnet_ctx *ctx, int M, int K, int N)
{
    if (!ctx || !gemm_shape_ok(M, N, K)) return 0;
    return product_bytes(ctx, M, N, K, false);
}

size_t ssnet_product_bytes_conv(const ssnet_ctx *ctx, int B, int C, int H, int W, int Co, int kh, int kw, int stride,
                                int pad)
{
    if (!ctx || B < 1 || C < 1 || H < 1 || W < 1 || Co < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0) return 0;
    const int Ho = conv_out(H, kh, stride, pad), Wo = conv_out(W, kw, stride, pad);
    if (H + 2 * pad < kh || W + 2 * pad < kw || Ho < 1 || Wo < 1) return 0;
    const long M = (long)B * Ho * Wo, K = (long)C * kh * kw;
    if (!gemm_shape_ok(Co, M, K)) return 0;
    const size_t a = product_bytes(ctx, Co, (int)M, (int)K, false), b = product_bytes(ctx, Co, (int)M, (int)K, true);
    return a > b ? a : b;
}

int ssnet_linear_product_prepacked(ssnet_ctx *ctx, const void *d_x_packed, const void *d_w_packed, int M, int K, int N)
{
    if (!ctx || !d_x_packed || !d_w_packed || !gemm_shape_ok(M, N, K)) return SSNET_EINVAL;
    u64 *parts = reserve_pending(ctx, M, N, K, false);
    if (!parts) return SSNET_EWORKSPACE;
    timed tm(ctx, SSNET_PROF_GEMM);
    kernel_span ks(ctx);
    hipError_t e = ss_launch_gemm(d_x_packed, d_w_packed, parts, (size_t)ctx->n * M * N, ctx->n, M, N, K, (size_t)M * N,
                                  (size_t)N, INT_MAX, 0, ctx->stream, ks.started(), ks.stopped());
    ks.done(e);
    ctx->pending.on = e == hipSuccess;
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_conv1x1_product_prepacked(ssnet_ctx *ctx, const void *d_x_packed, const void *d_w_packed, int B, int C, int HW,
                                    int Co)
{
    if (!ctx || !d_x_packed || !d_w_packed || B < 1 || HW < 1 || (long)B * HW > (1L << 30) ||
        !gemm_shape_ok(Co, (long)B * HW, C))
        return SSNET_EINVAL;
    const int M = B * HW;
    u64 *parts = reserve_pending(ctx, Co, M, C, false);
    if (!parts) return SSNET_EWORKSPACE;
    timed tm(ctx, SSNET_PROF_GEMM);
    kernel_span ks(ctx);
    hipError_t e = ss_launch_gemm(d_w_packed, d_x_packed, parts, (size_t)ctx->n * Co * M, ctx->n, Co, M, C,
                                  (size_t)B * Co * HW, (size_t)HW, HW, (size_t)Co * HW, ctx->stream, ks.started(),
                                  ks.stopped());
    ks.done(e);
    ctx->pending.on = e == hipSuccess;
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_conv_product_planes(ssnet_ctx *ctx, const void *d_planes, const void *d_w_packed, int B, int C, int H, int W,
                              int Co, int kh, int kw, int stride, int pad)
{
    if (!ctx || !d_planes || !d_w_packed || !planes_shape_ok(B, C, H, W) || Co < 1 || kh < 1 || kw < 1 || stride < 1 ||
        pad < 0 || pad >= 32768)
        return SSNET_EINVAL;
    const int Ho = conv_out(H, kh, stride, pad), Wo = conv_out(W, kw, stride, pad);
    if (Ho < 1 || Wo < 1) return SSNET_EINVAL;
    const long M = (long)B * Ho * Wo, K = (long)C * kh * kw;
    if (!gemm_shape_ok(Co, M, K)) return SSNET_EINVAL;
    u64 *parts = reserve_pending(ctx, Co, (int)M, (int)K, true);
    if (!parts) return SSNET_EWORKSPACE;
    timed tm(ctx, SSNET_PROF_GEMM);
    kernel_span ks(ctx);
    hipError_t e = ss_launch_gemm_conv(d_w_packed, d_planes, parts, (size_t)ctx->n * Co * M, ctx->n, B, C, H, W, Co, kh, kw,
                                       stride, pad, Ho, Wo, ctx->stream, ks.started(), ks.stopped());
    ks.done(e);
    ctx->pending.on = e == hipSuccess;
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_linear_mod(ssnet_ctx *ctx, const uint64_t *d_x, const uint64_t *d_w, int M, int K, int N, uint64_t *d_y)
{
    if (!ctx || !d_x || !d_w || !d_y || !gemm_shape_ok(M, N, K)) return SSNET_EINVAL;
    const size_t part = align256(ss_gemm_scratch_bytes(ctx->n, M, N, K));
    const size_t xa = (size_t)ctx->n * ss_packed_bytes(M, K), wa = (size_t)ctx->n * ss_packed_bytes(N, K);
    if (!ws_fits(ctx, part + xa + wa)) return SSNET_EWORKSPACE;
    void *pw = ws_scratch(ctx) + part + xa;
    int rc = ssnet_pack_weights_linear(ctx, d_w, K, N, pw);
    if (rc) return rc;
    return ssnet_linear_mod_packed(ctx, d_x, pw, M, K, N, d_y);
}

int ssnet_conv_mod_packed(ssnet_ctx *ctx, const uint64_t *d_x, const void *d_w_packed, int B, int C, int H, int W,
                          int Co, int kh, int kw, int stride, int pad, uint64_t *d_y)
{
    if (!ctx || !d_x || !d_w_packed || !d_y || B < 1 || C < 1 || H < 1 || W < 1 || Co < 1 || kh < 1 || kw < 1 ||
        stride < 1 || pad < 0)
        return SSNET_EINVAL;
    const int Ho = conv_out(H, kh, stride, pad), Wo = conv_out(W, kw, stride, pad);
    if (H + 2 * pad < kh || W + 2 * pad < kw || Ho < 1 || Wo < 1) return SSNET_EINVAL;
    const long M = (long)B * Ho * Wo, K = (long)C * kh * kw;
    if (M > (1L << 30) || !gemm_shape_ok(Co, M, K)) return SSNET_EINVAL;
    const size_t part = align256(ss_gemm_scratch_bytes(ctx->n, Co, (int)M, (int)K));
    if (!ws_fits(ctx, part + (size_t)ctx->n * ss_packed_bytes((int)M, (int)K))) return SSNET_EWORKSPACE;
    void *px = ws_scratch(ctx) + part;
    {
        timed tm(ctx, SSNET_PROF_PACK_X);
        hipError_t e = ss_launch_pack_im2col(d_x, px, ctx->n, B, C, H, W, kh, kw, stride, pad, Ho, Wo, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e);
    }
    const size_t HW = (size_t)Ho * Wo;
    // rows = output channel, cols = (b, ho, wo): y[b][co][hw]
    return run_gemm(ctx, d_w_packed, px, d_y, Co, (int)M, (int)K, (size_t)B * Co * HW, HW, (int)HW, (size_t)Co * HW);
}

int ssnet_conv_mod(ssnet_ctx *ctx, const uint64_t *d_x, const uint64_t *d_w, int B, int C, int H, int W, int Co, int kh,
                   int kw, int stride, int pad, uint64_t *d_y)
{
    if (!ctx || !d_w) return SSNET_EINVAL;
    const size_t total = ssnet_workspace_bytes_conv(ctx, B, C, H, W, Co, kh, kw, stride, pad);
    if (total == 0) return SSNET_EINVAL;
    if (!ctx->ws || ctx->ws_bytes < total) return SSNET_EWORKSPACE;
    const long K = (long)C * kh * kw;
    if (K > SSNET_MAX_K) return SSNET_EINVAL;
    void *pw = (char *)ctx->ws + (total - (size_t)ctx->n * ss_packed_bytes(Co, (int)K));   // last part of the layout
    int rc = ssnet_pack_weights_conv(ctx, d_w, Co, (int)K, pw);
    if (rc) return rc;
    return ssnet_conv_mod_packed(ctx, d_x, pw, B, C, H, W, Co, kh, kw, stride, pad, d_y);
}

namespace {

static ss_dr_params make_dr_params(const ssnet_ctx *ctx, uint64_t stream_id)
{
    const int t = ctx->t, k = t + 1, nr = 2 * t + 1, n = ctx->n;
    ss_dr_params dp = {};
    dp.n = n;
    dp.t = t;
    for (int i = 0; i < nr; i++)
        for (int j = 1; j <= t; j++)
            dp.reshare_key[i][j - 1] = ss_key(ctx->seed, SSNET_DOM_RESHARE, stream_id, (u64)(i + 1), (u64)j);
    for (int j = 1; j <= t; j++) dp.zero_key[j - 1] = ss_key(ctx->seed, SSNET_DOM_ZERO, stream_id, 0, (u64)j);
    for (int i = 0; i < nr; i++) {
        for (int j = 0; j < k; j++) dp.ibinv[i][j] = ctx->ibinv[i][j];
        for (int m = 0; m < n; m++) dp.irmat[i][m] = ctx->irmat[i][m];
    }
    dp.dinv = ctx->dinv;
    for (int q = 0; q < k; q++) dp.ilambda[q] = ctx->ilambda_k[q];
    return dp;
}

static ss_tr_params make_tr_params(const ssnet_ctx *ctx, uint64_t stream_id)
{
    const int t = ctx->t;
    ss_tr_params tp = {};
    tp.n = ctx->n;
    tp.t = t;
    tp.f = ctx->f;
    tp.kdiv = 1;
    tp.e_range = 1u << (32 - ctx->f);
    tp.e_key = ss_key(ctx->seed, SSNET_DOM_MASK_E, stream_id, 0, 0);
    for (int j = 1; j <= t; j++) {
        tp.alpha_key[j - 1] = ss_key(ctx->seed, SSNET_DOM_MASK_ALPHA, stream_id, 0, (u64)j);
        tp.alphat_key[j - 1] = ss_key(ctx->seed, SSNET_DOM_MASK_ALPHAT, stream_id, 0, (u64)j);
        tp.gen_key[j - 1] = ss_key(ctx->seed, SSNET_DOM_TRUNC_GEN, stream_id, 0, (u64)j);
    }
    for (int q = 0; q <= t; q++) tp.ilambda[q] = ctx->ilambda_k[q];
    return tp;
}

}  // namespace

int ssnet_degree_reduce(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id, uint64_t *d_out)
{
    if (!ctx || !d_out || count == 0 || count > MAX_COUNT) return SSNET_EINVAL;
    const int k = ctx->t + 1, nr = 2 * ctx->t + 1, n = ctx->n;
    const size_t need = ((size_t)nr * k + (size_t)k * n) * count * 8;
    const u64 *c;
    ss_part_src ps;
    if (int rc = incoming_product(ctx, d_c, count, need, &c, &ps)) return rc;
    u64 *msg1 = (u64 *)ws_scratch(ctx), *msg2 = msg1 + (size_t)nr * k * count;
    timed tm(ctx, SSNET_PROF_DEGREE_REDUCE);
    hipError_t e = ss_launch_degree_reduce(c, msg1, msg2, d_out, count, make_dr_params(ctx, stream_id), ps, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

namespace {

// device address of `scratch` on the current device, looked up once per device
hipError_t static_scratch(void **out)
{
    constexpr int MAX_DEVICES = 64;
    static void *ptr[MAX_DEVICES];   // zero-initialised
    static std::mutex lock;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> guard(lock);
    if (!ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return hipSuccess;
}

}  // namespace

int ssnet_degree_reduce_static(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id, uint64_t *d_out)
{
    if (!ctx || !d_c || !d_out || count == 0 || count > MAX_COUNT) return SSNET_EINVAL;
    const int k = ctx->t + 1, nr = 2 * ctx->t + 1, n = ctx->n;
    const size_t words = (size_t)nr * k + (size_t)k * n;
    if (count > SSNET_STATIC_SCRATCH_BYTES / 8 / words) return SSNET_ESCRATCH;
    void *base = nullptr;
    hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return fail_hip(ctx, e);
    // both message arrays are written in full by the launch before anything reads them: nothing to clear
    u64 *msg1 = (u64 *)base, *msg2 = msg1 + (size_t)nr * k * count;
    e = ss_launch_degree_reduce(d_c, msg1, msg2, d_out, count, make_dr_params(ctx, stream_id), {1, 0}, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

namespace {

// the divisor of average pooling leaves at least one value of e: kdiv <= 2^(32-f) (Sec. VII-B)
static bool kdiv_fits(const ssnet_ctx *ctx, int kdiv)
{
    return kdiv >= 1 && kdiv <= SSNET_MAX_KDIV && (unsigned)kdiv <= (1u << (32 - ctx->f));
}

static void set_kdiv(const ssnet_ctx *ctx, ss_tr_params &tp, int kdiv)
{
    tp.kdiv = kdiv;
    tp.e_range = (1u << (32 - ctx->f)) / (unsigned)kdiv;
}

static int truncate_by(ssnet_ctx *ctx, const uint64_t *d_x, size_t count, int kdiv, uint64_t stream_id, uint64_t *d_out)
{
    if (!ctx || !d_x || !d_out || count == 0 || count > MAX_COUNT || !kdiv_fits(ctx, kdiv)) return SSNET_EINVAL;
    const int k = ctx->t + 1, n = ctx->n;
    const size_t need = ((size_t)k + n) * count * 8;
    if (!ws_fits(ctx, need)) return SSNET_EWORKSPACE;
    u64 *u = (u64 *)ws_scratch(ctx), *wsh = u + (size_t)k * count;
    ss_tr_params tp = make_tr_params(ctx, stream_id);
    set_kdiv(ctx, tp, kdiv);
    timed tm(ctx, SSNET_PROF_TRUNCATE);
    hipError_t e = ss_launch_truncate(d_x, u, wsh, d_out, count, tp, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

}  // namespace

int ssnet_truncate(ssnet_ctx *ctx, const uint64_t *d_x, size_t count, uint64_t stream_id, uint64_t *d_out)
{
    return truncate_by(ctx, d_x, count, 1, stream_id, d_out);
}

int ssnet_truncate_div(ssnet_ctx *ctx, const uint64_t *d_x, size_t count, int kdiv, uint64_t stream_id,
                       uint64_t *d_out)
{
    return truncate_by(ctx, d_x, count, kdiv, stream_id, d_out);
}

namespace {

// shared by the two fused entry points; d_rec == nullptr: no reconstruction
static int degree_reduce_truncate(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id, uint64_t *d_out,
                           const int *party_ids, int m, uint64_t *d_rec, int kdiv = 1)
{
    if (!ctx || !d_out || count == 0 || count > MAX_COUNT || !kdiv_fits(ctx, kdiv)) return SSNET_EINVAL;
    ss_recf_params rf = {};
    if (d_rec) {
        if (!party_ids || m < 1 || m > ctx->n) return SSNET_EINVAL;
        for (int i = 0; i < m; i++) {
            if (party_ids[i] < 1 || party_ids[i] > ctx->n) return SSNET_EID;
            for (int j = 0; j < i; j++)
                if (party_ids[j] == party_ids[i]) return SSNET_EID;
        }
        if (m < ctx->t + 1) return SSNET_ESHARES;
        int il[SS_MAXN];
        if (!h_lagrange_int(party_ids, m, il, &rf.dinv)) return SSNET_EINVAL;
        for (int i = 0; i < m; i++) rf.coef[party_ids[i] - 1] = il[i];
    }
    const int k = ctx->t + 1, nr = 2 * ctx->t + 1, n = ctx->n;
    const size_t need = ((size_t)nr * k + (size_t)k * n + k + n) * count * 8;
    const u64 *c;
    ss_part_src ps;
    if (int rc = incoming_product(ctx, d_c, count, need, &c, &ps)) return rc;
    u64 *msg1 = (u64 *)ws_scratch(ctx), *msg2 = msg1 + (size_t)nr * k * count;
    u64 *u = msg2 + (size_t)k * n * count, *wsh = u + (size_t)k * count;
    ss_tr_params tp = make_tr_params(ctx, stream_id);
    set_kdiv(ctx, tp, kdiv);
    timed tm(ctx, SSNET_PROF_DEGREE_REDUCE);
    hipError_t e = ss_launch_degree_reduce_truncate(c, msg1, msg2, u, wsh, d_out, d_rec, count,
                                                    make_dr_params(ctx, stream_id), tp, rf, ps, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

}  // namespace

int ssnet_degree_reduce_truncate(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id,
                                 uint64_t *d_out)
{
    return degree_reduce_truncate(ctx, d_c, count, stream_id, d_out, nullptr, 0, nullptr);
}

int ssnet_degree_reduce_truncate_div(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, int kdiv, uint64_t stream_id,
                                     uint64_t *d_out)
{
    return degree_reduce_truncate(ctx, d_c, count, stream_id, d_out, nullptr, 0, nullptr, kdiv);
}

int ssnet_degree_reduce_truncate_reconstruct(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id,
                                             uint64_t *d_out, const int *party_ids, int m, uint64_t *d_secret)
{
    if (!d_secret) return SSNET_EINVAL;
    return degree_reduce_truncate(ctx, d_c, count, stream_id, d_out, party_ids, m, d_secret);
}

namespace {

static bool make_nl_params(const ssnet_ctx *ctx, uint64_t stream_id, ss_nl_params *np)
{
    *np = {};
    np->n = ctx->n;
    np->t = ctx->t;
    np->bbits = SSNET_BETA_BITS;
    np->beta_key = ss_key(ctx->seed, SSNET_DOM_MASK_BETA, stream_id, 0, 0);
    for (int j = 1; j <= ctx->t; j++) {
        np->bgen_key[j - 1] = ss_key(ctx->seed, SSNET_DOM_BETA_GEN, stream_id, 0, (u64)j);
        np->bigen_key[j - 1] = ss_key(ctx->seed, SSNET_DOM_BETAINV_GEN, stream_id, 0, (u64)j);
    }
    int ids[2 * SS_MAXT + 1];
    for (int i = 0; i < 2 * ctx->t + 1; i++) ids[i] = i + 1;
    return h_lagrange_int(ids, 2 * ctx->t + 1, np->ilambda, &np->dinv);
}

}  // namespace

int ssnet_reduce_truncate_direct(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id,
                                 uint64_t *d_out, const int *party_ids, int m, uint64_t *d_secret)
{
    if (!ctx || !d_out || count == 0 || count > MAX_COUNT) return SSNET_EINVAL;
    ss_recf_params rf = {};
    if (d_secret) {
        if (!party_ids || m < 1 || m > ctx->n) return SSNET_EINVAL;
        for (int i = 0; i < m; i++) {
            if (party_ids[i] < 1 || party_ids[i] > ctx->n) return SSNET_EID;
            for (int j = 0; j < i; j++)
                if (party_ids[j] == party_ids[i]) return SSNET_EID;
        }
        if (m < ctx->t + 1) return SSNET_ESHARES;
        int il[SS_MAXN];
        if (!h_lagrange_int(party_ids, m, il, &rf.dinv)) return SSNET_EINVAL;
        for (int i = 0; i < m; i++) rf.coef[party_ids[i] - 1] = il[i];
    }
    ss_nl_params open_all;
    if (!make_nl_params(ctx, 0, &open_all)) return SSNET_EINVAL;
    const u64 *c = d_c;
    if (!d_c) {   // the pending product: this kernel reads one plane, so the planes are summed first
        ss_part_src ps;
        if (int rc = incoming_product(ctx, nullptr, count, 0, &c, &ps)) return rc;
        timed tm(ctx, SSNET_PROF_DEGREE_REDUCE);
        hipError_t e = ss_launch_sum_planes(ctx->pending.base, ctx->pending.base, (size_t)ctx->n * count, ps, ctx->stream);
        if (e != hipSuccess) return fail_hip(ctx, e);
        ctx->pending.planes = 1;
    }
    timed tm(ctx, SSNET_PROF_DEGREE_REDUCE);
    hipError_t e = ss_launch_reduce_truncate_direct(c, d_out, d_secret, count, open_all, make_tr_params(ctx, stream_id),
                                                    rf, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

namespace {

// positions per message plane of the layer-tail call: the threads of its one-launch kernel (blocks of 16
// pixels x 16 channels), or the elements themselves where the separate kernels run
static size_t tail_plane(const ssnet_ctx *ctx, int B, int C, int HW)
{
    const bool fused = (ctx->n == 5 && ctx->t == 2) || (ctx->n == 3 && ctx->t == 1);
    return fused ? (size_t)((B * HW + 15) / 16) * ((C + 15) / 16) * 256 : (size_t)B * C * HW;
}

}  // namespace

size_t ssnet_layer_tail_message_plane(const ssnet_ctx *ctx, int B, int C, int HW)
{
    if (!ctx || B < 1 || C < 1 || HW < 1 || (long)B * HW >= (1L << 30) || (size_t)B * C * HW > MAX_COUNT) return 0;
    return tail_plane(ctx, B, C, HW);
}

size_t ssnet_workspace_bytes_layer_tail(const ssnet_ctx *ctx, int B, int C, int HW)
{
    const size_t plane = ssnet_layer_tail_message_plane(ctx, B, C, HW);
    if (!plane) return 0;
    const size_t k = ctx->t + 1, nr = 2 * ctx->t + 1, n = ctx->n;
    return WS_HEADER_BYTES + align256((nr * k + k * n + k + n + nr + 1) * plane * 8);
}

int ssnet_reduce_truncate_relu(ssnet_ctx *ctx, const uint64_t *d_c, int B, int C, int HW, uint64_t stream_id,
                               const uint64_t *d_beta, const uint64_t *d_betainv, uint64_t *d_out, void *d_planes)
{
    if (!ctx || !d_beta || !d_betainv || !d_out || B < 1 || C < 1 || HW < 1) return SSNET_EINVAL;
    if ((long)B * HW >= (1L << 30) || (size_t)B * C * HW > MAX_COUNT) return SSNET_EINVAL;
    if (d_planes && (((uintptr_t)d_planes & 15) || C % 64 != 0)) return SSNET_EINVAL;
    const size_t count = (size_t)B * C * HW, plane = tail_plane(ctx, B, C, HW);
    const int k = ctx->t + 1, nr = 2 * ctx->t + 1, n = ctx->n;
    const u64 *c;
    ss_part_src ps;
    if (int rc = incoming_product(ctx, d_c, count, ((size_t)nr * k + (size_t)k * n + k + n + nr + 1) * plane * 8, &c, &ps))
        return rc;
    u64 *msg1 = (u64 *)ws_scratch(ctx), *msg2 = msg1 + (size_t)nr * k * plane;
    u64 *u = msg2 + (size_t)k * n * plane, *wsh = u + (size_t)k * plane;
    u64 *rmsg = wsh + (size_t)n * plane, *yplain = rmsg + (size_t)nr * plane;
    ss_nl_params np;
    if (!make_nl_params(ctx, 0, &np)) return SSNET_EINVAL;
    const ss_dr_params dp = make_dr_params(ctx, stream_id);
    const ss_tr_params tp = make_tr_params(ctx, stream_id);
    hipError_t e;
    if ((n == 5 && ctx->t == 2) || (n == 3 && ctx->t == 1)) {
        // from half a million elements on, the planes are written faster by the kernel that takes four
        // channels per thread than by the tail's one-element threads
        const bool planes_apart = d_planes && count >= ((size_t)1 << 19);
        {
            timed tm(ctx, SSNET_PROF_DEGREE_REDUCE);
            e = ss_launch_layer_tail(c, msg1, msg2, u, wsh, rmsg, yplain, d_beta, d_betainv, d_out,
                                     planes_apart ? nullptr : d_planes, B, C, HW, dp, tp, np, ps, ctx->stream);
        }
        if (e == hipSuccess && planes_apart) {
            const ss_keys none = {};
            timed tm(ctx, SSNET_PROF_PACK_X);
            e = ss_launch_planes(d_out, nullptr, d_planes, n, ctx->t, B, C, HW, false, none, ctx->stream);
        }
    } else {   // other schemes: the same steps, messages and results in three launches
        const ss_recf_params norec = {};
        {
            timed tm(ctx, SSNET_PROF_DEGREE_REDUCE);
            e = ss_launch_degree_reduce_truncate(c, msg1, msg2, u, wsh, d_out, nullptr, count, dp, tp, norec, ps,
                                                 ctx->stream);
        }
        if (e == hipSuccess) {
            timed tm(ctx, SSNET_PROF_NONLINEAR);
            e = ss_launch_relu(d_out, d_beta, d_betainv, rmsg, yplain, d_out, count, np, ctx->stream);
        }
        if (e == hipSuccess && d_planes) {
            const ss_keys none = {};
            timed tm(ctx, SSNET_PROF_PACK_X);
            e = ss_launch_planes(d_out, nullptr, d_planes, n, ctx->t, B, C, HW, false, none, ctx->stream);
        }
    }
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_reduce_truncate_relu_direct(ssnet_ctx *ctx, const uint64_t *d_c, int B, int C, int HW, const uint64_t *d_beta,
                                      const uint64_t *d_betainv, uint64_t *d_out, void *d_planes)
{
    if (!ctx || !d_beta || !d_betainv || !d_out || B < 1 || C < 1 || HW < 1) return SSNET_EINVAL;
    if ((long)B * HW >= (1L << 30) || (size_t)B * C * HW > MAX_COUNT) return SSNET_EINVAL;
    if (d_planes && (((uintptr_t)d_planes & 15) || C % 64 != 0)) return SSNET_EINVAL;
    const size_t count = (size_t)B * C * HW;
    const u64 *c;
    ss_part_src ps;
    if (d_c) {
        c = d_c;
        ps = {1, 0};
    } else if (int rc = incoming_product(ctx, nullptr, count, 0, &c, &ps)) {
        return rc;
    }
    ss_nl_params open_all;
    if (!make_nl_params(ctx, 0, &open_all)) return SSNET_EINVAL;
    timed tm(ctx, SSNET_PROF_DEGREE_REDUCE);
    hipError_t e = ss_launch_tail_direct(c, d_beta, d_betainv, d_out, d_planes, B, C, HW, open_all, make_tr_params(ctx, 0),
                                         ps, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_nonlinear_masks(ssnet_ctx *ctx, size_t count, uint64_t stream_id, uint64_t *d_beta, uint64_t *d_betainv)
{
    if (!ctx || !d_beta || !d_betainv || count == 0 || count > MAX_COUNT) return SSNET_EINVAL;
    ss_nl_params np;
    if (!make_nl_params(ctx, stream_id, &np)) return SSNET_EINVAL;
    timed tm(ctx, SSNET_PROF_NONLINEAR);
    hipError_t e = ss_launch_nonlinear_masks(d_beta, d_betainv, count, np, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_relu(ssnet_ctx *ctx, const uint64_t *d_x, const uint64_t *d_beta, const uint64_t *d_betainv, size_t count,
               uint64_t *d_out)
{
    if (!ctx || !d_x || !d_beta || !d_betainv || !d_out || count == 0 || count > MAX_COUNT) return SSNET_EINVAL;
    const int nr = 2 * ctx->t + 1;
    if (!ws_fits(ctx, (size_t)(nr + 1) * count * 8)) return SSNET_EWORKSPACE;
    ss_nl_params np;
    if (!make_nl_params(ctx, 0, &np)) return SSNET_EINVAL;
    u64 *msg = (u64 *)ws_scratch(ctx), *yplain = msg + (size_t)nr * count;
    timed tm(ctx, SSNET_PROF_NONLINEAR);
    hipError_t e = ss_launch_relu(d_x, d_beta, d_betainv, msg, yplain, d_out, count, np, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

namespace {

// 0 if the pooling geometry is not acceptable
static bool make_pool_geom(size_t planes, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw, int mode,
                    ss_pool_geom *g)
{
    if (planes < 1 || H < 1 || W < 1 || kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0) return false;
    if (ph >= kh || pw >= kw || kh > H + 2 * ph || kw > W + 2 * pw) return false;   // every kernel meets the plane
    if (H > (1 << 15) || W > (1 << 15) || (long)kh * kw > SSNET_MAX_KDIV || (mode != 0 && mode != 1)) return false;
    *g = {H, W, kh, kw, sh, sw, ph, pw, (H + 2 * ph - kh) / sh + 1, (W + 2 * pw - kw) / sw + 1,
          (sh == kh && sw == kw && ph == 0 && pw == 0) ? 1 : 0, mode};
    const size_t cin = (size_t)H * W, cout = (size_t)g->Ho * g->Wo;
    return planes <= MAX_COUNT / cin && planes <= MAX_COUNT / cout;
}

}  // namespace

uint64_t ssnet_field_prime(void) { return SS_P; }

int ssnet_pool_out_size(int H, int k, int s, int pad)
{
    if (H < 1 || k < 1 || s < 1 || pad < 0 || k > H + 2 * pad) return 0;
    return (H + 2 * pad - k) / s + 1;
}

int ssnet_pool_masks(ssnet_ctx *ctx, size_t planes, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
                     uint64_t stream_id, uint64_t *d_beta, uint64_t *d_betainv)
{
    ss_pool_geom g;
    if (!ctx || !d_beta || !d_betainv || !make_pool_geom(planes, H, W, kh, kw, sh, sw, ph, pw, 0, &g))
        return SSNET_EINVAL;
    ss_nl_params np;
    if (!make_nl_params(ctx, stream_id, &np)) return SSNET_EINVAL;
    timed tm(ctx, SSNET_PROF_NONLINEAR);
    hipError_t e = ss_launch_pool_masks(d_beta, d_betainv, planes, g, np, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

int ssnet_relu_pool(ssnet_ctx *ctx, const uint64_t *d_x, const uint64_t *d_beta, const uint64_t *d_betainv,
                    size_t planes, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw, int mode,
                    uint64_t *d_out)
{
    ss_pool_geom g;
    if (!ctx || !d_x || !d_beta || !d_betainv || !d_out ||
        !make_pool_geom(planes, H, W, kh, kw, sh, sw, ph, pw, mode, &g))
        return SSNET_EINVAL;
    const int nr = 2 * ctx->t + 1;
    const size_t cin = planes * H * W, cout = planes * g.Ho * g.Wo;
    {   // the pooled shares are written while other threads still read the input: no overlap allowed
        const uintptr_t x0 = (uintptr_t)d_x, x1 = x0 + (size_t)ctx->n * cin * 8, o0 = (uintptr_t)d_out,
                        o1 = o0 + (size_t)ctx->n * cout * 8;
        if (x0 < o1 && o0 < x1) return SSNET_EINVAL;
    }
    if (!ws_fits(ctx, ((size_t)(nr + 1) * cin + cout) * 8)) return SSNET_EWORKSPACE;
    ss_nl_params np;
    if (!make_nl_params(ctx, 0, &np)) return SSNET_EINVAL;
    u64 *msg = (u64 *)ws_scratch(ctx), *rplain = msg + (size_t)nr * cin, *yplain = rplain + cin;
    timed tm(ctx, SSNET_PROF_NONLINEAR);
    hipError_t e = ss_launch_relu_pool(d_x, d_beta, d_betainv, msg, rplain, yplain, d_out, planes, g, np, ctx->stream);
    return e == hipSuccess ? SSNET_OK : fail_hip(ctx, e);
}

uint64_t ssnet_rng_key(uint64_t seed, uint64_t domain, uint64_t stream_id, uint64_t party, uint64_t j)
{
    return ss_key(seed, domain, stream_id, party, j);
}

uint64_t ssnet_rng_draw(uint64_t key, uint64_t e) { return ss_draw(key, e); }

uint64_t ssnet_rng_field(uint64_t key, uint64_t e) { return ss_draw_field(key, e); }

int ssnet_host_lagrange(const ssnet_ctx *ctx, const int *party_ids, int m, uint64_t *out)
{
    if (!ctx || !party_ids || !out || m < 1 || m > ctx->n) return SSNET_EINVAL;
    for (int i = 0; i < m; i++) {
        if (party_ids[i] < 1 || party_ids[i] > ctx->n) return SSNET_EID;
        for (int j = 0; j < i; j++)
            if (party_ids[j] == party_ids[i]) return SSNET_EID;
    }
    h_lagrange(party_ids, m, out);
    return SSNET_OK;
}

int ssnet_host_reduction_matrix(const ssnet_ctx *ctx, uint64_t *out)
{
    if (!ctx || !out) return SSNET_EINVAL;
    const int k = ctx->t + 1, nr = 2 * ctx->t + 1;
    for (int i = 0; i < nr; i++)
        for (int m = 0; m < ctx->n; m++) {
            u64 acc = 0;
            for (int j = k - 1; j >= 0; j--) acc = ss_add(ss_mul(acc, (u64)(m + 1)), ctx->binv[i][j]);
            out[i * ctx->n + m] = acc;
        }
    return SSNET_OK;
}

const char *ssnet_strerror(int code)
{
    switch (code) {
        case SSNET_OK: return "ok";
        case SSNET_EINVAL: return "invalid argument";
        case SSNET_EPRIME: return "this library was built for another prime (see ssnet_field_prime)";
        case SSNET_ESHARES: return "too few shares for this degree";
        case SSNET_EID: return "party id out of range or repeated";
        case SSNET_EWORKSPACE: return "workspace missing or too small";
        case SSNET_EHIP: return "HIP error";
        case SSNET_ESCRATCH: return "count exceeds the fixed scratch of the entry point that allocates nothing";
        default: return "unknown error";
    }
}

int ssnet_last_hip_error(const ssnet_ctx *ctx) { return ctx ? ctx->last_hip : 0; }

}  // extern "C"
