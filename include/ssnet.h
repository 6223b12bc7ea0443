/*
 * ssnet.h - C ABI of the MI355X (gfx950) library for the per-party arithmetic
 * of Shamir-secret-sharing neural-network inference.
 *
 * All n parties of a (k = t+1, n) threshold scheme are simulated as the
 * leading (batch) dimension of every share tensor on one GPU; no data leaves
 * the device inside a call.  The field is F_p with p = 2^61 - 1; a field
 * element is a uint64_t in [0, p-1] (canonical: the value p never appears).
 *
 * The field is fixed when the library is compiled.  The same sources built
 * with -DSS_FIELD_P45 give a second library with this same ABI over the prime
 * of Sec. VII-A, p = 2^45 - 55 (16-bit operands, 13 bits of accumulation room):
 * field elements have 6 int8 limbs instead of 8, so limb tiles and limb planes
 * are three quarters the size (ask ssnet_packed_weight_bytes /
 * ssnet_conv_planes_bytes of the library in use) and a product costs 36 int8
 * multiply-adds instead of 64.  Wherever a comment below says 2^61 - 1, "61
 * bits" or "eight limbs", read the library's own prime (ssnet_field_prime) and
 * limb count.  Preconditions stated against p/2 scale with it: over the
 * 45-bit prime truncation needs |x| + 2^32 <= (p-1)/2 and the ReLU mask
 * |x| * 2^28 < p/2, i.e. |x| < 2^16, the paper's 16-bit budget (Sec. VII-B).
 *
 * Conventions for every entry point below
 *   - `d_` pointers are DEVICE pointers owned by the caller (8-byte aligned;
 *     16-byte aligned buffers take the faster vector path).  The library never
 *     allocates, frees or keeps them, except the workspace handed over with
 *     ssnet_set_workspace, which it uses until replaced or the context dies.
 *   - Share tensors are party-major: shares[i*count + e] is the share of
 *     element e held by the party with ID i+1 (IDs are 1..n, Sec. IV-A).
 *   - Work is enqueued on the HIP stream given at creation; calls do not
 *     synchronise.  Inputs and outputs must not alias unless stated.
 *   - Inputs must be canonical (< p); outputs always are.
 *   - Return value: SSNET_OK (0) or a negative SSNET_E* code; nothing throws.
 *   - Randomness: every random polynomial coefficient is a pure function of
 *     (seed, domain, stream_id, party, coefficient index, element index) by the
 *     counter-based generator documented with ssnet_rng_key / ssnet_rng_draw,
 *     so equal arguments give equal bits.  Use a fresh stream_id per call.
 */
#ifndef SSNET_H
#define SSNET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SSNET_OK 0
#define SSNET_EINVAL (-1)     /* null pointer, bad n/t/f/degree/shape                 */
#define SSNET_EPRIME (-2)     /* p is not the prime this library was built for         */
#define SSNET_ESHARES (-3)    /* fewer than degree+1 parties given to reconstruct      */
#define SSNET_EID (-4)        /* party id outside [1, n] or repeated                   */
#define SSNET_EWORKSPACE (-5) /* workspace missing or too small for this call          */
#define SSNET_EHIP (-6)       /* a HIP call failed; see ssnet_last_hip_error           */
#define SSNET_ESCRATCH (-7)   /* count beyond the fixed scratch of ssnet_degree_reduce_static */

#define SSNET_MAX_PARTIES 8   /* n <= 8                                                */
#define SSNET_MAX_T 3         /* t <= 3 (n >= 2t+1)                                    */
#define SSNET_MAX_K 16383     /* contraction length of linear/conv (int32 exactness)   */

#define SSNET_P61 0x1FFFFFFFFFFFFFFFULL /* 2^61 - 1                                    */
#define SSNET_P45 0x1FFFFFFFFFC9ULL     /* 2^45 - 55 (Sec. VII-A)                      */

/* The prime this library was built for: SSNET_P61 or SSNET_P45. */
uint64_t ssnet_field_prime(void);

typedef struct ssnet_ctx ssnet_ctx;

/* Context: parameters of the scheme plus host-computed constant tables
 * (Lagrange multipliers of Eq. 2 for IDs 1..k, the factors of the reduction
 * matrix R = B^-1 P B of Eq. 3).  Requires n >= 2t+1 (Sec. III-B), 1 <= t <=
 * SSNET_MAX_T, n <= SSNET_MAX_PARTIES, p == ssnet_field_prime(), 1 <= f <= 31.
 * `hip_stream` is a hipStream_t (NULL = the default stream).  Host-only work:
 * creating a context does not touch the GPU. */
int ssnet_create(ssnet_ctx **out, int n, int t, uint64_t p, int f, uint64_t seed, void *hip_stream);
int ssnet_destroy(ssnet_ctx *ctx);

/* Scratch memory for the inter-party messages of ssnet_degree_reduce /
 * ssnet_truncate on `count` elements, and for the int8 limb tiles and split
 * partial sums of ssnet_linear_mod / ssnet_conv_mod.  Sizes are in bytes; a
 * workspace of the maximum over the calls that will be made serves all of them.
 * The first SSNET_WS_HEADER_BYTES of a workspace are reserved; the messages of
 * ssnet_degree_reduce ([2t+1][k][count] then [k][n][count]) and of
 * ssnet_truncate ([k][count] then [n][count]) start right behind that header.
 * 16-byte aligned. */
#define SSNET_WS_HEADER_BYTES 65536
size_t ssnet_workspace_bytes_stream(const ssnet_ctx *ctx, size_t count);
size_t ssnet_workspace_bytes_linear(const ssnet_ctx *ctx, int M, int K, int N);
size_t ssnet_workspace_bytes_conv(const ssnet_ctx *ctx, int B, int C, int H, int W, int Co, int kh, int kw,
                                  int stride, int pad);
int ssnet_set_workspace(ssnet_ctx *ctx, void *d_workspace, size_t bytes);

/* GEN (Eq. 1): for each element e draw a_1..a_degree uniformly from F_p
 * (domain SHARE) and write share_i[e] = a0 + a1 i + ... + a_d i^d mod p for
 * i = 1..n.  d_secret [count] -> d_shares [n][count].  0 <= degree <= 2t. */
int ssnet_share(ssnet_ctx *ctx, const uint64_t *d_secret, size_t count, int degree, uint64_t stream_id,
                uint64_t *d_shares);

/* REC (Eq. 2): secret[e] = sum_{i in ids} lambda_i * shares[i-1][e] mod p with
 * lambda_i = prod_{j != i} j / (j - i).  `party_ids` is a HOST array of m
 * distinct IDs in [1, n]; m >= degree+1 else SSNET_ESHARES (degree = t or 2t).
 * d_shares [n][count] (only the m named planes are read) -> d_secret [count]. */
int ssnet_reconstruct(ssnet_ctx *ctx, const uint64_t *d_shares, size_t count, const int *party_ids, int m,
                      int degree, uint64_t *d_secret);

/* SSS-Linear step 1, dense (Sec. VI-A): every party multiplies its own share
 * matrices, y_i = x_i * w_i mod p.  d_x [n][M][K], d_w [n][K][N] -> d_y
 * [n][M][N], all row-major.  The result is a degree-2t sharing.
 * K <= SSNET_MAX_K.  Needs a workspace (ssnet_workspace_bytes_linear). */
int ssnet_linear_mod(ssnet_ctx *ctx, const uint64_t *d_x, const uint64_t *d_w, int M, int K, int N,
                     uint64_t *d_y);

/* SSS-Linear step 1, convolution (Sec. VI-A): per party, cross-correlation
 * (no kernel flip) with zero padding, mod p.  d_x [n][B][C][H][W], d_w
 * [n][Co][C][kh][kw] -> d_y [n][B][Co][Ho][Wo], Ho = (H+2*pad-kh)/stride+1.
 * C*kh*kw <= SSNET_MAX_K.  Needs a workspace (ssnet_workspace_bytes_conv). */
int ssnet_conv_mod(ssnet_ctx *ctx, const uint64_t *d_x, const uint64_t *d_w, int B, int C, int H, int W,
                   int Co, int kh, int kw, int stride, int pad, uint64_t *d_y);

/* Weights are fixed across inferences (Sec. II-B: preprocessing is done once
 * for a sequence of inferences), so their int8 limb tiles can be prepared
 * once: ssnet_pack_weights_* writes them to caller memory of
 * ssnet_packed_weight_bytes(rows, K) * n bytes, and the *_packed variants of
 * the two layer calls take that buffer in place of d_w.  rows = N (dense) or
 * Co (conv), K = contraction length.  Results are bit-identical. */
size_t ssnet_packed_weight_bytes(int rows, int K);
int ssnet_pack_weights_linear(ssnet_ctx *ctx, const uint64_t *d_w /*[n][K][N]*/, int K, int N, void *d_packed);
int ssnet_pack_weights_conv(ssnet_ctx *ctx, const uint64_t *d_w /*[n][Co][C][kh][kw]*/, int Co, int CKK,
                            void *d_packed);
int ssnet_linear_mod_packed(ssnet_ctx *ctx, const uint64_t *d_x, const void *d_w_packed, int M, int K, int N,
                            uint64_t *d_y);
int ssnet_conv_mod_packed(ssnet_ctx *ctx, const uint64_t *d_x, const void *d_w_packed, int B, int C, int H,
                          int W, int Co, int kh, int kw, int stride, int pad, uint64_t *d_y);

/* The input of a dense layer or of a 1x1, stride 1, unpadded convolution can be
 * shared and brought into limb tiles in one launch, and the layer then run on
 * the tiles alone:
 *   ssnet_share_packed: GEN (Eq. 1, degree t, domain SHARE) of d_secret
 *     [B][K][HW] -> d_shares [n][B][K][HW], the very values ssnet_share writes
 *     for the same stream_id, plus their tiles d_packed (n *
 *     ssnet_packed_weight_bytes(B*HW, K) bytes, 16-byte aligned).  Dense input
 *     [M][K]: B = M, HW = 1.  Conv input [B][C][H][W]: K = C, HW = H*W.
 *   ssnet_linear_mod_prepacked / ssnet_conv1x1_mod_prepacked: SSS-Linear step 1
 *     (Sec. VI-A) as ssnet_linear_mod_packed / ssnet_conv_mod_packed (kh = kw =
 *     stride = 1, pad = 0) compute it, bit-identical, from those tiles.  They
 *     need the workspace of the corresponding ssnet_workspace_bytes_* call. */
int ssnet_share_packed(ssnet_ctx *ctx, const uint64_t *d_secret, int B, int K, int HW, uint64_t stream_id,
                       uint64_t *d_shares, void *d_packed);
int ssnet_linear_mod_prepacked(ssnet_ctx *ctx, const void *d_x_packed, const void *d_w_packed, int M, int K, int N,
                               uint64_t *d_y);
int ssnet_conv1x1_mod_prepacked(ssnet_ctx *ctx, const void *d_x_packed, const void *d_w_packed, int B, int C, int HW,
                                int Co, uint64_t *d_y);

/* Convolution without a materialised im2col matrix (SSS-Linear step 1, Sec.
 * VI-A, for kh x kw kernels with C a multiple of 64): the input is kept as
 * channel-innermost int8 limb planes, per party [limb 0..7][b][h][w][c] plus a
 * 256-byte pad (ssnet_conv_planes_bytes(B, C, H, W) bytes per party, n parties
 * back to back, 16-byte aligned; 0 for an unsupported shape), from which the
 * product kernel gathers the 16 channels of one tap of one output pixel as 16
 * consecutive bytes; the weights are packed with contraction index (tap,
 * channel).
 *   ssnet_share_planes: GEN (Eq. 1, degree t, domain SHARE) of d_secret
 *     [B][C][H][W] -> d_shares [n][B][C][H][W] (the values of ssnet_share for
 *     the same stream_id) and their planes, in one launch.
 *   ssnet_split_planes: planes of existing shares d_x [n][B][C][H][W].
 *   ssnet_pack_weights_conv_taps: d_w [n][Co][C][kh][kw] -> tiles of
 *     ssnet_packed_weight_bytes(Co, C*kh*kw) bytes per party.
 *   ssnet_conv_mod_planes: d_y [n][B][Co][Ho][Wo], bit-identical to
 *     ssnet_conv_mod on the same shares; workspace as ssnet_workspace_bytes_conv. */
size_t ssnet_conv_planes_bytes(int B, int C, int H, int W);
int ssnet_share_planes(ssnet_ctx *ctx, const uint64_t *d_secret, int B, int C, int H, int W, uint64_t stream_id,
                       uint64_t *d_shares, void *d_planes);
int ssnet_split_planes(ssnet_ctx *ctx, const uint64_t *d_x, int B, int C, int H, int W, void *d_planes);
int ssnet_pack_weights_conv_taps(ssnet_ctx *ctx, const uint64_t *d_w, int Co, int C, int kh, int kw, void *d_packed);
int ssnet_conv_mod_planes(ssnet_ctx *ctx, const void *d_planes, const void *d_w_packed, int B, int C, int H, int W,
                          int Co, int kh, int kw, int stride, int pad, uint64_t *d_y);

/* SSS-Linear step 1 (Sec. VI-A) with the product shares left inside the
 * workspace for the reduction that follows (steps 2 and 3): the layers of a
 * batch-1 network are small, a product kernel then has fewer output tiles than
 * the chip has compute units and splits the contraction over them, and in this
 * form it does not gather the pieces: every workgroup stores what it has, as
 * planes whose sum mod p is the product, and the reduction adds the planes while
 * it reads them.  Nothing is exchanged or waited for inside the product kernel.
 *   ssnet_*_product_*: same operands, shapes and checks as ssnet_linear_mod_prepacked,
 *     ssnet_conv1x1_mod_prepacked and ssnet_conv_mod_planes, but no d_y: the
 *     product (count = M*N, resp. B*Co*Ho*Wo elements per party) becomes the
 *     context's pending product, kept in the last ssnet_product_bytes_* bytes of
 *     the workspace until the next ssnet_*_product_* or ssnet_set_workspace call.
 *   Consuming it: ssnet_degree_reduce, ssnet_degree_reduce_truncate(_div,
 *     _reconstruct), ssnet_reduce_truncate_direct and ssnet_reduce_truncate_relu
 *     take d_c = NULL for "the pending product" (count, resp. B*C*HW, must equal
 *     its element count, else SSNET_EINVAL; SSNET_EINVAL too if there is none).
 *     Results, messages and random draws are those of the same call on the d_y
 *     that the corresponding ssnet_*_mod_* call writes.  The call's messages
 *     start behind the workspace header as always, so the workspace must hold
 *     ssnet_workspace_bytes_stream(count) (ssnet_workspace_bytes_layer_tail for
 *     ssnet_reduce_truncate_relu) plus ssnet_product_bytes_*(...) bytes, else
 *     SSNET_EWORKSPACE. */
size_t ssnet_product_bytes_linear(const ssnet_ctx *ctx, int M, int K, int N);
size_t ssnet_product_bytes_conv(const ssnet_ctx *ctx, int B, int C, int H, int W, int Co, int kh, int kw, int stride,
                                int pad);
int ssnet_linear_product_prepacked(ssnet_ctx *ctx, const void *d_x_packed, const void *d_w_packed, int M, int K, int N);
int ssnet_conv1x1_product_prepacked(ssnet_ctx *ctx, const void *d_x_packed, const void *d_w_packed, int B, int C, int HW,
                                    int Co);
int ssnet_conv_product_planes(ssnet_ctx *ctx, const void *d_planes, const void *d_w_packed, int B, int C, int H, int W,
                              int Co, int kh, int kw, int stride, int pad);

/* RED by resharing (Sec. IV-B, the three protocol steps with the matrix of
 * Eq. 3) followed by RERAND (Sec. IV-C), all n parties:
 *   1. parties 1..2t+1: GEN(c_i, k, k) towards parties 1..k   (domain RESHARE, party i)
 *   2. parties 1..k: received row vector times R               -> one value per party 1..n
 *   3. parties 1..n: REC of the k values received, then add the party's share
 *      of a fresh degree-t sharing of zero                     (domain ZERO)
 * d_c [n][count] (degree 2t) -> d_out [n][count] (degree t).  The messages of
 * steps 1 and 2 are materialised in the workspace ([2t+1][k][count] and
 * [k][n][count]).  d_out may alias d_c.  d_c = NULL: the pending product. */
int ssnet_degree_reduce(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id, uint64_t *d_out);

/* ssnet_degree_reduce for callers that cannot allocate device memory or hand a
 * workspace over: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same random draws, same d_out and the
 * same two message arrays as ssnet_degree_reduce, but the messages go to a fixed
 * array of SSNET_STATIC_SCRATCH_BYTES inside the library's device image (each
 * GPU the library runs on holds it until the process ends) instead of the
 * workspace; no workspace is needed and the call allocates and frees nothing.
 * Limit: (2t+1)(t+1) + (t+1)n message words per element must fit, i.e. count <=
 * SSNET_STATIC_SCRATCH_BYTES / 8 / ((2t+1)(t+1) + (t+1)n) (34952 elements for
 * n = 5, t = 2), else SSNET_ESCRATCH and nothing is launched.  Every call on a
 * GPU uses that GPU's one array (nothing in it needs clearing: a launch writes
 * each message before it is read), so calls that overlap on one GPU, from any
 * context or stream, race on it; calls on one stream are ordered and safe.
 * The device current at the call must be the one the context's stream is on.
 * d_out may alias d_c. */
#define SSNET_STATIC_SCRATCH_BYTES (8u << 20)
int ssnet_degree_reduce_static(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id,
                               uint64_t *d_out);

/* SSS-Truncation (Sec. VI-B) by r = 2^f: shares of floor(x / 2^f), x read as a
 * signed value in [-(p-1)/2, (p-1)/2].
 *   1. parties 1..k add their share of alpha = e*2^f, e uniform in [1, 2^(32-f)]
 *      (Sec. VII-B; domains MASK_E, MASK_ALPHA)
 *   2. the elite party reconstructs x+alpha, shifts right by f (arithmetic) and
 *      re-shares the result                                    (domain TRUNC_GEN)
 *   3. all n parties add their share of alpha~ = -e             (domain MASK_ALPHAT)
 * d_x [n][count] (degree t; planes 1..k are read) -> d_out [n][count].
 * Requires |x| + 2^32 <= (p-1)/2.  Messages go through the workspace.
 * d_out may alias d_x. */
int ssnet_truncate(ssnet_ctx *ctx, const uint64_t *d_x, size_t count, uint64_t stream_id, uint64_t *d_out);

/* SSS-Truncation followed by the rounding division that average pooling moves
 * into it (Sec. VI-C, extra step for AvgPooling; App. C): shares of
 * [floor(x / 2^f) / kdiv], kdiv = kh*kw of the pooling kernel that follows, so
 * that the pooling itself is a sum.  The mask becomes alpha = e*2^f*kdiv with
 * e uniform in [1, floor(2^(32-f) / kdiv)] (the smaller sample space of
 * Sec. VII-B, so that alpha stays in (0, 2^32]; the draw is that of
 * ssnet_truncate, reduced modulo the range instead of masked); [.] rounds to
 * the nearest integer, a remainder of ceil(kdiv/2) or more going up, on the
 * signed value.  1 <= kdiv <= min(SSNET_MAX_KDIV, 2^(32-f)), else
 * SSNET_EINVAL; kdiv = 1 is ssnet_truncate.  Requires |x| + 2^32 <= (p-1)/2,
 * as ssnet_truncate does.  Everything else as ssnet_truncate. */
#define SSNET_MAX_KDIV 4096
int ssnet_truncate_div(ssnet_ctx *ctx, const uint64_t *d_x, size_t count, int kdiv, uint64_t stream_id,
                       uint64_t *d_out);

/* SSS-Linear's reduction followed at once by SSS-Truncation (the default layer
 * order Linear - Truncation of Sec. VII-A): the result, every message and every
 * random draw are those of ssnet_degree_reduce(stream_id) followed by
 * ssnet_truncate(stream_id), in one launch.  Workspace behind the header:
 * [2t+1][k][count], [k][n][count] (reduction), then [k][count], [n][count]
 * (truncation).  d_out may alias d_c. */
int ssnet_degree_reduce_truncate(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id,
                                 uint64_t *d_out);

/* ssnet_degree_reduce(stream_id) followed by ssnet_truncate_div(kdiv, stream_id)
 * in one launch; workspace as for ssnet_degree_reduce_truncate. */
int ssnet_degree_reduce_truncate_div(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, int kdiv, uint64_t stream_id,
                                     uint64_t *d_out);

/* The same launch followed, per element, by REC (Eq. 2) of the truncated shares
 * of the parties party_ids[0..m) (distinct IDs in 1..n, m >= t+1): d_out
 * [n][count] is what ssnet_degree_reduce_truncate writes, d_secret [count] what
 * ssnet_reconstruct(d_out, party_ids, m, degree t) would then return.  The
 * layer-by-layer harness uses it where a layer's result is opened at once.
 * Errors as for the two calls; d_out may alias d_c, d_secret may not alias
 * either. */
int ssnet_degree_reduce_truncate_reconstruct(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id,
                                             uint64_t *d_out, const int *party_ids, int m, uint64_t *d_secret);

/* The outputs of ssnet_degree_reduce_truncate(_reconstruct) without the protocol:
 * they do not depend on the reshare and zero randomness (the elite party of the
 * truncation sees x + alpha, x being the secret of the incoming degree-2t
 * sharing), so with all parties on one device they follow from REC of the 2t+1
 * incoming shares and truncation steps 2 and 3.  d_out (and d_secret, if not
 * NULL) hold the very residues the protocol entry points write for the same
 * stream_id; no message is formed and no workspace is used.  This is a
 * simulation shortcut, reported beside the protocol path, never in its place.
 * d_out may alias d_c. */
int ssnet_reduce_truncate_direct(ssnet_ctx *ctx, const uint64_t *d_c, size_t count, uint64_t stream_id,
                                 uint64_t *d_out, const int *party_ids, int m, uint64_t *d_secret);

/* SSS-NonLinear with ReLU (Sec. VI-C), on shares that were truncated before
 * (order Linear - Truncation - NonLinear, Sec. VII-A).
 *   ssnet_nonlinear_masks: what the trusted source prepares ahead of the
 *     inference (Sec. VII-B): per element a mask beta, uniform in
 *     [1, 2^SSNET_BETA_BITS] (domain MASK_BETA), its inverse in F_p, and a
 *     degree-t sharing of each (domains BETA_GEN, BETAINV_GEN) -> d_beta,
 *     d_betainv [n][count].
 *   ssnet_relu: 1. parties 1..2t+1 multiply their share of x by their share of
 *     beta; 2. the elite party reconstructs x*beta from the 2t+1 products and
 *     applies max(., 0) to the signed value in the clear; 3. every party
 *     multiplies that plain value by its share of beta^-1.  d_x, d_beta,
 *     d_betainv, d_out [n][count]; d_out is a degree-t sharing of max(x, 0).
 *     Requires |x| * 2^SSNET_BETA_BITS < p/2, i.e. |x| < 2^32.  The 2t+1
 *     products and the plain value go through the workspace ([2t+1][count] then
 *     [count] behind the header; ssnet_workspace_bytes_stream(count) covers
 *     it).  d_out may alias d_x. */
#define SSNET_BETA_BITS 28
int ssnet_nonlinear_masks(ssnet_ctx *ctx, size_t count, uint64_t stream_id, uint64_t *d_beta, uint64_t *d_betainv);
int ssnet_relu(ssnet_ctx *ctx, const uint64_t *d_x, const uint64_t *d_beta, const uint64_t *d_betainv, size_t count,
               uint64_t *d_out);

/* SSS-NonLinear with ReLU followed by pooling (Sec. VI-C).  A tensor is `planes`
 * images of H x W (planes = batch * channels, [n][planes][H][W]); the pooling
 * kernel is kh x kw, moved by (sh, sw) over the image padded by ph / pw zeros
 * on each side, Ho = (H + 2*ph - kh) / sh + 1 = ssnet_pool_out_size(H, kh, sh,
 * ph) (0 for sizes that do not fit), Wo likewise.  Accepted: ph < kh, pw < kw,
 * kh <= H + 2*ph, kw <= W + 2*pw, H, W <= 2^15, kh*kw <= SSNET_MAX_KDIV.
 *   ssnet_pool_masks: the trusted source's masks.  beta is equal inside one
 *     pooling kernel: where the kernels partition the image (stride = kernel, no
 *     padding) one beta per kernel position, drawn at counter (plane*Ho + oh)*Wo
 *     + ow (elements beyond the last full kernel join the last one); where they
 *     overlap, one beta per plane, drawn at counter = plane (shared kernels link
 *     every element of a plane to every other).  The sharing coefficients are
 *     drawn per element.  d_beta [n][planes*H*W]; d_betainv [n][planes*Ho*Wo]
 *     shares beta^-1 of the pooled element's kernel.  Domains as
 *     ssnet_nonlinear_masks.
 *   ssnet_relu_pool: 1. parties 1..2t+1 multiply their shares of x and beta;
 *     2. the elite party reconstructs x*beta elementwise, applies max(., 0), and
 *     pools in the clear: mode SSNET_POOL_MAX the maximum, SSNET_POOL_SUM the sum
 *     over the kernel's elements inside the image (the division of an average is
 *     done before, by ssnet_truncate_div with kdiv = kh*kw); 3. every party
 *     multiplies the pooled plain value by its share of beta^-1.  d_out
 *     [n][planes*Ho*Wo] is a degree-t sharing of the pooled max(x, 0).
 *     Requires kh*kw * |x| * 2^SSNET_BETA_BITS < p/2 for the sum, |x| < 2^32 for
 *     the maximum.  Workspace behind the header: the products [2t+1][planes*H*W],
 *     the rectified plain values [planes*H*W], the pooled plain values
 *     [planes*Ho*Wo]; ssnet_workspace_bytes_stream(max of the two counts) covers
 *     it.  d_out must not overlap d_x (SSNET_EINVAL). */
#define SSNET_POOL_MAX 0
#define SSNET_POOL_SUM 1
int ssnet_pool_out_size(int H, int k, int s, int pad);
int ssnet_pool_masks(ssnet_ctx *ctx, size_t planes, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw,
                     uint64_t stream_id, uint64_t *d_beta, uint64_t *d_betainv);
int ssnet_relu_pool(ssnet_ctx *ctx, const uint64_t *d_x, const uint64_t *d_beta, const uint64_t *d_betainv,
                    size_t planes, int H, int W, int kh, int kw, int sh, int sw, int ph, int pw, int mode,
                    uint64_t *d_out);

/* The tail of a convolution layer in the default order Linear - Truncation -
 * NonLinear (Sec. VII-A) in one launch: ssnet_degree_reduce_truncate(stream_id)
 * of the product shares d_c [n][B][C][HW], then ssnet_relu with the masks
 * d_beta, d_betainv [n][B][C][HW]; d_out [n][B][C][HW] holds the residues these
 * two calls give, and d_planes, if not NULL, the same values as channel-innermost
 * limb planes for the next ssnet_conv_mod_planes (C a multiple of 64 then).
 * Messages behind the workspace header: those of the reduction and truncation,
 * then the 2t+1 masked products and the plain value of the ReLU, as planes of
 * P = ssnet_layer_tail_message_plane(B, C, HW) positions each
 * ([2t+1][k][P], [k][n][P], [k][P], [n][P], [2t+1][P], [P]).  For the schemes
 * (3,1) and (5,2), which run as one kernel, a plane is ordered by that kernel's
 * threads, blocks of 16 pixels x 16 channels: element (b, c, hw), pix = b*HW+hw,
 * sits at ((c/16) * ceil(B*HW/16) + pix/16) * 256 + (c%16/4) * 64 + (c%4) * 16 +
 * pix%16, and P counts the padded blocks; for other schemes P = B*C*HW in
 * element order.  ssnet_workspace_bytes_layer_tail gives the bytes needed.
 * d_out may alias d_c. */
size_t ssnet_layer_tail_message_plane(const ssnet_ctx *ctx, int B, int C, int HW);
size_t ssnet_workspace_bytes_layer_tail(const ssnet_ctx *ctx, int B, int C, int HW);
int ssnet_reduce_truncate_relu(ssnet_ctx *ctx, const uint64_t *d_c, int B, int C, int HW, uint64_t stream_id,
                               const uint64_t *d_beta, const uint64_t *d_betainv, uint64_t *d_out, void *d_planes);

/* The outputs of ssnet_reduce_truncate_relu without the protocol, for all
 * parties on one device (the companion of ssnet_reduce_truncate_direct for the
 * order Linear - Truncation - NonLinear of Sec. VII-A): d_out and, if not NULL,
 * d_planes hold the very residues the protocol entry point writes for any
 * stream_id, because they do not depend on the reshare, zero and truncation
 * randomness: the elite party of SSS-NonLinear (Sec. VI-C) sees floor(x / 2^f) *
 * beta, x being the secret of the incoming degree-2t sharing, and every party's
 * result is max(., 0) times its share of beta^-1.  One pass, no message, no
 * workspace (beyond a pending product, d_c = NULL).  A simulation shortcut,
 * reported beside the protocol path, never in its place.  Any scheme; shapes,
 * masks and planes as for ssnet_reduce_truncate_relu.  d_out may alias d_c. */
int ssnet_reduce_truncate_relu_direct(ssnet_ctx *ctx, const uint64_t *d_c, int B, int C, int HW, const uint64_t *d_beta,
                                      const uint64_t *d_betainv, uint64_t *d_out, void *d_planes);

/* Host-side generator, exposed so that its bits can be checked without a GPU.
 * key = absorb(seed, domain, stream_id, party, j) with h <- mix64((h ^ word) +
 * 0x9E3779B97F4A7C15) from h = 0, mix64 being the SplitMix64 output function;
 * draw(key, e) = mix64(key + (e+1) * 0x9E3779B97F4A7C15); the field element is
 * draw >> 3, with the single value p mapped to 0. */
#define SSNET_DOM_SHARE 1
#define SSNET_DOM_RESHARE 2
#define SSNET_DOM_ZERO 3
#define SSNET_DOM_MASK_E 4
#define SSNET_DOM_MASK_ALPHA 5
#define SSNET_DOM_MASK_ALPHAT 6
#define SSNET_DOM_TRUNC_GEN 7
#define SSNET_DOM_MASK_BETA 8
#define SSNET_DOM_BETA_GEN 9
#define SSNET_DOM_BETAINV_GEN 10
uint64_t ssnet_rng_key(uint64_t seed, uint64_t domain, uint64_t stream_id, uint64_t party, uint64_t j);
uint64_t ssnet_rng_draw(uint64_t key, uint64_t e);
uint64_t ssnet_rng_field(uint64_t key, uint64_t e);

/* Host-side constant tables of a context, for inspection: Lagrange multipliers
 * of an ID set (Eq. 2) into out[m]; the reduction matrix R (Eq. 3, row-vector
 * convention c' = c R) as [2t+1][n] row-major into out. */
int ssnet_host_lagrange(const ssnet_ctx *ctx, const int *party_ids, int m, uint64_t *out);
int ssnet_host_reduction_matrix(const ssnet_ctx *ctx, uint64_t *out);

/* Live kernel timing.  Between ssnet_profile_begin and ssnet_profile_end every
 * entry point brackets the kernels of each class below with a pair of HIP
 * events recorded on the context's stream.  ssnet_profile_end waits for those
 * events and writes, per class, the summed elapsed milliseconds and the number
 * of bracketed spans into two HOST arrays of SSNET_PROF_CLASSES entries.  A
 * span is what one entry-point call launches of that class: one kernel, two
 * where a call is documented as two launches.  An event recorded in front of a
 * launch is stamped when the queue reaches it, so a span contains the few
 * microseconds between that and the kernel's first wave.  Class
 * SSNET_PROF_GEMM_KERNEL has none of that: after ssnet_profile_begin_kernels
 * (instead of ssnet_profile_begin) it holds, for every product kernel (the
 * kernels of class SSNET_PROF_GEMM without the pass that adds planes up), the
 * time between the kernel's own start and end on the GPU, which is what a
 * profiler's kernel trace reports as its duration; the launches that take these
 * time stamps are slower to enqueue, so the bracketed spans of the same pass
 * are wider than after ssnet_profile_begin.  Not for use under stream capture. */
#define SSNET_PROF_SHARE 0
#define SSNET_PROF_RECONSTRUCT 1
#define SSNET_PROF_PACK_W 2
#define SSNET_PROF_PACK_X 3
#define SSNET_PROF_GEMM 4
#define SSNET_PROF_DEGREE_REDUCE 5
#define SSNET_PROF_TRUNCATE 6
#define SSNET_PROF_NONLINEAR 7
#define SSNET_PROF_GEMM_KERNEL 8
#define SSNET_PROF_CLASSES 9
int ssnet_profile_begin(ssnet_ctx *ctx);
int ssnet_profile_begin_kernels(ssnet_ctx *ctx);
int ssnet_profile_end(ssnet_ctx *ctx, double *ms_by_class, uint64_t *spans_by_class);

/* Measured ceilings of the machine, for roofline reports beside the published
 * peaks (bench support, not part of the share arithmetic; each call runs its
 * kernel reps + 1 times on the stream and waits for it):
 *   ssnet_probe_planes: `planes` copies of the `bytes` at d_src to d_dst
 *     (planes * bytes large), 16 bytes per lane, streaming stores: planes = 1 is
 *     a device copy, planes = n the traffic pattern of GEN (Eq. 1).  Result:
 *     moved gigabytes, (1 + planes) * bytes per run, per second.
 *   ssnet_probe_mfma_int8: a register-resident loop of v_mfma_i32_16x16x64_i8, two
 *     waves per SIMD with the operand and accumulator registers of the product
 *     kernel, on operand bytes from the generator (random_operands != 0: the clock
 *     this part holds under MFMA load depends on the data) or on constants.
 *     Result: int8 tera-operations per second.  d_sink: 4 device bytes. */
int ssnet_probe_planes(void *hip_stream, void *d_dst, const void *d_src, size_t bytes, int planes, int reps,
                       double *gb_per_s);
int ssnet_probe_mfma_int8(void *hip_stream, void *d_sink, int random_operands, int reps, double *tera_ops_per_s);

const char *ssnet_strerror(int code);
int ssnet_last_hip_error(const ssnet_ctx *ctx); /* hipError_t of the last failed HIP call, 0 if none */

#ifdef __cplusplus
}
#endif
#endif /* SSNET_H */
