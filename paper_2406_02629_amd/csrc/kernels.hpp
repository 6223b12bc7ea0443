// Internal launch interface between the C ABI (ssnet_api.hip) and the kernel
// files.  Every launcher enqueues on `stream` and returns hipGetLastError().
#pragma once
#include "field.hpp"

// Everything below lives in a namespace named after the field (ss61 / ss45), so that the two libraries built
// from these sources never share a C++ symbol or a kernel name.
namespace SS_NS {

#define SS_MAXDEG (2 * SS_MAXT)   // highest polynomial degree ssnet_share accepts

struct ss_keys {                  // generator keys, one per coefficient index j = 1..
    u64 k[SS_MAXDEG];
};

// Constant tables reach the kernels as small integers over a common
// denominator: value = dinv * sum(c_i * v_i), dinv = (denominator)^-1 in F_p.
// The multipliers of Eq. 2 and the entries of the matrix of Eq. 3 are ratios of
// small integers, so this replaces wide multiplications by narrow ones.
struct ss_rec_params {            // REC: which planes, which multipliers
    int m;
    int plane[SS_MAXN];
    int ilambda[SS_MAXN];         // lambda_i = ilambda[i] * dinv (for IDs up to 8, |ilambda| <= 448)
    u64 dinv;
};

struct ss_dr_params {             // RED + RERAND constants
    int n, t;
    u64 reshare_key[2 * SS_MAXT + 1][SS_MAXT];   // [party i][j]
    u64 zero_key[SS_MAXT];
    int ibinv[2 * SS_MAXT + 1][SS_MAXK];         // D * (first k columns of B^-1), Eq. 3
    int irmat[2 * SS_MAXT + 1][SS_MAXN];         // D * R, R = B^-1 P B, [reducing party][receiving party]
    u64 dinv;                                    // D^-1
    int ilambda[SS_MAXK];                        // Lagrange multipliers of IDs 1..k: (-1)^(q-1) C(k, q)
};

struct ss_tr_params {             // truncation constants
    int n, t, f;
    int kdiv;                     // > 1: rounding division by kdiv after the shift (average pooling, Sec. VI-C)
    unsigned e_range;             // e is uniform in [1, e_range], e_range = floor(2^(32-f) / kdiv), so that the mask
                                  // alpha = e * 2^f * kdiv stays in (0, 2^32] (Sec. VII-B)
    u64 e_key;
    u64 alpha_key[SS_MAXT], alphat_key[SS_MAXT], gen_key[SS_MAXT];
    int ilambda[SS_MAXK];
};

struct ss_recf_params {           // REC fused behind another step: multiplier of every party's share
    int coef[SS_MAXN];            // ilambda of the party, 0 for a party that does not take part
    u64 dinv;
};

struct ss_nl_params {             // SSS-NonLinear
    int n, t, bbits;              // beta uniform in [1, 2^bbits]
    u64 beta_key;
    u64 bgen_key[SS_MAXT], bigen_key[SS_MAXT];   // coefficients of [[beta]], [[beta^-1]]
    int ilambda[2 * SS_MAXT + 1]; // REC from the IDs 1..2t+1 (integers: (-1)^(i-1) C(2t+1, i))
    u64 dinv;
};

// Pooling kernel kh x kw moved by (sh, sw) over planes of H x W padded by ph / pw zeros (Sec. VI-C).
// tiled: the kernels partition the plane, one beta per kernel position; otherwise one beta per plane.
struct ss_pool_geom {
    int H, W, kh, kw, sh, sw, ph, pw, Ho, Wo;
    int tiled;
    int mode;                     // 0: maximum, 1: sum
};

// The incoming product shares of a reduction given as a sum of planes (the partial-sum form of the product
// kernels): share i of element e is the sum mod p of c[s * stride + i * count + e] over s < planes.
// planes <= 1: one plane, the plain tensor.
struct ss_part_src {
    int planes;
    size_t stride;
};

// ---- streaming family (stream_kernels.hip) ----
hipError_t ss_launch_share(const u64 *secret, u64 *shares, size_t count, int n, int degree,
                           const ss_keys &keys, hipStream_t stream);
hipError_t ss_launch_reconstruct(const u64 *shares, u64 *secret, size_t count, const ss_rec_params &rp,
                                 hipStream_t stream);
hipError_t ss_launch_degree_reduce(const u64 *c, u64 *msg1, u64 *msg2, u64 *out, size_t count,
                                   const ss_dr_params &dp, const ss_part_src &ps, hipStream_t stream);
// dst[i] = sum over the planes of c, i < total (dst may be c: for consumers that read one plane)
hipError_t ss_launch_sum_planes(u64 *dst, const u64 *c, size_t total, const ss_part_src &ps, hipStream_t stream);
hipError_t ss_launch_truncate(const u64 *x, u64 *u, u64 *wsh, u64 *out, size_t count, const ss_tr_params &tp,
                              hipStream_t stream);
// rec != nullptr: also REC of the truncated shares with the multipliers rf (one more output, same launch)
hipError_t ss_launch_degree_reduce_truncate(const u64 *c, u64 *msg1, u64 *msg2, u64 *u, u64 *wsh, u64 *out,
                                            u64 *rec, size_t count, const ss_dr_params &dp, const ss_tr_params &tp,
                                            const ss_recf_params &rf, const ss_part_src &ps, hipStream_t stream);

// outputs of reduction + truncation taken directly from the secret (no messages); open_all carries the
// multipliers of REC from the IDs 1..2t+1
hipError_t ss_launch_reduce_truncate_direct(const u64 *c, u64 *out, u64 *rec, size_t count, const ss_nl_params &open_all,
                                            const ss_tr_params &tp, const ss_recf_params &rf, hipStream_t stream);
// SSS-NonLinear (Sec. VI-C): the trusted source's masks, then ReLU under the mask
hipError_t ss_launch_nonlinear_masks(u64 *sh_b, u64 *sh_bi, size_t count, const ss_nl_params &np, hipStream_t stream);
hipError_t ss_launch_relu(const u64 *x, const u64 *sh_b, const u64 *sh_bi, u64 *msg, u64 *yplain, u64 *out,
                          size_t count, const ss_nl_params &np, hipStream_t stream);

// the same with pooling: masks equal inside a pooling kernel (sh_b [n][planes*H*W], sh_bi [n][planes*Ho*Wo]);
// ReLU under the mask elementwise (msg [2t+1][planes*H*W], rplain [planes*H*W]), then pooling in the clear
// and the mask-off (yplain [planes*Ho*Wo], out [n][planes*Ho*Wo])
hipError_t ss_launch_pool_masks(u64 *sh_b, u64 *sh_bi, size_t planes, const ss_pool_geom &g, const ss_nl_params &np,
                                hipStream_t stream);
hipError_t ss_launch_relu_pool(const u64 *x, const u64 *sh_b, const u64 *sh_bi, u64 *msg, u64 *rplain, u64 *yplain,
                               u64 *out, size_t planes, const ss_pool_geom &g, const ss_nl_params &np,
                               hipStream_t stream);

// reduction + RERAND + truncation + ReLU of c [n][B][C][HW] in one launch, result as shares and (planes !=
// nullptr) as limb planes; schemes (3,1) and (5,2) only (hipErrorInvalidValue otherwise, nothing launched)
hipError_t ss_launch_layer_tail(const u64 *c, u64 *msg1, u64 *msg2, u64 *umsg, u64 *wsh, u64 *rmsg, u64 *yplain,
                                const u64 *sh_b, const u64 *sh_bi, u64 *out, void *planes, int B, int C, int HW,
                                const ss_dr_params &dp, const ss_tr_params &tp, const ss_nl_params &np,
                                const ss_part_src &ps, hipStream_t stream);

// the tail's outputs (shares and, planes != nullptr, limb planes) taken directly from the secret: no messages;
// open_all carries the multipliers of REC from the IDs 1..2t+1, tp those of the IDs 1..k; any scheme
hipError_t ss_launch_tail_direct(const u64 *c, const u64 *sh_b, const u64 *sh_bi, u64 *out, void *planes, int B, int C,
                                 int HW, const ss_nl_params &open_all, const ss_tr_params &tp, const ss_part_src &ps,
                                 hipStream_t stream);

// ---- int8-limb MFMA family (gemm_kernels.hip) ----
// Packed operand: int8 tiles [row block of 16][k block of 64][limb 0..7][lane 0..63][16 bytes];
// byte b of lane l is limb `limb` of element (row = 16*rb + l%16, k = 64*kb + 16*(l/16) + b).
size_t ss_packed_bytes(int rows, int K);

// element (r, k) of party i is src[i*party_stride + r*stride_r + k*stride_k]; taps > 0: packed index k =
// tap*C + c reads source index c*taps + tap (C = K / taps)
hipError_t ss_launch_pack_matrix(const u64 *src, void *dst, int n, int rows, int K, size_t party_stride,
                                 size_t stride_r, size_t stride_k, int taps, hipStream_t stream);
// degree-t shares of secret [B][K][HW] -> shares [n][B][K][HW] and their packed operand (rows (b, hw), k)
hipError_t ss_launch_share_pack(const u64 *secret, u64 *shares, void *dst, int n, int t, int B, int K, int HW,
                                const ss_keys &keys, hipStream_t stream);
// Channel-innermost limb planes of a conv input: per party [limb 0..7][b][h][w][c] int8 and a 256-byte pad
// whose first 16 bytes are zero; C a multiple of 64.
size_t ss_planes_bytes(int B, int C, int H, int W);   // per party
// gen: `in` is the plaintext [B][C][HW] and the shares [n][B][C][HW] are written too; else `in` is the shares
hipError_t ss_launch_planes(const u64 *in, u64 *shares, void *planes, int n, int t, int B, int C, int HW, bool gen,
                            const ss_keys &keys, hipStream_t stream);
// convolution with the input given as planes and the weights packed with contraction index (tap, channel);
// out and part_stride as for ss_launch_gemm
// (started, stopped: see ss_launch_gemm)
hipError_t ss_launch_gemm_conv(const void *packedW, const void *planes, u64 *out, size_t part_stride, int n, int B, int C,
                               int H, int W, int Co, int kh, int kw, int stride, int pad, int Ho, int Wo,
                               hipStream_t stream, hipEvent_t started = nullptr, hipEvent_t stopped = nullptr);
// rows = (b, ho, wo), k = (c, r, s) of x [n][B][C][H][W]
hipError_t ss_launch_pack_im2col(const u64 *x, void *dst, int n, int B, int C, int H, int W, int kh, int kw,
                                 int stride, int pad, int Ho, int Wo, hipStream_t stream);
// product[i][row*stride_row + (col / cdiv)*stride_cb + col % cdiv] = sum_k A_i[row][k] * B_i[col][k] mod p, left as
// ss_gemm_planes(...) planes of that layout, part_stride elements apart, whose sum mod p is the product: a tile
// of the output may be computed in parts by several workgroups, each of which stores its part in a plane of
// its own; every position of every plane is written in every launch, nothing passes between workgroups.
// With one plane `out` is the product itself.
#define SS_GEMM_CUS 256
int ss_gemm_planes(int n, int rows, int cols, int K, bool planes_operand);
// bytes of the planes for either form of the second operand if there are several, else 0
size_t ss_gemm_scratch_bytes(int n, int rows, int cols, int K);
// started / stopped, if given, take the times at which the product kernel itself starts and ends on the GPU (the
// dispatch's own time stamps, without the gap between two launches that events recorded around a launch include)
hipError_t ss_launch_gemm(const void *packedA, const void *packedB, u64 *out, size_t part_stride, int n, int rows,
                          int cols, int K, size_t out_party_stride, size_t stride_row, int cdiv, size_t stride_cb,
                          hipStream_t stream, hipEvent_t started = nullptr, hipEvent_t stopped = nullptr);

}  // namespace SS_NS
