// Exact modular matrix product on int8 MFMA (SSS-Linear step 1, Sec. VI-A).
//
// A field element x < 2^61 is written in balanced radix 2^8,
//   x = sum_{i<8} d_i 2^(8i),  d_i in [-128, 127],
// which is one add and one xor: the bytes of x + 0x80..80 are d_i + 128.  The
// integer dot product sum_k x_k w_k is then sum_{i,j} 2^(8(i+j)) sum_k d_i(x_k)
// d_j(w_k): 64 int8 dot products.  Only the 15 anti-diagonal sums
//   D_s = sum_{i+j=s} sum_k d_i(x_k) d_j(w_k),   |D_s| <= 8 K 2^14 < 2^31 for K <= 16383,
// are needed, so the 64 MFMA 16x16x64 products of a 16 x 16 tile of field
// outputs accumulate straight into 15 int32 accumulator tiles (the MFMA's own
// C operand does the diagonal sum).  The epilogue turns the 15 sums of each
// output into a 61-bit residue with 2^61 = 1 (mod p) and stores the canonical
// field element.
//
// Built for p = 2^45 - 55 (Sec. VII-A) an element has 6 digits (x < 2^45 leaves
// digits 6 and 7 zero): 36 products, 11 diagonal sums, tiles and limb planes
// three quarters the size, and the epilogue folds with 2^45 = 55 (mod p).
#include "kernels.hpp"
#include "eval.hpp"
#include "digits.hpp"

namespace SS_NS {

typedef int v4i __attribute__((ext_vector_type(4)));

namespace {

// NL digits per field element (8 for p = 2^61 - 1, 6 for p = 2^45 - 55: the digits above are zero), hence
// ND anti-diagonal sums; a packed tile (16 rows x 64 contraction indices) is NL limb slices of 64 lanes x
// 16 bytes = TILE 16-byte words
constexpr int NL = SS_NLIMB, ND = 2 * NL - 1, TILE = NL * 64;

// Digit words of four consecutive contraction indices -> one dword per limb
// (byte c of dword `limb` is digit `limb` of y[c]) and store them: the thread
// owns bytes [4*(kq%4), +4) of lane (row + 16*(kq/4)) in each of the eight limb
// slices of its tile.
__device__ __forceinline__ void store_digits(const u64 (&y)[4], v4i *tile, int row, int kq)
{
    u32 *base = reinterpret_cast<u32 *>(tile) + (row + 16 * (kq >> 2)) * 4 + (kq & 3);
#pragma unroll
    for (int limb = 0; limb < NL; limb++) {
        const int i = limb & 3;
        const u32 a = limb < 4 ? (u32)y[0] : (u32)(y[0] >> 32), b = limb < 4 ? (u32)y[1] : (u32)(y[1] >> 32);
        const u32 c = limb < 4 ? (u32)y[2] : (u32)(y[2] >> 32), d = limb < 4 ? (u32)y[3] : (u32)(y[3] >> 32);
        // v_perm_b32: selector byte k picks byte k of {second operand (0..3), first operand (4..7)}; 0x0c = zero
        const u32 sel = (u32)i | ((u32)(4 + i) << 8) | 0x0c0c0000u;
        const u32 ab = __builtin_amdgcn_perm(b, a, sel), cd = __builtin_amdgcn_perm(d, c, sel);
        base[limb * 256] = __builtin_amdgcn_perm(cd, ab, 0x05040100u);
    }
}

// One workgroup per (row block, k block) tile, one thread per (row, 4 contraction indices).
// grid (Rb, Kb, n), block 256: thread t -> row t%16, k group t/16.
// taps > 0: the contraction index of the packed operand runs (tap, channel) while the source runs (channel,
// tap) with `taps` taps per channel (convolution weights for the kernel that reads its other operand from
// channel-innermost planes); stride_k is then the stride of the source's own index.
__global__ __launch_bounds__(256) void pack_matrix_kernel(const u64 *__restrict__ src, v4i *__restrict__ dst,
                                                          int rows, int K, int Kb, size_t party_stride,
                                                          size_t stride_r, size_t stride_k, size_t dst_party_stride,
                                                          int taps)
{
    const int rb = blockIdx.x, kb = blockIdx.y, r16 = threadIdx.x & 15, kq = threadIdx.x >> 4;
    const int row = rb * 16 + r16, k0 = kb * 64 + 4 * kq;
    const u64 *s = src + (size_t)blockIdx.z * party_stride + (size_t)row * stride_r;
    const int C = taps ? K / taps : 1;
    u64 y[4];
#pragma unroll
    for (int c = 0; c < 4; c++) {
        const int k = k0 + c, ks = taps ? (k % C) * taps + k / C : k;
        y[c] = (row < rows && k < K) ? balanced_digits(s[(size_t)ks * stride_k]) : 0;
    }
    store_digits(y, dst + (size_t)blockIdx.z * dst_party_stride + ((size_t)rb * Kb + kb) * TILE, r16, kq);
}

// rows = (b, ho, wo), k = (c, r, s) gathered from x [n][B][C][H][W]; zero padding
__global__ __launch_bounds__(256) void pack_im2col_kernel(const u64 *__restrict__ x, v4i *__restrict__ dst, int B,
                                                          int C, int H, int W, int kh, int kw, int stride, int pad,
                                                          int Ho, int Wo, int Kb, size_t dst_party_stride)
{
    const int rb = blockIdx.x, kb = blockIdx.y, r16 = threadIdx.x & 15, kq = threadIdx.x >> 4;
    const int M = B * Ho * Wo, K = C * kh * kw;
    const int row = rb * 16 + r16, k0 = kb * 64 + 4 * kq;
    const u64 *xi = x + (size_t)blockIdx.z * B * C * H * W;
    u64 y[4] = {0, 0, 0, 0};
    if (row < M) {
        const int wo = row % Wo, ho = (row / Wo) % Ho, b = row / (Wo * Ho);
        int c = k0 / (kh * kw), rs = k0 % (kh * kw), r = rs / kw, s = rs % kw;
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const int hi = ho * stride - pad + r, wi = wo * stride - pad + s;
            if (k0 + q < K && hi >= 0 && hi < H && wi >= 0 && wi < W)
                y[q] = balanced_digits(xi[(((size_t)b * C + c) * H + hi) * W + wi]);
            if (++s == kw) { s = 0; if (++r == kh) { r = 0; ++c; } }
        }
    }
    store_digits(y, dst + (size_t)blockIdx.z * dst_party_stride + ((size_t)rb * Kb + kb) * TILE, r16, kq);
}

// The two kernels below take one element per thread: lane l of a wave holds row (or pixel) l%16 and the
// contraction index (or channel) 4 g + l/16 of the wave's group g of four.  The four lanes of a row swap
// their digit words (ds_bpermute), after which each of them owns all four and writes two of the eight limb
// dwords.  The layers of a batch-1 network are small: one element per thread is what fills the chip.

// shares of element e of the plaintext tensor, as GEN (Eq. 1) draws them (element index = position in the
// tensor, so the values are those of the plain share kernel): stored, and returned as digit words
template <int N, int T>
__device__ __forceinline__ void gen_digits(const u64 *__restrict__ secret, u64 *__restrict__ shares, size_t count,
                                           size_t e, int n, int t, const ss_keys &keys, u64 (&dig)[N ? N : SS_MAXN])
{
    constexpr int MAXP = N ? N : SS_MAXN, MAXD = T ? T : SS_MAXT;
    const u64 a0 = secret[e], counter = ss_counter(e);
    u64 c[MAXD];
#pragma unroll
    for (int j = 0; j < MAXD; j++) c[j] = (j < t) ? ss_draw_field_at(keys.k[j], counter) : 0;
    if constexpr (N != 0) {
        eval_points<T, N>(a0, c, [&](int p, u64 v) {
            shares[(size_t)p * count + e] = v;
            dig[p] = balanced_digits(v);
        });
    } else {
#pragma unroll
        for (int p = 0; p < MAXP; p++) {
            if (p < n) {
                const u64 v = ss_poly_eval<MAXD>(a0, c, t, p + 1);
                shares[(size_t)p * count + e] = v;
                dig[p] = balanced_digits(v);
            }
        }
    }
}

// GEN (Eq. 1) of the input of a dense or 1x1 convolution layer and its limb
// tiles in one pass.  The secret is [B][K][HW] (dense: HW = 1); operand row
// (b, hw), contraction index k.  grid (row blocks, 4 Kb), block 256: wave w of
// block (rb, y) takes the group of four contraction indices 4 y + w of row block
// rb.  N, T > 0 fix the scheme at compile time, 0 takes the run-time values.
template <int N, int T>
__global__ __launch_bounds__(256) void share_pack_kernel(const u64 *__restrict__ secret, u64 *__restrict__ shares,
                                                         v4i *__restrict__ dst, int B, int K, int HW, int Kb,
                                                         size_t dst_party_stride, int n_rt, int t_rt, ss_keys keys)
{
    constexpr int MAXP = N ? N : SS_MAXN;
    const int n = N ? N : n_rt, t = T ? T : t_rt;
    const int lane = threadIdx.x & 63, r16 = lane & 15, j = lane >> 4;
    const int g = blockIdx.y * 4 + (threadIdx.x >> 6), kb = g >> 4, kq = g & 15;
    const int rb = blockIdx.x, row = rb * 16 + r16, k = kb * 64 + 4 * kq + j, rows = B * HW;
    u64 dig[MAXP];
#pragma unroll
    for (int p = 0; p < MAXP; p++) dig[p] = 0;   // digits of padding rows and columns
    if (row < rows && k < K) {
        const int b = row / HW, hw = row - b * HW;
        gen_digits<N, T>(secret, shares, (size_t)B * K * HW, ((size_t)b * K + k) * HW + hw, n, t, keys, dig);
    }
    u32 *base = reinterpret_cast<u32 *>(dst + ((size_t)rb * Kb + kb) * TILE) + (r16 + 16 * (kq >> 2)) * 4 + (kq & 3);
#pragma unroll
    for (int p = 0; p < MAXP; p++) {
        if (p < n) {
            u64 y[4];
#pragma unroll
            for (int q = 0; q < 4; q++) y[q] = __shfl(dig[p], r16 + 16 * q);
            u32 *bp = base + (size_t)p * dst_party_stride * 4;
            if (2 * j < NL) {   // lane group j writes limbs 2j and 2j+1
                bp[(2 * j) * 256] = limb_dword(y, 2 * j);
                bp[(2 * j + 1) * 256] = limb_dword(y, 2 * j + 1);
            }
        }
    }
}

// Conv input [B][C][H][W] -> channel-innermost limb planes [party][limb][b][h][w][c] (int8), the form the
// convolution kernel gathers its second operand from (16 consecutive channels of one tap of one output pixel
// are 16 consecutive bytes).  GEN: the input is the plaintext tensor and the kernel also is GEN (Eq. 1):
// it writes the n shares and their planes; otherwise the input is the share tensor [n][B][C][H][W].
// grid (pixel blocks of 16, C / 16), block 256: wave w of block (x, y) takes channels 16 y + 4 w .. +3.
// Every party's planes end in a pad whose first 16 bytes are zero (the source of taps in the padding).
template <int N, int T, bool GEN>
__global__ __launch_bounds__(256) void planes_kernel(const u64 *__restrict__ in, u64 *__restrict__ shares,
                                                     signed char *__restrict__ planes, int B, int C, int HW,
                                                     size_t party_bytes, int n_rt, int t_rt, ss_keys keys)
{
    constexpr int MAXP = N ? N : SS_MAXN;
    const int n = N ? N : n_rt, t = T ? T : t_rt;
    const int lane = threadIdx.x & 63, r16 = lane & 15, j = lane >> 4;
    const int pix = blockIdx.x * 16 + r16, c0 = blockIdx.y * 16 + 4 * (threadIdx.x >> 6);
    const size_t plane = (size_t)B * HW * C;
    if (blockIdx.x == 0 && blockIdx.y == 0 && (int)threadIdx.x < n)
        *reinterpret_cast<v4i *>(planes + threadIdx.x * party_bytes + NL * plane) = (v4i){0, 0, 0, 0};
    u64 dig[MAXP];
#pragma unroll
    for (int p = 0; p < MAXP; p++) dig[p] = 0;
    const bool live = pix < B * HW;
    if (live) {
        const int b = pix / HW, hw = pix - b * HW;
        const size_t e = ((size_t)b * C + (c0 + j)) * HW + hw;
        if constexpr (GEN) {
            gen_digits<N, T>(in, shares, plane, e, n, t, keys, dig);
        } else {
#pragma unroll
            for (int p = 0; p < MAXP; p++)
                if (p < n) dig[p] = balanced_digits(in[(size_t)p * plane + e]);
        }
    }
#pragma unroll
    for (int p = 0; p < MAXP; p++) {
        if (p < n) {
            u64 y[4];
#pragma unroll
            for (int q = 0; q < 4; q++) y[q] = __shfl(dig[p], r16 + 16 * q);
            if (live && 2 * j < NL) {
                u32 *bp = reinterpret_cast<u32 *>(planes + p * party_bytes + (size_t)pix * C + c0);
                bp[(2 * j) * (plane / 4)] = limb_dword(y, 2 * j);
                bp[(2 * j + 1) * (plane / 4)] = limb_dword(y, 2 * j + 1);
            }
        }
    }
}

// The same with four channels per thread (thread t of block (pixel block, channel block of 64): pixel t%16,
// channels from 4 (t/16)): fewer, longer threads, the better shape for large tensors.
template <int N, int T, bool GEN>
__global__ __launch_bounds__(256) void planes4_kernel(const u64 *__restrict__ in, u64 *__restrict__ shares,
                                                     signed char *__restrict__ planes, int B, int C, int HW,
                                                     size_t party_bytes, int n_rt, int t_rt, ss_keys keys)
{
    constexpr int MAXP = N ? N : SS_MAXN, MAXD = T ? T : SS_MAXT;
    const int n = N ? N : n_rt, t = T ? T : t_rt;
    const int pix = blockIdx.x * 16 + (threadIdx.x & 15), c0 = blockIdx.y * 64 + 4 * (threadIdx.x >> 4);
    const size_t plane = (size_t)B * HW * C, count = plane;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < MAXP && (int)threadIdx.x < n)
        *reinterpret_cast<v4i *>(planes + threadIdx.x * party_bytes + NL * plane) = (v4i){0, 0, 0, 0};
    if (pix >= B * HW) return;
    const int b = pix / HW, hw = pix - b * HW;
    u64 y[MAXP][4];
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const size_t e = ((size_t)b * C + (c0 + q)) * HW + hw;
        if constexpr (GEN) {
            const u64 a0 = in[e], counter = ss_counter(e);
            u64 c[MAXD];
#pragma unroll
            for (int j = 0; j < MAXD; j++) c[j] = (j < t) ? ss_draw_field_at(keys.k[j], counter) : 0;
            if constexpr (N != 0) {
                eval_points<T, N>(a0, c, [&](int p, u64 v) {
                    shares[(size_t)p * count + e] = v;
                    y[p][q] = balanced_digits(v);
                });
            } else {
#pragma unroll
                for (int p = 0; p < MAXP; p++) {
                    if (p < n) {
                        const u64 v = ss_poly_eval<MAXD>(a0, c, t, p + 1);
                        shares[(size_t)p * count + e] = v;
                        y[p][q] = balanced_digits(v);
                    }
                }
            }
        } else {
#pragma unroll
            for (int p = 0; p < MAXP; p++)
                if (p < n) y[p][q] = balanced_digits(in[(size_t)p * count + e]);
        }
    }
#pragma unroll
    for (int p = 0; p < MAXP; p++) {
        if (p < n) {
            u32 *dst = reinterpret_cast<u32 *>(planes + p * party_bytes + (size_t)pix * C + c0);
#pragma unroll
            for (int limb = 0; limb < NL; limb++) dst[limb * (plane / 4)] = limb_dword(y[p], limb);
        }
    }
}

struct gemm_args {
    const v4i *A, *B;          // packed operands, all parties
    u64 *out;
    u64 *partials;             // [tile][slot][64*64] residues of tiles shared between workgroups
    unsigned *counters;        // [tile], zero between launches
    int rows, cols, Rb, Cb, Kb, RT, CT;
    unsigned units;            // tiles * Kb (< 2^31), or 0: one whole tile per workgroup
    unsigned wlast, wrow;      // cost of one unit of the last column tile; of one k block over a whole tile row
    unsigned long long cost;   // of all units
    int slots;                 // partial slots per tile
    size_t a_party_stride, b_party_stride, out_party_stride, stride_row, stride_cb;
    int cdiv;
    u64 negbias;
    // second operand read straight from channel-innermost limb planes (convolution without a materialised
    // im2col): planes [party][limb][b][h][w][c] int8, contraction index (tap, channel), C a multiple of 64
    const v4i *planes, *zero;          // zero: 16 zero bytes, for taps that fall into the padding
    unsigned plane16, party16;         // strides of a limb plane and of a party, in 16-byte units
    int cvH, cvW, cvC16, cvKw, cvStride, cvPad, cvHoWo, cvWo, cvKbTap;   // C16 = C/16, KbTap = C/64
};

// where one wave's block of a unit comes from: limb slice q is the 64 lanes x 16 bytes at base + q * qs
struct wave_src {
    const v4i *p;    // block pointer (packed operand), or the party's planes (implicit operand)
    int hw, bpix;    // implicit operand: (h0 << 16) | (w0 & 0xffff) of this lane's output pixel, and the
                     // pixel index of its image, -1 if the lane's column is past the matrix
};

// the ND diagonal sums of one output -> canonical field element
#if defined(SS_FIELD_P45)
__device__ __forceinline__ u64 fold_diagonals(const v4i (&acc)[ND], int r, u64 negbias)
{
    u32 U[ND];
#pragma unroll
    for (int s = 0; s < ND; s++) U[s] = (u32)acc[s][r] ^ 0x80000000u;   // D_s + 2^31, non-negative
    const u64 g0 = (u64)U[0] + ((u64)U[1] << 8) + ((u64)U[2] << 16) + ((u64)U[3] << 24);   // < 2^57
    const u64 g1 = (u64)U[4] + ((u64)U[5] << 8) + ((u64)U[6] << 16) + ((u64)U[7] << 24);
    const u64 g2 = (u64)U[8] + ((u64)U[9] << 8) + ((u64)U[10] << 16);
    // g0 + g1 2^32 + g2 2^64.  With g = a 2^13 + b: g 2^32 = a 2^45 + b 2^32 = 55 a + b 2^32, and
    // 2^64 = 55 2^19 (mod p)
    const u64 r1 = ss_reduce(g1), r2 = ss_reduce(g2);
    const u64 t1 = SS_PC * (r1 >> 13) + ((r1 & 0x1FFFull) << 32);   // < 2^38 + 2^45
    const u64 t2 = ss_mul(r2, SS_PC << 19);
    return ss_reduce(ss_fold(g0) + t1 + t2 + negbias);   // minus the 2^31 offsets
}
#else
__device__ __forceinline__ u64 fold_diagonals(const v4i (&acc)[15], int r, u64 negbias)
{
    u32 U[15];
#pragma unroll
    for (int s = 0; s < 15; s++) U[s] = (u32)acc[s][r] ^ 0x80000000u;   // D_s + 2^31, non-negative
    const u64 g0 = (u64)U[0] + ((u64)U[1] << 8) + ((u64)U[2] << 16) + ((u64)U[3] << 24);
    const u64 g1 = (u64)U[4] + ((u64)U[5] << 8) + ((u64)U[6] << 16) + ((u64)U[7] << 24);
    const u64 g2 = (u64)U[8] + ((u64)U[9] << 8) + ((u64)U[10] << 16) + ((u64)U[11] << 24);
    const u64 g3 = (u64)U[12] + ((u64)U[13] << 8) + ((u64)U[14] << 16);
    // g0 + g1 2^32 + g2 2^64 + g3 2^96 with 2^61 = 1: 2^64 = 2^3, 2^96 = 2^35
    const u64 tot = g0 + ((g1 & ((1ULL << 29) - 1)) << 32) + (g1 >> 29) + (g2 << 3) +
                    ((g3 & ((1ULL << 26) - 1)) << 35) + (g3 >> 26);
    return ss_reduce(ss_fold(tot) + negbias);   // minus the 2^31 offsets
}
#endif

// The units are dealt to the workgroups by cost, not by count: a unit of a full
// tile costs SS_UNIT_COST, a unit of the last column tile, where only some of
// the four column blocks exist and the MFMAs of the others are skipped, costs
// less (see unit_cost).  With cp(u) the summed cost of all units before u,
// workgroup s of G owns the units with floor(s cost / G) <= cp(u) <
// floor((s+1) cost / G).  cost / G >= SS_UNIT_COST, so no range is empty.
constexpr unsigned SS_UNIT_COST = 9;
// what one hand-over of a shared tile costs a workgroup, in the same scale: about 3.3 us, i.e. 1.3 units of
// eight limbs (2.5 us each) or 2.2 units of six (1.6 us each)
constexpr unsigned SS_HANDOVER_COST = SS_NLIMB == 8 ? 12 : 20;

// cost position of unit j of tile `tile`
__device__ __forceinline__ unsigned long long cost_before(const gemm_args &g, unsigned tile, unsigned j)
{
    const unsigned ct = tile % (unsigned)g.CT, rg = tile / (unsigned)g.CT;
    return (unsigned long long)rg * ((unsigned)g.Kb * g.wrow) + ct * SS_UNIT_COST * (unsigned)g.Kb +
           j * (ct == (unsigned)g.CT - 1 ? g.wlast : SS_UNIT_COST);
}

// first unit whose cost position is >= x
__device__ __forceinline__ unsigned unit_at(const gemm_args &g, unsigned long long x)
{
    const unsigned rowcost = (unsigned)g.Kb * g.wrow, tilecost = SS_UNIT_COST * (unsigned)g.Kb;
    const unsigned rg = (unsigned)(x / rowcost), rem = (unsigned)(x - (unsigned long long)rg * rowcost);
    const unsigned full = ((unsigned)g.CT - 1) * tilecost;
    unsigned ct, j;
    if (rem < full) {
        ct = rem / tilecost;
        j = (rem - ct * tilecost + SS_UNIT_COST - 1) / SS_UNIT_COST;
    } else {
        ct = (unsigned)g.CT - 1;
        j = (rem - full + g.wlast - 1) / g.wlast;
    }
    return (rg * (unsigned)g.CT + ct) * (unsigned)g.Kb + j;   // j == Kb: first unit of the next tile
}

// workgroup that owns the unit at cost position cp
__device__ __forceinline__ int owner_of(const gemm_args &g, unsigned long long cp, unsigned G)
{
    return (int)(((cp + 1) * G - 1) / g.cost);
}

// this wave's source block of tile `tile`: block `wave` of A for waves 0..3, of
// B for waves 4..7; blocks past the end are clamped (their products are
// computed and never stored)
template <bool IMPLICIT>
__device__ __forceinline__ wave_src tile_source(const gemm_args &g, unsigned tile, int wave, int lane)
{
    const int ct = (int)(tile % (unsigned)g.CT);
    const unsigned rem = tile / (unsigned)g.CT;
    const int rt = (int)(rem % (unsigned)g.RT), party = (int)(rem / (unsigned)g.RT);
    wave_src ws = {nullptr, 0, 0};
    if (wave < 4) {
        ws.p = g.A + (size_t)party * g.a_party_stride + (size_t)min(rt * 4 + wave, g.Rb - 1) * g.Kb * TILE + lane;
    } else if (!IMPLICIT) {
        ws.p = g.B + (size_t)party * g.b_party_stride + (size_t)min(ct * 4 + wave - 4, g.Cb - 1) * g.Kb * TILE + lane;
    } else {
        // lane l of a block holds column 16 cb + l%16 = output pixel (b, ho, wo)
        const int col = min(ct * 4 + wave - 4, g.Cb - 1) * 16 + (lane & 15);
        const int cc = min(col, g.cols - 1), b = cc / g.cvHoWo, r = cc - b * g.cvHoWo, ho = r / g.cvWo, wo = r - ho * g.cvWo;
        ws.p = g.planes + (size_t)party * g.party16;
        ws.hw = (int)((unsigned)(ho * g.cvStride - g.cvPad) << 16) | ((wo * g.cvStride - g.cvPad) & 0xffff);
        ws.bpix = col < g.cols ? b * g.cvH * g.cvW : -1;
    }
    return ws;
}

// base address and limb stride (16-byte units) of the wave's block for k block kb
template <bool IMPLICIT>
__device__ __forceinline__ const v4i *unit_base(const gemm_args &g, const wave_src &ws, int kb, int wave, int lane,
                                                unsigned &qs)
{
    if (!IMPLICIT || wave < 4) {
        qs = 64;
        return ws.p + (size_t)kb * TILE;
    }
    // k block kb = channels [64 (kb % KbTap), +64) of tap kb / KbTap; this lane: 16 of them
    const int tap = kb / g.cvKbTap, c16 = (kb - tap * g.cvKbTap) * 4 + (lane >> 4);
    const int r = tap / g.cvKw, sx = tap - r * g.cvKw;
    const int hi = (ws.hw >> 16) + r, wi = (int)(short)(ws.hw & 0xffff) + sx;
    const bool ok = ws.bpix >= 0 && (unsigned)hi < (unsigned)g.cvH && (unsigned)wi < (unsigned)g.cvW;
    qs = ok ? g.plane16 : 0;
    return ok ? ws.p + (size_t)(ws.bpix + hi * g.cvW + wi) * g.cvC16 + c16 : g.zero;
}

// Persistent kernel, one workgroup of 8 waves (4 x 2) per CU.  The work is the
// flat list of units (output tile of 64 x 64, k block of 64), tile-major; each
// workgroup takes one contiguous range of it, of equal cost, so every CU gets
// the same amount of work whatever the layer shape, and a tile whose k range is
// cut by a range boundary is finished by the hand-over below.  Wave (wr, wc) owns row block wr
// and column blocks 2wc, 2wc+1 of the tile (2 x 15 accumulator tiles); the two
// waves of a SIMD differ in wc.
//
// Per unit the workgroup needs four row blocks of A and four column blocks of
// B, 8 KB each and already in MFMA lane order, so wave w copies block w (A for
// w < 4, B otherwise) straight into LDS with eight 1 KB global->LDS loads; two
// stages, the next unit's loads (also across a tile boundary) in flight during
// the 128 MFMAs per wave of the current one.
//
// Hand-over of a tile shared by several workgroups (which may sit on different
// XCDs with separate L2s): each contributor folds its partial sums to residues,
// stores them with agent-scope atomic stores, waits for these stores and bumps
// the tile's counter; the contributor that arrives last adds the others'
// residues (agent-scope atomic loads) to its own and writes the output.  No
// cache-wide fence is used: it would evict the operand tiles that all other
// workgroups are reusing.  Integer sums are exact, so the result does not
// depend on how the units were dealt or on arrival order.
template <bool IMPLICIT>
__global__ __launch_bounds__(512) void gemm_limb_kernel(gemm_args g)
{
    extern __shared__ v4i lds[];   // 2 stages x (4 A blocks + 4 B blocks) x TILE
    constexpr int STAGE = 8 * TILE;
    __shared__ unsigned arrival;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wr = wave & 3, wc = wave >> 2;
    const unsigned G = gridDim.x;
    // consecutive ranges go to workgroups of the same XCD (workgroups are dealt
    // round-robin to the 8 XCDs), so that neighbours in the list share an L2
    const unsigned slot = (G % 8 == 0) ? (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8 : blockIdx.x;
    unsigned u0, u1;
    if (g.units) {
        u0 = unit_at(g, (unsigned long long)slot * g.cost / G);
        u1 = unit_at(g, (unsigned long long)(slot + 1) * g.cost / G);
    } else {   // one whole tile per workgroup; unit numbers are relative to it
        u0 = 0;
        u1 = (unsigned)g.Kb;
    }
    if (u0 >= u1) return;
    v4i *mine = lds + wave * TILE;   // wave-uniform LDS destination of this wave's block

    unsigned tile = g.units ? u0 / (unsigned)g.Kb : slot;
    int kb = (int)(u0 - (g.units ? tile * (unsigned)g.Kb : 0));
    wave_src src = tile_source<IMPLICIT>(g, tile, wave, lane);
    {
        unsigned qs;
        const v4i *ub = unit_base<IMPLICIT>(g, src, kb, wave, lane, qs);
#pragma unroll
        for (int q = 0; q < NL; q++) __builtin_amdgcn_global_load_lds(ub + (size_t)q * qs, mine + q * 64, 16, 0, 0);
    }
    int st = 0;

    // column blocks of this wave that lie inside the matrix (0 if its row block lies outside): MFMAs of
    // blocks past the edge are skipped, so a ragged last tile costs only its valid part
    auto valid_blocks = [&](unsigned t) {
        const int ct = (int)(t % (unsigned)g.CT), rt = (int)(t / (unsigned)g.CT % (unsigned)g.RT);
        if (rt * 4 + wr >= g.Rb) return 0;
        return max(0, min(2, g.Cb - (ct * 4 + 2 * wc)));
    };

    unsigned u = u0;
    while (u < u1) {
        const int nblk = valid_blocks(tile);
        const int kb_first = kb;
        v4i acc[2][ND];
#pragma unroll
        for (int h = 0; h < 2; h++)
#pragma unroll
            for (int s = 0; s < ND; s++) acc[h][s] = (v4i){0, 0, 0, 0};

        // units of this tile that belong to this workgroup
        const int kb_end = min(g.Kb, kb + (int)(u1 - u));
        wave_src next_src = src;
        for (; kb < kb_end; kb++, u++) {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of the unit is in LDS
            __syncthreads();                      // everyone's part is; stage st^1 is no longer read
            if (u + 1 < u1) {
                int nkb = kb + 1;
                if (nkb == g.Kb) {
                    nkb = 0;
                    next_src = tile_source<IMPLICIT>(g, tile + 1, wave, lane);
                }
                if constexpr (!IMPLICIT) {
#pragma unroll
                    for (int q = 0; q < NL; q++)
                        __builtin_amdgcn_global_load_lds(next_src.p + (size_t)nkb * TILE + q * 64,
                                                         mine + (st ^ 1) * STAGE + q * 64, 16, 0, 0);
                } else {
                    unsigned qs;
                    const v4i *ub = unit_base<true>(g, next_src, nkb, wave, lane, qs);
#pragma unroll
                    for (int q = 0; q < NL; q++)
                        __builtin_amdgcn_global_load_lds(ub + (size_t)q * qs, mine + (st ^ 1) * STAGE + q * 64, 16, 0, 0);
                }
            }
            const v4i *sa = lds + st * STAGE + wr * TILE + lane;
            const v4i *sb = lds + st * STAGE + 4 * TILE + wc * 2 * TILE + lane;
            if (nblk == 2) {   // the usual case, kept free of branches so that loads and MFMAs interleave
                v4i a[NL];
#pragma unroll
                for (int i = 0; i < NL; i++) a[i] = sa[i * 64];
#pragma unroll
                for (int h = 0; h < 2; h++) {
                    v4i b[NL];
#pragma unroll
                    for (int j = 0; j < NL; j++) b[j] = sb[h * TILE + j * 64];
#pragma unroll
                    for (int i = 0; i < NL; i++)
#pragma unroll
                        for (int j = 0; j < NL; j++)
                            acc[h][i + j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[h][i + j], 0, 0, 0);
                }
            } else if (nblk == 1) {   // ragged edge: only the first column block is inside the matrix
                v4i a[NL], b[NL];
#pragma unroll
                for (int i = 0; i < NL; i++) {
                    a[i] = sa[i * 64];
                    b[i] = sb[i * 64];
                }
#pragma unroll
                for (int i = 0; i < NL; i++)
#pragma unroll
                    for (int j = 0; j < NL; j++)
                        acc[0][i + j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[0][i + j], 0, 0, 0);
            }
            st ^= 1;
        }
        // lane holds, per column block h, column lane%16 and rows 4*(lane/16)+r
        u64 v[2][4];
#pragma unroll
        for (int h = 0; h < 2; h++)
#pragma unroll
            for (int r = 0; r < 4; r++) v[h][r] = fold_diagonals(acc[h], r, g.negbias);

        const int ct = (int)(tile % (unsigned)g.CT);
        const unsigned rem = tile / (unsigned)g.CT;
        const int rt = (int)(rem % (unsigned)g.RT), party = (int)(rem / (unsigned)g.RT);
        const int lrow = wr * 16 + 4 * (lane >> 4), lcol = wc * 32 + (lane & 15);   // within the 64 x 64 tile
        bool finish = true;
        if (kb_first != 0 || kb_end != g.Kb) {   // the tile is shared: uniform over the workgroup
            const int first = owner_of(g, cost_before(g, tile, 0), G),
                      last = owner_of(g, cost_before(g, tile, (unsigned)g.Kb - 1), G);
            u64 *part = g.partials + (size_t)tile * g.slots * 4096;
            const int my = (int)slot - first;
#pragma unroll
            for (int h = 0; h < 2; h++)
#pragma unroll
                for (int r = 0; r < 4; r++)
                    __hip_atomic_store(&part[(size_t)my * 4096 + (lrow + r) * 64 + lcol + 16 * h], v[h][r],
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the stores above are done
            __syncthreads();
            if (tid == 0)
                arrival = __hip_atomic_fetch_add(&g.counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            finish = arrival == (unsigned)(last - first);
            if (finish) {
                if (tid == 0) __hip_atomic_store(&g.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int s = 0; s <= last - first; s++) {
                    if (s == my) continue;
#pragma unroll
                    for (int h = 0; h < 2; h++)
#pragma unroll
                        for (int r = 0; r < 4; r++)
                            v[h][r] = ss_add(v[h][r],
                                             __hip_atomic_load(&part[(size_t)s * 4096 + (lrow + r) * 64 + lcol + 16 * h],
                                                               __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                }
            }
            __syncthreads();   // `arrival` may be rewritten by the next tile
        }
        if (finish) {
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int col = ct * 64 + lcol + 16 * h;
                u64 *op = g.out + (size_t)party * g.out_party_stride + (size_t)(col / g.cdiv) * g.stride_cb + (col % g.cdiv);
#pragma unroll
                for (int r = 0; r < 4; r++) {
                    const int row = rt * 64 + lrow + r;
                    if (row < g.rows && col < g.cols) op[(size_t)row * g.stride_row] = v[h][r];
                }
            }
        }
        if (kb == g.Kb) {
            kb = 0;
            tile++;
            src = next_src;
        }
    }
}

// The same contraction for a first operand of at most 16 rows (dense layers at a small batch, convolutions
// with few output channels).  There the time goes into reading the second operand once, so a launch is as
// fast as it keeps bytes in flight: a workgroup's tile is 16 rows x 128 columns, one row block and eight
// column blocks per unit, twice the column blocks of the square tile in the same LDS, and no MFMA is spent on
// row blocks that do not exist.  Wave w copies column block w and limb slice w of the row block, and owns
// the 16 x 16 outputs of column block w.  Units, ranges, hand-over and epilogue are those of the kernel above
// (a shared tile has 16 x 128 partial residues).
constexpr int SKINNY_COLS = 128, SKINNY_PART = 16 * SKINNY_COLS;

__global__ __launch_bounds__(512) void gemm_skinny_kernel(gemm_args g)
{
    extern __shared__ v4i lds[];   // 2 stages x (1 row block + 8 column blocks) x TILE
    __shared__ unsigned arrival;
    constexpr int STAGE = 9 * TILE;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const unsigned G = gridDim.x;
    const unsigned slot = (G % 8 == 0) ? (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8 : blockIdx.x;
    unsigned u0, u1;
    if (g.units) {
        u0 = unit_at(g, (unsigned long long)slot * g.cost / G);
        u1 = unit_at(g, (unsigned long long)(slot + 1) * g.cost / G);
    } else {
        u0 = 0;
        u1 = (unsigned)g.Kb;
    }
    if (u0 >= u1) return;

    // this wave's column block of tile t (clamped past the edge: computed, never stored) and its limb slice
    // of the party's row block
    auto b_source = [&](unsigned t) {
        const int ct = (int)(t % (unsigned)g.CT), party = (int)(t / (unsigned)g.CT);
        return g.B + (size_t)party * g.b_party_stride + (size_t)min(ct * 8 + wave, g.Cb - 1) * g.Kb * TILE + lane;
    };
    auto a_source = [&](unsigned t) {
        const int party = (int)(t / (unsigned)g.CT);
        return g.A + (size_t)party * g.a_party_stride + min(wave, NL - 1) * 64 + lane;
    };
    auto copy_unit = [&](const v4i *as, const v4i *bs, int k, int stage) {
        v4i *dst = lds + stage * STAGE;
#pragma unroll
        for (int q = 0; q < NL; q++)
            __builtin_amdgcn_global_load_lds(bs + (size_t)k * TILE + q * 64, dst + (1 + wave) * TILE + q * 64, 16, 0, 0);
        if (wave < NL) __builtin_amdgcn_global_load_lds(as + (size_t)k * TILE, dst + wave * 64, 16, 0, 0);
    };

    unsigned tile = g.units ? u0 / (unsigned)g.Kb : slot;
    int kb = (int)(u0 - (g.units ? tile * (unsigned)g.Kb : 0));
    const v4i *as = a_source(tile), *bs = b_source(tile);
    copy_unit(as, bs, kb, 0);
    int st = 0;

    unsigned u = u0;
    while (u < u1) {
        const int ct = (int)(tile % (unsigned)g.CT), party = (int)(tile / (unsigned)g.CT);
        const bool inside = ct * 8 + wave < g.Cb;   // this wave's column block lies inside the matrix
        const int kb_first = kb;
        v4i acc[ND];
#pragma unroll
        for (int s = 0; s < ND; s++) acc[s] = (v4i){0, 0, 0, 0};

        const int kb_end = min(g.Kb, kb + (int)(u1 - u));
        const v4i *next_as = as, *next_bs = bs;
        for (; kb < kb_end; kb++, u++) {
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of the unit is in LDS
            __syncthreads();                      // everyone's part is; stage st^1 is no longer read
            if (u + 1 < u1) {
                int nkb = kb + 1;
                if (nkb == g.Kb) {
                    nkb = 0;
                    next_as = a_source(tile + 1);
                    next_bs = b_source(tile + 1);
                }
                copy_unit(next_as, next_bs, nkb, st ^ 1);
            }
            if (inside) {
                const v4i *sa = lds + st * STAGE + lane, *sb = lds + st * STAGE + (1 + wave) * TILE + lane;
                v4i a[NL], b[NL];
#pragma unroll
                for (int i = 0; i < NL; i++) {
                    a[i] = sa[i * 64];
                    b[i] = sb[i * 64];
                }
#pragma unroll
                for (int i = 0; i < NL; i++)
#pragma unroll
                    for (int j = 0; j < NL; j++)
                        acc[i + j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[i + j], 0, 0, 0);
            }
            st ^= 1;
        }

        // lane holds column lane%16 of its block and rows 4*(lane/16)+r
        u64 v[4];
#pragma unroll
        for (int r = 0; r < 4; r++) v[r] = fold_diagonals(acc, r, g.negbias);
        const int lrow = 4 * (lane >> 4), lcol = wave * 16 + (lane & 15);   // within the 16 x 128 tile
        bool finish = true;
        if (kb_first != 0 || kb_end != g.Kb) {   // the tile is shared: uniform over the workgroup
            const int first = owner_of(g, cost_before(g, tile, 0), G),
                      last = owner_of(g, cost_before(g, tile, (unsigned)g.Kb - 1), G);
            u64 *part = g.partials + (size_t)tile * g.slots * SKINNY_PART;
            const int my = (int)slot - first;
#pragma unroll
            for (int r = 0; r < 4; r++)
                __hip_atomic_store(&part[(size_t)my * SKINNY_PART + (lrow + r) * SKINNY_COLS + lcol], v[r], __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the stores above are done
            __syncthreads();
            if (tid == 0)
                arrival = __hip_atomic_fetch_add(&g.counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __syncthreads();
            finish = arrival == (unsigned)(last - first);
            if (finish) {
                if (tid == 0) __hip_atomic_store(&g.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                for (int s = 0; s <= last - first; s++) {
                    if (s == my) continue;
#pragma unroll
                    for (int r = 0; r < 4; r++)
                        v[r] = ss_add(v[r], __hip_atomic_load(&part[(size_t)s * SKINNY_PART + (lrow + r) * SKINNY_COLS + lcol],
                                                              __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                }
            }
            __syncthreads();   // `arrival` may be rewritten by the next tile
        }
        if (finish) {
            const int col = ct * SKINNY_COLS + lcol;
            u64 *op = g.out + (size_t)party * g.out_party_stride + (size_t)(col / g.cdiv) * g.stride_cb + (col % g.cdiv);
#pragma unroll
            for (int r = 0; r < 4; r++)
                if (lrow + r < g.rows && col < g.cols) op[(size_t)(lrow + r) * g.stride_row] = v[r];
        }
        if (kb == g.Kb) {
            kb = 0;
            tile++;
            as = next_as;
            bs = next_bs;
        }
    }
}

__global__ void zero_words_kernel(unsigned *p, size_t nwords)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) p[i] = 0;
}

// residue of sum_{s<ND} 2^31 2^(8s), negated
u64 neg_bias()
{
    u64 b = 0, w = ss_reduce(1ULL << 31);
    for (int s = 0; s < ND; s++) {
        b = ss_add(b, w);
        w = ss_mul(w, 256);
    }
    return ss_neg(b);
}

struct gemm_plan {
    bool skinny;               // first operand of at most 16 rows: tiles of 16 x 128 (gemm_skinny_kernel)
    long tiles, units;
    int Kb, G, slots;
    unsigned wlast, wrow;
    unsigned long long cost;
};

// relative duration of a unit in which `vb` of the four column blocks exist:
// a fixed part (copy, barrier, LDS reads) plus one part per column block, as
// measured; the full unit is SS_UNIT_COST
unsigned unit_cost(int vb)
{
    static const unsigned w[5] = {0, 4, 6, 7, SS_UNIT_COST};
    return w[vb];
}

// How the units are dealt: one workgroup per CU unless there are fewer units
// than CUs; slots = the most workgroups that can share one tile.  When there are
// more tiles than arrival counters every workgroup gets whole tiles.
gemm_plan plan_gemm(int n, int rows, int cols, int K, bool allow_skinny)
{
    gemm_plan p;
    p.skinny = allow_skinny && rows <= 16;
    p.Kb = (K + 63) / 64;
    p.tiles = p.skinny ? (long)n * ((cols + SKINNY_COLS - 1) / SKINNY_COLS)
                       : (long)n * ((rows + 63) / 64) * ((cols + 63) / 64);
    p.units = p.tiles * p.Kb;
    if (p.tiles > SS_GEMM_MAX_SPLIT_TILES || p.units >= (1L << 31)) {
        p.G = (int)(p.tiles < (1L << 30) ? p.tiles : 0);   // 0: not launchable, rejected by the caller
        p.slots = 0;
        p.units = 0;
        p.wlast = p.wrow = SS_UNIT_COST;
        p.cost = 0;
        return p;
    }
    if (p.skinny) {   // every unit copies the same nine blocks: one cost for all
        const int CT = (cols + SKINNY_COLS - 1) / SKINNY_COLS;
        p.wlast = SS_UNIT_COST;
        p.wrow = (unsigned)CT * SS_UNIT_COST;
        p.cost = (unsigned long long)n * p.Kb * p.wrow;
    } else {
        const int CT = (cols + 63) / 64, Cb = (cols + 15) / 16;
        p.wlast = unit_cost(Cb - 4 * (CT - 1));
        p.wrow = (unsigned)(CT - 1) * SS_UNIT_COST + p.wlast;
        p.cost = (unsigned long long)n * ((rows + 63) / 64) * p.Kb * p.wrow;
    }
    // Whole tiles or shared tiles?  Dealt by cost, a workgroup runs cost / G and hands over at both ends of its
    // range (measured: each hand-over costs about SS_HANDOVER_COST / SS_UNIT_COST units).  With one whole tile
    // per workgroup nothing is handed over and the launch lasts as many tiles as the fullest CU gets.  With a
    // single k block tiles are never shared, so there is nothing to choose.
    if (p.Kb > 1) {
        const unsigned long long rounds = ((unsigned long long)p.tiles + SS_GEMM_CUS - 1) / SS_GEMM_CUS;
        const unsigned long long whole = rounds * p.Kb * SS_UNIT_COST;
        const unsigned long long g = p.cost / SS_UNIT_COST < SS_GEMM_CUS ? (p.cost / SS_UNIT_COST ? p.cost / SS_UNIT_COST : 1) : SS_GEMM_CUS;
        const unsigned long long shared = p.cost / g + 2 * SS_HANDOVER_COST;
        if (whole <= shared) {
            p.G = (int)p.tiles;
            p.slots = 0;
            p.units = 0;
            p.cost = 0;
            return p;
        }
    }
    // every range must hold at least one unit start: cost / G >= SS_UNIT_COST
    const unsigned long long most = p.cost / SS_UNIT_COST;
    p.G = (int)(most < SS_GEMM_CUS ? (most ? most : 1) : SS_GEMM_CUS);
    // a tile of cost <= SS_UNIT_COST Kb meets at most this many ranges of length >= cost / G
    const unsigned long long share = p.cost / p.G;
    p.slots = (int)(((unsigned long long)SS_UNIT_COST * p.Kb + share - 1) / share) + 1;
    return p;
}

}  // namespace


size_t ss_gemm_scratch_bytes(int n, int rows, int cols, int K)
{
    // room for either form (an operand given as limb planes never takes the 16-row form)
    const gemm_plan p = plan_gemm(n, rows, cols, K, false), q = plan_gemm(n, rows, cols, K, true);
    const size_t a = (size_t)p.tiles * p.slots * 4096, b = q.skinny ? (size_t)q.tiles * q.slots * SKINNY_PART : 0;
    return (a > b ? a : b) * sizeof(u64);
}

hipError_t ss_launch_zero_counters(unsigned *counters, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_words_kernel, dim3((SS_GEMM_MAX_SPLIT_TILES + 255) / 256), dim3(256), 0, stream, counters,
                       (size_t)SS_GEMM_MAX_SPLIT_TILES);
    return hipGetLastError();
}

size_t ss_packed_bytes(int rows, int K)
{
    return (size_t)((rows + 15) / 16) * (size_t)((K + 63) / 64) * (TILE * 16);
}

hipError_t ss_launch_pack_matrix(const u64 *src, void *dst, int n, int rows, int K, size_t party_stride,
                                 size_t stride_r, size_t stride_k, int taps, hipStream_t stream)
{
    const int Rb = (rows + 15) / 16, Kb = (K + 63) / 64;
    hipLaunchKernelGGL(pack_matrix_kernel, dim3(Rb, Kb, n), dim3(256), 0, stream, src, (v4i *)dst, rows, K, Kb,
                       party_stride, stride_r, stride_k, ss_packed_bytes(rows, K) / 16, taps);
    return hipGetLastError();
}

hipError_t ss_launch_share_pack(const u64 *secret, u64 *shares, void *dst, int n, int t, int B, int K, int HW,
                                const ss_keys &keys, hipStream_t stream)
{
    const int rows = B * HW, Rb = (rows + 15) / 16, Kb = (K + 63) / 64;
    const dim3 grid(Rb, Kb * 4), block(256);
    const size_t stride = ss_packed_bytes(rows, K) / 16;
#define SS_SHARE_PACK(NC, TC) \
    hipLaunchKernelGGL((share_pack_kernel<NC, TC>), grid, block, 0, stream, secret, shares, (v4i *)dst, B, K, HW, Kb, stride, n, t, keys)
    if (n == 5 && t == 2)
        SS_SHARE_PACK(5, 2);
    else if (n == 3 && t == 1)
        SS_SHARE_PACK(3, 1);
    else
        SS_SHARE_PACK(0, 0);
#undef SS_SHARE_PACK
    return hipGetLastError();
}

hipError_t ss_launch_planes(const u64 *in, u64 *shares, void *planes, int n, int t, int B, int C, int HW, bool gen,
                            const ss_keys &keys, hipStream_t stream)
{
    // one element per thread fills the chip for the small tensors of a batch-1 network; from about half a
    // million elements on, four per thread move the data with fewer instructions
    const bool big = (size_t)B * HW * C >= ((size_t)1 << 19);
    const dim3 grid((B * HW + 15) / 16, big ? C / 64 : C / 16), block(256);
    const size_t party_bytes = ss_planes_bytes(B, C, HW, 1);
#define SS_PLANES(NC, TC, G)                                                                                        \
    do {                                                                                                            \
        if (big)                                                                                                    \
            hipLaunchKernelGGL((planes4_kernel<NC, TC, G>), grid, block, 0, stream, in, shares, (signed char *)planes, B, \
                               C, HW, party_bytes, n, t, keys);                                                     \
        else                                                                                                        \
            hipLaunchKernelGGL((planes_kernel<NC, TC, G>), grid, block, 0, stream, in, shares, (signed char *)planes, B,  \
                               C, HW, party_bytes, n, t, keys);                                                     \
    } while (0)
    if (!gen)
        SS_PLANES(0, 0, false);
    else if (n == 5 && t == 2)
        SS_PLANES(5, 2, true);
    else if (n == 3 && t == 1)
        SS_PLANES(3, 1, true);
    else
        SS_PLANES(0, 0, true);
#undef SS_PLANES
    return hipGetLastError();
}

hipError_t ss_launch_pack_im2col(const u64 *x, void *dst, int n, int B, int C, int H, int W, int kh, int kw,
                                 int stride, int pad, int Ho, int Wo, hipStream_t stream)
{
    const int M = B * Ho * Wo, K = C * kh * kw;
    const int Rb = (M + 15) / 16, Kb = (K + 63) / 64;
    hipLaunchKernelGGL(pack_im2col_kernel, dim3(Rb, Kb, n), dim3(256), 0, stream, x, (v4i *)dst, B, C, H, W, kh, kw,
                       stride, pad, Ho, Wo, Kb, ss_packed_bytes(M, K) / 16);
    return hipGetLastError();
}

namespace {

struct conv_planes {   // geometry of an operand given as channel-innermost limb planes
    const void *planes;
    int B, C, H, W, kh, kw, stride, pad, Ho, Wo;
};

hipError_t launch_gemm(const void *packedA, const void *packedB, const conv_planes *cv, u64 *out, int n, int rows,
                       int cols, int K, size_t out_party_stride, size_t stride_row, int cdiv, size_t stride_cb,
                       unsigned *counters, u64 *partials, hipStream_t stream)
{
    static bool lds_opt_in = false;
    constexpr int LDS_BYTES = 2 * 8 * TILE * 16, LDS_BYTES_SKINNY = 2 * 9 * TILE * 16;
    if (!lds_opt_in) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_limb_kernel<false>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)gemm_limb_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    LDS_BYTES);
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)gemm_skinny_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    LDS_BYTES_SKINNY);
        if (e != hipSuccess) return e;
        lds_opt_in = true;
    }
    const gemm_plan p = plan_gemm(n, rows, cols, K, cv == nullptr);
    if (p.G <= 0) return hipErrorInvalidValue;
    gemm_args g = {};
    g.A = (const v4i *)packedA;
    g.B = (const v4i *)packedB;
    g.out = out;
    g.partials = partials;
    g.counters = counters;
    g.rows = rows;
    g.cols = cols;
    g.Rb = (rows + 15) / 16;
    g.Cb = (cols + 15) / 16;
    g.Kb = p.Kb;
    g.RT = p.skinny ? 1 : (rows + 63) / 64;
    g.CT = p.skinny ? (cols + SKINNY_COLS - 1) / SKINNY_COLS : (cols + 63) / 64;
    g.units = (unsigned)p.units;
    g.wlast = p.wlast;
    g.wrow = p.wrow;
    g.cost = p.cost;
    g.slots = p.slots;
    g.a_party_stride = ss_packed_bytes(rows, K) / 16;
    g.b_party_stride = ss_packed_bytes(cols, K) / 16;
    g.out_party_stride = out_party_stride;
    g.stride_row = stride_row;
    g.stride_cb = stride_cb;
    g.cdiv = cdiv;
    g.negbias = neg_bias();
    if (cv) {
        const size_t plane = (size_t)cv->B * cv->H * cv->W * cv->C;   // bytes
        g.planes = (const v4i *)cv->planes;
        g.plane16 = (unsigned)(plane / 16);
        g.party16 = (unsigned)(ss_planes_bytes(cv->B, cv->C, cv->H, cv->W) / 16);
        g.zero = g.planes + (size_t)NL * g.plane16;   // the pad behind the first party's planes
        g.cvH = cv->H, g.cvW = cv->W, g.cvC16 = cv->C / 16, g.cvKw = cv->kw, g.cvStride = cv->stride, g.cvPad = cv->pad;
        g.cvHoWo = cv->Ho * cv->Wo, g.cvWo = cv->Wo, g.cvKbTap = cv->C / 64;
    }
    if (p.skinny)
        hipLaunchKernelGGL(gemm_skinny_kernel, dim3((unsigned)p.G), dim3(512), LDS_BYTES_SKINNY, stream, g);
    else if (cv)
        hipLaunchKernelGGL(gemm_limb_kernel<true>, dim3((unsigned)p.G), dim3(512), LDS_BYTES, stream, g);
    else
        hipLaunchKernelGGL(gemm_limb_kernel<false>, dim3((unsigned)p.G), dim3(512), LDS_BYTES, stream, g);
    return hipGetLastError();
}

}  // namespace

size_t ss_planes_bytes(int B, int C, int H, int W)
{
    return (size_t)NL * B * H * W * C + 256;   // the limb planes and a pad that starts with 16 zero bytes
}

hipError_t ss_launch_gemm(const void *packedA, const void *packedB, u64 *out, int n, int rows, int cols, int K,
                          size_t out_party_stride, size_t stride_row, int cdiv, size_t stride_cb, unsigned *counters,
                          u64 *partials, hipStream_t stream)
{
    return launch_gemm(packedA, packedB, nullptr, out, n, rows, cols, K, out_party_stride, stride_row, cdiv, stride_cb,
                       counters, partials, stream);
}

hipError_t ss_launch_gemm_conv(const void *packedW, const void *planes, u64 *out, int n, int B, int C, int H, int W,
                               int Co, int kh, int kw, int stride, int pad, int Ho, int Wo, unsigned *counters,
                               u64 *partials, hipStream_t stream)
{
    const conv_planes cv = {planes, B, C, H, W, kh, kw, stride, pad, Ho, Wo};
    const size_t HW = (size_t)Ho * Wo;
    // rows = output channel, cols = (b, ho, wo): y[b][co][hw]
    return launch_gemm(packedW, nullptr, &cv, out, n, Co, (int)(B * HW), C * kh * kw, (size_t)B * Co * HW, HW, (int)HW,
                       (size_t)Co * HW, counters, partials, stream);
}

}  // namespace SS_NS
