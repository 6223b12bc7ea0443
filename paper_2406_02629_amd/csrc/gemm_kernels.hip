// Exact modular matrix product on int8 MFMA (SSS-Linear step 1, Sec. VI-A).
//
// A field element x < 2^61 is written in balanced radix 2^8,
//   x = sum_{i<8} d_i 2^(8i),  d_i in [-128, 127],
// which is one add and one xor: the bytes of x + 0x80..80 are d_i + 128.  The
// integer dot product sum_k x_k w_k is then sum_{i,j} 2^(8(i+j)) sum_k d_i(x_k)
// d_j(w_k): 64 int8 dot products, each exact in int32 for K <= 16383.  They are
// one int8 GEMM of shape (8 rows) x K x (8 cols): the limb index multiplies the
// row and column counts, so one wave holds a 16 x 16 tile of field outputs as
// 8 x 8 MFMA 16x16x64 accumulators.  The epilogue adds the 64 accumulators of
// each output along anti-diagonals, propagates them into a 61-bit residue with
// 2^61 = 1 (mod p) and stores the canonical field element.
#include "kernels.hpp"

typedef int v4i __attribute__((ext_vector_type(4)));

namespace {

constexpr u64 BAL = 0x8080808080808080ULL;

// balanced digits of x as 8 signed bytes
__device__ __forceinline__ u64 balanced_digits(u64 x) { return (x + BAL) ^ BAL; }

// bytes `limb` of 16 digit words -> one 16-byte MFMA operand row
__device__ __forceinline__ v4i gather_limb(const u64 (&y)[16], int limb)
{
    v4i o;
#pragma unroll
    for (int w = 0; w < 4; w++) {
        u32 acc = 0;
#pragma unroll
        for (int c = 0; c < 4; c++) acc |= (u32)((y[4 * w + c] >> (8 * limb)) & 0xFF) << (8 * c);
        o[w] = (int)acc;
    }
    return o;
}

__device__ __forceinline__ void store_tiles(const u64 (&y)[16], v4i *dst, int rb, int kb, int Kb, int lane)
{
    v4i *tile = dst + ((size_t)rb * Kb + kb) * 512 + lane;
#pragma unroll
    for (int limb = 0; limb < 8; limb++) tile[limb * 64] = gather_limb(y, limb);
}

// grid (Rb, ceil(Kb/4), n), block (64, 4): one wave per (row block, k block)
__global__ __launch_bounds__(256) void pack_matrix_kernel(const u64 *__restrict__ src, v4i *__restrict__ dst,
                                                          int rows, int K, int Kb, size_t party_stride,
                                                          size_t stride_r, size_t stride_k, size_t dst_party_stride)
{
    const int lane = threadIdx.x, kb = blockIdx.y * 4 + threadIdx.y, rb = blockIdx.x;
    if (kb >= Kb) return;
    const int row = rb * 16 + (lane & 15), k0 = kb * 64 + 16 * (lane >> 4);
    const u64 *s = src + (size_t)blockIdx.z * party_stride + (size_t)row * stride_r;
    u64 y[16];
#pragma unroll
    for (int b = 0; b < 16; b++) {
        const int k = k0 + b;
        y[b] = (row < rows && k < K) ? balanced_digits(s[(size_t)k * stride_k]) : 0;
    }
    store_tiles(y, dst + (size_t)blockIdx.z * dst_party_stride, rb, kb, Kb, lane);
}

// rows = (b, ho, wo), k = (c, r, s) gathered from x [n][B][C][H][W]; zero padding
__global__ __launch_bounds__(256) void pack_im2col_kernel(const u64 *__restrict__ x, v4i *__restrict__ dst, int B,
                                                          int C, int H, int W, int kh, int kw, int stride, int pad,
                                                          int Ho, int Wo, int Kb, size_t dst_party_stride)
{
    const int lane = threadIdx.x, kb = blockIdx.y * 4 + threadIdx.y, rb = blockIdx.x;
    if (kb >= Kb) return;
    const int M = B * Ho * Wo, K = C * kh * kw;
    const int row = rb * 16 + (lane & 15), k0 = kb * 64 + 16 * (lane >> 4);
    const u64 *xi = x + (size_t)blockIdx.z * B * C * H * W;
    u64 y[16];
    if (row < M) {
        const int wo = row % Wo, ho = (row / Wo) % Ho, b = row / (Wo * Ho);
        int c = k0 / (kh * kw), rs = k0 % (kh * kw), r = rs / kw, s = rs % kw;
#pragma unroll
        for (int q = 0; q < 16; q++) {
            const int hi = ho * stride - pad + r, wi = wo * stride - pad + s;
            const bool ok = (k0 + q < K) && hi >= 0 && hi < H && wi >= 0 && wi < W;
            y[q] = ok ? balanced_digits(xi[(((size_t)b * C + c) * H + hi) * W + wi]) : 0;
            if (++s == kw) { s = 0; if (++r == kh) { r = 0; ++c; } }
        }
    } else {
#pragma unroll
        for (int q = 0; q < 16; q++) y[q] = 0;
    }
    store_tiles(y, dst + (size_t)blockIdx.z * dst_party_stride, rb, kb, Kb, lane);
}

// One workgroup = 4 waves (2 x 2) = 32 x 32 field outputs.  Per k block the
// workgroup stages two row blocks of A and two of B (16 KB each, already in
// MFMA lane order) through LDS, double buffered, with the next block's global
// loads in flight during the 64 MFMAs of the current one.
__global__ __launch_bounds__(256, 1) void gemm_limb_kernel(const v4i *__restrict__ A, const v4i *__restrict__ Bm,
                                                           u64 *__restrict__ out, int rows, int cols, int Rb,
                                                           int Cb, int Kb, size_t a_party_stride,
                                                           size_t b_party_stride, size_t out_party_stride,
                                                           size_t stride_row, int cdiv, size_t stride_cb, u64 negbias)
{
    __shared__ v4i lds[2][2048];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wr = wave >> 1, wc = wave & 1;
    const int rb0 = blockIdx.y * 2, cb0 = blockIdx.x * 2;
    const v4i *Ap = A + (size_t)blockIdx.z * a_party_stride;
    const v4i *Bp = Bm + (size_t)blockIdx.z * b_party_stride;

    // slot q of this thread: element tid + 256 q of a 1024-entry chunk; q = 0, 1
    // lie in the first block of the pair, q = 2, 3 in the second.  Blocks past
    // the end are clamped: their products are computed and never stored.
    const v4i *asrc[4], *bsrc[4];
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int half = q >> 1, within = (tid + 256 * q) & 511;
        const int rb = min(rb0 + half, Rb - 1), cb = min(cb0 + half, Cb - 1);
        asrc[q] = Ap + (size_t)rb * Kb * 512 + within;
        bsrc[q] = Bp + (size_t)cb * Kb * 512 + within;
    }

    v4i acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 8; j++) acc[i][j] = (v4i){0, 0, 0, 0};

    v4i pa[4], pb[4];
#pragma unroll
    for (int q = 0; q < 4; q++) {
        pa[q] = asrc[q][0];
        pb[q] = bsrc[q][0];
    }
#pragma unroll
    for (int q = 0; q < 4; q++) {
        lds[0][tid + 256 * q] = pa[q];
        lds[0][1024 + tid + 256 * q] = pb[q];
    }
    __syncthreads();

    for (int kb = 0; kb < Kb; kb++) {
        const int cur = kb & 1;
        const bool more = kb + 1 < Kb;
        if (more) {
#pragma unroll
            for (int q = 0; q < 4; q++) {
                pa[q] = asrc[q][(size_t)(kb + 1) * 512];
                pb[q] = bsrc[q][(size_t)(kb + 1) * 512];
            }
        }
        v4i a[8], b[8];
#pragma unroll
        for (int i = 0; i < 8; i++) {
            a[i] = lds[cur][wr * 512 + i * 64 + lane];
            b[i] = lds[cur][1024 + wc * 512 + i * 64 + lane];
        }
#pragma unroll
        for (int i = 0; i < 8; i++)
#pragma unroll
            for (int j = 0; j < 8; j++)
                acc[i][j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        if (more) {
#pragma unroll
            for (int q = 0; q < 4; q++) {
                lds[cur ^ 1][tid + 256 * q] = pa[q];
                lds[cur ^ 1][1024 + tid + 256 * q] = pb[q];
            }
        }
        __syncthreads();
    }

    // lane holds column lane%16 and rows 4*(lane/16)+r of the wave's 16 x 16 tile
    const int col = (cb0 + wc) * 16 + (lane & 15);
    u64 *op = out + (size_t)blockIdx.z * out_party_stride + (size_t)(col / cdiv) * stride_cb + (col % cdiv);
#pragma unroll
    for (int r = 0; r < 4; r++) {
        u32 U[15];
#pragma unroll
        for (int s = 0; s < 15; s++) {
            int d = 0;
#pragma unroll
            for (int i = 0; i < 8; i++)
                if (s - i >= 0 && s - i < 8) d += acc[i][s - i][r];
            U[s] = (u32)d ^ 0x80000000u;   // d + 2^31, non-negative
        }
        const u64 g0 = (u64)U[0] + ((u64)U[1] << 8) + ((u64)U[2] << 16) + ((u64)U[3] << 24);
        const u64 g1 = (u64)U[4] + ((u64)U[5] << 8) + ((u64)U[6] << 16) + ((u64)U[7] << 24);
        const u64 g2 = (u64)U[8] + ((u64)U[9] << 8) + ((u64)U[10] << 16) + ((u64)U[11] << 24);
        const u64 g3 = (u64)U[12] + ((u64)U[13] << 8) + ((u64)U[14] << 16);
        // g0 + g1 2^32 + g2 2^64 + g3 2^96 with 2^61 = 1: 2^64 = 2^3, 2^96 = 2^35
        const u64 tot = g0 + ((g1 & ((1ULL << 29) - 1)) << 32) + (g1 >> 29) + (g2 << 3) +
                        ((g3 & ((1ULL << 26) - 1)) << 35) + (g3 >> 26);
        const u64 v = ss_reduce(ss_fold(tot) + negbias);   // minus the 2^31 offsets
        const int row = (rb0 + wr) * 16 + 4 * (lane >> 4) + r;
        if (row < rows && col < cols) op[(size_t)row * stride_row] = v;
    }
}

// residue of sum_{s<15} 2^31 2^(8s), negated
u64 neg_bias()
{
    u64 b = 0;
    for (int s = 0; s < 15; s++) b = ss_add(b, 1ULL << ((31 + 8 * s) % 61));
    return ss_neg(b);
}

}  // namespace

size_t ss_packed_bytes(int rows, int K)
{
    return (size_t)((rows + 15) / 16) * (size_t)((K + 63) / 64) * 8192;
}

hipError_t ss_launch_pack_matrix(const u64 *src, void *dst, int n, int rows, int K, size_t party_stride,
                                 size_t stride_r, size_t stride_k, hipStream_t stream)
{
    const int Rb = (rows + 15) / 16, Kb = (K + 63) / 64;
    hipLaunchKernelGGL(pack_matrix_kernel, dim3(Rb, (Kb + 3) / 4, n), dim3(64, 4), 0, stream, src, (v4i *)dst, rows, K,
                       Kb, party_stride, stride_r, stride_k, ss_packed_bytes(rows, K) / 16);
    return hipGetLastError();
}

hipError_t ss_launch_pack_im2col(const u64 *x, void *dst, int n, int B, int C, int H, int W, int kh, int kw,
                                 int stride, int pad, int Ho, int Wo, hipStream_t stream)
{
    const int M = B * Ho * Wo, K = C * kh * kw;
    const int Rb = (M + 15) / 16, Kb = (K + 63) / 64;
    hipLaunchKernelGGL(pack_im2col_kernel, dim3(Rb, (Kb + 3) / 4, n), dim3(64, 4), 0, stream, x, (v4i *)dst, B, C, H, W,
                       kh, kw, stride, pad, Ho, Wo, Kb, ss_packed_bytes(M, K) / 16);
    return hipGetLastError();
}

hipError_t ss_launch_gemm(const void *packedA, const void *packedB, u64 *out, int n, int rows, int cols, int K,
                          size_t out_party_stride, size_t stride_row, int cdiv, size_t stride_cb, hipStream_t stream)
{
    const int Rb = (rows + 15) / 16, Cb = (cols + 15) / 16, Kb = (K + 63) / 64;
    hipLaunchKernelGGL(gemm_limb_kernel, dim3((Cb + 1) / 2, (Rb + 1) / 2, n), dim3(256), 0, stream,
                       (const v4i *)packedA, (const v4i *)packedB, out, rows, cols, Rb, Cb, Kb,
                       ss_packed_bytes(rows, K) / 16, ss_packed_bytes(cols, K) / 16, out_party_stride, stride_row, cdiv,
                       stride_cb, neg_bias());
    return hipGetLastError();
}
