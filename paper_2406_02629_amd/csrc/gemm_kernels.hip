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

struct gemm_args {
    const v4i *A, *B;          // packed operands, all parties
    u64 *out;
    u64 *partials;             // [tile][S][64*64] field elements, used when S > 1
    unsigned *counters;        // [tile], zero between launches
    int rows, cols, Rb, Cb, Kb, RT, CT, S;
    size_t a_party_stride, b_party_stride, out_party_stride, stride_row, stride_cb;
    int cdiv;
    u64 negbias;
};

// 15 diagonal sums of one output -> canonical field element
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

// One workgroup = 8 waves (4 x 2) = 64 x 64 field outputs over the k blocks
// [kb0, kb1) of its split; wave (wr, wc) owns row block wr and column blocks
// 2wc, 2wc+1 (2 x 15 accumulator tiles).  Per k block the workgroup needs four
// row blocks of A and four column blocks of B, 8 KB each and already in MFMA
// lane order, so wave w copies block w (A for w < 4, B otherwise) straight
// into LDS with eight 1 KB global->LDS loads; two stages, the next block's
// loads in flight during the 128 MFMAs per wave of the current one.
//
// With S > 1 splits of the contraction, every split stores its residues to the
// partials buffer and bumps the tile's counter; the split that arrives last
// adds the others' residues to its own and writes the output.  Integer sums
// are exact, so the result does not depend on S or on arrival order.
__global__ __launch_bounds__(512) void gemm_limb_kernel(gemm_args g)
{
    extern __shared__ v4i lds[];   // 2 stages x (4 A blocks + 4 B blocks) x 512
    __shared__ unsigned arrival;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wr = wave >> 1, wc = wave & 1;
    int item = blockIdx.x;
    const int ks = item % g.S;
    item /= g.S;
    const int ct = item % g.CT;
    item /= g.CT;
    const int rt = item % g.RT, party = item / g.RT;
    const int kb0 = (int)((long)ks * g.Kb / g.S), kb1 = (int)((long)(ks + 1) * g.Kb / g.S);

    // this wave's source block; blocks past the end are clamped (their
    // products are computed and never stored)
    const v4i *src;
    if (wave < 4)
        src = g.A + (size_t)party * g.a_party_stride + (size_t)min(rt * 4 + wave, g.Rb - 1) * g.Kb * 512 + lane;
    else
        src = g.B + (size_t)party * g.b_party_stride + (size_t)min(ct * 4 + wave - 4, g.Cb - 1) * g.Kb * 512 + lane;
    v4i *mine = lds + wave * 512;   // wave-uniform LDS destination of this wave's block

    v4i acc[2][15];
#pragma unroll
    for (int h = 0; h < 2; h++)
#pragma unroll
        for (int s = 0; s < 15; s++) acc[h][s] = (v4i){0, 0, 0, 0};

#pragma unroll
    for (int u = 0; u < 8; u++)
        __builtin_amdgcn_global_load_lds(src + (size_t)kb0 * 512 + u * 64, mine + u * 64, 16, 0, 0);

    for (int kb = kb0; kb < kb1; kb++) {
        const int st = (kb - kb0) & 1;
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of block kb is in LDS
        __syncthreads();                      // everyone's part is; stage st^1 is no longer read
        if (kb + 1 < kb1) {
#pragma unroll
            for (int u = 0; u < 8; u++)
                __builtin_amdgcn_global_load_lds(src + (size_t)(kb + 1) * 512 + u * 64,
                                                 mine + (st ^ 1) * 4096 + u * 64, 16, 0, 0);
        }
        const v4i *sa = lds + st * 4096 + wr * 512 + lane;
        const v4i *sb = lds + st * 4096 + 2048 + wc * 1024 + lane;
        v4i a[8];
#pragma unroll
        for (int i = 0; i < 8; i++) a[i] = sa[i * 64];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            v4i b[8];
#pragma unroll
            for (int j = 0; j < 8; j++) b[j] = sb[h * 512 + j * 64];
#pragma unroll
            for (int i = 0; i < 8; i++)
#pragma unroll
                for (int j = 0; j < 8; j++)
                    acc[h][i + j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[h][i + j], 0, 0, 0);
        }
    }

    // lane holds, per column block h, column lane%16 and rows 4*(lane/16)+r
    u64 v[2][4];
#pragma unroll
    for (int h = 0; h < 2; h++)
#pragma unroll
        for (int r = 0; r < 4; r++) v[h][r] = fold_diagonals(acc[h], r, g.negbias);

    const int lrow = wr * 16 + 4 * (lane >> 4), lcol = wc * 32 + (lane & 15);   // within the 64 x 64 tile
    if (g.S > 1) {
        // Hand-over between workgroups that may sit on different XCDs (separate
        // L2s): the residues and the counter are moved with agent-scope atomic
        // accesses, which are performed at the device's coherence point, and the
        // counter is bumped only after this workgroup's stores have completed.
        // No cache-wide fence is used: it would evict the operand tiles that all
        // other workgroups are reusing.
        const size_t tile = ((size_t)party * g.RT + rt) * g.CT + ct;
        u64 *part = g.partials + (tile * g.S) * 4096;
#pragma unroll
        for (int h = 0; h < 2; h++)
#pragma unroll
            for (int r = 0; r < 4; r++)
                __hip_atomic_store(&part[(size_t)ks * 4096 + (lrow + r) * 64 + lcol + 16 * h], v[h][r],
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): the stores above are done
        __syncthreads();
        if (tid == 0)
            arrival = __hip_atomic_fetch_add(&g.counters[tile], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (arrival != (unsigned)(g.S - 1)) return;
        if (tid == 0) __hip_atomic_store(&g.counters[tile], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        for (int s = 0; s < g.S; s++) {
            if (s == ks) continue;
#pragma unroll
            for (int h = 0; h < 2; h++)
#pragma unroll
                for (int r = 0; r < 4; r++)
                    v[h][r] = ss_add(v[h][r],
                                     __hip_atomic_load(&part[(size_t)s * 4096 + (lrow + r) * 64 + lcol + 16 * h],
                                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
        }
    }
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

__global__ void zero_words_kernel(unsigned *p, size_t nwords)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) p[i] = 0;
}

// residue of sum_{s<15} 2^31 2^(8s), negated
u64 neg_bias()
{
    u64 b = 0;
    for (int s = 0; s < 15; s++) b = ss_add(b, 1ULL << ((31 + 8 * s) % 61));
    return ss_neg(b);
}

}  // namespace

// Number of splits of the contraction: enough workgroups to occupy every CU a
// few times over, but each split keeps at least two k blocks.  Modelled cost per
// workgroup: a fixed part worth about 1.5 k blocks plus its k blocks; the CUs
// take the workgroups in rounds.
int ss_gemm_splits(int n, int rows, int cols, int K)
{
    const long tiles = (long)n * ((rows + 63) / 64) * ((cols + 63) / 64);
    const int Kb = (K + 63) / 64;
    if (tiles > SS_GEMM_MAX_SPLIT_TILES) return 1;
    int best = 1;
    double best_cost = 1e300;
    for (int S = 1; S <= 32 && S <= Kb; S++) {
        if (S > 1 && Kb / S < 2) break;
        const long rounds = (tiles * S + SS_GEMM_CUS - 1) / SS_GEMM_CUS;
        const double cost = (double)rounds * ((Kb + S - 1) / S + 1.5 + (S > 1 ? 0.5 : 0.0));
        if (cost < best_cost - 1e-9) {
            best_cost = cost;
            best = S;
        }
    }
    return best;
}

size_t ss_gemm_scratch_bytes(int n, int rows, int cols, int K)
{
    const size_t tiles = (size_t)n * ((rows + 63) / 64) * ((cols + 63) / 64);
    const int S = ss_gemm_splits(n, rows, cols, K);
    return S > 1 ? tiles * S * 4096 * sizeof(u64) : 0;
}

hipError_t ss_launch_zero_counters(unsigned *counters, hipStream_t stream)
{
    hipLaunchKernelGGL(zero_words_kernel, dim3((SS_GEMM_MAX_SPLIT_TILES + 255) / 256), dim3(256), 0, stream, counters,
                       (size_t)SS_GEMM_MAX_SPLIT_TILES);
    return hipGetLastError();
}

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
                          size_t out_party_stride, size_t stride_row, int cdiv, size_t stride_cb, unsigned *counters,
                          u64 *partials, hipStream_t stream)
{
    static bool lds_opt_in = false;
    constexpr int LDS_BYTES = 2 * 4096 * 16;
    if (!lds_opt_in) {
        hipError_t e = hipFuncSetAttribute((const void *)gemm_limb_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                           LDS_BYTES);
        if (e != hipSuccess) return e;
        lds_opt_in = true;
    }
    gemm_args g;
    g.A = (const v4i *)packedA;
    g.B = (const v4i *)packedB;
    g.out = out;
    g.partials = partials;
    g.counters = counters;
    g.rows = rows;
    g.cols = cols;
    g.Rb = (rows + 15) / 16;
    g.Cb = (cols + 15) / 16;
    g.Kb = (K + 63) / 64;
    g.RT = (rows + 63) / 64;
    g.CT = (cols + 63) / 64;
    g.S = ss_gemm_splits(n, rows, cols, K);
    g.a_party_stride = ss_packed_bytes(rows, K) / 16;
    g.b_party_stride = ss_packed_bytes(cols, K) / 16;
    g.out_party_stride = out_party_stride;
    g.stride_row = stride_row;
    g.stride_cb = stride_cb;
    g.cdiv = cdiv;
    g.negbias = neg_bias();
    const long items = (long)n * g.RT * g.CT * g.S;
    hipLaunchKernelGGL(gemm_limb_kernel, dim3((unsigned)items), dim3(512), LDS_BYTES, stream, g);
    return hipGetLastError();
}
