// Measured ceilings of the machine for the roofline reports: what a plain device copy, the write pattern of
// GEN (one plane read, several written) and a register-resident int8 MFMA loop reach on this GPU.  Bench
// support only: nothing here is on the share path.
#include "../../include/ssnet.h"

#include "field.hpp"

namespace SS_NS {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

// dst plane q (q < planes) <- src, 16 bytes per lane: planes = 1 is a copy, planes = n the traffic of GEN
__global__ __launch_bounds__(256) void probe_planes_kernel(v4i *__restrict__ dst, const v4i *__restrict__ src, size_t n16,
                                                           int planes)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n16) return;
    const v4i v = src[i];
    for (int q = 0; q < planes; q++) __builtin_nontemporal_store(v, dst + (size_t)q * n16 + i);
}

// Two waves per SIMD, each with eight + eight operand registers and fifteen accumulator tiles as in the
// product kernel, 64 products per round, nothing but MFMAs in the loop.  random != 0: operand bytes from the
// generator (the clock this part sustains depends on how many bits toggle), else small constants.
__global__ __launch_bounds__(512) void probe_mfma_kernel(int rounds, int random, int *sink)
{
    v4i a[8], b[8], acc[15];
    const u64 lane_key = ss_mix64(0x1234 + threadIdx.x + 512ull * blockIdx.x);
#pragma unroll
    for (int i = 0; i < 8; i++) {
        const u64 x = ss_mix64(lane_key + i), y = ss_mix64(lane_key + 64 + i);
        a[i] = random ? (v4i){(int)x, (int)(x >> 32), (int)y, (int)(y >> 32)} : (v4i){1, 2, 3, i};
        const u64 z = ss_mix64(lane_key + 128 + i), w = ss_mix64(lane_key + 192 + i);
        b[i] = random ? (v4i){(int)z, (int)(z >> 32), (int)w, (int)(w >> 32)} : (v4i){4, 5, i, 7};
    }
#pragma unroll
    for (int s = 0; s < 15; s++) acc[s] = (v4i){0, 0, 0, 0};
    for (int r = 0; r < rounds; r++) {
#pragma unroll
        for (int i = 0; i < 8; i++)
#pragma unroll
            for (int j = 0; j < 8; j++) acc[i + j] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a[i], b[j], acc[i + j], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int q = 0; q < 15; q++) s += acc[q][0] ^ acc[q][1] ^ acc[q][2] ^ acc[q][3];
    if (s == 0x7FFFFFF1) sink[0] = s;   // keeps the loop alive
}

// elapsed milliseconds of `reps` runs of launch() on `stream`, after one warm-up run
template <typename F>
hipError_t timed_runs(hipStream_t stream, int reps, float *ms, F &&launch)
{
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) {
        (void)hipEventDestroy(e0);
        return e;
    }
    launch();
    e = hipEventRecord(e0, stream);
    for (int r = 0; r < reps && e == hipSuccess; r++) launch();
    if (e == hipSuccess) e = hipGetLastError();
    if (e == hipSuccess) e = hipEventRecord(e1, stream);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return e;
}

}  // namespace
}  // namespace SS_NS

using namespace SS_NS;

extern "C" {

int ssnet_probe_planes(void *hip_stream, void *d_dst, const void *d_src, size_t bytes, int planes, int reps,
                       double *gb_per_s)
{
    if (!d_dst || !d_src || !gb_per_s || bytes < 16 || bytes % 16 || planes < 1 || planes > 64 || reps < 1 ||
        ((uintptr_t)d_dst & 15) || ((uintptr_t)d_src & 15) || bytes / 16 > ((size_t)1 << 39))
        return SSNET_EINVAL;
    const size_t n16 = bytes / 16;
    float ms = 0.f;
    hipError_t e = timed_runs((hipStream_t)hip_stream, reps, &ms, [&]() {
        hipLaunchKernelGGL(probe_planes_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, (hipStream_t)hip_stream,
                           (v4i *)d_dst, (const v4i *)d_src, n16, planes);
    });
    if (e != hipSuccess) return SSNET_EHIP;
    *gb_per_s = (double)bytes * (1 + planes) * reps / (ms * 1e-3) / 1e9;
    return SSNET_OK;
}

int ssnet_probe_mfma_int8(void *hip_stream, void *d_sink, int random_operands, int reps, double *tera_ops_per_s)
{
    if (!d_sink || !tera_ops_per_s || reps < 1 || ((uintptr_t)d_sink & 3)) return SSNET_EINVAL;
    const int rounds = 512, blocks = 256;   // one workgroup of eight waves per compute unit
    float ms = 0.f;
    hipError_t e = timed_runs((hipStream_t)hip_stream, reps, &ms, [&]() {
        hipLaunchKernelGGL(probe_mfma_kernel, dim3(blocks), dim3(512), 0, (hipStream_t)hip_stream, rounds, random_operands,
                           (int *)d_sink);
    });
    if (e != hipSuccess) return SSNET_EHIP;
    const double ops = (double)blocks * 8 * rounds * 64 * (2.0 * 16 * 16 * 64) * reps;
    *tera_ops_per_s = ops / (ms * 1e-3) / 1e12;
    return SSNET_OK;
}

}  // extern "C"
