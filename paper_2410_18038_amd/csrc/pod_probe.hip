// Two micro-kernels that measure what this GPU can sustain: a coalesced HBM read stream and an
// MFMA issue loop.  The benchmark reports the attention kernels against these measured peaks
// next to the datasheet ones.
#include <hip/hip_runtime.h>

#include "../../include/pod_attn.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kThreads = 256;
constexpr int kUnroll = 8;

// Every lane reads 16 bytes per load, a wavefront 1 KiB of consecutive memory; kUnroll loads are
// in flight per lane.  The xor keeps the loads alive; the store never happens for real data.
__global__ __launch_bounds__(kThreads) void hbm_read_kernel(const u32x4 *src, size_t n_vec, uint32_t *sink)
{
    const size_t stride = (size_t)gridDim.x * kThreads;
    size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (kUnroll - 1) * stride < n_vec; i += kUnroll * stride) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= v[u];
    }
    for (; i < n_vec; i += stride) acc ^= src[i];
    if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9e3779b9u) sink[0] = acc.x;
}

__global__ __launch_bounds__(kThreads) void mfma_loop_kernel(int iters, float *sink)
{
    f16x8 a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (_Float16)(0.001f * (float)(threadIdx.x + i));
        b[i] = (_Float16)(0.002f * (float)(threadIdx.x - i));
    }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
    }
    const float s = c0[0] + c1[1] + c2[2] + c3[3];
    if (s == 12345.678f) sink[0] = s;
}

}  // namespace

extern "C" {

pod_status pod_attn_probe_hbm_read(const void *buf, size_t bytes, void *sink, void *stream)
{
    if (!buf || !sink || bytes < 16) return POD_ERR_INVALID_ARG;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess) return POD_ERR_HIP;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    hbm_read_kernel<<<dim3(cus * 8), dim3(kThreads), 0, (hipStream_t)stream>>>(
        (const u32x4 *)buf, bytes / 16, (uint32_t *)sink);
    return hipGetLastError() == hipSuccess ? POD_OK : POD_ERR_HIP;
}

pod_status pod_attn_probe_mfma(int32_t iters, void *sink, double *flops_out, void *stream)
{
    if (!sink || iters <= 0) return POD_ERR_INVALID_ARG;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess) return POD_ERR_HIP;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const int grid = cus * 2;                       // 8 wavefronts per compute unit, 2 per SIMD
    mfma_loop_kernel<<<dim3(grid), dim3(kThreads), 0, (hipStream_t)stream>>>(iters, (float *)sink);
    if (flops_out) *flops_out = (double)grid * (kThreads / 64) * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
    return hipGetLastError() == hipSuccess ? POD_OK : POD_ERR_HIP;
}

}  // extern "C"
