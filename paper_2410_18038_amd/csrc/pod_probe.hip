// Micro-kernels.  Two measure what this GPU can sustain: a coalesced HBM read stream and an MFMA
// issue loop; the benchmark reports the attention kernels against these measured peaks next to
// the datasheet ones.  A third group is the co-location experiment of the paper's Section 3.3
// (a compute-bound and a memory-bound operation, run one after the other, fused by workgroup
// index, and fused with roles bound per compute unit at run time).
#include <hip/hip_runtime.h>

#include "../../include/pod_attn.h"

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kUnroll = 8;

// Every lane reads 16 bytes per load, a wavefront 1 KiB of consecutive memory; kUnroll loads are
// in flight per lane; every workgroup walks a contiguous region of its own.  Of the patterns tried
// (grid-stride, one region per workgroup, one region per wavefront; 256 to 1024 threads; one to
// eight workgroups per compute unit; with and without the non-temporal hint) this one, with two
// workgroups of 256 threads per unit, read fastest on MI355X: 7.2-7.3 TB/s against 6.2-6.3 for a
// grid-stride loop with eight workgroups per unit.  The xor keeps the loads alive; the store never
// happens for real data.
__global__ __launch_bounds__(kThreads) void hbm_read_kernel(const u32x4 *src, size_t n_vec, uint32_t *sink)
{
    const size_t per = (n_vec + gridDim.x - 1) / gridDim.x;
    const size_t end = per * (blockIdx.x + 1) < n_vec ? per * (blockIdx.x + 1) : n_vec;
    size_t i = per * blockIdx.x + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (; i + (kUnroll - 1) * kThreads < end; i += kUnroll * kThreads) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + u * kThreads);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) acc ^= v[u];
    }
    for (; i < end; i += kThreads) acc ^= src[i];
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

// ---- co-location experiment (Section 3.3, Figure 7) -------------------------------------------
// Compute item: every thread runs `iters` rounds of eight independent multiply-adds.  Memory
// item: c = a + b over a chunk of n_vec 16-byte vectors, coalesced.  Both use 256 threads and
// few registers, so eight workgroups of either kind fit on a compute unit.
struct ColoArgs {
    const f32x4 *a, *b;
    f32x4 *c;
    uint32_t *ctr;                  // [1024] per-unit tickets, then [2] next item of each kind
    float *sink;
    uint32_t n_vec;                 // vectors per memory item
    int32_t n_cmp, n_mem, iters;
};

__device__ __forceinline__ void colo_compute(const ColoArgs &g, int item)
{
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = 0.001f * (float)(threadIdx.x + i + item);
    const float m = 1.0000001f, d = 1e-7f;
    for (int it = 0; it < g.iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = __builtin_fmaf(x[i], m, d);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += x[i];
    if (s == 12345.678f) g.sink[0] = s;
}

__device__ __forceinline__ void colo_memory(const ColoArgs &g, int item)
{
    const size_t base = (size_t)item * g.n_vec;
    for (uint32_t i = threadIdx.x; i < g.n_vec; i += 4 * kThreads) {
        f32x4 va[4], vb[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = i + u * kThreads;
            if (j < g.n_vec) {
                va[u] = __builtin_nontemporal_load(g.a + base + j);
                vb[u] = __builtin_nontemporal_load(g.b + base + j);
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t j = i + u * kThreads;
            if (j < g.n_vec) {
                const f32x4 r = va[u] + vb[u];
                __builtin_nontemporal_store(r, g.c + base + j);
            }
        }
    }
}

__global__ __launch_bounds__(kThreads) void colo_compute_kernel(ColoArgs g) { colo_compute(g, blockIdx.x); }
__global__ __launch_bounds__(kThreads) void colo_memory_kernel(ColoArgs g) { colo_memory(g, blockIdx.x); }

// Fusion by workgroup index: the first n_cmp workgroups compute, the rest move memory.  Which
// compute unit a workgroup lands on, and when, is the hardware's choice.
__global__ __launch_bounds__(kThreads) void colo_fused_by_index_kernel(ColoArgs g)
{
    if ((int)blockIdx.x < g.n_cmp) colo_compute(g, blockIdx.x);
    else colo_memory(g, blockIdx.x - g.n_cmp);
}

// Fusion with run-time binding (Section 4.1): the workgroup asks which compute unit it is on,
// takes that unit's next ticket, alternates between the two operations by ticket parity, claims
// the next item of its operation, and takes the other operation's work when its own has run out.
__global__ __launch_bounds__(kThreads) void colo_fused_bound_kernel(ColoArgs g)
{
    __shared__ int pick[2];
    if (threadIdx.x == 0) {
        const unsigned cu = __smid() & 1023u;
        const uint32_t ticket = atomicAdd(&g.ctr[cu], 1u);
        int role = (int)(ticket & 1u);                       // 0 compute, 1 memory
        int item = (int)atomicAdd(&g.ctr[1024 + role], 1u);
        if (item >= (role == 0 ? g.n_cmp : g.n_mem)) {
            role ^= 1;
            item = (int)atomicAdd(&g.ctr[1024 + role], 1u);
            if (item >= (role == 0 ? g.n_cmp : g.n_mem)) role = -1;
        }
        pick[0] = role;
        pick[1] = item;
    }
    __syncthreads();
    if (pick[0] == 0) colo_compute(g, pick[1]);
    else if (pick[0] == 1) colo_memory(g, pick[1]);
}


// ---- instruction-mix probe ------------------------------------------------------------------
// What a SIMD of this chip can overlap: dense matrix instructions alone, and beside the vector
// work a softmax does per score (scale-and-shift, 2^x, a maximum, rounding to 16 bit, the weight
// sum), with the sum taken either by plain additions or by two-element dot products.  The
// prefill loop's choices (where its time goes, why the weight sum matters, why one wavefront per
// SIMD with a wider tile does not pay) rest on these figures.  Every variant is a loop over
// "turns"; the mix of a turn is fixed at compile time and held in place by scheduling barriers.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int NM, int NE, int NF, int NC, int NX, int ND>
__global__ __launch_bounds__(kThreads) void issue_mix_kernel(int iters, float seed, float *sink)
{
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = seed * (float)(i + r);
    bf16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (__bf16)(seed + (float)i); b[i] = (__bf16)(seed * (float)i); }
    float e[8], f[8], m[4], d[2];
    uint32_t c[4];
    for (int i = 0; i < 8; ++i) { e[i] = seed * (float)(threadIdx.x + i) * 1e-3f; f[i] = seed + (float)i; }
    for (int i = 0; i < 4; ++i) { m[i] = seed - (float)i; c[i] = (uint32_t)i; }
    d[0] = d[1] = seed;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < NM; ++t) {
            acc[t & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[t & 3], 0, 0, 0);
#pragma unroll
            for (int i = 0; i < NE; ++i) asm volatile("v_exp_f32 %0, %0" : "+v"(e[(t * NE + i) & 7]));
#pragma unroll
            for (int i = 0; i < NF; ++i) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(f[(t * NF + i) & 7]) : "v"(seed));
#pragma unroll
            for (int i = 0; i < NC; ++i)
                asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(c[(t * NC + i) & 3]) : "v"(f[(i + 4) & 7]), "v"(e[(i + 4) & 7]));
#pragma unroll
            for (int i = 0; i < NX; ++i)
                asm volatile("v_max3_f32 %0, %0, %1, %2" : "+v"(m[(t * NX + i) & 3]) : "v"(f[(i + 5) & 7]), "v"(e[(i + 5) & 7]));
#pragma unroll
            for (int i = 0; i < ND; ++i)
                asm volatile("v_dot2_f32_bf16 %0, %1, %2, %0" : "+v"(d[i & 1]) : "v"(c[(i + 2) & 3]), "v"(c[(i + 3) & 3]));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = d[0] + d[1];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    for (int i = 0; i < 8; ++i) s += e[i] + f[i];
    for (int i = 0; i < 4; ++i) s += m[i] + (float)c[i];
    if (s == 12345.678f) sink[0] = s;
}

// A turn of a software-pipelined tile loop: one 16-byte LDS fragment read (three turns ahead), NMF
// matrix instructions that share the fragment, and the softmax work of NMF scores per lane in
// three stages that are one turn apart, so that no instruction depends on a result of its own turn.
template <int NMF>
__global__ __launch_bounds__(kThreads) void issue_turn_kernel(int iters, float seed, float *sink)
{
    __shared__ u32x4 lds[1024];
    for (int i = threadIdx.x; i < 1024; i += kThreads) lds[i] = u32x4{1u, 2u, 3u, (uint32_t)i};
    __syncthreads();
    f32x16 acc[4];
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = seed * (float)(i + r);
    bf16x8 b;
    for (int i = 0; i < 8; ++i) b[i] = (__bf16)(seed * (float)i);
    float s1[NMF], s2[NMF], s3[NMF], lsum = 0.f, mx = seed;
    uint32_t pw = 0;
    for (int i = 0; i < NMF; ++i) { s1[i] = seed * (float)i; s2[i] = seed + (float)i; s3[i] = seed - (float)i; }
    u32x4 frag[3];
    const __attribute__((address_space(3))) u32x4 *lp = (const __attribute__((address_space(3))) u32x4 *)lds + (threadIdx.x & 63);
    frag[0] = lp[0]; frag[1] = lp[64]; frag[2] = lp[128];
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            const bf16x8 a = __builtin_bit_cast(bf16x8, frag[t]);
#pragma unroll
            for (int mm = 0; mm < NMF; ++mm)
                acc[(t * NMF + mm) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[(t * NMF + mm) & 3], 0, 0, 0);
            frag[t] = lp[((it * 3 + t) & 15) * 64];            // lands in the register it is used from, three turns on
#pragma unroll
            for (int mm = 0; mm < NMF; mm += 2)
                asm volatile("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(pw) : "v"(s3[mm]), "v"(s3[(mm + 1) % NMF]));
#pragma unroll
            for (int mm = 0; mm < NMF; ++mm) asm volatile("v_add_f32 %0, %0, %1" : "+v"(lsum) : "v"(s3[mm]));
#pragma unroll
            for (int mm = 0; mm < NMF; ++mm) asm volatile("v_exp_f32 %0, %1" : "=v"(s3[mm]) : "v"(s2[mm]));
#pragma unroll
            for (int mm = 0; mm < NMF; ++mm) asm volatile("v_fma_f32 %0, %1, %2, %2" : "=v"(s2[mm]) : "v"(s1[mm]), "v"(seed));
#pragma unroll
            for (int mm = 0; mm < NMF; ++mm) asm volatile("v_max_f32 %0, %0, %1" : "+v"(mx) : "v"(s1[mm]));
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    float s = lsum + mx + (float)pw;
    for (int i = 0; i < 4; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    if (s == 12345.678f) sink[0] = s;
}

// Vector instructions alone: eight independent chains of one instruction kind.  What one wavefront
// can issue by itself and what two reach together on a SIMD.
template <int KIND>
__global__ __launch_bounds__(kThreads) void issue_valu_kernel(int iters, float seed, float *sink)
{
    float x[8];
    for (int i = 0; i < 8; ++i) x[i] = seed * 0.5f + 0.001f * (float)(threadIdx.x + i);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if (KIND == 0) asm volatile("v_fma_f32 %0, %0, %1, %1" : "+v"(x[i]) : "v"(seed));
            else asm volatile("v_exp_f32 %0, %0" : "+v"(x[i]));
        }
    }
    float s = 0.f;
    for (int i = 0; i < 8; ++i) s += x[i];
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
    hbm_read_kernel<<<dim3(cus * 2), dim3(kThreads), 0, (hipStream_t)stream>>>(
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

pod_status pod_attn_probe_issue(int32_t variant, int32_t iters, int32_t wgs_per_unit, void *sink,
                                double *matrix_ops_per_wave, void *stream)
{
    if (!sink || iters <= 0 || wgs_per_unit < 1 || wgs_per_unit > 2) return POD_ERR_INVALID_ARG;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess) return POD_ERR_HIP;
    (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    const dim3 grid(cus * wgs_per_unit), block(kThreads);
    hipStream_t s = (hipStream_t)stream;
    float *out = (float *)sink;
    double per_iter = 4.0;
    switch (variant) {
    case 0: issue_mix_kernel<4, 0, 0, 0, 0, 0><<<grid, block, 0, s>>>(iters, 1.0f, out); break;
    case 1: issue_mix_kernel<4, 1, 0, 0, 0, 0><<<grid, block, 0, s>>>(iters, 1.0f, out); break;
    case 2: issue_mix_kernel<4, 1, 2, 1, 1, 0><<<grid, block, 0, s>>>(iters, 1.0f, out); break;
    case 3: issue_mix_kernel<4, 1, 2, 1, 1, 1><<<grid, block, 0, s>>>(iters, 1.0f, out); break;
    case 4: issue_mix_kernel<4, 0, 0, 0, 0, 1><<<grid, block, 0, s>>>(iters, 1.0f, out); break;
    case 5: issue_turn_kernel<1><<<grid, block, 0, s>>>(iters, 1.0f, out); per_iter = 3.0; break;
    case 6: issue_turn_kernel<2><<<grid, block, 0, s>>>(iters, 1.0f, out); per_iter = 6.0; break;
    case 7: issue_valu_kernel<0><<<grid, block, 0, s>>>(iters, 1.0f, out); per_iter = 8.0; break;
    case 8: issue_valu_kernel<1><<<grid, block, 0, s>>>(iters, 1.0f, out); per_iter = 8.0; break;
    default: return POD_ERR_INVALID_ARG;
    }
    if (matrix_ops_per_wave) *matrix_ops_per_wave = per_iter * (double)iters;
    return hipGetLastError() == hipSuccess ? POD_OK : POD_ERR_HIP;
}

pod_status pod_attn_probe_colocation(int32_t variant, const void *a, const void *b, void *c,
                                     size_t bytes_per_item, int32_t n_memory_items,
                                     int32_t n_compute_items, int32_t compute_iters, void *counters,
                                     void *sink, void *stream)
{
    if (variant < 0 || variant > 3 || !sink) return POD_ERR_INVALID_ARG;
    if (n_memory_items < 0 || n_compute_items < 0 || compute_iters < 0) return POD_ERR_INVALID_ARG;
    if (bytes_per_item % 16 != 0 || bytes_per_item / 16 > 0xffffffffull) return POD_ERR_INVALID_ARG;
    const bool uses_memory = variant != 0 && n_memory_items > 0;
    if (uses_memory && (!a || !b || !c)) return POD_ERR_INVALID_ARG;
    if (variant == 3 && !counters) return POD_ERR_INVALID_ARG;
    ColoArgs g;
    g.a = (const f32x4 *)a; g.b = (const f32x4 *)b; g.c = (f32x4 *)c;
    g.ctr = (uint32_t *)counters; g.sink = (float *)sink;
    g.n_vec = (uint32_t)(bytes_per_item / 16);
    g.n_cmp = n_compute_items; g.n_mem = n_memory_items; g.iters = compute_iters;
    hipStream_t s = (hipStream_t)stream;
    const int n_both = n_compute_items + n_memory_items;
    switch (variant) {
    case 0:
        if (n_compute_items > 0) colo_compute_kernel<<<dim3(n_compute_items), dim3(kThreads), 0, s>>>(g);
        break;
    case 1:
        if (n_memory_items > 0) colo_memory_kernel<<<dim3(n_memory_items), dim3(kThreads), 0, s>>>(g);
        break;
    case 2:
        if (n_both > 0) colo_fused_by_index_kernel<<<dim3(n_both), dim3(kThreads), 0, s>>>(g);
        break;
    default:
        if (n_both > 0) {
            if (hipMemsetAsync(counters, 0, 1026 * sizeof(uint32_t), s) != hipSuccess) return POD_ERR_HIP;
            colo_fused_bound_kernel<<<dim3(n_both), dim3(kThreads), 0, s>>>(g);
        }
        break;
    }
    return hipGetLastError() == hipSuccess ? POD_OK : POD_ERR_HIP;
}

}  // extern "C"
