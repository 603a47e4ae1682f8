// Micro-kernels that measure what the machine delivers, for the benchmark's
// roofline fractions: a streaming read of a buffer and back-to-back matrix
// instructions.  They compute nothing of the method.
#include <hip/hip_runtime.h>

#include "slim_internal.h"

namespace slim {

typedef float float16v_t __attribute__((ext_vector_type(16)));

// Every workgroup of 512 threads reads runs of 64 KiB (8 x 16 bytes per thread) with
// a grid stride; the bytes past the last whole run are not read.
__global__ __launch_bounds__(512) void probe_read_kernel(const uint4_t *p, size_t n16, uint32_t *sink)
{
    uint4_t acc = {0u, 0u, 0u, 0u};
    const size_t run = (size_t)512 * 8;
    for (size_t base = (size_t)blockIdx.x * run; base + run <= n16; base += (size_t)gridDim.x * run) {
        uint4_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + base + u * 512 + threadIdx.x);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9e3779b9u) *sink = 1u;       // keeps the loads alive
}

// Four independent accumulator chains per wavefront, `iters` rounds: dense
// V_MFMA_F32_32X32X16_F16 (SPARSE = false) or V_SMFMAC_F32_32X32X32_F16.
template <bool SPARSE>
__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float *sink)
{
    const int lane = threadIdx.x & 63;
    half8_t a;
    half16_t b16;
#pragma unroll
    for (int i = 0; i < 8; ++i) a[i] = (half_t)(0.001f * (float)(lane + i));
#pragma unroll
    for (int i = 0; i < 16; ++i) b16[i] = (half_t)(0.002f * (float)(lane - i));
    half8_t b8;
#pragma unroll
    for (int i = 0; i < 8; ++i) b8[i] = b16[i];
    float16v_t c0, c1, c2, c3;
#pragma unroll
    for (int e = 0; e < 16; ++e) c0[e] = c1[e] = c2[e] = c3[e] = 0.f;
    for (int i = 0; i < iters; ++i) {
        if constexpr (SPARSE) {
            c0 = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b16, c0, 0x4444, 0, 0);
            c1 = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b16, c1, 0x4444, 0, 0);
            c2 = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b16, c2, 0x4444, 0, 0);
            c3 = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a, b16, c3, 0x4444, 0, 0);
        } else {
            c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b8, c0, 0, 0, 0);
            c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b8, c1, 0, 0, 0);
            c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b8, c2, 0, 0, 0);
            c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b8, c3, 0, 0, 0);
        }
    }
    float s = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) s += c0[e] + c1[e] + c2[e] + c3[e];
    if (s == 123.456f) *sink = s;
}

}  // namespace slim

using namespace slim;

extern "C" int slim_probe_read(const void *buf, size_t bytes, int32_t repeats, size_t stride, void *sink, void *stream)
{
    if (!buf || !sink) return SLIM_ERR_NULL;
    if (!aligned16(buf) || !aligned16(sink) || stride % 16) return SLIM_ERR_ALIGN;
    if (bytes < 65536 || repeats < 1) return SLIM_ERR_SHAPE;
    const size_t runs = bytes / 65536;
    const unsigned grid = (unsigned)(runs < 2048 ? runs : 2048);
    for (int r = 0; r < repeats; ++r)
        hipLaunchKernelGGL(probe_read_kernel, dim3(grid), dim3(512), 0, static_cast<hipStream_t>(stream),
                           reinterpret_cast<const uint4_t *>(static_cast<const char *>(buf) + (size_t)r * stride), bytes / 16,
                           static_cast<uint32_t *>(sink));
    return hip_status(hipGetLastError());
}

extern "C" int slim_probe_mfma(int32_t sparse, int32_t iters, int32_t workgroups, void *sink, double *flops, void *stream)
{
    if (!sink || !flops) return SLIM_ERR_NULL;
    if (iters < 1 || workgroups < 1 || workgroups > 65536) return SLIM_ERR_SHAPE;
    // per instruction: 32 x 32 outputs x 16 (dense) or 32 (sparse, counted as the dense product it stands for) inputs
    *flops = (double)workgroups * 4.0 * (double)iters * 4.0 * 2.0 * 32.0 * 32.0 * (sparse ? 32.0 : 16.0);
    if (sparse)
        hipLaunchKernelGGL(probe_mfma_kernel<true>, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters,
                           static_cast<float *>(sink));
    else
        hipLaunchKernelGGL(probe_mfma_kernel<false>, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), iters,
                           static_cast<float *>(sink));
    return hip_status(hipGetLastError());
}
