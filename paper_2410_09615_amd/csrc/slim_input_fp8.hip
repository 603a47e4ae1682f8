// 8-bit input quantization as the paper evaluates it (App. "Input Quantization"): AbsMax
// quantization of an input tensor to FP8 with one scale per tensor; the quantized values,
// back on the fp16 grid, are what the layer then sees.  E4M3 (largest value 448) unless the
// tensor's maximum exceeds that, then E5M2 (largest value 57344).
#include <hip/hip_runtime.h>

#include "slim_internal.h"

namespace slim {

constexpr int kInMaxBlocks = 256;

// partial maxima of |X|, one per workgroup (X as 16-byte pieces of 8 halves; `tail` halves after them)
__global__ __launch_bounds__(256) void input_absmax_kernel(const half_t *__restrict__ X, size_t count, float *part)
{
    __shared__ float red[4];
    const size_t n8 = count / 8;
    float a = 0.f;
    // four independent loads per lane and round: the grid is small (one partial per workgroup)
    const half8_t *X8 = reinterpret_cast<const half8_t *>(X);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    auto take = [&](const half8_t &v) {
#pragma unroll
        for (int e = 0; e < 8; ++e) a = fmaxf(a, fabsf((float)v[e]));
    };
    for (; i + 3 * stride < n8; i += 4 * stride) {
        const half8_t v0 = X8[i], v1 = X8[i + stride], v2 = X8[i + 2 * stride], v3 = X8[i + 3 * stride];
        take(v0);
        take(v1);
        take(v2);
        take(v3);
    }
    for (; i < n8; i += stride) take(X8[i]);
    if (blockIdx.x == 0)
        for (size_t t = n8 * 8 + threadIdx.x; t < count; t += blockDim.x) a = fmaxf(a, fabsf((float)X[t]));
    a = wave_max(a);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = a;
    __syncthreads();
    if (threadIdx.x == 0) part[blockIdx.x] = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// nearest value of the format (mantissa bits P, smallest normal exponent EMIN, largest value fmax) to |v|, ties to even
template <int P, int EMIN>
__device__ __forceinline__ float fp8_round_abs(float v, float fmax)
{
    const float a = fminf(fabsf(v), fmax);
    int e = (int)((__float_as_uint(a) >> 23) & 0xFFu) - 127;     // floor(log2 a) for a normal a; zero and tiny values fall below EMIN
    e = e > EMIN ? e : EMIN;
    const float q = __uint_as_float((uint32_t)(e - P + 127) << 23);      // spacing of the format at this magnitude
    const float qinv = __uint_as_float((uint32_t)(P - e + 127) << 23);   // 1 / q, a power of two as well: a * qinv = a / q exactly
    return fminf(rintf(a * qinv) * q, fmax);
}

// The 8-bit code of a value r >= 0 that lies on the format's grid (P mantissa bits, exponent bias BIAS,
// smallest normal exponent EMIN): exponent field and mantissa from r's binary32 bits; subnormals count
// in units of the format's smallest spacing.
template <int P, int EMIN, int BIAS>
__device__ __forceinline__ uint32_t fp8_bits_abs(float r)
{
    const uint32_t b = __float_as_uint(r);
    const int e = (int)((b >> 23) & 0xFFu) - 127;
    if (r == 0.f) return 0u;
    if (e < EMIN) return (uint32_t)(r * __uint_as_float((uint32_t)(P - EMIN + 127) << 23));      // r / 2^(EMIN - P), an integer below 2^P
    return ((uint32_t)(e + BIAS) << P) | ((b >> (23 - P)) & ((1u << P) - 1u));
}

__global__ __launch_bounds__(256) void input_fp8_kernel(const half_t *__restrict__ X, size_t count, const float *part, int nparts,
                                                        half_t *Xq, uint8_t *Xb, float *info)
{
    __shared__ float red[4];
    float a = (int)threadIdx.x < nparts ? part[threadIdx.x] : 0.f;
    a = wave_max(a);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = a;
    __syncthreads();
    const float M = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const bool e5 = M > 448.0f;
    const float fmax = e5 ? 57344.0f : 448.0f;
    const float s = M == 0.f ? 1.0f : M / fmax;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        info[0] = s;
        info[1] = e5 ? 1.0f : 0.0f;
    }
    // The sign is carried over as a bit: the product's conversion to half may be contracted into a
    // fused multiply-add with a +0 addend, which would turn a result of -0 into +0.
    // code: the 8-bit code of the same value (sign bit 7), for the kernels that take FP8 operands
    auto one = [&](half_t x, uint32_t &code) {
        const float v = (float)x / s;
        const float r = e5 ? fp8_round_abs<2, -14>(v, fmax) : fp8_round_abs<3, -6>(v, fmax);
        // product rounded to binary32, then to binary16 (two roundings, as defined): the empty asm hides the
        // product from the compiler, which would otherwise fuse the two into one mixed-precision
        // multiply-add that rounds once
        float prod = r * s;
        asm volatile("" : "+v"(prod));
        const half_t h = (half_t)prod;
        const uint16_t sign = (uint16_t)(__builtin_bit_cast(uint16_t, x) & 0x8000u);
        const uint16_t bits = (uint16_t)(__builtin_bit_cast(uint16_t, h) | sign);
        code = (e5 ? fp8_bits_abs<2, -14, 15>(r) : fp8_bits_abs<3, -6, 7>(r)) | (uint32_t)(sign >> 8);
        return __builtin_bit_cast(half_t, bits);
    };
    const size_t n8 = count / 8;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8; i += (size_t)gridDim.x * blockDim.x) {
        const half8_t v = reinterpret_cast<const half8_t *>(X)[i];
        half8_t o;
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            uint32_t c;
            o[e] = one(v[e], c);
            if (e < 4)
                lo |= c << (8 * e);
            else
                hi |= c << (8 * (e - 4));
        }
        if (Xq) reinterpret_cast<half8_t *>(Xq)[i] = o;
        if (Xb) reinterpret_cast<uint2_t *>(Xb)[i] = uint2_t{lo, hi};
    }
    if (blockIdx.x == 0)
        for (size_t i = n8 * 8 + threadIdx.x; i < count; i += blockDim.x) {
            uint32_t c;
            const half_t h = one(X[i], c);
            if (Xq) Xq[i] = h;
            if (Xb) Xb[i] = (uint8_t)c;
        }
}

}  // namespace slim

using namespace slim;

extern "C" int slim_input_quant_fp8_codes(const slim_half *X, size_t count, slim_half *Xq, uint8_t *Xb, float *info,
                                          void *workspace, size_t workspace_bytes, void *stream)
{
    if (!X || (!Xq && !Xb) || !info || !workspace) return SLIM_ERR_NULL;
    if (count < 1) return SLIM_ERR_SHAPE;
    if (!aligned16(X) || (Xq && !aligned16(Xq)) || !aligned16(workspace) || (Xb && !aligned16(Xb))) return SLIM_ERR_ALIGN;
    if (workspace_bytes < kInMaxBlocks * sizeof(float)) return SLIM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const size_t g = (count / 8 + 255) / 256;
    const unsigned grid_a = (unsigned)(g < 1 ? 1 : (g < kInMaxBlocks ? g : kInMaxBlocks));
    const unsigned grid_q = (unsigned)(g < 1 ? 1 : (g < 2048 ? g : 2048));
    float *part = static_cast<float *>(workspace);
    hipLaunchKernelGGL(input_absmax_kernel, dim3(grid_a), dim3(256), 0, st, reinterpret_cast<const half_t *>(X), count, part);
    hipLaunchKernelGGL(input_fp8_kernel, dim3(grid_q), dim3(256), 0, st, reinterpret_cast<const half_t *>(X), count,
                       (const float *)part, (int)grid_a, reinterpret_cast<half_t *>(Xq), Xb, info);
    return hip_status(hipGetLastError());
}

extern "C" int slim_input_quant_fp8(const slim_half *X, size_t count, slim_half *Xq, float *info, void *workspace,
                                    size_t workspace_bytes, void *stream)
{
    if (!Xq) return SLIM_ERR_NULL;
    return slim_input_quant_fp8_codes(X, count, Xq, nullptr, info, workspace, workspace_bytes, stream);
}
