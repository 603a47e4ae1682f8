// 4-bit adapters (Sec. 3.3, "Low-rank Adapter Quantization"): AbsMax group
// quantization of L and R, groups of 128 consecutive elements of a row, codes
// in [-8, 7], one fp16 scale per group.
//
//   scale  max|a| of the group / 7 as one binary32 division, rounded to binary16
//          (1 for a group of zeros; the smallest positive binary16 number if
//          the rounding gives zero);
//   code   round-half-even(a / scale) with the quotient in binary32, clamped.
//
// slim_pack_adapters_q4 quantizes and writes the device layout (slim_internal.h),
// slim_unpack_adapters_q4 inverts the layout (tests), and q4_to_tiled_fp16
// expands a quantized adapter into the fp16 adapter layout for the kernels that
// read fp16 (prefill; decode where the one-launch kernel does not apply).
#include "slim_internal.h"

namespace slim {

constexpr int kGroup = 128;

// One matrix to quantize: A fp16 [rows][K] row-major -> codes, scales in the device layout.
struct Q4PackJob {
    const half_t *A;
    int rows, K;
    uint8_t *codes;
    half_t *scales;
    unsigned blocks;                     // workgroups of this job
};

// One wavefront per (row, group): a lane owns two neighbouring columns = one byte.  Both adapters
// of a layer in one launch: the first j0.blocks workgroups work on j0, the others on j1.
__global__ __launch_bounds__(256) void adapter_q4_pack_kernel(Q4PackJob j0, Q4PackJob j1)
{
    const bool second = blockIdx.x >= j0.blocks;
    const half_t *A = second ? j1.A : j0.A;
    const int rows = second ? j1.rows : j0.rows, K = second ? j1.K : j0.K;
    uint8_t *codes = second ? j1.codes : j0.codes;
    half_t *scales = second ? j1.scales : j0.scales;
    const int lane = threadIdx.x & (kWave - 1);
    const int groups = (int)q4_groups(K);
    const long pair = (long)(blockIdx.x - (second ? j0.blocks : 0u)) * (blockDim.x / kWave) + threadIdx.x / kWave;
    const int row = (int)(pair / groups), g = (int)(pair % groups);
    if (row >= (int)q4_rows(rows)) return;
    const int col = g * kGroup + 2 * lane;
    float x0 = 0.f, x1 = 0.f;
    if (row < rows) {
        if (col < K) x0 = (float)A[(size_t)row * K + col];
        if (col + 1 < K) x1 = (float)A[(size_t)row * K + col + 1];
    }
    const float amax = wave_max(fmaxf(fabsf(x0), fabsf(x1)));
    const bool real = row < rows && g * kGroup < K;         // a group of the matrix (not padding)
    half_t s16 = (half_t)(amax / 7.0f);
    if (amax == 0.f) s16 = real ? (half_t)1.0f : (half_t)0.0f;
    else if ((float)s16 == 0.f) s16 = __builtin_bit_cast(half_t, (unsigned short)1);
    const float s = (float)s16;
    int c0 = 0, c1 = 0;
    if (amax != 0.f) {
        c0 = (int)fminf(fmaxf(__builtin_rintf(x0 / s), -8.f), 7.f);
        c1 = (int)fminf(fmaxf(__builtin_rintf(x1 / s), -8.f), 7.f);
    }
    const uint32_t c64 = (uint32_t)(2 * g + (lane >> 5));
    codes[q4_piece((uint32_t)row, c64, q4_ctiles(K)) + (lane & 31)] = (uint8_t)((c0 & 15) | ((c1 & 15) << 4));
    if (lane == 0) scales[(size_t)row * groups + g] = s16;
}

// codes int8 [rows][K] and scales fp16 [rows][ceil(K / 128)], row-major
__global__ __launch_bounds__(256) void adapter_q4_unpack_kernel(const uint8_t *codes, const half_t *scales, int rows,
                                                                 int K, int8_t *out_codes, half_t *out_scales)
{
    const long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= (long)rows * K) return;
    const int row = (int)(e / K), col = (int)(e % K);
    const uint8_t b = codes[q4_piece((uint32_t)row, (uint32_t)col / 64, q4_ctiles(K)) + (col % 64) / 2];
    out_codes[e] = (int8_t)nibble_to_int((col & 1) ? (b >> 4) : (b & 15u));
    if (col % kGroup == 0) out_scales[(size_t)row * ((K + kGroup - 1) / kGroup) + col / kGroup] =
        scales[(size_t)row * q4_groups(K) + col / kGroup];
}

// Expand into the fp16 adapter layout [rows_t][cols_t] (tiles of 32 x 16): a
// thread writes one piece of 8 columns.  value = fp16(code * scale), the same
// rounding as a half-precision multiply.
__global__ __launch_bounds__(256) void adapter_q4_expand_kernel(const uint8_t *codes, const half_t *scales, int rows,
                                                                 int K, int rows_t, int cols_t, half_t *out)
{
    const long e = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const int c8n = cols_t / 8;
    if (e >= (long)rows_t * c8n) return;
    const int row = (int)(e / c8n), c8 = (int)(e % c8n);
    half8_t v = {0, 0, 0, 0, 0, 0, 0, 0};
    if (row < rows && 8 * c8 < K) {
        const uint32_t q = *reinterpret_cast<const uint32_t *>(codes + q4_piece((uint32_t)row, (uint32_t)c8 / 8, q4_ctiles(K)) +
                                                               (c8 % 8) * 4);
        const half_t s = scales[(size_t)row * q4_groups(K) + (8 * c8) / kGroup];
        v = codes_to_half8(q) * s;
    }
    *reinterpret_cast<half8_t *>(reinterpret_cast<char *>(out) + tl_piece((uint32_t)row, (uint32_t)c8, (uint32_t)cols_t)) = v;
}

void launch_q4_expand(const uint8_t *codes, const half_t *scales, int rows, int K, int rows_t, int cols_t, half_t *out,
                      hipStream_t st)
{
    const long total = (long)rows_t * (cols_t / 8);
    hipLaunchKernelGGL(adapter_q4_expand_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, codes, scales, rows,
                       K, rows_t, cols_t, out);
}

}  // namespace slim

using namespace slim;

extern "C" int slim_adapter_q4_sizes(int32_t rows, int32_t cols, size_t *codes_bytes, size_t *scales_bytes)
{
    if (rows < 1 || cols < 1) return SLIM_ERR_SHAPE;
    if (codes_bytes) *codes_bytes = q4_code_bytes(rows, cols);
    if (scales_bytes) *scales_bytes = q4_scale_bytes(rows, cols);
    return SLIM_OK;
}

static Q4PackJob pack_job(const slim_half *A, int rows, int K, uint8_t *codes, slim_half *scales)
{
    const long pairs = (long)q4_rows(rows) * q4_groups(K);
    return Q4PackJob{reinterpret_cast<const half_t *>(A), rows, K, codes, reinterpret_cast<half_t *>(scales), (unsigned)((pairs + 3) / 4)};
}

extern "C" int slim_pack_adapters_q4(const slim_half *L, const slim_half *R, slim_shape shape, uint8_t *Lq,
                                     slim_half *Ls, uint8_t *Rq, slim_half *Rs, void *stream)
{
    if (!L || !R || !Lq || !Ls || !Rq || !Rs) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 128 || shape.k % 128 || shape.rank < 1) return SLIM_ERR_SHAPE;
    if (!aligned16(L) || !aligned16(R) || !aligned16(Lq) || !aligned16(Ls) || !aligned16(Rq) || !aligned16(Rs))
        return SLIM_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const Q4PackJob jl = pack_job(L, shape.n, shape.rank, Lq, Ls), jr = pack_job(R, shape.rank, shape.k, Rq, Rs);
    hipLaunchKernelGGL(adapter_q4_pack_kernel, dim3(jl.blocks + jr.blocks), dim3(256), 0, st, jl, jr);
    return hip_status(hipGetLastError());
}

extern "C" int slim_unpack_adapters_q4(const uint8_t *codes, const slim_half *scales, int32_t rows, int32_t cols,
                                       int8_t *out_codes, slim_half *out_scales, void *stream)
{
    if (!codes || !scales || !out_codes || !out_scales) return SLIM_ERR_NULL;
    if (rows < 1 || cols < 1) return SLIM_ERR_SHAPE;
    const long total = (long)rows * cols;
    hipLaunchKernelGGL(adapter_q4_unpack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), codes, reinterpret_cast<const half_t *>(scales), rows, cols,
                       out_codes, reinterpret_cast<half_t *>(out_scales));
    return hip_status(hipGetLastError());
}
