// slim_linear_gemv: decode-shaped forward (1 <= m <= 16 tokens).
//
// Two launches.  Kernel 1 treats the adapter factor R as `rank_pad` more
// output rows of the same X: one wavefront per row streams either a packed
// weight row (codes + positions, dequantized in registers) or a fp16 row of R,
// reduces its partial sums across the 64 lanes and writes the scaled
// quantized term acc[m][o] or T[m][j] = (X R^T)[m][j] in fp32.  Kernel 2
// streams L and writes Y[m][o] = fp16(acc[m][o] + sum_j T[m][j] L[o][j]).
#include "slim_internal.h"

namespace slim {

constexpr int kMaxTokens = 16;
constexpr int kGemvThreads = 256;
constexpr int kGemvWaves = kGemvThreads / kWave;

__global__ __launch_bounds__(kGemvThreads) void gemv_rows_kernel(
    const uint8_t *__restrict__ qvals, const uint8_t *__restrict__ meta, const float *__restrict__ scale,
    const half_t *__restrict__ R, const half_t *__restrict__ X, int n, int k, int rank_pad, int m,
    float *__restrict__ acc_out, float *__restrict__ T_out)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = blockIdx.x * kGemvWaves + threadIdx.x / kWave;
    const int nwaves = gridDim.x * kGemvWaves;
    const int rows = n + rank_pad;
    for (int row = wave; row < rows; row += nwaves) {
        float acc[kMaxTokens];
#pragma unroll
        for (int t = 0; t < kMaxTokens; ++t) acc[t] = 0.0f;
        if (row < n) {
            const uint8_t *qrow = qvals + (size_t)row * (k / 4);
            const uint8_t *mrow = meta + (size_t)row * (k / 8);
            // a lane takes 8 groups (32 inputs) per step
            for (int g0 = lane * 8; g0 < k / 4; g0 += kWave * 8) {
                uint2_t q = *reinterpret_cast<const uint2_t *>(qrow + g0);
                uint32_t me = *reinterpret_cast<const uint32_t *>(mrow + g0 / 2);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    uint32_t b = ((j < 4 ? q.x : q.y) >> (8 * (j & 3))) & 0xFFu;
                    uint32_t nib = (me >> (4 * j)) & 0xFu;
                    float c0 = (float)nibble_to_int(b & 0xFu);
                    float c1 = (float)nibble_to_int(b >> 4);
                    int k0 = 4 * (g0 + j) + (int)(nib & 3u);
                    int k1 = 4 * (g0 + j) + (int)(nib >> 2);
#pragma unroll
                    for (int t = 0; t < kMaxTokens; ++t)
                        if (t < m) {
                            acc[t] = fmaf(c0, (float)X[(size_t)t * k + k0], acc[t]);
                            acc[t] = fmaf(c1, (float)X[(size_t)t * k + k1], acc[t]);
                        }
                }
            }
            const float s = scale[row];
#pragma unroll
            for (int t = 0; t < kMaxTokens; ++t)
                if (t < m) {
                    float v = wave_sum(acc[t]);
                    if (lane == 0) acc_out[(size_t)t * n + row] = s * v;
                }
        } else {
            const int j = row - n;
            const half_t *rrow = R + (size_t)j * k;
            for (int c0 = lane * 8; c0 < k; c0 += kWave * 8) {
                half8_t rv = *reinterpret_cast<const half8_t *>(rrow + c0);
#pragma unroll
                for (int t = 0; t < kMaxTokens; ++t)
                    if (t < m) {
                        half8_t xv = *reinterpret_cast<const half8_t *>(X + (size_t)t * k + c0);
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[t] = fmaf((float)rv[e], (float)xv[e], acc[t]);
                    }
            }
#pragma unroll
            for (int t = 0; t < kMaxTokens; ++t)
                if (t < m) {
                    float v = wave_sum(acc[t]);
                    if (lane == 0) T_out[(size_t)t * rank_pad + j] = v;
                }
        }
    }
}

// Y[t][o] = fp16(base[t][o] + sum_j T[t][j] L[o][j]); base == nullptr reads 0,
// accumulate != 0 adds the fp16 value already in Y.
__global__ __launch_bounds__(kGemvThreads) void gemv_adapter_out_kernel(
    const float *__restrict__ base, const float *__restrict__ T, const half_t *__restrict__ L, int n,
    int rank_pad, int m, int accumulate, half_t *__restrict__ Y)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = blockIdx.x * kGemvWaves + threadIdx.x / kWave;
    const int nwaves = gridDim.x * kGemvWaves;
    for (int o = wave; o < n; o += nwaves) {
        float acc[kMaxTokens];
#pragma unroll
        for (int t = 0; t < kMaxTokens; ++t) acc[t] = 0.0f;
        const half_t *lrow = L + (size_t)o * rank_pad;
        for (int j0 = lane * 8; j0 < rank_pad; j0 += kWave * 8) {
            half8_t lv = *reinterpret_cast<const half8_t *>(lrow + j0);
#pragma unroll
            for (int t = 0; t < kMaxTokens; ++t)
                if (t < m) {
                    const float *tp = T + (size_t)t * rank_pad + j0;
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[t] = fmaf((float)lv[e], tp[e], acc[t]);
                }
        }
#pragma unroll
        for (int t = 0; t < kMaxTokens; ++t)
            if (t < m) {
                float v = wave_sum(acc[t]);
                if (lane == 0) {
                    if (base) v += base[(size_t)t * n + o];
                    if (accumulate) v += (float)Y[(size_t)t * n + o];
                    Y[(size_t)t * n + o] = (half_t)v;
                }
            }
    }
}

// Y[t][o] = fp16(base[t][o]) for a layer without adapters.
__global__ __launch_bounds__(256) void gemv_store_kernel(const float *__restrict__ base, size_t total,
                                                         half_t *__restrict__ Y)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x)
        Y[i] = (half_t)base[i];
}

static int wave_grid(int rows)
{
    int blocks = (rows + kGemvWaves - 1) / kGemvWaves;
    const int cap = 256 * 8;
    return blocks < cap ? (blocks < 1 ? 1 : blocks) : cap;
}

int launch_lowrank_decode(const half_t *X, int m, const half_t *R, const half_t *L, int n, int k, int rank_pad,
                          half_t *Y, int accumulate, float *T, hipStream_t st)
{
    hipLaunchKernelGGL(gemv_rows_kernel, dim3(wave_grid(rank_pad)), dim3(kGemvThreads), 0, st, nullptr, nullptr,
                       nullptr, R, X, 0, k, rank_pad, m, nullptr, T);
    hipLaunchKernelGGL(gemv_adapter_out_kernel, dim3(wave_grid(n)), dim3(kGemvThreads), 0, st, nullptr, T, L, n,
                       rank_pad, m, accumulate, Y);
    return hip_status(hipGetLastError());
}

}  // namespace slim

using namespace slim;

extern "C" int slim_linear_gemv(const slim_layer *layer, const slim_half *X, int32_t m, slim_half *Y,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    if (!layer || !X || !Y) return SLIM_ERR_NULL;
    const slim_shape s = layer->shape;
    if (!layer->qvals || !layer->meta || !layer->scale) return SLIM_ERR_NULL;
    if (s.rank > 0 && (!layer->L || !layer->R)) return SLIM_ERR_NULL;
    if (s.n < 1 || s.k < 128 || s.k % 128 || s.rank < 0 || m < 1 || m > kMaxTokens) return SLIM_ERR_SHAPE;
    if (layer->rank_pad != slim_rank_pad(s.rank)) return SLIM_ERR_SHAPE;
    if (!aligned16(layer->qvals) || !aligned16(layer->meta) || !aligned16(layer->scale) || !aligned16(X) ||
        !aligned16(Y) || !aligned16(layer->L) || !aligned16(layer->R) || !aligned16(workspace))
        return SLIM_ERR_ALIGN;
    WorkspacePlan p = plan_workspace(s.n, s.k, layer->rank_pad, m);
    if (!workspace || workspace_bytes < p.total) return SLIM_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *T = reinterpret_cast<float *>(ws + p.t_off);
    float *acc = reinterpret_cast<float *>(ws + p.acc_off);
    const int rp = layer->rank_pad;
    hipLaunchKernelGGL(gemv_rows_kernel, dim3(wave_grid(s.n + rp)), dim3(kGemvThreads), 0, st, layer->qvals,
                       layer->meta, layer->scale, reinterpret_cast<const half_t *>(layer->R),
                       reinterpret_cast<const half_t *>(X), s.n, s.k, rp, m, acc, T);
    if (rp > 0)
        hipLaunchKernelGGL(gemv_adapter_out_kernel, dim3(wave_grid(s.n)), dim3(kGemvThreads), 0, st, acc, T,
                           reinterpret_cast<const half_t *>(layer->L), s.n, rp, m, 0,
                           reinterpret_cast<half_t *>(Y));
    else
        hipLaunchKernelGGL(gemv_store_kernel, dim3(wave_grid(s.n)), dim3(256), 0, st, acc, (size_t)m * s.n,
                           reinterpret_cast<half_t *>(Y));
    return hip_status(hipGetLastError());
}
