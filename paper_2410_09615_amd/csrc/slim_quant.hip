// slim_quant_search: the per-tensor scale of SLiM-Quant (Sec. 3.1, Eq. 4-7,
// Alg. 1): alpha* minimises E_quant(alpha) + E_clip(alpha), the squared error of
// the symmetric 4-bit quantizer with full scale alpha, integrated over the
// histogram of |W| (every element of a bin taken at the bin's centre).
//
//   histogram  B = max(512, min(n k / 1000, 20000)) uniform bins over [0, M],
//              M = max|W|; bin = min(B - 1, floor(|w| * (B / M))), quotient and
//              product in binary32 (so the counts are reproducible integers)
//   coarse     E at alpha = M i / 10, i = 1..10 (the last one is AbsMax)
//   fine       E at 21 samples of a tenth of that spacing around the best
//              coarse one (those inside (0, M])
//   alpha*     the first minimum over all of them; scale = alpha* / 7 (binary32)
//
// Three passes over memory in all: max, histogram (both read W once, HBM-bound),
// and the candidates, which only touch the histogram.  Everything stays on the
// device; the error sums are fp64.
#include "slim_internal.h"

namespace slim {

constexpr int kCoarse = 10;
constexpr int kFine = 21;
constexpr int kMaxBins = 20000;
constexpr int kMaxBlocks = 1024;        // workgroups of the maximum pass (one partial maximum each)

// workspace (32-bit words): [0] bits of M, [16 .. 77] errors (31 doubles from byte 64),
// [128 .. 128 + B) counts, then kMaxBlocks per-workgroup maxima
struct QuantWs {
    unsigned *mbits;
    double *err;
    unsigned *counts;
};
__host__ __device__ inline QuantWs quant_ws(void *ws)
{
    QuantWs q;
    q.mbits = static_cast<unsigned *>(ws);
    q.err = reinterpret_cast<double *>(static_cast<char *>(ws) + 64);
    q.counts = static_cast<unsigned *>(ws) + 128;
    return q;
}

__host__ __device__ inline int quant_bins(long numel)
{
    const long b = numel / 1000 < kMaxBins ? numel / 1000 : kMaxBins;
    return (int)(b > 512 ? b : 512);
}

// partial maxima of |W|, one per workgroup (no atomics: thousands of them on one
// address would serialize at memory)
__global__ __launch_bounds__(256) void quant_absmax_kernel(const float *__restrict__ W, size_t numel4, float *bmax,
                                                           unsigned *ws, int words)
{
    __shared__ float part[4];
    // the words the later kernels add into start at zero (this kernel runs before them)
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < words; i += gridDim.x * blockDim.x) ws[i] = 0u;
    float a = 0.f;
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < numel4; i += (size_t)gridDim.x * blockDim.x) {
        const float4 v = reinterpret_cast<const float4 *>(W)[i];
        a = fmaxf(a, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
    }
    a = wave_max(a);
    if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = a;
    __syncthreads();
    if (threadIdx.x == 0) bmax[blockIdx.x] = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
}

// per-workgroup histogram in LDS, then one global add per non-empty bin
__global__ __launch_bounds__(1024) void quant_hist_kernel(const float *__restrict__ W, size_t numel4, int B,
                                                          const float *bmax, int nblocks, unsigned *mbits, unsigned *counts)
{
    extern __shared__ unsigned hist[];
    __shared__ float part[16];
    for (int i = threadIdx.x; i < B; i += blockDim.x) hist[i] = 0u;
    // M from the partial maxima (every workgroup for itself; workgroup 0 publishes it)
    float a = (int)threadIdx.x < nblocks ? bmax[threadIdx.x] : 0.f;
    a = wave_max(a);
    if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = a;
    __syncthreads();
    float M = part[0];
    for (int w = 1; w < (int)blockDim.x / kWave; ++w) M = fmaxf(M, part[w]);
    if (blockIdx.x == 0 && threadIdx.x == 0) *mbits = __float_as_uint(M);
    if (M > 0.f) {
        const float inv = (float)B / M;
        auto put = [&](float w) {
            const int b = (int)floorf(fabsf(w) * inv);
            atomicAdd(&hist[b < B - 1 ? b : B - 1], 1u);
        };
        const float4 *W4 = reinterpret_cast<const float4 *>(W);
        const size_t stride = (size_t)gridDim.x * blockDim.x;
        size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
        for (; i + stride < numel4; i += 2 * stride) {       // two loads in flight per lane
            const float4 v = W4[i], u = W4[i + stride];
            put(v.x);
            put(v.y);
            put(v.z);
            put(v.w);
            put(u.x);
            put(u.y);
            put(u.z);
            put(u.w);
        }
        if (i < numel4) {
            const float4 v = W4[i];
            put(v.x);
            put(v.y);
            put(v.z);
            put(v.w);
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < B; i += blockDim.x)
        if (hist[i]) atomicAdd(&counts[i], hist[i]);
}

// E(alpha) over the histogram: one workgroup, fp64
__device__ __forceinline__ double quant_error_block(const unsigned *counts, int B, double M, double alpha, double *red)
{
    const double step = alpha / 7.0, width = M / B;
    double e = 0.0;
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        const double x = ((double)b + 0.5) * width;
        const double d = x <= alpha ? rint(x / step) * step - x : alpha - x;
        e += (double)counts[b] * (d * d);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) e += __shfl_xor(e, off, kWave);
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = e;
    __syncthreads();
    double t = 0.0;
    for (int w = 0; w < (int)blockDim.x / kWave; ++w) t += red[w];
    return t;
}

// candidates 0..9 coarse, 10..30 fine (the fine ones need the coarse errors: second launch)
__global__ __launch_bounds__(1024) void quant_eval_kernel(const unsigned *mbits, const unsigned *counts, int B, double *err,
                                                          int first)
{
    __shared__ double red[16];
    const int c = first + blockIdx.x;
    const double M = (double)__uint_as_float(*mbits);
    if (M == 0.0) return;
    const double eta = M / 10.0;
    double alpha;
    if (c < kCoarse) {
        alpha = eta * (c + 1);
    } else {
        int best = 0;
        for (int i = 1; i < kCoarse; ++i)
            if (err[i] < err[best]) best = i;
        alpha = eta * (best + 1) + eta * ((c - kCoarse - 10) / 10.0);
        if (!(alpha > 0.0 && alpha <= M)) {
            if (threadIdx.x == 0) err[c] = __builtin_inf();
            return;
        }
    }
    const double e = quant_error_block(counts, B, M, alpha, red);
    if (threadIdx.x == 0) err[c] = e;
}

// alpha* = first minimum; scale_out[o] = alpha* / 7 for every row
__global__ __launch_bounds__(256) void quant_pick_kernel(const unsigned *mbits, const double *err, float *scale_out, int n,
                                                         float *alpha_out)
{
    const double M = (double)__uint_as_float(*mbits);
    float alpha = 0.f, s = 1.f;
    if (M > 0.0) {
        const double eta = M / 10.0;
        int best = 0;
        for (int i = 1; i < kCoarse; ++i)
            if (err[i] < err[best]) best = i;
        const double lo = eta * (best + 1);
        int pick = best;
        for (int c = kCoarse; c < kCoarse + kFine; ++c)
            if (err[c] < err[pick]) pick = c;
        const double a = pick < kCoarse ? eta * (pick + 1) : lo + eta * ((pick - kCoarse - 10) / 10.0);
        alpha = (float)a;
        s = alpha / 7.0f;
    }
    for (int o = blockIdx.x * blockDim.x + threadIdx.x; o < n; o += gridDim.x * blockDim.x) scale_out[o] = s;
    if (alpha_out && blockIdx.x == 0 && threadIdx.x == 0) *alpha_out = alpha;
}

// ---- the same search with one scale per output row: one workgroup per row, everything in LDS ----
// (the histogram of a row has quant_bins(k) bins: 512 for every k below 513000)
__global__ __launch_bounds__(256) void quant_rows_kernel(const float *__restrict__ W, int n, int k, int B, float *scale_out,
                                                         float *alpha_out)
{
    extern __shared__ unsigned hist[];
    __shared__ double err[kCoarse + kFine];
    __shared__ double psum[(kCoarse + kFine) * 24];
    __shared__ float part[4];
    const int k4 = k / 4;
    for (int row = blockIdx.x; row < n; row += gridDim.x) {
        const float4 *w4 = reinterpret_cast<const float4 *>(W + (size_t)row * k);
        float a = 0.f;
        for (int i = threadIdx.x; i < k4; i += blockDim.x) {
            const float4 v = w4[i];
            a = fmaxf(a, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
        }
        a = wave_max(a);
        __syncthreads();                      // the previous row is done with hist, part and err
        if ((threadIdx.x & (kWave - 1)) == 0) part[threadIdx.x / kWave] = a;
        for (int i = threadIdx.x; i < B; i += blockDim.x) hist[i] = 0u;
        __syncthreads();
        const float Mf = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
        float alpha_f = 0.f, s = 1.f;
        if (Mf > 0.f) {
            const float inv = (float)B / Mf;
            auto put = [&](float w) {
                const int b = (int)floorf(fabsf(w) * inv);
                atomicAdd(&hist[b < B - 1 ? b : B - 1], 1u);
            };
            for (int i = threadIdx.x; i < k4; i += blockDim.x) {
                const float4 v = w4[i];
                put(v.x);
                put(v.y);
                put(v.z);
                put(v.w);
            }
            __syncthreads();
            const double M = (double)Mf, eta = M / 10.0;
            // all candidates of a stage at once: G lanes share a candidate, each takes every G-th bin
            auto eval = [&](int c, double alpha, bool ok, int j, int G) {
                double e = 0.0;
                if (ok) {
                    // rint(x / step) without the binary64 division wherever that cannot change the result:
                    // x * (1 / step) is within a few ulp of the quotient (at most 700), so the two round to the
                    // same integer unless the product lies within 1e-9 of a half; there the quotient decides.
                    // Empty bins add an exact zero and are skipped.
                    const double step = alpha / 7.0, width = M / B, inv_step = 1.0 / step;
                    for (int b = j; b < B; b += G) {
                        const unsigned cnt = hist[b];
                        if (cnt == 0u) continue;
                        const double x = ((double)b + 0.5) * width;
                        double d = alpha - x;
                        if (x <= alpha) {
                            const double q = x * inv_step;
                            double r = rint(q);
                            if (fabs(q - r) > 0.5 - 1e-9) r = rint(x / step);
                            d = r * step - x;
                        }
                        e += (double)cnt * (d * d);
                    }
                }
                // the G partial sums of a candidate are added up in lane order by its first lane
                if (c < kCoarse + kFine) psum[c * 24 + j] = e;
                __syncthreads();
                if (j == 0 && c < kCoarse + kFine) {
                    double t = 0.0;
                    for (int i = 0; i < G; ++i) t += psum[c * 24 + i];
                    err[c] = ok ? t : __builtin_inf();
                }
            };
            {
                const int c = threadIdx.x / 24;                     // 24 lanes per coarse candidate: 240 of 256 busy
                eval(c, eta * (c + 1), c < kCoarse, threadIdx.x - 24 * c, 24);
            }
            __syncthreads();
            int best = 0;
            for (int i = 1; i < kCoarse; ++i)
                if (err[i] < err[best]) best = i;
            const double lo = eta * (best + 1);
            {
                const int f = threadIdx.x / 12;                     // 12 lanes per fine candidate: 252 of 256 busy
                const double alpha = lo + eta * ((f - 10) / 10.0);
                eval(kCoarse + f, alpha, f < kFine && alpha > 0.0 && alpha <= M, threadIdx.x - 12 * f, 12);
            }
            __syncthreads();
            int pick = best;
            for (int c = kCoarse; c < kCoarse + kFine; ++c)
                if (err[c] < err[pick]) pick = c;
            const double al = pick < kCoarse ? eta * (pick + 1) : lo + eta * ((pick - kCoarse - 10) / 10.0);
            alpha_f = (float)al;
            s = alpha_f / 7.0f;
        }
        if (threadIdx.x == 0) {
            scale_out[row] = s;
            if (alpha_out) alpha_out[row] = alpha_f;
        }
    }
}

}  // namespace slim

using namespace slim;

extern "C" int slim_quant_workspace_bytes(slim_shape shape, size_t *bytes)
{
    if (!bytes) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 8 || shape.k % 8) return SLIM_ERR_SHAPE;
    *bytes = (size_t)(128 + quant_bins((long)shape.n * shape.k) + kMaxBlocks) * 4;
    return SLIM_OK;
}

extern "C" int slim_quant_search(const float *W, slim_shape shape, float *scale_out, float *alpha_out, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    if (!W || !scale_out || !workspace) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 8 || shape.k % 8) return SLIM_ERR_SHAPE;
    if (!aligned16(W) || !aligned16(workspace)) return SLIM_ERR_ALIGN;
    const size_t numel = (size_t)shape.n * shape.k;
    const int B = quant_bins((long)numel);
    if (workspace_bytes < (size_t)(128 + B + kMaxBlocks) * 4) return SLIM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const QuantWs q = quant_ws(workspace);
    const size_t numel4 = numel / 4;
    size_t g = (numel4 + 255) / 256;
    const unsigned grid_a = (unsigned)(g < (size_t)kMaxBlocks ? g : (size_t)kMaxBlocks);
    float *bmax = reinterpret_cast<float *>(q.counts + B);
    g = (numel4 + 1023) / 1024;
    // every workgroup ends with one global add per non-empty bin of its own histogram: few workgroups
    // (one per compute unit; half of that below 2^25 elements, where those adds outweigh the reading)
    const size_t hcap = numel < ((size_t)1 << 25) ? 128 : 256;
    const unsigned grid_h = (unsigned)(g < hcap ? g : hcap);
    hipLaunchKernelGGL(quant_absmax_kernel, dim3(grid_a), dim3(256), 0, st, W, numel4, bmax, q.mbits, 128 + B);
    hipLaunchKernelGGL(quant_hist_kernel, dim3(grid_h), dim3(1024), (size_t)B * 4, st, W, numel4, B, bmax, (int)grid_a, q.mbits,
                       q.counts);
    hipLaunchKernelGGL(quant_eval_kernel, dim3(kCoarse), dim3(1024), 0, st, q.mbits, q.counts, B, q.err, 0);
    hipLaunchKernelGGL(quant_eval_kernel, dim3(kFine), dim3(1024), 0, st, q.mbits, q.counts, B, q.err, kCoarse);
    hipLaunchKernelGGL(quant_pick_kernel, dim3((unsigned)((shape.n + 255) / 256)), dim3(256), 0, st, q.mbits, q.err,
                       scale_out, shape.n, alpha_out);
    return hip_status(hipGetLastError());
}

extern "C" int slim_quant_search_rows(const float *W, slim_shape shape, float *scale_out, float *alpha_out, void *stream)
{
    if (!W || !scale_out) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 8 || shape.k % 8) return SLIM_ERR_SHAPE;
    if (!aligned16(W)) return SLIM_ERR_ALIGN;
    const int B = quant_bins((long)shape.k);
    const unsigned grid = (unsigned)(shape.n < 4096 ? shape.n : 4096);
    hipLaunchKernelGGL(quant_rows_kernel, dim3(grid), dim3(256), (size_t)B * 4, static_cast<hipStream_t>(stream), W, shape.n,
                       shape.k, B, scale_out, alpha_out);
    return hip_status(hipGetLastError());
}
