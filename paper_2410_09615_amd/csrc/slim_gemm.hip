// slim_linear_gemm and slim_lowrank: prefill-shaped forward on the matrix cores.
//
// One tiled kernel computes C[o][t] = sum_k A[o][k] B[t][k] for a 128 x 128
// tile of (output rows o) x (tokens t) per workgroup, in up to two phases that
// share the fp32 accumulators:
//   phase S  A = packed 2:4 int4 weights, expanded to dense fp16 tiles in LDS
//            (codes only; exact), B = X;
//   scale    accumulators times the fp32 row scale;
//   phase D  A = dense fp16 rows (L, or R for the T = X R^T product), B = fp16
//            (T, or X).
// so the adapter term rides on the same accumulators as extra k-steps and Y
// is rounded to fp16 once.
#include "slim_internal.h"

namespace slim {

constexpr int BO = 128;            // output rows per workgroup tile
constexpr int BT = 128;            // tokens per workgroup tile
constexpr int BK = 64;             // inputs per k-step
constexpr int LDS_LD = BK + 8;     // padded row length in halves (144 B: 16-byte aligned)
constexpr int kGemmThreads = 256;

enum OutMode { OUT_STORE = 0, OUT_ACCUM = 1, OUT_PARTIAL = 2 };

struct GemmArgs {
    int n_rows;            // extent of o
    int m;                 // extent of t
    // phase S (ks == 0: absent)
    const uint8_t *qvals;  // [n_rows][ks/4]
    const uint8_t *meta;   // [n_rows][ks/8]
    const float *scale;    // [n_rows]
    const half_t *Bs;      // [m][ks]
    int ks;
    // phase D (kd == 0: absent); grid.z splits its k range
    const half_t *Ad;      // [n_rows][kd]
    const half_t *Bd;      // [m][kd]
    int kd;
    // output: Y[t][o] fp16 (ld = n_rows) or P[z][t][o] fp32
    half_t *Y;
    float *P;
    int mode;
};

__device__ __forceinline__ uint16_t code_to_half_bits(int c)
{
    half_t h = (half_t)(float)c;
    return __builtin_bit_cast(uint16_t, h);
}

// 8 packed groups (8 code bytes, 8 position nibbles) -> 32 fp16, as 4 x 16 B.
__device__ __forceinline__ void expand8(uint2_t q, uint32_t me, uint4_t out[4])
{
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        uint32_t b = ((j < 4 ? q.x : q.y) >> (8 * (j & 3))) & 0xFFu;
        uint32_t nib = (me >> (4 * j)) & 0xFu;
        uint64_t h0 = code_to_half_bits(nibble_to_int(b & 0xFu));
        uint64_t h1 = code_to_half_bits(nibble_to_int(b >> 4));
        uint64_t v = (h0 << (16 * (nib & 3u))) | (h1 << (16 * (nib >> 2)));
        if (j & 1) {
            out[j >> 1].z = (uint32_t)v;
            out[j >> 1].w = (uint32_t)(v >> 32);
        } else {
            out[j >> 1].x = (uint32_t)v;
            out[j >> 1].y = (uint32_t)(v >> 32);
        }
    }
}

__global__ __launch_bounds__(kGemmThreads) void gemm_kernel(GemmArgs a)
{
    __shared__ __attribute__((aligned(16))) half_t As[BO * LDS_LD];
    __shared__ __attribute__((aligned(16))) half_t Bs[BT * LDS_LD];

    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int wo = wave & 1, wt = wave >> 1;
    const int o0 = blockIdx.x * BO;
    const int t0 = blockIdx.y * BT;

    // loader role: one tile row and one 32-input half of the k-step
    const int lrow = tid >> 1;
    const int lhalf = tid & 1;

    float16_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    uint4_t areg[4], breg[4];
    uint2_t qreg;
    uint32_t mreg;

    auto load_b = [&](const half_t *B, int ldb, int kbase, int kend) {
        const int t = t0 + lrow;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int kk = kbase + lhalf * 32 + c * 8;
            uint4_t v = {0u, 0u, 0u, 0u};
            if (t < a.m && kk < kend) v = *reinterpret_cast<const uint4_t *>(B + (size_t)t * ldb + kk);
            breg[c] = v;
        }
    };
    auto load_a_dense = [&](int kbase, int kend) {
        const int o = o0 + lrow;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int kk = kbase + lhalf * 32 + c * 8;
            uint4_t v = {0u, 0u, 0u, 0u};
            if (o < a.n_rows && kk < kend) v = *reinterpret_cast<const uint4_t *>(a.Ad + (size_t)o * a.kd + kk);
            areg[c] = v;
        }
    };
    auto load_a_packed = [&](int kbase) {
        const int o = o0 + lrow;
        qreg = uint2_t{0u, 0u};
        mreg = 0x44444444u;            // positions (0, 1) with zero codes
        if (o < a.n_rows) {
            const int g = (kbase + lhalf * 32) / 4;
            qreg = *reinterpret_cast<const uint2_t *>(a.qvals + (size_t)o * (a.ks / 4) + g);
            mreg = *reinterpret_cast<const uint32_t *>(a.meta + (size_t)o * (a.ks / 8) + g / 2);
        }
    };
    auto store_lds = [&]() {
        uint4_t *ad = reinterpret_cast<uint4_t *>(As + lrow * LDS_LD + lhalf * 32);
        uint4_t *bd = reinterpret_cast<uint4_t *>(Bs + lrow * LDS_LD + lhalf * 32);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            ad[c] = areg[c];
            bd[c] = breg[c];
        }
    };
    auto compute = [&]() {
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            half8_t af[2], bf[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                af[i] = *reinterpret_cast<const half8_t *>(As + (wo * 64 + i * 32 + (lane & 31)) * LDS_LD + ks * 16 +
                                                           8 * (lane >> 5));
                bf[i] = *reinterpret_cast<const half8_t *>(Bs + (wt * 64 + i * 32 + (lane & 31)) * LDS_LD + ks * 16 +
                                                           8 * (lane >> 5));
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    };

    // ---- phase S: packed weights against X ----
    if (a.ks > 0) {
        const int nk = a.ks / BK;
        load_a_packed(0);
        load_b(a.Bs, a.ks, 0, a.ks);
        for (int kt = 0; kt < nk; ++kt) {
            expand8(qreg, mreg, areg);
            __syncthreads();
            store_lds();
            __syncthreads();
            if (kt + 1 < nk) {
                load_a_packed((kt + 1) * BK);
                load_b(a.Bs, a.ks, (kt + 1) * BK, a.ks);
            }
            compute();
        }
        // row scale on the fp32 accumulators
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int blk = 0; blk < 4; ++blk)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int o = o0 + wo * 64 + i * 32 + 8 * blk + 4 * (lane >> 5) + e;
                    const float s = o < a.n_rows ? a.scale[o] : 0.0f;
#pragma unroll
                    for (int j = 0; j < 2; ++j) acc[i][j][4 * blk + e] *= s;
                }
    }

    // ---- phase D: dense fp16 rows ----
    if (a.kd > 0) {
        const int steps = (a.kd + BK - 1) / BK;
        const int per = (steps + gridDim.z - 1) / gridDim.z;
        const int kt0 = blockIdx.z * per;
        const int kt1 = min(steps, kt0 + per);
        if (kt0 < kt1) {
            load_a_dense(kt0 * BK, a.kd);
            load_b(a.Bd, a.kd, kt0 * BK, a.kd);
        }
        for (int kt = kt0; kt < kt1; ++kt) {
            __syncthreads();
            store_lds();
            __syncthreads();
            if (kt + 1 < kt1) {
                load_a_dense((kt + 1) * BK, a.kd);
                load_b(a.Bd, a.kd, (kt + 1) * BK, a.kd);
            }
            compute();
        }
    }

    // ---- output ----
    const bool vec_ok = (a.n_rows % 4) == 0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int t = t0 + wt * 64 + j * 32 + (lane & 31);
            if (t >= a.m) continue;
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
                const int o = o0 + wo * 64 + i * 32 + 8 * blk + 4 * (lane >> 5);
                if (o >= a.n_rows) continue;
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * blk + e];
                if (a.mode == OUT_PARTIAL) {
                    float *p = a.P + ((size_t)blockIdx.z * a.m + t) * a.n_rows + o;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (o + e < a.n_rows) p[e] = v[e];
                } else {
                    half_t *y = a.Y + (size_t)t * a.n_rows + o;
                    if (vec_ok) {
                        half4_t h;
                        if (a.mode == OUT_ACCUM) {
                            half4_t old = *reinterpret_cast<const half4_t *>(y);
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] += (float)old[e];
                        }
#pragma unroll
                        for (int e = 0; e < 4; ++e) h[e] = (half_t)v[e];
                        *reinterpret_cast<half4_t *>(y) = h;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (o + e < a.n_rows) {
                                float x = v[e];
                                if (a.mode == OUT_ACCUM) x += (float)y[e];
                                y[e] = (half_t)x;
                            }
                    }
                }
            }
        }
}

// T[i] = fp16(sum_z P[z][i])
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ P, int splits, size_t count,
                                                              half_t *__restrict__ T)
{
    for (size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x; i < count;
         i += (size_t)gridDim.x * blockDim.x) {
        float s = 0.0f;
        for (int z = 0; z < splits; ++z) s += P[(size_t)z * count + i];
        T[i] = (half_t)s;
    }
}

// Split-K factor for T = X R^T so that the launch has enough workgroups.
int gemm_t_splits(int32_t m, int32_t rank_pad, int32_t k)
{
    long tiles = (long)((rank_pad + BO - 1) / BO) * ((m + BT - 1) / BT);
    int s = 1;
    while (tiles * s < 192 && s < 8 && (k / BK) / (s * 2) >= 4) s *= 2;
    return s;
}

// T fp16 [m][rank_pad] = X R^T.
static void launch_t(const half_t *X, int m, const half_t *R, int k, int rank_pad, half_t *T, float *P, int splits,
                     hipStream_t st)
{
    GemmArgs g{};
    g.n_rows = rank_pad;
    g.m = m;
    g.Ad = R;
    g.Bd = X;
    g.kd = k;
    g.Y = T;
    g.P = P;
    g.mode = splits > 1 ? OUT_PARTIAL : OUT_STORE;
    dim3 grid((rank_pad + BO - 1) / BO, (m + BT - 1) / BT, splits);
    hipLaunchKernelGGL(gemm_kernel, grid, dim3(kGemmThreads), 0, st, g);
    if (splits > 1) {
        size_t count = (size_t)m * rank_pad;
        int blocks = (int)((count + 255) / 256 < 4096 ? (count + 255) / 256 : 4096);
        hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks), dim3(256), 0, st, P, splits, count, T);
    }
}

int launch_gemm_sparse(const uint8_t *qvals, const uint8_t *meta, const float *scale, const half_t *X, const half_t *L,
                       const half_t *T, half_t *Y, int n, int k, int rank_pad, int m,
                       hipStream_t st);   // slim_gemm_sparse.hip

int launch_lowrank_decode(const half_t *X, int m, const half_t *R, const half_t *L, int n, int k, int rank_pad,
                          half_t *Y, int accumulate, float *T, unsigned *counter, hipStream_t st);   // slim_gemv.hip

}  // namespace slim

using namespace slim;

extern "C" int slim_linear_gemm(const slim_layer *layer, const slim_half *X, int32_t m, slim_half *Y,
                                void *workspace, size_t workspace_bytes, void *stream)
{
    if (!layer || !X || !Y) return SLIM_ERR_NULL;
    const slim_shape s = layer->shape;
    if (!layer->qvals || !layer->meta || !layer->scale) return SLIM_ERR_NULL;
    if (s.rank > 0 && (!layer->L || !layer->R)) return SLIM_ERR_NULL;
    if (s.n < 1 || s.k < 128 || s.k % 128 || s.rank < 0 || m < 1) return SLIM_ERR_SHAPE;
    if (layer->rank_pad != slim_rank_pad(s.rank)) return SLIM_ERR_SHAPE;
    if (!aligned16(layer->qvals) || !aligned16(layer->meta) || !aligned16(layer->scale) || !aligned16(X) ||
        !aligned16(Y) || !aligned16(layer->L) || !aligned16(layer->R) || !aligned16(workspace))
        return SLIM_ERR_ALIGN;
    // 32-bit offsets into the weights and into L
    if ((uint64_t)s.n * (uint64_t)(s.k / 4) > 0xFFFFFFFFull || (uint64_t)s.n * (uint64_t)layer->rank_pad * 2 > 0xFFFFFFFFull)
        return SLIM_ERR_SHAPE;
    WorkspacePlan p = plan_workspace(s.n, s.k, layer->rank_pad, m);
    if (!workspace || workspace_bytes < p.total) return SLIM_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    half_t *T = reinterpret_cast<half_t *>(ws + p.t_off);
    float *P = reinterpret_cast<float *>(ws + p.part_off);
    const int rp = layer->rank_pad;
    const half_t *Xh = reinterpret_cast<const half_t *>(X);
    if (rp > 0) launch_t(Xh, m, reinterpret_cast<const half_t *>(layer->R), s.k, rp, T, P, p.splits, st);

    return launch_gemm_sparse(layer->qvals, layer->meta, layer->scale, Xh, reinterpret_cast<const half_t *>(layer->L),
                              T, reinterpret_cast<half_t *>(Y), s.n, s.k, rp, m, st);
}

extern "C" int slim_lowrank(const slim_half *X, int32_t m, const slim_half *R, const slim_half *L, slim_shape shape,
                            int32_t rank_pad, slim_half *Y, int accumulate, void *workspace,
                            size_t workspace_bytes, void *stream)
{
    if (!X || !R || !L || !Y) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 128 || shape.k % 128 || shape.rank < 1 || m < 1) return SLIM_ERR_SHAPE;
    if (rank_pad != slim_rank_pad(shape.rank)) return SLIM_ERR_SHAPE;
    if (!aligned16(X) || !aligned16(R) || !aligned16(L) || !aligned16(Y) || !aligned16(workspace))
        return SLIM_ERR_ALIGN;
    WorkspacePlan p = plan_workspace(shape.n, shape.k, rank_pad, m);
    if (!workspace || workspace_bytes < p.total) return SLIM_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    const half_t *Xh = reinterpret_cast<const half_t *>(X);
    const half_t *Rh = reinterpret_cast<const half_t *>(R);
    const half_t *Lh = reinterpret_cast<const half_t *>(L);
    half_t *Yh = reinterpret_cast<half_t *>(Y);
    if (m <= 16)
        return launch_lowrank_decode(Xh, m, Rh, Lh, shape.n, shape.k, rank_pad, Yh, accumulate,
                                     reinterpret_cast<float *>(ws + p.dec_off + 256),
                                     reinterpret_cast<unsigned *>(ws + p.dec_off), st);

    half_t *T = reinterpret_cast<half_t *>(ws + p.t_off);
    launch_t(Xh, m, Rh, shape.k, rank_pad, T, reinterpret_cast<float *>(ws + p.part_off), p.splits, st);
    GemmArgs g{};
    g.n_rows = shape.n;
    g.m = m;
    g.Ad = Lh;
    g.Bd = T;
    g.kd = rank_pad;
    g.Y = Yh;
    g.mode = accumulate ? OUT_ACCUM : OUT_STORE;
    dim3 grid((shape.n + BO - 1) / BO, (m + BT - 1) / BT, 1);
    hipLaunchKernelGGL(gemm_kernel, grid, dim3(kGemmThreads), 0, st, g);
    return hip_status(hipGetLastError());
}
