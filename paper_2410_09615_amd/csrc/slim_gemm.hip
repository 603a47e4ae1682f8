// slim_linear_gemm and slim_lowrank: prefill-shaped forward on the matrix cores.
//
// The dense products of the path, C[t][o] (+)= sum_k A[o][k] B[t][k] with fp16
// operands and fp32 accumulation, all go through one kernel:
//   T = X R^T        (A = R, B = X; split along k when there are few tiles),
//   Y (+)= T L^T     (A = L, B = T; slim_lowrank with more than 16 tokens).
// The quantized term and its adapter continuation are in slim_gemm_sparse.hip.
#include "slim_mma.h"

namespace slim {

enum OutMode { OUT_STORE = 0, OUT_ACCUM = 1, OUT_PARTIAL = 2 };

struct DenseGemmArgs {
    const half_t *A;     // [rows][kt] in the tiled adapter layout, or (AQ) null and
    const uint8_t *Aq;   //   the 4-bit codes of A [aq_rows][kt] (4-bit adapter layout)
    const half_t *As;    //   with their group scales
    int aq_rows;
    const half_t *B;     // [m][kt] fp16, or (BF != 0) 8-bit codes, one byte per value
    const float *b_scale; // BF != 0: the scale of B's tensor (device memory); the result is multiplied by it
    int rows, m, kt;     // kt: row length of A and B (the full k extent)
    int ks;              // inputs per split (multiple of 128); grid.y splits
    half_t *Y;           // fp16 [m][rows]   (OUT_STORE, OUT_ACCUM)
    float *P;            // fp32 [splits][m][rows]   (OUT_PARTIAL)
    int mode;
    int tiles_o;         // row tiles of 128 AT
};

// Eight 8-bit codes (two dwords) -> eight fp16 values, exactly: E4M3 (BF 1) and E5M2 (BF 2) values all lie
// on the fp16 grid.
template <int BF>
__device__ __forceinline__ uint4_t fp8x8_to_half8(uint32_t lo, uint32_t hi)
{
    uint4_t out;
#pragma unroll
    for (int d = 0; d < 2; ++d) {
        const int src = (int)(d ? hi : lo);
        typedef float f2_t __attribute__((ext_vector_type(2)));
        const f2_t p0 = BF == 1 ? __builtin_amdgcn_cvt_pk_f32_fp8(src, false) : __builtin_amdgcn_cvt_pk_f32_bf8(src, false);
        const f2_t p1 = BF == 1 ? __builtin_amdgcn_cvt_pk_f32_fp8(src, true) : __builtin_amdgcn_cvt_pk_f32_bf8(src, true);
        out[2 * d] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p0[0], p0[1]));       // exact: nothing to round
        out[2 * d + 1] = __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_pkrtz(p1[0], p1[1]));
    }
    return out;
}

// Workgroup: 4 wavefronts, tile (128 AT) rows x 128 tokens, each wavefront
// (32 AT) rows x 128 tokens on fixed accumulators; the k-loop is dense_phase().
// BF: 0 = B in fp16; 1, 2 = B as E4M3 / E5M2 codes with one scale for the tensor (App. "Input
// Quantization"): half the bytes of B are requested, the codes become fp16 on their way into LDS,
// and the result is multiplied by the scale.
// AQ: A as 4-bit codes (Sec. 3.3), turned into fp16 in registers (dense_phase_q4()).
template <int AT, int BF = 0, bool AQ = false>
__global__ __launch_bounds__(256, 1) void gemm_dense_kernel(DenseGemmArgs a)
{
    constexpr int WROWS = 32 * AT;
    extern __shared__ __attribute__((aligned(16))) half_t lds[];   // two stage buffers
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int li = lane & 31;
    const int lb = lane >> 5;
    // the workgroups of a die (index mod 8) take neighbouring positions of the blocked order
    const int gx = (int)gridDim.x;
    const int q = gx % kDies == 0 ? ((int)blockIdx.x % kDies) * (gx / kDies) + (int)blockIdx.x / kDies : (int)blockIdx.x;
    const int w = blocked_tile(q, a.tiles_o, gx / a.tiles_o);
    const int o0 = (w % a.tiles_o) * (4 * WROWS) + wave * WROWS;
    const int t0 = (w / a.tiles_o) * 128;
    const int t_end = min(a.m, t0 + 128);
    const int k0 = blockIdx.y * a.ks;
    const int klen = max(0, min(a.ks, a.kt - k0));      // a split past the end adds zeros

    acc_reserve<AT>();
    static_for<16 * AT * NT>([&](auto r) { acc_write<r>(0.0f); });

    const uint32_t kt = (uint32_t)a.kt;
    const half_t *const lr = lds + li * SG_LD + 8 * lb;
    const rsrc_t da = make_rsrc(a.A, AQ ? 0u : (uint32_t)tl_bytes(a.rows, a.kt));
    const uint32_t av = tl_piece((uint32_t)o0 + li, (uint32_t)k0 / 8 + lb, kt);      // k0 is a multiple of 128
    const half_t *const lrq = lds + li * SG_LD + 32 * lb;
    Q4Rows aq{};
    if constexpr (AQ) aq = q4_rows_operand(a.Aq, a.As, a.aq_rows, a.kt, o0, li, lb, k0);
    float b_scale = 1.0f;
    if constexpr (BF == 0) {
        // 16 lanes per token row (256 contiguous bytes), 16 rows per pass
        const int srow = tid >> 4, scol = (tid & 15) * 8;
        half_t *const lw = lds + srow * SG_LD + scol;
        uint4_t xs[XR];
        auto stage_store = [&](int u, const uint4_t (&reg)[XR], int only = -1) {
#pragma unroll
            for (int p = 0; p < XR; ++p)
                if (only < 0 || only == p) *reinterpret_cast<uint4_t *>(lw + u * SG_STAGE + p * 16 * SG_LD) = reg[p];
        };
        const rsrc_t db = make_rsrc(a.B, (uint32_t)a.m * kt * 2u);
        const uint32_t bv = ((uint32_t)(t0 + srow) * kt + (uint32_t)k0 + (uint32_t)scol) * 2u;
        if constexpr (AQ)
            dense_phase_q4<AT>(aq, db, bv, 32u * kt, scol, klen, lrq, xs, stage_store);
        else
            dense_phase<AT>(da, av, (kt / 16) * 1024u, 1024u, db, bv, 32u * kt, klen, lr, xs, stage_store);
    } else {
        // 8 lanes per token row (128 contiguous bytes = 128 codes), 32 rows per pass; a load of 16 codes
        // becomes two pieces of 8 halves in LDS
        b_scale = *a.b_scale;
        const int srow = tid >> 3, scol = (tid & 7) * 16;
        half_t *const lw = lds + srow * SG_LD + scol;
        uint4_t xs[XR / 2];
        auto stage_store = [&](int u, const uint4_t (&reg)[XR / 2], int only = -1) {
#pragma unroll
            for (int p = 0; p < XR / 2; ++p) {
                if (only >= 0 && only != p) continue;
                half_t *d = lw + u * SG_STAGE + p * 32 * SG_LD;
                *reinterpret_cast<uint4_t *>(d) = fp8x8_to_half8<BF>(reg[p][0], reg[p][1]);
                *reinterpret_cast<uint4_t *>(d + 8) = fp8x8_to_half8<BF>(reg[p][2], reg[p][3]);
            }
        };
        const rsrc_t db = make_rsrc(a.B, (uint32_t)a.m * kt);
        const uint32_t bv = (uint32_t)(t0 + srow) * kt + (uint32_t)k0 + (uint32_t)scol;
        if constexpr (AQ)
            dense_phase_q4<AT, 1>(aq, db, bv, 32u * kt, scol, klen, lrq, xs, stage_store);
        else
            dense_phase<AT, 1>(da, av, (kt / 16) * 1024u, 1024u, db, bv, 32u * kt, klen, lr, xs, stage_store);
    }
    acc_settle();

    // lane holds token t0 + 32 it + li, rows o .. o + 3 per (i, blk)
    const bool vec_ok = (a.rows & 3) == 0;
    static_for<NT>([&](auto itc) {
        constexpr int it = itc;
        const int t = t0 + 32 * it + li;
        if (t >= t_end) return;
        static_for<AT>([&](auto ic) {
            constexpr int i = ic;
            static_for<4>([&](auto bc) {
                constexpr int blk = bc;
                const int o = o0 + 32 * i + 8 * blk + 4 * lb;
                if (o >= a.rows) return;
                float v[4];
                v[0] = acc_read<16 * (i * NT + it) + 4 * blk + 0>();
                v[1] = acc_read<16 * (i * NT + it) + 4 * blk + 1>();
                v[2] = acc_read<16 * (i * NT + it) + 4 * blk + 2>();
                v[3] = acc_read<16 * (i * NT + it) + 4 * blk + 3>();
                if constexpr (BF != 0) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) v[e] *= b_scale;
                }
                if (a.mode == OUT_PARTIAL) {
                    float *pp = a.P + ((size_t)blockIdx.y * a.m + t) * a.rows + o;
                    if (vec_ok) {
                        *reinterpret_cast<float4_t *>(pp) = float4_t{v[0], v[1], v[2], v[3]};
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (o + e < a.rows) pp[e] = v[e];
                    }
                } else {
                    half_t *y = a.Y + (size_t)t * a.rows + o;
                    if (vec_ok) {
                        if (a.mode == OUT_ACCUM) {
                            const half4_t old = *reinterpret_cast<const half4_t *>(y);
#pragma unroll
                            for (int e = 0; e < 4; ++e) v[e] += (float)old[e];
                        }
                        half4_t h;
#pragma unroll
                        for (int e = 0; e < 4; ++e) h[e] = (half_t)v[e];
                        *reinterpret_cast<half4_t *>(y) = h;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (o + e < a.rows) {
                                float x = v[e];
                                if (a.mode == OUT_ACCUM) x += (float)y[e];
                                y[e] = (half_t)x;
                            }
                    }
                }
            });
        });
    });
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

// One dense product on up to 2^32 - 1 bytes of B: C = A B^T over `splits` k ranges.
template <int AT, int BF = 0, bool AQ = false>
static void launch_dense(DenseGemmArgs a, int splits, hipStream_t st)
{
    a.tiles_o = (a.rows + 128 * AT - 1) / (128 * AT);
    const int tiles_t = (a.m + 127) / 128;
    const size_t lds = (size_t)2 * SG_STAGE * sizeof(half_t);
    hipLaunchKernelGGL((gemm_dense_kernel<AT, BF, AQ>), dim3((unsigned)(a.tiles_o * tiles_t), (unsigned)splits), dim3(256),
                       lds, st, a);
}

// Largest token count whose rows of `row_halves` halves stay below 4 GiB
// (buffer offsets are 32 bits wide), as a multiple of 128; 0 if even 128 do not.
static int token_chunk(int row_halves)
{
    return (int)((0xFFFFFFFFull / (2ull * (uint64_t)row_halves)) / 128 * 128);
}

// Split-K factor for T = X R^T so that the launch has enough workgroups: row
// tiles of 256 ranks x 128 tokens, k ranges of at least 512 inputs.
int gemm_t_splits(int32_t m, int32_t rank_pad, int32_t k)
{
    const long tiles = (long)((rank_pad + 255) / 256) * ((m + 127) / 128);
    int s = 1;
    while (tiles * s < 192 && s < 8 && k / (2 * s) >= 512) s *= 2;
    return s;
}

// T fp16 [m][rank_pad] = X R^T.  xf: 0 = X fp16; 1, 2 = X as E4M3 / E5M2 codes (one byte per value) with the
// tensor's scale at x_scale: T = scale * (value(X) R^T).
// R: fp16 [rank_pad][k] in the adapter layout, or null with Rq / Rs: the 4-bit codes and scales of R [rank][k].
static int launch_t(const half_t *X, int m, const half_t *R, int k, int rank_pad, half_t *T, float *P, int splits,
                    hipStream_t st, int xf = 0, const float *x_scale = nullptr, const uint8_t *Rq = nullptr,
                    const half_t *Rs = nullptr, int rank = 0)
{
    if ((uint64_t)rank_pad * (uint64_t)k * 2 > 0xFFFFFFFFull) return SLIM_ERR_SHAPE;
    const int chunk = token_chunk(k);
    if (chunk < 128) return SLIM_ERR_SHAPE;
    DenseGemmArgs g{};
    g.A = R;
    g.Aq = Rq;
    g.As = Rs;
    g.aq_rows = rank;
    g.rows = rank_pad;
    g.kt = k;
    g.ks = ((k / 128 + splits - 1) / splits) * 128;
    g.mode = splits > 1 ? OUT_PARTIAL : OUT_STORE;
    for (int t0 = 0; t0 < m; t0 += chunk) {
        g.m = m - t0 < chunk ? m - t0 : chunk;
        g.B = reinterpret_cast<const half_t *>(reinterpret_cast<const char *>(X) + (size_t)t0 * k * (xf ? 1 : 2));
        g.b_scale = x_scale;
        g.Y = T + (size_t)t0 * rank_pad;
        g.P = P;
        if (!R) {
            if (xf == 0)
                launch_dense<2, 0, true>(g, splits, st);
            else if (xf == 1)
                launch_dense<2, 1, true>(g, splits, st);
            else
                launch_dense<2, 2, true>(g, splits, st);
        } else if (xf == 0)
            launch_dense<2>(g, splits, st);
        else if (xf == 1)
            launch_dense<2, 1>(g, splits, st);
        else
            launch_dense<2, 2>(g, splits, st);
        if (splits > 1) {
            const size_t count = (size_t)g.m * rank_pad;
            const int blocks = (int)((count + 255) / 256 < 4096 ? (count + 255) / 256 : 4096);
            hipLaunchKernelGGL(reduce_partials_kernel, dim3(blocks), dim3(256), 0, st, P, splits, count, g.Y);
        }
    }
    return hip_status(hipGetLastError());
}

int launch_gemm_sparse(const uint8_t *qvals, const uint8_t *meta, const float *scale, const half_t *X, const half_t *L,
                       const half_t *T, half_t *Y, int n, int k, int rank_pad, int m, hipStream_t st, int xf,
                       const float *x_scale, const uint8_t *Lq, const half_t *Ls, int rank);   // slim_gemm_sparse.hip

int launch_lowrank_decode(const half_t *X, int m, const half_t *R, const half_t *L, int n, int k, int rank, int rank_pad,
                          half_t *Y, int accumulate, float *T, void *T16, unsigned *ctrl, hipStream_t st);   // slim_gemv.hip

}  // namespace slim

using namespace slim;

// X: fp16 [m][k] (xf = 0), or 8-bit codes [m][k] with x_info = {scale, format} in device memory (xf = 1: E4M3,
// 2: E5M2).
static int linear_gemm(const slim_layer *layer_in, const void *X, int xf, const float *x_info, int32_t m, slim_half *Y,
                       void *workspace, size_t workspace_bytes, void *stream)
{
    if (!layer_in || !X || !Y) return SLIM_ERR_NULL;
    if (xf != 0 && !x_info) return SLIM_ERR_NULL;
    if (xf < 0 || xf > 2) return SLIM_ERR_SHAPE;
    const slim_layer *layer = layer_in;
    const slim_shape s = layer->shape;
    if (!layer->qvals || !layer->meta || !layer->scale) return SLIM_ERR_NULL;
    const bool q4 = layer->adapter_bits == 4 && s.rank > 0;
    if (q4 && (!layer->Lq || !layer->Ls || !layer->Rq || !layer->Rs)) return SLIM_ERR_NULL;
    if (!q4 && s.rank > 0 && (!layer->L || !layer->R)) return SLIM_ERR_NULL;
    if (s.n < 1 || s.k < 128 || s.k % 128 || s.rank < 0 || m < 1) return SLIM_ERR_SHAPE;
    if (layer->rank_pad != slim_rank_pad(s.rank)) return SLIM_ERR_SHAPE;
    if (!aligned16(layer->qvals) || !aligned16(layer->meta) || !aligned16(layer->scale) || !aligned16(X) ||
        !aligned16(Y) || (!q4 && (!aligned16(layer->L) || !aligned16(layer->R))) || !aligned16(workspace))
        return SLIM_ERR_ALIGN;
    if (q4 && (!aligned16(layer->Lq) || !aligned16(layer->Ls) || !aligned16(layer->Rq) || !aligned16(layer->Rs)))
        return SLIM_ERR_ALIGN;
    // 32-bit offsets into the weights and into L
    if ((uint64_t)s.n * (uint64_t)(s.k / 4) > 0xFFFFFFFFull || (uint64_t)s.n * (uint64_t)layer->rank_pad * 2 > 0xFFFFFFFFull)
        return SLIM_ERR_SHAPE;
    WorkspacePlan p = plan_workspace(s.n, s.k, layer->rank_pad, m, q4);
    if (!workspace || workspace_bytes < p.total) return SLIM_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    // 4-bit adapters: both products read the codes themselves (dense_phase_q4())
    if (q4 && ((uint64_t)q4_code_bytes(s.n, s.rank) > 0xFFFFFFFFull || (uint64_t)q4_code_bytes(s.rank, s.k) > 0xFFFFFFFFull))
        return SLIM_ERR_SHAPE;
    half_t *T = reinterpret_cast<half_t *>(ws + p.t_off);
    float *P = reinterpret_cast<float *>(ws + p.part_off);
    const int rp = layer->rank_pad;
    const half_t *Xh = reinterpret_cast<const half_t *>(X);
    const half_t *Lh = q4 ? nullptr : reinterpret_cast<const half_t *>(layer->L);
    const half_t *Rh = q4 ? nullptr : reinterpret_cast<const half_t *>(layer->R);
    const half_t *Ls = reinterpret_cast<const half_t *>(layer->Ls), *Rs = reinterpret_cast<const half_t *>(layer->Rs);
    if (rp > 0) {
        const int rc = launch_t(Xh, m, Rh, s.k, rp, T, P, p.splits, st, xf, x_info, layer->Rq, Rs, s.rank);
        if (rc != SLIM_OK) return rc;
    }

    return launch_gemm_sparse(layer->qvals, layer->meta, layer->scale, Xh, Lh, T, reinterpret_cast<half_t *>(Y), s.n, s.k, rp,
                              m, st, xf, x_info, layer->Lq, Ls, s.rank);
}

extern "C" int slim_linear_gemm(const slim_layer *layer, const slim_half *X, int32_t m, slim_half *Y, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    return linear_gemm(layer, X, 0, nullptr, m, Y, workspace, workspace_bytes, stream);
}

extern "C" int slim_linear_gemm_fp8(const slim_layer *layer, const uint8_t *X8, const float *x_info, int32_t format, int32_t m,
                                    slim_half *Y, void *workspace, size_t workspace_bytes, void *stream)
{
    if (format != 0 && format != 1) return SLIM_ERR_SHAPE;
    return linear_gemm(layer, X8, 1 + format, x_info, m, Y, workspace, workspace_bytes, stream);
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
    WorkspacePlan p = plan_workspace(shape.n, shape.k, rank_pad, m, false);
    if (!workspace || workspace_bytes < p.total) return SLIM_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    const half_t *Xh = reinterpret_cast<const half_t *>(X);
    const half_t *Rh = reinterpret_cast<const half_t *>(R);
    const half_t *Lh = reinterpret_cast<const half_t *>(L);
    half_t *Yh = reinterpret_cast<half_t *>(Y);
    if (m <= 16) {
        // the decode kernels use 2^31 as "past the end of every buffer"
        if (tl_bytes(shape.n, rank_pad) >= 0x80000000ull || tl_bytes(rank_pad, shape.k) >= 0x80000000ull) return SLIM_ERR_SHAPE;
        return launch_lowrank_decode(Xh, m, Rh, Lh, shape.n, shape.k, shape.rank, rank_pad, Yh, accumulate,
                                     reinterpret_cast<float *>(ws + p.dec_off + 256), ws + p.t16_off,
                                     reinterpret_cast<unsigned *>(ws + p.dec_off), st);
    }

    if ((uint64_t)shape.n * (uint64_t)rank_pad * 2 > 0xFFFFFFFFull) return SLIM_ERR_SHAPE;
    half_t *T = reinterpret_cast<half_t *>(ws + p.t_off);
    const int rc = launch_t(Xh, m, Rh, shape.k, rank_pad, T, reinterpret_cast<float *>(ws + p.part_off), p.splits, st);
    if (rc != SLIM_OK) return rc;
    const int chunk = token_chunk(rank_pad);
    if (chunk < 128) return SLIM_ERR_SHAPE;
    DenseGemmArgs g{};
    g.A = Lh;
    g.rows = shape.n;
    g.kt = rank_pad;
    g.ks = (rank_pad + 127) / 128 * 128;
    g.mode = accumulate ? OUT_ACCUM : OUT_STORE;
    for (int t0 = 0; t0 < m; t0 += chunk) {
        g.m = m - t0 < chunk ? m - t0 : chunk;
        g.B = T + (size_t)t0 * rank_pad;
        g.Y = Yh + (size_t)t0 * shape.n;
        // the tallest row tile that still gives every compute unit a workgroup
        const long tt = (g.m + 127) / 128;
        const long cus = device_info().cus;
        if ((long)((shape.n + 511) / 512) * tt >= cus)
            launch_dense<4>(g, 1, st);
        else if ((long)((shape.n + 255) / 256) * tt >= cus)
            launch_dense<2>(g, 1, st);
        else
            launch_dense<1>(g, 1, st);
    }
    return hip_status(hipGetLastError());
}
