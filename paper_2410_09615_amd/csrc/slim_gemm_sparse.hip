// Prefill main kernel: Y = scale * (X Wc^T) + T L^T on the matrix cores, with
// the 2:4 weights as the sparse A operand of V_SMFMAC_F32_32X32X32_F16.
//
// Workgroup tile: 256 output rows x 128 tokens, 4 wavefronts, each 64 rows x
// 128 tokens (2 x 4 accumulator tiles of 32 x 32, 128 VGPRs).
//   A (weights): never touches LDS.  Per 128 inputs a lane loads 16 bytes of
//     codes and 8 bytes of positions of its row straight from global memory
//     (two stages ahead), turns 4 code bytes into 8 fp16 values in registers, and passes the 16
//     position bits of those 4 groups as the index operand (the canonical
//     metadata is that operand's format).  Each wavefront converts only its
//     own rows, once, and uses them against all 128 tokens.
//   B (X): 128 tokens x 128 inputs per stage, double-buffered in LDS.
//   Then the accumulators are multiplied by the row scale and the adapter
//   term continues on them with the dense instruction: A = L rows from global
//   memory, B = T (fp16, from the workspace) staged through the same LDS
//   buffers.  One rounding to fp16 at the store.
#include "slim_internal.h"

namespace slim {

constexpr int SG_BO = 256;              // output rows per workgroup
constexpr int SG_BT = 128;              // tokens per workgroup
constexpr int SG_BK = 128;              // inputs per stage
constexpr int SG_LD = SG_BK + 8;        // LDS row length in halves (272 B)
constexpr int SG_THREADS = 256;
constexpr int SG_STAGE = SG_BT * SG_LD; // halves per LDS buffer

struct SparseGemmArgs {
    const uint8_t *qvals;
    const uint8_t *meta;
    const float *scale;
    const half_t *X;     // [m][k]
    const half_t *L;     // [n][rank_pad]
    const half_t *T;     // [m][rank_pad] fp16
    half_t *Y;           // [m][n]
    int n, k, rank_pad, m;
    int tiles_o;         // row tiles
    int tiles_total;     // row tiles x token tiles
    int n_full;          // workgroups [0, n_full) take whole tiles, the rest half tiles (64 tokens)
};

// Copy a [128 tokens][128 inputs] piece of a row-major fp16 matrix (leading
// dimension ld, valid extent rows x cols) into registers: lane -> 16 lanes per
// row (256 contiguous bytes), 16 rows per step, 8 steps.
__device__ __forceinline__ void stage_load(const half_t *src, int ld, int rows, int cols, int row0, int col0,
                                           uint4_t (&reg)[8])
{
    const int tid = threadIdx.x;
    const int c = col0 + (tid & 15) * 8;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int r = row0 + s * 16 + (tid >> 4);
        uint4_t v = {0u, 0u, 0u, 0u};
        if (r < rows && c < cols) v = *reinterpret_cast<const uint4_t *>(src + (size_t)r * ld + c);
        reg[s] = v;
    }
}

__device__ __forceinline__ void stage_store(half_t *buf, const uint4_t (&reg)[8])
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int s = 0; s < 8; ++s)
        *reinterpret_cast<uint4_t *>(buf + (s * 16 + (tid >> 4)) * SG_LD + (tid & 15) * 8) = reg[s];
}

__global__ __launch_bounds__(SG_THREADS, 2) void gemm_sparse_kernel(SparseGemmArgs a)
{
    extern __shared__ __attribute__((aligned(16))) half_t lds[];   // two stage buffers
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int li = lane & 31;            // A row / B token within a 32-tile
    const int lb = lane >> 5;            // k-block of the lane
    // Whole tiles first; the tiles that would make up a last, partly filled round
    // of workgroups are cut in two along the tokens, so that round is short.
    const int b = blockIdx.x;
    const bool half_tile = b >= a.n_full;
    const int w = half_tile ? a.n_full + (b - a.n_full) / 2 : b;
    const int nt = half_tile ? 2 : 4;                        // 32-token accumulator tiles in use
    const int o0 = (w % a.tiles_o) * SG_BO + wave * 64;
    const int t0 = (w / a.tiles_o) * SG_BT + (half_tile ? 64 * ((b - a.n_full) & 1) : 0);
    const int t_end = min(a.m, t0 + 32 * nt);                // tokens of this workgroup: [t0, t_end)

    float16_t acc[2][4];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;

    // this lane's two weight rows (clamped: rows past n are computed and dropped)
    const int orow0 = min(o0 + li, a.n - 1);
    const int orow1 = min(o0 + 32 + li, a.n - 1);
    // 32-bit byte offsets from the (uniform) base pointers keep address registers few
    const uint32_t q0o = (uint32_t)orow0 * (uint32_t)(a.k / 4) + 16u * lb;
    const uint32_t q1o = (uint32_t)orow1 * (uint32_t)(a.k / 4) + 16u * lb;
    const uint32_t m0o = (uint32_t)orow0 * (uint32_t)(a.k / 8) + 8u * lb;
    const uint32_t m1o = (uint32_t)orow1 * (uint32_t)(a.k / 8) + 8u * lb;

    uint4_t xreg[8];
    const int nsteps = a.k / SG_BK;

    // weights of stages s, s+1, s+2: loaded two stages ahead into three rotating
    // register slots (the main loop is unrolled by 6 so that the slots are static)
    uint4_t qa[3][2];
    uint2_t ma[3][2];
    auto load_a = [&](int s, uint4_t (&q)[2], uint2_t (&mm)[2]) {
        const int sc = min(s, nsteps - 1);                           // past the end: a harmless reload
        q[0] = *reinterpret_cast<const uint4_t *>(a.qvals + (q0o + (uint32_t)sc * (SG_BK / 4)));
        q[1] = *reinterpret_cast<const uint4_t *>(a.qvals + (q1o + (uint32_t)sc * (SG_BK / 4)));
        mm[0] = *reinterpret_cast<const uint2_t *>(a.meta + (m0o + (uint32_t)sc * (SG_BK / 8)));
        mm[1] = *reinterpret_cast<const uint2_t *>(a.meta + (m1o + (uint32_t)sc * (SG_BK / 8)));
    };

    // prologue: stage 0
    stage_load(a.X, a.k, t_end, a.k, t0, 0, xreg);
    load_a(0, qa[0], ma[0]);
    load_a(1, qa[1], ma[1]);
    stage_store(lds, xreg);
    __syncthreads();

    // B fragment address of this lane inside a stage buffer: token li of tile
    // it, inputs 16 t + 8 lb (values 0-7) and 64 + 16 t + 8 lb (values 8-15)
    const int boff = li * SG_LD + 8 * lb;

    for (int s0 = 0; s0 < nsteps; s0 += 6) {
#pragma unroll
      for (int u = 0; u < 6; ++u) {
        const int s = s0 + u;
        if (s >= nsteps) break;
        const half_t *buf = lds + (u & 1) * SG_STAGE;               // stage s sits in buffer s & 1 (6 is even)
        if (s + 1 < nsteps) stage_load(a.X, a.k, t_end, a.k, t0, (s + 1) * SG_BK, xreg);
        load_a(s + 2, qa[(u + 2) % 3], ma[(u + 2) % 3]);
        const uint4_t (&qc)[2] = qa[u % 3];
        const uint2_t (&mc)[2] = ma[u % 3];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const half8_t a0 = codes_to_half8(qc[0][t]);
            const half8_t a1 = codes_to_half8(qc[1][t]);
            const int idx0 = (int)mc[0][t >> 1];
            const int idx1 = (int)mc[1][t >> 1];
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                if (it >= nt) break;
                const half_t *bp = buf + it * 32 * SG_LD + boff + 16 * t;
                const half8_t b1 = *reinterpret_cast<const half8_t *>(bp);
                const half8_t b2 = *reinterpret_cast<const half8_t *>(bp + 64);
                const half16_t bv =
                    __builtin_shufflevector(b1, b2, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
                if (t & 1) {
                    acc[0][it] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a0, bv, acc[0][it], idx0, 0, 1);
                    acc[1][it] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a1, bv, acc[1][it], idx1, 0, 1);
                } else {
                    acc[0][it] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a0, bv, acc[0][it], idx0, 0, 0);
                    acc[1][it] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(a1, bv, acc[1][it], idx1, 0, 0);
                }
            }
        }
        if (s + 1 < nsteps) stage_store(lds + ((u + 1) & 1) * SG_STAGE, xreg);
        __syncthreads();
      }
    }

    // row scale: accumulator element 4 blk + e of tile io is row 32 io + 8 blk + 4 lb + e
#pragma unroll
    for (int io = 0; io < 2; ++io)
#pragma unroll
        for (int blk = 0; blk < 4; ++blk)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int o = o0 + 32 * io + 8 * blk + 4 * lb + e;
                const float sc = o < a.n ? a.scale[o] : 0.0f;
#pragma unroll
                for (int it = 0; it < 4; ++it) acc[io][it][4 * blk + e] *= sc;
            }

    // adapter term: dense steps of 16 ranks; T staged like X, L rows from global
    if (a.rank_pad > 0) {
        const int rp = a.rank_pad;
        const half_t *l0p = a.L + (size_t)orow0 * rp + 8 * lb;
        const half_t *l1p = a.L + (size_t)orow1 * rp + 8 * lb;
        const int rstages = (rp + SG_BK - 1) / SG_BK;
        stage_load(a.T, rp, t_end, rp, t0, 0, xreg);
        stage_store(lds, xreg);
        __syncthreads();
        const int boff2 = li * SG_LD + 8 * lb;
        for (int s = 0; s < rstages; ++s) {
            const half_t *buf = lds + (s & 1) * SG_STAGE;
            if (s + 1 < rstages) stage_load(a.T, rp, t_end, rp, t0, (s + 1) * SG_BK, xreg);
            const int jn = min(SG_BK, rp - s * SG_BK) / 16;      // dense steps in this stage
            uint4_t la[2], ln[2];
            la[0] = *reinterpret_cast<const uint4_t *>(l0p + s * SG_BK);
            la[1] = *reinterpret_cast<const uint4_t *>(l1p + s * SG_BK);
            for (int j = 0; j < jn; ++j) {
                if (j + 1 < jn) {
                    ln[0] = *reinterpret_cast<const uint4_t *>(l0p + s * SG_BK + 16 * (j + 1));
                    ln[1] = *reinterpret_cast<const uint4_t *>(l1p + s * SG_BK + 16 * (j + 1));
                }
                const half8_t a0 = __builtin_bit_cast(half8_t, la[0]);
                const half8_t a1 = __builtin_bit_cast(half8_t, la[1]);
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    if (it >= nt) break;
                    const half8_t bv = *reinterpret_cast<const half8_t *>(buf + it * 32 * SG_LD + boff2 + 16 * j);
                    acc[0][it] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a0, bv, acc[0][it], 0, 0, 0);
                    acc[1][it] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a1, bv, acc[1][it], 0, 0, 0);
                }
                la[0] = ln[0];
                la[1] = ln[1];
            }
            if (s + 1 < rstages) stage_store(lds + ((s + 1) & 1) * SG_STAGE, xreg);
            __syncthreads();
        }
    }

    // store: lane holds token t0 + 32 it + li, rows o .. o + 3 per (io, blk)
    const bool vec_ok = (a.n & 3) == 0;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int t = t0 + 32 * it + li;
        if (t >= t_end) continue;
#pragma unroll
        for (int io = 0; io < 2; ++io)
#pragma unroll
            for (int blk = 0; blk < 4; ++blk) {
                const int o = o0 + 32 * io + 8 * blk + 4 * lb;
                if (o >= a.n) continue;
                half_t *y = a.Y + (size_t)t * a.n + o;
                if (vec_ok) {
                    half4_t h;
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = (half_t)acc[io][it][4 * blk + e];
                    *reinterpret_cast<half4_t *>(y) = h;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (o + e < a.n) y[e] = (half_t)acc[io][it][4 * blk + e];
                }
            }
    }
}

int launch_gemm_sparse(const uint8_t *qvals, const uint8_t *meta, const float *scale, const half_t *X, const half_t *L,
                       const half_t *T, half_t *Y, int n, int k, int rank_pad, int m, hipStream_t st)
{
    SparseGemmArgs a{};
    a.qvals = qvals;
    a.meta = meta;
    a.scale = scale;
    a.X = X;
    a.L = L;
    a.T = T;
    a.Y = Y;
    a.n = n;
    a.k = k;
    a.rank_pad = rank_pad;
    a.m = m;
    a.tiles_o = (n + SG_BO - 1) / SG_BO;
    const int tiles_t = (m + SG_BT - 1) / SG_BT;
    a.tiles_total = a.tiles_o * tiles_t;
    // two workgroups per CU are resident: whole rounds of tiles stay whole, the
    // remainder is cut into half tiles when those fit into one round
    const int slots = 2 * 256;
    const int rem = a.tiles_total % slots;
    a.n_full = (rem != 0 && 2 * rem <= slots) ? a.tiles_total - rem : a.tiles_total;
    const int blocks = a.n_full + 2 * (a.tiles_total - a.n_full);
    const size_t lds = (size_t)2 * SG_STAGE * sizeof(half_t);
    hipLaunchKernelGGL(gemm_sparse_kernel, dim3((unsigned)blocks), dim3(SG_THREADS), lds, st, a);
    return hip_status(hipGetLastError());
}

}  // namespace slim
