// Shared device code of the prefill kernels (matrix-core GEMMs with 128 tokens per
// workgroup): buffer loads with and without compiler tracking, accumulators held
// in the accumulation registers by number, and the dense k-loop both kernels use.
#ifndef SLIM_MMA_H
#define SLIM_MMA_H

#include <utility>

#include "slim_internal.h"

namespace slim {

constexpr int SG_BK = 128;              // inputs per stage
constexpr int SG_LD = SG_BK + 8;        // LDS row length in halves (272 B)
constexpr int SG_STAGE = 128 * SG_LD;   // halves per LDS buffer (128 tokens)
constexpr int NT = 4;                   // token tiles of 32 per wavefront
constexpr int XR = 8;                   // 128-bit pieces of an X stage per lane (16 token rows per pass)

// Compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>).
template <int... Is, class F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, Is...>, F &&f)
{
    (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// Accumulators of a wavefront that owns 128 x 128 outputs: 256 registers, the
// whole accumulation half of the register file, with everything else in the
// ordinary half.  The compiler's allocator does not find this split (it spills),
// so the accumulation registers are addressed by number from asm: tile T
// occupies a[16 T .. 16 T + 15] and the compiler never sees a value in them.  It
// is told that they are in use (clobber list at kernel entry) and the library is
// built with spilling into accumulation registers switched off, so it has no
// reason to touch them.  Being asm, these instructions are outside the
// compiler's hazard bookkeeping: acc_settle() goes wherever accumulators pass
// between matrix instructions and reads or writes of them.
#define SLIM_A10(b) "a" #b "0", "a" #b "1", "a" #b "2", "a" #b "3", "a" #b "4", "a" #b "5", "a" #b "6", "a" #b "7", \
                    "a" #b "8", "a" #b "9"
#define SLIM_ACC_REGS_64                                                                                             \
    "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", SLIM_A10(1), SLIM_A10(2), SLIM_A10(3), SLIM_A10(4),  \
        SLIM_A10(5), "a60", "a61", "a62", "a63"
#define SLIM_ACC_REGS_128                                                                                            \
    SLIM_ACC_REGS_64, "a64", "a65", "a66", "a67", "a68", "a69", SLIM_A10(7), SLIM_A10(8), SLIM_A10(9), SLIM_A10(10), \
        SLIM_A10(11), "a120", "a121", "a122", "a123", "a124", "a125", "a126", "a127"
#define SLIM_ACC_REGS_256                                                                                            \
    SLIM_ACC_REGS_128, "a128", "a129", SLIM_A10(13), SLIM_A10(14), SLIM_A10(15), SLIM_A10(16), SLIM_A10(17),         \
        SLIM_A10(18), SLIM_A10(19), SLIM_A10(20), SLIM_A10(21), SLIM_A10(22), SLIM_A10(23), SLIM_A10(24), "a250",    \
        "a251", "a252", "a253", "a254", "a255"

// The accumulators of a kernel with AT row tiles per wavefront: a[0 .. 64 AT).  Fewer reserved
// registers let two (AT = 2) or three (AT = 1) wavefronts share a SIMD.
template <int AT>
__device__ __forceinline__ void acc_reserve()
{
    if constexpr (AT == 1)
        asm volatile("" : : : SLIM_ACC_REGS_64);
    else if constexpr (AT == 2)
        asm volatile("" : : : SLIM_ACC_REGS_128);
    else
        asm volatile("" : : : SLIM_ACC_REGS_256);
}

template <int R>
__device__ __forceinline__ void acc_write(float v)
{
    asm volatile("v_accvgpr_write_b32 a[%1], %0" : : "v"(v), "n"(R));
}
template <int R>
__device__ __forceinline__ float acc_read()
{
    float v;
    asm volatile("v_accvgpr_read_b32 %0, a[%1]" : "=v"(v) : "n"(R));
    return v;
}
// longest result latency of a matrix instruction (16 passes) plus margin
__device__ __forceinline__ void acc_settle() { asm volatile("s_nop 15\n\ts_nop 7"); }

// Sparse step on accumulator tile T: a[16 T ..] += A(sparse, 32 x 32) B(32 x 32).
// HI: the index operand's bits 31..16 hold this slice's positions, else bits 15..0.
template <int T, bool HI>
__device__ __forceinline__ void smfmac_fixed(half8_t av, half16_t bv, int idx)
{
    if (HI)
        asm volatile("v_smfmac_f32_32x32x32_f16 a[%3:%4], %0, %1, %2 abid:1"
                     :
                     : "v"(av), "v"(bv), "v"(idx), "n"(16 * T), "n"(16 * T + 15));
    else
        asm volatile("v_smfmac_f32_32x32x32_f16 a[%3:%4], %0, %1, %2"
                     :
                     : "v"(av), "v"(bv), "v"(idx), "n"(16 * T), "n"(16 * T + 15));
}
template <int T>
__device__ __forceinline__ void mfma_fixed(half8_t av, half8_t bv)
{
    asm volatile("v_mfma_f32_32x32x16_f16 a[%2:%3], %0, %1, a[%2:%3]"
                 :
                 : "v"(av), "v"(bv), "n"(16 * T), "n"(16 * T + 15));
}

// The order in which the prefill kernels hand output tiles (row tile x token tile) to workgroups.
// These kernels are bound by the bytes their workgroups request from L2, and a die's L2 serves the
// workgroups whose index is congruent to the die's modulo 8 (the dispatcher deals workgroups to the
// dies in turn).  With tiles handed out in index order the 32 workgroups a die holds at a time are
// scattered over the layer (8192 x 8192: 2 row tiles x 16 token tiles, 42 MB of distinct operands for
// 4 MB of L2); in blocks of 4 row tiles x 8 token tiles they share 4 weight tiles and 8 X tiles
// (28 MB), and the main kernel is 13 % faster on that layer.
//   q -> tile: blocks of kBlkR x kBlkT tiles, row blocks fastest within a band of kBlkT token tiles,
//   the tiles of a block rows fastest; ragged blocks at the edges just have fewer tiles.  Returns
//   row tile + tiles_o * token tile.
constexpr int kDies = 8, kBlkR = 4, kBlkT = 8;
__host__ __device__ __forceinline__ int blocked_tile(int q, int tiles_o, int tiles_t)
{
    const int band = tiles_o * kBlkT;                       // tiles per band
    const int tb_last = (tiles_t - 1) / kBlkT, rb_last = (tiles_o - 1) / kBlkR;
    const int tb = q / band < tb_last ? q / band : tb_last;
    const int bt = tiles_t - tb * kBlkT < kBlkT ? tiles_t - tb * kBlkT : kBlkT;            // token tiles in this band
    const int q2 = q - tb * band;
    const int rb = q2 / (kBlkR * bt) < rb_last ? q2 / (kBlkR * bt) : rb_last;
    const int br = tiles_o - rb * kBlkR < kBlkR ? tiles_o - rb * kBlkR : kBlkR;            // row tiles in this block
    const int e = q2 - rb * kBlkR * bt;
    return (tb * kBlkT + e / br) * tiles_o + rb * kBlkR + e % br;
}

// Dense continuation on the fixed accumulators: acc(i, it) += A_i B_it^T over K
// inputs (K a multiple of 32), 16 per step of V_MFMA_F32_32X32X16_F16.
//   A: rows from global memory, 16 bytes per lane, row tile and step (da, av:
//      this lane's offset for tile 0, step 0; a_tile: bytes between row tiles;
//      a_step: bytes between steps), fetched three steps ahead into four rotating sets;
//   B: 128 tokens x 128 inputs per stage staged through the LDS buffers like X
//      (db, bv: this lane's staging offset for stage 0; b_pass: bytes between
//      the passes of 16-byte loads; a stage is 128 BB bytes further), next stage's
//      loads issued during steps 0-3 of the current one.  BB = 2: B is fp16, eight
//      loads per lane and stage; BB = 1: B is 8-bit codes, four loads, which
//      stage_store(buffer, registers, piece: one of them, or all with -1) expands to fp16 on their way into LDS.
// Loads past the end stay inside the descriptors or read as zero and are not
// used; issuing them anyway keeps one path through the loop body.
// Starts and ends with every wavefront past a barrier.
template <int AT, int BB = 2, class Store>
__device__ __forceinline__ void dense_phase(rsrc_t da, uint32_t av, uint32_t a_tile, uint32_t a_step, rsrc_t db,
                                            uint32_t bv,
                                            uint32_t b_pass, int K, const half_t *lr, uint4_t (&xs)[XR * BB / 2],
                                            Store &&stage_store)
{
    constexpr int XRN = XR * BB / 2;              // 16-byte loads of a stage per lane
    const int nst = K / 16;                       // steps
    const int stages = (K + SG_BK - 1) / SG_BK;
    uint4_t la[4][AT];
#pragma unroll
    for (int p = 0; p < XRN; ++p) xs[p] = load16(db, bv, (uint32_t)p * b_pass);
#pragma unroll
    for (int g = 0; g < 3; ++g)
#pragma unroll
        for (int i = 0; i < AT; ++i) la[g][i] = load16(da, av, (uint32_t)i * a_tile + (uint32_t)g * a_step);
    stage_store(0, xs);
    __syncthreads();
    for (int s = 0; s < stages; ++s) {
        const int u = s & 1;
        const int jn = min(8, nst - 8 * s);       // steps in this stage
        half8_t b_cur[NT], b_nxt[NT];
#pragma unroll
        for (int it = 0; it < NT; ++it)
            b_cur[it] = *reinterpret_cast<const half8_t *>(lr + u * SG_STAGE + it * 32 * SG_LD);
        static_for<8>([&](auto jc) {
            constexpr int j = jc;
            if (j >= jn) return;
            const int g = 8 * s + j;
            static_for<NT>([&](auto itc) {
                constexpr int it = itc;
                if constexpr (it < AT)
                    la[(j + 3) & 3][it] = load16(da, av, (uint32_t)it * a_tile + (uint32_t)(g + 3) * a_step);
                if constexpr (j < 4 && it < XRN / 4)
                    xs[(XRN / 4) * j + it] =
                        load16(db, bv, (uint32_t)(s + 1) * (SG_BK * BB) + (uint32_t)((XRN / 4) * j + it) * b_pass);
                if constexpr (j + 1 < 8)
                    b_nxt[it] = *reinterpret_cast<const half8_t *>(lr + u * SG_STAGE + it * 32 * SG_LD + 16 * (j + 1));
                // the next stage's B, loaded four steps ago, goes into the other buffer (nobody reads it during
                // this stage) piece by piece, not in the stage's tail
                if constexpr (j >= 4 && it < XRN / 4)
                    if (s + 1 < stages) stage_store(u ^ 1, xs, (XRN / 4) * (j - 4) + it);
                __builtin_amdgcn_sched_barrier(0);
                static_for<AT>([&](auto ic) {
                    constexpr int i = ic;
                    mfma_fixed<i * NT + it>(__builtin_bit_cast(half8_t, la[j & 3][i]), b_cur[it]);
                });
                __builtin_amdgcn_sched_barrier(0);
            });
#pragma unroll
            for (int it = 0; it < NT; ++it) b_cur[it] = b_nxt[it];
        });
        __syncthreads();
    }
}

// The A operand of dense_phase_q4(): the rows of a matrix [rows][K] stored as 4-bit codes with one
// fp16 scale per group of 128 columns (slim_internal.h: tiles of 16 rows x 256 columns, a row's 256
// columns in 128 contiguous bytes).
struct Q4Rows {
    rsrc_t codes, scales;
    uint32_t cv, c_tile;     // code bytes: this lane's offset for row tile 0, columns 0-255; bytes between row tiles of 32
    uint32_t sv, s_tile;     // scale bytes: this lane's offset for row tile 0, group 0; bytes between row tiles of 32
    uint32_t g0;             // group of 128 columns at which the k range starts
};

// Lane (li, lb) of a wavefront whose row tile 0 starts at row o0 (a multiple of 32), k range from k0 (a
// multiple of 128).  Rows past the last tile of 16 lie past the end of both descriptors and read as zero.
__device__ __forceinline__ Q4Rows q4_rows_operand(const uint8_t *codes, const half_t *scales, int rows, int K, int o0,
                                                  int li, int lb, int k0)
{
    const uint32_t ct = q4_ctiles(K);
    Q4Rows q;
    q.codes = make_rsrc(codes, (uint32_t)q4_code_bytes(rows, K));
    q.scales = make_rsrc(scales, (uint32_t)q4_scale_bytes(rows, K));
    q.cv = ((uint32_t)(o0 / 16 + (li >> 4)) * ct) * 2048u + (uint32_t)(li & 15) * 128u + (uint32_t)lb * 16u;
    q.c_tile = 2u * ct * 2048u;
    q.sv = (uint32_t)(o0 + li) * (2u * ct) * 2u;
    q.s_tile = 32u * (2u * ct) * 2u;
    q.g0 = (uint32_t)k0 / 128u;
    return q;
}

// dense_phase() with the A operand read as 4-bit codes: acc(i, it) += A_i B_it^T over K inputs (K a
// multiple of 32), B staged through LDS exactly as there.
//   A: per stage of 128 inputs (one scale group) a lane loads 2 x 16 bytes of codes and one scale per row
//      tile: 3 AT loads per stage where fp16 rows take 8 AT.  One register set: the half of a stage that
//      steps 0-3 use is refilled for the next stage at step 3, the other half at step 7, four steps
//      before the first use either way.  A dword of codes becomes eight fp16 values (the 13-instruction
//      conversion of the weights) times the scale (four packed multiplies: the value is
//      fp16(code * scale), what the expansion to fp16 stores), one step ahead, in pieces of two values
//      pinned behind the matrix instructions.
//   Order of the inputs inside a stage: the 16 bytes a lane loads are 32 consecutive columns of its row,
//      so that a load instruction asks for 32 contiguous bytes of each of 32 rows and the two loads of
//      a stage use up half a line of every row.  Step 4 q + j therefore multiplies columns
//      64 q + 32 lb + 8 j + [0, 8) on lane half lb, and the B fragments are read from LDS in that order
//      (lrq: this lane's token row at column 32 lb), one step ahead; a sum over the inputs does
//      not care.  A partly valid stage runs whole groups of four steps: bcol = first column of the
//      lane's share of a B stage, whose columns past K are replaced by zeros on their way into LDS.
// Starts and ends with every wavefront past a barrier.
template <int AT, int BB = 2, class Store>
__device__ __forceinline__ void dense_phase_q4(const Q4Rows &qa, rsrc_t db, uint32_t bv, uint32_t b_pass, int bcol,
                                               int K, const half_t *lrq, uint4_t (&xs)[XR * BB / 2],
                                               Store &&stage_store)
{
    constexpr int XRN = XR * BB / 2;
    static_assert(AT <= NT, "one load per block refills a half stage");
    const int stages = (K + SG_BK - 1) / SG_BK;
    uint4_t cq[2][AT];             // [half of the stage][row tile]
    half_t sc[AT], sc_nxt[AT];
    auto fetch_codes = [&](int h, int i, int s) {
        const uint32_t sg = qa.g0 + (uint32_t)s;
        cq[h][i] = load16(qa.codes, qa.cv, (uint32_t)i * qa.c_tile + (sg >> 1) * 2048u + (sg & 1u) * 64u + (uint32_t)h * 32u);
    };
    auto fetch_scale = [&](int i, int s, half_t (&dst)[AT]) {
        dst[i] = load_half(qa.scales, qa.sv, (uint32_t)i * qa.s_tile + (qa.g0 + (uint32_t)s) * 2u);
    };
    auto zero_tail = [&](int s) {
        if (SG_BK * s + bcol >= K) {
#pragma unroll
            for (int p = 0; p < XRN; ++p) xs[p] = uint4_t{0u, 0u, 0u, 0u};
        }
    };
    auto read_b = [&](int u, int it, int jj) {
        return *reinterpret_cast<const half8_t *>(lrq + u * SG_STAGE + it * 32 * SG_LD + 64 * (jj >> 2) + 8 * (jj & 3));
    };
#pragma unroll
    for (int p = 0; p < XRN; ++p) xs[p] = load16(db, bv, (uint32_t)p * b_pass);
#pragma unroll
    for (int i = 0; i < AT; ++i) {
        fetch_codes(0, i, 0);
        fetch_codes(1, i, 0);
        fetch_scale(i, 0, sc);
    }
    zero_tail(0);
    stage_store(0, xs);
    __syncthreads();
    half8_t a_cur[AT], a_nxt[AT];
#pragma unroll
    for (int i = 0; i < AT; ++i) a_cur[i] = codes_to_half8(cq[0][i][0]) * sc[i];
    for (int s = 0; s < stages; ++s) {
        const int u = s & 1;
        const int jn = min(8, 4 * ((K - SG_BK * s + 63) / 64));       // steps in this stage
        half8_t b_cur[NT], b_nxt[NT];
#pragma unroll
        for (int it = 0; it < NT; ++it) b_cur[it] = read_b(u, it, 0);
        static_for<8>([&](auto jc) {
            constexpr int jj = jc;
            if (jj >= jn) return;
            constexpr int nq = ((jj + 1) & 7) >> 2, nd = (jj + 1) & 3;      // where the codes of the next step are
            static_for<NT>([&](auto itc) {
                constexpr int it = itc;
                if constexpr (jj == 2 && it < AT) fetch_scale(it, s + 1, sc_nxt);
                if constexpr (jj == 3 && it < AT) fetch_codes(0, it, s + 1);
                if constexpr (jj == 7 && it < AT) fetch_codes(1, it, s + 1);
                if constexpr (jj < 4 && it < XRN / 4)
                    xs[(XRN / 4) * jj + it] =
                        load16(db, bv, (uint32_t)(s + 1) * (SG_BK * BB) + (uint32_t)((XRN / 4) * jj + it) * b_pass);
                if constexpr (jj + 1 < 8) b_nxt[it] = read_b(u, it, jj + 1);
                if constexpr (jj >= 4 && it < XRN / 4) {
                    constexpr int p = (XRN / 4) * (jj - 4) + it;
                    if (s + 1 < stages) {
                        if (SG_BK * (s + 1) + bcol >= K) xs[p] = uint4_t{0u, 0u, 0u, 0u};
                        stage_store(u ^ 1, xs, p);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
                static_for<AT>([&](auto ic) {
                    constexpr int i = ic;
                    mfma_fixed<i * NT + it>(a_cur[i], b_cur[it]);
                    // 4 AT pieces of two values over AT NT matrix instructions
                    constexpr int pc = it * AT + i, tile = pc / 4, g = pc % 4;
                    if constexpr (tile < AT) {
                        const half_t sv = jj == 7 ? sc_nxt[tile] : sc[tile];
                        const half2_t h = code_pair(codes_bias(cq[nq][tile][nd]), g) * sv;
                        a_nxt[tile][2 * g] = h[0];
                        a_nxt[tile][2 * g + 1] = h[1];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
            });
#pragma unroll
            for (int it = 0; it < NT; ++it) b_cur[it] = b_nxt[it];
#pragma unroll
            for (int i = 0; i < AT; ++i) a_cur[i] = a_nxt[i];
        });
#pragma unroll
        for (int i = 0; i < AT; ++i) sc[i] = sc_nxt[i];
        __syncthreads();
    }
}

}  // namespace slim

#endif  // SLIM_MMA_H
