// Prefill main kernel: Y = scale * (X Wc^T) + T L^T on the matrix cores, with
// the 2:4 weights as the sparse A operand of V_SMFMAC_F32_32X32X32_F16.
//
// Workgroup: 4 wavefronts, one per SIMD; tile (128 AT) output rows x 128 tokens;
// each wavefront owns (32 AT) rows x 128 tokens = AT x 4 accumulator tiles of
// 32 x 32.  AT = 4 is the working configuration (128 x 128 outputs per
// wavefront); AT = 2 finishes the row tiles left over after the last whole
// round of workgroups.
//   A (weights): never touches LDS.  Per 128 inputs a lane loads 16 bytes of
//     codes and 8 bytes of positions of each of its rows straight from global
//     memory (one stage ahead), turns 4 code bytes into 8 fp16 values in
//     registers, and passes the 16 position bits of those 4 groups as the index
//     operand (the canonical metadata is that operand's format).  Each wavefront
//     converts only its own rows, once, and uses them against all its tokens.
//   B (X): 128 tokens x 128 inputs per stage, double-buffered in LDS, loaded
//     from global memory two stages ahead through registers.  Every B fragment
//     read from LDS feeds AT matrix instructions.
//   Then the accumulators are multiplied by the row scale and the adapter
//   term continues on them with the dense instruction: A = L rows from global
//   memory, B = T (fp16, from the workspace) staged through the same LDS
//   buffers.  One rounding to fp16 at the store.
// All global reads are buffer loads: a uniform descriptor and a 32-bit offset,
// and rows past the end of a matrix read as zero.
#include <utility>

#include "slim_internal.h"

namespace slim {

constexpr int SG_BK = 128;              // inputs per stage
constexpr int SG_LD = SG_BK + 8;        // LDS row length in halves (272 B)
constexpr int SG_STAGE = 128 * SG_LD;   // halves per LDS buffer (128 tokens)
constexpr int NT = 4;                   // token tiles of 32 per wavefront
constexpr int XR = 8;                   // 128-bit pieces of an X stage per lane (16 token rows per pass)

struct SparseGemmArgs {
    const uint8_t *qvals;
    const uint8_t *meta;
    const float *scale;
    const half_t *X;     // [m][k]
    const half_t *L;     // [n][rank_pad]
    const half_t *T;     // [m][rank_pad] fp16
    half_t *Y;           // [m][n]
    int n, k, rank_pad, m;
    int tiles_o;         // row tiles of 512
    int tiles_total;     // row tiles x token tiles
    int n_full;          // tiles [0, n_full) run whole (AT = 4), the rest as two halves of 256 rows (AT = 2)
};

typedef __amdgpu_buffer_rsrc_t rsrc_t;

// Raw buffer descriptor over `bytes` bytes at p (32-bit data format word of gfx9).
__device__ __forceinline__ rsrc_t make_rsrc(const void *p, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)bytes, 0x00020000);
}

// The whole byte offset goes into the per-lane offset operand: that is the part
// the hardware checks against the descriptor's size (the scalar offset operand
// is added to the address without a check).
__device__ __forceinline__ uint4_t load16(rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(uint4_t,
                              __builtin_amdgcn_raw_buffer_load_b128(r, (int)(lane_off + uniform_off), 0, 0));
}

// Loads the compiler does not track.  Its wait-count pass is conservative
// around loops that carry loads in flight from one iteration to the next (it
// waited for loads issued moments earlier), so the main loop issues its global
// loads from asm and places the waits itself with vm_wait_*(): loads complete in
// order, vm_wait<N> returns once at most N are still in flight, and the values it
// names only count as defined from there on.  Every such load must have landed
// (vm_wait<0>) before its destination registers may die.
__device__ __forceinline__ uint4_t load16_untracked(uint4_t desc, uint32_t off)
{
    uint4_t v;
    asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(v) : "v"(off), "s"(desc));
    return v;
}
__device__ __forceinline__ uint2_t load8_untracked(uint4_t desc, uint32_t off)
{
    uint2_t v;
    asm volatile("buffer_load_dwordx2 %0, %1, %2, 0 offen" : "=v"(v) : "v"(off), "s"(desc));
    return v;
}
template <int N>
__device__ __forceinline__ void vm_wait_a(uint4_t (&q)[4], uint2_t (&mm)[4])
{
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+v"(q[0]), "+v"(q[1]), "+v"(q[2]), "+v"(q[3]), "+v"(mm[0]), "+v"(mm[1]), "+v"(mm[2]), "+v"(mm[3])
                 : "n"(N));
}
template <int N>
__device__ __forceinline__ void vm_wait_a(uint4_t (&q)[2], uint2_t (&mm)[2])
{
    asm volatile("s_waitcnt vmcnt(%4)" : "+v"(q[0]), "+v"(q[1]), "+v"(mm[0]), "+v"(mm[1]) : "n"(N));
}
template <int N>
__device__ __forceinline__ void vm_wait_x(uint4_t (&x)[8])
{
    asm volatile("s_waitcnt vmcnt(%8)"
                 : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
                 : "n"(N));
}
// Descriptor words for a raw buffer of `bytes` bytes (same as make_rsrc).
__device__ __forceinline__ uint4_t make_desc(const void *p, uint32_t bytes)
{
    const uint64_t a = reinterpret_cast<uint64_t>(p);
    return uint4_t{(uint32_t)a, (uint32_t)(a >> 32) & 0xFFFFu, bytes, 0x00020000u};
}

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
#define SLIM_ALL_ACC_REGS                                                                                            \
    "a0", "a1", "a2", "a3", "a4", "a5", "a6", "a7", "a8", "a9", SLIM_A10(1), SLIM_A10(2), SLIM_A10(3), SLIM_A10(4),  \
        SLIM_A10(5), SLIM_A10(6), SLIM_A10(7), SLIM_A10(8), SLIM_A10(9), SLIM_A10(10), SLIM_A10(11), SLIM_A10(12),   \
        SLIM_A10(13), SLIM_A10(14), SLIM_A10(15), SLIM_A10(16), SLIM_A10(17), SLIM_A10(18), SLIM_A10(19),            \
        SLIM_A10(20), SLIM_A10(21), SLIM_A10(22), SLIM_A10(23), SLIM_A10(24), "a250", "a251", "a252", "a253",        \
        "a254", "a255"

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

// AT row tiles of 32 per wavefront; accumulator tile (i, it) is a[16 (i NT + it) ..].
template <int AT>
__global__ __launch_bounds__(256, 1) void gemm_sparse_kernel(SparseGemmArgs a)
{
    constexpr int WROWS = 32 * AT;       // rows per wavefront
    constexpr int NB = 4 * NT;           // (slice, token tile) blocks per stage
    constexpr int HB = NB / 2;
    extern __shared__ __attribute__((aligned(16))) half_t lds[];   // two stage buffers
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const int li = lane & 31;            // A row / B token within a 32-tile
    const int lb = lane >> 5;            // k-block of the lane

    // AT = 4: workgroup b takes tile b.  AT = 2: workgroup b takes rows
    // 256 (b & 1) .. + 255 of tile n_full + b / 2.
    const int b = blockIdx.x;
    constexpr int split = 4 / AT;
    const int w = a.n_full * (split - 1) + b / split;
    const int o0 = (w % a.tiles_o) * 512 + (b % split) * (4 * WROWS) + wave * WROWS;
    const int t0 = (w / a.tiles_o) * 128;
    const int t_end = min(a.m, t0 + 128);                    // tokens of this workgroup: [t0, t_end)

    asm volatile("" : : : SLIM_ALL_ACC_REGS);
    static_for<16 * AT * NT>([&](auto r) { acc_write<r>(0.0f); });

    const uint32_t k = (uint32_t)a.k;
    const int nsteps = a.k / SG_BK;

    // this lane's row of tile 0 (rows past n read as zero); tile i and stage s
    // are uniform terms
    const uint32_t qv = (uint32_t)(o0 + li) * (k / 4) + 16u * lb;
    const uint32_t mv = (uint32_t)(o0 + li) * (k / 8) + 8u * lb;
    uint4_t qa[2][AT];
    uint2_t ma[2][AT];

    // X / T staging: 16 lanes per token row (256 contiguous bytes), 16 rows per pass
    const int srow = tid >> 4, scol = (tid & 15) * 8;
    const uint32_t xv = ((uint32_t)(t0 + srow) * k + (uint32_t)scol) * 2u;
    half_t *const lw = lds + srow * SG_LD + scol;
    uint4_t xr[2][XR];
    auto stage_store = [&](int u, const uint4_t (&reg)[XR]) {
#pragma unroll
        for (int p = 0; p < XR; ++p) *reinterpret_cast<uint4_t *>(lw + u * SG_STAGE + p * 16 * SG_LD) = reg[p];
    };

    // B fragment address of this lane inside a stage buffer: token li of tile
    // it, inputs 16 t + 8 lb (values 0-7) and 64 + 16 t + 8 lb (values 8-15)
    const half_t *const lr = lds + li * SG_LD + 8 * lb;
    auto read_b = [&](int u, int t, int it) {
        const half_t *bp = lr + u * SG_STAGE + it * 32 * SG_LD + 16 * t;
        const half8_t b1 = *reinterpret_cast<const half8_t *>(bp);
        const half8_t b2 = *reinterpret_cast<const half8_t *>(bp + 64);
        return __builtin_shufflevector(b1, b2, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
    };

    // One stage = 4 k-slices (t) x NT token tiles (it), software-pipelined by
    // hand: the LDS reads of the next (t, it) are issued before the matrix
    // instructions of the current one.  With one wavefront per SIMD nothing else
    // fills the matrix pipe's shadow, so the conversion of the next slice's codes
    // is cut into pieces of one group (3-4 instructions) and one piece follows
    // each matrix instruction, pinned there by scheduling barriers.
    // `fetch(bi)` is called once per block, bi = t NT + it, right after the
    // block's LDS reads: the place to issue a share of the next stages' loads.
    auto compute_stage = [&](int u, const uint4_t (&q)[AT], const uint2_t (&mm)[AT], auto &&fetch) {
        half8_t a_cur[AT], a_nxt[AT];
#pragma unroll
        for (int i = 0; i < AT; ++i) a_cur[i] = codes_to_half8(q[i][0]);
        half16_t b_cur = read_b(u, 0, 0), b_nxt = b_cur;
        static_for<4>([&](auto tc) {
            constexpr int t = tc;
            static_for<NT>([&](auto itc) {
                constexpr int it = itc;
                if (it + 1 < NT)
                    b_nxt = read_b(u, t, it + 1);
                else if (t + 1 < 4)
                    b_nxt = read_b(u, t + 1, 0);
                fetch(std::integral_constant<int, t * NT + it>{});
                __builtin_amdgcn_sched_barrier(0);      // keep the reads ahead of the matrix work
                static_for<AT>([&](auto ic) {
                    constexpr int i = ic;
                    // even slice: index bits 15..0, odd slice: bits 31..16 of the position dword
                    smfmac_fixed<i * NT + it, (t & 1) != 0>(a_cur[i], b_cur, (int)mm[i][t >> 1]);
                    if constexpr (t + 1 < 4) {
                        // 4 AT pieces per slice over AT NT matrix instructions
                        constexpr int pc = it * AT + i, tile = pc / 4, g = pc % 4;
                        if constexpr (tile < AT) {
                            const half2_t h = code_pair(codes_bias(q[tile][t + 1]), g);
                            a_nxt[tile][2 * g] = h[0];
                            a_nxt[tile][2 * g + 1] = h[1];
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                });
                b_cur = b_nxt;
            });
#pragma unroll
            for (int i = 0; i < AT; ++i) a_cur[i] = a_nxt[i];
        });
    };

    // The global loads are spread over the stage, one or two per block, so the
    // four wavefronts do not all queue sixteen loads at the address unit right
    // after the barrier (that burst stalled the first slice of every stage).
    // Weights of stage s + 1 go out in the first half of stage s; X of stage
    // s + 2 in the second half, to be written to LDS at the end of stage s + 1.
    // Fetches past the last stage stay inside the descriptors or read as zero and
    // are never used.
    {
        const uint4_t dq = make_desc(a.qvals, (uint32_t)a.n * (k / 4));
        const uint4_t dm = make_desc(a.meta, (uint32_t)a.n * (k / 8));
        const uint4_t dx = make_desc(a.X, (uint32_t)a.m * k * 2);
        auto fetch_a = [&](int j, int s, uint4_t (&q)[AT], uint2_t (&mm)[AT]) {    // j < 2 AT
            if (j < AT)
                q[j] = load16_untracked(dq, qv + (uint32_t)j * 8u * k + (uint32_t)s * (SG_BK / 4));
            else
                mm[j - AT] = load8_untracked(dm, mv + (uint32_t)(j - AT) * 4u * k + (uint32_t)s * (SG_BK / 8));
        };
        auto fetch_x = [&](int p, int s, uint4_t (&reg)[XR]) {
            reg[p] = load16_untracked(dx, xv + (uint32_t)s * (SG_BK * 2) + (uint32_t)p * 32u * k);
        };
        // in flight after the prologue, oldest first: X(0), A(0), X(1)
#pragma unroll
        for (int p = 0; p < XR; ++p) fetch_x(p, 0, xr[0]);
#pragma unroll
        for (int j = 0; j < 2 * AT; ++j) fetch_a(j, 0, qa[0], ma[0]);
#pragma unroll
        for (int p = 0; p < XR; ++p) fetch_x(p, 1, xr[1]);
        vm_wait_x<2 * AT + XR>(xr[0]);
        stage_store(0, xr[0]);
        __syncthreads();
        for (int s0 = 0; s0 < nsteps; s0 += 2) {
            static_for<2>([&](auto uc) {
                constexpr int u = uc;
                const int s = s0 + u;
                if (s >= nsteps) return;
                // in flight here, oldest first: A(s), X(s + 1)
                vm_wait_a<XR>(qa[u], ma[u]);
                compute_stage(u, qa[u], ma[u], [&](auto bc) {
                    constexpr int bi = bc;
                    if constexpr (bi < HB) {
                        constexpr int per = (2 * AT + HB - 1) / HB;      // weights of stage s + 1
#pragma unroll
                        for (int j = bi * per; j < (bi + 1) * per && j < 2 * AT; ++j)
                            fetch_a(j, s + 1, qa[u ^ 1], ma[u ^ 1]);
                    } else {
                        constexpr int per = (XR + HB - 1) / HB;          // X of stage s + 2
#pragma unroll
                        for (int p = (bi - HB) * per; p < (bi - HB + 1) * per && p < XR; ++p)
                            fetch_x(p, s + 2, xr[u]);
                    }
                });
                // in flight, oldest first: X(s + 1), A(s + 1), X(s + 2)
                vm_wait_x<2 * AT + XR>(xr[u ^ 1]);
                stage_store(u ^ 1, xr[u ^ 1]);
                __syncthreads();
            });
        }
        // the fetches past the last stage must land before their registers are reused
        vm_wait_a<0>(qa[0], ma[0]);
        vm_wait_a<0>(qa[1], ma[1]);
        vm_wait_x<0>(xr[0]);
        vm_wait_x<0>(xr[1]);
    }

    // row scale: accumulator element 4 blk + e of tile i is row 32 i + 8 blk + 4 lb + e
    {
        acc_settle();
        const rsrc_t rs = make_rsrc(a.scale, (uint32_t)a.n * 4u);
        static_for<AT>([&](auto ic) {
            constexpr int i = ic;
            uint4_t sv[4];
#pragma unroll
            for (int blk = 0; blk < 4; ++blk)
                sv[blk] = load16(rs, (uint32_t)(o0 + 4 * lb) * 4u, (uint32_t)(32 * i + 8 * blk) * 4u);
            static_for<NT>([&](auto itc) {
                constexpr int it = itc;
                static_for<16>([&](auto ec) {
                    constexpr int e = ec;
                    // (bit-casting the vector element in place reads element 0 with this
                    // compiler; go through a scalar)
                    const uint32_t sbits = sv[e / 4][e % 4];
                    const float sc = __builtin_bit_cast(float, sbits);
                    acc_write<16 * (i * NT + it) + e>(acc_read<16 * (i * NT + it) + e>() * sc);
                });
            });
        });
        acc_settle();
    }

    // adapter term: dense steps of 16 ranks; T staged like X, L rows from global
    if (a.rank_pad > 0) {
        const uint32_t rp = (uint32_t)a.rank_pad;
        const rsrc_t rl = make_rsrc(a.L, (uint32_t)a.n * rp * 2u);
        const rsrc_t rt = make_rsrc(a.T, (uint32_t)a.m * rp * 2u);
        const uint32_t lv = ((uint32_t)(o0 + li) * rp + 8u * lb) * 2u;
        const uint32_t tv = ((uint32_t)(t0 + srow) * rp + (uint32_t)scol) * 2u;
        const int rstages = ((int)rp + SG_BK - 1) / SG_BK;
        auto stage_load_t = [&](int s) {
#pragma unroll
            for (int p = 0; p < XR; ++p) xr[0][p] = load16(rt, tv, (uint32_t)s * (SG_BK * 2) + (uint32_t)p * 32u * rp);
        };
        // columns past rank_pad in the last stage hold other rows' data; they are
        // staged but never multiplied (jn below)
        stage_load_t(0);
        stage_store(0, xr[0]);
        __syncthreads();
        for (int s = 0; s < rstages; ++s) {
            const int u = s & 1;
            if (s + 1 < rstages) stage_load_t(s + 1);
            const int jn = min(SG_BK, (int)rp - s * SG_BK) / 16;      // dense steps in this stage
            uint4_t la[AT], ln[AT];
#pragma unroll
            for (int i = 0; i < AT; ++i) la[i] = load16(rl, lv, ((uint32_t)i * 32u * rp + (uint32_t)s * SG_BK) * 2u);
            for (int j = 0; j < jn; ++j) {
                if (j + 1 < jn) {
#pragma unroll
                    for (int i = 0; i < AT; ++i)
                        ln[i] = load16(rl, lv, ((uint32_t)i * 32u * rp + (uint32_t)(s * SG_BK + 16 * (j + 1))) * 2u);
                }
                static_for<NT>([&](auto itc) {
                    constexpr int it = itc;
                    const half8_t bv =
                        *reinterpret_cast<const half8_t *>(lr + u * SG_STAGE + it * 32 * SG_LD + 16 * j);
                    static_for<AT>([&](auto ic) {
                        constexpr int i = ic;
                        mfma_fixed<i * NT + it>(__builtin_bit_cast(half8_t, la[i]), bv);
                    });
                });
#pragma unroll
                for (int i = 0; i < AT; ++i) la[i] = ln[i];
            }
            if (s + 1 < rstages) stage_store(u ^ 1, xr[0]);
            __syncthreads();
        }
        acc_settle();
    }

    // store: lane holds token t0 + 32 it + li, rows o .. o + 3 per (i, blk)
    const bool vec_ok = (a.n & 3) == 0;
    static_for<NT>([&](auto itc) {
        constexpr int it = itc;
        const int t = t0 + 32 * it + li;
        if (t >= t_end) return;
        static_for<AT>([&](auto ic) {
            constexpr int i = ic;
            static_for<4>([&](auto bc) {
                constexpr int blk = bc;
                const int o = o0 + 32 * i + 8 * blk + 4 * lb;
                if (o >= a.n) return;
                float v[4];
                v[0] = acc_read<16 * (i * NT + it) + 4 * blk + 0>();
                v[1] = acc_read<16 * (i * NT + it) + 4 * blk + 1>();
                v[2] = acc_read<16 * (i * NT + it) + 4 * blk + 2>();
                v[3] = acc_read<16 * (i * NT + it) + 4 * blk + 3>();
                half_t *y = a.Y + (size_t)t * a.n + o;
                if (vec_ok) {
                    half4_t h;
#pragma unroll
                    for (int e = 0; e < 4; ++e) h[e] = (half_t)v[e];
                    *reinterpret_cast<half4_t *>(y) = h;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (o + e < a.n) y[e] = (half_t)v[e];
                }
            });
        });
    });
}

// Whole rounds of tiles (one workgroup per CU) stay whole; the remainder is cut
// into halves of 256 rows (a second launch) when those fit into one round.
static void plan_tiles(SparseGemmArgs &a, int slots)
{
    a.tiles_o = (a.n + 511) / 512;
    const int tiles_t = (a.m + 127) / 128;
    a.tiles_total = a.tiles_o * tiles_t;
    const int rem = a.tiles_total % slots;
    a.n_full = (rem != 0 && 2 * rem <= slots) ? a.tiles_total - rem : a.tiles_total;
}

// Buffer offsets are 32 bits wide: the caller has checked that the weight and
// adapter matrices stay below 4 GiB each; X, T and Y are walked in token chunks
// that do.
int launch_gemm_sparse(const uint8_t *qvals, const uint8_t *meta, const float *scale, const half_t *X, const half_t *L,
                       const half_t *T, half_t *Y, int n, int k, int rank_pad, int m, hipStream_t st)
{
    SparseGemmArgs a{};
    a.qvals = qvals;
    a.meta = meta;
    a.scale = scale;
    a.L = L;
    a.n = n;
    a.k = k;
    a.rank_pad = rank_pad;
    const uint64_t row_bytes = 2ull * (uint64_t)(k > rank_pad ? k : rank_pad);
    const int chunk = (int)((0xFFFFFFFFull / row_bytes) / 128 * 128);
    if (chunk < 128) return SLIM_ERR_SHAPE;
    const size_t lds = (size_t)2 * SG_STAGE * sizeof(half_t);
    for (int t0 = 0; t0 < m; t0 += chunk) {
        a.m = m - t0 < chunk ? m - t0 : chunk;
        a.X = X + (size_t)t0 * k;
        a.T = T ? T + (size_t)t0 * rank_pad : nullptr;
        a.Y = Y + (size_t)t0 * n;
        plan_tiles(a, 256);
        const int n_half = 2 * (a.tiles_total - a.n_full);
        if (a.n_full > 0) hipLaunchKernelGGL(gemm_sparse_kernel<4>, dim3((unsigned)a.n_full), dim3(256), lds, st, a);
        if (n_half > 0) hipLaunchKernelGGL(gemm_sparse_kernel<2>, dim3((unsigned)n_half), dim3(256), lds, st, a);
    }
    return hip_status(hipGetLastError());
}

}  // namespace slim
