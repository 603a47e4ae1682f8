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
//     memory (two stages ahead; the packed layout makes each load instruction one
//     contiguous KiB or half KiB), turns 4 code bytes into 8 fp16 values in
//     registers, and passes the 16 position bits of those 4 groups as the index
//     operand (the canonical metadata is that operand's format).  Each wavefront
//     converts only its own rows, once, and uses them against all its tokens.
//   B (X): 128 tokens x 128 inputs per stage, double-buffered in LDS, loaded
//     from global memory two stages ahead through registers.  Every B fragment
//     read from LDS feeds AT matrix instructions.
//   Then the accumulators are multiplied by the row scale and the adapter
//   term continues on them with the dense instruction: A = L rows from global
//   memory (fp16, or 4-bit codes turned into fp16 in registers), B = T (fp16,
//   from the workspace) staged through the same LDS buffers.  One rounding to
//   fp16 at the store.
// All global reads are buffer loads: a uniform descriptor and a 32-bit offset,
// and rows past the end of a matrix read as zero.
#include "slim_mma.h"

namespace slim {

typedef int int4_t __attribute__((ext_vector_type(4)));
typedef int int8v_t __attribute__((ext_vector_type(8)));

struct SparseGemmArgs {
    const uint8_t *qvals;
    const uint8_t *meta;
    const float *scale;
    const half_t *X;     // [m][k] fp16, or (XF != 0) the same tensor as 8-bit codes, one byte per value
    const float *x_scale; // XF != 0: the tensor's scale (device memory)
    const half_t *L;     // [n][rank_pad], or null with the 4-bit form:
    const uint8_t *Lq;   // codes of L [n][rank] (4-bit adapter layout)
    const half_t *Ls;    // their group scales
    int rank;
    const half_t *T;     // [m][rank_pad] fp16
    half_t *Y;           // [m][n]
    int n, k, rank_pad, m;
    int tiles_o;         // row tiles of 512
    int tiles_total;     // row tiles x token tiles
    int n_full;          // tiles [0, n_full) run whole (AT = 4), the rest as halves of 256 rows (AT = 2) or quarters (AT = 1)
    int rem_split;       // pieces per remaining tile: 1 (none remain), 2 or 4
    int per_die;         // workgroup slots per die (slots / 8), 0: the number of compute units is not a multiple of 8
};

// Which tile a workgroup works on: position q of the blocked order (blocked_tile(), slim_mma.h).  In
// whole rounds of `slots` workgroups die d takes positions d * per_die .. of the round, i.e. one
// block of 4 row tiles x 8 token tiles where the layer has them (interleave); elsewhere q = w.
__host__ __device__ __forceinline__ int tile_of_workgroup(const SparseGemmArgs &a, int w, bool interleave)
{
    int q = w;
    if (interleave && a.per_die > 0) {
        const int slots = a.per_die * kDies;
        if (w < (a.n_full / slots) * slots) q = (w / slots) * slots + (w % kDies) * a.per_die + (w % slots) / kDies;
    }
    return blocked_tile(q, a.tiles_o, a.tiles_total / a.tiles_o);
}

// Sparse step with 8-bit operands on accumulator tile T: a[16 T ..] += A(sparse, 32 x 64, E5M2 codes of
// the integer weights) B(64 x 32, FP8 inputs: E4M3, or E5M2 with E5).  The index operand is one
// dword: 8 groups of four inputs per lane.
template <int T, bool E5>
__device__ __forceinline__ void smfmac8_fixed(int4_t av, int8v_t bv, int idx)
{
    if (E5)
        asm volatile("v_smfmac_f32_32x32x64_bf8_bf8 a[%3:%4], %0, %1, %2"
                     :
                     : "v"(av), "v"(bv), "v"(idx), "n"(16 * T), "n"(16 * T + 15));
    else
        asm volatile("v_smfmac_f32_32x32x64_bf8_fp8 a[%3:%4], %0, %1, %2"
                     :
                     : "v"(av), "v"(bv), "v"(idx), "n"(16 * T), "n"(16 * T + 15));
}

// Eight codes (a dword) -> eight E5M2 bytes: the integers -8 .. 7 as fp16 have nothing below their two
// top mantissa bits, so the E5M2 code of a value is the high byte of its fp16 code.
__device__ __forceinline__ uint2_t codes_to_e5m2x8(uint32_t q)
{
    const uint4_t h = __builtin_bit_cast(uint4_t, codes_to_half8(q));
    return uint2_t{__builtin_amdgcn_perm(h[1], h[0], 0x07050301u), __builtin_amdgcn_perm(h[3], h[2], 0x07050301u)};
}
// Half of that: codes 4 h .. 4 h + 3 of a dword already in offset-by-8 form (codes_bias()).
__device__ __forceinline__ uint32_t codes_to_e5m2x4(uint32_t biased, int h)
{
    const uint32_t p0 = __builtin_bit_cast(uint32_t, code_pair(biased, 2 * h));
    const uint32_t p1 = __builtin_bit_cast(uint32_t, code_pair(biased, 2 * h + 1));
    return __builtin_amdgcn_perm(p1, p0, 0x07050301u);
}

// AT row tiles of 32 per wavefront; accumulator tile (i, it) is a[16 (i NT + it) ..].
// XF: 0 = X in fp16; 1, 2 = X as 8-bit codes (E4M3, E5M2) with one scale for the tensor
// (App. "Input Quantization"): the weight term then runs on the 8-bit sparse instruction, 64 inputs
// per step, on half the bytes of X; the adapter term is unchanged (its T comes from the caller's
// fp16 copy of the quantized X).
template <int AT, int XF = 0>
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

    // AT = 4: workgroup b takes tile b.  AT = 2 (1): workgroup b takes the half
    // (quarter) b % split of tile n_full + b / split.
    const int b = blockIdx.x;
    constexpr int split = 4 / AT;
    const int w = tile_of_workgroup(a, (split > 1 ? a.n_full : 0) + b / split, split == 1);
    const int o0 = (w % a.tiles_o) * 512 + (b % split) * (4 * WROWS) + wave * WROWS;
    const int t0 = (w / a.tiles_o) * 128;
    const int t_end = min(a.m, t0 + 128);                    // tokens of this workgroup: [t0, t_end)

    acc_reserve<AT>();
    static_for<16 * AT * NT>([&](auto r) { acc_write<r>(0.0f); });

    const uint32_t k = (uint32_t)a.k;
    const int nsteps = a.k / SG_BK;

    // this lane's piece of row tile 0, stage 0 in the packed layout (one KiB of
    // codes, 512 bytes of positions per row tile and stage); tile i and stage s are
    // uniform terms; row tiles past the end read as zero
    const uint32_t qv = (uint32_t)(o0 / 32) * (k / 128) * 1024u + (uint32_t)(lb * 32 + li) * 16u;
    const uint32_t mv = (uint32_t)(o0 / 32) * (k / 128) * 512u + (uint32_t)(lb * 32 + li) * 8u;
    uint4_t qa[3][AT];
    uint2_t ma[3][AT];

    // X / T staging: 16 lanes per token row (256 contiguous bytes), 16 rows per pass
    const int srow = tid >> 4, scol = (tid & 15) * 8;
    const uint32_t xv = ((uint32_t)(t0 + srow) * k + (uint32_t)scol) * 2u;
    half_t *const lw = lds + srow * SG_LD + scol;
    uint4_t xr[2][XR];
    auto stage_store = [&](int u, const uint4_t (&reg)[XR], int only = -1) {
#pragma unroll
        for (int p = 0; p < XR; ++p)
            if (only < 0 || only == p) *reinterpret_cast<uint4_t *>(lw + u * SG_STAGE + p * 16 * SG_LD) = reg[p];
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
    // each matrix instruction, pinned there by scheduling barriers; the pieces
    // behind the last slice convert the first slice of the next stage (qn: its
    // codes, loaded a stage ago), so that no stage begins with a conversion.
    // a_cur: the first slice of this stage on entry, of the next stage on exit.
    // `fetch(bi)` is called once per block, bi = t NT + it, right after the
    // block's LDS reads: the place to issue a share of the next stages' loads.
    auto compute_stage = [&](int u, const uint4_t (&q)[AT], const uint4_t (&qn)[AT], const uint2_t (&mm)[AT],
                             half8_t (&a_cur)[AT], auto &&fetch) {
        half8_t a_nxt[AT];
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
                    {
                        // 4 AT pieces per slice over AT NT matrix instructions; the last slice converts the
                        // first one of the next stage
                        constexpr int pc = it * AT + i, tile = pc / 4, g = pc % 4;
                        if constexpr (tile < AT) {
                            const half2_t h = code_pair(codes_bias(t + 1 < 4 ? q[tile][(t + 1) & 3] : qn[tile][0]), g);
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

    if constexpr (XF != 0) {
        // ---- 8-bit inputs ----
        // A stage is 128 tokens x 128 inputs = 16 KiB in LDS, rows of 144 bytes.  Within a row the
        // inputs are stored in the order in which the lanes of the 8-bit instruction want them: for
        // step u (64 inputs of the stage) lane half h takes 32 contiguous bytes at 64 u + 32 h, the
        // inputs 32 u + 16 h + [0, 16) and 64 + 32 u + 16 h + [0, 16) -- the packed layout gives lane
        // half lb the inputs 16 t + 8 lb + [0, 8) and 64 + 16 t + 8 lb + [0, 8) of slice t, and a step is
        // two slices.  (Checked on the GPU with one-hot inputs.)  A staging thread moves 16 contiguous
        // bytes.
        constexpr int F8_LD = 144, F8_STAGE = 128 * F8_LD;
        unsigned char *const lds8 = reinterpret_cast<unsigned char *>(lds);
        const rsrc_t dq = make_rsrc(a.qvals, (uint32_t)pk_qbytes(a.n, a.k));
        const rsrc_t dm = make_rsrc(a.meta, (uint32_t)pk_mbytes(a.n, a.k));
        const rsrc_t dx = make_rsrc(a.X, (uint32_t)a.m * k);
        const int srow8 = tid >> 3, c16 = tid & 7;
        const uint32_t xv8 = (uint32_t)(t0 + srow8) * k + 16u * (uint32_t)c16;
        unsigned char *const lw8 = lds8 + srow8 * F8_LD + 64 * ((c16 & 3) >> 1) + 32 * (c16 & 1) + 16 * (c16 >> 2);
        const unsigned char *const lr8 = lds8 + li * F8_LD + 32 * lb;
        uint4_t x8[2][4];
        auto fetch_x8 = [&](int p, int s, uint4_t (&reg)[4]) {
            reg[p] = load16(dx, xv8, (uint32_t)s * 128u + (uint32_t)p * 32u * k);
        };
        auto stage_store8 = [&](int u, const uint4_t (&reg)[4]) {
#pragma unroll
            for (int p = 0; p < 4; ++p) *reinterpret_cast<uint4_t *>(lw8 + u * F8_STAGE + p * 32 * F8_LD) = reg[p];
        };
        auto read_b8 = [&](int ub, int u, int it) {
            const unsigned char *bp = lr8 + ub * F8_STAGE + it * 32 * F8_LD + 64 * u;
            const uint4_t b1 = *reinterpret_cast<const uint4_t *>(bp);
            const uint4_t b2 = *reinterpret_cast<const uint4_t *>(bp + 16);
            return int8v_t{(int)b1[0], (int)b1[1], (int)b1[2], (int)b1[3], (int)b2[0], (int)b2[1], (int)b2[2], (int)b2[3]};
        };
        auto fetch_a = [&](int j, int s, uint4_t (&q)[AT], uint2_t (&mm)[AT]) {    // j < 2 AT
            if (j < AT)
                q[j] = load16(dq, qv, ((uint32_t)j * (k / 128) + (uint32_t)s) * 1024u);
            else
                mm[j - AT] = load8(dm, mv, ((uint32_t)(j - AT) * (k / 128) + (uint32_t)s) * 512u);
        };
        // One stage = 2 steps (u) x NT token tiles: 2 NT blocks of AT matrix instructions.  Every matrix
        // instruction is followed by one piece of conversion (four codes -> four E5M2 bytes, 7 instructions):
        // during step 0 the pieces of this stage's step 1, during step 1 those of the next stage's step 0
        // (a0: this stage's step-0 operands on entry, the next stage's on exit), so that no conversion stands
        // between two stages.  qn: the codes of the next stage, loaded a stage ago.
        auto compute_stage8 = [&](int ub, const uint4_t (&q)[AT], const uint4_t (&qn)[AT], const uint2_t (&mm)[AT],
                                  int4_t (&a0)[AT], auto &&fetch) {
            int4_t a1[AT], an[AT];
            int8v_t b_cur = read_b8(ub, 0, 0), b_nxt = b_cur;
            static_for<2>([&](auto uc) {
                constexpr int u = uc;
                static_for<NT>([&](auto itc) {
                    constexpr int it = itc;
                    if (it + 1 < NT)
                        b_nxt = read_b8(ub, u, it + 1);
                    else if (u + 1 < 2)
                        b_nxt = read_b8(ub, u + 1, 0);
                    fetch(std::integral_constant<int, u * NT + it>{});
                    __builtin_amdgcn_sched_barrier(0);
                    static_for<AT>([&](auto ic) {
                        constexpr int i = ic;
                        smfmac8_fixed<i * NT + it, XF == 2>(u == 0 ? a0[i] : a1[i], b_cur, (int)mm[i][u]);
                        // 4 AT pieces over AT NT matrix instructions: piece `part` of a tile is half
                        // (part & 1) of code dword (part >> 1) of the step
                        constexpr int pc = it * AT + i, tile = pc / 4, part = pc % 4;
                        if constexpr (tile < AT) {
                            if constexpr (u == 0)
                                a1[tile][part] = (int)codes_to_e5m2x4(codes_bias(q[tile][2 + (part >> 1)]), part & 1);
                            else
                                an[tile][part] = (int)codes_to_e5m2x4(codes_bias(qn[tile][part >> 1]), part & 1);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    });
                    b_cur = b_nxt;
                });
                asm volatile("s_nop 3");       // the last piece is written right before the next step reads it
            });
#pragma unroll
            for (int i = 0; i < AT; ++i) a0[i] = an[i];
        };
        uint4_t qa8[3][AT];
        uint2_t ma8[3][AT];
#pragma unroll
        for (int p = 0; p < 4; ++p) fetch_x8(p, 0, x8[0]);
#pragma unroll
        for (int j = 0; j < 2 * AT; ++j) fetch_a(j, 0, qa8[0], ma8[0]);
#pragma unroll
        for (int p = 0; p < 4; ++p) fetch_x8(p, 1, x8[1]);
#pragma unroll
        for (int j = 0; j < 2 * AT; ++j) fetch_a(j, 1, qa8[1], ma8[1]);
        stage_store8(0, x8[0]);
        int4_t a0[AT];
#pragma unroll
        for (int i = 0; i < AT; ++i) {
            const uint2_t c0 = codes_to_e5m2x8(qa8[0][i][0]), c1 = codes_to_e5m2x8(qa8[0][i][1]);
            a0[i] = int4_t{(int)c0[0], (int)c0[1], (int)c1[0], (int)c1[1]};
        }
        __syncthreads();
        // weights two stages ahead in three register sets (stage s uses set s mod 3), X two stages ahead in two
        // sets and two LDS buffers (s mod 2): the loop body is written out for six stages
        for (int s0 = 0; s0 < nsteps; s0 += 6) {
            static_for<6>([&](auto vc) {
                constexpr int u = vc % 2, w = vc % 3, w1 = (vc + 1) % 3, w2 = (vc + 2) % 3;
                const int s = s0 + vc;
                if (s >= nsteps) return;
                compute_stage8(u, qa8[w], qa8[w1], ma8[w], a0, [&](auto bc) {
                    constexpr int bi = bc;           // 0 .. 2 NT - 1
                    if constexpr (bi < NT) {
                        constexpr int per = (2 * AT + NT - 1) / NT;      // weights of stage s + 2
#pragma unroll
                        for (int j = bi * per; j < (bi + 1) * per && j < 2 * AT; ++j)
                            fetch_a(j, s + 2, qa8[w2], ma8[w2]);
                    } else {
                        fetch_x8(bi - NT, s + 2, x8[u]);                 // X of stage s + 2: four loads
                    }
                });
                stage_store8(u ^ 1, x8[u ^ 1]);
                __syncthreads();
            });
        }
    } else {
    // The global loads are spread over the stage, one or two per block, so the
    // four wavefronts do not all queue sixteen loads at the address unit right
    // after the barrier (that burst stalled the first slice of every stage).
    // Weights of stage s + 2 go out in the first half of stage s; X of stage
    // s + 2 in the second half, to be written to LDS at the end of stage s + 1.
    // Fetches past the last stage stay inside the descriptors or read as zero and
    // are never used.
    {
        const rsrc_t dq = make_rsrc(a.qvals, (uint32_t)pk_qbytes(a.n, a.k));
        const rsrc_t dm = make_rsrc(a.meta, (uint32_t)pk_mbytes(a.n, a.k));
        const rsrc_t dx = make_rsrc(a.X, (uint32_t)a.m * k * 2);
        auto fetch_a = [&](int j, int s, uint4_t (&q)[AT], uint2_t (&mm)[AT]) {    // j < 2 AT
            if (j < AT)
                q[j] = load16(dq, qv, ((uint32_t)j * (k / 128) + (uint32_t)s) * 1024u);
            else
                mm[j - AT] = load8(dm, mv, ((uint32_t)(j - AT) * (k / 128) + (uint32_t)s) * 512u);
        };
        auto fetch_x = [&](int p, int s, uint4_t (&reg)[XR]) {
            reg[p] = load16(dx, xv, (uint32_t)s * (SG_BK * 2) + (uint32_t)p * 32u * k);
        };
#pragma unroll
        for (int p = 0; p < XR; ++p) fetch_x(p, 0, xr[0]);
#pragma unroll
        for (int j = 0; j < 2 * AT; ++j) fetch_a(j, 0, qa[0], ma[0]);
#pragma unroll
        for (int p = 0; p < XR; ++p) fetch_x(p, 1, xr[1]);
#pragma unroll
        for (int j = 0; j < 2 * AT; ++j) fetch_a(j, 1, qa[1], ma[1]);
        stage_store(0, xr[0]);
        half8_t a_first[AT];
#pragma unroll
        for (int i = 0; i < AT; ++i) a_first[i] = codes_to_half8(qa[0][i][0]);
        __syncthreads();
        // weights two stages ahead in three register sets (stage s uses set s mod 3), X two stages ahead in
        // two sets and two LDS buffers (s mod 2): the loop body is written out for six stages
        for (int s0 = 0; s0 < nsteps; s0 += 6) {
            static_for<6>([&](auto vc) {
                constexpr int u = vc % 2, w = vc % 3, w1 = (vc + 1) % 3, w2 = (vc + 2) % 3;
                const int s = s0 + vc;
                if (s >= nsteps) return;
                compute_stage(u, qa[w], qa[w1], ma[w], a_first, [&](auto bc) {
                    constexpr int bi = bc;
                    if constexpr (bi < HB) {
                        constexpr int per = (2 * AT + HB - 1) / HB;      // weights of stage s + 2
#pragma unroll
                        for (int j = bi * per; j < (bi + 1) * per && j < 2 * AT; ++j)
                            fetch_a(j, s + 2, qa[w2], ma[w2]);
                    } else {
                        constexpr int per = (XR + HB - 1) / HB;          // X of stage s + 2
#pragma unroll
                        for (int p = (bi - HB) * per; p < (bi - HB + 1) * per && p < XR; ++p) {
                            fetch_x(p, s + 2, xr[u]);
                            // X of stage s + 1 (loaded a stage ago) goes into the other LDS buffer, which nobody
                            // reads during this stage, piece by piece instead of in the stage's tail
                            *reinterpret_cast<uint4_t *>(lw + (u ^ 1) * SG_STAGE + p * 16 * SG_LD) = xr[u ^ 1][p];
                        }
                    }
                });
                __syncthreads();
            });
        }
    }

    }

    // row scale (times the scale of the 8-bit inputs): accumulator element 4 blk + e of tile i is row 32 i + 8 blk + 4 lb + e
    {
        float xs = 1.0f;
        if constexpr (XF != 0) xs = *a.x_scale;
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
                    const float sc = __builtin_bit_cast(float, sbits) * xs;
                    acc_write<16 * (i * NT + it) + e>(acc_read<16 * (i * NT + it) + e>() * sc);
                });
            });
        });
        acc_settle();
    }

    // adapter term: acc += L T^T as dense steps of 16 ranks; T staged like X; L in its
    // tiled layout: one contiguous KiB per row tile and step
    if (a.rank_pad > 0) {
        const uint32_t rp = (uint32_t)a.rank_pad;
        const rsrc_t dl = make_rsrc(a.L, a.L ? (uint32_t)tl_bytes(a.n, a.rank_pad) : 0u);
        const rsrc_t dt = make_rsrc(a.T, (uint32_t)a.m * rp * 2u);
        const uint32_t lv = tl_piece((uint32_t)o0 + li, lb, rp);
        const uint32_t tv = ((uint32_t)(t0 + srow) * rp + (uint32_t)scol) * 2u;
        if (a.Lq) {
            const Q4Rows lq = q4_rows_operand(a.Lq, a.Ls, a.n, a.rank, o0, li, lb, 0);
            dense_phase_q4<AT>(lq, dt, tv, 32u * rp, scol, (int)rp, lds + li * SG_LD + 32 * lb, xr[0], stage_store);
        } else {
            dense_phase<AT>(dl, lv, (rp / 16) * 1024u, 1024u, dt, tv, 32u * rp, (int)rp, lr, xr[0], stage_store);
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
// into quarters of 128 rows or halves of 256 rows (a second launch) when those
// fit into one round: more compute units busy for a shorter time.
static void plan_tiles(SparseGemmArgs &a, int slots)
{
    a.tiles_o = (a.n + 511) / 512;
    const int tiles_t = (a.m + 127) / 128;
    a.tiles_total = a.tiles_o * tiles_t;
    const int rem = a.tiles_total % slots;
    a.rem_split = 1;
    if (rem != 0 && 4 * rem <= slots)
        a.rem_split = 4;
    else if (rem != 0 && 2 * rem <= slots)
        a.rem_split = 2;
    a.n_full = a.rem_split > 1 ? a.tiles_total - rem : a.tiles_total;
    a.per_die = slots % kDies == 0 ? slots / kDies : 0;
}

// Buffer offsets are 32 bits wide: the caller has checked that the weight and
// adapter matrices stay below 4 GiB each; X, T and Y are walked in token chunks
// that do.
// xf: 0 = X fp16; 1, 2 = X as E4M3 / E5M2 codes (one byte per value) with the tensor's scale at x_scale
// L: fp16 [n][rank_pad] in the adapter layout, or null with Lq / Ls: the 4-bit codes and scales of L [n][rank]
int launch_gemm_sparse(const uint8_t *qvals, const uint8_t *meta, const float *scale, const half_t *X, const half_t *L,
                       const half_t *T, half_t *Y, int n, int k, int rank_pad, int m, hipStream_t st, int xf,
                       const float *x_scale, const uint8_t *Lq, const half_t *Ls, int rank)
{
    SparseGemmArgs a{};
    a.qvals = qvals;
    a.meta = meta;
    a.scale = scale;
    a.L = L;
    a.Lq = L ? nullptr : Lq;
    a.Ls = Ls;
    a.rank = rank;
    a.n = n;
    a.k = k;
    a.rank_pad = rank_pad;
    a.x_scale = x_scale;
    const size_t xbytes = xf ? 1 : 2;       // bytes per value of X
    const uint64_t row_bytes = 2ull * (uint64_t)(k > rank_pad ? k : rank_pad);
    const int chunk = (int)((0xFFFFFFFFull / row_bytes) / 128 * 128);
    if (chunk < 128) return SLIM_ERR_SHAPE;
    const size_t lds = (size_t)2 * SG_STAGE * sizeof(half_t);
    for (int t0 = 0; t0 < m; t0 += chunk) {
        a.m = m - t0 < chunk ? m - t0 : chunk;
        a.X = reinterpret_cast<const half_t *>(reinterpret_cast<const char *>(X) + (size_t)t0 * k * xbytes);
        a.T = T ? T + (size_t)t0 * rank_pad : nullptr;
        a.Y = Y + (size_t)t0 * n;
        plan_tiles(a, device_info().cus);
        const int n_rem = a.rem_split * (a.tiles_total - a.n_full);
        auto launch = [&](auto atc, unsigned grid) {
            constexpr int AT = decltype(atc)::value;
            if (xf == 0)
                hipLaunchKernelGGL((gemm_sparse_kernel<AT, 0>), dim3(grid), dim3(256), lds, st, a);
            else if (xf == 1)
                hipLaunchKernelGGL((gemm_sparse_kernel<AT, 1>), dim3(grid), dim3(256), lds, st, a);
            else
                hipLaunchKernelGGL((gemm_sparse_kernel<AT, 2>), dim3(grid), dim3(256), lds, st, a);
        };
        if (a.n_full > 0) launch(std::integral_constant<int, 4>{}, (unsigned)a.n_full);
        if (n_rem > 0 && a.rem_split == 2) launch(std::integral_constant<int, 2>{}, (unsigned)n_rem);
        if (n_rem > 0 && a.rem_split == 4) launch(std::integral_constant<int, 1>{}, (unsigned)n_rem);
    }
    return hip_status(hipGetLastError());
}

}  // namespace slim

using namespace slim;

extern "C" int slim_gemm_tile_order(int32_t n, int32_t m, int32_t *out, size_t count)
{
    if (!out) return SLIM_ERR_NULL;
    if (n < 1 || m < 1) return SLIM_ERR_SHAPE;
    SparseGemmArgs a{};
    a.n = n;
    a.m = m;
    plan_tiles(a, device_info().cus);
    if (count < (size_t)a.tiles_total + 2) return SLIM_ERR_SHAPE;
    out[0] = a.tiles_total;
    out[1] = a.n_full;
    for (int w = 0; w < a.tiles_total; ++w) out[2 + w] = tile_of_workgroup(a, w, w < a.n_full);
    return SLIM_OK;
}

