// slim_linear_gemv: decode-shaped forward (1 <= m <= 16 tokens), HBM-bound.
//
// Two launches; the kernel boundary is the only device-wide synchronisation
// (an in-kernel wait of all blocks on one counter was measured at about 18 us
// on this eight-die part, a launch boundary costs about 3 us).
//
//  part 1  A wavefront owns "units" of 16 rows x a slice of inputs, streams
//          them with 128-bit loads straight into registers, and feeds the
//          matrix cores with the tokens as the 16 columns of the B operand.
//          Rows are the packed weight rows AND the rank_pad rows of R (the
//          adapter stage T = X R^T is just more output rows of the same X):
//           - packed rows: the two int4 codes of a group become two fp16
//             values in registers and go, with the group's 2-bit position
//             pair as the index operand, into the structured-sparse matrix
//             instruction (V_SMFMAC_F32_16X16X64_F16), which picks the
//             matching X values itself: the canonical metadata bytes are
//             exactly that instruction's index format;
//           - R rows: dense fp16 matrix instruction.
//          X (the block's k-chunk of it) sits in LDS in fp16, zero-padded to
//          whole units and with one extra all-zero row that the lanes of
//          unused token columns read, so the inner loop has no branches.
//          A packed-row task writes partial sums to P[slot][token][row]; an R
//          unit adds its partial sums to T with fp32 atomics.  The loads of
//          the next unit are in flight while the current one is computed.
//  part 2  Y[t][o] = fp16(scale[o] * sum_slot P[slot][t][o] + sum_j T[t][j] L[o][j]):
//          L rows stream through the dense matrix instruction against T held
//          in LDS as an fp16 hi/lo pair (T keeps fp32 accuracy).
//
// All operands are read in their tiled layouts: a load instruction of a
// wavefront covers four runs of 256 contiguous bytes (R, L, codes) or of 128
// (positions).
//
// Nothing is carried between calls: T (fp32 [16][rank_pad] in the head of the
// workspace) is zeroed by a small kernel ahead of part 1, which adds into it.
// (Earlier the calls cleaned a second T buffer for one another; that breaks as
// soon as layers of different rank share a workspace.)
#include <atomic>
#include <cstdlib>
#include <cstring>

#include "slim_decode.h"

namespace slim {

constexpr int kDecThreads = 256;
constexpr int kDecWaves = kDecThreads / kWave;
constexpr int kLdsBudget = 72 * 1024;      // bytes of LDS per block: two blocks per CU
constexpr int kUnitK = 1024;               // inputs per packed-row unit
constexpr int kUnitR = 256;                // inputs per R unit

struct DecodeArgs {
    const uint8_t *qvals;
    const uint8_t *meta;
    const float *scale;
    const half_t *R;
    const half_t *L;
    const half_t *X;
    half_t *Y;
    float *P;            // [slots][m][n]; nullptr: no packed term (slim_lowrank)
    float *T;            // two buffers of [16][rank_pad] fp32
    unsigned *ctrl;      // control words of the workspace (not used by these kernels)
    int n, k, rank_pad, m;
    int mp;              // token rows of the LDS tiles (1, 4, 8 or 16) before the zero row
    int n_packed;        // rows with a packed term in part 1 (n, or 0)
    int kc;              // inputs per chunk (multiple of kUnitK)
    int nch;             // number of chunks
    int sl;              // inputs per packed-row task (multiple of kUnitK)
    int rsl;             // inputs per R task (multiple of kUnitR): fewer, larger atomic updates of T
    int wsl_full;        // tasks per row tile in a full chunk
    int slots;           // total partial slots
    int accumulate;      // slim_lowrank only: add the fp16 value already in Y
};

// One unit of part 1: which rows, which inputs, and where its task stands.
struct Unit {
    int q;         // task index within this wave's chunk (-1: none)
    int u;         // unit within the task
    int tile;      // row tile (16 rows)
    int k0;        // first input, chunk-relative
    int k1;        // end of the inputs of this unit, chunk-relative
    int slot_s;    // packed rows: slice index of the task in the chunk
    bool is_r;
    bool last;     // last unit of its task
};

// Geometry of part 1 for one block (one k-chunk).
struct Part1Geom {
    int kbeg, klen, rsub, n_rtasks, wsl, n_tasks, gstride;
};

__device__ __forceinline__ Unit describe_unit(const DecodeArgs &a, const Part1Geom &g, int q, int u)
{
    Unit d;
    d.q = q;
    d.u = u;
    d.tile = d.k0 = d.k1 = d.slot_s = 0;
    d.is_r = false;
    d.last = true;
    if (q >= g.n_tasks) {
        d.q = -1;
    } else if (q < g.n_rtasks) {
        d.is_r = true;
        d.tile = q / g.rsub;
        const int t0 = (q - d.tile * g.rsub) * a.rsl;
        const int t1 = min(g.klen, t0 + a.rsl);
        d.k0 = t0 + u * kUnitR;
        d.k1 = min(t1, d.k0 + kUnitR);
        d.last = d.k0 + kUnitR >= t1;
    } else {
        const int qq = q - g.n_rtasks;
        d.tile = qq / g.wsl;
        d.slot_s = qq - d.tile * g.wsl;
        const int t0 = d.slot_s * a.sl;
        const int t1 = min(g.klen, t0 + a.sl);
        d.k0 = t0 + u * kUnitK;
        d.k1 = min(t1, d.k0 + kUnitK);
        d.last = d.k0 + kUnitK >= t1;
    }
    return d;
}

// Loads of one unit: up to 8 x 128 bit per lane.
//  R unit:      8 inputs of row lx per matrix step (8 steps of 32 inputs)
//  packed unit: per 512 inputs (two halves per unit): 2 quads of codes, 1 of
//               positions, for the lane's 128 inputs of row lx
// Whatever lies beyond the end of the unit's inputs or rows is loaded as zero.
__device__ __forceinline__ void issue_unit(const DecodeArgs &a, const Part1Geom &g, const Unit &d, int lx, int ly,
                                           UnitRegs &b)
{
    const uint4_t zero = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < 8; ++i) b.r[i] = zero;      // every register defined on every path
    if (d.q < 0) return;
    if (d.is_r) {
        // R in its tiled layout: step t reads the pieces (row, 4 t + ly) of the unit,
        // four runs of 256 contiguous bytes per load instruction
        const char *base = reinterpret_cast<const char *>(a.R) +
                           tl_piece(16u * d.tile + lx, (uint32_t)(g.kbeg + d.k0) / 8 + ly, (uint32_t)a.k);
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const bool valid = d.k0 + 32 * t < d.k1;
            b.r[t] = valid ? *reinterpret_cast<const uint4_t *>(base + 2048 * t) : zero;     // 4 pieces = 2 tiles on
        }
    } else {
        const int o = 16 * d.tile + lx;
        const bool rowok = o < a.n_packed;
        const size_t row = rowok ? o : 0;
        const int kl0 = d.k0 + 128 * ly;
        const int kl1 = kl0 + 512;
        const bool valid0 = rowok && kl0 < d.k1;
        const bool valid1 = rowok && kl1 < d.k1;
        const int kg0 = g.kbeg + (valid0 ? kl0 : 0);
        const int kg1 = g.kbeg + (valid1 ? kl1 : 0);
        // The lane's 128 inputs are one tile column of the packed layout: its two
        // pieces of codes lie 512 bytes apart, its two pieces of positions 256.
        const uint32_t kt = pk_ktiles(a.k);
        const uint8_t *qp0 = a.qvals + pk_qoff((uint32_t)row, (uint32_t)kg0 / 4, kt);
        const uint8_t *mp0 = a.meta + pk_moff((uint32_t)row, (uint32_t)kg0 / 8, kt);
        const uint8_t *qp1 = a.qvals + pk_qoff((uint32_t)row, (uint32_t)kg1 / 4, kt);
        const uint8_t *mp1 = a.meta + pk_moff((uint32_t)row, (uint32_t)kg1 / 8, kt);
        auto q16 = [](const uint8_t *p) { return *reinterpret_cast<const uint4_t *>(p); };
        auto m16 = [](const uint8_t *p) {
            const uint2_t lo = *reinterpret_cast<const uint2_t *>(p), hi = *reinterpret_cast<const uint2_t *>(p + 256);
            return uint4_t{lo[0], lo[1], hi[0], hi[1]};
        };
        b.r[0] = valid0 ? q16(qp0) : zero;
        b.r[1] = valid0 ? q16(qp0 + 512) : zero;
        b.r[2] = valid0 ? m16(mp0) : zero;
        b.r[3] = valid1 ? q16(qp1) : zero;
        b.r[4] = valid1 ? q16(qp1 + 512) : zero;
        b.r[5] = valid1 ? m16(mp1) : zero;
    }
}

// ---- part 1: packed rows -> P, R rows -> T (atomics) ----
__global__ __launch_bounds__(kDecThreads, 2) __attribute__((amdgpu_waves_per_eu(2, 2))) void decode_part1_kernel(DecodeArgs a)
{
    extern __shared__ __attribute__((aligned(16))) half_t lds[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int lx = lane & 15;       // A-operand row / B-operand token
    const int ly = lane >> 4;       // k-block of the lane
    const int chunk = blockIdx.x % a.nch;
    const int rp = a.rank_pad;
    const int ldx = a.kc + kLdsPad;

    Part1Geom g;
    g.kbeg = chunk * a.kc;
    g.klen = min(a.k, g.kbeg + a.kc) - g.kbeg;
    g.rsub = (g.klen + a.rsl - 1) / a.rsl;
    g.n_rtasks = (rp / 16) * g.rsub;
    g.wsl = (g.klen + a.sl - 1) / a.sl;
    g.n_tasks = g.n_rtasks + ((a.n_packed + 15) / 16) * g.wsl;
    g.gstride = (gridDim.x / a.nch) * kDecWaves;

    // first loads go out before anything else
    UnitRegs bufA, bufB;
    Unit cur = describe_unit(a, g, (blockIdx.x / a.nch) * kDecWaves + wave, 0);
    issue_unit(a, g, cur, lx, ly, bufA);

    // T of this call: zeroed ahead of this kernel
    float *Tcur = a.T;

    // stage this chunk of X: mp token rows (rows >= m zero), inputs beyond the
    // chunk zero up to kc, then one all-zero row
    // (loads are issued in batches of 8 per lane before the LDS stores, so the
    // copy costs a few memory round trips, not one per element)
    {
        const int per_row = a.kc / 8;                       // 128-bit pieces per row
        const int total = (a.mp + 1) * per_row;
        for (int e0 = threadIdx.x; e0 < total; e0 += 8 * kDecThreads) {
            uint4_t v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + i * kDecThreads;
                const int row = e / per_row, c = e - row * per_row;
                v[i] = uint4_t{0u, 0u, 0u, 0u};
                if (e < total && row < a.m && c * 8 < g.klen)
                    v[i] = *reinterpret_cast<const uint4_t *>(a.X + (size_t)row * a.k + g.kbeg + c * 8);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + i * kDecThreads;
                const int row = e / per_row, c = e - row * per_row;
                if (e < total) *reinterpret_cast<uint4_t *>(lds + row * ldx + c * 8) = v[i];
            }
        }
    }
    __syncthreads();

    // this lane's B-operand row: its token, or the zero row
    const half_t *xrow = lds + (lx < a.mp ? lx : a.mp) * ldx;
    const half_t *xrow_packed = xrow + 128 * (ly >> 1) + 8 * (ly & 1);
    const half_t *xrow_r = xrow + 8 * ly;
    float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = acc0;
    while (cur.q >= 0) {
        const Unit nxt = cur.last ? describe_unit(a, g, cur.q + g.gstride, 0) : describe_unit(a, g, cur.q, cur.u + 1);
        issue_unit(a, g, nxt, lx, ly, bufB);
        if (cur.is_r) {
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const half8_t bv = *reinterpret_cast<const half8_t *>(xrow_r + cur.k0 + 32 * t);
                const half8_t av = __builtin_bit_cast(half8_t, bufA.r[t]);
                if (t & 1)
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc1, 0, 0, 0);
                else
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc0, 0, 0, 0);
            }
        } else {
            packed_half<0>(bufA, xrow_packed + cur.k0, acc0, acc1);
            packed_half<1>(bufA, xrow_packed + cur.k0 + 512, acc0, acc1);
        }
        if (cur.last) {
            // lane holds token lx, rows 16 tile + 4 ly .. + 3
            const float4_t acc = acc0 + acc1;
            acc0 = float4_t{0.f, 0.f, 0.f, 0.f};
            acc1 = acc0;
            if (lx < a.m) {
                if (cur.is_r) {
                    float *tp = Tcur + (size_t)lx * rp + 16 * cur.tile + 4 * ly;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        __hip_atomic_fetch_add(tp + v, acc[v], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    const int slot = chunk * a.wsl_full + cur.slot_s;
                    const int ob = 16 * cur.tile + 4 * ly;
                    float *pp = a.P + ((size_t)slot * a.m + lx) * a.n + ob;
                    if (ob + 3 < a.n && (a.n & 3) == 0) {
                        *reinterpret_cast<float4_t *>(pp) = acc;
                    } else {
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (ob + v < a.n) pp[v] = acc[v];
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) bufA.r[i] = bufB.r[i];
        cur = nxt;
    }

}

// ---- part 2: Y = scale * sum P + T L^T ----
// Sixteen wavefronts per workgroup: four tiles of 16 output rows at a time, and
// the ranks of each tile dealt out to four wavefronts (wavefront sp takes the
// steps of 32 ranks sp, sp + 4, ...), so a layer with few row tiles still puts
// enough loads in flight to stream L at memory speed.  The three partial sums
// meet the first wavefront of the tile in LDS.  NB = 128-bit L loads a lane issues at
// once (one per step); the next batch, or the first of the next tile, is in
// flight during the matrix work.
constexpr int kP2Waves = 16;
constexpr int kP2Threads = kP2Waves * kWave;
constexpr int kP2Split = 4;                          // wavefronts per tile
constexpr int kP2Tiles = kP2Waves / kP2Split;        // tiles per workgroup and round
constexpr int kP2RedBytes = 2 * kP2Tiles * (kP2Split - 1) * kWave * 16;   // two alternating sets of partial sums

template <int NB>
__global__ __launch_bounds__(kP2Threads, 1) void decode_part2_kernel(DecodeArgs a)
{
    extern __shared__ __attribute__((aligned(16))) half_t lds[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int ts = wave / kP2Split;      // tile slot of this wavefront
    const int sp = wave % kP2Split;      // its share of the ranks
    const int lx = lane & 15;
    const int ly = lane >> 4;
    const int rp = a.rank_pad;
    const int wtiles = (a.n + 15) / 16;
    const int steps = rp / 32;
    const int cnt = (steps - sp + kP2Split - 1) / kP2Split;          // steps of this wavefront (sp < steps or 0)
    const int nbatch = cnt > 0 ? (cnt + NB - 1) / NB : 0;
    const int tile0 = blockIdx.x * kP2Tiles + ts;
    const int tstride = gridDim.x * kP2Tiles;
    const int rounds = (wtiles - blockIdx.x * kP2Tiles + tstride - 1) / tstride;   // same for the whole workgroup

    // L of the first tile goes out first: it does not depend on T
    uint4_t lvA[NB], lvB[NB];
    auto issue_l = [&](int ot, int batch, uint4_t (&lv)[NB]) {
        const int o = 16 * ot + lx;
        const bool rowok = batch < nbatch && ot < wtiles && o < a.n;
        // step t = sp + 4 (batch NB + x) takes ranks 32 t + 8 ly .. + 7 of row o: piece (o, 4 t + ly)
        // of the tiled layout; consecutive steps of this wavefront lie 8 KiB apart
        const int tb = sp + kP2Split * (rowok ? batch : 0) * NB;
        const char *lp = reinterpret_cast<const char *>(a.L) + tl_piece((uint32_t)(rowok ? o : 0), 4u * tb + ly, (uint32_t)rp);
#pragma unroll
        for (int x = 0; x < NB; ++x) {
            const bool ok = rowok && tb + kP2Split * x < steps;
            lv[x] = ok ? *reinterpret_cast<const uint4_t *>(lp + 2048 * kP2Split * x) : uint4_t{0u, 0u, 0u, 0u};
        }
    };
    if (nbatch > 0) issue_l(tile0, 0, lvA);

    const float *T0 = a.T;

    // T -> LDS as fp16 hi + lo, mp token rows then one zero row
    const int ldt = rp + kLdsPad;
    half_t *t_hi = lds;
    half_t *t_lo = lds + (a.mp + 1) * ldt;
    float *red = reinterpret_cast<float *>(lds + 2 * (a.mp + 1) * ldt);
    if (rp > 0) {
        // 4 ranks per piece, up to 4 pieces per lane in flight before the LDS stores
        const int per_row = rp / 4;
        const int total = (a.mp + 1) * per_row;
        for (int e0 = threadIdx.x; e0 < total; e0 += 4 * kP2Threads) {
            float4_t v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = e0 + i * kP2Threads;
                const int row = e / per_row, c = e - row * per_row;
                v[i] = float4_t{0.f, 0.f, 0.f, 0.f};
                if (e < total && row < a.m)
                    v[i] = *reinterpret_cast<const float4_t *>(T0 + (size_t)row * rp + 4 * c);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = e0 + i * kP2Threads;
                const int row = e / per_row, c = e - row * per_row;
                if (e < total) {
                    half4_t hi, lo;
#pragma unroll
                    for (int x = 0; x < 4; ++x) {
                        hi[x] = (half_t)v[i][x];
                        lo[x] = (half_t)(v[i][x] - (float)hi[x]);
                    }
                    *reinterpret_cast<half4_t *>(t_hi + row * ldt + 4 * c) = hi;
                    *reinterpret_cast<half4_t *>(t_lo + row * ldt + 4 * c) = lo;
                }
            }
        }
    }
    __syncthreads();
    const int trow = lx < a.mp ? lx : a.mp;
    const half_t *th = t_hi + trow * ldt + 8 * ly;
    const half_t *tl = t_lo + trow * ldt + 8 * ly;

    for (int round = 0; round < rounds; ++round) {
        const int ot = tile0 + round * tstride;          // may lie past the last tile: then nothing is loaded or stored
        float4_t acc = {0.f, 0.f, 0.f, 0.f}, accb = acc;
        const int ob = 16 * ot + 4 * ly;
        const bool vec = (ob + 3 < a.n) && (a.n & 3) == 0;
        // packed term of this lane's 4 outputs (first wavefront of the tile): its
        // loads go out before the matrix work
        float q[4] = {0.f, 0.f, 0.f, 0.f};
        float sc[4] = {0.f, 0.f, 0.f, 0.f};
        if (sp == 0 && a.P && lx < a.m && ot < wtiles) {
            for (int slot = 0; slot < a.slots; ++slot) {
                const float *pp = a.P + ((size_t)slot * a.m + lx) * a.n + ob;
                if (vec) {
                    const float4_t p4 = *reinterpret_cast<const float4_t *>(pp);
#pragma unroll
                    for (int v = 0; v < 4; ++v) q[v] += p4[v];
                } else {
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (ob + v < a.n) q[v] += pp[v];
                }
            }
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (ob + v < a.n) sc[v] = a.scale[ob + v];
        }
        for (int batch = 0; batch < nbatch; ++batch) {
            // next batch (of this tile or the first of the next tile) while this one is used
            if (batch + 1 < nbatch)
                issue_l(ot, batch + 1, lvB);
            else
                issue_l(ot + tstride, 0, lvB);
#pragma unroll
            for (int x = 0; x < NB; ++x) {
                // steps past the end carry zero L values and read T inside the padded row
                const int t = min(sp + kP2Split * (batch * NB + x), steps - 1);
                const half8_t bh = *reinterpret_cast<const half8_t *>(th + 32 * t);
                const half8_t bl = *reinterpret_cast<const half8_t *>(tl + 32 * t);
                const half8_t av = __builtin_bit_cast(half8_t, lvA[x]);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bh, acc, 0, 0, 0);
                accb = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bl, accb, 0, 0, 0);
            }
#pragma unroll
            for (int x = 0; x < NB; ++x) lvA[x] = lvB[x];
        }
        acc += accb;
        // partial sums of the other three wavefronts of the tile (alternating sets,
        // so one barrier per round is enough)
        float *rset = red + (size_t)((round & 1) * kP2Tiles + ts) * (kP2Split - 1) * kWave * 4;
        if (sp != 0) *reinterpret_cast<float4_t *>(rset + ((sp - 1) * kWave + lane) * 4) = acc;
        __syncthreads();
        if (sp == 0 && lx < a.m && ot < wtiles) {
#pragma unroll
            for (int w = 0; w < kP2Split - 1; ++w) acc += *reinterpret_cast<const float4_t *>(rset + (w * kWave + lane) * 4);
            half_t *yp = a.Y + (size_t)lx * a.n + ob;
            float y[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                y[v] = acc[v] + sc[v] * q[v];
                if (a.accumulate && ob + v < a.n) y[v] += (float)yp[v];
            }
            if (vec) {
                half4_t h = {(half_t)y[0], (half_t)y[1], (half_t)y[2], (half_t)y[3]};
                *reinterpret_cast<half4_t *>(yp) = h;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (ob + v < a.n) yp[v] = (half_t)y[v];
            }
        }
    }
}

static int pad_tokens(int m) { return m <= 1 ? 1 : (m <= 4 ? 4 : (m <= 8 ? 8 : 16)); }

// Chunk and slice geometry for a decode call (host side).
DecodePlan plan_decode(int n, int k, int rank_pad, int m)
{
    DecodePlan p{};
    p.mp = pad_tokens(m);
    // largest chunk (whole units) whose X tile, with its zero row, fits the LDS budget
    int kc_max = (kLdsBudget / (2 * (p.mp + 1)) - kLdsPad) / kUnitK * kUnitK;
    if (kc_max < kUnitK) kc_max = kUnitK;
    const int kpad = (k + kUnitK - 1) / kUnitK * kUnitK;
    p.kc = kpad < kc_max ? kpad : kc_max;
    p.nch = (k + p.kc - 1) / p.kc;
    // Every chunk gets the same number of workgroups, so chunks should be equal:
    // of the chunk counts nch .. nch + 2 take the one that wastes the fewest units.
    {
        const int units = kpad / kUnitK;
        int best = p.nch, best_waste = 1 << 30;
        for (int c = p.nch; c <= p.nch + 2 && c <= units; ++c) {
            const int waste = c * ((units + c - 1) / c) - units;
            if (waste < best_waste) {
                best_waste = waste;
                best = c;
            }
        }
        p.kc = ((units + best - 1) / best) * kUnitK;
        p.nch = (k + p.kc - 1) / p.kc;
    }
    // inputs per packed-row task: one unit for small layers (more tasks in
    // flight), more for large ones (fewer partial slots to write and re-read)
    const long tiles = (n + 15) / 16;
    int sl = kUnitK;
    while (sl < p.kc && tiles * ((k + sl - 1) / sl) > 8192) sl *= 2;
    p.sl = sl;
    // R tasks: every task ends in one fp32 atomic per T element it touches, and
    // those go to memory, so with many tokens take 4 units per task
    // (only when there is enough work that waves run several tasks anyway).
    const long small_tasks = tiles * ((k + sl - 1) / sl) + (long)(rank_pad / 16) * ((k + kUnitR - 1) / kUnitR);
    p.rsl = (p.mp > 4 && small_tasks > 4096) ? 4 * kUnitR : kUnitR;
    p.wsl_full = (p.kc + sl - 1) / sl;
    const int klast = k - (p.nch - 1) * p.kc;
    p.slots = (p.nch - 1) * p.wsl_full + (klast + sl - 1) / sl;
    return p;
}

__global__ void decode_zero_t_kernel(float *T, int count)
{
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < count; i += gridDim.x * blockDim.x) T[i] = 0.0f;
}

static int launch_decode(const DecodeArgs &a, const DecodePlan &p, hipStream_t st)
{
    const size_t lds1 = (size_t)(p.mp + 1) * (p.kc + kLdsPad) * sizeof(half_t);
    const size_t lds2 = (size_t)2 * (p.mp + 1) * (a.rank_pad + kLdsPad) * sizeof(half_t) + kP2RedBytes;
    const DeviceInfo dev = device_info();
    if (lds1 > dev.lds || lds2 > dev.lds) return SLIM_ERR_SHAPE;
    const long units_r = (long)(a.rank_pad / 16) * ((p.kc + p.rsl - 1) / p.rsl);
    const long tasks_w = (long)((a.n_packed + 15) / 16) * p.wsl_full;
    // blocks per chunk: at most about four per CU, and such that every wave gets
    // the same number of tasks
    const long tasks = units_r + tasks_w;
    long resident = (long)dev.lds / (long)(lds1 > 0 ? lds1 : 1);    // blocks of this LDS size a CU holds
    if (resident > 4) resident = 4;
    if (resident < 1) resident = 1;
    const long cap = dev.cus * resident / p.nch > 0 ? dev.cus * resident / p.nch : 1;
    const long per_wave = (tasks + cap * kDecWaves - 1) / (cap * kDecWaves);
    long b1 = (tasks + per_wave * kDecWaves - 1) / (per_wave * kDecWaves);
    if (b1 < 1) b1 = 1;
    if (a.rank_pad > 0) {
        const int count = kMaxTokens * a.rank_pad;
        hipLaunchKernelGGL(decode_zero_t_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, st, a.T, count);
    }
    if (units_r + tasks_w > 0)
        hipLaunchKernelGGL(decode_part1_kernel, dim3((unsigned)(b1 * p.nch)), dim3(kDecThreads), lds1, st, a);
    long b2 = ((a.n + 15) / 16 + kP2Tiles - 1) / kP2Tiles;
    if (b2 > 512) b2 = 512;
    // L loads per lane and batch: the steps of 32 ranks are dealt out to 4 wavefronts
    const int l_loads = (a.rank_pad / 32 + kP2Split - 1) / kP2Split;
    const dim3 g2((unsigned)b2), blk(kP2Threads);
    if (l_loads > 4)
        hipLaunchKernelGGL(decode_part2_kernel<7>, g2, blk, lds2, st, a);
    else if (l_loads > 2)
        hipLaunchKernelGGL(decode_part2_kernel<4>, g2, blk, lds2, st, a);
    else
        hipLaunchKernelGGL(decode_part2_kernel<2>, g2, blk, lds2, st, a);
    return hip_status(hipGetLastError());
}

static void fill_plan(DecodeArgs &a, const DecodePlan &p)
{
    a.mp = p.mp;
    a.kc = p.kc;
    a.nch = p.nch;
    a.sl = p.sl;
    a.rsl = p.rsl;
    a.wsl_full = p.wsl_full;
    a.slots = p.slots;
}

// The one-launch kernel without its packed items where the geometry allows it (slim_decode_override with
// path 0 keeps the two-part kernels, as for slim_linear_gemv); T16: the one-launch path's pieces of T.
int launch_lowrank_decode(const half_t *X, int m, const half_t *R, const half_t *L, int n, int k, int rank, int rank_pad,
                          half_t *Y, int accumulate, float *T, void *T16, unsigned *ctrl, hipStream_t st)
{
    {
        const FusedPlan f = plan_fused(n, k, rank_pad, m);
        if (f.ok && f.n_r > 0 && decode_path_override() != 0) {
            slim_layer lay{};
            lay.shape = slim_shape{n, k, rank};
            lay.L = reinterpret_cast<const slim_half *>(L);
            lay.R = reinterpret_cast<const slim_half *>(R);
            lay.rank_pad = rank_pad;
            lay.adapter_bits = 16;
            return launch_decode_fused(&lay, X, m, Y, T16, ctrl + 2, ctrl + 3, f, 2, st, accumulate ? 2 : 1);
        }
    }
    DecodePlan p = plan_decode(n, k, rank_pad, m);
    DecodeArgs a{};
    a.R = R;
    a.L = L;
    a.X = X;
    a.Y = Y;
    a.T = T;
    a.ctrl = ctrl;
    a.n = n;
    a.k = k;
    a.rank_pad = rank_pad;
    a.m = m;
    a.n_packed = 0;
    fill_plan(a, p);
    a.slots = 0;
    a.accumulate = accumulate;
    return launch_decode(a, p, st);
}

}  // namespace slim

using namespace slim;

// Scratch of slim_linear_gemv_static: the workspace of a decode call inside the library's own
// code object, one copy per GPU, zero at load time (a zero-filled workspace is what the decode
// kernels expect before their first call) and held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress; kernels and copies get the address it returns.
static __device__ __align__(256) unsigned char scratch[SLIM_STATIC_SCRATCH_BYTES];

namespace slim {

constexpr int kMaxDevices = 64;
static std::atomic<void *> g_scratch_ptr[kMaxDevices];

// Address of `scratch` on the current device, looked up once per device.
int scratch_of_current_device(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SLIM_ERR_HIP;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return SLIM_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);     // every thread finds the same address
    }
    *out = p;
    return SLIM_OK;
}

// 2: one launch, 1: its roles as two launches, 3: the Y role alone (test of the bounded wait), -1: the two-launch kernels
static int decode_mode(const FusedPlan &f)
{
    const int forced = decode_path_override();
    if (!f.ok || forced == 0) return -1;
    return forced == 1 ? 1 : (forced == 3 ? 3 : 2);
}

// The decode kernels address every buffer with 32-bit byte offsets and use 2^31 as "past the end".
static bool decode_buffers_addressable(int n, int k, int rank_pad, int m)
{
    const uint64_t lim = 0x80000000ull;
    return pk_qbytes(n, k) < lim && tl_bytes(n, rank_pad) < lim && tl_bytes(rank_pad, k) < lim &&
           (uint64_t)m * (uint64_t)k * 2 < lim && (uint64_t)m * (uint64_t)n * 2 < lim;
}

// own_scratch: the workspace is the library's array; it has to hold what the chosen path uses
// (the caller's has to hold slim_workspace_bytes, whatever the path).
static int linear_gemv(const slim_layer *layer_in, const slim_half *X, int32_t m, slim_half *Y, void *workspace,
                       size_t workspace_bytes, void *stream, bool own_scratch);

}  // namespace slim

extern "C" int slim_linear_gemv(const slim_layer *layer, const slim_half *X, int32_t m, slim_half *Y, void *workspace,
                                size_t workspace_bytes, void *stream)
{
    return linear_gemv(layer, X, m, Y, workspace, workspace_bytes, stream, false);
}

extern "C" int slim_linear_gemv_static(const slim_layer *layer, const slim_half *X, int32_t m, slim_half *Y, void *stream)
{
    // arguments and size are checked on the host first; the array's address is looked up after that
    return linear_gemv(layer, X, m, Y, nullptr, (size_t)SLIM_STATIC_SCRATCH_BYTES, stream, true);
}

int slim::linear_gemv(const slim_layer *layer_in, const slim_half *X, int32_t m, slim_half *Y, void *workspace,
                      size_t workspace_bytes, void *stream, bool own_scratch)
{
    if (!layer_in || !X || !Y) return SLIM_ERR_NULL;
    const slim_layer *layer = layer_in;
    const slim_shape s = layer->shape;
    if (!layer->qvals || !layer->meta || !layer->scale) return SLIM_ERR_NULL;
    const bool q4 = layer->adapter_bits == 4 && s.rank > 0;
    if (q4 && (!layer->Lq || !layer->Ls || !layer->Rq || !layer->Rs)) return SLIM_ERR_NULL;
    if (!q4 && s.rank > 0 && (!layer->L || !layer->R)) return SLIM_ERR_NULL;
    if (s.n < 1 || s.k < 128 || s.k % 128 || s.rank < 0 || m < 1 || m > kMaxTokens) return SLIM_ERR_SHAPE;
    if (layer->rank_pad != slim_rank_pad(s.rank)) return SLIM_ERR_SHAPE;
    if (!decode_buffers_addressable(s.n, s.k, layer->rank_pad, m)) return SLIM_ERR_SHAPE;
    if (!aligned16(layer->qvals) || !aligned16(layer->meta) || !aligned16(layer->scale) || !aligned16(X) ||
        !aligned16(Y) || (!q4 && (!aligned16(layer->L) || !aligned16(layer->R))) || !aligned16(workspace))
        return SLIM_ERR_ALIGN;
    if (q4 && (!aligned16(layer->Lq) || !aligned16(layer->Ls) || !aligned16(layer->Rq) || !aligned16(layer->Rs)))
        return SLIM_ERR_ALIGN;
    WorkspacePlan w = plan_workspace(s.n, s.k, layer->rank_pad, m, q4);
    if (!own_scratch && (!workspace || workspace_bytes < w.total)) return SLIM_ERR_WORKSPACE;

    char *ws = nullptr;
    // Path: one launch where X fits the LDS of a compute unit, else the two-part
    // kernels; slim_decode_override forces one (tests, measurement).
    {
        const FusedPlan f = plan_fused(s.n, s.k, layer->rank_pad, m);
        const int mode = decode_mode(f);
        // the one-launch kernel uses the head of the workspace only (control words and T)
        if (own_scratch) {
            if (workspace_bytes < (mode > 0 ? w.dec_off + w.dec_bytes : w.total)) return SLIM_ERR_WORKSPACE;
            const int rc = scratch_of_current_device(&workspace);
            if (rc != SLIM_OK) return rc;
        }
        ws = static_cast<char *>(workspace);
        if (mode > 0)
            return launch_decode_fused(layer, reinterpret_cast<const half_t *>(X), m, reinterpret_cast<half_t *>(Y),
                                       ws + w.t16_off, reinterpret_cast<unsigned *>(ws + w.dec_off) + 2,
                                       reinterpret_cast<unsigned *>(ws + w.dec_off) + 3, f, mode,
                                       static_cast<hipStream_t>(stream));
    }
    // the two-launch kernels read fp16 adapters: 4-bit ones are expanded in the workspace first
    slim_layer expanded;
    if (q4) {
        const int rc = expand_q4_adapters(layer, w, ws, &expanded, static_cast<hipStream_t>(stream));
        if (rc != SLIM_OK) return rc;
        layer = &expanded;
    }
    DecodePlan p = plan_decode(s.n, s.k, layer->rank_pad, m);
    DecodeArgs a{};
    a.qvals = layer->qvals;
    a.meta = layer->meta;
    a.scale = layer->scale;
    a.R = reinterpret_cast<const half_t *>(layer->R);
    a.L = reinterpret_cast<const half_t *>(layer->L);
    a.X = reinterpret_cast<const half_t *>(X);
    a.Y = reinterpret_cast<half_t *>(Y);
    a.P = reinterpret_cast<float *>(ws + w.acc_off);
    a.T = reinterpret_cast<float *>(ws + w.dec_off + 256);
    a.ctrl = reinterpret_cast<unsigned *>(ws + w.dec_off);
    a.n = s.n;
    a.k = s.k;
    a.rank_pad = layer->rank_pad;
    a.m = m;
    a.n_packed = s.n;
    fill_plan(a, p);
    a.accumulate = 0;
    return launch_decode(a, p, static_cast<hipStream_t>(stream));
}

// What slim_linear_gemv would launch for this layer and token count (no launch, no device access).
extern "C" int slim_decode_plan(const slim_layer *layer, int32_t m, int32_t *out)
{
    if (!layer || !out) return SLIM_ERR_NULL;
    const slim_shape s = layer->shape;
    if (s.n < 1 || s.k < 128 || s.k % 128 || s.rank < 0 || m < 1 || m > kMaxTokens) return SLIM_ERR_SHAPE;
    if (layer->rank_pad != slim_rank_pad(s.rank)) return SLIM_ERR_SHAPE;
    const FusedPlan f = plan_fused(s.n, s.k, layer->rank_pad, m);
    const int mode = decode_mode(f);
    for (int i = 0; i < 12; ++i) out[i] = 0;
    out[0] = mode > 0 ? (mode == 3 ? 2 : mode) : 0;
    if (mode > 0) {
        out[1] = f.n_r + f.ygrid;
        out[2] = (f.waves + f.helpers) * kWave;
        out[3] = (int32_t)f.lds;
        out[4] = f.n_r;
        out[5] = f.kh;
        out[6] = f.S;
        out[7] = f.waves;
        out[8] = f.helpers;
        out[9] = f.kc;
        out[10] = f.nch;
        out[11] = f.ygrid;
    }
    return SLIM_OK;
}
