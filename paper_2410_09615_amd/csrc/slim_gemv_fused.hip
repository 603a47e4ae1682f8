// slim_linear_gemv in one launch, for layers whose X (all inputs, the padded
// token rows) fits the LDS of a compute unit.
//
// Two kinds of workgroups share one grid:
//
//  R role  (the first rank_pad / 16 workgroups) one tile of 16 ranks each:
//          T[:, tile] = X R[tile, :]^T over all inputs.  The wavefronts take
//          units of 16 ranks x 256 inputs (R and X straight from memory into
//          registers, dense 16 x 16 x 32 matrix instruction), add their partial
//          tiles in LDS, and wavefront 0 writes the tile of T as fp16, makes it
//          visible to the device and raises the tile's flag to the epoch of
//          this call.  These workgroups wait for nothing.
//  Y role  (all others) S wavefronts per tile of 16 output rows, 8 / S tiles
//          per workgroup and round.  Wavefront s of a tile takes the halves
//          (512 inputs) s, s + S, ... of the packed row tile through the
//          structured-sparse matrix instruction against X held in LDS, then the
//          steps of 32 ranks s, s + S, ... of the L row tile against T held in
//          LDS.  Between the two it waits (once per workgroup) until every
//          flag shows this call's epoch.  The S partial results, each already
//          scale * packed + low-rank, meet in LDS and wavefront 0 of the tile
//          stores Y.  Nothing goes through memory between the two terms: no
//          partial sums, no atomics, no second launch.
//
// Progress: workgroups start in the order of their index, so every R-role
// workgroup has started before any Y-role workgroup can wait for it, and the
// wait is bounded anyway (it gives up after kSpinLimit polls and records that
// in the control words; the call then returns wrong numbers, not a hang).
//
// The same kernel also runs the roles as two launches (mode 0, then mode 1),
// with the kernel boundary in place of the flags.
//
// T is rounded to fp16 once here, as in the prefill path.
#include <atomic>

#include "slim_decode.h"

namespace slim {

constexpr int kFusedMaxThreads = 512;
constexpr int kSpinLimit = 1 << 16;

struct FusedArgs {
    const uint8_t *qvals;
    const uint8_t *meta;
    const float *scale;
    const half_t *R;
    const half_t *L;
    const half_t *X;
    half_t *Y;
    half_t *T;           // fp16 [16][rank_pad]
    unsigned *flags;     // per tile of 16 ranks: epoch of the call that last completed it
    unsigned *err;       // set to 1 when a wait gave up
    unsigned epoch;
    int n, k, rank_pad, m;
    int mp;              // token rows of the LDS tiles (1, 4, 8, 16)
    int kpad;            // k rounded up to 1024: extent of an X row in LDS
    int S;               // wavefronts per row tile
    int n_r;             // R-role workgroups (rank_pad / 16)
    int mode;            // 0: R role only; 1: Y role only, T complete; 2: both roles in this grid
};

// ---- R role ----
__device__ __forceinline__ void role_r(const FusedArgs &a, half_t *lds_h, int rt)
{
    float *red = reinterpret_cast<float *>(lds_h);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int nw = blockDim.x / kWave;
    const int lx = lane & 15;       // A: rank within the tile; B, C: token
    const int ly = lane >> 4;
    const int rp = a.rank_pad;
    const int units = (a.k + 255) / 256;
    const uint4_t zero = {0u, 0u, 0u, 0u};

    auto issue_r = [&](int u, UnitRegs &b) {
#pragma unroll
        for (int t = 0; t < 8; ++t) b.r[t] = zero;
        if (u >= units) return;
        // step t reads the pieces (rank, 32 u + 4 t + ly): two tiles (2 KiB) further per step
        const char *base = reinterpret_cast<const char *>(a.R) + tl_piece(16u * rt + lx, 32u * u + ly, (uint32_t)a.k);
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (256 * u + 32 * t < a.k) b.r[t] = *reinterpret_cast<const uint4_t *>(base + 2048 * t);
    };
    auto issue_x = [&](int u, uint4_t (&xb)[8]) {
#pragma unroll
        for (int t = 0; t < 8; ++t) xb[t] = zero;
        if (u >= units || lx >= a.m) return;
        const half_t *xp = a.X + (size_t)lx * a.k + 256 * u + 8 * ly;
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (256 * u + 32 * t < a.k) xb[t] = *reinterpret_cast<const uint4_t *>(xp + 32 * t);
    };

    // two units per wavefront in flight at once (all of a 4096-input layer)
    UnitRegs bufA, bufB;
    uint4_t xa[8], xb[8];
    float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = acc0;
    auto mma = [&](const UnitRegs &b, const uint4_t (&x)[8]) {
#pragma unroll
        for (int t = 0; t < 8; ++t) {
            const half8_t av = __builtin_bit_cast(half8_t, b.r[t]);
            const half8_t bv = __builtin_bit_cast(half8_t, x[t]);
            if (t & 1)
                acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc1, 0, 0, 0);
            else
                acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc0, 0, 0, 0);
        }
    };
    for (int u = wave; u < units; u += 2 * nw) {
        issue_r(u, bufA);
        issue_x(u, xa);
        issue_r(u + nw, bufB);       // past the last unit: zeros
        issue_x(u + nw, xb);
        mma(bufA, xa);
        mma(bufB, xb);
    }
    // lane holds token lx, ranks 16 rt + 4 ly .. + 3
    float4_t acc = acc0 + acc1;
    if (wave != 0) *reinterpret_cast<float4_t *>(red + ((wave - 1) * kWave + lane) * 4) = acc;
    __syncthreads();
    if (wave == 0) {
        for (int w = 0; w < nw - 1; ++w) acc += *reinterpret_cast<const float4_t *>(red + (w * kWave + lane) * 4);
        const half4_t h = {(half_t)acc[0], (half_t)acc[1], (half_t)acc[2], (half_t)acc[3]};
        *reinterpret_cast<half4_t *>(a.T + (size_t)lx * rp + 16 * rt + 4 * ly) = h;
        if (a.mode == 2) {
            // the tile of T, then the flag: the fence makes this wavefront's
            // stores visible device-wide before the flag can be seen
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            if (lane == 0) __hip_atomic_store(a.flags + rt, a.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// ---- Y role ----
__device__ __forceinline__ void role_y(const FusedArgs &a, half_t *lds, int yb, int ygrid)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int nw = blockDim.x / kWave;
    const int lx = lane & 15;
    const int ly = lane >> 4;
    const int S = a.S;
    const int tpw = nw / S;              // tiles per workgroup and round
    const int ts = wave / S;             // tile slot of this wavefront
    const int s = wave - ts * S;         // its share of the inputs and of the ranks
    const int rp = a.rank_pad;
    const int rows_x = a.mp < kMaxTokens ? a.mp + 1 : kMaxTokens;    // token rows, then a zero row if a lane needs one
    const int ldx = a.kpad + kLdsPad;
    const int ldt = rp + kLdsPad;
    half_t *x_lds = lds;
    half_t *t_lds = lds + rows_x * ldx;
    float *red = reinterpret_cast<float *>(t_lds + rows_x * ldt);
    const int wtiles = (a.n + 15) / 16;
    const int H = (a.k + 511) / 512;             // halves of a row
    const int Hp = a.kpad / 512;
    const int steps = rp / 32;                   // steps of 32 ranks
    const int cnt_h = s < H ? (H - s + S - 1) / S : 0;
    const int cnt_l = s < steps ? (steps - s + S - 1) / S : 0;
    const int nP = (cnt_h + 1) / 2;              // items of two halves
    const int nL = (cnt_l + 7) / 8;              // items of eight steps
    const int nI = nP + nL;
    const int tile0 = yb * tpw + ts;
    const int tstride = ygrid * tpw;
    const int rounds = (wtiles - yb * tpw + tstride - 1) / tstride;      // same for the whole workgroup
    const uint32_t kt = pk_ktiles(a.k);
    const uint4_t zero = {0u, 0u, 0u, 0u};

    // Loads of item j of row tile ot: what lies past the rows, the inputs or the ranks is zero.
    auto issue_item = [&](int ot, int j, UnitRegs &b) {
#pragma unroll
        for (int i = 0; i < 8; ++i) b.r[i] = zero;
        const int o = 16 * ot + lx;
        if (j >= nI || ot >= wtiles || o >= a.n) return;
        if (j < nP) {
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int h = s + S * (2 * j + x);
                const int kl = 512 * h + 128 * ly;          // the lane's 128 inputs: one tile column of the packed layout
                if (h < H && kl < a.k) {
                    const uint8_t *qp = a.qvals + pk_qoff((uint32_t)o, (uint32_t)kl / 4, kt);
                    const uint8_t *mp = a.meta + pk_moff((uint32_t)o, (uint32_t)kl / 8, kt);
                    b.r[3 * x] = load_q16(qp);
                    b.r[3 * x + 1] = load_q16(qp + 512);
                    b.r[3 * x + 2] = load_m16(mp);
                }
            }
        } else {
            // step t = s + S (8 jl + i) takes ranks 32 t + 8 ly .. + 7 of row o: piece (o, 4 t + ly)
            const int t0 = s + S * 8 * (j - nP);
            const char *lp = reinterpret_cast<const char *>(a.L) + tl_piece((uint32_t)o, 4u * t0 + ly, (uint32_t)rp);
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (t0 + S * i < steps) b.r[i] = *reinterpret_cast<const uint4_t *>(lp + (size_t)2048 * S * i);
        }
    };

    // the first loads go out before anything else
    UnitRegs bufA, bufB;
    issue_item(tile0, 0, bufA);

    // X -> LDS: rows >= m zero, inputs past k zero up to kpad
    {
        const int per_row = a.kpad / 8;
        const int total = rows_x * per_row;
        for (int e0 = threadIdx.x; e0 < total; e0 += 8 * (int)blockDim.x) {
            uint4_t v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + i * (int)blockDim.x;
                const int row = e / per_row, c = e - row * per_row;
                v[i] = zero;
                if (e < total && row < a.m && c * 8 < a.k)
                    v[i] = *reinterpret_cast<const uint4_t *>(a.X + (size_t)row * a.k + c * 8);
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int e = e0 + i * (int)blockDim.x;
                const int row = e / per_row, c = e - row * per_row;
                if (e < total) *reinterpret_cast<uint4_t *>(x_lds + row * ldx + c * 8) = v[i];
            }
        }
    }
    // T -> LDS (all threads; the caller has made T visible)
    auto stage_t = [&]() {
        const int per_row = rp / 8;
        const int total = rows_x * per_row;
        for (int e = threadIdx.x; e < total; e += blockDim.x) {
            const int row = e / per_row, c = e - row * per_row;
            uint4_t v = zero;
            if (row < a.m) v = *reinterpret_cast<const uint4_t *>(a.T + (size_t)row * rp + c * 8);
            *reinterpret_cast<uint4_t *>(t_lds + row * ldt + c * 8) = v;
        }
    };
    // mode 2: wait for the flags of all rank tiles, then stage T
    auto wait_and_stage_t = [&]() {
        if (wave == 0) {
            bool done = false;
            for (int spin = 0; spin < kSpinLimit && !done; ++spin) {
                bool mine = true;
                for (int r = lane; r < a.n_r; r += kWave)
                    mine = mine && __hip_atomic_load(a.flags + r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == a.epoch;
                done = __all(mine);
                if (!done) __builtin_amdgcn_s_sleep(8);
            }
            if (!done && lane == 0) __hip_atomic_store(a.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            // what the R-role workgroups stored before raising their flags is read after this
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        __syncthreads();
        stage_t();
        __syncthreads();
    };
    bool t_ready = rp == 0;
    if (a.mode == 1 && rp > 0) {
        stage_t();
        t_ready = true;
    }
    __syncthreads();

    // this lane's B-operand rows: its token, or the zero row
    const int trow = lx < a.mp ? lx : a.mp;       // mp == 16: always lx
    const half_t *xrow_packed = x_lds + trow * ldx + 128 * (ly >> 1) + 8 * (ly & 1);
    const half_t *trow_l = t_lds + trow * ldt + 8 * ly;

    for (int round = 0; round < rounds; ++round) {
        const int ot = tile0 + round * tstride;     // past the last tile: nothing is loaded or stored
        const int ob = 16 * ot + 4 * ly;
        const bool vec = (ob + 3 < a.n) && (a.n & 3) == 0;
        float sc[4] = {0.f, 0.f, 0.f, 0.f};
        if (ot < wtiles) {
            if (vec) {
                const float4_t s4 = *reinterpret_cast<const float4_t *>(a.scale + ob);
#pragma unroll
                for (int v = 0; v < 4; ++v) sc[v] = s4[v];
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (ob + v < a.n) sc[v] = a.scale[ob + v];
            }
        }
        float4_t accp0 = {0.f, 0.f, 0.f, 0.f}, accp1 = accp0, accl0 = accp0, accl1 = accp0;
        for (int j = 0; j < nI; ++j) {
            if (j == nP && !t_ready) {
                wait_and_stage_t();
                t_ready = true;
            }
            if (j + 1 < nI)
                issue_item(ot, j + 1, bufB);
            else
                issue_item(ot + tstride, 0, bufB);
            if (j < nP) {
                const int h0 = min(s + S * (2 * j), Hp - 1), h1 = min(s + S * (2 * j + 1), Hp - 1);
                packed_half<0>(bufA, xrow_packed + 512 * h0, accp0, accp1);
                packed_half<1>(bufA, xrow_packed + 512 * h1, accp0, accp1);
            } else {
                const int t0 = s + S * 8 * (j - nP);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    // steps past the end carry zero L values and read T inside the row
                    const int t = min(t0 + S * i, steps - 1);
                    const half8_t bv = *reinterpret_cast<const half8_t *>(trow_l + 32 * t);
                    const half8_t av = __builtin_bit_cast(half8_t, bufA.r[i]);
                    if (i & 1)
                        accl1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, accl1, 0, 0, 0);
                    else
                        accl0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, accl0, 0, 0, 0);
                }
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) bufA.r[i] = bufB.r[i];
        }
        if (!t_ready) {          // a wavefront without rank steps still takes part in the barriers
            wait_and_stage_t();
            t_ready = true;
        }
        // lane holds token lx, rows 16 ot + 4 ly .. + 3
        const float4_t accp = accp0 + accp1;
        float4_t y = accl0 + accl1;
#pragma unroll
        for (int v = 0; v < 4; ++v) y[v] += sc[v] * accp[v];
        if (S > 1) {
            float *rset = red + (size_t)ts * (S - 1) * kWave * 4;
            if (s != 0) *reinterpret_cast<float4_t *>(rset + ((s - 1) * kWave + lane) * 4) = y;
            __syncthreads();
            if (s == 0)
                for (int w = 0; w < S - 1; ++w) y += *reinterpret_cast<const float4_t *>(rset + (w * kWave + lane) * 4);
        }
        if (s == 0 && lx < a.m && ot < wtiles) {
            half_t *yp = a.Y + (size_t)lx * a.n + ob;
            if (vec) {
                const half4_t h = {(half_t)y[0], (half_t)y[1], (half_t)y[2], (half_t)y[3]};
                *reinterpret_cast<half4_t *>(yp) = h;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (ob + v < a.n) yp[v] = (half_t)y[v];
            }
        }
        if (S > 1 && round + 1 < rounds) __syncthreads();      // the partial sums are read before the next round writes
    }
}

__global__ __launch_bounds__(kFusedMaxThreads, 1) void decode_fused_kernel(FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) half_t lds[];
    if (a.mode == 0) {
        role_r(a, lds, blockIdx.x);
    } else if (a.mode == 1) {
        role_y(a, lds, blockIdx.x, gridDim.x);
    } else if ((int)blockIdx.x < a.n_r) {
        role_r(a, lds, blockIdx.x);
    } else {
        role_y(a, lds, (int)blockIdx.x - a.n_r, (int)gridDim.x - a.n_r);
    }
}

static int pad_tokens16(int m) { return m <= 1 ? 1 : (m <= 4 ? 4 : (m <= 8 ? 8 : 16)); }

// Which layers take this path, and with what geometry.
FusedPlan plan_fused(int n, int k, int rank_pad, int m)
{
    FusedPlan p{};
    p.mp = pad_tokens16(m);
    p.kpad = (k + 1023) / 1024 * 1024;
    p.waves = kFusedMaxThreads / kWave;
    p.n_r = rank_pad / 16;
    const int rows_x = p.mp < kMaxTokens ? p.mp + 1 : kMaxTokens;
    const long wtiles = (n + 15) / 16;
    // Every workgroup should have a compute unit of its own (slots).  S wavefronts
    // per row tile make a round S times shorter and ask for S times as many
    // workgroup-rounds: take the S with the least rounds / S, the smaller S on a tie.
    const int slots = 256 - (p.n_r < 128 ? p.n_r : 128);
    p.S = 1;
    double best = 1e30;
    for (int S = 1; S <= p.waves; S *= 2) {
        const int tpw = p.waves / S;
        const long wgs = (wtiles + tpw - 1) / tpw;
        const double cost = (double)((wgs + slots - 1) / slots) / S;
        if (cost < best * 0.999) {
            best = cost;
            p.S = S;
        }
    }
    const int tpw = p.waves / p.S;
    long yg = (wtiles + tpw - 1) / tpw;
    if (yg > slots) yg = slots;
    p.ygrid = (int)yg;
    const size_t red_y = p.S > 1 ? (size_t)tpw * (p.S - 1) * kWave * 16 : 0;
    const size_t red_r = (size_t)(p.waves - 1) * kWave * 16;
    const size_t lds_y = (size_t)rows_x * ((p.kpad + kLdsPad) + (rank_pad + kLdsPad)) * sizeof(half_t) + red_y;
    p.lds = lds_y > red_r ? lds_y : red_r;
    p.ok = p.lds <= 160 * 1024 && p.n_r <= 128;
    return p;
}

static std::atomic<unsigned> g_epoch{0};

// mode: 2 = one launch, 1 = the two roles as two launches
int launch_decode_fused(const slim_layer *layer, const half_t *X, int m, half_t *Y, half_t *T, unsigned *flags,
                        unsigned *err, const FusedPlan &p, int mode, hipStream_t st)
{
    FusedArgs a{};
    a.qvals = layer->qvals;
    a.meta = layer->meta;
    a.scale = layer->scale;
    a.R = reinterpret_cast<const half_t *>(layer->R);
    a.L = reinterpret_cast<const half_t *>(layer->L);
    a.X = X;
    a.Y = Y;
    a.T = T;
    a.flags = flags;
    a.err = err;
    unsigned e = ++g_epoch;
    if (e == 0) e = ++g_epoch;          // flags start as zeros: epoch 0 is never used
    a.epoch = e;
    a.n = layer->shape.n;
    a.k = layer->shape.k;
    a.rank_pad = layer->rank_pad;
    a.m = m;
    a.mp = p.mp;
    a.kpad = p.kpad;
    a.S = p.S;
    a.n_r = p.n_r;
    const dim3 blk(p.waves * kWave);
    if (mode == 2 || p.n_r == 0) {
        a.mode = p.n_r == 0 ? 1 : 2;
        hipLaunchKernelGGL(decode_fused_kernel, dim3((unsigned)(p.n_r + p.ygrid)), blk, p.lds, st, a);
    } else {
        a.mode = 0;
        hipLaunchKernelGGL(decode_fused_kernel, dim3((unsigned)p.n_r), blk, p.lds, st, a);
        a.mode = 1;
        hipLaunchKernelGGL(decode_fused_kernel, dim3((unsigned)p.ygrid), blk, p.lds, st, a);
    }
    return hip_status(hipGetLastError());
}

}  // namespace slim
