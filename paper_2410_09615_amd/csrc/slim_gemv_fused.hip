// slim_linear_gemv in one launch: X lives in the LDS of a compute unit, all of
// it where the token rows of all inputs fit, else in chunks that stream through
// two buffers while the accumulators stay in registers.
//
// Two kinds of workgroups share one grid:
//
//  R role  (the first workgroups of the grid) one tile of 16 ranks and one share
//          of the inputs each: T[:, tile] += X R[tile, share]^T.  The wavefronts
//          take units of 16 ranks x 256 inputs (R and X straight from memory
//          into registers, dense 16 x 16 x 32 matrix instruction), add their
//          partial tiles in LDS, and wavefront 0 stores the tile as fp16 in
//          16-byte pieces {epoch of this call, four ranks of one token, checksum},
//          written through to memory.  These workgroups wait for nothing.
//  Y role  (all others) S wavefronts per tile of 16 output rows.  Wavefront s
//          of a tile takes the halves (512 inputs) s, s + S, ... of the packed
//          row tile through the structured-sparse matrix instruction against X
//          held in LDS, then the steps of 32 ranks s, s + S, ... of the L row
//          tile against T held in LDS.  One to eight more wavefronts of the
//          workgroup (helpers) move what is not a plain stream: they stage X
//          with loads that write LDS directly, and they fetch T: they re-read
//          its pieces until every piece carries this call's epoch and its
//          checksum, add the shares and put the sum into LDS, while the others
//          are busy with the packed term; the workgroup meets at one barrier
//          before its first rank step.  The
//          S partial results, each already scale * packed + low-rank, meet in
//          LDS and wavefront 0 of the tile stores Y.  Nothing goes through
//          memory between the two terms but T itself: no partial sums, no
//          atomics, no second launch.
//
// A piece is valid by itself (its epoch is unique to the call, process-wide), so
// there are no flags to order against the data, nothing to reset between calls,
// and a workspace may serve different layers in turn.
//
// Progress: the planner admits a geometry only if all workgroups of the grid are
// resident at once, so none that is waited for can be queued behind one that
// waits (workgroups also start in the order of their index, which lets the R
// role start first), and the wait is bounded anyway (a helper gives up after kSpinLimit reads and records
// that in the control words and puts NaN in place of the T it did not get, so the
// outputs of its workgroup are NaN: a failed call cannot pass for a result).
//
// The same kernel also runs the roles as two launches (mode 0, then mode 1).
//
// T is rounded to fp16 once per share here (prefill: once).
#include <atomic>
#include <cstdlib>
#include <type_traits>

#include "slim_decode.h"

namespace slim {

constexpr int kFusedMaxThreads = 1024;     // 8 working wavefronts + up to 8 helpers
constexpr int kScopeDevice = 16;      // cache policy of a buffer access: device scope (written through / read from memory)
constexpr int kMaxShares = 4;         // R role: at most this many shares of the inputs (planes of T)
constexpr int kFusedWavesPerSimd = 4;   // the kernel is compiled for 128 registers: 16 wavefronts per compute unit
constexpr int kSpinLimit = 1 << 16;
constexpr int kSpinLimitShort = 256;   // test of the bounded wait (mode bit 3)
constexpr int kWaitVm0 = 0x0F70;       // s_waitcnt vmcnt(0) (expcnt, lgkmcnt left alone): all vector memory loads of the wavefront are back
constexpr uint32_t kNowhere = 0x80000000u;       // byte offset past the end of every buffer here (all are < 2 GiB)

struct FusedArgs {
    const uint8_t *qvals;
    const uint8_t *meta;
    const float *scale;
    const half_t *R;     // fp16 adapters in the adapter layout, or
    const half_t *L;
    const uint8_t *Rq;   // 4-bit adapters: codes in the 4-bit adapter layout and group scales
    const uint8_t *Lq;
    const half_t *Rs;
    const half_t *Ls;
    const half_t *X;
    half_t *Y;
    uint4_t *T;          // pieces {epoch, 4 ranks fp16, checksum} [kh][16][rank_pad / 4]: T is the sum of the planes
    unsigned *err;       // set to 1 when a wait gave up
    unsigned epoch;      // this call's number (top bit clear, never 0), or
    const unsigned *epoch_ptr;   // under stream capture: where a small kernel ahead of this one has put it (top bit set)
    int n, k, rank_pad, m;
    int rank;            // true rank (rows of R, columns of L that exist in the 4-bit buffers)
    int kpad;            // k rounded up to 1024
    int kc;              // inputs per chunk of X in LDS (multiple of 1024; kpad: all of X at once)
    int nch;             // chunks: more than one -> two LDS buffers, the helpers stage chunk c + 1 during chunk c
    int S;               // wavefronts per row tile
    int n_r;             // R-role workgroups: (rank_pad / 16) tiles x kh shares of the inputs
    int kh;              // shares of the inputs in the R role = planes of T
    int upk;             // units of 256 inputs per share
    int helpers;         // wavefronts of a workgroup that only fetch T (Y role)
    int mode;            // 0: R role only; 1: Y role only, T complete; 2: both roles in this grid;
                         // + 4 (low-rank term alone, both roles): add to what Y holds
                         // + 8 (test of the bounded wait): the helpers give up after kSpinLimitShort polls
};

// The number that tags this call's pieces of T.  A launch argument normally; a launch that is
// being captured into a graph would replay with the same number and take the pieces of the
// previous replay for its own, so there the number lives in the workspace and a one-thread
// kernel ahead of this one advances it on every replay.  The top bit keeps the two kinds apart.
__device__ __forceinline__ unsigned call_epoch(const FusedArgs &a)
{
    return a.epoch_ptr ? (__builtin_nontemporal_load(a.epoch_ptr) | 0x80000000u) : a.epoch;
}

__global__ void decode_epoch_bump_kernel(unsigned *ctr)
{
    const unsigned v = (*ctr + 1u) & 0x7FFFFFFFu;
    *ctr = v ? v : 1u;
}

// A piece of T: {epoch, two dwords of four fp16 ranks, epoch ^ dword ^ dword}.  The reader accepts it only if
// the first dword is this call's epoch and the last one is the checksum of the three before it, so a piece
// whose dwords come from two different stores (should a 128-bit store ever become visible in parts) is
// taken for "not there yet" and read again, unless the old and the new data have the same checksum --
// which they do when they are the same data.  Only single dwords need to be atomic for that.
__device__ __forceinline__ bool piece_valid(const uint4_t &pc, unsigned epoch)
{
    return pc[0] == epoch && pc[3] == (pc[0] ^ pc[1] ^ pc[2]);
}
constexpr unsigned short kHalfNaNBits = 0x7E00;
#define kHalfNaN __builtin_bit_cast(half_t, kHalfNaNBits)

// The loads of one item of the Y role: eight 128-bit loads.
struct ItemRegs {
    uint4_t r[8];
};

// One half (512 inputs) of a packed item: 8 sparse matrix instructions (V_SMFMAC_F32_16X16X64_F16) on
// registers r[4 H], r[4 H + 1] (codes) and the low halves of r[4 H + 2], r[4 H + 3] (positions of the
// lane's inputs 0-63 and 64-127).  xh and the B operand as in packed_half().
template <int H>
__device__ __forceinline__ void packed_half_item(const ItemRegs &b, const half_t *xh, float4_t &acc0, float4_t &acc1)
{
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const uint32_t qd = t < 4 ? b.r[4 * H][t] : b.r[4 * H + 1][t - 4];
        const half8_t av = codes_to_half8(qd);
        const half8_t b1 = *reinterpret_cast<const half8_t *>(xh + 16 * t);
        const half8_t b2 = *reinterpret_cast<const half8_t *>(xh + 256 + 16 * t);
        const half16_t bv = __builtin_shufflevector(b1, b2, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
        const int idx = (int)(t < 4 ? b.r[4 * H + 2][t >> 1] : b.r[4 * H + 3][(t >> 1) - 2]);
        // even t: index bits 15..0, odd t: bits 31..16 of the position dword
        if (t & 1)
            acc1 = __builtin_amdgcn_smfmac_f32_16x16x64_f16(av, bv, acc1, idx, 0, 1);
        else
            acc0 = __builtin_amdgcn_smfmac_f32_16x16x64_f16(av, bv, acc0, idx, 0, 0);
    }
}

// ---- R role ----
template <bool Q4>
__device__ __forceinline__ void role_r(const FusedArgs &a, half_t *lds_h, int rb)
{
    const int rt = rb / a.kh;                  // tile of 16 ranks
    const int kh = rb - rt * a.kh;             // share of the inputs

    float *red = reinterpret_cast<float *>(lds_h);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);    // uniform: lets the compiler keep what derives from it in scalar registers
    const int nw = blockDim.x / kWave;
    const int lx = lane & 15;       // A: rank within the tile; B, C: token
    const int ly = lane >> 4;
    const int rp = a.rank_pad;
    const int units = (a.k + 255) / 256;
    const int u0 = kh * a.upk, u1 = min(units, u0 + a.upk);

    // Buffer loads: one 32-bit offset per lane, no branches; an offset past the
    // end of the buffer (kNowhere) reads as zero.
    const rsrc_t x_rs = make_rsrc(a.X, (uint32_t)a.m * a.k * 2u);
    UnitRegs buf;
    uint4_t xb[8];
    float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = acc0;
    if constexpr (!Q4) {
        // Two register sets for R alternate (both go out at once; a wavefront with more
        // units refills a set as soon as it is consumed); the X operand, an L2 hit, is
        // loaded when its unit is due.
        const rsrc_t r_rs = make_rsrc(a.R, (uint32_t)tl_bytes(rp, a.k));
        auto issue_r = [&](int u, UnitRegs &b) {
            // step t reads the pieces (rank, 32 u + 4 t + ly): two tiles (2 KiB) further per step
            const uint32_t rbase = tl_piece(16u * rt + lx, 32u * u + ly, (uint32_t)a.k);
#pragma unroll
            for (int t = 0; t < 8; ++t)
                b.r[t] = load16(r_rs, (u < u1 && 256 * u + 32 * t < a.k) ? rbase + 2048u * t : kNowhere, 0);
        };
        auto unit = [&](int u, const UnitRegs &b) {
            const uint32_t xbase = ((uint32_t)lx * a.k + 256 * u + 8 * ly) * 2u;
#pragma unroll
            for (int t = 0; t < 8; ++t)
                xb[t] = load16(x_rs, (lx < a.m && 256 * u + 32 * t < a.k) ? xbase + 64u * t : kNowhere, 0);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const half8_t av = __builtin_bit_cast(half8_t, b.r[t]);
                const half8_t bv = __builtin_bit_cast(half8_t, xb[t]);
                if (t & 1)
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc1, 0, 0, 0);
                else
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc0, 0, 0, 0);
            }
        };
        UnitRegs buf2;
        const int ua = u0 + wave;
        issue_r(ua, buf);
        issue_r(ua + nw, buf2);
        for (int u = ua; u < u1; u += 2 * nw) {
            unit(u, buf);
            issue_r(u + 2 * nw, buf);
            if (u + nw < u1) {
                unit(u + nw, buf2);
                issue_r(u + 3 * nw, buf2);
            }
        }
    } else {
        // 4-bit R: lane (rank lx, quarter ly) owns 64 consecutive inputs of the unit (32
        // bytes of codes, one scale: a quarter lies inside one group of 128); step t
        // takes its inputs 8 t .. 8 t + 7, and the X operand follows the same order.
        // (rows of R past the last stored tile of 16 lie past the end of the buffers: zeros)
        const rsrc_t q_rs = make_rsrc(a.Rq, (uint32_t)q4_code_bytes(a.rank, a.k));
        const rsrc_t s_rs = make_rsrc(a.Rs, (uint32_t)q4_scale_bytes(a.rank, a.k));
        const uint32_t ct = q4_ctiles(a.k), gs = q4_groups(a.k);
        for (int u = u0 + wave; u < u1; u += nw) {
            const bool ok = 256 * u + 64 * ly < a.k;
            const uint32_t qbase = ok ? q4_piece(16u * rt + lx, 4u * u + ly, ct) : kNowhere;
            const uint32_t xbase = (ok && lx < a.m) ? ((uint32_t)lx * a.k + 256 * u + 64 * ly) * 2u : kNowhere;
            buf.r[0] = load16(q_rs, qbase, 0);
            buf.r[1] = load16(q_rs, qbase, 16);
            const unsigned short sb = (unsigned short)__builtin_amdgcn_raw_buffer_load_b16(
                s_rs, ok ? (int)(((16u * rt + lx) * gs + 2u * u + (ly >> 1)) * 2u) : (int)kNowhere, 0, 0);
#pragma unroll
            for (int t = 0; t < 8; ++t) xb[t] = load16(x_rs, xbase, 16u * t);
            const half_t sc = __builtin_bit_cast(half_t, sb);
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                const half8_t av = codes_to_half8(buf.r[t >> 2][t & 3]) * sc;
                const half8_t bv = __builtin_bit_cast(half8_t, xb[t]);
                if (t & 1)
                    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc1, 0, 0, 0);
                else
                    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc0, 0, 0, 0);
            }
        }
    }
    // lane holds token lx, ranks 16 rt + 4 ly .. + 3
    float4_t acc = acc0 + acc1;
    if (wave != 0) *reinterpret_cast<float4_t *>(red + ((wave - 1) * kWave + lane) * 4) = acc;
    __syncthreads();
    if (wave == 0) {
        for (int w = 0; w < nw - 1; ++w) acc += *reinterpret_cast<const float4_t *>(red + (w * kWave + lane) * 4);
        const half4_t h = {(half_t)acc[0], (half_t)acc[1], (half_t)acc[2], (half_t)acc[3]};
        const uint2_t hb = __builtin_bit_cast(uint2_t, h);
        // one 16-byte store per lane, through to memory: the piece with its epoch
        const rsrc_t t_rs = make_rsrc(a.T, (uint32_t)a.kh * kMaxTokens * (rp / 4) * 16u);
        const uint32_t off = (((uint32_t)kh * kMaxTokens + lx) * (rp / 4) + 4 * rt + ly) * 16u;
        typedef unsigned int store4_t __attribute__((__vector_size__(16)));
        const unsigned ep = call_epoch(a);
        const store4_t piece = {ep, hb[0], hb[1], ep ^ hb[0] ^ hb[1]};
        __builtin_amdgcn_raw_buffer_store_b128(piece, t_rs, (int)off, 0, kScopeDevice);
    }
}

// ---- Y role ----
// LR: the low-rank term alone (slim_lowrank): no packed items, no X in LDS, no row
// scales; the barrier sequence is that of a layer whose X is one chunk.
template <bool Q4, bool LR = false>
__device__ __forceinline__ void role_y(const FusedArgs &a, half_t *lds, int yb, int ygrid)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);    // uniform: lets the compiler keep what derives from it in scalar registers
    const int nw = blockDim.x / kWave;
    const int lx = lane & 15;
    const int ly = lane >> 4;
    const int S = a.S;
    const int nwc = nw - a.helpers;      // working wavefronts; the helpers come after them
    const int tpw = nwc / S;             // tiles per workgroup and round
    const int ts = wave / S;             // tile slot of this wavefront
    const int s = wave - ts * S;         // its share of the inputs and of the ranks
    const int rp = a.rank_pad;
    const int rows_x = a.m;              // token rows in LDS; the lanes of the other columns of a matrix
                                         // operand read row 0 and their results are not stored
    const int ldx = a.kc + kLdsPad;
    const int ldt = rp + kLdsPad;
    const int nch = LR ? 1 : a.nch;
    // LDS: one X buffer, then T, then the partial results; with chunks: two X
    // buffers, T takes the place of the buffer that is free during the last chunk
    half_t *x_lds = lds;
    const int xbuf = rows_x * ldx;               // halves per X buffer
    half_t *t_lds = nch > 1 ? lds + (nch & 1) * xbuf : lds + xbuf;
    float *red = reinterpret_cast<float *>(nch > 1 ? lds + 2 * xbuf : lds + xbuf + rows_x * ldt);
    const int wtiles = (a.n + 15) / 16;
    const int H = (a.k + 511) / 512;             // halves of a row
    const int hc = a.kc / 512;                   // halves per chunk
    const int steps = rp / 32;                   // steps of 32 ranks
    // halves of this wavefront per chunk: s, s + S, ... < hc (with chunks S divides hc: the same for all)
    const int hpc = s < hc ? (hc - s + S - 1) / S : 0;
    const int ipc = LR ? 0 : (hpc + 1) / 2;      // items (of two halves) per chunk
    const int ipd = LR ? 1 : ipc;                // as a divisor (no packed items: never used)
    // rank work of this wavefront: steps of 32 ranks s, s + S, ... (fp16), or units of 256 ranks (4-bit)
    const int units_l = (int)q4_ctiles(rp);
    const int cnt_l = Q4 ? (s < units_l ? (units_l - s + S - 1) / S : 0) : (s < steps ? (steps - s + S - 1) / S : 0);
    const int nP = nch * ipc;
    const int nL = Q4 ? (cnt_l + 1) / 2 : (cnt_l + 7) / 8;    // items of eight steps, or of two units
    const int nI = nP + nL;
    const int tile0 = yb * tpw + ts;
    const int tstride = ygrid * tpw;
    const int rounds = (wtiles - yb * tpw + tstride - 1) / tstride;      // same for the whole workgroup
    const uint32_t kt = pk_ktiles(a.k);

    auto tile_of = [&](int r) { return tile0 + r * tstride; };   // r >= rounds: past the last tile, loads read zeros
    // Loads of item j of the row tile of round r: ALWAYS the same eight load instructions, whatever the
    // item is (packed inputs, rank steps, or nothing), with the descriptors and offsets chosen by
    // uniform selects.  The compiler keeps count of the loads in flight per register: with one
    // instruction sequence per item it knows, at every use, how many younger loads there are, and
    // waits for exactly the set it needs while the other set stays in flight (with loads under
    // branches it waits for everything, every time).  Offsets: one 32-bit value per lane, no
    // branches around loads; rows past n inside the last tile of 32 are zero bytes in the tiled
    // layouts, tiles past the last one lie past the end of the buffer, and what lies past the
    // inputs or the ranks gets the offset kNowhere: all zeros.
    //   packed item (two halves x):  r[4x], r[4x+1] codes; r[4x+2], r[4x+3] positions (the low
    //                                8 bytes of each 16-byte load are the lane's)
    //   rank item, fp16:             r[i] = the lane's piece of L for step i
    //   rank item, 4-bit (units x):  r[4x], r[4x+1] codes; r[4x+2] the 16 bytes that hold the scale
    const rsrc_t q_rs = make_rsrc(a.qvals, (uint32_t)pk_qbytes(a.n, a.k));
    const rsrc_t m_rs = make_rsrc(a.meta, (uint32_t)pk_mbytes(a.n, a.k));
    const rsrc_t l_rs = Q4 ? make_rsrc(a.Lq, (uint32_t)q4_code_bytes(a.n, rp)) : make_rsrc(a.L, (uint32_t)tl_bytes(a.n, rp));
    const rsrc_t ls_rs = make_rsrc(Q4 ? a.Ls : nullptr, Q4 ? (uint32_t)q4_scale_bytes(a.n, rp) : 0u);
    const rsrc_t sc_rs = make_rsrc(LR ? nullptr : a.scale, LR ? 0u : (uint32_t)a.n * 4u);
    auto issue_item = [&](int r, int j, ItemRegs &b) {
        const int ot = tile_of(r);                   // r >= rounds: past the last tile
        const bool tile_ok = ot < wtiles;
        const uint32_t o = 16u * ot + lx;
        const bool packed = j < nP;
        uint32_t off[8];
        if (packed) {
            const int c = j / ipd, jj = j - c * ipd;        // chunk, item within the chunk
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int hl = s + S * (2 * jj + x);        // half within the chunk
                const int h = c * hc + hl;
                const int kl = 512 * h + 128 * ly;          // the lane's 128 inputs: one tile column of the packed layout
                const bool ok = hl < hc && h < H && kl < a.k && tile_ok;
                const uint32_t qo = ok ? (uint32_t)pk_qoff(o, (uint32_t)kl / 4, kt) : kNowhere;
                const uint32_t mo = ok ? (uint32_t)pk_moff(o, (uint32_t)kl / 8, kt) : kNowhere;
                off[4 * x] = qo;
                off[4 * x + 1] = qo + 512u;
                off[4 * x + 2] = mo;
                off[4 * x + 3] = mo + 256u;
            }
        } else if constexpr (!Q4) {
            // step t = s + S (8 jl + i) takes ranks 32 t + 8 ly .. + 7 of row o: piece (o, 4 t + ly)
            const int t0 = s + S * 8 * (j - nP);
            const uint32_t base = tl_piece(o, 4u * t0 + ly, (uint32_t)rp);
#pragma unroll
            for (int i = 0; i < 8; ++i) off[i] = (j < nI && tile_ok && t0 + S * i < steps) ? base + 2048u * S * i : kNowhere;
        } else {
            // two units of 256 ranks: 32 bytes of codes and a scale per lane and unit
            const uint32_t ct = q4_ctiles(rp), gs = q4_groups(rp);
#pragma unroll
            for (int x = 0; x < 2; ++x) {
                const int uu = s + S * (2 * (j - nP) + x);
                const bool ok = j < nI && tile_ok && uu < units_l && 256 * uu + 64 * ly < rp;
                const uint32_t qo = ok ? q4_piece(o, 4u * uu + ly, ct) : kNowhere;
                off[4 * x] = qo;
                off[4 * x + 1] = qo + 16u;
                off[4 * x + 2] = ok ? ((o * gs + 2u * uu + (ly >> 1)) * 2u) & ~3u : kNowhere;    // the dword that holds the scale
                off[4 * x + 3] = kNowhere;
            }
        }
        // descriptors per slot: codes / positions of the packed rows, or the adapter buffers
        const rsrc_t d0 = packed ? q_rs : l_rs;
        const rsrc_t d1 = packed ? m_rs : (Q4 ? ls_rs : l_rs);
        const rsrc_t d2 = packed ? m_rs : l_rs;                 // 4-bit rank items: offset kNowhere, any descriptor
        b.r[0] = load16(d0, off[0], 0);
        b.r[1] = load16(d0, off[1], 0);
        b.r[2] = load16(d1, off[2], 0);
        b.r[3] = load16(d2, off[3], 0);
        b.r[4] = load16(d0, off[4], 0);
        b.r[5] = load16(d0, off[5], 0);
        b.r[6] = load16(d1, off[6], 0);
        b.r[7] = load16(d2, off[7], 0);
    };

    // A wavefront's work is a sequence of items, nIe per round (a wavefront without any still takes
    // part in the barriers), numbered through the rounds.  Two register sets alternate: the loads
    // of the item after next go out as soon as an item is done.  Nothing may move across the
    // boundaries between "use a set" and "load a set": the instruction scheduler would otherwise
    // sink the loads to the end of the loop and wait for all of them at its top.
    const int nIe = nI > 0 ? nI : 1;
    const int total = rounds * nIe;                  // items of this wavefront
    auto advance = [&](int &r, int &j) {
        const bool wrap = j + 1 >= nIe;
        j = wrap ? 0 : j + 1;
        r += wrap ? 1 : 0;
    };
    int ir = 0, ij = 0;              // next item to load
    ItemRegs bufA, bufB;

    // the first two items' loads go out before anything else
    __builtin_amdgcn_sched_barrier(0);
    if (wave < nwc) {
        issue_item(ir, ij, bufA);
        advance(ir, ij);
        __builtin_amdgcn_sched_barrier(0);
        issue_item(ir, ij, bufB);
        advance(ir, ij);
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- helpers: T -> LDS ----
    // A helper lane owns (token, four ranks) pairs hl, hl + 64 helpers, ...; a pair
    // has one piece per share.  It re-reads its pieces (device scope) until each
    // carries this call's epoch, adds the shares and writes four halves to LDS.
    if (wave >= nwc) {
        // X -> LDS, by the helpers alone, with loads that write LDS directly (no
        // registers: a wavefront keeps dozens of KiB in flight).  One load
        // instruction moves a row segment of 512 inputs (64 lanes x 16 bytes,
        // contiguous in LDS); inputs past k read as zero.  Chunk c goes into
        // buffer c & 1; chunks 0 and 1 go out at once, chunk c + 1 when the working
        // wavefronts have left chunk c - 1 (the barrier that opens chunk c).
        {
            const rsrc_t x_rs = make_rsrc(a.X, (uint32_t)a.m * a.k * 2u);
            const int hw = wave - nwc;                        // helper index
            auto stage_chunk = [&](int c) {
                half_t *dst = x_lds + (c & 1) * xbuf;
                for (int idx = hw; idx < rows_x * hc; idx += a.helpers) {
                    const int row = idx / hc, seg = idx - row * hc;
                    const int col = c * a.kc + seg * 512 + lane * 8;
                    const uint32_t off = col < a.k ? ((uint32_t)row * a.k + col) * 2u : kNowhere;
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(
                        x_rs, (__attribute__((address_space(3))) void *)(dst + row * ldx + seg * 512), 16, (int)off, 0, 0, 0);
                }
            };
            if constexpr (!LR) stage_chunk(0);
            if (nch > 1) {
                stage_chunk(1);
                // chunk 0 is complete when at most the loads of chunk 1 are outstanding;
                // they return in order, so waiting for all of them is the simple upper bound
            }
            __builtin_amdgcn_s_waitcnt(kWaitVm0);
            __syncthreads();                                  // chunk 0 (and 1) in LDS
            for (int c = 1; c < nch; ++c) {
                __syncthreads();                              // opens chunk c: chunk c - 1 is done with
                if (c + 1 < nch) {
                    stage_chunk(c + 1);
                    __builtin_amdgcn_s_waitcnt(kWaitVm0);
                }
            }
        }
        const rsrc_t t_rs = make_rsrc(a.T, (uint32_t)a.kh * kMaxTokens * (rp / 4) * 16u);
        const int hl = (int)threadIdx.x - nwc * kWave;
        const int hn = a.helpers * kWave;
        const int qpr = rp / 4;                           // pairs per token
        const int pairs = a.m * qpr;
        int spins = 0;
        bool gave_up = false;
        const int spin_limit = (a.mode & 8) ? kSpinLimitShort : kSpinLimit;
        const unsigned epoch = call_epoch(a);
        auto piece_off = [&](int pair, int share) {
            const int row = pair / qpr, q = pair - row * qpr;
            return pair < pairs ? (((uint32_t)share * kMaxTokens + row) * qpr + q) * 16u : kNowhere;
        };
        auto fetch = [&](auto khc) {
            constexpr int KH = decltype(khc)::value;
            constexpr int PB = 8 / KH;                    // pairs per batch: 8 loads in flight
            for (int p0 = hl; p0 < pairs; p0 += PB * hn) {        // p0 differs per lane: every lane runs its own count
                uint4_t pc[PB * KH];
                bool all_there = false;
                while (!all_there) {
#pragma unroll
                    for (int i = 0; i < PB; ++i)
#pragma unroll
                        for (int h = 0; h < KH; ++h)
                            pc[i * KH + h] = __builtin_bit_cast(
                                uint4_t, __builtin_amdgcn_raw_buffer_load_b128(t_rs, (int)piece_off(p0 + i * hn, h), 0, kScopeDevice));
                    all_there = true;
#pragma unroll
                    for (int i = 0; i < PB; ++i)
#pragma unroll
                        for (int h = 0; h < KH; ++h)
                            all_there = all_there && (p0 + i * hn >= pairs || piece_valid(pc[i * KH + h], epoch));
                    if (!all_there) {
                        if (++spins >= spin_limit) {
                            gave_up = true;
                            break;
                        }
                        __builtin_amdgcn_s_sleep(4);
                    }
                }
#pragma unroll
                for (int i = 0; i < PB; ++i) {
                    const int pair = p0 + i * hn;
                    half4_t sum = {0, 0, 0, 0};
#pragma unroll
                    for (int h = 0; h < KH; ++h) sum += __builtin_bit_cast(half4_t, uint2_t{pc[i * KH + h][1], pc[i * KH + h][2]});
                    // a wait that gave up must not pass for a result: NaN in T makes every output of this workgroup NaN
                    if (gave_up) sum = half4_t{kHalfNaN, kHalfNaN, kHalfNaN, kHalfNaN};
                    if (pair < pairs) {
                        const int row = pair / qpr, q = pair - row * qpr;
                        *reinterpret_cast<half4_t *>(t_lds + row * ldt + 4 * q) = sum;
                    }
                }
            }
        };
        if (rp > 0) {
            if (a.kh == 1)
                fetch(std::integral_constant<int, 1>{});
            else if (a.kh == 2)
                fetch(std::integral_constant<int, 2>{});
            else
                fetch(std::integral_constant<int, 4>{});
            if ((gave_up || spins >= spin_limit) && a.err) __hip_atomic_store(a.err, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // the barriers of the working wavefronts: T, then those of every round
        if (rp > 0) __syncthreads();
        for (int r = 0; r < rounds; ++r)
            if (S > 1) {
                __syncthreads();
                if (r + 1 < rounds) __syncthreads();
            }
        return;
    }
    __syncthreads();                 // the helpers have put chunk 0 of X into LDS
    bool t_ready = rp == 0;
    auto meet_for_t = [&]() { __syncthreads(); };     // the helpers arrive when T is in LDS

    // this lane's B-operand rows: its token, or any row at all
    const int trow = lx < a.m ? lx : 0;
    const half_t *xrow_packed = x_lds + trow * ldx + 128 * (ly >> 1) + 8 * (ly & 1);
    const half_t *trow_l = t_lds + trow * ldt + 8 * ly;

    float4_t acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = acc0, sc4 = acc0;
    // item j of round r, its loads in cur
    auto step = [&](int r, int j, const ItemRegs &cur) {
        const int ot = tile_of(r);
        const int ob = 16 * ot + 4 * ly;
        const bool vec = (ob + 3 < a.n) && (a.n & 3) == 0;
        if (j == nP) {
            // the packed term is scaled once; the rank steps go on in the same registers.  (This use of the
            // scales stands ahead of their load in the code on purpose: what it waits for was loaded at
            // least one item ago, and the compiler's count of loads in flight then lets the other register
            // set stay in flight.  Without packed items there is nothing to scale.)
            if (nP > 0) {
                acc0 = (acc0 + acc1) * sc4;
                acc1 = float4_t{0.f, 0.f, 0.f, 0.f};
            }
            if (!t_ready) {
                meet_for_t();
                t_ready = true;
            }
        }
        if (j == 0) {
            acc0 = float4_t{0.f, 0.f, 0.f, 0.f};
            acc1 = acc0;
            // row scales of this lane's four outputs (rows past n read as zero): needed when the packed
            // items are done
            sc4 = __builtin_bit_cast(float4_t, load16(sc_rs, (!LR && ot < wtiles) ? (uint32_t)ob * 4u : kNowhere, 0));
        }
        if (j < nP) {
            const int c = j / ipd, jj = j - c * ipd;
            if (c > 0 && jj == 0) __syncthreads();     // chunk c is in LDS; everybody has left chunk c - 1
            const half_t *xc = xrow_packed + (c & 1) * xbuf;
            const int h0 = min(s + S * (2 * jj), hc - 1), h1 = min(s + S * (2 * jj + 1), hc - 1);
            packed_half_item<0>(cur, xc + 512 * h0, acc0, acc1);
            packed_half_item<1>(cur, xc + 512 * h1, acc0, acc1);
        } else if (j < nI) {
            if constexpr (!Q4) {
                const int t0 = s + S * 8 * (j - nP);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    // steps past the end carry zero L values and read T inside the row
                    const int t = min(t0 + S * i, steps - 1);
                    const half8_t bv = *reinterpret_cast<const half8_t *>(trow_l + 32 * t);
                    const half8_t av = __builtin_bit_cast(half8_t, cur.r[i]);
                    if (i & 1)
                        acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc1, 0, 0, 0);
                    else
                        acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc0, 0, 0, 0);
                }
            } else {
                const uint32_t gs = q4_groups(rp);
#pragma unroll
                for (int x = 0; x < 2; ++x) {
                    const int uu = s + S * (2 * (j - nP) + x);
                    // the scale is one half of the dword that was loaded: which, by its byte address
                    const uint32_t sa = ((16u * ot + lx) * gs + 2u * uu + (ly >> 1)) * 2u;
                    const uint32_t sd = cur.r[4 * x + 2][0];
                    const half_t sc = __builtin_bit_cast(half_t, (unsigned short)((sa & 2u) ? (sd >> 16) : (sd & 0xFFFFu)));
#pragma unroll
                    for (int t = 0; t < 8; ++t) {
                        // ranks 256 uu + 64 ly + 8 t .. + 7; past the end the codes are zero and T is read inside the row
                        const int col = min(256 * uu + 64 * ly + 8 * t, rp - 8);
                        const half8_t bv = *reinterpret_cast<const half8_t *>(t_lds + trow * ldt + col);
                        const half8_t av = codes_to_half8(cur.r[4 * x + (t >> 2)][t & 3]) * sc;
                        if (t & 1)
                            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc1, 0, 0, 0);
                        else
                            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, bv, acc0, 0, 0, 0);
                    }
                }
            }
        }
        if (j != nIe - 1) return;
        // ---- end of the round ----
        if (nP == nIe) {             // no rank steps on this wavefront
            acc0 = (acc0 + acc1) * sc4;
            acc1 = float4_t{0.f, 0.f, 0.f, 0.f};
            if (!t_ready) {          // it still takes part in the barriers
                meet_for_t();
                t_ready = true;
            }
        }
        // lane holds token lx, rows 16 ot + 4 ly .. + 3
        float4_t y = acc0 + acc1;
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
                if (LR && (a.mode & 4)) {
                    const half4_t old = *reinterpret_cast<const half4_t *>(yp);
#pragma unroll
                    for (int v = 0; v < 4; ++v) y[v] += (float)old[v];
                }
                const half4_t h = {(half_t)y[0], (half_t)y[1], (half_t)y[2], (half_t)y[3]};
                *reinterpret_cast<half4_t *>(yp) = h;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (ob + v < a.n) yp[v] = (half_t)(LR && (a.mode & 4) ? y[v] + (float)yp[v] : y[v]);
            }
        }
        if (S > 1 && r + 1 < rounds) __syncthreads();      // the partial sums are read before the next round writes
    };

    // Items in pairs: set A, then set B; an odd total ends with a pair whose second half is skipped
    // (its loads were all past the end and brought zeros).
    int cr = 0, cj = 0;              // item being worked on
    for (int g = 0; g < total; g += 2) {
        __builtin_amdgcn_sched_barrier(0);
        step(cr, cj, bufA);
        advance(cr, cj);
        __builtin_amdgcn_sched_barrier(0);
        issue_item(ir, ij, bufA);
        advance(ir, ij);
        __builtin_amdgcn_sched_barrier(0);
        if (g + 1 < total) {
            step(cr, cj, bufB);
            advance(cr, cj);
        }
        __builtin_amdgcn_sched_barrier(0);
        issue_item(ir, ij, bufB);
        advance(ir, ij);
        __builtin_amdgcn_sched_barrier(0);
    }
}

template <bool Q4, bool LR = false>
__global__ __launch_bounds__(kFusedMaxThreads, kFusedWavesPerSimd) void decode_fused_kernel(FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) half_t lds[];
    // mode & 3: 0 = every workgroup in the R role, 1 = every workgroup in the Y role, 2 = the first n_r in
    // the R role and the others in the Y role (one copy of each role's code)
    const int split = (a.mode & 3) == 2 ? a.n_r : ((a.mode & 3) == 0 ? (int)gridDim.x : 0);
    if ((int)blockIdx.x < split)
        role_r<Q4>(a, lds, blockIdx.x);
    else
        role_y<Q4, LR>(a, lds, (int)blockIdx.x - split, (int)gridDim.x - split);
}

static int pad_tokens16(int m) { return m <= 1 ? 1 : (m <= 4 ? 4 : (m <= 8 ? 8 : 16)); }

// Geometry for one workgroup size: all of X in LDS at once if it fits, else
// chunks of 4096, 2048 or 1024 inputs in two buffers; the shares of the R role;
// the largest S (wavefronts per row tile) with which every workgroup is
// resident at once.
static FusedPlan plan_fused_waves(int n, int k, int rank_pad, int m, int waves, const DeviceInfo &dev, size_t lds_limit)
{
    FusedPlan p{};
    p.mp = pad_tokens16(m);
    p.kpad = (k + 1023) / 1024 * 1024;
    p.waves = waves;
    const long wtiles = (n + 15) / 16;
    const int kcs[4] = {p.kpad, 4096, 2048, 1024};
    // LDS of a compute unit; slim_decode_override can lower what the geometry plans with (tests: chunks on small layers)
    const size_t lds_cu = dev.lds;
    size_t lds_cap = lds_cu;
    if (lds_limit >= 16 * 1024 && lds_limit < lds_cap) lds_cap = lds_limit;
    for (int ci = 0; ci < 4 && !p.ok; ++ci) {
        const int kc = kcs[ci];
        if (ci > 0 && kc >= p.kpad) continue;
        const int nch = (p.kpad + kc - 1) / kc;
        const int hc = kc / 512;
        if (nch > 1 && rank_pad > kc) continue;          // T takes the place of an X buffer
        // helpers: they stage X (about 32 KiB per wavefront in flight) and fetch T (8 loads per
        // lane and batch).  Beside 8 working wavefronts up to 4 of them fit the compute unit
        // anyway; beside 4, fewer helpers mean more workgroups per compute unit.
        // (with more than 8 tokens eight: T is then one batch per lane, and the workgroup has
        // the compute unit to itself anyway)
        int helpers = m > 8 ? 8 : 4;
        if (waves == 7) {
            helpers = 1;                               // up to 4 tokens: X and T are a few loads per lane
        } else if (waves < 8) {
            const int by_t = m <= 4 ? 1 : (m <= 8 ? 2 : 4);
            const int by_x = (int)(((size_t)m * kc * 2 + 32767) / 32768);
            helpers = by_x > by_t ? by_x : by_t;
            if (helpers > 4) helpers = 4;
        }
        const int total = waves + helpers;            // wavefronts of a workgroup
        // Shares of the inputs in the R role (1, 2 or 4): up to one unit per wavefront, so that
        // T is there early; fewer if the workgroups would no longer all be resident.
        const int units = (k + 255) / 256;
        const int want = (units + 7) / 8;              // as if eight wavefronts: also spreads R over more compute units
        const int kh_max = want <= 1 ? 1 : (want <= 2 ? 2 : kMaxShares);
        const size_t lds_x = nch == 1 ? (size_t)m * ((kc + kLdsPad) + (rank_pad + kLdsPad)) * sizeof(half_t)
                                      : (size_t)2 * m * (kc + kLdsPad) * sizeof(half_t);
        const size_t red_r = (size_t)(total - 1) * kWave * 16;
        for (int S = waves; S >= 1; S /= 2) {
            if (waves % S) continue;                         // whole row tiles per workgroup
            if (nch > 1 && (S > hc || hc % S)) continue;     // every wavefront has the same items in every chunk
            const int tpw = waves / S;
            const size_t red_y = S > 1 ? (size_t)tpw * (S - 1) * kWave * 16 : 0;
            const size_t lds = lds_x + red_y > red_r ? lds_x + red_y : red_r;
            if (lds > lds_cap) continue;
            // Workgroups a compute unit is sure to hold: the wavefronts of a workgroup are dealt to the
            // four SIMDs in turn, so one SIMD gets ceil(total / 4) of them, and a SIMD holds
            // kFusedWavesPerSimd.  (Counting wavefronts per compute unit alone admitted three
            // workgroups of five, which the hardware does not always place: the last ones then
            // started only when the R role had ended, 7 us late on the largest layer.)
            long per_cu = kFusedWavesPerSimd / ((total + 3) / 4);
            if (per_cu > (long)(lds_cu / lds)) per_cu = (long)(lds_cu / lds);
            const long wgs = (wtiles + tpw - 1) / tpw;
            int kh = kh_max;
            while (kh > 1 && wgs + (long)(rank_pad / 16) * kh > dev.cus * per_cu) kh /= 2;
            const int n_r = (rank_pad / 16) * kh;
            if (wgs + n_r <= dev.cus * per_cu) {
                p.S = S;
                p.ygrid = (int)wgs;
                p.lds = lds;
                p.kc = kc;
                p.nch = nch;
                p.helpers = helpers;
                p.kh = kh;
                p.upk = (units + kh - 1) / kh;
                p.n_r = n_r;
                p.ok = n_r <= 512;
                break;
            }
        }
    }
    return p;
}

// Which layers take this path, and with what geometry.  Workgroups of 8 working
// wavefronts, one per compute unit, measured best wherever they fit; layers with
// more row tiles than that allows run, up to 4 tokens, workgroups of 7 working
// wavefronts and one helper (two per compute unit, every SIMD evenly loaded:
// 28672 x 8192 is then 256 workgroups of 7 row tiles), else workgroups of 4
// working wavefronts, two per compute unit.
FusedPlan plan_fused(int n, int k, int rank_pad, int m)
{
    // The plan is a pure function of these seven numbers; a decode loop asks for the same few over and
    // over, so each thread keeps the last ones it computed.
    struct Key {
        int n, k, rank_pad, m, cus;
        size_t lds, limit;
        bool operator==(const Key &o) const
        {
            return n == o.n && k == o.k && rank_pad == o.rank_pad && m == o.m && cus == o.cus && lds == o.lds && limit == o.limit;
        }
    };
    constexpr int kSlots = 16;
    thread_local Key keys[kSlots];
    thread_local FusedPlan plans[kSlots];
    thread_local int used = 0, next = 0;
    const DeviceInfo dev = device_info();
    const Key key{n, k, rank_pad, m, dev.cus, dev.lds, decode_lds_limit()};
    for (int i = 0; i < used; ++i)
        if (keys[i] == key) return plans[i];
    FusedPlan p = plan_fused_waves(n, k, rank_pad, m, 8, dev, key.limit);
    if (!p.ok && m <= 4) p = plan_fused_waves(n, k, rank_pad, m, 7, dev, key.limit);
    if (!p.ok) p = plan_fused_waves(n, k, rank_pad, m, 4, dev, key.limit);
    keys[next] = key;
    plans[next] = p;
    next = (next + 1) % kSlots;
    if (used < kSlots) ++used;
    return p;
}

static std::atomic<unsigned> g_epoch{0};

// mode: 2 = one launch, 1 = the two roles as two launches.  lowrank: 0 = the layer; 1, 2 = the
// low-rank term alone on the layer's fp16 adapters (its packed buffers are not read), 2 adds to Y.
int launch_decode_fused(const slim_layer *layer, const half_t *X, int m, half_t *Y, void *T, unsigned *err, unsigned *epoch_ctr, const FusedPlan &p, int mode, hipStream_t st, int lowrank)
{
    if (lowrank && (layer->adapter_bits == 4 || p.n_r == 0)) return SLIM_ERR_SHAPE;
    FusedArgs a{};
    a.qvals = layer->qvals;
    a.meta = layer->meta;
    a.scale = layer->scale;
    a.R = reinterpret_cast<const half_t *>(layer->R);
    a.L = reinterpret_cast<const half_t *>(layer->L);
    a.Rq = layer->Rq;
    a.Lq = layer->Lq;
    a.Rs = reinterpret_cast<const half_t *>(layer->Rs);
    a.Ls = reinterpret_cast<const half_t *>(layer->Ls);
    a.X = X;
    a.Y = Y;
    a.T = static_cast<uint4_t *>(T);
    a.err = err;
    unsigned e = ++g_epoch & 0x7FFFFFFFu;
    if (e == 0) e = ++g_epoch & 0x7FFFFFFFu;      // a zero-filled workspace must not look valid: epoch 0 is never used
    a.epoch = e;
    a.epoch_ptr = nullptr;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) == hipSuccess && cap == hipStreamCaptureStatusActive) {
        hipLaunchKernelGGL(decode_epoch_bump_kernel, dim3(1), dim3(1), 0, st, epoch_ctr);
        a.epoch_ptr = epoch_ctr;
    }
    a.n = layer->shape.n;
    a.k = layer->shape.k;
    a.rank_pad = layer->rank_pad;
    a.rank = layer->shape.rank;
    a.m = m;
    a.kpad = p.kpad;
    a.kc = p.kc;
    a.nch = p.nch;
    a.S = p.S;
    a.n_r = p.n_r;
    a.helpers = p.helpers;
    a.kh = p.kh;
    a.upk = p.upk;
    const dim3 blk((p.waves + p.helpers) * kWave);
    const bool q4 = layer->adapter_bits == 4 && p.n_r > 0;
    auto launch = [&](unsigned grid) {
        if (lowrank)
            hipLaunchKernelGGL((decode_fused_kernel<false, true>), dim3(grid), blk, p.lds, st, a);
        else if (q4)
            hipLaunchKernelGGL(decode_fused_kernel<true>, dim3(grid), blk, p.lds, st, a);
        else
            hipLaunchKernelGGL(decode_fused_kernel<false>, dim3(grid), blk, p.lds, st, a);
    };
    if (mode == 3 && p.n_r > 0) {
        // test of the bounded wait: the Y role alone, so the pieces of T it waits for never come; the
        // helpers give up after a few polls, the outputs are NaN and the error word is set
        a.mode = 1 | 8;
        launch((unsigned)p.ygrid);
    } else if (mode == 2 || p.n_r == 0) {
        a.mode = p.n_r == 0 ? 1 : (lowrank == 2 ? 6 : 2);
        launch((unsigned)(p.n_r + p.ygrid));
    } else {
        a.mode = 0;
        launch((unsigned)p.n_r);
        a.mode = 1;
        launch((unsigned)p.ygrid);
    }
    return hip_status(hipGetLastError());
}

}  // namespace slim
