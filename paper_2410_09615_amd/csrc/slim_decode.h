// Device code shared by the decode kernels (slim_gemv.hip, slim_gemv_fused.hip).
#pragma once

#include "slim_internal.h"

namespace slim {

constexpr int kMaxTokens = 16;
constexpr int kLdsPad = 8;                 // halves of padding per LDS row (16 B)

struct UnitRegs {
    uint4_t r[8];  // the 8 x 128-bit loads of one unit
};

// 128-bit load of code bytes; the two 64-bit pieces of positions of a lane's
// 128 inputs (256 bytes apart in the packed layout) as one register quad.
__device__ __forceinline__ uint4_t load_q16(const uint8_t *p) { return *reinterpret_cast<const uint4_t *>(p); }
__device__ __forceinline__ uint4_t load_m16(const uint8_t *p)
{
    const uint2_t lo = *reinterpret_cast<const uint2_t *>(p), hi = *reinterpret_cast<const uint2_t *>(p + 256);
    return uint4_t{lo[0], lo[1], hi[0], hi[1]};
}

// One half (512 inputs) of a packed unit: 8 sparse matrix instructions
// (V_SMFMAC_F32_16X16X64_F16) on registers r[3 H] and r[3 H + 1] (codes) and
// r[3 H + 2] (positions).  xh is the lane's B-operand row at the first input
// of the half, already moved to the lane's share: + 128 (ly >> 1) + 8 (ly & 1).
// B operand of instruction t: values 0-7 pair with the A lanes of k-block
// (ly >> 1), values 8-15 with k-block 2 + (ly >> 1); inside the lane's 128
// inputs they are the 8 inputs at 16 t + 8 (ly & 1).
template <int H>
__device__ __forceinline__ void packed_half(const UnitRegs &b, const half_t *xh, float4_t &acc0, float4_t &acc1)
{
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        const uint32_t qd = t < 4 ? b.r[3 * H][t] : b.r[3 * H + 1][t - 4];
        const half8_t av = codes_to_half8(qd);
        const half8_t b1 = *reinterpret_cast<const half8_t *>(xh + 16 * t);
        const half8_t b2 = *reinterpret_cast<const half8_t *>(xh + 256 + 16 * t);
        const half16_t bv = __builtin_shufflevector(b1, b2, 0, 1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15);
        const int idx = (int)b.r[3 * H + 2][t >> 1];
        // even t: index bits 15..0, odd t: bits 31..16 of the position dword
        if (t & 1)
            acc1 = __builtin_amdgcn_smfmac_f32_16x16x64_f16(av, bv, acc1, idx, 0, 1);
        else
            acc0 = __builtin_amdgcn_smfmac_f32_16x16x64_f16(av, bv, acc0, idx, 0, 0);
    }
}

// Geometry and launch of the one-launch decode path (slim_gemv_fused.hip).
struct FusedPlan {
    bool ok;            // the layer and token count fit this path
    int mp, kpad, kc, nch, S, waves, helpers, n_r, kh, upk, ygrid;
    size_t lds;
};
FusedPlan plan_fused(int n, int k, int rank_pad, int m);
// mode 2: one launch; mode 1: the two roles as two launches
// err, epoch_ctr: two control words of the workspace (error flag; call counter used under stream capture)
// lowrank 1, 2: the low-rank term alone on the layer's fp16 adapters (packed buffers not read); 2 adds to Y
int launch_decode_fused(const slim_layer *layer, const half_t *X, int m, half_t *Y, void *T, unsigned *err, unsigned *epoch_ctr,
                        const FusedPlan &p, int mode, hipStream_t st, int lowrank = 0);

}  // namespace slim
