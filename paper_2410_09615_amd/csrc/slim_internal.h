// Internal helpers shared by the libslim translation units (device + host).
// Not part of the public boundary (include/slim.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "slim.h"

namespace slim {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef _Float16 half16_t __attribute__((ext_vector_type(16)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));

constexpr int kWave = 64;

// Sum over the 64 lanes of a wavefront; every lane gets the total.
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
    return v;
}

// Two's-complement nibble -> int in [-8, 7].
__device__ __forceinline__ int nibble_to_int(uint32_t v) { return (int)(v & 7u) - (int)(v & 8u); }

// Code bytes -> fp16 in matrix-operand order.  codes_bias() turns the four
// two's-complement nibble pairs of a dword into offset-by-8 form; code_pair()
// then yields group g's two values: (low nibble, high nibble) of byte g.
__device__ __forceinline__ uint32_t codes_bias(uint32_t q) { return q ^ 0x88888888u; }

__device__ __forceinline__ half2_t code_pair(uint32_t x, int g)
{
    const half2_t mul = {(half_t)1.0f, (half_t)0.0625f};
    const half2_t add = {(half_t)-1032.0f, (half_t)-72.0f};
    // bytes [b, 0x64, b, 0x64]: both halves read 1024 + b; keep the low
    // nibble in the low half and the high nibble (x16) in the high half.
    // Selector bytes 4..7 pick bytes of the first operand, 0..3 of the second.
    const uint32_t sel = ((4u + g) << 16) | (4u + g);
    uint32_t v = __builtin_amdgcn_perm(x, 0x64646464u, sel);
    v &= 0x64F0640Fu;
    const half2_t h = __builtin_bit_cast(half2_t, v);
    return __builtin_elementwise_fma(h, mul, add);   // (1024+n0)-1032, (1024+16 n1)/16-72
}

// Four packed groups (one dword of code bytes) -> eight fp16 values: value 2g
// is the low nibble of byte g, value 2g+1 its high nibble.
__device__ __forceinline__ half8_t codes_to_half8(uint32_t q)
{
    const uint32_t x = codes_bias(q);
    half8_t out;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const half2_t h = code_pair(x, g);
        out[2 * g] = h[0];
        out[2 * g + 1] = h[1];
    }
    return out;
}

// ---- device layout of the fp16 adapters (what slim_pack_adapters writes) ----
// A matrix [rows][K] is stored as tiles of 32 rows x 16 columns, 1 KiB each,
// row tile major; inside a tile the 64 pieces of 8 halves (16 bytes) are ordered
// (column half, row): piece (r, h) at ((h * 32) + r) * 16.  That is the order in
// which the 64 lanes of a wavefront hold the A operand of a 32 x 32 x 16 matrix
// instruction, so one load instruction reads one contiguous KiB; the 16 x 16 x 32
// instruction of the decode path reads four runs of 256 bytes.  rows is padded
// to 32 and K to 16 with zeros.
__host__ __device__ inline uint32_t tl_rows(int rows) { return (uint32_t)(rows + 31) / 32 * 32; }
__host__ __device__ inline uint32_t tl_cols(int K) { return (uint32_t)(K + 15) / 16 * 16; }
__host__ __device__ inline size_t tl_bytes(int rows, int K) { return (size_t)tl_rows(rows) * tl_cols(K) * 2; }
// byte offset of the piece holding columns 8 c8 .. 8 c8 + 7 of `row`
__host__ __device__ inline uint32_t tl_piece(uint32_t row, uint32_t c8, uint32_t kcols)
{
    return ((row >> 5) * (kcols >> 4) + (c8 >> 1)) * 1024u + (((c8 & 1u) << 5) + (row & 31u)) * 16u;
}

// ---- device layout of the packed weights (what slim_pack writes) ----
// The canonical bytes (qvals[o][g], one per group of 4 inputs; meta[o][g / 2]) are
// stored as tiles of 32 rows x 128 inputs, row tile major: 1 KiB of codes and
// 512 bytes of positions per tile.  Inside a tile the 64 pieces of 64 inputs
// (16 code bytes / 8 position bytes) are ordered (input half, row): lane order of
// the sparse 32 x 32 x 32 matrix instruction, so one load instruction reads one
// contiguous KiB (codes) or 512 bytes (positions).  Rows are padded to 32 and
// inputs to 128 with zero bytes.
__host__ __device__ inline uint32_t pk_ktiles(int k) { return (uint32_t)(k + 127) / 128; }
__host__ __device__ inline size_t pk_qbytes(int n, int k) { return (size_t)((n + 31) / 32) * pk_ktiles(k) * 1024; }
__host__ __device__ inline size_t pk_mbytes(int n, int k) { return (size_t)((n + 31) / 32) * pk_ktiles(k) * 512; }
// byte offsets of canonical qvals[o][g] and meta[o][b]
__host__ __device__ inline size_t pk_qoff(uint32_t o, uint32_t g, uint32_t kt)
{
    return ((size_t)(o >> 5) * kt + (g >> 5)) * 1024u + ((((g >> 4) & 1u) << 5) + (o & 31u)) * 16u + (g & 15u);
}
__host__ __device__ inline size_t pk_moff(uint32_t o, uint32_t b, uint32_t kt)
{
    return ((size_t)(o >> 5) * kt + (b >> 4)) * 512u + ((((b >> 3) & 1u) << 5) + (o & 31u)) * 8u + (b & 7u);
}

// ---- device layout of 4-bit adapters (what slim_pack_adapters_q4 writes) ----
// Codes of a matrix [rows][K] (two's-complement nibbles, the even column in the
// low nibble) are stored as tiles of 16 rows x 256 columns, 2 KiB each, row tile
// major; inside a tile the piece of row r and quarter q (64 columns, 32 bytes)
// starts at (4 r + q) * 32: lane (row, quarter) of a wavefront reads its 64
// columns with two 128-bit loads and the wavefront reads the tile as one
// contiguous run.  Rows are padded to 16 and columns to 256 with zero codes.
// Scales: fp16 [rows16][2 * tiles per row], one per group of 128 columns.
__host__ __device__ inline uint32_t q4_ctiles(int K) { return (uint32_t)(K + 255) / 256; }
__host__ __device__ inline uint32_t q4_rows(int rows) { return (uint32_t)(rows + 15) / 16 * 16; }
__host__ __device__ inline uint32_t q4_groups(int K) { return 2 * q4_ctiles(K); }
__host__ __device__ inline size_t q4_code_bytes(int rows, int K) { return (size_t)(q4_rows(rows) / 16) * q4_ctiles(K) * 2048; }
__host__ __device__ inline size_t q4_scale_bytes(int rows, int K) { return (size_t)q4_rows(rows) * q4_groups(K) * 2; }
// byte offset of the piece holding columns 64 c64 .. 64 c64 + 63 of `row`
__host__ __device__ inline uint32_t q4_piece(uint32_t row, uint32_t c64, uint32_t ctiles)
{
    return ((row >> 4) * ctiles + (c64 >> 2)) * 2048u + ((row & 15u) * 4u + (c64 & 3u)) * 32u;
}

#ifdef __HIPCC__
// ---- buffer loads: descriptor + 32-bit byte offset, out-of-range reads return zero ----
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

__device__ __forceinline__ uint2_t load8(rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(uint2_t, __builtin_amdgcn_raw_buffer_load_b64(r, (int)(lane_off + uniform_off), 0, 0));
}

__device__ __forceinline__ half_t load_half(rsrc_t r, uint32_t lane_off, uint32_t uniform_off)
{
    return __builtin_bit_cast(half_t, __builtin_amdgcn_raw_buffer_load_b16(r, (int)(lane_off + uniform_off), 0, 0));
}

#endif

// What the planners need to know of the device that is current: compute units and LDS bytes per compute
// unit, read once per device from its properties (the nominal MI355X figures, 256 and 160 KiB, where no
// device can be asked: the planners are host logic and also run without one).
struct DeviceInfo {
    int cus;
    size_t lds;
};
DeviceInfo device_info();

// Process-wide test and measurement control of the decode geometry (slim_decode_override).
int decode_path_override();      // -1: automatic, 0: two-launch kernels, 1: the roles as two launches, 2: one launch
size_t decode_lds_limit();       // 0: the device's LDS; else bytes the one-launch geometry may plan with

// Device address of the library's own scratch array on the current device (slim_gemv.hip).
int scratch_of_current_device(void **out);

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int hip_status(hipError_t e) { return e == hipSuccess ? SLIM_OK : SLIM_ERR_HIP; }

// Workspace carve-up used by the forward entry points (offsets in bytes,
// each a multiple of 256).
struct WorkspacePlan {
    size_t dec_off, dec_bytes;    // decode state: 256 B of control words, then T fp32 [16][rank_pad] of the two-launch path (room for two),
                                  // then (one-launch path) T as up to four planes [16][rank_pad / 4] of 16-byte pieces
    size_t t16_off;               // the last, as an offset into the workspace
    size_t t_off, t_bytes;        // gemm: T = X R^T as fp16 [m][rank_pad]
    size_t acc_off, acc_bytes;    // decode: partial quantized term, fp32 [slots][m][n]
    size_t part_off, part_bytes;  // gemm: split-K partials of T, fp32 [splits][m][rank_pad]
    size_t exp_off, exp_bytes;    // 4-bit adapters expanded to fp16 (adapter layout): L then R
    int splits;                   // split-K factor of the T product
    size_t total;
};

// Geometry of a decode call: padded token count, k-chunk per block, inputs per
// packed-row task, tasks per row tile in a full chunk, partial slots.
struct DecodePlan {
    int mp, kc, nch, sl, rsl, wsl_full, slots;
};

DecodePlan plan_decode(int n, int k, int rank_pad, int m);

WorkspacePlan plan_workspace(int32_t n, int32_t k, int32_t rank_pad, int32_t m, bool q4);

// 4-bit adapters of a layer -> fp16 in the workspace; returns the layer to run with (fp16 adapters).
int expand_q4_adapters(const slim_layer *layer, const WorkspacePlan &w, char *ws, slim_layer *out, hipStream_t st);

}  // namespace slim
