// slim_pack / slim_unpack / slim_pack_adapters: the encoding side of the layer.
//
// slim_pack is a streaming kernel bound by HBM: it reads 4 bytes per weight
// and writes 3 bits per weight.  One workgroup owns one output row: it keeps
// the row in registers while the row maximum is reduced (so W is read from
// memory once), then each lane encodes the groups of 4 it holds.
#include "slim_internal.h"

namespace slim {

constexpr int kPackSlotsMax = 12;   // float4 groups a lane keeps at most: rows up to 4 * 1024 * 12 inputs stay in registers

// Kept positions of one group: order by (|w| descending, position ascending),
// take two, return them as i0 < i1 packed as i0 | (i1 << 2).
__device__ __forceinline__ uint32_t keep_two(float a0, float a1, float a2, float a3)
{
    int first = 0;
    float best = a0;
    if (a1 > best) { best = a1; first = 1; }
    if (a2 > best) { best = a2; first = 2; }
    if (a3 > best) { best = a3; first = 3; }
    int second = -1;
    float sb = -1.0f;
    if (first != 0 && a0 > sb) { sb = a0; second = 0; }
    if (first != 1 && a1 > sb) { sb = a1; second = 1; }
    if (first != 2 && a2 > sb) { sb = a2; second = 2; }
    if (first != 3 && a3 > sb) { sb = a3; second = 3; }
    int i0 = first < second ? first : second;
    int i1 = first < second ? second : first;
    return (uint32_t)i0 | ((uint32_t)i1 << 2);
}

__device__ __forceinline__ uint32_t quantize_code(float w, float s)
{
    float q = rintf(w / s);               // IEEE division, round half to even
    q = fminf(fmaxf(q, -8.0f), 7.0f);
    return (uint32_t)(int)q & 0xFu;
}

// Encode one group: returns the qvals byte, *m4 the metadata nibble.  sal: the
// saliency of the four inputs (all ones: the magnitude mask); the products are
// single binary32 multiplications.
__device__ __forceinline__ uint32_t encode_group(float4 v, float s, uint32_t *m4, float4 sal = make_float4(1.f, 1.f, 1.f, 1.f))
{
    uint32_t sel = keep_two(fabsf(v.x) * sal.x, fabsf(v.y) * sal.y, fabsf(v.z) * sal.z, fabsf(v.w) * sal.w);
    uint32_t i0 = sel & 3u, i1 = sel >> 2;
    float w[4] = {v.x, v.y, v.z, v.w};
    float w0 = i0 == 0 ? w[0] : (i0 == 1 ? w[1] : w[2]);
    float w1 = i1 == 1 ? w[1] : (i1 == 2 ? w[2] : w[3]);
    *m4 = sel;
    return quantize_code(w0, s) | (quantize_code(w1, s) << 4);
}

// THREADS lanes per row; SLOTS = float4 groups of the row each lane keeps in
// registers (the row has at most 4 THREADS SLOTS inputs); 0 = rows of any
// length, read twice.  Few slots per lane keep the register count low enough
// for eight wavefronts per SIMD, which is what hides the load latency here.
// The kernel is as much bound by its vector ALU work (top-2 selection, two IEEE
// divisions per group) as by memory, so the stores stay plain byte stores: lane
// t writes group t + i THREADS of slot i, whose place in the packed layout is a
// per-lane base plus a constant per slot.
// EX: the variant behind slim_pack_ex: saliency [k] (or null) weighs the
// magnitudes in the 2:4 choice, scale_in [n] (or null) replaces AbsMax / 7.
template <int THREADS, int SLOTS, bool EX = false>
__global__ __launch_bounds__(THREADS) void pack_kernel(const float *__restrict__ W, int n, int k,
                                                            uint8_t *__restrict__ qvals,
                                                            uint8_t *__restrict__ meta,
                                                            float *__restrict__ scale,
                                                            const float *__restrict__ saliency = nullptr,
                                                            const float *__restrict__ scale_in = nullptr)
{
    __shared__ float wave_part[THREADS / kWave];
    const int ngroups = k / 4;
    const int tid = threadIdx.x;
    const uint32_t kt = pk_ktiles(k);
    const int gpad = (int)kt * 32;             // groups per row of the packed layout
    const int npad = (n + 31) / 32 * 32;
    // Workgroups go to the 8 dies round-robin and each die has its own L2.  The 32
    // rows of a row tile write into the same cache lines, so they are kept on one
    // die: die x takes a contiguous range of row tiles, its workgroups walk that
    // range row by row.  (The grid is a multiple of 8.)
    const int die = blockIdx.x & 7, local = blockIdx.x >> 3, per_die = gridDim.x >> 3;
    const int rows_per_die = ((npad / 32 + 7) / 8) * 32;
    const int o_end = min(npad, (die + 1) * rows_per_die);
    for (int o = die * rows_per_die + local; o < o_end; o += per_die) {
        // this lane's byte of slot 0 in the packed layout (group tid, position byte tid / 2)
        uint8_t *const ql = qvals + pk_qoff(o, tid, kt);
        uint8_t *const ml = meta + pk_moff(o, tid >> 1, kt);
        constexpr size_t q_slot = (size_t)(THREADS / 32) * 1024, m_slot = (size_t)(THREADS / 32) * 512;
        if (o >= n) {
            // padding row of the last row tile: zero bytes
            for (int g = tid, i = 0; g < gpad; g += THREADS, ++i) {
                ql[i * q_slot] = 0;
                if ((g & 1) == 0) ml[i * m_slot] = 0;
            }
            continue;
        }
        const float4 *row = reinterpret_cast<const float4 *>(W + (size_t)o * k);
        constexpr bool CACHED = SLOTS > 0;
        float4 cache[CACHED ? SLOTS : 1];
        float a = 0.0f;
        if (CACHED) {
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) {
                int g = tid + i * THREADS;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (g < ngroups) v = row[g];
                cache[i] = v;
                a = fmaxf(a, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
            }
        } else {
            for (int g = tid; g < ngroups; g += THREADS) {
                float4 v = row[g];
                a = fmaxf(a, fmaxf(fmaxf(fabsf(v.x), fabsf(v.y)), fmaxf(fabsf(v.z), fabsf(v.w))));
            }
        }
        a = wave_max(a);
        __syncthreads();                       // wave_part is reused across rows
        if ((tid & (kWave - 1)) == 0) wave_part[tid / kWave] = a;
        __syncthreads();
        a = wave_part[0];
#pragma unroll
        for (int w = 1; w < THREADS / kWave; ++w) a = fmaxf(a, wave_part[w]);
        float s = (a == 0.0f) ? 1.0f : a / 7.0f;
        if (EX && scale_in) s = scale_in[o];
        if (tid == 0) scale[o] = s;

        // Lanes g and g^1 hold the two groups of one position byte (the stride is
        // even, so both are active together).  Groups past the end of the row
        // (padding of the last tile) are zero bytes.
        auto emit = [&](int i, int g, float4 v) {
            uint32_t q = 0, m4 = 0;
            if (g < ngroups) {
                if (EX && saliency)
                    q = encode_group(v, s, &m4, reinterpret_cast<const float4 *>(saliency)[g]);
                else
                    q = encode_group(v, s, &m4);
            }
            const uint32_t other = __shfl_xor(m4, 1, kWave);
            if (g < gpad) {
                ql[i * q_slot] = (uint8_t)q;
                if ((g & 1) == 0) ml[i * m_slot] = (uint8_t)(m4 | (other << 4));
            }
        };
        if (CACHED) {
#pragma unroll
            for (int i = 0; i < SLOTS; ++i) emit(i, tid + i * THREADS, cache[i]);
        } else {
            for (int g0 = 0, i = 0; g0 < gpad; g0 += THREADS, ++i) {
                const int g = g0 + tid;
                emit(i, g, g < ngroups ? row[g] : make_float4(0.f, 0.f, 0.f, 0.f));
            }
        }
    }
}

// One lane decodes one group: 4 codes and 4 mask bytes, one dword store each.
__global__ __launch_bounds__(256) void unpack_kernel(const uint8_t *__restrict__ qvals,
                                                     const uint8_t *__restrict__ meta, int n, int k,
                                                     int8_t *__restrict__ codes, uint8_t *__restrict__ mask)
{
    const uint32_t ngroups = (uint32_t)k / 4, kt = pk_ktiles(k);
    const size_t total_groups = (size_t)n * ngroups;
    for (size_t g = blockIdx.x * (size_t)blockDim.x + threadIdx.x; g < total_groups;
         g += (size_t)gridDim.x * blockDim.x) {
        const uint32_t o = (uint32_t)(g / ngroups), gi = (uint32_t)(g - (size_t)o * ngroups);
        uint32_t q = qvals[pk_qoff(o, gi, kt)];
        uint32_t m4 = (meta[pk_moff(o, gi >> 1, kt)] >> (4 * (gi & 1))) & 0xFu;
        uint32_t i0 = m4 & 3u, i1 = m4 >> 2;
        uint32_t c0 = (uint32_t)nibble_to_int(q & 0xFu) & 0xFFu;
        uint32_t c1 = (uint32_t)nibble_to_int(q >> 4) & 0xFFu;
        // a malformed nibble with i1 == i0 keeps the later write, as a
        // sequential decoder would
        uint32_t cw = (i0 == i1) ? (c1 << (8 * i1)) : ((c0 << (8 * i0)) | (c1 << (8 * i1)));
        uint32_t mw = (1u << (8 * i0)) | (1u << (8 * i1));
        reinterpret_cast<uint32_t *>(codes)[g] = cw;
        reinterpret_cast<uint32_t *>(mask)[g] = mw;
    }
}

// dst (tiled layout of a [rows][kcols] matrix, see slim_internal.h) <- src
// [src_rows][src_cols] row-major, zero outside the source.  One lane per piece
// of 8 halves, pieces in destination order: the stores are contiguous.
__global__ __launch_bounds__(256) void tile_copy_kernel(const uint16_t *__restrict__ src, int src_rows,
                                                        int src_cols, uint16_t *__restrict__ dst, uint32_t rows,
                                                        uint32_t kcols)
{
    const size_t pieces = (size_t)rows * (kcols / 8);
    for (size_t p = blockIdx.x * (size_t)blockDim.x + threadIdx.x; p < pieces;
         p += (size_t)gridDim.x * blockDim.x) {
        const uint32_t tile = (uint32_t)(p >> 6), q = (uint32_t)p & 63u;
        const uint32_t rt = tile / (kcols >> 4), kt = tile - rt * (kcols >> 4);
        const int row = (int)(rt * 32 + (q & 31u));
        const int c0 = (int)(kt * 16 + (q >> 5) * 8);
        uint16_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = (row < src_rows && c0 + e < src_cols) ? src[(size_t)row * src_cols + c0 + e] : (uint16_t)0;
        uint4_t out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = (uint32_t)v[2 * e] | ((uint32_t)v[2 * e + 1] << 16);
        reinterpret_cast<uint4_t *>(dst)[p] = out;
    }
}

// Workgroups for slim_pack: one per row up to `cap`, a multiple of 8.
static int pack_grid(int npad, int cap)
{
    int g = npad < cap ? npad : cap;
    return (g + 7) / 8 * 8;
}

static int grid_for(size_t items, int threads, int cap = 256 * 16)
{
    size_t b = (items + threads - 1) / threads;
    if (b > (size_t)cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

}  // namespace slim

using namespace slim;

template <bool EX>
static int launch_pack(const float *W, slim_shape shape, uint8_t *qvals, uint8_t *meta, float *scale,
                       const float *saliency, const float *scale_in, hipStream_t st)
{
    const int npad = (shape.n + 31) / 32 * 32;      // the padding rows of the last tile get a workgroup too
    // lanes per row: enough that a lane keeps at most 4 groups, up to 1024
    const int groups = shape.k / 4;
    // (two rounds of resident workgroups at most; a workgroup walks the rows it owns)
#define SLIM_PACK_LAUNCH(T, S)                                                                                    \
    hipLaunchKernelGGL((pack_kernel<T, S, EX>), dim3(pack_grid(npad, 256 * (4096 / T))), dim3(T), 0, st, W, shape.n, \
                       shape.k, qvals, meta, scale, saliency, scale_in)
    if (groups <= 256 * 2)
        SLIM_PACK_LAUNCH(256, 2);
    else if (groups <= 256 * 4)
        SLIM_PACK_LAUNCH(256, 4);
    else if (groups <= 512 * 4)
        SLIM_PACK_LAUNCH(512, 4);
    else if (groups <= 1024 * 4)
        SLIM_PACK_LAUNCH(1024, 4);
    else if (groups <= 1024 * 8)
        SLIM_PACK_LAUNCH(1024, 8);
    else if (groups <= 1024 * kPackSlotsMax)
        SLIM_PACK_LAUNCH(1024, kPackSlotsMax);
    else
        SLIM_PACK_LAUNCH(1024, 0);
#undef SLIM_PACK_LAUNCH
    return hip_status(hipGetLastError());
}

extern "C" int slim_pack(const float *W, slim_shape shape, uint8_t *qvals, uint8_t *meta, float *scale,
                         void *stream)
{
    if (!W || !qvals || !meta || !scale) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 8 || shape.k % 8) return SLIM_ERR_SHAPE;
    if (!aligned16(W) || !aligned16(qvals) || !aligned16(meta) || !aligned16(scale)) return SLIM_ERR_ALIGN;
    return launch_pack<false>(W, shape, qvals, meta, scale, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

extern "C" int slim_pack_ex(const float *W, slim_shape shape, const float *saliency, const float *scale_in,
                            uint8_t *qvals, uint8_t *meta, float *scale, void *stream)
{
    if (!W || !qvals || !meta || !scale) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 8 || shape.k % 8) return SLIM_ERR_SHAPE;
    if (!aligned16(W) || !aligned16(qvals) || !aligned16(meta) || !aligned16(scale) || !aligned16(saliency) ||
        !aligned16(scale_in))
        return SLIM_ERR_ALIGN;
    return launch_pack<true>(W, shape, qvals, meta, scale, saliency, scale_in, static_cast<hipStream_t>(stream));
}

extern "C" int slim_unpack(const uint8_t *qvals, const uint8_t *meta, slim_shape shape, int8_t *codes,
                           uint8_t *mask, void *stream)
{
    if (!qvals || !meta || !codes || !mask) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 8 || shape.k % 8) return SLIM_ERR_SHAPE;
    if (!aligned16(qvals) || !aligned16(meta) || !aligned16(codes) || !aligned16(mask)) return SLIM_ERR_ALIGN;
    size_t groups = (size_t)shape.n * (shape.k / 4);
    hipLaunchKernelGGL(unpack_kernel, dim3(grid_for(groups, 256)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), qvals, meta, shape.n, shape.k, codes, mask);
    return hip_status(hipGetLastError());
}

extern "C" int slim_pack_adapters(const slim_half *L, const slim_half *R, slim_shape shape, slim_half *L_pad,
                                  slim_half *R_pad, void *stream)
{
    if (!L || !R || !L_pad || !R_pad) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 8 || shape.k % 8 || shape.rank < 1) return SLIM_ERR_SHAPE;
    if (!aligned16(L_pad) || !aligned16(R_pad)) return SLIM_ERR_ALIGN;
    int rp = slim_rank_pad(shape.rank);
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(tile_copy_kernel, dim3(grid_for(tl_bytes(shape.n, rp) / 16, 256)), dim3(256), 0, st, L, shape.n,
                       shape.rank, L_pad, tl_rows(shape.n), tl_cols(rp));
    hipLaunchKernelGGL(tile_copy_kernel, dim3(grid_for(tl_bytes(rp, shape.k) / 16, 256)), dim3(256), 0, st, R,
                       shape.rank, shape.k, R_pad, tl_rows(rp), tl_cols(shape.k));
    return hip_status(hipGetLastError());
}
