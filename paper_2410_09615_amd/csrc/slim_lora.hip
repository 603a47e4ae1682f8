// Low-rank adapter computation: Naive-LoRA and SLiM-LoRA (paper Sec. 3.2, Eq. 8-11, Alg. 2).
//
//   E = W - W^C,  x = x~ + min|x~|,  S = E diag(x)            ([n][k], input channels are columns)
//   S ~= L R~ with L [n][r] orthonormal columns spanning the r leading left singular vectors,
//   R~ = L^T S;   R = R~ diag(1 / x)                          (W ~= W^C + L R)
//
// The truncated SVD is reached by subspace iteration: Q <- orth(S orth(S^T Q)), started from a
// seeded random block of r columns.  The product Q Q^T S converges to the best rank-r
// approximation of S (Eckart-Young); how far it is from it after `iters` rounds shows in the
// captured energy ||Q^T S||_F^2 the call reports.  Everything is dense fp32 work on the matrix
// cores (V_MFMA_F32_32X32X2_F32): five GEMM shapes through one kernel, orthonormalisation as
// Cholesky QR (Gram matrix, Cholesky factor, inverse of the factor, one more GEMM).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "slim_internal.h"

namespace slim {

typedef float float16v_t __attribute__((ext_vector_type(16)));

// ---- C = A B or A^T B, fp32, row-major, optional split over K with atomic adds ----
struct SgemmArgs {
    const float *A, *B;
    float *C;
    int M, N, K;          // C is [M][N]; K is the summed dimension
    int lda, ldb, ldc;    // A is [M][K] (lda >= K), or [K][M] when transposed (lda >= M); B is [K][N]
    int kchunk;           // K values per grid.z slice (a multiple of 16); C is added to atomically when there are several
};

constexpr int kGM = 128, kGN = 128, kGK = 16, kGLd = kGK + 4;      // LDS rows of 16 k-values, padded to 20 floats

// Workgroup of 4 wavefronts, tile 128 x 128, each wavefront 64 x 64 = 2 x 2 matrix
// instruction blocks.  Both operand tiles sit in LDS as [row or column][k]: lane
// (r = lane % 32, h = lane / 32) of a block reads the four k-values 8 s + 4 h .. + 3 of
// its row with one 128-bit read and feeds them to four instructions; A and B use the
// same assignment of k-values to (lane half, instruction), so the sum is complete.
template <bool TA>
__global__ __launch_bounds__(256) void sgemm_kernel(SgemmArgs a)
{
    __shared__ __attribute__((aligned(16))) float As[kGM * kGLd];
    __shared__ __attribute__((aligned(16))) float Bs[kGN * kGLd];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = blockIdx.y * kGM, n0 = blockIdx.x * kGN;
    const int kb = blockIdx.z * a.kchunk, ke = min(a.K, kb + a.kchunk);
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;
    const int r = lane & 31, h = lane >> 5;

    float16v_t acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    float4_t ra[2], rb[2];
    // loads of the k-slab starting at k0 into registers (zeros outside the matrices)
    auto load_slab = [&](int k0) {
        if constexpr (!TA) {
            // A [M][K]: thread -> row tid / 4 (+ 64), k-values 4 (tid % 4) .. + 3
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int row = m0 + (tid >> 2) + 64 * i, kk = k0 + (tid & 3) * 4;
                ra[i] = (row < a.M && kk < ke) ? *reinterpret_cast<const float4_t *>(a.A + (size_t)row * a.lda + kk)
                                               : float4_t{0.f, 0.f, 0.f, 0.f};
            }
        } else {
            // A [K][M]: thread -> k-value tid / 32 (+ 8), rows 4 (tid % 32) .. + 3
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int kk = k0 + (tid >> 5) + 8 * i, row = m0 + (tid & 31) * 4;
                ra[i] = (kk < ke && row < a.M) ? *reinterpret_cast<const float4_t *>(a.A + (size_t)kk * a.lda + row)
                                               : float4_t{0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int kk = k0 + (tid >> 5) + 8 * i, col = n0 + (tid & 31) * 4;
            rb[i] = (kk < ke && col < a.N) ? *reinterpret_cast<const float4_t *>(a.B + (size_t)kk * a.ldb + col)
                                           : float4_t{0.f, 0.f, 0.f, 0.f};
        }
    };
    auto store_slab = [&]() {
        if constexpr (!TA) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                *reinterpret_cast<float4_t *>(As + ((tid >> 2) + 64 * i) * kGLd + (tid & 3) * 4) = ra[i];
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) As[((tid & 31) * 4 + e) * kGLd + (tid >> 5) + 8 * i] = ra[i][e];
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int e = 0; e < 4; ++e) Bs[((tid & 31) * 4 + e) * kGLd + (tid >> 5) + 8 * i] = rb[i][e];
    };

    // M and N are multiples of 4 wherever a 128-bit load straddles the edge (row counts
    // that are not appear only as K or as the row index of an untransposed A)
    load_slab(kb);
    for (int k0 = kb; k0 < ke; k0 += kGK) {
        __syncthreads();                      // the previous slab has been read
        store_slab();
        __syncthreads();
        if (k0 + kGK < ke) load_slab(k0 + kGK);
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            float4_t av[2], bv[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) av[i] = *reinterpret_cast<const float4_t *>(As + (wm + 32 * i + r) * kGLd + 8 * s + 4 * h);
#pragma unroll
            for (int j = 0; j < 2; ++j) bv[j] = *reinterpret_cast<const float4_t *>(Bs + (wn + 32 * j + r) * kGLd + 8 * s + 4 * h);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < 2; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i][e], bv[j][e], acc[i][j], 0, 0, 0);
        }
    }
    // register 4 b + e of a block: row 8 b + 4 h + e, column r
    const bool add = gridDim.z > 1;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn + 32 * j + r;
            if (col >= a.N) continue;
#pragma unroll
            for (int b = 0; b < 4; ++b)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int row = m0 + wm + 32 * i + 8 * b + 4 * h + e;
                    if (row >= a.M) continue;
                    float *c = a.C + (size_t)row * a.ldc + col;
                    if (add)
                        atomicAdd(c, acc[i][j][4 * b + e]);
                    else
                        *c = acc[i][j][4 * b + e];
                }
        }
}

__global__ void fill_kernel(float *p, size_t count, float v)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}

static int launch_fill(float *p, size_t count, float v, hipStream_t st)
{
    const unsigned grid = (unsigned)std::min<size_t>((count + 255) / 256, 2048);
    hipLaunchKernelGGL(fill_kernel, dim3(grid ? grid : 1), dim3(256), 0, st, p, count, v);
    return hip_status(hipGetLastError());
}

// C = op(A) B.  Few tiles and a long K: K is split over grid.z and C, zeroed first, is added to.
static int sgemm(bool ta, const float *A, int lda, const float *B, int ldb, float *C, int ldc, int M, int N, int K,
                 hipStream_t st)
{
    SgemmArgs a{A, B, C, M, N, K, lda, ldb, ldc, 0};
    const int tm = (M + kGM - 1) / kGM, tn = (N + kGN - 1) / kGN;
    int splits = 1;
    if (tm * tn < 512) splits = (512 + tm * tn - 1) / (tm * tn);
    const int kslabs = (K + kGK - 1) / kGK;
    if (splits > kslabs / 4) splits = kslabs / 4 > 0 ? kslabs / 4 : 1;      // at least 64 k-values per slice
    a.kchunk = (kslabs + splits - 1) / splits * kGK;
    splits = (K + a.kchunk - 1) / a.kchunk;
    if (splits > 1) {
        if (ldc == N) {
            const int rc = launch_fill(C, (size_t)M * N, 0.f, st);
            if (rc != SLIM_OK) return rc;
        } else {
            return SLIM_ERR_SHAPE;      // not used: every C here is contiguous
        }
    }
    const dim3 grid(tn, tm, splits);
    if (ta)
        hipLaunchKernelGGL(sgemm_kernel<true>, grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(sgemm_kernel<false>, grid, dim3(256), 0, st, a);
    return hip_status(hipGetLastError());
}

// ---- x = x~ + min|x~| (Alg. 2), or ones ----
__global__ __launch_bounds__(1024) void lora_shift_kernel(const float *xt, int k, float *x)
{
    __shared__ float red[16];
    float mn = INFINITY;
    if (xt)
        for (int i = threadIdx.x; i < k; i += blockDim.x) mn = fminf(mn, fabsf(xt[i]));
    mn = -wave_max(-mn);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mn;
    __syncthreads();
    mn = red[0];
    for (int w = 1; w < (int)blockDim.x / 64; ++w) mn = fminf(mn, red[w]);
    for (int i = threadIdx.x; i < k; i += blockDim.x) x[i] = xt ? xt[i] + mn : 1.0f;
}

// ---- S = (W - W^C) diag(x); the packed bytes are read in their tiled layout ----
// One thread per group of four inputs.  sq[0] += ||S||_F^2.
__global__ __launch_bounds__(256) void lora_error_kernel(const float *W, const uint8_t *qvals, const uint8_t *meta,
                                                         const float *scale, const float *x, int n, int k, float *S,
                                                         float *sq)
{
    const int groups = k / 4;
    const size_t total = (size_t)n * groups;
    const uint32_t kt = pk_ktiles(k);
    float part = 0.f;
    for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (size_t)gridDim.x * blockDim.x) {
        const uint32_t o = (uint32_t)(t / groups), g = (uint32_t)(t % groups);
        const uint32_t q = qvals[pk_qoff(o, g, kt)];
        const uint32_t mb = meta[pk_moff(o, g >> 1, kt)];
        const uint32_t m4 = (g & 1) ? (mb >> 4) : (mb & 15u);
        const float s = scale[o];
        float wc[4] = {0.f, 0.f, 0.f, 0.f};
        wc[m4 & 3u] = (float)nibble_to_int(q & 15u) * s;
        wc[(m4 >> 2) & 3u] = (float)nibble_to_int(q >> 4) * s;
        const float4_t w = *reinterpret_cast<const float4_t *>(W + (size_t)o * k + 4 * g);
        const float4_t xv = *reinterpret_cast<const float4_t *>(x + 4 * g);
        float4_t e;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            e[i] = (w[i] - wc[i]) * xv[i];
            part += e[i] * e[i];
        }
        *reinterpret_cast<float4_t *>(S + (size_t)o * k + 4 * g) = e;
    }
    part = wave_sum(part);
    if ((threadIdx.x & 63) == 0) atomicAdd(sq, part);
}

// ---- start block: uniform in (-1, 1) from a hash of (seed, element), columns >= r zero ----
__device__ __forceinline__ uint32_t mix32(uint32_t v)
{
    v ^= v >> 16;
    v *= 0x7feb352du;
    v ^= v >> 15;
    v *= 0x846ca68bu;
    v ^= v >> 16;
    return v;
}

__global__ void lora_init_kernel(float *Z, int rows, int l, int r, uint32_t seed)
{
    const size_t total = (size_t)rows * l;
    for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (size_t)gridDim.x * blockDim.x) {
        const int c = (int)(t % l);
        const uint32_t hsh = mix32(mix32((uint32_t)t ^ seed) + (uint32_t)(t >> 32) + 0x9e3779b9u * seed);
        Z[t] = c < r ? ((float)(hsh >> 8) + 0.5f) * (2.0f / 16777216.0f) - 1.0f : 0.f;
    }
}

// ---- Cholesky factor of the Gram matrix, in place (lower triangle), one workgroup ----
// A pivot below 1e-9 of the largest diagonal entry marks a column that lies in the span of
// the ones before it (or a padding column of zeros): it gets pivot 1 and a zero column, so
// the orthonormalised block carries a zero column there.
constexpr int kMaxBlock = 1024;          // columns of the iteration block (rank_pad)

__global__ __launch_bounds__(1024) void lora_chol_kernel(float *G, int l)
{
    __shared__ float col[kMaxBlock];
    __shared__ float red[16];
    __shared__ float piv;
    const int tid = threadIdx.x, T = blockDim.x;
    float mx = 0.f;
    for (int i = tid; i < l; i += T) mx = fmaxf(mx, G[(size_t)i * l + i]);
    mx = wave_max(mx);
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = red[0];
    for (int w = 1; w < T / 64; ++w) mx = fmaxf(mx, red[w]);
    const float floor_ = mx * 1e-9f;
    for (int j = 0; j < l; ++j) {
        if (tid == 0) {
            const float d = G[(size_t)j * l + j];
            piv = d > floor_ ? sqrtf(d) : 0.f;
        }
        __syncthreads();
        const float p = piv;
        const float inv = p > 0.f ? 1.0f / p : 0.f;
        for (int i = j + 1 + tid; i < l; i += T) {
            const float v = G[(size_t)i * l + j] * inv;
            G[(size_t)i * l + j] = v;
            col[i] = v;
        }
        if (tid == 0) G[(size_t)j * l + j] = p > 0.f ? p : 1.0f;
        __syncthreads();
        // trailing update of the lower triangle: G[i][c] -= col[i] col[c], j < c <= i
        const int cnt = l - j - 1;
        if (p > 0.f)
            for (int idx = tid; idx < cnt * cnt; idx += T) {
                const int i = j + 1 + idx / cnt, c = j + 1 + idx % cnt;
                if (c <= i) G[(size_t)i * l + c] -= col[i] * col[c];
            }
        __syncthreads();
    }
}

// ---- B = (inverse of the lower factor)^T: B[j][i] = X[i][j], X = Lc^-1; thread per column j of X ----
__global__ __launch_bounds__(64) void lora_trinv_kernel(const float *Lc, float *B, int l)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= l) return;
    float *row = B + (size_t)j * l;                 // column j of X, as a row of B
    for (int i = 0; i < j; ++i) row[i] = 0.f;
    row[j] = 1.0f / Lc[(size_t)j * l + j];
    for (int i = j + 1; i < l; ++i) {
        const float *li = Lc + (size_t)i * l;
        float s = 0.f;
        for (int p = j; p < i; ++p) s += li[p] * row[p];
        row[i] = -s / li[i];
    }
}

// ---- results: L fp16 [n][r] = Q[:, :r];  R fp16 [r][k] = R~[:r] / x;  sq[1] += ||R~[:r]||_F^2 ----
__global__ void lora_out_l_kernel(const float *Q, int n, int l, int r, half_t *L)
{
    const size_t total = (size_t)n * r;
    for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (size_t)gridDim.x * blockDim.x) {
        const size_t i = t / r, c = t % r;
        L[t] = (half_t)Q[i * l + c];
    }
}

__global__ __launch_bounds__(256) void lora_out_r_kernel(const float *Rt, const float *x, int k, int r, half_t *R, float *sq)
{
    const size_t total = (size_t)r * k;
    float part = 0.f;
    for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += (size_t)gridDim.x * blockDim.x) {
        const size_t j = t % k;
        const float v = Rt[t];
        part += v * v;
        R[t] = (half_t)(v / x[j]);
    }
    part = wave_sum(part);
    if ((threadIdx.x & 63) == 0) atomicAdd(sq + 1, part);
}

// sq[2] = max |G - I| over the leading r x r block (orthonormality of the final Q)
__global__ __launch_bounds__(256) void lora_ortho_kernel(const float *G, int l, int r, float *sq)
{
    float mx = 0.f;
    for (int t = blockIdx.x * blockDim.x + threadIdx.x; t < r * r; t += gridDim.x * blockDim.x) {
        const int i = t / r, c = t % r;
        mx = fmaxf(mx, fabsf(G[(size_t)i * l + c] - (i == c ? 1.0f : 0.f)));
    }
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) atomicMax(reinterpret_cast<unsigned *>(sq + 2), __float_as_uint(mx));   // non-negative floats order as integers
}

struct LoraPlan {
    int l;                      // columns of the iteration block: rank padded as the layer's adapters are
    size_t x, S, Q, Y, Z, G, B, Rt, sq, total;      // byte offsets
};

static size_t up256(size_t v) { return (v + 255) / 256 * 256; }

static LoraPlan plan_lora(int n, int k, int rank)
{
    LoraPlan p{};
    p.l = slim_rank_pad(rank);
    const size_t l = p.l, big = n > k ? n : k;
    size_t off = 0;
    auto take = [&](size_t floats) {
        const size_t at = off;
        off += up256(floats * sizeof(float));
        return at;
    };
    p.x = take(k);
    p.S = take((size_t)n * k);
    p.Q = take(big * l);
    p.Y = take(big * l);
    p.Z = take((size_t)k * l);
    p.G = take(l * l);
    p.B = take(l * l);
    p.Rt = take(l * k);
    p.sq = take(64);
    p.total = off;
    return p;
}

}  // namespace slim

using namespace slim;

extern "C" int slim_adapters_workspace_bytes(slim_shape shape, size_t *bytes)
{
    if (!bytes) return SLIM_ERR_NULL;
    if (shape.n < 1 || shape.k < 128 || shape.k % 128 || shape.rank < 1 || shape.rank > shape.n || shape.rank > shape.k ||
        slim_rank_pad(shape.rank) > kMaxBlock)
        return SLIM_ERR_SHAPE;
    *bytes = plan_lora(shape.n, shape.k, shape.rank).total;
    return SLIM_OK;
}

extern "C" int slim_compute_adapters(const float *W, const uint8_t *qvals, const uint8_t *meta, const float *scale,
                                     slim_shape shape, const float *x_tilde, int32_t iters, uint32_t seed, slim_half *L,
                                     slim_half *R, float *diag, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!W || !qvals || !meta || !scale || !L || !R) return SLIM_ERR_NULL;
    const int n = shape.n, k = shape.k, r = shape.rank;
    if (n < 1 || k < 128 || k % 128 || r < 1 || r > n || r > k || slim_rank_pad(r) > kMaxBlock || iters < 0 || iters > 1000)
        return SLIM_ERR_SHAPE;
    if (!aligned16(W) || !aligned16(qvals) || !aligned16(meta) || !aligned16(scale) || !aligned16(L) || !aligned16(R) ||
        (x_tilde && !aligned16(x_tilde)) || !aligned16(workspace))
        return SLIM_ERR_ALIGN;
    const LoraPlan p = plan_lora(n, k, r);
    if (!workspace || workspace_bytes < p.total) return SLIM_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    float *x = reinterpret_cast<float *>(ws + p.x), *S = reinterpret_cast<float *>(ws + p.S);
    float *Q = reinterpret_cast<float *>(ws + p.Q), *Y = reinterpret_cast<float *>(ws + p.Y);
    float *Z = reinterpret_cast<float *>(ws + p.Z), *G = reinterpret_cast<float *>(ws + p.G);
    float *B = reinterpret_cast<float *>(ws + p.B), *Rt = reinterpret_cast<float *>(ws + p.Rt);
    float *sq = reinterpret_cast<float *>(ws + p.sq);
    const int l = p.l;
    const int q = iters == 0 ? 16 : iters;
    int rc;
#define SLIM_TRY(call)            \
    do {                          \
        rc = (call);              \
        if (rc != SLIM_OK) return rc; \
    } while (0)
    auto launched = [&]() { return hip_status(hipGetLastError()); };
    auto grid_for = [](size_t count) { return dim3((unsigned)std::min<size_t>((count + 255) / 256, 4096)); };

    SLIM_TRY(launch_fill(sq, 64, 0.f, st));
    hipLaunchKernelGGL(lora_shift_kernel, dim3(1), dim3(1024), 0, st, x_tilde, k, x);
    SLIM_TRY(launched());
    hipLaunchKernelGGL(lora_error_kernel, grid_for((size_t)n * (k / 4)), dim3(256), 0, st, W, qvals, meta, scale,
                       (const float *)x, n, k, S, sq);
    SLIM_TRY(launched());
    hipLaunchKernelGGL(lora_init_kernel, grid_for((size_t)k * l), dim3(256), 0, st, Z, k, l, r, seed);
    SLIM_TRY(launched());

    // out = orth(in) for a block [rows][l]: G = in^T in = Lc Lc^T, out = in Lc^-T
    auto orth = [&](const float *in, float *out, int rows) -> int {
        int e = sgemm(true, in, l, in, l, G, l, l, l, rows, st);
        if (e != SLIM_OK) return e;
        hipLaunchKernelGGL(lora_chol_kernel, dim3(1), dim3(1024), 0, st, G, l);
        if ((e = launched()) != SLIM_OK) return e;
        hipLaunchKernelGGL(lora_trinv_kernel, dim3((l + 63) / 64), dim3(64), 0, st, (const float *)G, B, l);
        if ((e = launched()) != SLIM_OK) return e;
        return sgemm(false, in, l, B, l, out, l, rows, l, l, st);
    };

    SLIM_TRY(sgemm(false, S, k, Z, l, Y, l, n, l, k, st));          // Y = S Z           [n][l]
    SLIM_TRY(orth(Y, Q, n));
    for (int it = 0; it < q; ++it) {
        SLIM_TRY(sgemm(true, S, k, Q, l, Y, l, k, l, n, st));       // Y = S^T Q         [k][l]
        SLIM_TRY(orth(Y, Z, k));
        SLIM_TRY(sgemm(false, S, k, Z, l, Y, l, n, l, k, st));      // Y = S Z           [n][l]
        SLIM_TRY(orth(Y, Q, n));
    }
    SLIM_TRY(orth(Q, Y, n));                                        // second pass: orthonormal to rounding
    SLIM_TRY(sgemm(true, Y, l, S, k, Rt, k, l, k, n, st));          // R~ = Q^T S        [l][k]
    SLIM_TRY(sgemm(true, Y, l, Y, l, G, l, l, l, n, st));           // Gram of the final block, for the report
    hipLaunchKernelGGL(lora_ortho_kernel, grid_for((size_t)r * r), dim3(256), 0, st, (const float *)G, l, r, sq);
    SLIM_TRY(launched());
    hipLaunchKernelGGL(lora_out_l_kernel, grid_for((size_t)n * r), dim3(256), 0, st, (const float *)Y, n, l, r,
                       reinterpret_cast<half_t *>(L));
    SLIM_TRY(launched());
    hipLaunchKernelGGL(lora_out_r_kernel, grid_for((size_t)r * k), dim3(256), 0, st, (const float *)Rt, (const float *)x, k,
                       r, reinterpret_cast<half_t *>(R), sq);
    SLIM_TRY(launched());
    if (diag) {
        const hipError_t e = hipMemcpyAsync(diag, sq, 4 * sizeof(float), hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return SLIM_ERR_HIP;
    }
#undef SLIM_TRY
    return SLIM_OK;
}
