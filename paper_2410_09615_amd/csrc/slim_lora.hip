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
// cores (V_MFMA_F32_32X32X2_F32), all GEMM shapes through one kernel; orthonormalisation is
// Cholesky QR in blocks of 64 columns (Gram matrix, then per block a small factor-and-invert
// kernel and GEMMs for the panel, the trailing update and the application to the block).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "slim_internal.h"

namespace slim {

typedef float float16v_t __attribute__((ext_vector_type(16)));

// ---- C = alpha op(A) op(B) + beta C, fp32, row-major, optional split over K with atomic adds ----
struct SgemmArgs {
    const float *A, *B;
    float *C;
    int M, N, K;          // C is [M][N]; K is the summed dimension
    int lda, ldb, ldc;    // A is [M][K], or [K][M] when TA; B is [K][N], or [N][K] when TB
    int kchunk;           // K values per grid.z slice (a multiple of 16); C is added to atomically when there are several
    float alpha;
    int beta;             // 0: C is overwritten (zeroed first when K is split), 1: added to
};

constexpr int kGM = 128, kGN = 128, kGK = 16, kGLd = kGK + 4;      // LDS rows of 16 k-values, padded to 20 floats

// Workgroup of 4 wavefronts, tile 128 x 128, each wavefront 64 x 64 = 2 x 2 matrix
// instruction blocks.  Both operand tiles sit in LDS as [row or column][k]: lane
// (r = lane % 32, h = lane / 32) of a block reads the four k-values 8 s + 4 h .. + 3 of
// its row with one 128-bit read and feeds them to four instructions; A and B use the
// same assignment of k-values to (lane half, instruction), so the sum is complete.
template <bool TA, bool TB>
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
        if constexpr (TB) {
            // B [N][K]: as the untransposed A
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int col = n0 + (tid >> 2) + 64 * i, kk = k0 + (tid & 3) * 4;
                rb[i] = (col < a.N && kk < ke) ? *reinterpret_cast<const float4_t *>(a.B + (size_t)col * a.ldb + kk)
                                               : float4_t{0.f, 0.f, 0.f, 0.f};
            }
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int kk = k0 + (tid >> 5) + 8 * i, col = n0 + (tid & 31) * 4;
                rb[i] = (kk < ke && col < a.N) ? *reinterpret_cast<const float4_t *>(a.B + (size_t)kk * a.ldb + col)
                                               : float4_t{0.f, 0.f, 0.f, 0.f};
            }
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
        if constexpr (TB) {
#pragma unroll
            for (int i = 0; i < 2; ++i)
                *reinterpret_cast<float4_t *>(Bs + ((tid >> 2) + 64 * i) * kGLd + (tid & 3) * 4) = rb[i];
        } else {
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int e = 0; e < 4; ++e) Bs[((tid & 31) * 4 + e) * kGLd + (tid >> 5) + 8 * i] = rb[i][e];
        }
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
                    const float v = a.alpha * acc[i][j][4 * b + e];
                    if (add)
                        atomicAdd(c, v);
                    else
                        *c = a.beta ? *c + v : v;
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

// C = alpha op(A) op(B) + beta C.  Few tiles and a long K: K is split over grid.z and C
// (zeroed first when beta = 0) is added to.
static int sgemm(bool ta, bool tb, const float *A, int lda, const float *B, int ldb, float *C, int ldc, int M, int N, int K,
                 hipStream_t st, float alpha = 1.0f, int beta = 0)
{
    if (M <= 0 || N <= 0 || K <= 0) return SLIM_OK;
    SgemmArgs a{A, B, C, M, N, K, lda, ldb, ldc, 0, alpha, beta};
    const int tm = (M + kGM - 1) / kGM, tn = (N + kGN - 1) / kGN;
    int splits = 1;
    if (tm * tn < 512) splits = (512 + tm * tn - 1) / (tm * tn);
    const int kslabs = (K + kGK - 1) / kGK;
    if (splits > kslabs / 4) splits = kslabs / 4 > 0 ? kslabs / 4 : 1;      // at least 64 k-values per slice
    a.kchunk = (kslabs + splits - 1) / splits * kGK;
    splits = (K + a.kchunk - 1) / a.kchunk;
    if (splits > 1 && !beta) {
        if (ldc == N) {
            const int rc = launch_fill(C, (size_t)M * N, 0.f, st);
            if (rc != SLIM_OK) return rc;
        } else {
            return SLIM_ERR_SHAPE;      // not used: a C that is overwritten with K split is contiguous here
        }
    }
    const dim3 grid(tn, tm, splits);
    if (ta && !tb)
        hipLaunchKernelGGL((sgemm_kernel<true, false>), grid, dim3(256), 0, st, a);
    else if (!ta && tb)
        hipLaunchKernelGGL((sgemm_kernel<false, true>), grid, dim3(256), 0, st, a);
    else if (!ta && !tb)
        hipLaunchKernelGGL((sgemm_kernel<false, false>), grid, dim3(256), 0, st, a);
    else
        return SLIM_ERR_SHAPE;          // A^T B^T is not needed here
    return hip_status(hipGetLastError());
}

// One atomic add per workgroup of 256 threads (adds to one address serialise).
__device__ __forceinline__ void block_add(float part, float *dst)
{
    __shared__ float red4[4];
    part = wave_sum(part);
    if ((threadIdx.x & 63) == 0) red4[threadIdx.x >> 6] = part;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(dst, red4[0] + red4[1] + red4[2] + red4[3]);
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
    block_add(part, sq);
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

// ---- Cholesky QR in blocks of 64 columns ----
// G = Lc Lc^T is factored block column by block column: the 64 x 64 diagonal block and its
// inverse in one small workgroup (below), the panel under it and the trailing update as
// GEMMs.  A pivot below 1e-9 of the largest diagonal entry of G marks a column that lies in
// the span of the ones before it (or a padding column of zeros): it gets pivot 1 and a zero
// column, so the orthonormalised block carries a (numerically) zero column there.
constexpr int kMaxBlock = 1024;          // columns of the iteration block (rank_pad)
constexpr int kCb = 64;                  // block width of the factorisation

__global__ __launch_bounds__(1024) void lora_diagmax_kernel(const float *G, int l, float *out)
{
    __shared__ float red[16];
    float mx = 0.f;
    for (int i = threadIdx.x; i < l; i += blockDim.x) mx = fmaxf(mx, G[(size_t)i * l + i]);
    mx = wave_max(mx);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < (int)blockDim.x / 64; ++w) mx = fmaxf(mx, red[w]);
        *out = mx;
    }
}

// Diagonal block at (j0, j0), width w <= 64: L11 replaces its lower triangle in G, and
// X11 = L11^-1 (lower triangular, zeros above) goes to D[j0 .. j0 + w)[0 .. 64).
// Column c of the factor and row c of the inverse are final after step c: the forward
// substitution L X = I runs along with the factorisation (x starts as the identity).
// The block lives in registers: 256 threads as a 16 x 16 grid, thread (ty, tx) owns the
// elements (ty + 16 p, tx + 16 q) of a and of x.  A step needs column c of a and row c of x:
// their owners publish them in LDS (two buffers in turn, one barrier per step), everybody
// reads the four values of its rows and of its columns, and the update is 32 predicated
// multiply-adds on registers.  Scaled column c and row c are final then and go to LDS
// for the write-out at the end.
__global__ __launch_bounds__(256) void lora_chol_diag_kernel(float *G, int l, int j0, int w, const float *gmax, float *D)
{
    __shared__ float col[2][kCb];        // column c of a, as it stands at step c (unscaled)
    __shared__ float xrow[2][kCb];       // row c of x (unscaled)
    __shared__ float lout[kCb][kCb + 1];
    __shared__ float xout[kCb][kCb + 1];
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    float av[4][4], xv[4][4];
#pragma unroll
    for (int p = 0; p < 4; ++p)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int i = ty + 16 * p, cc = tx + 16 * q;
            av[p][q] = (i < w && cc < w) ? G[(size_t)(j0 + i) * l + j0 + cc] : 0.f;
            xv[p][q] = i == cc ? 1.0f : 0.f;
        }
    for (int idx = tid; idx < kCb * kCb; idx += 256) {
        lout[idx / kCb][idx % kCb] = 0.f;
        xout[idx / kCb][idx % kCb] = 0.f;
    }
    const float floor_ = *gmax * 1e-9f;
    for (int c = 0; c < w; ++c) {
        const int b = c & 1, cq = c >> 4, cr = c & 15;
        // publish: column c of a from the threads with tx == c mod 16, row c of x from those with ty == c mod 16
        if (tx == cr) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (q == cq) {
#pragma unroll
                    for (int p = 0; p < 4; ++p) col[b][ty + 16 * p] = av[p][q];
                }
        }
        if (ty == cr) {
#pragma unroll
            for (int p = 0; p < 4; ++p)
                if (p == cq) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) xrow[b][tx + 16 * q] = xv[p][q];
                }
        }
        __syncthreads();
        const float d = col[b][c];
        const float pv = d > floor_ ? sqrtf(d) : 0.f;        // 0: a column in the span of the ones before it
        const float inv = pv > 0.f ? 1.0f / pv : 0.f;
        const float dinv = pv > 0.f ? 1.0f / pv : 1.0f;
        float li[4], lc[4], xr[4];
#pragma unroll
        for (int p = 0; p < 4; ++p) li[p] = col[b][ty + 16 * p] * inv;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            lc[q] = col[b][tx + 16 * q] * inv;
            xr[q] = xrow[b][tx + 16 * q] * dinv;
        }
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int i = ty + 16 * p, cc = tx + 16 * q;
                if (i > c && cc > c && cc <= i) av[p][q] -= li[p] * lc[q];
                if (i > c && cc <= c) xv[p][q] -= li[p] * xr[q];
            }
        // what is final now: column c of the factor (threads 0..63), row c of the inverse (64..127)
        if (tid < kCb) {
            if (tid > c)
                lout[tid][c] = col[b][tid] * inv;
            else if (tid == c)
                lout[tid][c] = pv > 0.f ? pv : 1.0f;
        } else if (tid < 2 * kCb) {
            const int cc = tid - kCb;
            if (cc <= c) xout[c][cc] = xrow[b][cc] * dinv;
        }
    }
    __syncthreads();
    for (int idx = tid; idx < w * w; idx += 256) {
        const int i = idx / w, c = idx % w;
        if (c <= i) G[(size_t)(j0 + i) * l + j0 + c] = lout[i][c];
    }
    for (int idx = tid; idx < w * kCb; idx += 256) {
        const int i = idx / kCb, c = idx % kCb;
        D[(size_t)(j0 + i) * kCb + c] = c < w ? xout[i][c] : 0.f;
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
    block_add(part, sq + 1);
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

// the four numbers of the report, out of the workspace (a kernel, so that the call is kernels only)
__global__ void lora_report_kernel(const float *sq, float *diag)
{
    if (threadIdx.x < 4) diag[threadIdx.x] = threadIdx.x < 3 ? sq[threadIdx.x] : 0.f;
}

struct LoraPlan {
    int l;                      // columns of the iteration block: rank padded as the layer's adapters are
    size_t x, S, Q, Y, Z, G, B, Rt, sq, total;      // byte offsets (B: the inverses of the diagonal blocks, [l][64])
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
    p.B = take(l * kCb);
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
    hipLaunchKernelGGL(lora_error_kernel, dim3(std::min(grid_for((size_t)n * (k / 4)).x, 1024u)), dim3(256), 0, st, W, qvals, meta, scale,
                       (const float *)x, n, k, S, sq);
    SLIM_TRY(launched());
    hipLaunchKernelGGL(lora_init_kernel, grid_for((size_t)k * l), dim3(256), 0, st, Z, k, l, r, seed);
    SLIM_TRY(launched());

    // out = orth(in) for a block [rows][l] (in is overwritten): G = in^T in = Lc Lc^T, out = in Lc^-T
    auto orth = [&](float *in, float *out, int rows) -> int {
        int e = sgemm(true, false, in, l, in, l, G, l, l, l, rows, st);
        if (e != SLIM_OK) return e;
        hipLaunchKernelGGL(lora_diagmax_kernel, dim3(1), dim3(1024), 0, st, (const float *)G, l, sq + 4);
        if ((e = launched()) != SLIM_OK) return e;
        for (int j0 = 0; j0 < l; j0 += kCb) {
            const int w = std::min(kCb, l - j0), below = l - j0 - w;
            hipLaunchKernelGGL(lora_chol_diag_kernel, dim3(1), dim3(256), 0, st, G, l, j0, w, (const float *)(sq + 4), B);
            if ((e = launched()) != SLIM_OK) return e;
            float *panel = G + (size_t)(j0 + w) * l + j0;
            // panel under the block: L21 = A21 L11^-T (in place: a workgroup has read its rows before it writes them)
            if ((e = sgemm(false, true, panel, l, B + (size_t)j0 * kCb, kCb, panel, l, below, w, w, st)) != SLIM_OK) return e;
            // what is left: A22 -= L21 L21^T
            if ((e = sgemm(false, true, panel, l, panel, l, G + (size_t)(j0 + w) * l + j0 + w, l, below, below, w, st, -1.0f, 1)) != SLIM_OK)
                return e;
        }
        // out = in Lc^-T by block columns: out_j = (in_j - out_{<j} Lc[j, <j]^T) X_jj^T
        for (int j0 = 0; j0 < l; j0 += kCb) {
            const int w = std::min(kCb, l - j0);
            if ((e = sgemm(false, true, out, l, G + (size_t)j0 * l, l, in + j0, l, rows, w, j0, st, -1.0f, 1)) != SLIM_OK) return e;
            if ((e = sgemm(false, true, in + j0, l, B + (size_t)j0 * kCb, kCb, out + j0, l, rows, w, w, st)) != SLIM_OK) return e;
        }
        return SLIM_OK;
    };

    SLIM_TRY(sgemm(false, false, S, k, Z, l, Y, l, n, l, k, st));          // Y = S Z           [n][l]
    SLIM_TRY(orth(Y, Q, n));
    for (int it = 0; it < q; ++it) {
        SLIM_TRY(sgemm(true, false, S, k, Q, l, Y, l, k, l, n, st));       // Y = S^T Q         [k][l]
        SLIM_TRY(orth(Y, Z, k));
        SLIM_TRY(sgemm(false, false, S, k, Z, l, Y, l, n, l, k, st));      // Y = S Z           [n][l]
        SLIM_TRY(orth(Y, Q, n));
    }
    SLIM_TRY(orth(Q, Y, n));                                        // second pass: orthonormal to rounding
    SLIM_TRY(sgemm(true, false, Y, l, S, k, Rt, k, l, k, n, st));          // R~ = Q^T S        [l][k]
    SLIM_TRY(sgemm(true, false, Y, l, Y, l, G, l, l, l, n, st));           // Gram of the final block, for the report
    hipLaunchKernelGGL(lora_ortho_kernel, grid_for((size_t)r * r), dim3(256), 0, st, (const float *)G, l, r, sq);
    SLIM_TRY(launched());
    hipLaunchKernelGGL(lora_out_l_kernel, grid_for((size_t)n * r), dim3(256), 0, st, (const float *)Y, n, l, r,
                       reinterpret_cast<half_t *>(L));
    SLIM_TRY(launched());
    hipLaunchKernelGGL(lora_out_r_kernel, dim3(std::min(grid_for((size_t)r * k).x, 1024u)), dim3(256), 0, st, (const float *)Rt, (const float *)x, k,
                       r, reinterpret_cast<half_t *>(R), sq);
    SLIM_TRY(launched());
    if (diag) {
        hipLaunchKernelGGL(lora_report_kernel, dim3(1), dim3(64), 0, st, (const float *)sq, diag);
        SLIM_TRY(launched());
    }
#undef SLIM_TRY
    return SLIM_OK;
}
