/*
 * libslim -- forward pass of one SLiM-compressed linear layer on MI355X (gfx950).
 *
 *     Y = X . dequant(Wq (.) M_2:4)^T + (X . R^T) . L^T
 *
 * Wq: symmetric 4-bit codes under a 2:4 semi-structured mask, one fp32 scale
 * per output row; L, R: fp16 low-rank adapters.  This is the inference form
 * of the paper's decomposition W ~= W^C + L R (arXiv 2410.09615, Sec. 3.2),
 * written in nn.Linear orientation: W is [n][k] = d_out x d_in, L is [n][rank],
 * R is [rank][k], X is [m][k], Y is [m][n].  (The paper stores W as
 * d_in x d_out and names the d_in-side factor L: its L is R^T here and its R
 * is L^T here.)
 *
 * Conventions for every entry point
 *   - returns 0 (SLIM_OK) or a negative slim_status; never throws, never exits;
 *   - every pointer is a DEVICE pointer owned by the caller (except the
 *     out-parameters of the size queries, which are host pointers);
 *   - matrices are row-major, contiguous, 16-byte aligned;
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream);
 *     all work is enqueued on it and the call returns without synchronizing;
 *   - the library allocates nothing; the forward entry points enqueue kernels only
 *     (no memset, copy or synchronization) and may be captured into a HIP graph;
 *   - what the library keeps between calls is: a process-wide call counter (the
 *     number that tags a decode call's intermediate result), what it has read of
 *     each device's properties (compute units, LDS), per thread the last decode
 *     launch plans it computed, the device address of its own scratch array
 *     (slim_linear_gemv_static) and the setting of slim_decode_override.  No result
 *     depends on an earlier call;
 *   - arguments are validated on the host before anything is launched; on an
 *     error nothing has been enqueued.
 * fp16 values are IEEE binary16 bit patterns (`slim_half`).
 *
 * Canonical packed bytes:
 *   group g of row o = inputs 4g .. 4g+3; i0 < i1 are its two kept positions
 *   qvals[o][g]  = (code(i0) & 15) | ((code(i1) & 15) << 4)   two's-complement nibbles
 *   meta[o][g/2] = m4(2*(g/2)) | (m4(2*(g/2)+1) << 4),  m4(g) = i0 | (i1 << 2)
 *   scale[o]     = fp32
 * 3 bits per original weight.
 *
 * Packed layout (written by slim_pack, read by every kernel, inverted by
 * slim_unpack): a byte permutation of the canonical arrays.  They are cut into
 * tiles of 32 rows x 128 inputs (32 bytes of qvals, 16 of meta per row), stored
 * row tile major, KT = ceil(k / 128) tiles per row tile, 1024 bytes of qvals and
 * 512 of meta each; inside a tile the pieces of 64 inputs (16 / 8 bytes) are
 * ordered (input half, row):
 *   qvals[o][g] at ((o/32) * KT + g/32) * 1024 + (((g%32)/16) * 32 + o%32) * 16 + g%16
 *   meta[o][b]  at ((o/32) * KT + b/16) *  512 + (((b%16)/8)  * 32 + o%32) *  8 + b%8
 * Rows are padded to a multiple of 32 and inputs to a multiple of 128 with zero
 * bytes.  This is the lane order of the sparse matrix instructions' A operand, so
 * a wavefront's load of a tile is contiguous.  scale stays [n].
 *
 * Adapter layout (written by slim_pack_adapters, read by every kernel): an fp16
 * matrix [rows][cols] (L: [n][rank_pad], R: [rank_pad][k]) is stored as tiles of
 * 32 rows x 16 columns (1 KiB), row tile major, rows padded to 32 and columns to
 * 16 with zeros; inside a tile the 64 pieces of 8 columns (16 bytes) are ordered
 * (column half, row).  The piece with columns 8 c .. 8 c + 7 of row r starts at byte
 *   ((r / 32) * (cols16 / 16) + c / 2) * 1024 + ((c % 2) * 32 + r % 32) * 16,
 * cols16 = cols rounded up to 16.  This is the order in which a wavefront holds
 * the A operand of the matrix instructions, so its loads are contiguous.
 */
#ifndef SLIM_H
#define SLIM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef uint16_t slim_half;

typedef enum {
    SLIM_OK = 0,
    SLIM_ERR_NULL = -1,       /* a required pointer is NULL                          */
    SLIM_ERR_SHAPE = -2,      /* a dimension is out of the documented range           */
    SLIM_ERR_ALIGN = -3,      /* a pointer is not 16-byte aligned                     */
    SLIM_ERR_WORKSPACE = -4,  /* workspace missing or smaller than slim_workspace_bytes */
    SLIM_ERR_HIP = -5,        /* a HIP runtime call failed (launch error)             */
    SLIM_ERR_WAIT = -6        /* slim_workspace_check: a decode call gave up waiting  */
} slim_status;

/* d_out, d_in and the true adapter rank (0 = layer without adapters). */
typedef struct {
    int32_t n, k, rank;
} slim_shape;

/* One compressed layer: device pointers to caller-owned buffers. */
typedef struct {
    slim_shape shape;
    const uint8_t *qvals;   /* canonical [n][k/4] in the packed layout               */
    const uint8_t *meta;    /* canonical [n][k/8] in the packed layout               */
    const float *scale;     /* [n]                                                   */
    const slim_half *L;     /* [n][rank_pad] in the adapter layout, columns >= rank zero (NULL if rank == 0) */
    const slim_half *R;     /* [rank_pad][k] in the adapter layout, rows >= rank zero    (NULL if rank == 0) */
    int32_t rank_pad;       /* slim_rank_pad(rank)                                   */
    /* 4-bit adapters (Sec. 3.3): with adapter_bits == 4 the kernels read Lq, Ls, Rq, Rs
     * (from slim_pack_adapters_q4) and ignore L and R; 0 or 16: fp16 adapters in L, R. */
    int32_t adapter_bits;
    const uint8_t *Lq;      /* codes of L [n][rank] in the 4-bit adapter layout      */
    const slim_half *Ls;    /* its group scales                                      */
    const uint8_t *Rq;      /* codes of R [rank][k]                                  */
    const slim_half *Rs;    /* its group scales                                      */
} slim_layer;

/* Text for a status code; a static string, never NULL. */
const char *slim_status_string(int status);

/* Padded rank the kernels work with: rank rounded up to a multiple of 32
 * (the k-extent of one matrix-core instruction); 0 stays 0. */
int32_t slim_rank_pad(int32_t rank);

/*
 * Buffer sizes, in bytes, of the packed layer for a given shape.  All
 * out-pointers are HOST pointers and may be NULL individually.
 * Errors: SLIM_ERR_SHAPE unless n >= 1, k >= 8, k % 8 == 0, rank >= 0.
 */
int slim_packed_sizes(slim_shape shape, size_t *qvals_bytes, size_t *meta_bytes,
                      size_t *scale_bytes, int32_t *rank_pad, size_t *L_bytes, size_t *R_bytes);

/*
 * slim_pack -- dense weights in, compressed layer out.
 *   mask   2:4 magnitude pruning: of every 4 consecutive inputs keep the two of
 *          largest |w| (ties: lower position first);
 *   scale  AbsMax per output row (Sec. 2): scale[o] = max_k |W[o][k]| / 7 as one
 *          binary32 division (1.0 for an all-zero row);
 *   codes  symmetric uniform 4-bit quantization (Sec. 2; Sec. 3.1 Eq. 2):
 *          round-half-even(W / scale) in binary32, clamped to [-8, 7];
 *   bytes  the canonical bytes above, written in the packed layout.
 * W [n][k] fp32 in; qvals, meta (sizes from slim_packed_sizes), scale [n] out.
 * W must be finite.  Errors: NULL, SHAPE (k % 8 != 0, n < 1), ALIGN, HIP.
 */
int slim_pack(const float *W, slim_shape shape, uint8_t *qvals, uint8_t *meta, float *scale,
              void *stream);

/*
 * slim_pack_ex -- slim_pack with the two choices the paper's own pipeline makes
 * differently (either pointer may be NULL, which gives slim_pack's behaviour):
 *   saliency [k]  non-negative, one per input: the 2:4 mask keeps the two largest
 *                 |w| * saliency[input] of a group (one binary32 product each;
 *                 ties: lower position first).  With the activation norms of the
 *                 inputs this is Wanda's metric, the pruning the paper applies
 *                 (Sec. 3, Sec. 4); the vector is the caller's.
 *   scale_in [n]  the scales to quantize with (copied to scale), e.g. the
 *                 per-tensor alpha / 7 of slim_quant_search; values beyond the
 *                 grid saturate at the codes -8 and 7.
 */
int slim_pack_ex(const float *W, slim_shape shape, const float *saliency, const float *scale_in,
                 uint8_t *qvals, uint8_t *meta, float *scale, void *stream);

/*
 * slim_quant_search -- the per-tensor scale of SLiM-Quant (Sec. 3.1, Eq. 4-7,
 * Alg. 1): alpha* minimises E_quant(alpha) + E_clip(alpha) of the symmetric
 * 4-bit quantizer, integrated numerically over the histogram of |W|:
 *   histogram  B = max(512, min(n k / 1000, 20000)) uniform bins over
 *              [0, M], M = max|W| (App. "Implementation Details"); an element
 *              counts at the centre of its bin; bin = min(B - 1, floor(|w| * (B / M)))
 *              in binary32;
 *   coarse     alpha = M i / 10, i = 1..10 (i = 10 is AbsMax);
 *   fine       21 samples of a tenth of that spacing around the best coarse one,
 *              those inside (0, M];
 *   alpha*     the first minimum over all of them (fp64 error sums).  The errors are,
 *              up to the factor M^2, rationals with a small denominator, so two
 *              candidates can have exactly equal errors; which of two candidates
 *              whose errors agree to the rounding error of the sum is returned is
 *              then decided by the order of the additions in the kernel.
 * W [n][k] fp32 in; scale_out [n] = alpha* / 7 in every row (1 for a zero
 * tensor), ready for slim_pack_ex; alpha_out (one float, may be NULL) = alpha*.
 * workspace: slim_quant_workspace_bytes (HOST out-pointer), need not be zeroed.
 */
int slim_quant_workspace_bytes(slim_shape shape, size_t *bytes);
int slim_quant_search(const float *W, slim_shape shape, float *scale_out, float *alpha_out,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * slim_quant_search_rows -- the same search (Sec. 3.1, Alg. 1) with one scale per
 * output row, the granularity of this format: row o is its own tensor of k
 * weights (histogram of max(512, min(k / 1000, 20000)) bins over [0, max|W[o]|]).
 * scale_out [n] = alpha*(o) / 7 (1 for a zero row), alpha_out [n] (may be NULL).
 * No workspace.  Errors: NULL, SHAPE (k % 8 != 0), ALIGN, HIP.
 */
int slim_quant_search_rows(const float *W, slim_shape shape, float *scale_out, float *alpha_out,
                           void *stream);

/*
 * slim_compute_adapters -- the low-rank adapters of a compressed layer: Naive-LoRA
 * and SLiM-LoRA (Sec. 3.2, Eq. 8-11, Alg. 2).  With E = W - W^C (so that
 * W ~= W^C + L R), x = x_tilde + min|x_tilde| and the error saliency
 * S = E diag(x) (input channels are the columns of W here), the adapters are the
 * rank-r truncation of S with the saliency taken out again:
 *   L [n][rank]  orthonormal columns spanning the leading left singular vectors of S,
 *   R [rank][k]  (L^T S) diag(1 / x),
 * both fp16, row-major (what slim_pack_adapters takes); L R minimises
 * ||(W - W^C - L R) diag(x)||_F over rank-r products.
 *   W [n][k] fp32, the dense weights; qvals, meta, scale: the layer slim_pack made of them;
 *   x_tilde [k]  fp32, the mean magnitude of the calibration inputs per input channel,
 *                positive and finite (the caller's; not checked); NULL: x = 1, Naive-LoRA;
 *   shape.rank   1 <= rank <= min(n, k), slim_rank_pad(rank) <= 1024;
 *   iters        rounds of the subspace iteration Q <- orth(S orth(S^T Q)) that stands in
 *                for the SVD (0: 16).  It starts from a block of `rank` columns drawn
 *                from `seed`; its distance from the exact truncation shows in diag
 *                (16 rounds: weighted residual within 0.3 % of the optimum for rank <=
 *                min(n, k) / 4 on compression errors; a rank close to min(n, k) leaves a few
 *                nearly equal singular values to separate and wants more rounds);
 *                sums use atomic adds, so results differ in the last bits from call to call;
 *   diag         (may be NULL) four floats out: ||S||_F^2, the captured part
 *                ||L^T S||_F^2 (the exact truncation captures the sum of the rank
 *                largest squared singular values), max |L^T L - I|, 0.
 * All dense work is fp32 on the matrix cores.  workspace:
 * slim_adapters_workspace_bytes (HOST out-pointer; about 4 n k bytes plus the
 * blocks), need not be zeroed.  Errors: NULL, SHAPE, ALIGN, WORKSPACE, HIP.
 */
int slim_adapters_workspace_bytes(slim_shape shape, size_t *bytes);
int slim_compute_adapters(const float *W, const uint8_t *qvals, const uint8_t *meta, const float *scale,
                          slim_shape shape, const float *x_tilde, int32_t iters, uint32_t seed,
                          slim_half *L, slim_half *R, float *diag, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * slim_pack_adapters -- lay the fp16 adapters out for the kernels: L [n][rank]
 * and R [rank][k], row-major, go into L_pad = [n][rank_pad] and R_pad =
 * [rank_pad][k] in the adapter layout above (sizes from slim_packed_sizes),
 * zero-filling the padding.  No arithmetic.  rank must be >= 1.
 */
int slim_pack_adapters(const slim_half *L, const slim_half *R, slim_shape shape,
                       slim_half *L_pad, slim_half *R_pad, void *stream);

/*
 * 4-bit adapters (Sec. 3.3, "Low-rank Adapter Quantization"): AbsMax group
 * quantization, groups of 128 consecutive elements of a row of L [n][rank] or
 * R [rank][k] (the last group of a row may be shorter):
 *   scale = max|a| / 7 as one binary32 division, rounded to binary16 (1 for a
 *           group of zeros; the smallest positive binary16 if that rounds to 0);
 *   code  = round-half-even(a / scale) in binary32, clamped to [-8, 7].
 * 4-bit adapter layout: codes as two's-complement nibbles (even column in the
 * low nibble) in tiles of 16 rows x 256 columns (2 KiB), row tile major; inside
 * a tile the 32 bytes of row r, columns 64 q .. 64 q + 63 start at (4 r + q) * 32;
 * rows padded to 16, columns to 256 with zero codes.  Scales: fp16
 * [rows16][2 * ceil(cols / 256)], row-major, entry g = group g of the row.
 * Sizes from slim_adapter_q4_sizes (HOST out-pointers).  A value is used as
 * fp16(code * scale).  The forward calls read the codes directly (a quarter of
 * the adapter bytes) and turn them into fp16 in registers; only the two-launch
 * decode kernels (layers whose one-launch geometry does not fit) expand them to
 * fp16 in the workspace first.  slim_unpack_adapters_q4 returns codes int8 [rows][cols] and scales
 * fp16 [rows][ceil(cols / 128)], row-major (tests, inspection).
 * slim_pack_adapters_q4 requires k % 128 == 0, as the forward calls do (SHAPE
 * otherwise); n and rank are free.
 */
int slim_adapter_q4_sizes(int32_t rows, int32_t cols, size_t *codes_bytes, size_t *scales_bytes);
int slim_pack_adapters_q4(const slim_half *L, const slim_half *R, slim_shape shape, uint8_t *Lq,
                          slim_half *Ls, uint8_t *Rq, slim_half *Rs, void *stream);
int slim_unpack_adapters_q4(const uint8_t *codes, const slim_half *scales, int32_t rows, int32_t cols,
                            int8_t *out_codes, slim_half *out_scales, void *stream);

/*
 * slim_unpack -- inverse of slim_pack's bytes (packed layout and canonical
 * format), for tests and inspection: codes [n][k] int8 (0 where dropped) and
 * mask [n][k] uint8 (1 where kept), row-major.
 */
int slim_unpack(const uint8_t *qvals, const uint8_t *meta, slim_shape shape, int8_t *codes,
                uint8_t *mask, void *stream);

/*
 * Scratch the forward calls need for a layer at m tokens (a HOST out-pointer).
 * The same size covers slim_linear_gemv (m <= 16), slim_linear_gemm and
 * slim_lowrank.
 * The workspace must be ZERO-FILLED ONCE before its first use (hipMemset):
 * its first bytes hold the decode path's T = X R^T between the kernels' two
 * phases (pieces tagged with a call number, never 0), and a fresh workspace
 * must not look like finished work (under stream capture the call number
 * lives in word 3 of the workspace and a one-thread kernel enqueued ahead of
 * the decode kernel advances it on every replay).  No result is carried between calls: one
 * workspace (of the largest size needed) can serve any sequence of layers and
 * token counts.  Two calls that overlap in time need two workspaces.
 * Diagnostics: the one-launch decode kernel waits, inside the kernel, for its own
 * T = X R^T; the wait is bounded.  Should it ever run out (it never should),
 * the outputs that depend on the missing part are NaN -- a failed call cannot
 * pass for a result -- and word 2 of the workspace is set to 1.
 * slim_workspace_check reads that word back: it synchronizes `stream` (so it is
 * not for graph capture), returns SLIM_ERR_WAIT and clears the word if a call on
 * this workspace gave up since the last check, else SLIM_OK.  workspace == NULL
 * checks the library's own scratch array on the current device
 * (slim_linear_gemv_static).
 */
int slim_workspace_bytes(const slim_layer *layer, int32_t m, size_t *bytes);
int slim_workspace_check(void *workspace, void *stream);

/*
 * slim_linear_gemv -- decode-shaped forward, 1 <= m <= 16 tokens (decoding runs
 * on small batches: Sec. 4 "Speedup").  Streams the packed
 * rows and the adapters once; fp16 inputs, fp32 accumulation, Y rounded once
 * to fp16.  X [m][k] fp16 in, Y [m][n] fp16 out.
 * One kernel launch wherever the geometry fits the device (every configured
 * LLaMA-2 shape at every token count: X streams through the LDS of a compute
 * unit in chunks where it does not fit whole), the two-launch kernels otherwise
 * (rank_pad above the chunk size, more row tiles than resident workgroups).
 * In the one-launch kernel T = X R^T is rounded to fp16 (per share of the
 * inputs, at most four, added in fp16), so |T| must stay below 65504 -- four
 * orders of magnitude above what N(0, 1) inputs with x20 outlier channels and
 * N(0, 0.01) adapters give; the two-launch kernels keep T in fp32.
 * Requires k % 128 == 0 and every buffer (packed codes, L, R, X, Y) below
 * 2 GiB: the kernels address them with 32-bit offsets.
 * Errors: NULL, SHAPE (m out of range, k, a buffer of 2 GiB or more), ALIGN,
 * WORKSPACE, HIP.
 */
int slim_linear_gemv(const slim_layer *layer, const slim_half *X, int32_t m, slim_half *Y,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * slim_linear_gemv_static -- slim_linear_gemv for callers that cannot allocate or
 * carry a workspace: code recorded under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same kernels, same results; the
 * workspace is an array of SLIM_STATIC_SCRATCH_BYTES inside the library's own code
 * object (one copy per GPU, zero when the library is loaded, held until the process
 * ends).  The call allocates and frees nothing and enqueues kernels only.
 *   - A call that needs more scratch than SLIM_STATIC_SCRATCH_BYTES is refused with
 *     SLIM_ERR_WORKSPACE and nothing is enqueued.  The one-launch kernel needs
 *     256 + 192 rank_pad + 256 * ceil(rank_pad / 4) bytes or so (under 200 KiB at rank 820);
 *     where the two-launch kernels run, the whole of slim_workspace_bytes (partial sums of
 *     slots x m x n floats; with 4-bit adapters also their fp16 expansion).  Every
 *     configured LLaMA-2 shape up to 28672 x 8192, rank 820, 16 tokens fits, with fp16
 *     and with 4-bit adapters.
 *   - The array belongs to the device that is current at the call (the device of
 *     `stream`); its address is looked up on the first call on each device -- make
 *     that first call outside stream capture.
 *   - Every call on a GPU shares that GPU's array: calls that overlap in time on one
 *     GPU (two streams, two threads) race on it.  Calls in stream order do not, and
 *     nothing has to be cleared between them (the kernels tag what they leave there
 *     with a call number, as in a caller-owned workspace).
 * Errors: as slim_linear_gemv, SLIM_ERR_WORKSPACE as above, SLIM_ERR_HIP if the
 * array's address cannot be obtained.
 */
#define SLIM_STATIC_SCRATCH_BYTES (8u << 20)
int slim_linear_gemv_static(const slim_layer *layer, const slim_half *X, int32_t m, slim_half *Y,
                            void *stream);

/*
 * slim_decode_override -- test and measurement control, process-wide: which of
 * its launch geometries slim_linear_gemv (and slim_lowrank up to 16 tokens)
 * takes from now on.  Not for production use: the automatic choice is the
 * product path.
 *   path    -1 automatic; 0 the two-launch kernels; 1 the one-launch kernel's two
 *           roles as two launches (where that geometry fits, else as 0); 2 as -1;
 *           3 a test of the kernel's bounded wait: where the one-launch geometry
 *           fits, only the half of the kernel that waits for T is launched, with
 *           the wait cut to 256 polls, so it gives up: every wavefront still ends
 *           normally, Y is NaN and the workspace's error word is set
 *           (slim_workspace_check then reports SLIM_ERR_WAIT);
 *   lds_kb  0: plan with the device's LDS; 16..160: with at most this many KiB
 *           (X then streams through the LDS in chunks on small layers too).
 * Errors: SHAPE (a value outside these ranges).
 */
int slim_decode_override(int32_t path, int32_t lds_kb);

/*
 * slim_decode_plan -- what slim_linear_gemv would launch for this layer (only
 * shape, rank_pad and adapter_bits are read) at m tokens; nothing is launched.
 * out: 12 ints (HOST pointer): [0] path (2: one launch, 1: its two roles as two
 * launches, 0: the two-launch kernels); for paths 1 and 2: [1] workgroups, [2]
 * threads per workgroup, [3] LDS bytes per workgroup, [4] workgroups of the
 * R role, [5] shares of the inputs in the R role, [6] wavefronts per row tile,
 * [7] working and [8] helper wavefronts per workgroup, [9] inputs per chunk of
 * X, [10] chunks, [11] workgroups of the Y role.  Errors: NULL, SHAPE.
 */
int slim_decode_plan(const slim_layer *layer, int32_t m, int32_t *out);

/*
 * slim_gemm_tile_order -- which output tile (512 rows x 128 tokens) each
 * workgroup of slim_linear_gemm's main kernel works on, for a layer of n rows
 * at m tokens (m below the chunk the call walks X in); host logic only, nothing
 * is launched (inspection and tests).  out (HOST pointer, count ints):
 * [0] tiles = ceil(n / 512) * ceil(m / 128), [1] how many of them the launch
 * with whole tiles takes (the others are cut into halves or quarters by a
 * second launch, in the same order), [2 + w] = row tile + ceil(n / 512) *
 * token tile of workgroup w.  Every tile appears exactly once.  The order
 * hands the workgroups that share a die's L2 a compact block of the layer.
 * Errors: NULL, SHAPE (n or m < 1, count < tiles + 2).
 */
int slim_gemm_tile_order(int32_t n, int32_t m, int32_t *out, size_t count);

/*
 * slim_linear_gemm -- prefill-shaped forward, any m >= 1 (meant for m >= 64):
 * Y = X W^C + (X L) R of Sec. 3.2 in this header's orientation; by the count of
 * App. "Computation Reduction Analysis" (Eq. 13) the 2:4 mask halves the
 * multiply-adds of the weight term, quantization saves none, and the adapters
 * add 2 m r (n + k).
 * Matrix-core GEMM over the compressed weights with the adapter product
 * T = X R^T (rounded once to fp16) folded in as extra k-steps, row scale
 * applied to the fp32 accumulators, Y rounded once to fp16.
 * Requires k % 128 == 0.  Errors as slim_linear_gemv.
 */
int slim_linear_gemm(const slim_layer *layer, const slim_half *X, int32_t m, slim_half *Y,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * slim_lowrank -- the adapter term alone (Sec. 3.2; cost O(2 b r d^2), App.
 * "Rank Analysis"):  Y = (X R^T) L^T  or, with accumulate != 0,  Y += ...
 * L, R as in slim_layer (adapter layout); shape.rank >= 1;
 * k % 128 == 0.  In accumulate mode Y is read as fp16, added to in fp32 and
 * rounded back once.  Up to 16 tokens the call is slim_linear_gemv's kernel
 * without the packed term (one launch where that geometry fits), above that
 * two dense matrix-core products with T = X R^T rounded to fp16 in between.
 * Workspace as for the forward calls (slim_workspace_bytes of a layer of this
 * shape); kernels only, so the call can be captured into a HIP graph like them.
 */
int slim_lowrank(const slim_half *X, int32_t m, const slim_half *R, const slim_half *L,
                 slim_shape shape, int32_t rank_pad, slim_half *Y, int accumulate,
                 void *workspace, size_t workspace_bytes, void *stream);

/*
 * slim_input_quant_fp8 -- 8-bit input quantization as the paper evaluates it
 * (App. "Input Quantization"): AbsMax quantization of an input tensor to FP8
 * with one scale per tensor; Xq holds the quantized values back on the fp16
 * grid, which is what the layer is then run on.
 *   M = max|X|;  format E4M3 (largest value 448) unless M > 448, then E5M2
 *   (largest value 57344);  scale = M / (largest value), one binary32 division
 *   (1 for a zero tensor);  Xq = fp16( fp8(x / scale) * scale ), quotient and
 *   product in binary32, fp8(): nearest value of the format, ties to even,
 *   subnormals included.
 * X, Xq: `count` fp16 values (Xq may be X); info: two floats out (scale; 0 for
 * E4M3, 1 for E5M2); workspace: at least 1024 bytes, need not be zeroed.
 * X must be finite.  Errors: NULL, SHAPE (count = 0), ALIGN, WORKSPACE, HIP.
 */
int slim_input_quant_fp8(const slim_half *X, size_t count, slim_half *Xq, float *info, void *workspace,
                         size_t workspace_bytes, void *stream);

/*
 * slim_input_quant_fp8_codes -- slim_input_quant_fp8 that also writes the 8-bit
 * codes of the quantized values (Xb: `count` bytes): sign in bit 7, then the
 * exponent field (4 bits, bias 7, for E4M3; 5 bits, bias 15, for E5M2) and the
 * mantissa (3 or 2 bits), subnormals with exponent field 0 -- the OCP 8-bit
 * formats.  value(Xb[i]) * scale is the quantized value before its rounding to
 * fp16 in Xq.  Either of Xq and Xb may be NULL (not both).  Errors as
 * slim_input_quant_fp8; ALIGN also for Xb.
 */
int slim_input_quant_fp8_codes(const slim_half *X, size_t count, slim_half *Xq, uint8_t *Xb, float *info,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * slim_linear_gemm_fp8 -- slim_linear_gemm on an input tensor quantized to 8 bits
 * (App. "Input Quantization": AbsMax FP8 quantization of the layer's input, one
 * scale per tensor):  with Xv = scale * value(X8), the exact quantized values,
 *   Y = Xv W^C + (Xv L) R   in the orientation of Sec. 3.2.
 * The weight term runs on the 8-bit structured-sparse matrix instruction (the
 * int4 weights are exact in E5M2, the products exact in binary32); the adapter
 * product T = Xv R^T reads the codes too (half the bytes), turns them into
 * fp16 exactly and goes on as in slim_linear_gemm.
 *   X8      [m][k] 8-bit codes, x_info = {scale, format} (DEVICE pointers): outputs
 *           of slim_input_quant_fp8_codes for the tensor;
 *   format  0 = E4M3, 1 = E5M2: what x_info[1] holds (the caller reads it back
 *           once, or knows it from the range of its activations: E4M3 unless
 *           max|X| > 448).
 * Everything else, the workspace included, as slim_linear_gemm.  Errors as
 * slim_linear_gemm; SHAPE also for a format other than 0 or 1.
 */
int slim_linear_gemm_fp8(const slim_layer *layer, const uint8_t *X8, const float *x_info, int32_t format, int32_t m,
                         slim_half *Y, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement aids (they compute nothing of the method): what this machine
 * delivers on a plain streaming read and on back-to-back matrix instructions,
 * to set beside the nominal peaks when a kernel's roofline fraction is quoted
 * (Sec. 4 "Speedup" measures layers; these give the ceilings such a layer has
 * here).
 *   slim_probe_read  `repeats` launches; launch i reads `bytes` (>= 64 KiB; whole
 *                    runs of 64 KiB) at buf + i * stride once, with 128-bit loads
 *                    from up to 2048 workgroups (the buffer must hold
 *                    (repeats - 1) * stride + bytes; a stride of at least
 *                    `bytes` makes every launch read cold data).  The caller
 *                    times the call.  sink: 4 device bytes, left unchanged.
 *   slim_probe_mfma  `workgroups` x 4 wavefronts each issue 4 x iters matrix
 *                    instructions on four independent accumulators:
 *                    V_MFMA_F32_32X32X16_F16 (sparse = 0) or
 *                    V_SMFMAC_F32_32X32X32_F16 (sparse = 1, counted as the dense
 *                    32 x 32 x 32 product it stands for).  *flops (HOST pointer)
 *                    receives the FLOPs of the launch; sink: 4 device bytes.
 */
int slim_probe_read(const void *buf, size_t bytes, int32_t repeats, size_t stride, void *sink,
                    void *stream);
int slim_probe_mfma(int32_t sparse, int32_t iters, int32_t workgroups, void *sink, double *flops,
                    void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SLIM_H */
