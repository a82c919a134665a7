/*
 * mp8 -- the 8-bit floating point (s=1, e=5, m=2) training primitive of
 * "Mixed Precision Training With 8-bit Floating Point" (arXiv 1905.12334) for AMD
 * MI355X (gfx950).  C ABI of libmp8.so.
 *
 * General rules for every entry point that takes a `stream`:
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library never
 *     allocates, frees or keeps them.  Tensors are row-major, last dimension contiguous.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call only
 *     enqueues work on that stream and returns; it never synchronises.
 *   - Errors are return codes.  Every check of a call, including those of the later launches of
 *     a call made of several launches, is done before its first launch: on any error other
 *     than MP8_ERR_HIP nothing has been enqueued.  (MP8_ERR_HIP reports that the runtime refused
 *     a launch; for a call made of several launches the earlier ones may then be enqueued.)
 *   - `stats`, where present, is a nullable DEVICE pointer to an mp8_stats that the caller
 *     zeroes; calls accumulate into it (atomic max / atomic add), so one struct can collect
 *     a whole step.
 *   - Random bits for stochastic rounding come from Philox4x32-10 keyed by `seed`, with the
 *     call's `offset` in the upper counter words and the element's row-major linear index
 *     selecting counter and halfword (see mp8_sr_bits).  The same (seed, offset, index)
 *     always gives the same bits, whatever the launch shape.
 */
#ifndef MP8_H
#define MP8_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MP8_OK = 0,
    MP8_ERR_INVALID_ARG = 1, /* null pointer, negative size, bad enum value            */
    MP8_ERR_UNSUPPORTED = 2, /* a shape or stride the kernels cannot handle            */
    MP8_ERR_ALIGNMENT = 3,   /* pointer or leading dimension not aligned as required   */
    MP8_ERR_WORKSPACE = 4,   /* workspace missing or smaller than the query says       */
    MP8_ERR_HIP = 5          /* the HIP runtime refused the launch                     */
} mp8_status;

/* Rounding of a down-conversion (Section 3.2): round to nearest even, or stochastic
 * rounding with 16 random bits per element. */
typedef enum { MP8_RNE = 0, MP8_SR = 1 } mp8_round;

/* Which of the three training GEMMs (Section 3, Figure 1a). */
typedef enum { MP8_FWD = 0, MP8_BWD_DATA = 1, MP8_WGRAD = 2 } mp8_op;

enum {
    /* Finite values beyond the largest normal (57344) become +-57344 instead of +-Inf. */
    MP8_FLAG_SATURATE = 1,
    /* mp8_gemm_fp8 only: an operand is stored with the contraction index as the slow one:
     * a as [kc, rows] (out[r, c] = sum_j a[j, r] * ...), b as [kc, cols].  With both flags the
     * weight gradient reads X8 [M, K] and dY8 [M, N] as the Q node writes them; with the b flag
     * alone the forward GEMM reads W8 [K, N]: no transposed copy of any tensor is needed.
     * (a alone is not supported.) */
    MP8_FLAG_A_CONTRACTION_MAJOR = 2,
    MP8_FLAG_B_CONTRACTION_MAJOR = 4,
    MP8_FLAG_CONTRACTION_MAJOR = 6
};

typedef struct {
    uint32_t amax_bits; /* max over elements of the FP32 bit pattern of |value before
                           rounding|; any NaN counts as 0x7FC00000                     */
    uint32_t nonfinite; /* number of produced (quantize, gemm) or consumed (update)
                           8-bit codes that are Inf or NaN                             */
    uint32_t zeroed;    /* number of non-zero values that were rounded to +-0          */
    uint32_t rsvd;
} mp8_stats;

/*
 * The Q node of Figure 1a: dst[i] = Q(fl32(src[i] * scale)), one IEEE single multiply
 * followed by one rounding to the 8-bit format.  `scale` is where the loss scale of
 * Section 3.1 is applied to error tensors (1.0f otherwise).
 *   src        [rows, cols] FP32, or IEEE half if src_is_f16 != 0; 16-byte aligned
 *   dst        [rows, cols] 8-bit codes; 16-byte aligned
 *   dst_t      nullable; [cols, rows], the same codes transposed (rounded once, stored
 *              twice); 16-byte aligned
 *   NaN -> 0x7F.  Overflow -> +-Inf (0x7C/0xFC), or +-57344 with MP8_FLAG_SATURATE.
 *   rows*cols == 0 is valid and does nothing.
 */
mp8_status mp8_quantize_e5m2(const void *src, int src_is_f16, uint8_t *dst, uint8_t *dst_t,
                             int64_t rows, int64_t cols, float scale, mp8_round round,
                             int flags, uint64_t seed, uint64_t offset, mp8_stats *stats,
                             void *stream);

/*
 * Several Q nodes in one launch: a training step quantises its activations and its errors (and
 * whatever else is due) at the same point of the flow of Figure 1a, and short tensors cost
 * little more than their bytes when they run beside a long one.  Item i gives exactly the
 * result of
 *     mp8_quantize_e5m2(src, src_is_f16, dst, NULL, 1, n, scale, round, flags, seed, offset, stats)
 * (flat tensors, no transposed copy; SR uses the element index).  `items` is a host array, read
 * before the call returns; count <= MP8_QUANTIZE_BATCH_MAX.  Items must not overlap each other's
 * outputs; items may share one mp8_stats.  On error nothing is enqueued.
 */
#define MP8_QUANTIZE_BATCH_MAX 8
typedef struct {
    const void *src;  /* device, FP32 or IEEE half, 16-byte aligned */
    int src_is_f16;
    uint8_t *dst;     /* device, 16-byte aligned */
    int64_t n;        /* elements; 0 is valid */
    float scale;
    mp8_round round;
    int flags;        /* MP8_FLAG_SATURATE or 0 */
    uint64_t seed, offset;
    mp8_stats *stats; /* nullable, device */
} mp8_quantize_item;
mp8_status mp8_quantize_e5m2_batch(const mp8_quantize_item *items, int count, void *stream);

/*
 * The FP8 compute primitive of Section 3: two 8-bit operands, FP32 accumulation, and the
 * result rounded once to 8 bits in the epilogue (the Q node after each GEMM in Figure 1a).
 *
 * (M, N, K) are always the LAYER dimensions X[M,K] . W[K,N] = Y[M,N]; `op` selects the
 * contraction.  Both operands are passed with the contraction index contiguous:
 *        out[r, c] = sum_j a[r, j] * b[c, j]
 *     MP8_FWD       a = X8   [M, K]   b = W8^T  [N, K]   out [M, N]   contraction K
 *     MP8_BWD_DATA  a = dY8  [M, N]   b = W8    [K, N]   out [M, K]   contraction N
 *     MP8_WGRAD     a = X8^T [K, M]   b = dY8^T [N, M]   out [K, N]   contraction M
 *   lda, ldb   leading dimensions in elements (>= contraction length, multiples of 16; with
 *              a contraction-major flag: >= rows resp. cols of the output)
 *   a, b       16-byte aligned
 *   alpha      out8 = Q(fl32(alpha * acc)); acc itself is stored unscaled
 *   acc        nullable FP32 [rows, cols] (16-byte aligned).  acc_mode 0: not touched;
 *              1: receives the FP32 accumulator; 2: acc += accumulator, and out8 is the
 *              rounding of the updated acc (accumulation across calls, e.g. timesteps)
 *   out8       nullable [rows, cols] 8-bit result; out8_t nullable [cols, rows] transposed
 *   round      rounding of the epilogue; SR uses index r*cols + c
 *   workspace  device scratch, 16-byte aligned, contents undefined afterwards.  It is needed
 *              when the contraction is split (few output tiles, long contraction), for
 *              acc_mode 2, for out8_t, and when cols is not a multiple of 16;
 *              mp8_gemm_fp8_workspace_bytes(op, M, N, K) is enough in every case.  A call
 *              that does not need it accepts NULL.
 * Any contraction length >= 1 and any rows/cols >= 1 are accepted (ragged shapes run on a
 * slower kernel); a zero dimension is valid and does nothing.  Partial sums of a split
 * contraction are combined in FP32, in a fixed order, before the single rounding, so results
 * are bit-reproducible run to run.
 */
mp8_status mp8_gemm_fp8(mp8_op op, int64_t M, int64_t N, int64_t K, const uint8_t *a,
                        int64_t lda, const uint8_t *b, int64_t ldb, float alpha, float *acc,
                        int acc_mode, uint8_t *out8, uint8_t *out8_t, mp8_round round,
                        int flags, uint64_t seed, uint64_t offset, mp8_stats *stats,
                        void *workspace, size_t workspace_bytes, void *stream);

/* Upper bound of the scratch mp8_gemm_fp8 can need for this shape, whatever the options
 * (0 for shapes that take the generic kernel). */
size_t mp8_gemm_fp8_workspace_bytes(mp8_op op, int64_t M, int64_t N, int64_t K);

/*
 * mp8_gemm_fp8 for callers that cannot allocate device memory and have no workspace at hand:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and, bit for bit, the same results as mp8_gemm_fp8 (automatic kernel choice), but
 * the scratch of the two-pass paths lives in a static device array inside the library instead of
 * a caller's workspace.  The call allocates and frees nothing.
 *   - Limit: shapes for which mp8_gemm_fp8_workspace_bytes(op, M, N, K) exceeds
 *     MP8_STATIC_SCRATCH_BYTES (32 MiB, also returned by mp8_static_scratch_bytes()) are
 *     rejected with MP8_ERR_WORKSPACE.  Each GPU the library runs on holds that array until the
 *     process ends.
 *   - The array is looked up once per device, on the first call with that device current (a
 *     symbol look-up, no allocation); the call must be made with the device of the tensors and
 *     of `stream` current.
 *   - Every call on a GPU shares that GPU's array: two calls whose kernels may overlap on one
 *     GPU (different streams, no dependency between them) race on it; calls on one stream, or
 *     ordered by events, are safe.  Nothing in the array has to be cleared between calls.
 */
#define MP8_STATIC_SCRATCH_BYTES (32u << 20)
mp8_status mp8_gemm_fp8_static(mp8_op op, int64_t M, int64_t N, int64_t K, const uint8_t *a,
                               int64_t lda, const uint8_t *b, int64_t ldb, float alpha, float *acc,
                               int acc_mode, uint8_t *out8, uint8_t *out8_t, mp8_round round,
                               int flags, uint64_t seed, uint64_t offset, mp8_stats *stats,
                               void *stream);
size_t mp8_static_scratch_bytes(void);

/*
 * As mp8_gemm_fp8 with the kernel choice made by the caller (for tuning and tests):
 * tile_config 0 = automatic, otherwise an index below mp8_gemm_num_tile_configs() + 1;
 * split_k 0 = automatic, otherwise the number of contraction slices.  Workspace need:
 * mp8_gemm_fp8_workspace_bytes_tuned with the same two values.
 */
mp8_status mp8_gemm_fp8_tuned(mp8_op op, int64_t M, int64_t N, int64_t K, const uint8_t *a,
                              int64_t lda, const uint8_t *b, int64_t ldb, float alpha,
                              float *acc, int acc_mode, uint8_t *out8, uint8_t *out8_t,
                              mp8_round round, int flags, uint64_t seed, uint64_t offset,
                              mp8_stats *stats, void *workspace, size_t workspace_bytes,
                              void *stream, int tile_config, int split_k);
size_t mp8_gemm_fp8_workspace_bytes_tuned(mp8_op op, int64_t M, int64_t N, int64_t K,
                                          int tile_config, int split_k);
/* Host only: which kernel an aligned call with these arguments would take -- *tile_out the tile
 * configuration (1-based; 0 = the any-shape kernel), *splits_out the number of contraction
 * slices.  For tests and tuning. */
mp8_status mp8_gemm_fp8_plan(mp8_op op, int64_t M, int64_t N, int64_t K, int flags, int tile_config,
                             int split_k, int *tile_out, int *splits_out);
int mp8_gemm_num_tile_configs(void);
/* Writes "BMxBNxBK" style description of tile_config (1-based) into buf. */
int mp8_gemm_tile_config_name(int tile_config, char *buf, size_t buflen);
/* Diagnostic (needs a device): bytes of statically allocated LDS of the row-major kernel of
 * tile_config (1-based) with epilogue variant epi (0 FP32 tiles, 1 RNE only, 2 complete), as the
 * runtime reports them; -1 on error.  The number of workgroups a CU holds hangs on it, so the
 * tests pin it to what the tile shape implies. */
int mp8_gemm_tile_config_lds_bytes(int tile_config, int epi);

/*
 * The same primitive for a 3x3 convolution (stride 1, zero padding 1; Section 3 applies the
 * 8-bit format to every convolution and GEMM kernel, Section 4 trains residual networks), as
 * an implicit GEMM: no lowered (im2col) copy of the activations exists.
 *
 * Activations and errors are channels-last on the ZERO-PADDED pixel grid: a tensor with C
 * channels is [prows, C] with prows >= B*(H+2)*(W+2); row (b*(H+2) + y)*(W+2) + x holds pixel
 * (y-1, x-1) of image b, rows with y in {0, H+1} or x in {0, W+1} and rows beyond the last
 * image are padding and hold zero codes.  The operand `a` (read at shifted pixel positions)
 * must in addition be readable for W+3 rows before its first and after its last row, and
 * those guard rows must hold finite codes (they only ever meet padding).  Weights are
 * w8 [3, 3, Cin, Cout].
 *     MP8_FWD       a = x8 [prows, Cin]   b = w8                out  y8  [prows, Cout]
 *     MP8_BWD_DATA  a = e8 [prows, Cout]  b = w8                out  dx8 [prows, Cin]
 *     MP8_WGRAD     a = x8 [prows, Cin]   b = e8 [prows, Cout]  out  dw8 [3, 3, Cin, Cout]
 * Padding rows of y8 / dx8 are written as zero codes (so an output can be the next input) and
 * do not enter the statistics; acc, if requested, has the shape of out and its padding rows are
 * unspecified.  SR uses the row-major index of the output matrix.  Cin and Cout must be
 * multiples of 64 (the residual networks of Section 4 start at 64 channels) below 32768, W below
 * 32768, and prows a multiple of 128 for MP8_WGRAD (MP8_ERR_UNSUPPORTED otherwise).
 * Everything else (alpha, acc_mode, round, flags = MP8_FLAG_SATURATE or 0, stats, workspace)
 * as for mp8_gemm_fp8.
 */
mp8_status mp8_conv3x3_fp8(mp8_op op, int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout,
                           int64_t prows, const uint8_t *a, const uint8_t *b, float alpha,
                           float *acc, int acc_mode, uint8_t *out8, mp8_round round, int flags,
                           uint64_t seed, uint64_t offset, mp8_stats *stats, void *workspace,
                           size_t workspace_bytes, void *stream);
size_t mp8_conv3x3_fp8_workspace_bytes(mp8_op op, int64_t B, int64_t H, int64_t W, int64_t Cin,
                                       int64_t Cout, int64_t prows);

/*
 * The weight-update path of Figure 1b on half-precision master weights, per element:
 *     g    = fl32(value(g8[i]) * inv_loss_scale)     un-scaling in full precision
 *     w    = float(w16[i])
 *     w'   = fmaf(-lr, g, w)                         32-bit update
 *     w16[i] = half(w') rounded by `round` (SR uses index i)
 *   w16              in/out IEEE half codes, 16-byte aligned
 *   g8               8-bit weight gradients, 16-byte aligned
 *   skip_if_nonzero  nullable device word; if it is non-zero when the kernel runs, nothing
 *                    is written (an overflowed step is skipped without a host round trip)
 *   w8_out           nullable; receives Q_RNE(new w16[i]), the next step's 8-bit weights
 *   stats->nonfinite counts Inf/NaN codes in g8 (counted even when skipping)
 */
mp8_status mp8_sgd_update_fp16_sr(uint16_t *w16, const uint8_t *g8, int64_t n, float lr,
                                  float inv_loss_scale, mp8_round round, uint64_t seed,
                                  uint64_t offset, const uint32_t *skip_if_nonzero,
                                  uint8_t *w8_out, mp8_stats *stats, void *stream);

/*
 * The same path with the momentum optimizer of Figure 1b and the L2 regularisation term of
 * Eq. 1 (its gradient enters as weight_decay * w), per element:
 *     g  = fmaf(weight_decay, w, fl32(value(g8[i]) * inv_loss_scale))
 *     v' = fmaf(momentum, velocity[i], g)        velocity is FP32, in/out, 16-byte aligned
 *     w' = fmaf(-lr, v', w);   w16[i] = half(w') rounded by `round`
 * With momentum = weight_decay = 0 the weights equal those of mp8_sgd_update_fp16_sr.  Other
 * arguments as there; a skipped step leaves the velocity untouched too.
 */
mp8_status mp8_sgd_momentum_fp16_sr(uint16_t *w16, float *velocity, const uint8_t *g8, int64_t n,
                                    float lr, float inv_loss_scale, float momentum,
                                    float weight_decay, mp8_round round, uint64_t seed,
                                    uint64_t offset, const uint32_t *skip_if_nonzero,
                                    uint8_t *w8_out, mp8_stats *stats, void *stream);

/*
 * The same path with the ADAM optimizer, which Section 4 names for the translation networks
 * (the paper gives no formula: Kingma & Ba, Algorithm 1), with the regularisation gradient of
 * Eq. 1 as above.  Per element, every operation a separately rounded FP32 operation:
 *     g  = fmaf(weight_decay, w, fl32(value(g8[i]) * inv_loss_scale))
 *     m' = fmaf(beta1, m[i], (1 - beta1) * g);   v' = fmaf(beta2, v[i], (1 - beta2) * (g * g))
 *     w' = fmaf(-lr, (m' / c1) / (sqrt(v' / c2) + eps), w),   c_i = fl32(1 - beta_i^step)
 *     w16[i] = half(w') rounded by `round`
 *   m, v    FP32 moments, in/out, 16-byte aligned (a skipped step leaves them untouched)
 *   step    number of this update, counted from 1 (beta_i^step is formed in double on the host)
 * Other arguments as for mp8_sgd_update_fp16_sr.  21 bytes of traffic per element.
 */
mp8_status mp8_adam_fp16_sr(uint16_t *w16, float *m, float *v, const uint8_t *g8, int64_t n, float lr,
                            float inv_loss_scale, float beta1, float beta2, float eps,
                            float weight_decay, int64_t step, mp8_round round, uint64_t seed,
                            uint64_t offset, const uint32_t *skip_if_nonzero, uint8_t *w8_out,
                            mp8_stats *stats, void *stream);

/*
 * Figure 1b from the weight-gradient GEMM to the next step's weights in one call: the weight
 * gradient is accumulated in FP32 and rounded once to 8 bits (as mp8_gemm_fp8 with MP8_WGRAD:
 * a, lda, b, ldb, alpha, flags incl. the contraction-major ones, g_round / g_seed / g_offset for
 * that rounding, stats), and the finishing pass that rounds it also applies
 * mp8_sgd_update_fp16_sr to the master weights w16 [K, N] with the codes it has just produced
 * (lr, inv_loss_scale, w_round / w_seed / w_offset, skip_if_nonzero, w8_out as there).  The
 * results are bit for bit those of the two separate calls.
 *   skip_if_nonzero  as there.  The finishing pass reads the flag when it starts, so a flag that
 *              earlier work on the stream has written (the overflow count of the error tensor's
 *              Q node) is honoured as it is.  A flag that lies inside *stats would still be
 *              counted by this very call (the gradient's own Inf/NaN codes) while the pass that
 *              reads it runs: such a call runs the weight gradient and the update as two
 *              launches, the update then sees the final count; it needs g8_out
 *              (MP8_ERR_INVALID_ARG without it).
 *   g8_out     nullable [K, N]: the 8-bit weight gradient, if the caller wants to keep it
 *   workspace  at least mp8_gemm_fp8_workspace_bytes(MP8_WGRAD, M, N, K) bytes, always needed
 *              when that is non-zero
 * Shapes that only the any-shape GEMM kernel takes run as the two separate launches and need
 * g8_out (MP8_ERR_UNSUPPORTED without it).  A weight gradient whose contraction is not split
 * rounds in the GEMM's own epilogue; it is then followed by the update kernel instead of being
 * forced through a finishing pass (cheaper: no FP32 copy of the result is written), with the codes
 * in g8_out, or in the first K*N bytes of the workspace if the caller passes no g8_out and the
 * workspace is that large.
 */
mp8_status mp8_wgrad_update_fp16_sr(int64_t M, int64_t N, int64_t K, const uint8_t *a, int64_t lda,
                                    const uint8_t *b, int64_t ldb, float alpha, uint8_t *g8_out,
                                    mp8_round g_round, int flags, uint64_t g_seed, uint64_t g_offset,
                                    mp8_stats *stats, uint16_t *w16, float lr, float inv_loss_scale,
                                    mp8_round w_round, uint64_t w_seed, uint64_t w_offset,
                                    const uint32_t *skip_if_nonzero, uint8_t *w8_out, void *workspace,
                                    size_t workspace_bytes, void *stream);

/* The same for the weight gradient of the 3x3 convolution (operands as mp8_conv3x3_fp8 with
 * MP8_WGRAD: x8 and e8 padded channels-last; w16, g8_out, w8_out are [3, 3, Cin, Cout]).  The
 * workspace (mp8_conv3x3_fp8_workspace_bytes for MP8_WGRAD, at least 36 * Cin * Cout bytes) is
 * always needed. */
mp8_status mp8_conv3x3_wgrad_update_fp16_sr(
    int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t prows, const uint8_t *x8,
    const uint8_t *e8, float alpha, uint8_t *g8_out, mp8_round g_round, int flags, uint64_t g_seed,
    uint64_t g_offset, mp8_stats *stats, uint16_t *w16, float lr, float inv_loss_scale,
    mp8_round w_round, uint64_t w_seed, uint64_t w_offset, const uint32_t *skip_if_nonzero,
    uint8_t *w8_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The Q node on the activations and the forward GEMM it feeds (Figure 1a) in one call:
 *     x8_out = Q(fl32(x * x_scale))            exactly as mp8_quantize_e5m2 (FP32 source, x_round,
 *                                              x_flags, x_seed / x_offset, x_stats)
 *     out    = x8_out [M, K] . w8 [K, N]       exactly as mp8_gemm_fp8 with MP8_FWD and
 *                                              MP8_FLAG_B_CONTRACTION_MAJOR (alpha, acc, acc_mode,
 *                                              out8, out8_t, round, flags, seed / offset, stats)
 * The results are bit for bit those of the two separate calls.  When the layer has at most 128
 * output columns (N a multiple of 16, K a multiple of 128) the GEMM reads the activations only
 * once, and one kernel does both: it reads x, rounds it, writes x8_out (the weight gradient needs
 * it later) and multiplies from the codes it holds.  Every other shape runs as the two calls.
 *   x          [M, K] FP32, dense, 16-byte aligned (device)
 *   x8_out     [M, K] 8-bit codes, dense, 16-byte aligned; always written
 *   w8         [K, N] 8-bit codes, row stride ldw >= N (the layout mp8_sgd_update_fp16_sr's
 *              w8_out produces); 16-byte aligned rows for the fused kernel
 *   flags      MP8_FLAG_SATURATE or 0, for the output rounding; x_flags the same for x8_out
 *   workspace  as mp8_gemm_fp8_workspace_bytes(MP8_FWD, M, N, K) says; the fused kernel needs none
 * M*K == 0 or N == 0 is valid.  On error nothing is enqueued.
 */
mp8_status mp8_quantize_gemm_fwd_fp8(int64_t M, int64_t N, int64_t K, const float *x, float x_scale,
                                     mp8_round x_round, int x_flags, uint64_t x_seed, uint64_t x_offset,
                                     mp8_stats *x_stats, uint8_t *x8_out, const uint8_t *w8, int64_t ldw,
                                     float alpha, float *acc, int acc_mode, uint8_t *out8,
                                     uint8_t *out8_t, mp8_round round, int flags, uint64_t seed,
                                     uint64_t offset, mp8_stats *stats, void *workspace,
                                     size_t workspace_bytes, void *stream);

/*
 * mp8_wgrad_update_fp16_sr and mp8_conv3x3_wgrad_update_fp16_sr with the momentum optimizer of
 * mp8_sgd_momentum_fp16_sr in the finishing pass (the weight-update path of Figure 1b passes the
 * un-scaled gradients to a momentum optimizer): velocity [K, N] (or [3, 3, Cin, Cout]) FP32, in/out, 16-byte aligned; momentum
 * and weight_decay as there; every other argument as in the calls they extend.  The results --
 * gradient codes, master weights, velocity, 8-bit weights -- are bit for bit those of the
 * weight-gradient call followed by mp8_sgd_momentum_fp16_sr.
 */
mp8_status mp8_wgrad_momentum_fp16_sr(int64_t M, int64_t N, int64_t K, const uint8_t *a, int64_t lda,
                                      const uint8_t *b, int64_t ldb, float alpha, uint8_t *g8_out,
                                      mp8_round g_round, int flags, uint64_t g_seed, uint64_t g_offset,
                                      mp8_stats *stats, uint16_t *w16, float *velocity, float lr,
                                      float inv_loss_scale, float momentum, float weight_decay,
                                      mp8_round w_round, uint64_t w_seed, uint64_t w_offset,
                                      const uint32_t *skip_if_nonzero, uint8_t *w8_out, void *workspace,
                                      size_t workspace_bytes, void *stream);
mp8_status mp8_conv3x3_wgrad_momentum_fp16_sr(
    int64_t B, int64_t H, int64_t W, int64_t Cin, int64_t Cout, int64_t prows, const uint8_t *x8,
    const uint8_t *e8, float alpha, uint8_t *g8_out, mp8_round g_round, int flags, uint64_t g_seed,
    uint64_t g_offset, mp8_stats *stats, uint16_t *w16, float *velocity, float lr, float inv_loss_scale,
    float momentum, float weight_decay, mp8_round w_round, uint64_t w_seed, uint64_t w_offset,
    const uint32_t *skip_if_nonzero, uint8_t *w8_out, void *workspace, size_t workspace_bytes,
    void *stream);

/*
 * The same with ADAM (mp8_adam_fp16_sr: m, v [K, N] FP32 moments in place, beta1, beta2, eps,
 * weight_decay, step counted from 1) in the finishing pass of the weight-gradient GEMM; bit for
 * bit the weight-gradient call followed by mp8_adam_fp16_sr.
 */
mp8_status mp8_wgrad_adam_fp16_sr(int64_t M, int64_t N, int64_t K, const uint8_t *a, int64_t lda,
                                  const uint8_t *b, int64_t ldb, float alpha, uint8_t *g8_out,
                                  mp8_round g_round, int flags, uint64_t g_seed, uint64_t g_offset,
                                  mp8_stats *stats, uint16_t *w16, float *m, float *v, float lr,
                                  float inv_loss_scale, float beta1, float beta2, float eps,
                                  float weight_decay, int64_t step, mp8_round w_round, uint64_t w_seed,
                                  uint64_t w_offset, const uint32_t *skip_if_nonzero, uint8_t *w8_out,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * Diagnostic, for benchmarks: a kernel that only moves bytes, in the access pattern and with the
 * read:write ratio of the streaming kernels above (Section 3 calls the weight update a
 * bandwidth-bound operation; this is the stick that bound is measured with).  Reads read_bytes
 * from src (device, 16-byte aligned, a multiple of 16) and writes read_bytes / reads_per_write
 * bytes to dst: reads_per_write = 4 is the Q node's ratio (FP32 in, one byte out), 1 a plain copy
 * (the optimizers with FP32 state).  The bytes written are a function of the bytes read, of no
 * other use.
 */
mp8_status mp8_stream_probe(const void *src, void *dst, int64_t read_bytes, int reads_per_write,
                            void *stream);

/* out[i] = the 16 random bits element i would use (device array of n uint16), for tests. */
mp8_status mp8_sr_bits(uint16_t *out, int64_t n, uint64_t seed, uint64_t offset, void *stream);

/* Host: one Philox4x32-10 block (Salmon et al., SC'11).  Host pointers. */
void mp8_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/*
 * Host-side loss scaler of Section 3.1: back-off dynamic scaling with a minimum threshold
 * that the caller raises as training proceeds.  update(): nonfinite != 0 halves the scale
 * (not below `floor`), resets the clean-step count and returns 1 (skip the step);
 * otherwise counts a clean step, doubles the scale after growth_interval of them (growth stops
 * at MP8_SCALER_MAX = 2^32: the scale and its reciprocal stay exact FP32 numbers, and a run
 * without overflows does not double without end), returns 0.
 */
#define MP8_SCALER_MAX 4294967296.0
typedef struct {
    double scale;
    double floor;
    int64_t growth_interval;
    int64_t good_steps;
} mp8_scaler;
void mp8_scaler_init(mp8_scaler *s, double scale, double floor, int64_t growth_interval);
int mp8_scaler_update(mp8_scaler *s, uint32_t nonfinite);
void mp8_scaler_set_floor(mp8_scaler *s, double floor);

const char *mp8_status_string(mp8_status status);

#ifdef __cplusplus
}
#endif
#endif /* MP8_H */
