/*
 * adapt_mi355 -- approximate-multiplier GEMM / convolution by table lookup on MI355X (gfx950).
 *
 * C ABI of the hot path of AdaPT (arXiv 2203.04071): per layer
 *     quantise (Sec. III-A)  ->  matrix product in which every b-bit x b-bit
 *     multiply is one entry of a 2^b x 2^b table (Sec. III-C, IV)  ->  dequantise,
 * for linear layers, 2-D convolutions (Sec. III-B) and transposed convolutions
 * (the generator networks of Sec. V), plus the small fp32 operations that sit
 * between approximate layers in the CNN / LSTM / GAN workloads.
 *
 * General rules
 *   - Every function returns ADAPT_OK (0) or a negative error code; nothing
 *     throws, aborts or synchronises the device unless stated.  A text for the
 *     last error of the calling thread is available from adapt_last_error().
 *   - Pointers named *_dev are DEVICE pointers owned by the caller; pointers
 *     named *_host are HOST pointers.  The library never frees caller memory
 *     and never keeps a caller pointer after the call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Kernels are enqueued on it and the call returns without waiting.
 *   - Tensors are dense, row-major, in the layouts stated per function.
 *   - b = bits, H = 2^(b-1), Q = H - 1.  Quantised operands are signed integers
 *     in [-H, H-1] stored one per int8.  Passing values outside that range for
 *     the table's bit width is a caller error (the kernels wrap them into range,
 *     they never read outside the table).
 *   - Accumulators are int32 with two's-complement wrap-around.
 *   - Output buffers are overwritten, never accumulated into.
 *   - Handles (adapt_lut) own their device memory and belong to the device that
 *     was current when they were created.
 *   - Two calls that overlap in time on different streams are safe for the plain
 *     entry points (workspaces are allocated per call in stream order).  A packed
 *     weights handle owns a grow-only workspace: calls with the SAME handle must not
 *     overlap in time; once a handle has run at its largest input size its calls
 *     allocate nothing and may be recorded into a HIP graph (which a later call
 *     at a larger size, re-allocating the workspace, would invalidate).
 *   - Environment variables the library reads (debugging and measurement aids; results never depend on them):
 *     ADAPT_POISON_ALLOC   any value: every device allocation the library makes is filled with 0xA5 bytes before
 *                          use, so that code relying on fresh memory being zero shows up in tests.
 *     ADAPT_STE_TILE       64 or 128: forces the output tile of the gradient products of adapt_ste_*_backward_f32
 *     ADAPT_STE_KS         1 or 2: forces four or eight waves per workgroup there (both normally chosen from the shape).
 */
#ifndef ADAPT_MI355_H
#define ADAPT_MI355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ADAPT_OK 0
#define ADAPT_ERR_INVALID_ARGUMENT (-1) /* null pointer, bits outside [2,8], non-positive dims, bad geometry */
#define ADAPT_ERR_UNSUPPORTED (-2)      /* valid request this build does not implement */
#define ADAPT_ERR_LUT_RANGE (-3)        /* reserved: table entry not representable */
#define ADAPT_ERR_HIP (-4)              /* a HIP runtime call or kernel launch failed */
#define ADAPT_ERR_OUT_OF_MEMORY (-5)

/* thread-local text of the most recent error on this thread ("" if none); static storage */
const char *adapt_last_error(void);

/* Number of compute units of the current device (used by callers to report rooflines). <0 on error. */
int adapt_device_cu_count(void);

/* ------------------------------------------------------------------------------------------------
 * Multiplier table (Sec. III-C: one look-up table per approximate compute unit, a 1:1 image of the
 * multiplier; Sec. III: the unit may differ from layer to layer, so it is a per-call argument).
 *
 * table_host: HOST int32 [2^b][2^b]; the product of activation a and weight w, both in [-H, H-1],
 * is table_host[(a + H) * 2^b + (w + H)].  The table may be arbitrary (not symmetric, not zero for a
 * zero operand).  The call copies it (synchronously) into a device image in the library's private
 * order; the host array may be freed afterwards.
 * storage chosen: 0 = one int16 table (all entries in [-32768, 32767]);
 *                 1 = two 16-bit tables (high and low halves of int32 entries; kernels run twice).
 * ---------------------------------------------------------------------------------------------- */
typedef struct adapt_lut adapt_lut;

int adapt_lut_create(adapt_lut **out, int bits, const int32_t *table_host);
int adapt_lut_destroy(adapt_lut *lut);
int adapt_lut_info(const adapt_lut *lut, int *bits, int *storage, int32_t *min_entry, int32_t *max_entry);

/* ------------------------------------------------------------------------------------------------
 * Quantiser (Sec. III-A: affine map real = scale * q, zero point 0, any bit width).
 * ---------------------------------------------------------------------------------------------- */

/* amax_dev[0] = max |x_i| over n fp32 values (NaNs skipped; 0 for n == 0).  This is the "max absolute
 * number" scale choice of Sec. III-A; scale = amax / Q. */
int adapt_absmax_f32(const float *x_dev, size_t n, float *amax_dev, void *stream);

/* q_i = clamp(round_half_even(x_i / scale), -Q, Q), NaN -> 0.  scale > 0. */
int adapt_quantize_f32(const float *x_dev, int8_t *q_dev, size_t n, float scale, int bits, void *stream);

/* Dequantiser: y = float(acc) * scale, then (if bias_dev) + bias[c]; two separately rounded fp32
 * operations (Sec. III-A real = A * q; Sec. III-B "+ b").  Element (o, c, i) sits at
 * ((o * channels) + c) * inner + i:  linear -> outer = M, channels = N, inner = 1;
 * convolution NCHW -> outer = N, channels = Cout, inner = Hout * Wout.  scale = s_x * s_w, formed in
 * fp32 by the caller.  bias_dev: [channels] or NULL. */
int adapt_dequant_i32(const int32_t *acc_dev, float *y_dev, size_t outer, size_t channels, size_t inner,
                      float scale, const float *bias_dev, void *stream);

/* The quantiser as the paper configures it (Sec. III-A "Parameter calibration": weight ranges per output channel,
 * activation range calib_max from a histogram calibrator at a 99.9 % percentile; scale = range / Q as above).
 * The paper names the method, not the histogram; this library's definition: `bins` equal-width bins over [0, amax],
 * width = amax / bins, bin(v) = min(bins - 1, trunc(|v| / width)) (IEEE fp32 divisions), NaN not counted;
 * calib_max = (k + 1) * width for the first bin k whose cumulative count reaches ceil(total * num / den).
 * Values beyond calib_max saturate in the quantiser's clamp. */

/* amax_dev[r] = max |x[r][0..cols)| for rows of a dense [rows][cols] matrix (weights: one row per output channel) */
int adapt_absmax_rows_f32(const float *x_dev, size_t rows, size_t cols, float *amax_dev, void *stream);
/* q[r][c] = quantise(x[r][c], scales_dev[r], bits) as adapt_quantize_f32; every scale must be > 0 */
int adapt_quantize_rows_f32(const float *x_dev, int8_t *q_dev, size_t rows, size_t cols, const float *scales_dev, int bits,
                            void *stream);
/* adapt_dequant_i32 with one scale per channel: y = float(acc) * scales_dev[c] (+ bias[c]); scales_dev[c] = s_x * s_w[c] */
int adapt_dequant_i32_per_channel(const int32_t *acc_dev, float *y_dev, size_t outer, size_t channels, size_t inner,
                                  const float *scales_dev, const float *bias_dev, void *stream);
/* counts_dev[bin(x_i)] += 1 for i < n (uint32 [bins], 1 <= bins <= 4096; accumulated into, so the caller zeroes it
 * first and may add several batches); amax > 0 is the range (e.g. from adapt_absmax_f32) */
int adapt_histogram_abs_f32(const float *x_dev, size_t n, float amax, int bins, uint32_t *counts_dev, void *stream);
/* calib_max_dev[0] for the fraction num / den (99.9 %: 999 / 1000; den <= 2^20) of the counted values */
int adapt_percentile_from_histogram(const uint32_t *counts_dev, int bins, float amax, unsigned num, unsigned den,
                                    float *calib_max_dev, void *stream);
/* calib_max_dev[0] by least squared quantisation error (Sec. III-A names an MSE calibrator as an alternative, without a
 * definition; this one is: candidates are the bin edges t_k = (k + 1) * amax / bins; with the scale t_k / Q a value at
 * the centre c_j of bin j is reproduced as min(Q, rint(c_j / s)) * s; the candidate's error is sum_j counts[j] *
 * (c_j - that)^2 in fp64; the first candidate with the smallest error wins).  2 <= bits <= 16. */
int adapt_mse_from_histogram(const uint32_t *counts_dev, int bins, float amax, int bits, float *calib_max_dev, void *stream);
/* calib_max_dev[0] by least information loss (Sec. III-A names an entropy calibrator as the other alternative, without a
 * definition; this one is: with L = 2^(bits-1) levels, candidate k = min(L, bins) .. bins keeps the first k bins.
 * Reference p: the kept counts, everything beyond added to the last kept bin (where saturated values land).  Quantised q:
 * the kept counts alone, merged into min(L, k) groups of bins [g k / L, (g+1) k / L) and spread back evenly over each
 * group's non-empty bins.  The candidate's loss is the Kullback-Leibler divergence sum_j (p_j / P) log((p_j / P) /
 * (q_j / Q)) over its bins with p_j > 0 (P, Q the two totals; +inf when such a bin has q_j = 0), in fp64, j ascending;
 * the first candidate with the smallest loss wins: calib_max = k * amax / bins.  An empty histogram keeps amax.
 * 2 <= bits <= 16. */
int adapt_entropy_from_histogram(const uint32_t *counts_dev, int bins, float amax, int bits, float *calib_max_dev,
                                 void *stream);

/* ------------------------------------------------------------------------------------------------
 * Approximate layers (Sec. III-B, IV): every inner-product term is one table entry.
 * ---------------------------------------------------------------------------------------------- */

/* Linear layer y = x A^T:  acc[m][n] = sum_k T[a[m][k]][w[n][k]].
 * a_dev [M][K], w_dev [N][K], acc_dev [M][N].  M, N >= 0 (empty is a no-op), K >= 0 (K == 0 writes zeros). */
int adapt_approx_linear(const adapt_lut *lut, const int8_t *a_dev, const int8_t *w_dev, int32_t *acc_dev,
                        int M, int K, int N, void *stream);

/* adapt_approx_linear for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same integers.  The call makes no allocation of any kind (no
 * hipMalloc / hipMallocAsync / hipFree, also none hidden in a library routine): the row offsets it derives from w_dev
 * live in a static device array of 4 MiB that is part of the library's code object (each GPU the library runs on holds
 * it until the process ends; the first call on a device looks its address up).  Limit: K * (N rounded up to a multiple
 * of 16) * 4 bytes <= 4 MiB (e.g. K = N = 1024), beyond that ADAPT_ERR_UNSUPPORTED and nothing is launched.  Every
 * shape runs on the whole-table kernel (long matrices are faster through adapt_approx_linear or a packed handle).
 * All calls on one GPU share that array: two calls that overlap in time on one GPU (different streams or threads) race;
 * calls on one stream are ordered.  Nothing in the array has to start at zero (every call rewrites what it reads). */
int adapt_approx_linear_noalloc(const adapt_lut *lut, const int8_t *a_dev, const int8_t *w_dev, int32_t *acc_dev,
                                int M, int K, int N, void *stream);

/* 2-D convolution, x NCHW [N][Cin][H][W], w [Cout][Cin/groups][kh][kw], acc [N][Cout][Hout][Wout],
 * Hout = (H + 2 pad_h - dil_h (kh-1) - 1) / stride_h + 1 (likewise Wout).  The layer is the product of
 * the expanded input matrix with the filter matrix (Sec. III-B); a tap that falls into the padding is
 * an entry of that matrix equal to quantised zero, so T[0][w] IS added for it.
 * groups > 1 (Sec. III-B: "groups"; groups = Cin is the depthwise half of the separable convolution, eq. (1)):
 * output channel co belongs to group co / (Cout / groups) and meets only the Cin / groups input channels of that
 * group.  Cin and Cout must be multiples of groups (else ADAPT_ERR_INVALID_ARGUMENT). */
int adapt_approx_conv2d(const adapt_lut *lut, const int8_t *x_dev, const int8_t *w_dev, int32_t *acc_dev,
                        int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w,
                        int pad_h, int pad_w, int dil_h, int dil_w, int groups, void *stream);

/* Transposed 2-D convolution (generator networks), x [N][Cin][H][W], w [Cin][Cout][kh][kw],
 * acc [N][Cout][Hout][Wout], Hout = (H-1) stride - 2 pad + kh; input pixel (iy, ix) meets tap (ky, kx)
 * at output (iy stride - pad + ky, ix stride - pad + kx).  Only real (input, weight) pairs are looked
 * up; the zeros implied between input pixels never enter the multiplier.  output_padding 0, dilation 1. */
int adapt_approx_conv_transpose2d(const adapt_lut *lut, const int8_t *x_dev, const int8_t *w_dev,
                                  int32_t *acc_dev, int N, int Cin, int H, int W, int Cout, int kh, int kw,
                                  int stride, int pad, void *stream);

/* ------------------------------------------------------------------------------------------------
 * Pre-packed weights (the weights of a trained layer are static; the paper expands the filters into
 * a 2-D matrix once, Sec. III-B, and generates the table offline, Sec. III-C).  Packing combines the
 * two: for every inner index k and every block of 8 output channels it stores the table entries
 * T[a][w[n][k]] for all activations a, in the orders the two long-matrix kernels stream them (128-byte
 * lines; 256-byte lines of two-digit entries for the kernel that sums on the matrix pipe; both are made
 * by the pack call, nothing is added to a handle later, so a handle may be used from several threads).
 * The handle owns 2 * K * N * 2^b * 2 bytes of device memory, K and N rounded up to the kernels' tiles
 * (the first order twice for tables with entries beyond int16, which only that order serves) and
 * is tied to the device, the table contents and the weight values at pack time; w_dev may be freed
 * once the stream has passed the call.  The handle keeps a pointer to `lut`: the table handle must stay alive as long
 * as the weights handle is used (short linear layers run on the whole-table kernel with pre-packed row offsets).  The packed entry points give the same integers as the plain
 * ones; they skip the per-call packing that the plain entry points do for long matrices.
 * ---------------------------------------------------------------------------------------------- */
typedef struct adapt_weights adapt_weights;

/* w_dev [N][K] (linear layer, y = x A^T) */
int adapt_weights_pack_linear(adapt_weights **out, const adapt_lut *lut, const int8_t *w_dev, int K, int N,
                              void *stream);
/* w_dev [Cout][Cin][kh][kw] (groups = 1) */
int adapt_weights_pack_conv2d(adapt_weights **out, const adapt_lut *lut, const int8_t *w_dev, int Cout, int Cin,
                              int kh, int kw, void *stream);
/* w_dev [Cin][Cout][kh][kw], transposed convolution with the given stride (Sec. V generator networks).  When kh and kw
 * are multiples of the stride the layer is stored as stride^2 ordinary stride-1 convolutions (one per residue of the
 * output position modulo the stride), each over kh/stride x kw/stride taps.  The handle also keeps a copy of the
 * weights and a pointer to `lut` for geometries that form does not cover (a single input pixel, kernel or output sizes
 * that are no multiple of the stride): the table handle must stay alive as long as this handle is used. */
int adapt_weights_pack_conv_transpose2d(adapt_weights **out, const adapt_lut *lut, const int8_t *w_dev, int Cin, int Cout,
                                        int kh, int kw, int stride, void *stream);
int adapt_weights_destroy(adapt_weights *w);

/* Diagnostic, host only (no device call when cu > 0): how a product on a packed handle of this shape is spread over the
 * chip (Sec. IV: the matrix product is where the time goes, so which kernel runs it and in which launch shape is what a
 * profile has to be read against).  kind 0 linear (kh = kw = 1), 1 conv2d, 2 transposed conv2d with `stride`; storage as
 * adapt_lut_info reports it; rows = rows of the product (linear: M; convolution: N Ho Wo; transposed convolution: N Ho Wo
 * / stride^2, the rows of one phase), Wo = output width of one image row (linear: M; transposed: Wo / stride), sw =
 * horizontal stride; cu = compute units to plan for (<= 0: those of the current device).
 * *kernel: -1 whole-table kernel (lut_rows_kernel), 0 lut_lines_kernel, 1 lut_lines_fast_kernel, 2 the same on the
 * x-major copy, 3 lut_quad_kernel; *rows_per_workgroup; *ksplit = workgroups that share an output tile, each with a slice
 * of the inner dimension; *steps = table steps of the whole inner dimension (16 inner indices each for kernel 3, 8
 * otherwise); *workgroups = size of the launch.  Any output pointer may be NULL. */
int adapt_plan_packed(int kind, int bits, int storage, int Cout, int Cin, int kh, int kw, int stride, int rows, int Wo, int sw, int cu,
                      int *kernel, int *rows_per_workgroup, int *ksplit, int *steps, int *workgroups);

/* same results as adapt_approx_linear / adapt_approx_conv2d with the weights and table given at pack time */
int adapt_approx_linear_packed(const adapt_weights *w, const int8_t *a_dev, int32_t *acc_dev, int M, void *stream);
int adapt_approx_conv2d_packed(const adapt_weights *w, const int8_t *x_dev, int32_t *acc_dev, int N, int H, int W,
                               int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, void *stream);

/* same results as adapt_approx_conv_transpose2d (real pairs only: no term for a tap without an input pixel) */
int adapt_approx_conv_transpose2d_packed(const adapt_weights *w, const int8_t *x_dev, int32_t *acc_dev, int N, int H, int W,
                                         int pad, void *stream);

/* A grouped convolution as one call (Sec. III-B; depthwise: groups = Cin, the first half of the separable convolution,
 * eq. (1)).  The sums are rescaled as in adapt_conv2d_layer_f32 (s_out or s_out_vec_dev, bias, act) and written to y_dev
 * (fp32 [N][Cout][Ho][Wo]) and, when `next` != NULL (a prepared conv2d handle, e.g. the pointwise half), also as next's
 * quantised input copy as in adapt_conv2d_layer_chain_f32.  w_dev int8 [Cout][Cin/groups][kh][kw].
 *   Groups with fewer than 8 output channels: one kernel, x is quantised with s_x while it is staged; y_dev may be NULL
 *     when `next` is given.  Shapes whose input rows do not fit the kernel's staging buffer and two-pass tables return
 *     ADAPT_ERR_UNSUPPORTED (use the separate calls).
 *   Groups with 8 or more output channels (groups = 1 included): the quantiser, then the whole-table product kernel over
 *     a group dimension with the finishing pass in its epilogue (single-pass table, no tanh, no `next`) or in place
 *     afterwards; y_dev is required; the quantised input lives in a stream-ordered temporary. */
int adapt_conv2d_grouped_layer_f32(const adapt_lut *lut, const float *x_dev, const int8_t *w_dev, float *y_dev, int N,
                                   int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w,
                                   int pad_h, int pad_w, int dil_h, int dil_w, int groups, float s_x, float s_out,
                                   const float *s_out_vec_dev, const float *bias_dev, int act,
                                   const adapt_weights *next, float s_next, void *stream);

/* Chained convolution layers (Sec. III-A / IV: quantise -> table-lookup layer -> dequantise per layer; here the
 * re-quantisation for the NEXT layer happens in this layer's epilogue).  adapt_conv2d_chain_prepare fixes the place
 * and layout of `h`'s quantised, zero-padded input copy for one input geometry and zeroes it (borders and padded
 * channels stay zero afterwards); it may re-allocate the handle's workspace, so call it before recording a graph.
 * adapt_conv2d_layer_chain_f32 is adapt_conv2d_layer_f32 with two additions:
 *   x_dev == NULL: the input copy is already in the prepared workspace of `h` (written by the layer before);
 *   next != NULL : y is ALSO written into the prepared workspace of `next` as its input copy, quantised with
 *                  s_next exactly as adapt_quantize_f32 would quantise y_dev.  y_dev is written too, unless it is NULL:
 *                  a caller that wants nothing but next's copy may pass y_dev == NULL with next != NULL.  That works
 *                  where the product kernel, or the kernel that adds the sums of a layer whose inner dimension is
 *                  split over workgroups, finishes the sums and writes the copy; a layer whose sums are finished in
 *                  a separate pass over the output (two-pass tables; split layers whose output width or plane size is
 *                  no multiple of 4) returns ADAPT_ERR_UNSUPPORTED with next's copy untouched and needs the buffer.
 * `next` must have been prepared for N images of this layer's output size and have as many input channels as this
 * layer has output channels, and must be another handle than `w`; otherwise ADAPT_ERR_INVALID_ARGUMENT.  An ordinary call on a prepared handle with
 * another geometry ends its prepared state.  Results are identical to the unchained calls.
 * A handle remembers whether the call that last wrote its input copy applied ReLU (act = 1): all codes are then >= 0 and
 * the consuming call streams only the table lines such codes can select.  That is decided when the consuming call is
 * made; a recorded graph keeps the decision of the time of recording, so record producer and consumer together (or
 * record the consumer after a producer with the same `act` has run).  These calls change state of `w` and `next`: do
 * not run two chains over the same handles from two threads at once. */
int adapt_conv2d_chain_prepare(const adapt_weights *w, int N, int H, int W, int stride_h, int stride_w, int pad_h,
                               int pad_w, int dil_h, int dil_w, void *stream);
int adapt_conv2d_layer_chain_f32(const adapt_weights *w, const float *x_dev, float *y_dev, int N, int H, int W,
                                 int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, float s_x,
                                 float s_out, const float *s_out_vec_dev, const float *bias_dev,
                                 const float *residual_dev, int act, const adapt_weights *next, float s_next,
                                 void *stream);

/* ------------------------------------------------------------------------------------------------
 * Whole layers on packed weights with fp32 activations on both sides (Sec. III-A/III-B: a layer quantises its input,
 * multiplies through the table and rescales the sums):
 *     q = quantise(x, s_x, bits of the table)                 exactly as adapt_quantize_f32
 *     acc = table product of q with the packed weights        exactly as the *_packed entry points
 *     y = float(acc) * s_out, then + bias[c] if bias_dev      exactly as adapt_dequant_i32
 *     act 0: nothing; 1: y = y > 0 ? y : 0 (adapt_relu_f32); 2: adapt_tanh_f32
 * The quantiser runs inside the kernel that lays the activations out for the product, and (single-pass tables) the
 * rescaling inside the product kernel, so a layer is two launches instead of four or five and the int8 / int32
 * intermediates never reach memory.  y_dev has the shape of the int32 output of the corresponding *_packed call
 * and also serves as scratch for the sums where they cannot be rescaled in the product kernel.  s_out = s_x * s_w,
 * formed in fp32 by the caller; with per-channel weight ranges s_out_vec_dev [channels] holds s_x * s_w[c] instead
 * (then s_out is ignored; NULL otherwise); bias_dev [channels] or NULL.  The convolution also takes residual_dev,
 * an fp32 tensor of the output's shape (not aliasing y_dev) or NULL: y = y + residual (adapt_add_f32) after the bias
 * and before act -- the residual connection of a ResNet block without a pass of its own.
 * ---------------------------------------------------------------------------------------------- */
int adapt_linear_layer_f32(const adapt_weights *w, const float *x_dev, float *y_dev, int M, float s_x, float s_out,
                           const float *s_out_vec_dev, const float *bias_dev, int act, void *stream);
int adapt_conv2d_layer_f32(const adapt_weights *w, const float *x_dev, float *y_dev, int N, int H, int W, int stride_h,
                           int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, float s_x, float s_out,
                           const float *s_out_vec_dev, const float *bias_dev, const float *residual_dev, int act,
                           void *stream);
int adapt_conv_transpose2d_layer_f32(const adapt_weights *w, const float *x_dev, float *y_dev, int N, int H, int W, int pad,
                                     float s_x, float s_out, const float *s_out_vec_dev, const float *bias_dev, int act,
                                     void *stream);

/* ------------------------------------------------------------------------------------------------
 * fp32 operations between approximate layers.  Each element is produced by single IEEE fp32
 * operations in the stated order (no fused multiply-add unless stated), so that the integers the next
 * quantiser produces are reproducible.  In-place use (y_dev == x_dev) is allowed.
 * ---------------------------------------------------------------------------------------------- */

/* y = x > 0 ? x : 0 */
int adapt_relu_f32(const float *x_dev, float *y_dev, size_t n, void *stream);
/* y = a + b, optionally followed by the ReLU above (relu != 0): residual connection */
int adapt_add_f32(const float *a_dev, const float *b_dev, float *y_dev, size_t n, int relu, void *stream);
/* y[i] = (sequential row-major fp32 sum of x[i][0..HW-1]) * (1.0f / HW): global average pool */
int adapt_avgpool_hw_f32(const float *x_dev, float *y_dev, size_t NC, size_t HW, void *stream);
/* parameter-free residual shortcut: y[n][c][oy][ox] = x[n][c - (Cout-Cin)/2][2 oy][2 ox] or 0 outside;
 * y is [N][Cout][(H+1)/2][(W+1)/2] */
int adapt_shortcut_a_f32(const float *x_dev, float *y_dev, int N, int Cin, int H, int W, int Cout, void *stream);
/* y = tanh(x) computed as sign(x) (1 - e) / (1 + e), e = exp(-2|x|), with the library's written-out
 * exp (range reduction by ln 2 in two fused steps, degree-7 Horner polynomial with fused multiply-adds) */
int adapt_tanh_f32(const float *x_dev, float *y_dev, size_t n, void *stream);
/* y = 1 / (1 + exp(-x)) with the same exp */
int adapt_sigmoid_f32(const float *x_dev, float *y_dev, size_t n, void *stream);
/* LSTM memory cell (Sec. III-B "RNN Layer"), gate order i, f, g, o along the 4*Hs axis:
 *   pre = (float(acc_ih) * s_ih + float(acc_hh) * s_hh) + bias   (bias_dev NULL = 0)
 *   c = f * c + i * g  (two products, then one sum);  h = o * tanh(c)
 * acc_ih_dev, acc_hh_dev [B][4 Hs] int32; c_dev [B][Hs] updated in place; h_dev [B][Hs] written. */
int adapt_lstm_cell_f32(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh,
                        const float *bias_dev, float *c_dev, float *h_dev, int B, int Hs, void *stream);

/* The same cell, and in the same kernel the next step's operand: qh = quantise(h, s_h, bits) exactly as
 * adapt_quantize_f32 would (Sec. III-A); qh_dev [B][Hs] int8. */
int adapt_lstm_cell_q_f32(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh,
                          const float *bias_dev, float *c_dev, float *h_dev, int8_t *qh_dev, float s_h, int bits, int B,
                          int Hs, void *stream);

/* GRU memory cell (Sec. III-B "RNN Layer"), gate order r, z, n along the 3*Hs axis, every operation one rounded
 * fp32 operation in this order:
 *   gi = float(acc_ih) * s_ih + b_ih;  gh = float(acc_hh) * s_hh + b_hh      (a NULL bias adds nothing)
 *   r = sigmoid(gi_r + gh_r);  z = sigmoid(gi_z + gh_z);  n = tanh(gi_n + r * gh_n);  h' = (1 - z) * n + z * h
 * acc_ih_dev, acc_hh_dev [B][3 Hs] int32; b_ih_dev, b_hh_dev [3 Hs] or NULL; h_prev_dev, h_dev [B][Hs] (may be the
 * same buffer).  qh_dev [B][Hs] int8 or NULL: when given, also qh = quantise(h', s_h, bits) as adapt_quantize_f32. */
int adapt_gru_cell_f32(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh,
                       const float *b_ih_dev, const float *b_hh_dev, const float *h_prev_dev, float *h_dev,
                       int8_t *qh_dev, float s_h, int bits, int B, int Hs, void *stream);

/* Plain recurrent cell (Sec. III-B "RNN Layer"): h' = act((float(acc_ih) * s_ih + float(acc_hh) * s_hh) + bias),
 * act = tanh (relu == 0) or max(., 0) (relu != 0).  acc_ih_dev, acc_hh_dev, h_dev [B][Hs]; bias_dev [Hs] or NULL;
 * qh_dev as above. */
int adapt_rnn_cell_f32(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh,
                       const float *bias_dev, int relu, float *h_dev, int8_t *qh_dev, float s_h, int bits, int B, int Hs,
                       void *stream);

/* Chained transposed convolutions (the generator networks of Sec. V are stacks of them): as adapt_conv2d_chain_prepare /
 * adapt_conv2d_layer_chain_f32, for handles of adapt_weights_pack_conv_transpose2d.
 * adapt_conv_transpose2d_chain_prepare fixes the place and layout of h's input copy for inputs [N][Cin][H][W] and padding
 * `pad` and zeroes it; afterwards a layer whose `next` is h writes its output there, and h runs with x_dev == NULL.
 * Only geometries that take the phase form (filter sizes multiples of the stride, 2 pad a multiple of it, more than
 * one input pixel) can be prepared: ADAPT_ERR_UNSUPPORTED otherwise.
 * adapt_conv_transpose2d_layer_chain_f32: adapt_conv_transpose2d_layer_f32 with x_dev == NULL allowed (prepared handle)
 * and, when next != NULL (a prepared conv2d or transposed-conv2d handle whose input is this layer's output), the output
 * also written as next's quantised input copy with scale s_next.  y_dev may be NULL when next != NULL, under the same
 * condition as for adapt_conv2d_layer_chain_f32 (ADAPT_ERR_UNSUPPORTED otherwise).  Every geometry is accepted as a
 * producer. */
int adapt_conv_transpose2d_chain_prepare(const adapt_weights *h, int N, int H, int W, int pad, void *stream);
int adapt_conv_transpose2d_layer_chain_f32(const adapt_weights *h, const float *x_dev, float *y_dev, int N, int H, int W,
                                           int pad, float s_x, float s_out, const float *s_out_vec_dev,
                                           const float *bias_dev, int act, const adapt_weights *next, float s_next,
                                           void *stream);

/* One whole time step of the recurrent part of an LSTM layer in one kernel:
 *     acc_hh = table product of qh_dev [B][Hs] with the packed W_hh [4 Hs][Hs]   (adapt_approx_linear_packed)
 *     (c, h) = cell(acc_ih, acc_hh);  qh_next = quantise(h, s_h)                   (adapt_lstm_cell_q_f32)
 * with the same integers and floats as those two calls.  w_hh: handle of adapt_weights_pack_linear for W_hh.
 * acc_ih_dev [B][4 Hs]; c_dev [B][Hs] in place; h_dev [B][Hs]; qh_next_dev [B][Hs], must not alias qh_dev.
 * Covers even Hs and single-pass tables; otherwise ADAPT_ERR_UNSUPPORTED and the caller uses the two calls above. */
int adapt_lstm_step_f32(const adapt_weights *w_hh, const int8_t *qh_dev, const int32_t *acc_ih_dev, float s_ih, float s_hh,
                        float s_h, const float *bias_dev, float *c_dev, float *h_dev, int8_t *qh_next_dev, int B, int Hs,
                        void *stream);

/* One whole time step of the recurrent part of a GRU layer in one kernel:
 *     acc_hh = table product of qh_dev [B][Hs] with the packed W_hh [3 Hs][Hs]   (adapt_approx_linear_packed)
 *     h' = cell(acc_ih, acc_hh, h_prev);  qh_next = quantise(h', s_h)              (adapt_gru_cell_f32)
 * with the same integers and floats as those two calls.  w_hh: handle of adapt_weights_pack_linear for W_hh (rows in
 * gate order r, z, n).  acc_ih_dev [B][3 Hs]; b_ih_dev, b_hh_dev [3 Hs] or NULL; h_prev_dev, h_dev [B][Hs] (may be the
 * same buffer); qh_next_dev [B][Hs], must not alias qh_dev.
 * Covers even Hs and single-pass tables; otherwise ADAPT_ERR_UNSUPPORTED and the caller uses the two calls above. */
int adapt_gru_step_f32(const adapt_weights *w_hh, const int8_t *qh_dev, const int32_t *acc_ih_dev, float s_ih, float s_hh,
                       float s_h, const float *b_ih_dev, const float *b_hh_dev, const float *h_prev_dev, float *h_dev,
                       int8_t *qh_next_dev, int B, int Hs, void *stream);

/* One whole time step of a plain recurrent layer in one kernel: the table product of qh_dev [B][Hs] with the packed
 * W_hh [Hs][Hs], then adapt_rnn_cell_f32 (same integers and floats as those two calls).  acc_ih_dev, h_dev [B][Hs];
 * bias_dev [Hs] or NULL; relu != 0: max(., 0) instead of tanh; qh_next_dev [B][Hs], must not alias qh_dev.
 * Covers even Hs and single-pass tables; otherwise ADAPT_ERR_UNSUPPORTED and the caller uses the two calls. */
int adapt_rnn_step_f32(const adapt_weights *w_hh, const int8_t *qh_dev, const int32_t *acc_ih_dev, float s_ih, float s_hh,
                       float s_h, const float *bias_dev, int relu, float *h_dev, int8_t *qh_next_dev, int B, int Hs,
                       void *stream);

/* ------------------------------------------------------------------------------------------------
 * Operands wider than 8 bits and multipliers given as functions (Sec. III-C "Framework operation": a
 * table per multiplier or, for large bitwidths, the multiplier described as a function - both a 1-1
 * representation of the unit; Sec. V evaluates a 12-bit unit).  Operands are int16 in [-H, H-1],
 * H = 2^(bits-1); same index convention, same sums (int32 wrap-around), padded convolution taps meet
 * activation 0.  Out-of-range operands are reduced modulo 2^bits in the table form.
 * ---------------------------------------------------------------------------------------------- */

typedef struct adapt_lut16 adapt_lut16;

/* Device copy of a host table T[(a + H) * 2^bits + (w + H)] of int32 entries, 2 <= bits <= 12 (bits = 12:
 * 64 MiB, kept in device memory; the kernels gather from it).  Synchronous.  The handle owns its memory. */
int adapt_lut16_create(adapt_lut16 **out, int bits, const int32_t *table_host);
/* The table of a function-described multiplier, generated on the device (the table generator of Sec. III-C).
 * kind 0: exact product.  kind 1: both operands lose their `param` low bits (arithmetic shift), exact multiply,
 * product shifted back by 2 param.  kind 2: Mitchell's logarithmic multiplier on the magnitudes, sign restored
 * (param ignored but must be 0 <= param < bits). */
int adapt_lut16_create_from_func(adapt_lut16 **out, int kind, int param, int bits);
int adapt_lut16_destroy(adapt_lut16 *lut);
int adapt_lut16_bits(const adapt_lut16 *lut);

/* q = clamp(rint(x / scale), -Q, Q), Q = 2^(bits-1) - 1, 2 <= bits <= 16: the quantiser of Sec. III-A into int16 */
int adapt_quantize_i16_f32(const float *x_dev, int16_t *q_dev, size_t n, float scale, int bits, void *stream);

/* acc[m][n] = sum_k T[a[m][k]][w[n][k]]; a_dev [M][K], w_dev [N][K] int16, acc_dev [M][N] int32 */
int adapt_approx_linear_i16(const adapt_lut16 *lut, const int16_t *a_dev, const int16_t *w_dev, int32_t *acc_dev,
                            int M, int K, int N, void *stream);
/* 2-D convolution as adapt_approx_conv2d with groups = 1; x [N][Cin][H][W], w [Cout][Cin][kh][kw] int16 */
int adapt_approx_conv2d_i16(const adapt_lut16 *lut, const int16_t *x_dev, const int16_t *w_dev, int32_t *acc_dev,
                            int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w,
                            int pad_h, int pad_w, int dil_h, int dil_w, void *stream);
/* The same two layers with the multiplier (kind, param as above) evaluated as a function instead of read from a
 * table: no table memory, operands of 2 <= bits <= 16.  Identical results to the table form of the same multiplier. */
int adapt_approx_linear_func_i16(int kind, int param, int bits, const int16_t *a_dev, const int16_t *w_dev,
                                 int32_t *acc_dev, int M, int K, int N, void *stream);
int adapt_approx_conv2d_func_i16(int kind, int param, int bits, const int16_t *x_dev, const int16_t *w_dev,
                                 int32_t *acc_dev, int N, int Cin, int H, int W, int Cout, int kh, int kw,
                                 int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, void *stream);

/* Whole layers on operands of up to 16 bits (Sec. III-A quantiser, the products above, Sec. III-A rescaling), one call each:
 *     q   = quantise(x, s_x, bits)                      exactly as adapt_quantize_i16_f32 (stream-ordered temporary)
 *     acc = product of q with w_dev                     exactly as the *_i16 / *_func_i16 entry points above
 *     y   = float(acc) * s_out (or s_out_vec_dev[n]), + bias_dev[n] if given, then act (0 none, 1 ReLU, 2 tanh)
 * with the last step in the product kernel's epilogue (two kernels per call).  lut != NULL: table form, `bits` is the
 * table's and kind / param / bits are ignored; lut == NULL: the function form (kind, param, bits) as in
 * adapt_approx_linear_func_i16.  x_dev fp32 [M][K] / [N][Cin][H][W]; w_dev int16 codes [N][K] / [Cout][Cin][kh][kw];
 * y_dev fp32 [M][N] / [N][Cout][Ho][Wo]. */
int adapt_linear_layer_i16_f32(const adapt_lut16 *lut, int kind, int param, int bits, const float *x_dev, const int16_t *w_dev,
                               float *y_dev, int M, int K, int N, float s_x, float s_out, const float *s_out_vec_dev,
                               const float *bias_dev, int act, void *stream);
int adapt_conv2d_layer_i16_f32(const adapt_lut16 *lut, int kind, int param, int bits, const float *x_dev, const int16_t *w_dev,
                               float *y_dev, int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w,
                               int pad_h, int pad_w, int dil_h, int dil_w, float s_x, float s_out, const float *s_out_vec_dev,
                               const float *bias_dev, int act, void *stream);

/* ------------------------------------------------------------------ retraining: backward pass */

/* Backward pass of an approximate linear layer y = s_x s_w (table product of q(x), q(w)) + b under the straight-through
 * estimator (Sec. III-A, "Retraining": training continues through fake-quantisation modules; the estimator stands in
 * for the derivative of the quantiser, the forward pass goes through the multiplier table).  The quantiser passes a
 * gradient where its clamp did not act, |rint(x / s)| <= Q = 2^(bits-1) - 1, decided in fp32 exactly as
 * adapt_quantize_f32 decides; the table is differentiated as the exact product it approximates:
 *     dx[m][k] = inside(x[m][k], s_x) * sum_n dy[m][n] * (s_w * q(w)[n][k])
 *     dw[n][k] = inside(w[n][k], s_w) * sum_m dy[m][n] * (s_x * q(x)[m][k])
 *     db[n]    = sum_m dy[m][n]
 * dy_dev [M][N], x_dev [M][K], w_dev [N][K]: fp32 device pointers, row-major, dense, the un-quantised operands of the
 * forward pass; s_x, s_w: the scales the forward pass quantised them with; 2 <= bits <= 16.  dx_dev [M][K], dw_dev
 * [N][K], db_dev [N]: device pointers, fully overwritten; any of them may be NULL (not computed); none may alias an
 * input.  Products and sums are fp32 (matrix instructions for dx / dw, a fixed order for db); NaN inputs get no
 * gradient.  Asynchronous on `stream`, no allocation.  Errors: ADAPT_ERR_INVALID_ARGUMENT (NULL / misaligned pointer,
 * negative size, bits, scales), ADAPT_ERR_UNSUPPORTED (M or N above 65535 * 64), ADAPT_ERR_HIP. */
int adapt_ste_linear_backward_f32(const float *dy_dev, const float *x_dev, const float *w_dev, int M, int K, int N, float s_x,
                                  float s_w, int bits, float *dx_dev, float *dw_dev, float *db_dev, void *stream);

/* The same backward pass for an approximate 2-D convolution with groups = 1 (Sec. III-A "Retraining"; Sec. III-B: the
 * convolution as a matrix product over the unfolded input).  With x^ = s_x q(x), w^ = s_w q(w) and zero outside the image:
 *     dw[o][c][ky][kx] = inside(w) * sum_{n,oy,ox} dy[n][o][oy][ox] * x^[n][c][oy s - p + ky d][ox s - p + kx d]
 *     dx[n][c][iy][ix] = inside(x) * sum over the (o, ky, kx, oy, ox) whose tap lands on (iy, ix) of dy * w^
 *     db[o]            = sum_{n,oy,ox} dy[n][o][oy][ox]
 * dy_dev [N][Cout][Ho][Wo], x_dev [N][Cin][H][W], w_dev [Cout][Cin][kh][kw]: fp32 device pointers, dense; geometry as in
 * adapt_approx_conv2d.  dx_dev, dw_dev, db_dev: shapes of x, w and [Cout]; fully overwritten; NULL = not computed; none
 * may alias an input.  workspace_dev: device memory of at least the number of bytes that
 * adapt_ste_conv2d_backward_workspace reports for the same arguments (want_dx / want_dw: whether dx_dev / dw_dev are
 * given), aligned to 256 bytes, owned by the caller, contents undefined afterwards; it holds dy as rows, the gradient of
 * the unfolded input and partial sums (the unfolded input itself is read from x_dev, never written).  fp32 sums (matrix instructions for the products, a fixed tap order for dx).  Asynchronous on `stream`, no
 * allocation.  Errors: ADAPT_ERR_INVALID_ARGUMENT (pointers, geometry, bits, scales, workspace too small or misaligned),
 * ADAPT_ERR_UNSUPPORTED (N Ho Wo above 65535 * 64), ADAPT_ERR_HIP. */
int adapt_ste_conv2d_backward_workspace(int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w, int pad_h,
                                        int pad_w, int dil_h, int dil_w, int want_dx, int want_dw, size_t *bytes);
int adapt_ste_conv2d_backward_f32(const float *dy_dev, const float *x_dev, const float *w_dev, int N, int Cin, int H, int W, int Cout,
                                  int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, float s_x,
                                  float s_w, int bits, float *dx_dev, float *dw_dev, float *db_dev, void *workspace_dev,
                                  size_t workspace_bytes, void *stream);

/* Gradient through the ReLU that the layer calls fuse (act = 1), for the backward pass of Sec. III-A's retraining:
 * dx[i] = y[i] > 0 ? dy[i] : 0, y being the layer's output.  n floats each on the device; dx_dev may be dy_dev (in place).
 * Asynchronous on `stream`.  Errors: ADAPT_ERR_INVALID_ARGUMENT (NULL pointer), ADAPT_ERR_HIP. */
int adapt_relu_backward_f32(const float *dy_dev, const float *y_dev, float *dx_dev, size_t n, void *stream);

/* One plain stochastic-gradient step, the optimiser the paper retrains with (Sec. V-A, "Quantization and retraining":
 * SGD, learning rate 1e-4): w[i] <- w[i] - lr * g[i] in fp32, the product and the difference rounded separately.
 * w_dev, g_dev: n floats each on the device, distinct; in place on w_dev.  Asynchronous on `stream`.
 * Errors: ADAPT_ERR_INVALID_ARGUMENT (NULL pointer, w_dev == g_dev), ADAPT_ERR_HIP. */
int adapt_sgd_step_f32(float *w_dev, const float *g_dev, size_t n, float lr, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ADAPT_MI355_H */
