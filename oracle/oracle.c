/*
 * CPU oracle for the approximate-multiplier hot path (AdaPT, arXiv 2203.04071).
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing here is part of the product path: only the
 * test-suite, the smoke check and the benchmark's cpu_baseline leg may load this
 * file.  It shares no source, header, table or helper with the HIP library.
 *
 * Everything is the plain definition written out: nested loops, one table read
 * per multiply-accumulate, 32-bit wrap-around accumulation, one IEEE fp32
 * operation per stated step (compile with -ffp-contract=off, no fast-math).
 * The only parallelism is an OpenMP `parallel for` over the batch / output rows,
 * which mirrors the paper's thread parallelism over batches (Sec. IV-A) and does
 * not change any result.
 *
 * Conventions (Sec. III-A, III-B, III-C of the paper; readings where it is
 * silent are listed in the design notes of the repository):
 *   - b = bits, H = 2^(b-1), Q = H-1.  Operands are signed integers in [-H, H-1]
 *     stored as int8.
 *   - The multiplier table T has 2^b x 2^b int32 entries; the entry for
 *     (activation a, weight w) is T[(a+H)*2^b + (w+H)]            (Sec. III-C).
 *   - Every inner product term of a matrix multiply / convolution is one table
 *     entry (Sec. IV): acc = sum_k T[a_k][w_k].
 *
 * Pinned by tests/test_oracle_*.py (hand-computed tiny cases, exact-product
 * table == integer GEMM / library convolution, linearity in the table,
 * projections, constant tables, quantiser closed forms).  The paper prints no
 * worked numeric example, so no pin comes from printed values.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_BAD_ARG (-1)
#define ORC_NO_MEM (-5)

static int in_range(const int8_t *p, size_t n, int bits) {
    const int h = 1 << (bits - 1);
    for (size_t i = 0; i < n; ++i)
        if (p[i] < -h || p[i] > h - 1) return 0;
    return 1;
}

/* table entry for signed operands (a, w)  -- Sec. III-C (one table per multiplier) */
static inline uint32_t lut_at(const int32_t *T, int bits, int a, int w) {
    const int n = 1 << bits, h = n >> 1;
    return (uint32_t)T[(size_t)(a + h) * (size_t)n + (size_t)(w + h)];
}

/* ---------------------------------------------------------------------------
 * Linear layer y = x A^T (Sec. III-B "Linear Layer") with every product taken
 * from the table (Sec. IV):  acc[m][n] = sum_k T[A[m][k]][W[n][k]].
 * A is [M][K], W is [N][K], acc is [M][N]; int32 wrap-around accumulation.
 * ------------------------------------------------------------------------- */
int orc_approx_linear(const int32_t *T, int bits, const int8_t *A, const int8_t *W, int32_t *acc,
                      long M, long K, long N, int threads) {
    if (!T || !A || !W || !acc || bits < 2 || bits > 8 || M < 0 || K < 0 || N < 0) return ORC_BAD_ARG;
    if (!in_range(A, (size_t)M * K, bits) || !in_range(W, (size_t)N * K, bits)) return ORC_BAD_ARG;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (long m = 0; m < M; ++m) {
        for (long n = 0; n < N; ++n) {
            uint32_t s = 0;
            for (long k = 0; k < K; ++k) s += lut_at(T, bits, A[m * K + k], W[n * K + k]);
            acc[m * N + n] = (int32_t)s;
        }
    }
    return ORC_OK;
}

static long out_dim(long in, long k, long s, long p, long d) { return (in + 2 * p - d * (k - 1) - 1) / s + 1; }

/* ---------------------------------------------------------------------------
 * 2-D convolution (Sec. III-B "Convolution Layer"), direct form.
 * x [N][Cin][H][W], w [Cout][Cin/g][kh][kw], acc [N][Cout][Ho][Wo].
 * A tap that falls outside the image contributes the table entry of a zero
 * activation: the convolution is defined as the product of the expanded input
 * matrix with the filter matrix, and pad elements are entries of that matrix.
 * ------------------------------------------------------------------------- */
int orc_approx_conv2d_direct(const int32_t *T, int bits, const int8_t *x, const int8_t *w, int32_t *acc,
                             long N, long Cin, long H, long W, long Cout, long kh, long kw,
                             long sh, long sw, long ph, long pw, long dh, long dw, long groups,
                             int threads) {
    if (!T || !x || !w || !acc || bits < 2 || bits > 8) return ORC_BAD_ARG;
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || kh < 1 || kw < 1 || sh < 1 || sw < 1 ||
        ph < 0 || pw < 0 || dh < 1 || dw < 1 || groups < 1 || Cin % groups || Cout % groups)
        return ORC_BAD_ARG;
    const long Ho = out_dim(H, kh, sh, ph, dh), Wo = out_dim(W, kw, sw, pw, dw);
    if (Ho < 1 || Wo < 1) return ORC_BAD_ARG;
    const long cg = Cin / groups, og = Cout / groups;
    if (!in_range(x, (size_t)N * Cin * H * W, bits) || !in_range(w, (size_t)Cout * cg * kh * kw, bits))
        return ORC_BAD_ARG;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (long n = 0; n < N; ++n)
        for (long co = 0; co < Cout; ++co) {
            const long g = co / og;
            for (long oy = 0; oy < Ho; ++oy)
                for (long ox = 0; ox < Wo; ++ox) {
                    uint32_t s = 0;
                    for (long c = 0; c < cg; ++c)
                        for (long ky = 0; ky < kh; ++ky)
                            for (long kx = 0; kx < kw; ++kx) {
                                const long iy = oy * sh - ph + ky * dh, ix = ox * sw - pw + kx * dw;
                                int a = 0;
                                if (iy >= 0 && iy < H && ix >= 0 && ix < W)
                                    a = x[((n * Cin + g * cg + c) * H + iy) * W + ix];
                                s += lut_at(T, bits, a, w[((co * cg + c) * kh + ky) * kw + kx]);
                            }
                    acc[((n * Cout + co) * Ho + oy) * Wo + ox] = (int32_t)s;
                }
        }
    return ORC_OK;
}

/* Expanded input matrix of one channel group: col[m][k], m = (n, oy, ox),
 * k = (c, ky, kx), zero where the tap is outside the image. */
int orc_im2col_i8(const int8_t *x, int8_t *col, long N, long Cin, long H, long W, long c0, long cg,
                  long kh, long kw, long sh, long sw, long ph, long pw, long dh, long dw) {
    if (!x || !col) return ORC_BAD_ARG;
    const long Ho = out_dim(H, kh, sh, ph, dh), Wo = out_dim(W, kw, sw, pw, dw);
    const long K = cg * kh * kw;
    for (long n = 0; n < N; ++n)
        for (long oy = 0; oy < Ho; ++oy)
            for (long ox = 0; ox < Wo; ++ox) {
                int8_t *row = col + ((n * Ho + oy) * Wo + ox) * K;
                for (long c = 0; c < cg; ++c)
                    for (long ky = 0; ky < kh; ++ky)
                        for (long kx = 0; kx < kw; ++kx) {
                            const long iy = oy * sh - ph + ky * dh, ix = ox * sw - pw + kx * dw;
                            int8_t a = 0;
                            if (iy >= 0 && iy < H && ix >= 0 && ix < W)
                                a = x[((n * Cin + c0 + c) * H + iy) * W + ix];
                            row[(c * kh + ky) * kw + kx] = a;
                        }
            }
    return ORC_OK;
}

/* Same convolution as the product of the two expanded matrices (Sec. III-B):
 * (expanded input [M][K]) x (filters as a matrix [Cout/g][K]) per group. */
int orc_approx_conv2d_im2col(const int32_t *T, int bits, const int8_t *x, const int8_t *w, int32_t *acc,
                             long N, long Cin, long H, long W, long Cout, long kh, long kw,
                             long sh, long sw, long ph, long pw, long dh, long dw, long groups,
                             int threads) {
    if (!T || !x || !w || !acc || groups < 1 || Cin % groups || Cout % groups) return ORC_BAD_ARG;
    const long Ho = out_dim(H, kh, sh, ph, dh), Wo = out_dim(W, kw, sw, pw, dw);
    if (Ho < 1 || Wo < 1) return ORC_BAD_ARG;
    const long cg = Cin / groups, og = Cout / groups, K = cg * kh * kw, M = N * Ho * Wo;
    int8_t *col = (int8_t *)malloc((size_t)(M > 0 ? M : 1) * K);
    int32_t *tmp = (int32_t *)malloc(sizeof(int32_t) * (size_t)(M > 0 ? M : 1) * og);
    if (!col || !tmp) { free(col); free(tmp); return ORC_NO_MEM; }
    int rc = ORC_OK;
    for (long g = 0; g < groups && rc == ORC_OK; ++g) {
        rc = orc_im2col_i8(x, col, N, Cin, H, W, g * cg, cg, kh, kw, sh, sw, ph, pw, dh, dw);
        if (rc == ORC_OK) rc = orc_approx_linear(T, bits, col, w + g * og * K, tmp, M, K, og, threads);
        if (rc != ORC_OK) break;
        for (long n = 0; n < N; ++n)
            for (long o = 0; o < og; ++o)
                for (long p = 0; p < Ho * Wo; ++p)
                    acc[(n * Cout + g * og + o) * Ho * Wo + p] = tmp[(n * Ho * Wo + p) * og + o];
    }
    free(col);
    free(tmp);
    return rc;
}

/* ---------------------------------------------------------------------------
 * Transposed 2-D convolution (the generator-network layer of the GAN family,
 * Sec. V Table I), the usual definition: input pixel (iy, ix) meets filter tap
 * (ky, kx) at output (iy*s - p + ky, ix*s - p + kx).  x [N][Cin][H][W],
 * w [Cin][Cout][kh][kw], acc [N][Cout][Ho][Wo], Ho = (H-1)s - 2p + kh.
 * Only real input/weight pairs are multiplied; the implied zeros between input
 * pixels never enter the multiplier.
 * ------------------------------------------------------------------------- */
int orc_approx_conv_transpose2d(const int32_t *T, int bits, const int8_t *x, const int8_t *w, int32_t *acc,
                                long N, long Cin, long H, long W, long Cout, long kh, long kw,
                                long stride, long pad, int threads) {
    if (!T || !x || !w || !acc || bits < 2 || bits > 8) return ORC_BAD_ARG;
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0)
        return ORC_BAD_ARG;
    const long Ho = (H - 1) * stride - 2 * pad + kh, Wo = (W - 1) * stride - 2 * pad + kw;
    if (Ho < 1 || Wo < 1) return ORC_BAD_ARG;
    if (!in_range(x, (size_t)N * Cin * H * W, bits) || !in_range(w, (size_t)Cin * Cout * kh * kw, bits))
        return ORC_BAD_ARG;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (long n = 0; n < N; ++n) {
        uint32_t *out = (uint32_t *)(acc + n * Cout * Ho * Wo);
        memset(out, 0, sizeof(uint32_t) * (size_t)(Cout * Ho * Wo));
        for (long ci = 0; ci < Cin; ++ci)
            for (long iy = 0; iy < H; ++iy)
                for (long ix = 0; ix < W; ++ix) {
                    const int a = x[((n * Cin + ci) * H + iy) * W + ix];
                    for (long co = 0; co < Cout; ++co)
                        for (long ky = 0; ky < kh; ++ky)
                            for (long kx = 0; kx < kw; ++kx) {
                                const long oy = iy * stride - pad + ky, ox = ix * stride - pad + kx;
                                if (oy < 0 || oy >= Ho || ox < 0 || ox >= Wo) continue;
                                out[(co * Ho + oy) * Wo + ox] +=
                                    lut_at(T, bits, a, w[((ci * Cout + co) * kh + ky) * kw + kx]);
                            }
                }
    }
    return ORC_OK;
}

/* ---------------------------------------------------------------------------
 * Quantiser (Sec. III-A): affine map real = scale * q with zero point 0.
 * ------------------------------------------------------------------------- */

/* largest |x| of a tensor; NaNs are skipped (the "max absolute number" scale) */
float orc_absmax_f32(const float *x, size_t n) {
    float m = 0.0f;
    for (size_t i = 0; i < n; ++i) {
        const float a = fabsf(x[i]);
        if (a > m) m = a;
    }
    return m;
}

/* scale that maps amax onto the largest quantised magnitude Q = 2^(b-1) - 1 */
float orc_scale_from_amax(float amax, int bits) {
    const float q = (float)((1 << (bits - 1)) - 1);
    if (!(amax > 0.0f)) return 1.0f;
    return amax / q;
}

/* q = clamp(round_half_even(x / scale), -Q, Q); NaN -> 0 */
int orc_quantize_f32(const float *x, int8_t *q, size_t n, float scale, int bits) {
    if (!x || !q || bits < 2 || bits > 8 || !(scale > 0.0f)) return ORC_BAD_ARG;
    const float Q = (float)((1 << (bits - 1)) - 1);
    for (size_t i = 0; i < n; ++i) {
        float r = rintf(x[i] / scale);
        if (r != r) r = 0.0f;
        if (r > Q) r = Q;
        if (r < -Q) r = -Q;
        q[i] = (int8_t)r;
    }
    return ORC_OK;
}

/* y = float(acc) * scale (+ bias[c]); element (o, c, i) at ((o*channels)+c)*inner+i.
 * Two separately rounded fp32 operations (Sec. III-A real = A*q; Sec. III-B "+ b"). */
int orc_dequant_i32(const int32_t *acc, float *y, size_t outer, size_t channels, size_t inner, float scale,
                    const float *bias) {
    if (!acc || !y) return ORC_BAD_ARG;
    for (size_t o = 0; o < outer; ++o)
        for (size_t c = 0; c < channels; ++c)
            for (size_t i = 0; i < inner; ++i) {
                const size_t idx = (o * channels + c) * inner + i;
                float v = (float)acc[idx] * scale;
                if (bias) v = v + bias[c];
                y[idx] = v;
            }
    return ORC_OK;
}

/* ---------------------------------------------------------------------------
 * The quantiser as the paper uses it (Sec. III-A "Parameter calibration"): weight ranges per output channel,
 * activation ranges per tensor from a histogram calibrator at a 99.9 % percentile, instead of the plain maximum.
 * The paper names the method but not the histogram; the reading taken here:
 *   bins equal-width bins over [0, amax], width = amax / bins (one fp32 division);
 *   bin(v) = min(bins - 1, (long) trunc(|v| / width)) (one fp32 division); NaN is not counted;
 *   calib_max = upper edge of the first bin at which the cumulative count reaches ceil(num / den * total),
 *             = (float)(k + 1) * width (one fp32 multiplication);  then scale = calib_max / Q as before, and
 *   the quantiser's clamp saturates what lies beyond calib_max.
 * ------------------------------------------------------------------------- */

/* amax[r] = max |x[r][c]| over the cols of row r (weights [Cout][Cin*kh*kw]: one row per output channel) */
int orc_absmax_rows_f32(const float *x, size_t rows, size_t cols, float *amax) {
    if ((!x && rows && cols) || (!amax && rows)) return ORC_BAD_ARG;
    for (size_t r = 0; r < rows; ++r) {
        float m = 0.0f;
        for (size_t c = 0; c < cols; ++c) {
            const float a = fabsf(x[r * cols + c]);
            if (a > m) m = a;
        }
        amax[r] = m;
    }
    return ORC_OK;
}

/* q[r][c] = clamp(round_half_even(x[r][c] / scale[r]), -Q, Q): the quantiser above with one scale per row */
int orc_quantize_rows_f32(const float *x, int8_t *q, size_t rows, size_t cols, const float *scale, int bits) {
    if (!x || !q || !scale || bits < 2 || bits > 8) return ORC_BAD_ARG;
    const float Q = (float)((1 << (bits - 1)) - 1);
    for (size_t r = 0; r < rows; ++r) {
        if (!(scale[r] > 0.0f)) return ORC_BAD_ARG;
        for (size_t c = 0; c < cols; ++c) {
            float v = rintf(x[r * cols + c] / scale[r]);
            if (v != v) v = 0.0f;
            if (v > Q) v = Q;
            if (v < -Q) v = -Q;
            q[r * cols + c] = (int8_t)v;
        }
    }
    return ORC_OK;
}

/* y = float(acc) * scale[c] (+ bias[c]): the dequantiser with one scale per output channel (= s_x * s_w[c]) */
int orc_dequant_i32_per_channel(const int32_t *acc, float *y, size_t outer, size_t channels, size_t inner,
                                const float *scale, const float *bias) {
    if (!acc || !y || !scale) return ORC_BAD_ARG;
    for (size_t o = 0; o < outer; ++o)
        for (size_t c = 0; c < channels; ++c)
            for (size_t i = 0; i < inner; ++i) {
                const size_t idx = (o * channels + c) * inner + i;
                float v = (float)acc[idx] * scale[c];
                if (bias) v = v + bias[c];
                y[idx] = v;
            }
    return ORC_OK;
}

/* counts[bin(x_i)] += 1 for every i (counts is accumulated into, so several batches can share it) */
int orc_histogram_abs_f32(const float *x, size_t n, float amax, int bins, uint32_t *counts) {
    if ((!x && n) || !counts || bins < 1 || !(amax > 0.0f)) return ORC_BAD_ARG;
    const float width = amax / (float)bins;
    for (size_t i = 0; i < n; ++i) {
        const float a = fabsf(x[i]);
        if (a != a) continue;
        const float t = a / width;
        long b = t >= (float)bins ? (long)bins - 1 : (long)t;
        if (b > bins - 1) b = bins - 1;
        counts[b] += 1u;
    }
    return ORC_OK;
}

/* calib_max for the fraction num / den of the counted values (e.g. 999 / 1000) */
int orc_percentile_from_histogram(const uint32_t *counts, int bins, float amax, unsigned long long num,
                                  unsigned long long den, float *calib_max) {
    if (!counts || !calib_max || bins < 1 || !(amax > 0.0f) || den == 0 || num > den) return ORC_BAD_ARG;
    unsigned long long total = 0;
    for (int b = 0; b < bins; ++b) total += counts[b];
    const unsigned long long target = (total * num + den - 1) / den;     /* ceil(total * num / den) */
    const float width = amax / (float)bins;
    unsigned long long cum = 0;
    int k = bins - 1;
    for (int b = 0; b < bins; ++b) {
        cum += counts[b];
        if (cum >= target) { k = b; break; }
    }
    *calib_max = (float)(k + 1) * width;
    return ORC_OK;
}

/* calib_max by least squared quantisation error (Sec. III-A names MSE as an alternative calibrator without defining it;
 * this is the reading of the design notes): every bin edge t_k = (k + 1) * width is a candidate range; with the scale
 * s = t_k / Q (fp32, as the quantiser would use it) a value at the centre c_j = (j + 0.5) * width of bin j is
 * reproduced as min(Q, rint(c_j / s)) * s; the candidate's error is sum_j counts[j] * (c_j - that)^2, all in fp64, j
 * ascending; the first candidate with the smallest error wins. */
int orc_mse_from_histogram(const uint32_t *counts, int bins, float amax, int bits, float *calib_max) {
    if (!counts || !calib_max || bins < 1 || !(amax > 0.0f) || bits < 2 || bits > 16) return ORC_BAD_ARG;
    const float width = amax / (float)bins;
    const float Qf = (float)((1 << (bits - 1)) - 1);
    const double Q = (double)Qf;
    double best = 0.0;
    int best_k = -1;
    for (int k = 0; k < bins; ++k) {
        const float t = (float)(k + 1) * width;
        const double s = (double)(t / Qf);
        double err = 0.0;
        for (int j = 0; j < bins; ++j) {
            if (!counts[j]) continue;
            const double c = ((double)j + 0.5) * (double)width;
            double q = rint(c / s);
            if (q > Q) q = Q;
            const double e = c - q * s;
            err = err + (double)counts[j] * (e * e);
        }
        if (best_k < 0 || err < best) { best = err; best_k = k; }
    }
    *calib_max = (float)(best_k + 1) * width;
    return ORC_OK;
}

/* calib_max by smallest information loss ("entropy" calibrator: Sec. III-A names it as a third alternative without
 * defining it; the definition below is this build's reading of the published idea - keep the range whose quantised
 * histogram diverges least, in the Kullback-Leibler sense, from the histogram it stands for).
 * L = 2^(bits-1) magnitude levels.  A candidate keeps the first k bins, k = L .. bins (k = bins alone when bins < L):
 *   reference  p_j = counts[j] for j < k - 1,  p_{k-1} = counts[k-1] + everything beyond (saturated values land there);
 *   quantised  the k kept bins WITHOUT that outlier mass are merged into L groups, group g = bins [g k / L, (g+1) k / L)
 *              (integer divisions); a bin with counts[j] > 0 gets q_j = (sum of its group) / (non-empty bins of its group),
 *              an empty bin q_j = 0;
 *   loss       KL_k = sum over j < k with p_j > 0, ascending, of (p_j / P) log((p_j / P) / (q_j / Q)),  P = sum p, Q = sum q;
 *              +inf when some p_j > 0 meets q_j = 0 (outliers pushed into an empty last bin).
 * fp64 throughout, every operation rounded on its own.  The first k with the smallest loss wins: calib_max = k * width.
 * kl (optional): KL_k for k = 1 .. bins at kl[k - 1] (+inf for k that are no candidates). */
int orc_entropy_from_histogram(const uint32_t *counts, int bins, float amax, int bits, float *calib_max, double *kl) {
    if (!counts || !calib_max || bins < 1 || !(amax > 0.0f) || bits < 2 || bits > 16) return ORC_BAD_ARG;
    const float width = amax / (float)bins;
    const long L = 1L << (bits - 1);
    unsigned long long total = 0;
    for (int j = 0; j < bins; ++j) total += counts[j];
    if (kl) for (int k = 0; k < bins; ++k) kl[k] = INFINITY;
    if (total == 0) { *calib_max = (float)bins * width; return ORC_OK; }
    const double P = (double)total;
    const int k_first = L < bins ? (int)L : bins;
    double best = 0.0;
    int best_k = -1;
    unsigned long long kept = 0;                 /* counts[0 .. k-1] */
    for (int j = 0; j < k_first - 1; ++j) kept += counts[j];
    for (int k = k_first; k <= bins; ++k) {
        kept += counts[k - 1];
        const unsigned long long outliers = total - kept;
        const long groups = L < k ? L : k;       /* (bins < L: one bin per group) */
        double Q = 0.0;                          /* sum of q over the kept bins = kept, formed the way q is formed */
        for (long g = 0; g < groups; ++g) {
            const long lo = g * k / groups, hi = (g + 1) * k / groups;
            unsigned long long sg = 0; long zg = 0;
            for (long j = lo; j < hi; ++j) { sg += counts[j]; zg += counts[j] > 0; }
            if (zg) Q = Q + (double)zg * ((double)sg / (double)zg);
        }
        double loss = 0.0;
        for (long g = 0; g < groups; ++g) {
            const long lo = g * k / groups, hi = (g + 1) * k / groups;
            unsigned long long sg = 0; long zg = 0;
            for (long j = lo; j < hi; ++j) { sg += counts[j]; zg += counts[j] > 0; }
            for (long j = lo; j < hi; ++j) {
                const unsigned long long pj = (unsigned long long)counts[j] + (j == k - 1 ? outliers : 0ULL);
                if (!pj) continue;
                if (!counts[j]) { loss = INFINITY; continue; }
                const double pn = (double)pj / P, qn = ((double)sg / (double)zg) / Q;
                loss = loss + pn * log(pn / qn);
            }
        }
        if (kl) kl[k - 1] = loss;
        if (best_k < 0 || loss < best) { best = loss; best_k = k; }
    }
    *calib_max = (float)best_k * width;
    return ORC_OK;
}

/* ---------------------------------------------------------------------------
 * fp32 glue between approximate layers.  Each is one IEEE operation per element
 * in the stated order, so that the integers produced by the next quantiser are
 * reproducible.
 * ------------------------------------------------------------------------- */
void orc_relu_f32(const float *x, float *y, size_t n) {
    for (size_t i = 0; i < n; ++i) y[i] = x[i] > 0.0f ? x[i] : 0.0f;
}

void orc_add_f32(const float *a, const float *b, float *y, size_t n) {
    for (size_t i = 0; i < n; ++i) y[i] = a[i] + b[i];
}

/* mean over (h, w): sequential row-major fp32 sum, then one multiply by 1/(H*W) */
void orc_avgpool_hw_f32(const float *x, float *y, size_t NC, size_t HW) {
    const float inv = 1.0f / (float)HW;
    for (size_t i = 0; i < NC; ++i) {
        float s = 0.0f;
        for (size_t j = 0; j < HW; ++j) s = s + x[i * HW + j];
        y[i] = s * inv;
    }
}

/* parameter-free residual shortcut: keep every second pixel, pad channels with
 * zeros, (Cout - Cin)/2 on each side */
void orc_shortcut_a_f32(const float *x, float *y, long N, long Cin, long H, long W, long Cout) {
    const long Ho = (H + 1) / 2, Wo = (W + 1) / 2, padc = (Cout - Cin) / 2;
    for (long n = 0; n < N; ++n)
        for (long c = 0; c < Cout; ++c)
            for (long oy = 0; oy < Ho; ++oy)
                for (long ox = 0; ox < Wo; ++ox) {
                    const long ci = c - padc;
                    float v = 0.0f;
                    if (ci >= 0 && ci < Cin) v = x[((n * Cin + ci) * H + 2 * oy) * W + 2 * ox];
                    y[((n * Cout + c) * Ho + oy) * Wo + ox] = v;
                }
}

/* exp(x) by a written-out algorithm (no libm), so that a device implementation
 * of the same steps gives the same bits:  clamp to [-87, 88];
 * n = rint(x*log2 e);  r = x - n*ln2 (two fused steps, hi/lo split);
 * degree-7 Taylor polynomial in Horner form with fused multiply-adds; scale by 2^n. */
float orc_exp_f32(float x) {
    const float LOG2E = 0x1.715476p+0f, LN2_HI = 0x1.62e400p-1f, LN2_LO = 0x1.7f7d1cp-20f;
    if (x != x) return x;
    if (x < -87.0f) x = -87.0f;
    if (x > 88.0f) x = 88.0f;
    const float n = rintf(x * LOG2E);
    float r = fmaf(n, -LN2_HI, x);
    r = fmaf(n, -LN2_LO, r);
    float p = 0x1.a01a02p-13f;          /* 1/5040 */
    p = fmaf(p, r, 0x1.6c16c2p-10f);    /* 1/720  */
    p = fmaf(p, r, 0x1.111112p-7f);     /* 1/120  */
    p = fmaf(p, r, 0x1.555556p-5f);     /* 1/24   */
    p = fmaf(p, r, 0x1.555556p-3f);     /* 1/6    */
    p = fmaf(p, r, 0.5f);
    p = fmaf(p, r, 1.0f);
    p = fmaf(p, r, 1.0f);
    return ldexpf(p, (int)n);
}

float orc_sigmoid_f32(float x) { return 1.0f / (1.0f + orc_exp_f32(-x)); }

float orc_tanh_f32(float x) {
    const float ax = fabsf(x);
    const float e = orc_exp_f32(-2.0f * ax);
    const float t = (1.0f - e) / (1.0f + e);
    return x < 0.0f ? -t : t;
}

void orc_tanh_vec_f32(const float *x, float *y, size_t n) {
    for (size_t i = 0; i < n; ++i) y[i] = orc_tanh_f32(x[i]);
}
void orc_sigmoid_vec_f32(const float *x, float *y, size_t n) {
    for (size_t i = 0; i < n; ++i) y[i] = orc_sigmoid_f32(x[i]);
}
void orc_exp_vec_f32(const float *x, float *y, size_t n) {
    for (size_t i = 0; i < n; ++i) y[i] = orc_exp_f32(x[i]);
}

/* LSTM memory cell (Sec. III-B "RNN Layer"), gate order i, f, g, o:
 *   pre = (float(acc_ih)*s_ih + float(acc_hh)*s_hh) + bias
 *   c' = f*c + i*g (two products, one sum);  h' = o * tanh(c')
 * acc_ih, acc_hh: [B][4*Hs];  c: [B][Hs] updated in place;  h: [B][Hs] written. */
void orc_lstm_cell_f32(const int32_t *acc_ih, const int32_t *acc_hh, float s_ih, float s_hh,
                       const float *bias, float *c, float *h, long B, long Hs) {
    for (long b = 0; b < B; ++b)
        for (long j = 0; j < Hs; ++j) {
            float pre[4];
            for (int g = 0; g < 4; ++g) {
                const long idx = b * 4 * Hs + g * Hs + j;
                const float u = (float)acc_ih[idx] * s_ih;
                const float v = (float)acc_hh[idx] * s_hh;
                float s = u + v;
                s = s + (bias ? bias[g * Hs + j] : 0.0f);
                pre[g] = s;
            }
            const float ig = orc_sigmoid_f32(pre[0]);
            const float fg = orc_sigmoid_f32(pre[1]);
            const float gg = orc_tanh_f32(pre[2]);
            const float og = orc_sigmoid_f32(pre[3]);
            const float fc = fg * c[b * Hs + j];
            const float igg = ig * gg;
            const float cn = fc + igg;
            c[b * Hs + j] = cn;
            h[b * Hs + j] = og * orc_tanh_f32(cn);
        }
}

/* GRU memory cell (Sec. III-B "RNN Layer": equivalent to the library layer), gate order r, z, n:
 *   gi = float(acc_ih)*s_ih + b_ih;   gh = float(acc_hh)*s_hh + b_hh        (per gate; a NULL bias adds nothing)
 *   r = sigmoid(gi_r + gh_r);  z = sigmoid(gi_z + gh_z);  n = tanh(gi_n + r*gh_n)   (product, then sum)
 *   h' = (1 - z)*n + z*h                                                    (two products, one sum)
 * acc_ih, acc_hh: [B][3*Hs];  h_prev, h_out: [B][Hs] (may be the same array). */
void orc_gru_cell_f32(const int32_t *acc_ih, const int32_t *acc_hh, float s_ih, float s_hh,
                      const float *b_ih, const float *b_hh, const float *h_prev, float *h_out, long B, long Hs) {
    for (long b = 0; b < B; ++b)
        for (long j = 0; j < Hs; ++j) {
            float gi[3], gh[3];
            for (int g = 0; g < 3; ++g) {
                const long idx = b * 3 * Hs + g * Hs + j;
                float u = (float)acc_ih[idx] * s_ih;
                if (b_ih) u = u + b_ih[g * Hs + j];
                float v = (float)acc_hh[idx] * s_hh;
                if (b_hh) v = v + b_hh[g * Hs + j];
                gi[g] = u;
                gh[g] = v;
            }
            const float r = orc_sigmoid_f32(gi[0] + gh[0]);
            const float z = orc_sigmoid_f32(gi[1] + gh[1]);
            const float rn = r * gh[2];
            const float n = orc_tanh_f32(gi[2] + rn);
            const float omz = 1.0f - z;
            const float a = omz * n;
            const float c = z * h_prev[b * Hs + j];
            h_out[b * Hs + j] = a + c;
        }
}

/* Plain recurrent cell (Sec. III-B "RNN Layer"): h' = act((float(acc_ih)*s_ih + float(acc_hh)*s_hh) + bias),
 * act = tanh (relu == 0) or max(., 0) (relu != 0).  acc_ih, acc_hh, h_out: [B][Hs]; bias [Hs] or NULL. */
void orc_rnn_cell_f32(const int32_t *acc_ih, const int32_t *acc_hh, float s_ih, float s_hh, const float *bias,
                      int relu, float *h_out, long B, long Hs) {
    for (long b = 0; b < B; ++b)
        for (long j = 0; j < Hs; ++j) {
            const long idx = b * Hs + j;
            const float u = (float)acc_ih[idx] * s_ih;
            const float v = (float)acc_hh[idx] * s_hh;
            float s = u + v;
            s = s + (bias ? bias[j] : 0.0f);
            h_out[idx] = relu ? (s > 0.0f ? s : 0.0f) : orc_tanh_f32(s);
        }
}

/* ===========================================================================
 * Operands wider than 8 bits and multipliers given as functions
 * (Sec. III-C "Framework operation": a table per multiplier, or - for large
 * bitwidths - the multiplier described as a function, "both a 1-1
 * representation" of the unit; Sec. V evaluates a 12-bit unit).
 * Operands are int16 in [-H, H-1], H = 2^(b-1); same table index convention
 * and the same sums as above.
 * ========================================================================= */

static int in_range16(const int16_t *p, size_t n, int bits) {
    const int h = 1 << (bits - 1);
    for (size_t i = 0; i < n; ++i)
        if (p[i] < -h || p[i] > h - 1) return 0;
    return 1;
}

/* Multipliers as functions of two signed operands.  kind 0: exact product.
 * kind 1: both operands lose their `param` low bits (arithmetic shift, i.e. floor) before an exact multiply, the
 *         product is shifted back: ((a >> t) * (w >> t)) << 2t.
 * kind 2: Mitchell's logarithmic multiplier on the magnitudes (sign restored afterwards): with a = 2^ka + xa,
 *         w = 2^kw + xw (ka, kw the positions of the leading ones), s = xa 2^kw + xw 2^ka:
 *         |a||w| ~ 2^(ka+kw) + s  if s < 2^(ka+kw),  else 2 s;   0 if an operand is 0.   (`param` unused.) */
int32_t orc_mul_func(int kind, int param, int a, int w) {
    if (kind == 0) return (int32_t)(a * w);
    if (kind == 1) {
        const int t = param;
        const int32_t pa = a >> t, pw = w >> t;      /* arithmetic shifts of negative values: floor */
        return (int32_t)((uint32_t)(pa * pw) << (2 * t));
    }
    const int neg = (a < 0) != (w < 0);
    uint32_t ma = (uint32_t)(a < 0 ? -a : a), mw = (uint32_t)(w < 0 ? -w : w);
    if (ma == 0 || mw == 0) return 0;
    int ka = 0, kw = 0;
    while ((ma >> (ka + 1)) != 0) ++ka;
    while ((mw >> (kw + 1)) != 0) ++kw;
    const uint32_t xa = ma - (1u << ka), xw = mw - (1u << kw);
    const uint32_t s = (xa << kw) + (xw << ka);
    const uint32_t one = 1u << (ka + kw);
    const uint32_t p = s < one ? one + s : 2u * s;
    return neg ? -(int32_t)p : (int32_t)p;
}

/* The table of a function-described multiplier (the table generator of Sec. III-C): T[(a+H) 2^b + (w+H)]. */
int orc_table_from_func(int kind, int param, int bits, int32_t *T) {
    if (!T || bits < 2 || bits > 12 || kind < 0 || kind > 2 || param < 0 || param >= bits) return ORC_BAD_ARG;
    const int n = 1 << bits, h = n >> 1;
    for (int a = -h; a < h; ++a)
        for (int w = -h; w < h; ++w) T[(size_t)(a + h) * n + (size_t)(w + h)] = orc_mul_func(kind, param, a, w);
    return ORC_OK;
}

/* acc[m][n] = sum_k T[A[m][k]][W[n][k]], int16 operands, 2 <= bits <= 12 */
int orc_approx_linear_i16(const int32_t *T, int bits, const int16_t *A, const int16_t *W, int32_t *acc,
                          long M, long K, long N, int threads) {
    if (!T || !A || !W || !acc || bits < 2 || bits > 12 || M < 0 || K < 0 || N < 0) return ORC_BAD_ARG;
    if (!in_range16(A, (size_t)M * K, bits) || !in_range16(W, (size_t)N * K, bits)) return ORC_BAD_ARG;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (long m = 0; m < M; ++m)
        for (long n = 0; n < N; ++n) {
            uint32_t s = 0;
            for (long k = 0; k < K; ++k) s += lut_at(T, bits, A[m * K + k], W[n * K + k]);
            acc[m * N + n] = (int32_t)s;
        }
    return ORC_OK;
}

/* acc[m][n] = sum_k f(A[m][k], W[n][k]) with the multiplier evaluated as a function, 2 <= bits <= 16 */
int orc_approx_linear_func_i16(int kind, int param, int bits, const int16_t *A, const int16_t *W, int32_t *acc,
                               long M, long K, long N, int threads) {
    if (!A || !W || !acc || bits < 2 || bits > 16 || kind < 0 || kind > 2 || param < 0 || param >= bits || M < 0 ||
        K < 0 || N < 0)
        return ORC_BAD_ARG;
    if (!in_range16(A, (size_t)M * K, bits) || !in_range16(W, (size_t)N * K, bits)) return ORC_BAD_ARG;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (long m = 0; m < M; ++m)
        for (long n = 0; n < N; ++n) {
            uint32_t s = 0;
            for (long k = 0; k < K; ++k) s += (uint32_t)orc_mul_func(kind, param, A[m * K + k], W[n * K + k]);
            acc[m * N + n] = (int32_t)s;
        }
    return ORC_OK;
}

/* 2-D convolution (Sec. III-B, groups = 1), int16 operands: T != NULL takes every product from the table
 * (bits <= 12), T == NULL evaluates the function (kind, param).  Padded taps meet activation 0 as above. */
int orc_approx_conv2d_i16(const int32_t *T, int kind, int param, int bits, const int16_t *x, const int16_t *w,
                          int32_t *acc, long N, long Cin, long H, long W, long Cout, long kh, long kw, long sh,
                          long sw, long ph, long pw, long dh, long dw, int threads) {
    if (!x || !w || !acc || bits < 2 || bits > (T ? 12 : 16)) return ORC_BAD_ARG;
    if (!T && (kind < 0 || kind > 2 || param < 0 || param >= bits)) return ORC_BAD_ARG;
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0 ||
        dh < 1 || dw < 1)
        return ORC_BAD_ARG;
    const long Ho = out_dim(H, kh, sh, ph, dh), Wo = out_dim(W, kw, sw, pw, dw);
    if (Ho < 1 || Wo < 1) return ORC_BAD_ARG;
    if (!in_range16(x, (size_t)N * Cin * H * W, bits) || !in_range16(w, (size_t)Cout * Cin * kh * kw, bits))
        return ORC_BAD_ARG;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (long n = 0; n < N; ++n)
        for (long co = 0; co < Cout; ++co)
            for (long oy = 0; oy < Ho; ++oy)
                for (long ox = 0; ox < Wo; ++ox) {
                    uint32_t s = 0;
                    for (long c = 0; c < Cin; ++c)
                        for (long ky = 0; ky < kh; ++ky)
                            for (long kx = 0; kx < kw; ++kx) {
                                const long iy = oy * sh - ph + ky * dh, ix = ox * sw - pw + kx * dw;
                                int a = 0;
                                if (iy >= 0 && iy < H && ix >= 0 && ix < W) a = x[((n * Cin + c) * H + iy) * W + ix];
                                const int wv = w[((co * Cin + c) * kh + ky) * kw + kx];
                                s += T ? lut_at(T, bits, a, wv) : (uint32_t)orc_mul_func(kind, param, a, wv);
                            }
                    acc[((n * Cout + co) * Ho + oy) * Wo + ox] = (int32_t)s;
                }
    return ORC_OK;
}

/* The quantiser of Sec. III-A for operands of up to 16 bits: q = clamp(rint(x / scale), -Q, Q), Q = 2^(b-1) - 1 */
int orc_quantize_i16_f32(const float *x, int16_t *q, size_t n, float scale, int bits) {
    if (!x || !q || bits < 2 || bits > 16 || !(scale > 0.0f)) return ORC_BAD_ARG;
    const float Q = (float)((1 << (bits - 1)) - 1);
    for (size_t i = 0; i < n; ++i) {
        float r = rintf(x[i] / scale);
        if (r != r) r = 0.0f;
        if (r > Q) r = Q;
        if (r < -Q) r = -Q;
        q[i] = (int16_t)r;
    }
    return ORC_OK;
}

