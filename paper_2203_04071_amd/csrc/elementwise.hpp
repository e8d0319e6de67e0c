// HBM-bound kernels of the path: max-abs calibration, quantiser, dequantiser (Sec. III-A of the
// paper) and the fp32 operations between approximate layers (Sec. III-B "RNN Layer" memory cell,
// residual adds, pooling).  gfx950 only; compiled with -ffp-contract=off so that every fp32 step
// rounds exactly where the text says it does.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace adapt {

constexpr int EW_THREADS = 256;

// Division of a 31-bit number by a launch-invariant divisor as multiply + shift: q = (n * M) >> k with
// k = 31 + ceil(log2 d), M = floor(2^k / d) + 1, exact for every n < 2^31 (the error term n / 2^k stays below 1 / d).
// An integer division costs about 35 vector instructions (a 64-bit one several times that), and the copy and
// element-wise kernels are bound by instruction count.
struct FastDiv {
    uint32_t M;
    int k;
    uint32_t d;
    __device__ __forceinline__ uint32_t div(uint32_t n) const { return (uint32_t)(((uint64_t)n * M) >> k); }
};

static __global__ void fill_u32_kernel(uint32_t *p, uint32_t v, size_t n) {       // any grid: strides over n
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = v;
}

// max |x|: the bit pattern of a non-negative float orders like an unsigned integer, so the final
// combine is an integer atomic max; NaNs fail the comparison and are skipped.
static __global__ __launch_bounds__(EW_THREADS) void absmax_kernel(const float *__restrict__ x, size_t n,
                                                            uint32_t *__restrict__ out_bits, int vec) {
    __shared__ float wave_max[EW_THREADS / 64];
    float m = 0.0f;
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    const size_t n4 = vec ? n / 4 : 0;   // vec: x is 16-byte aligned
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    auto fold = [&](const float4 v) {
        float a = fabsf(v.x); if (a > m) m = a;
        a = fabsf(v.y); if (a > m) m = a;
        a = fabsf(v.z); if (a > m) m = a;
        a = fabsf(v.w); if (a > m) m = a;
    };
    size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    for (; i + 3 * stride < n4; i += 4 * stride) {      // four loads in flight per lane
        const float4 v0 = x4[i], v1 = x4[i + stride], v2 = x4[i + 2 * stride], v3 = x4[i + 3 * stride];
        fold(v0); fold(v1); fold(v2); fold(v3);
    }
    for (; i < n4; i += stride) fold(x4[i]);
    for (size_t j = n4 * 4 + (size_t)blockIdx.x * EW_THREADS + threadIdx.x; j < n; j += stride) {
        const float a = fabsf(x[j]);
        if (a > m) m = a;
    }
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(m, off, 64);
        if (o > m) m = o;
    }
    // one atomic per workgroup: thousands of them on one address are what a short launch would otherwise wait for
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
#pragma unroll
        for (int w = 1; w < EW_THREADS / 64; ++w)
            if (wave_max[w] > m) m = wave_max[w];
        atomicMax(out_bits, __float_as_uint(m));
    }
}

__device__ __forceinline__ int quant1(float x, float scale, float Q) {
    float r = rintf(x / scale);          // IEEE divide, round half to even
    if (r != r) r = 0.0f;
    if (r > Q) r = Q;
    if (r < -Q) r = -Q;
    return (int)r;
}

static __global__ __launch_bounds__(EW_THREADS) void quantize_kernel(const float *__restrict__ x, int8_t *__restrict__ q,
                                                              size_t n, float scale, float Q, int vec) {
    // 16 values per thread step: four 16-byte loads, one 16-byte store (vec: both pointers 16-byte aligned)
    const size_t n16 = vec ? n / 16 : 0;
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    const float4 *x4 = reinterpret_cast<const float4 *>(x);
    uint4 *q16 = reinterpret_cast<uint4 *>(q);
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n16; i += stride) {
        uint32_t w[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 v = x4[i * 4 + j];
            const uint32_t b0 = (uint32_t)quant1(v.x, scale, Q) & 0xffu;
            const uint32_t b1 = (uint32_t)quant1(v.y, scale, Q) & 0xffu;
            const uint32_t b2 = (uint32_t)quant1(v.z, scale, Q) & 0xffu;
            const uint32_t b3 = (uint32_t)quant1(v.w, scale, Q) & 0xffu;
            w[j] = b0 | (b1 << 8) | (b2 << 16) | (b3 << 24);
        }
        q16[i] = make_uint4(w[0], w[1], w[2], w[3]);
    }
    for (size_t i = n16 * 16 + (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride)
        q[i] = (int8_t)quant1(x[i], scale, Q);
}

// ---- the quantiser as the paper configures it (Sec. III-A "Parameter calibration"): weight ranges per output
// channel, activation range from a histogram percentile

// amax[r] = max |x[r][0..cols)|; one workgroup per row
static __global__ __launch_bounds__(EW_THREADS) void absmax_rows_kernel(const float *__restrict__ x, size_t cols, float *__restrict__ amax) {
    __shared__ float part[EW_THREADS / 64];
    const float *row = x + (size_t)blockIdx.x * cols;
    float m = 0.0f;
    for (size_t c = threadIdx.x; c < cols; c += EW_THREADS) {
        const float a = fabsf(row[c]);
        if (a > m) m = a;          // NaN compares false and is skipped
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float o = __shfl_xor(m, off, 64);
        if (o > m) m = o;
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < EW_THREADS / 64; ++w)
            if (part[w] > m) m = part[w];
        amax[blockIdx.x] = m;
    }
}

// q[r][c] = quantise(x[r][c], scale[r])
static __global__ __launch_bounds__(EW_THREADS) void quantize_rows_kernel(const float *__restrict__ x, int8_t *__restrict__ q, size_t rows,
                                                                   size_t cols, const float *__restrict__ scale, float Q) {
    const size_t n = rows * cols;
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) q[i] = (int8_t)quant1(x[i], scale[i / cols], Q);
}

// y = float(acc) * scale[c] (+ bias[c])
static __global__ __launch_bounds__(EW_THREADS) void dequant_pc_kernel(const int32_t *__restrict__ acc, float *__restrict__ y, size_t n,
                                                                size_t channels, size_t inner, const float *__restrict__ scale,
                                                                const float *__restrict__ bias) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) {
        const size_t c = (i / inner) % channels;
        float v = (float)acc[i] * scale[c];
        if (bias) v = v + bias[c];
        y[i] = v;
    }
}

// counts[bin(|x_i|)] += 1 with bins equal bins over [0, amax]: bin(a) = min(bins - 1, trunc(a / width)), width = amax / bins
// (both IEEE fp32 divisions); NaN is not counted.  Per-workgroup histogram in LDS (bins <= 4096), then one atomic per
// non-empty bin.
static __global__ __launch_bounds__(EW_THREADS) void histogram_abs_kernel(const float *__restrict__ x, size_t n, float width, int bins,
                                                                   uint32_t *__restrict__ counts, int vec) {
    __shared__ uint32_t h[4096];
    for (int b = threadIdx.x; b < bins; b += EW_THREADS) h[b] = 0;
    __syncthreads();
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    auto count = [&](float v) {
        const float a = fabsf(v);
        if (a != a) return;
        const float t = a / width;
        const int b = t >= (float)bins ? bins - 1 : (int)t;
        atomicAdd(&h[b < bins ? b : bins - 1], 1u);
    };
    const size_t n4 = vec ? n / 4 : 0;      // vec: x is 16-byte aligned
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n4; i += stride) {
        const float4 v = reinterpret_cast<const float4 *>(x)[i];
        count(v.x); count(v.y); count(v.z); count(v.w);
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) count(x[i]);
    __syncthreads();
    for (int b = threadIdx.x; b < bins; b += EW_THREADS)
        if (h[b]) atomicAdd(&counts[b], h[b]);
}

// calib_max = (k + 1) * width for the first bin k at which the cumulative count reaches ceil(total * num / den)
static __global__ void percentile_kernel(const uint32_t *__restrict__ counts, int bins, float width, unsigned long long num,
                                  unsigned long long den, float *__restrict__ out) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    unsigned long long total = 0;
    for (int b = 0; b < bins; ++b) total += counts[b];
    const unsigned long long target = (total * num + den - 1) / den;
    unsigned long long cum = 0;
    int k = bins - 1;
    for (int b = 0; b < bins; ++b) {
        cum += counts[b];
        if (cum >= target) { k = b; break; }
    }
    out[0] = (float)(k + 1) * width;
}

// Least-squares range from the histogram: candidate k has range t_k = (k + 1) * width and scale s = t_k / Q (fp32); a
// value at the centre c_j = (j + 0.5) * width of bin j is reproduced as min(Q, rint(c_j / s)) * s; err[k] = sum_j
// counts[j] * (c_j - that)^2 in fp64, j ascending, every operation rounded on its own (the library is compiled without
// contraction).  One thread per candidate.
static __global__ __launch_bounds__(256) void mse_candidates_kernel(const uint32_t *__restrict__ counts, int bins, float width, float Qf,
                                                             double *__restrict__ err) {
    __shared__ uint32_t cnt[4096];
    for (int j = threadIdx.x; j < bins; j += 256) cnt[j] = counts[j];
    __syncthreads();
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= bins) return;
    const float t = (float)(k + 1) * width;
    const double s = (double)(t / Qf), Q = (double)Qf;
    double e2 = 0.0;
    for (int j = 0; j < bins; ++j) {
        const uint32_t n = cnt[j];
        if (!n) continue;
        const double c = ((double)j + 0.5) * (double)width;
        double q = rint(c / s);
        if (q > Q) q = Q;
        const double e = c - q * s;
        e2 = e2 + (double)n * (e * e);
    }
    err[k] = e2;
}

// the first candidate with the smallest error: calib_max = (k + 1) * width
static __global__ void mse_pick_kernel(const double *__restrict__ err, int bins, float width, float *__restrict__ out) {
    if (blockIdx.x != 0 || threadIdx.x != 0) return;
    int best_k = 0;
    double best = err[0];
    for (int k = 1; k < bins; ++k)
        if (err[k] < best) { best = err[k]; best_k = k; }
    out[0] = (float)(best_k + 1) * width;
}

// Information-loss range from the histogram (the third calibrator Sec. III-A names; the definition is this library's,
// stated in the header).  Candidate k keeps the first k bins, k = min(L, bins) .. bins with L = 2^(bits-1) levels.
// Reference p: the kept counts with everything beyond added to the last kept bin.  Quantised q: the kept counts alone,
// merged into min(L, k) groups [g k / L, (g+1) k / L) and spread evenly over each group's non-empty bins.  loss[k-1] =
// sum over the kept bins with p > 0, ascending, of (p/P) log((p/P) / (q/Q)), +inf where p > 0 meets q = 0; fp64, every
// operation rounded on its own.  One thread per candidate; loss of a k that is no candidate = +inf.  An empty
// histogram keeps the whole range (loss 0 at k = bins only).
static __global__ __launch_bounds__(256) void entropy_candidates_kernel(const uint32_t *__restrict__ counts, int bins, int levels,
                                                                 double *__restrict__ loss) {
    __shared__ uint32_t cnt[4096];
    for (int j = threadIdx.x; j < bins; j += 256) cnt[j] = counts[j];
    __syncthreads();
    const int k = blockIdx.x * 256 + threadIdx.x + 1;
    if (k > bins) return;
    const double inf = __builtin_inf();
    const int k_first = levels < bins ? levels : bins;
    if (k < k_first) { loss[k - 1] = inf; return; }
    unsigned long long total = 0, kept = 0;
    for (int j = 0; j < bins; ++j) { total += cnt[j]; if (j < k) kept += cnt[j]; }
    if (total == 0) { loss[k - 1] = k == bins ? 0.0 : inf; return; }
    const unsigned long long outliers = total - kept;
    const double P = (double)total;
    const long long groups = levels < k ? levels : k;
    double Q = 0.0;
    for (long long g = 0; g < groups; ++g) {
        const int lo = (int)(g * k / groups), hi = (int)((g + 1) * k / groups);
        unsigned long long sg = 0; int zg = 0;
        for (int j = lo; j < hi; ++j) { sg += cnt[j]; zg += cnt[j] > 0; }
        if (zg) Q = Q + (double)zg * ((double)sg / (double)zg);
    }
    double acc = 0.0;
    for (long long g = 0; g < groups; ++g) {
        const int lo = (int)(g * k / groups), hi = (int)((g + 1) * k / groups);
        unsigned long long sg = 0; int zg = 0;
        for (int j = lo; j < hi; ++j) { sg += cnt[j]; zg += cnt[j] > 0; }
        for (int j = lo; j < hi; ++j) {
            const unsigned long long pj = (unsigned long long)cnt[j] + (j == k - 1 ? outliers : 0ull);
            if (!pj) continue;
            if (!cnt[j]) { acc = inf; continue; }
            const double pn = (double)pj / P, qn = ((double)sg / (double)zg) / Q;
            acc = acc + pn * log(pn / qn);
        }
    }
    loss[k - 1] = acc;
}

// y = float(acc) * scale (+ bias[c]); channel of flat index i is (i / inner) % channels
static __global__ __launch_bounds__(EW_THREADS) void dequant_kernel(const int32_t *__restrict__ acc, float *__restrict__ y,
                                                             size_t n, size_t channels, size_t inner, float scale,
                                                             const float *__restrict__ bias, int vec) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    // vec: both pointers 16-byte aligned and four consecutive elements share one channel (or no bias)
    if (vec) {
        const size_t n4 = n / 4;
        const int4 *a4 = reinterpret_cast<const int4 *>(acc);
        float4 *y4 = reinterpret_cast<float4 *>(y);
        for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n4; i += stride) {
            const int4 a = a4[i];
            float4 v;
            v.x = (float)a.x * scale; v.y = (float)a.y * scale; v.z = (float)a.z * scale; v.w = (float)a.w * scale;
            if (bias) {
                const float b = bias[((i * 4) / inner) % channels];
                v.x = v.x + b; v.y = v.y + b; v.z = v.z + b; v.w = v.w + b;
            }
            y4[i] = v;
        }
        for (size_t i = n4 * 4 + (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) {
            float v = (float)acc[i] * scale;
            if (bias) v = v + bias[(i / inner) % channels];
            y[i] = v;
        }
    } else {
        for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) {
            float v = (float)acc[i] * scale;
            if (bias) v = v + bias[(i / inner) % channels];
            y[i] = v;
        }
    }
}

// vec: every pointer is 16-byte aligned - four elements per lane and iteration (the same operation on each element;
// y may be x itself)
static __global__ __launch_bounds__(EW_THREADS) void relu_kernel(const float *x, float *y, size_t n, int vec) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    const size_t n4 = vec ? n / 4 : 0;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n4; i += stride) {
        float4 v = reinterpret_cast<const float4 *>(x)[i];
        v.x = v.x > 0.0f ? v.x : 0.0f; v.y = v.y > 0.0f ? v.y : 0.0f; v.z = v.z > 0.0f ? v.z : 0.0f; v.w = v.w > 0.0f ? v.w : 0.0f;
        reinterpret_cast<float4 *>(y)[i] = v;
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) {
        const float v = x[i];
        y[i] = v > 0.0f ? v : 0.0f;
    }
}

static __global__ __launch_bounds__(EW_THREADS) void add_kernel(const float *a, const float *b, float *y, size_t n, int relu, int vec) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    const size_t n4 = vec ? n / 4 : 0;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n4; i += stride) {
        const float4 p = reinterpret_cast<const float4 *>(a)[i], q = reinterpret_cast<const float4 *>(b)[i];
        float4 v = make_float4(p.x + q.x, p.y + q.y, p.z + q.z, p.w + q.w);
        if (relu) { v.x = v.x > 0.0f ? v.x : 0.0f; v.y = v.y > 0.0f ? v.y : 0.0f; v.z = v.z > 0.0f ? v.z : 0.0f; v.w = v.w > 0.0f ? v.w : 0.0f; }
        reinterpret_cast<float4 *>(y)[i] = v;
    }
    for (size_t i = n4 * 4 + (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) {
        float v = a[i] + b[i];
        if (relu) v = v > 0.0f ? v : 0.0f;
        y[i] = v;
    }
}

// gradient through the fused ReLU: dx = dy where the layer's output y is positive
static __global__ __launch_bounds__(EW_THREADS) void relu_backward_kernel(const float *dy, const float *__restrict__ y, float *dx, size_t n) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) dx[i] = y[i] > 0.0f ? dy[i] : 0.0f;
}

// plain stochastic-gradient step of the retraining loop: w <- w - lr * g, the product and the difference rounded separately
static __global__ __launch_bounds__(EW_THREADS) void sgd_kernel(float *__restrict__ w, const float *__restrict__ g, size_t n, float lr) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) w[i] = w[i] - lr * g[i];
}

// one thread per (n, c) plane: the sum order (row-major, sequential) is part of the definition
static __global__ __launch_bounds__(EW_THREADS) void avgpool_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                             size_t NC, size_t HW) {
    const size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (i >= NC) return;
    const float inv = 1.0f / (float)HW;
    float s = 0.0f;
    for (size_t j = 0; j < HW; ++j) s = s + x[i * HW + j];
    y[i] = s * inv;
}

// The same for planes of 64 elements (an 8 x 8 feature map), 64 planes per workgroup of 64 lanes: the planes are read
// with coalesced 16-byte loads into LDS (row pitch 65 words, so that lane t summing plane t meets no bank conflict),
// then every lane adds up its plane in the same sequential order as above.
static __global__ __launch_bounds__(64) void avgpool64_kernel(const float *__restrict__ x, float *__restrict__ y, size_t NC) {
    __shared__ float tile[64 * 65];
    const size_t p0 = (size_t)blockIdx.x * 64;
    const int t = threadIdx.x;
    const size_t planes = NC - p0 < 64 ? NC - p0 : 64;
    const float4 *src = reinterpret_cast<const float4 *>(x + p0 * 64);
    for (int q = t; q < (int)planes * 16; q += 64) {       // float4 q = plane q / 16, elements 4 (q % 16) ..
        const float4 v = src[q];
        float *d = tile + (q >> 4) * 65 + (q & 15) * 4;
        d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
    }
    __syncthreads();
    if ((size_t)t >= planes) return;
    const float inv = 1.0f / 64.0f;
    float s = 0.0f;
#pragma unroll 8
    for (int j = 0; j < 64; ++j) s = s + tile[t * 65 + j];
    y[p0 + t] = s * inv;
}

static __global__ __launch_bounds__(EW_THREADS) void shortcut_a_kernel(const float *__restrict__ x, float *__restrict__ y,
                                                                int N, int Cin, int H, int W, int Cout, FastDiv dwo, FastDiv dho,
                                                                FastDiv dco, int fast) {
    const int Ho = (H + 1) / 2, Wo = (W + 1) / 2, padc = (Cout - Cin) / 2;
    const size_t total = (size_t)N * Cout * Ho * Wo;
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    if (fast) {         // fewer than 2^31 elements on both sides: 32-bit indices, divisions by multiply-and-shift
        for (uint32_t i = blockIdx.x * EW_THREADS + threadIdx.x; i < (uint32_t)total; i += (uint32_t)stride) {
            const uint32_t r1 = dwo.div(i), ox = i - r1 * (uint32_t)Wo;
            const uint32_t r2 = dho.div(r1), oy = r1 - r2 * (uint32_t)Ho;
            const uint32_t n = dco.div(r2), c = r2 - n * (uint32_t)Cout;
            const int ci = (int)c - padc;
            float v = 0.0f;
            if (ci >= 0 && ci < Cin) v = x[((n * (uint32_t)Cin + (uint32_t)ci) * (uint32_t)H + 2u * oy) * (uint32_t)W + 2u * ox];
            y[i] = v;
        }
        return;
    }
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < total; i += stride) {
        const int ox = (int)(i % Wo);
        const int oy = (int)((i / Wo) % Ho);
        const int c = (int)((i / ((size_t)Wo * Ho)) % Cout);
        const int n = (int)(i / ((size_t)Wo * Ho * Cout));
        const int ci = c - padc;
        float v = 0.0f;
        if (ci >= 0 && ci < Cin) v = x[(((size_t)n * Cin + ci) * H + 2 * oy) * W + 2 * ox];
        y[i] = v;
    }
}

// exp(x) written out so that host and device agree bit for bit: clamp to [-87, 88];
// n = rint(x * log2 e); r = x - n ln2 in two fused steps (hi/lo split of ln 2); degree-7 Taylor
// polynomial in Horner form, fused multiply-adds; exact scaling by 2^n.
__device__ __forceinline__ float exp_spec(float x) {
    const float LOG2E = 0x1.715476p+0f, LN2_HI = 0x1.62e400p-1f, LN2_LO = 0x1.7f7d1cp-20f;
    if (x != x) return x;
    if (x < -87.0f) x = -87.0f;
    if (x > 88.0f) x = 88.0f;
    const float n = rintf(x * LOG2E);
    float r = __builtin_fmaf(n, -LN2_HI, x);
    r = __builtin_fmaf(n, -LN2_LO, r);
    float p = 0x1.a01a02p-13f;
    p = __builtin_fmaf(p, r, 0x1.6c16c2p-10f);
    p = __builtin_fmaf(p, r, 0x1.111112p-7f);
    p = __builtin_fmaf(p, r, 0x1.555556p-5f);
    p = __builtin_fmaf(p, r, 0x1.555556p-3f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    return ldexpf(p, (int)n);
}

__device__ __forceinline__ float sigmoid_spec(float x) { return 1.0f / (1.0f + exp_spec(-x)); }

__device__ __forceinline__ float tanh_spec(float x) {
    const float ax = fabsf(x);
    const float e = exp_spec(-2.0f * ax);
    const float t = (1.0f - e) / (1.0f + e);
    return x < 0.0f ? -t : t;
}

static __global__ __launch_bounds__(EW_THREADS) void unary_kernel(const float *x, float *y, size_t n, int op) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) {
        const float v = x[i];
        y[i] = op == 0 ? tanh_spec(v) : (op == 1 ? sigmoid_spec(v) : exp_spec(v));
    }
}

static __global__ __launch_bounds__(EW_THREADS) void lstm_cell_kernel(const int32_t *__restrict__ acc_ih,
                                                               const int32_t *__restrict__ acc_hh, float s_ih,
                                                               float s_hh, const float *__restrict__ bias,
                                                               float *__restrict__ c, float *__restrict__ h, int B,
                                                               int Hs, int8_t *__restrict__ qh, float s_h, float Qh) {
    const size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (i >= (size_t)B * Hs) return;
    const int b = (int)(i / Hs), j = (int)(i % Hs);
    float pre[4];
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const size_t idx = (size_t)b * 4 * Hs + (size_t)g * Hs + j;
        const float u = (float)acc_ih[idx] * s_ih;
        const float v = (float)acc_hh[idx] * s_hh;
        float s = u + v;
        s = s + (bias ? bias[g * Hs + j] : 0.0f);
        pre[g] = s;
    }
    const float ig = sigmoid_spec(pre[0]);
    const float fg = sigmoid_spec(pre[1]);
    const float gg = tanh_spec(pre[2]);
    const float og = sigmoid_spec(pre[3]);
    const float fc = fg * c[i];
    const float igg = ig * gg;
    const float cn = fc + igg;
    c[i] = cn;
    const float hn = og * tanh_spec(cn);
    h[i] = hn;
    if (qh) qh[i] = (int8_t)quant1(hn, s_h, Qh);      // the next step's operand, same quantiser as quantize_kernel
}

// GRU memory cell (Sec. III-B "RNN Layer"), gate order r, z, n along the 3 Hs axis; every operation a single
// rounded fp32 operation in this order:
//   gi = float(acc_ih) * s_ih (+ b_ih);  gh = float(acc_hh) * s_hh (+ b_hh)
//   r = sigmoid(gi_r + gh_r);  z = sigmoid(gi_z + gh_z);  n = tanh(gi_n + r * gh_n);  h' = (1 - z) * n + z * h
static __global__ __launch_bounds__(EW_THREADS) void gru_cell_kernel(const int32_t *__restrict__ acc_ih, const int32_t *__restrict__ acc_hh,
                                                              float s_ih, float s_hh, const float *__restrict__ b_ih,
                                                              const float *__restrict__ b_hh, const float *h_prev, float *h, int B,
                                                              int Hs, int8_t *__restrict__ qh, float s_h, float Qh) {
    const size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (i >= (size_t)B * Hs) return;
    const int b = (int)(i / Hs), j = (int)(i % Hs);
    float gi[3], gh[3];
#pragma unroll
    for (int g = 0; g < 3; ++g) {
        const size_t idx = (size_t)b * 3 * Hs + (size_t)g * Hs + j;
        float u = (float)acc_ih[idx] * s_ih;
        if (b_ih) u = u + b_ih[g * Hs + j];
        float v = (float)acc_hh[idx] * s_hh;
        if (b_hh) v = v + b_hh[g * Hs + j];
        gi[g] = u;
        gh[g] = v;
    }
    const float r = sigmoid_spec(gi[0] + gh[0]);
    const float z = sigmoid_spec(gi[1] + gh[1]);
    const float rn = r * gh[2];
    const float n = tanh_spec(gi[2] + rn);
    const float omz = 1.0f - z;
    const float t0 = omz * n;
    const float t1 = z * h_prev[i];
    const float hn = t0 + t1;
    h[i] = hn;
    if (qh) qh[i] = (int8_t)quant1(hn, s_h, Qh);
}

// Plain recurrent cell: h' = act((float(acc_ih) * s_ih + float(acc_hh) * s_hh) + bias), act = tanh or ReLU
static __global__ __launch_bounds__(EW_THREADS) void rnn_cell_kernel(const int32_t *__restrict__ acc_ih, const int32_t *__restrict__ acc_hh,
                                                              float s_ih, float s_hh, const float *__restrict__ bias, int relu,
                                                              float *__restrict__ h, int B, int Hs, int8_t *__restrict__ qh, float s_h,
                                                              float Qh) {
    const size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x;
    if (i >= (size_t)B * Hs) return;
    const int j = (int)(i % Hs);
    const float u = (float)acc_ih[i] * s_ih;
    const float v = (float)acc_hh[i] * s_hh;
    float s = u + v;
    s = s + (bias ? bias[j] : 0.0f);
    const float hn = relu ? (s > 0.0f ? s : 0.0f) : tanh_spec(s);
    h[i] = hn;
    if (qh) qh[i] = (int8_t)quant1(hn, s_h, Qh);
}

}  // namespace adapt
