// Operands wider than 8 bits and multipliers given as functions (Sec. III-C "Framework operation": a table per
// multiplier or, for large bitwidths, the multiplier described as a function, both a 1-1 representation of the unit;
// Sec. V evaluates a 12-bit unit).
//
// A 2^b x 2^b table with b > 8 does not fit LDS (b = 12: 64 MB of int32), so the table form gathers from device memory:
// the table is stored weight-major, T[w + H][a + H], so that the 64 lanes of a wave - same weight, different
// activations - read inside ONE row of 2^b entries (16 KB at b = 12, and only the part of it that the activation
// distribution reaches), which the vector L1 and the L2 serve.  The function form evaluates the multiplier in the
// vector ALU and needs no memory at all; it covers operands of up to 16 bits.
//
// One kernel template serves both: lanes along the GEMM rows (output pixels), NT output channels per lane; per inner index
// the lane loads one activation and the NT weight words arrive through scalar loads (pre-packed [K][Npad] int32: element
// offset of the weight's table row, or the weight itself for the function form).  No LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elementwise.hpp"

namespace adapt {

// function form: 256 lanes, 8 channels per lane (the weight-side arithmetic is shared by the wave, the activation-side
// arithmetic by the 8 channels).  table form: 1024 lanes, 1 channel per lane, the waves of a workgroup kept in step by a
// barrier every four inner indices - all 16 waves then gather from the same table row at the same time and the vector L1
// (32 KB) serves most of their lines.  Measured on the 12-bit 3x3 layer (1.2 G lookups): 8 rows per step and free-running
// waves 3.7 ms with 30 L2 requests per gather instruction and a quarter of them missing L2 (20 GB fetched); the same with
// channel tiles spread over the XCDs 3.1 ms; 2 rows in step 1.7 ms; 1 row in step 1.6 ms with 7 L2 requests per gather.
constexpr int BIG_THREADS_FUNC = 256, BIG_NT_FUNC = 8;
constexpr int BIG_THREADS_TABLE = 1024, BIG_NT_TABLE = 1;

enum { FUNC_EXACT = 0, FUNC_TRUNC = 1, FUNC_MITCHELL = 2 };

// kind 0: exact product.  kind 1: both operands lose their t low bits (arithmetic shift = floor), exact multiply, shifted
// back.  kind 2: Mitchell's logarithmic multiplier on the magnitudes: a = 2^ka + xa, w = 2^kw + xw, s = xa 2^kw + xw 2^ka;
// |a||w| ~ 2^(ka+kw) + s if s < 2^(ka+kw), else 2 s; 0 for a zero operand; sign restored afterwards.
__device__ __forceinline__ int32_t mul_func(int kind, int t, int a, int w) {
    if (kind == FUNC_EXACT) return a * w;
    if (kind == FUNC_TRUNC) return (int32_t)((uint32_t)((a >> t) * (w >> t)) << (2 * t));
    // branch-free: a zero operand runs through the arithmetic with a harmless stand-in and is selected away at the end
    const uint32_t ma = (uint32_t)(a < 0 ? -a : a), mw = (uint32_t)(w < 0 ? -w : w);
    const int ka = 31 - __clz((int)(ma | 1u)), kw = 31 - __clz((int)(mw | 1u));
    const uint32_t s = ((ma - (1u << ka)) << kw) + ((mw - (1u << kw)) << ka);
    const uint32_t one = 1u << (ka + kw);
    uint32_t pr = s < one ? one + s : 2u * s;
    pr = (ma == 0 || mw == 0) ? 0u : pr;
    const uint32_t m = (uint32_t)((a ^ w) >> 31);       // all ones when the signs differ
    return (int32_t)((pr ^ m) - m);
}

struct MulTable {       // weight word = element offset of the table row of the weight
    const int32_t *T;
    int hoff, mask;
    __device__ __forceinline__ uint32_t operator()(int a, int wword) const { return (uint32_t)T[(size_t)wword + ((a + hoff) & mask)]; }
};
template <int KIND>
struct MulFunc {        // weight word = the weight
    int t;
    __device__ __forceinline__ uint32_t operator()(int a, int wword) const { return (uint32_t)mul_func(KIND, t, a, wword); }
};

// device table of a host table: Tdev[w + H][a + H] = Thost[a + H][w + H]
__global__ void big_transpose_kernel(const int32_t *__restrict__ src, int32_t *__restrict__ dst, int bits) {
    const size_t n = (size_t)1 << bits, total = n * n;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const size_t w = i >> bits, a = i & (n - 1);
        dst[i] = src[a * n + w];
    }
}

// device table of a function-described multiplier (the table generator of Sec. III-C), same layout
__global__ void big_table_from_func_kernel(int32_t *__restrict__ dst, int bits, int kind, int t) {
    const size_t n = (size_t)1 << bits, total = n * n;
    const int h = 1 << (bits - 1);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int w = (int)(i >> bits) - h, a = (int)(i & (n - 1)) - h;
        dst[i] = mul_func(kind, t, a, w);
    }
}

// weights [N][Cin][taps] int16 -> words [K = taps * Cin][Npad] int32, k = tap * Cin + ci (the order the kernel walks);
// table form (bits > 0): element offset of the weight's table row; function form (bits == 0): the weight
__global__ void big_pack_weights_kernel(const int16_t *__restrict__ w, int32_t *__restrict__ words, int K, int N, int Npad, int Cin,
                                        int taps, int bits) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)K * Npad) return;
    const int k = (int)(idx / Npad), n = (int)(idx % Npad);
    int32_t v = 0;
    if (n < N) {
        const int t = k / Cin, ci = k - t * Cin;
        const int wv = w[((size_t)n * Cin + ci) * taps + t];
        v = bits > 0 ? (int32_t)((uint32_t)((wv + (1 << (bits - 1))) & ((1 << bits) - 1)) << bits) : wv;
    }
    words[idx] = v;
}

struct BigParams {
    const int16_t *x;       // [M][K] or NCHW
    const int32_t *words;   // [K][Npad]
    int32_t *out;           // [M][N] or NCHW
    int M, N, Npad;
    int conv;               // 0: GEMM, 1: convolution
    int Cin, taps, kw;      // GEMM: Cin = K, taps = 1
    int H, W, Wo, HoWo;     // GEMM: HoWo = Wo = 1
    int sh, sw, ph, pw, dh, dw;
    int kstride, img_stride;
    // whole-layer form: deq != 0 stores fp32 y = float(acc) * scale (or scales[n]), + bias[n] if bias, then ReLU (act 1) or
    // tanh (act 2) instead of the integer sum
    int deq, act;
    float scale;
    const float *scales, *bias;
};

__device__ __forceinline__ uint32_t big_finish(const BigParams &p, uint32_t v, int n) {
    if (!p.deq) return v;
    float y = (float)(int32_t)v * (p.scales ? p.scales[n] : p.scale);
    if (p.bias) y = y + p.bias[n];
    if (p.act == 1) y = y > 0.0f ? y : 0.0f;
    else if (p.act == 2) y = tanh_spec(y);
    return __float_as_uint(y);
}

template <class Mul, int NT, int THREADS, bool IN_STEP>
__global__ __launch_bounds__(THREADS) void big_rows_kernel(const BigParams p, const Mul mul) {
    // workgroup id -> (channel tile fastest, then row tile): consecutive workgroups go to different XCDs, so each L2
    // serves the table rows of few channel tiles (with 8 tiles: of one) instead of all of them
    const int n_tiles = p.Npad / NT;
    const int n_tile = blockIdx.x % n_tiles, m_tile = blockIdx.x / n_tiles;
    const int m = m_tile * THREADS + threadIdx.x;
    const bool mvalid = m < p.M;
    const int mm = mvalid ? m : p.M - 1;
    const int n0 = n_tile * NT;
    const int img = mm / p.HoWo, pix = mm - img * p.HoWo;
    const int oy = pix / p.Wo, ox = pix - oy * p.Wo;
    const int16_t *xb = p.x + (size_t)img * p.img_stride;
    uint32_t acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = 0;
    for (int t = 0; t < p.taps; ++t) {
        int base = 0;
        bool valid = true;
        if (p.conv) {
            const int ky = t / p.kw, kx = t - ky * p.kw;
            const int iy = oy * p.sh - p.ph + ky * p.dh, ix = ox * p.sw - p.pw + kx * p.dw;
            valid = (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
            base = iy * p.W + ix;
        }
        const int16_t *xp = xb + (valid ? base : 0);
        const int32_t *wr = p.words + (size_t)t * p.Cin * p.Npad + n0;
        int c = 0;
        for (; c + 4 <= p.Cin; c += 4) {        // four activations, then their 4 x NT products (independent loads in flight)
            int a[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int v = xp[(size_t)(c + kk) * p.kstride];
                a[kk] = valid ? v : 0;          // a padded tap meets activation 0
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int32_t *w4 = wr + (size_t)(c + kk) * p.Npad;
                int32_t ww[NT];                 // the NT words of this inner index: one scalar load
#pragma unroll
                for (int n = 0; n < NT; ++n) ww[n] = w4[n];
#pragma unroll
                for (int n = 0; n < NT; ++n) acc[n] += mul(a[kk], ww[n]);
            }
            if (IN_STEP) __syncthreads();       // (uniform trip counts: every lane of the workgroup gets here)
        }
        for (; c < p.Cin; ++c) {
            const int v = xp[(size_t)c * p.kstride];
            const int a = valid ? v : 0;
            const int32_t *w1 = wr + (size_t)c * p.Npad;
#pragma unroll
            for (int n = 0; n < NT; ++n) acc[n] += mul(a, w1[n]);
        }
    }
    if (mvalid) {
        int32_t *o = p.out + (size_t)img * p.N * p.HoWo + pix;
#pragma unroll
        for (int n = 0; n < NT; ++n)
            if (n0 + n < p.N) o[(size_t)(n0 + n) * p.HoWo] = (int32_t)big_finish(p, acc[n], n0 + n);
    }
}

// q = clamp(rint(x / scale), -Q, Q) into int16 (Sec. III-A), the quantiser of elementwise.hpp for up to 16 bits
__global__ __launch_bounds__(256) void quantize_i16_kernel(const float *__restrict__ x, int16_t *__restrict__ q, size_t n, float scale,
                                                           float Q) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        float r = rintf(x[i] / scale);
        if (r != r) r = 0.0f;
        if (r > Q) r = Q;
        if (r < -Q) r = -Q;
        q[i] = (int16_t)(int)r;
    }
}

}  // namespace adapt
