// Backward pass of an approximate linear layer under the straight-through estimator (Sec. III-A, "Retraining"):
// the quantiser passes a gradient where its clamp did not act, the multiplier table is differentiated as the exact
// product.  Both gradients are dense fp32 contractions with one fake-quantised operand,
//
//     dx[m][k] = inside(x[m][k]) * sum_n dy[m][n] * w^[n][k]          w^ = s_w * q(w)
//     dw[n][k] = inside(w[n][k]) * sum_m dy[m][n] * x^[m][k]          x^ = s_x * q(x)
//
// so this is the one part of the library that belongs on the matrix pipe as a plain product: v_mfma_f32_32x32x2_f32,
// operands staged through LDS, the fake quantisation applied while a tile is staged and the clip mask in the epilogue
// (no quantised copy of x or w is ever written to memory).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "elementwise.hpp"

namespace adapt {

typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int STE_TR = 32;          // contraction indices per staged chunk
constexpr int STE_THREADS = 256;    // four waves, 2 x 2 over the workgroup's output tile (x KS, see the kernel)

// geometry of a convolution whose unfolded input takes part in a product (see the end of this file)
struct SteConvGeo {
    int N, C, H, W, O, kh, kw, sh, sw, ph, pw, dh, dw, Ho, Wo;
    FastDiv dK, dkw, dkhkw, dWo, dHoWo, dC, dW, dHW, dO, dP, dsh, dsw;      // the divisors of the index decodes below
};

// n / f.d: multiply-and-shift for 32-bit indices (exact below 2^31), a plain division otherwise
template <typename Idx>
__device__ __forceinline__ Idx ste_div(Idx n, const FastDiv &f) {
    if constexpr (sizeof(Idx) == 4) return (Idx)f.div((uint32_t)n);
    else return n / (Idx)f.d;
}

// c[i][j] = inside(o[i][j]) * sum_r A(i, r) * fq(b[r][j])
struct SteParams {
    const float *a;     // A_T: element (i, r) at a[r * lda + i]; else at a[i * lda + r]
    const float *b;     // [R][J], fake-quantised with scale sb while it is staged
    const float *o;     // [I][J], decides the clip mask with scale so; nullptr: no mask
    float *c;           // [I][J]
    int I, J, R, lda;
    float sb, so, Q;
    int cps;            // chunks of STE_TR contraction indices per grid z: z > 0 writes its partial sums to c + z * I * J
    int im2col;         // b is an NCHW image tensor x and stands for its unfolded matrix: b[r][j] = x(n, c, oy s - p + ky d, ...)
    SteConvGeo g;       //   with r = (n, oy, ox), j = (c, ky, kx) of this geometry, zero outside the image
};

__device__ __forceinline__ float ste_fake_quant(float x, float s, float Q) {
    float r = rintf(x / s);         // IEEE divide, round half to even: the forward quantiser's decision
    if (r != r) r = 0.0f;
    if (r > Q) r = Q;
    if (r < -Q) r = -Q;
    return r * s;
}

__device__ __forceinline__ bool ste_inside(float x, float s, float Q) { return fabsf(rintf(x / s)) <= Q; }     // NaN: false

// Four consecutive elements of a row-major matrix (col a multiple of 4).  FULL: the whole tile lies inside the matrix
// and rows are 16-byte aligned, one load.  Otherwise: zero outside the matrix, read without a branch from clamped
// addresses (rows, cols >= 1), so that the loads of a chunk stay in flight together.
template <bool FULL>
__device__ __forceinline__ float4 ste_load4(const float *__restrict__ base, int row, int col, int rows, int cols, int ld) {
    if (FULL) return *reinterpret_cast<const float4 *>(base + (size_t)row * (size_t)ld + (size_t)col);
    const float *q = base + (size_t)min(row, rows - 1) * (size_t)ld;
    const bool in_row = row < rows;
    float4 v;
    v.x = q[min(col + 0, cols - 1)];
    v.y = q[min(col + 1, cols - 1)];
    v.z = q[min(col + 2, cols - 1)];
    v.w = q[min(col + 3, cols - 1)];
    v.x = (in_row && col + 0 < cols) ? v.x : 0.0f;
    v.y = (in_row && col + 1 < cols) ? v.y : 0.0f;
    v.z = (in_row && col + 2 < cols) ? v.z : 0.0f;
    v.w = (in_row && col + 3 < cols) ? v.w : 0.0f;
    return v;
}

// Four consecutive elements of a row of the unfolded input of a convolution, read from the image itself (row = (n, oy, ox),
// col = (c, ky, kx), a multiple of 4): no unfolded copy exists.  Branch-free like the ragged loads above: the address of
// an element outside the matrix or the image is replaced by 0 and the value by zero.
__device__ __forceinline__ float4 ste_load4_unfolded(const float *__restrict__ x, int row, int col, int rows, int cols, const SteConvGeo &g) {
    const uint32_t m = (uint32_t)min(row, rows - 1);
    const uint32_t n = g.dHoWo.div(m), pix = m - n * (uint32_t)(g.Ho * g.Wo);
    const int oy = (int)g.dWo.div(pix), ox = (int)pix - oy * g.Wo;
    const int y0 = oy * g.sh - g.ph, x0 = ox * g.sw - g.pw;
    float v[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t k = (uint32_t)min(col + q, cols - 1);
        const uint32_t c = g.dkhkw.div(k), tap = k - c * (uint32_t)(g.kh * g.kw);
        const int ky = (int)g.dkw.div(tap), kx = (int)tap - ky * g.kw;
        const int iy = y0 + ky * g.dh, ix = x0 + kx * g.dw;
        const bool ok = row < rows && col + q < cols && iy >= 0 && iy < g.H && ix >= 0 && ix < g.W;
        const size_t at = ok ? (((size_t)n * g.C + c) * g.H + iy) * g.W + ix : 0;
        const float t = x[at];
        v[q] = ok ? t : 0.0f;
    }
    return make_float4(v[0], v[1], v[2], v[3]);
}

// TILE x TILE outputs per workgroup (128: four 32 x 32 blocks per wave; 64: one), FULL as above.  Chunks of 32
// contraction indices alternate between two LDS buffers: while the matrix pipe works on one, the next chunk's global
// loads are in flight and are fake-quantised into the other; one barrier per chunk.
// KS = 2: eight waves; waves w and w + 4 share an output quarter and take alternate pairs of contraction indices, their
// sums are added through LDS at the end (a fixed order).  For launches with about one workgroup per compute unit:
// two waves per SIMD, so that one wave's staging arithmetic runs under the other's matrix instructions.
// UNFOLD: b is an image tensor that stands for its unfolded matrix (p.im2col; a template parameter so that the plain
// products carry no trace of it: a run-time branch around the loads cost them 10 - 30 %).
template <bool A_T, int TILE, bool FULL, int KS, bool UNFOLD = false>
__global__ __launch_bounds__(STE_THREADS * KS) void ste_gemm_kernel(SteParams p) {
    constexpr int THREADS = STE_THREADS * KS;
    constexpr int LDB = TILE + 4;                   // LDS row length in floats: 16-byte rows, shifted by 4 banks per row
    constexpr int LDA = A_T ? TILE + 4 : TILE + 1;  // written element by element when the tile arrives transposed
    constexpr int PASSES = TILE * STE_TR / 4 / THREADS;     // staging passes of THREADS x 4 floats over a 32 x TILE chunk
    constexpr int TPR = TILE / 4;                   // threads per staged row
    constexpr int RPP = THREADS / TPR;              // rows per pass
    constexpr int IPP = THREADS / 8;                // rows of a transposed tile per pass
    constexpr int WT = TILE / 2, NB = WT / 32;
    __shared__ __align__(16) float As[2][STE_TR][LDA];      // [r][i]
    __shared__ __align__(16) float Bs[2][STE_TR][LDB];      // [r][j]
    const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) & 3, kh = tid >> 8;
    const int i0 = blockIdx.y * TILE, j0 = blockIdx.x * TILE;
    const int wi = (wave & 1) * WT, wj = (wave >> 1) * WT;

    f32x16_t acc[NB][NB];
#pragma unroll
    for (int bi = 0; bi < NB; ++bi)
#pragma unroll
        for (int bj = 0; bj < NB; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0.0f;

    float4 ra[PASSES], rb[PASSES];
    auto fetch = [&](int r0) {
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
            const int r = tid / TPR + RPP * pass, c4 = (tid % TPR) * 4;
            if constexpr (UNFOLD) rb[pass] = ste_load4_unfolded(p.b, r0 + r, j0 + c4, p.R, p.J, p.g);
            else rb[pass] = ste_load4<FULL>(p.b, r0 + r, j0 + c4, p.R, p.J, p.J);
            if (A_T) {
                ra[pass] = ste_load4<FULL>(p.a, r0 + r, i0 + c4, p.R, p.I, p.lda);
            } else {
                const int i = (tid >> 3) + IPP * pass, r4 = (tid & 7) * 4;
                ra[pass] = ste_load4<FULL>(p.a, i0 + i, r0 + r4, p.I, p.R, p.lda);
            }
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int pass = 0; pass < PASSES; ++pass) {
            const int r = tid / TPR + RPP * pass, c4 = (tid % TPR) * 4;
            float4 q;
            q.x = ste_fake_quant(rb[pass].x, p.sb, p.Q);
            q.y = ste_fake_quant(rb[pass].y, p.sb, p.Q);
            q.z = ste_fake_quant(rb[pass].z, p.sb, p.Q);
            q.w = ste_fake_quant(rb[pass].w, p.sb, p.Q);
            *reinterpret_cast<float4 *>(&Bs[buf][r][c4]) = q;
            if (A_T) {
                *reinterpret_cast<float4 *>(&As[buf][r][c4]) = ra[pass];
            } else {                                        // the tile arrives with r contiguous: transposed on the way in
                const int i = (tid >> 3) + IPP * pass, r4 = (tid & 7) * 4;
                As[buf][r4 + 0][i] = ra[pass].x;
                As[buf][r4 + 1][i] = ra[pass].y;
                As[buf][r4 + 2][i] = ra[pass].z;
                As[buf][r4 + 3][i] = ra[pass].w;
            }
        }
    };

    // this workgroup's share of the contraction (only the products over an unfolded input are ever split over grid z)
    const int ch0 = UNFOLD ? blockIdx.z * p.cps : 0;
    const int chunks = UNFOLD ? max(0, min((p.R + STE_TR - 1) / STE_TR, ch0 + p.cps) - ch0) : (p.R + STE_TR - 1) / STE_TR;
    float *const cout = UNFOLD ? p.c + (size_t)blockIdx.z * (size_t)p.I * (size_t)p.J : p.c;
    if (chunks > 0) { fetch(ch0 * STE_TR); stash(0); }
    __syncthreads();
    for (int ch = 0; ch < chunks; ++ch) {
        const int cur = ch & 1;
        const bool more = ch + 1 < chunks;
        if (more) fetch((ch0 + ch + 1) * STE_TR);
        // one instruction: lane l supplies A(i = l % 32, k = l / 32) and B(k = l / 32, j = l % 32)
        const int kr = lane >> 5, c = lane & 31;
        // all operands of the chunk are requested before its first matrix instruction: one LDS latency per chunk
        float av[STE_TR / 2 / KS][NB], bv[STE_TR / 2 / KS][NB];
#pragma unroll
        for (int k2 = 0; k2 < STE_TR / 2 / KS; ++k2)
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                av[k2][q] = As[cur][2 * (KS * k2 + kh) + kr][wi + 32 * q + c];
                bv[k2][q] = Bs[cur][2 * (KS * k2 + kh) + kr][wj + 32 * q + c];
            }
        __builtin_amdgcn_sched_barrier(0);          // (the scheduler would otherwise sink each read to its use)
#pragma unroll
        for (int k2 = 0; k2 < STE_TR / 2 / KS; ++k2)
#pragma unroll
            for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                for (int bj = 0; bj < NB; ++bj)
                    acc[bi][bj] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[k2][bi], bv[k2][bj], acc[bi][bj], 0, 0, 0);
        if (more) stash(cur ^ 1);           // the other buffer: every wave left it before the previous barrier
        __syncthreads();
    }

    if (KS == 2) {          // (the loop ended with a barrier: the staging buffers are free, but this has its own)
        __shared__ float red[KS == 2 ? 4 * NB * NB * 16 * 64 : 1];
        if (kh == 1) {
#pragma unroll
            for (int bi = 0; bi < NB; ++bi)
#pragma unroll
                for (int bj = 0; bj < NB; ++bj)
#pragma unroll
                    for (int v = 0; v < 16; ++v) red[((wave * NB * NB + bi * NB + bj) * 16 + v) * 64 + lane] = acc[bi][bj][v];
        }
        __syncthreads();
        if (kh == 1) return;
#pragma unroll
        for (int bi = 0; bi < NB; ++bi)
#pragma unroll
            for (int bj = 0; bj < NB; ++bj)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[bi][bj][v] += red[((wave * NB * NB + bi * NB + bj) * 16 + v) * 64 + lane];
    }

    // register v of lane l holds row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of a 32 x 32 block
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) {
#pragma unroll
        for (int bj = 0; bj < NB; ++bj) {
            const int j = j0 + wj + 32 * bj + (lane & 31);
            float ov[16];                   // the mask's operand first, all 16 requests together (c and o never overlap)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + wi + 32 * bi + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                ov[v] = (p.o && (FULL || (i < p.I && j < p.J))) ? p.o[(size_t)i * (size_t)p.J + (size_t)j] : 0.0f;
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + wi + 32 * bi + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (FULL || (i < p.I && j < p.J))
                    cout[(size_t)i * (size_t)p.J + (size_t)j] = (!p.o || ste_inside(ov[v], p.so, p.Q)) ? acc[bi][bj][v] : 0.0f;
            }
        }
    }
}

// c[i] = inside(o[i]) * (part[0][i] + part[1][i] + ... + part[S-1][i]), in that order: the partial sums of a product whose
// contraction was split over grid z
__global__ __launch_bounds__(256) void ste_reduce_masked_kernel(const float *__restrict__ part, int S, size_t n, const float *__restrict__ o,
                                                                float so, float Q, float *__restrict__ c) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        float s = part[i];
        for (int z = 1; z < S; ++z) s += part[(size_t)z * n + i];
        c[i] = (!o || ste_inside(o[i], so, Q)) ? s : 0.0f;
    }
}

// part[z][o] = sum over the images n = z, z + Z, ... and all pixels of dy[n][o][pix] from the NCHW tensor (grid: O x Z
// workgroups; every thread a strided share in ascending order, then a fixed tree); ste_reduce_masked_kernel adds the Z parts
__global__ __launch_bounds__(256) void ste_bias_grad_nchw_kernel(const float *__restrict__ dy, float *__restrict__ db, int N, int O, int P) {
    __shared__ float part[256];
    const int o = blockIdx.x;
    float s = 0.0f;
    for (int n = blockIdx.y; n < N; n += gridDim.y) {
        const float *q = dy + ((size_t)n * O + o) * (size_t)P;
        for (int e = threadIdx.x; e < P; e += 256) s += q[e];
    }
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) db[(size_t)blockIdx.y * O + o] = part[0];
}

// db[n] = sum_m dy[m][n]: 32 columns per workgroup, 32 threads per column take every 32nd row with four running sums
// each; fixed order, so the result does not depend on the launch
constexpr int STE_COLSUM_THREADS = 1024;
__global__ __launch_bounds__(STE_COLSUM_THREADS) void ste_colsum_kernel(const float *__restrict__ dy, float *__restrict__ db, int M, int N) {
    __shared__ float part[32][33];
    const int c = threadIdx.x & 31, ph = threadIdx.x >> 5;
    const int n = blockIdx.x * 32 + c;
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
    if (n < N) {
        const float *q = dy + n;
        int m = ph;
        for (; m + 96 < M; m += 128) {
            s0 += q[(size_t)m * (size_t)N];
            s1 += q[(size_t)(m + 32) * (size_t)N];
            s2 += q[(size_t)(m + 64) * (size_t)N];
            s3 += q[(size_t)(m + 96) * (size_t)N];
        }
        for (; m < M; m += 32) s0 += q[(size_t)m * (size_t)N];
    }
    part[ph][c] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    if (ph == 0 && n < N) {
        float t = part[0][c];
#pragma unroll
        for (int q = 1; q < 32; ++q) t += part[q][c];
        db[n] = t;
    }
}

// ---- convolution (groups = 1): the same two products over the unfolded input --------------------------------------
// y[m][o] = sum_k col(x^)[m][k] * w^[o][k] with m = (n, oy, ox), k = (c, ky, kx) (Sec. III-B: the convolution as a matrix
// product over the unfolded input), so dw = mask(w) . dy_rows^T . fq(col(x)) and dcol = dy_rows . fq(w), and dx gathers
// dcol back onto the image (a fixed order) under mask(x).  col(x) is never written: the product reads it from the image
// (ste_load4_unfolded); dy as rows, dcol and the partial sums live in a workspace of the caller.
// dy [N][O][P] -> rows [N * P][O]
template <typename Idx>
__global__ __launch_bounds__(256) void ste_rows_from_nchw_kernel(const float *__restrict__ dy, float *__restrict__ rows, SteConvGeo g, size_t total) {
    const Idx stride = (Idx)gridDim.x * 256;
    const int O = g.O, P = g.Ho * g.Wo;
    for (Idx i = (Idx)blockIdx.x * 256 + threadIdx.x; i < (Idx)total; i += stride) {
        const Idx m = ste_div<Idx>(i, g.dO), o = i - m * (Idx)O, n = ste_div<Idx>(m, g.dP), pix = m - n * (Idx)P;
        rows[i] = dy[((size_t)n * O + o) * P + pix];
    }
}

// w [O][C][T] -> wp [O][T][C] (T = kh kw taps): with the channel last in dcol's columns, the lanes of the gather kernel
// below, which run along channels, read consecutive floats
__global__ __launch_bounds__(256) void ste_taps_first_kernel(const float *__restrict__ w, float *__restrict__ wp, int O, int C, int T) {
    const size_t total = (size_t)O * C * T, stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < total; i += stride) {
        const size_t o = i / ((size_t)C * T), rem = i - o * (size_t)C * T, t = rem / C, c = rem - t * C;
        wp[i] = w[(o * C + c) * T + t];
    }
}

// dx[n][c][iy][ix] = inside(x) * sum over the taps (ky, kx ascending) that land on (iy, ix) of dcol[(n, oy, ox)][(ky, kx, c)]
template <typename Idx>
__global__ __launch_bounds__(256) void ste_col2im_kernel(const float *__restrict__ dcol, const float *__restrict__ x, float *__restrict__ dx,
                                                         SteConvGeo g, float s_x, float Q, size_t total) {
    const Idx stride = (Idx)gridDim.x * 256;
    const size_t K = (size_t)g.C * g.kh * g.kw;
    for (Idx i = (Idx)blockIdx.x * 256 + threadIdx.x; i < (Idx)total; i += stride) {
        // neighbouring lanes take neighbouring channels of one pixel: their reads of dcol are consecutive floats of one
        // row; the one store and the one read of x per lane are the strided side
        const Idx pixel = ste_div<Idx>(i, g.dC);
        const int c = (int)(i - pixel * (Idx)g.C);
        const Idx n = ste_div<Idx>(pixel, g.dHW);
        const int pin = (int)(pixel - n * (Idx)(g.H * g.W));
        const int iy = (int)g.dW.div((uint32_t)pin), ix = pin - iy * g.W;
        const size_t at = (((size_t)n * g.C + c) * g.H + iy) * g.W + ix;
        float s = 0.0f;
        for (int ky = 0; ky < g.kh; ++ky) {
            const int ty = iy + g.ph - ky * g.dh;
            if (ty < 0) continue;
            const int oy = (int)g.dsh.div((uint32_t)ty);
            if (oy * g.sh != ty || oy >= g.Ho) continue;
            for (int kx = 0; kx < g.kw; ++kx) {
                const int tx = ix + g.pw - kx * g.dw;
                if (tx < 0) continue;
                const int ox = (int)g.dsw.div((uint32_t)tx);
                if (ox * g.sw != tx || ox >= g.Wo) continue;
                s += dcol[(((size_t)n * g.Ho + oy) * g.Wo + ox) * K + (size_t)(ky * g.kw + kx) * g.C + c];
            }
        }
        dx[at] = ste_inside(x[at], s_x, Q) ? s : 0.0f;
    }
}

}  // namespace adapt
