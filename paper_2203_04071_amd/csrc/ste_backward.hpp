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

namespace adapt {

typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int STE_TILE = 128;       // output tile of a workgroup: 128 x 128, one 64 x 64 quarter per wave
constexpr int STE_TR = 16;          // contraction indices per staged chunk
constexpr int STE_LD = 132;         // LDS row length in floats (16-byte rows, shifted by 4 banks per row)
constexpr int STE_THREADS = 256;

// c[i][j] = inside(o[i][j]) * sum_r A(i, r) * fq(b[r][j])
struct SteParams {
    const float *a;     // A_T: element (i, r) at a[r * lda + i]; else at a[i * lda + r]
    const float *b;     // [R][J], fake-quantised with scale sb while it is staged
    const float *o;     // [I][J], decides the clip mask with scale so
    float *c;           // [I][J]
    int I, J, R, lda;
    float sb, so, Q;
    int vec_a, vec_b;   // 16-byte loads allowed (aligned base, row length a multiple of 4)
};

__device__ __forceinline__ float ste_fake_quant(float x, float s, float Q) {
    float r = rintf(x / s);         // IEEE divide, round half to even: the forward quantiser's decision
    if (r != r) r = 0.0f;
    if (r > Q) r = Q;
    if (r < -Q) r = -Q;
    return r * s;
}

__device__ __forceinline__ bool ste_inside(float x, float s, float Q) { return fabsf(rintf(x / s)) <= Q; }     // NaN: false

// four consecutive elements of a row-major matrix, zero outside it (col is a multiple of 4)
__device__ __forceinline__ float4 ste_load4(const float *__restrict__ base, int row, int col, int rows, int cols, int ld, int vec) {
    float4 v = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (row < rows && col < cols) {
        const float *q = base + (size_t)row * (size_t)ld + (size_t)col;
        if (vec && col + 3 < cols) {
            v = *reinterpret_cast<const float4 *>(q);
        } else {
            v.x = q[0];
            if (col + 1 < cols) v.y = q[1];
            if (col + 2 < cols) v.z = q[2];
            if (col + 3 < cols) v.w = q[3];
        }
    }
    return v;
}

template <bool A_T>
__global__ __launch_bounds__(STE_THREADS) void ste_gemm_kernel(SteParams p) {
    __shared__ __align__(16) float As[STE_TR][STE_LD];      // [r][i]
    __shared__ __align__(16) float Bs[STE_TR][STE_LD];      // [r][j]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int i0 = blockIdx.y * STE_TILE, j0 = blockIdx.x * STE_TILE;
    const int wi = (wave & 1) * 64, wj = (wave >> 1) * 64;

    f32x16_t acc[2][2];
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0.0f;

    float4 ra[2], rb[2];
    auto fetch = [&](int r0) {
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int r = (tid >> 5) + 8 * pass, c4 = (tid & 31) * 4;
            rb[pass] = ste_load4(p.b, r0 + r, j0 + c4, p.R, p.J, p.J, p.vec_b);
            if (A_T) {
                ra[pass] = ste_load4(p.a, r0 + r, i0 + c4, p.R, p.I, p.lda, p.vec_a);
            } else {
                const int i = (tid >> 2) + 64 * pass, r4 = (tid & 3) * 4;
                ra[pass] = ste_load4(p.a, i0 + i, r0 + r4, p.I, p.R, p.lda, p.vec_a);
            }
        }
    };
    auto stash = [&]() {
#pragma unroll
        for (int pass = 0; pass < 2; ++pass) {
            const int r = (tid >> 5) + 8 * pass, c4 = (tid & 31) * 4;
            float4 q;
            q.x = ste_fake_quant(rb[pass].x, p.sb, p.Q);
            q.y = ste_fake_quant(rb[pass].y, p.sb, p.Q);
            q.z = ste_fake_quant(rb[pass].z, p.sb, p.Q);
            q.w = ste_fake_quant(rb[pass].w, p.sb, p.Q);
            *reinterpret_cast<float4 *>(&Bs[r][c4]) = q;
            if (A_T) {
                *reinterpret_cast<float4 *>(&As[r][c4]) = ra[pass];
            } else {                                        // the tile arrives with r contiguous: transposed on the way in
                const int i = (tid >> 2) + 64 * pass, r4 = (tid & 3) * 4;
                As[r4 + 0][i] = ra[pass].x;
                As[r4 + 1][i] = ra[pass].y;
                As[r4 + 2][i] = ra[pass].z;
                As[r4 + 3][i] = ra[pass].w;
            }
        }
    };

    fetch(0);
    for (int r0 = 0; r0 < p.R; r0 += STE_TR) {
        __syncthreads();                    // every wave has finished reading the previous chunk
        stash();
        __syncthreads();
        if (r0 + STE_TR < p.R) fetch(r0 + STE_TR);          // in flight while this chunk is multiplied
        // one instruction: lane l supplies A(i = l % 32, k = l / 32) and B(k = l / 32, j = l % 32)
        const int kr = lane >> 5, c = lane & 31;
#pragma unroll
        for (int k = 0; k < STE_TR; k += 2) {
            const float a0 = As[k + kr][wi + c], a1 = As[k + kr][wi + 32 + c];
            const float b0 = Bs[k + kr][wj + c], b1 = Bs[k + kr][wj + 32 + c];
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
        }
    }

    // register v of lane l holds row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of a 32 x 32 block
#pragma unroll
    for (int bi = 0; bi < 2; ++bi) {
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) {
            const int j = j0 + wj + 32 * bj + (lane & 31);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = i0 + wi + 32 * bi + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (i < p.I && j < p.J) {
                    const size_t at = (size_t)i * (size_t)p.J + (size_t)j;
                    p.c[at] = ste_inside(p.o[at], p.so, p.Q) ? acc[bi][bj][v] : 0.0f;
                }
            }
        }
    }
}

// db[n] = sum_m dy[m][n]: 32 columns per workgroup, 8 threads per column take every eighth row, fixed order
__global__ __launch_bounds__(STE_THREADS) void ste_colsum_kernel(const float *__restrict__ dy, float *__restrict__ db, int M, int N) {
    __shared__ float part[8][32];
    const int c = threadIdx.x & 31, ph = threadIdx.x >> 5;
    const int n = blockIdx.x * 32 + c;
    float s = 0.0f;
    if (n < N)
        for (int m = ph; m < M; m += 8) s += dy[(size_t)m * (size_t)N + (size_t)n];
    part[ph][c] = s;
    __syncthreads();
    if (ph == 0 && n < N) {
        float t = part[0][c];
#pragma unroll
        for (int q = 1; q < 8; ++q) t += part[q][c];
        db[n] = t;
    }
}

}  // namespace adapt
