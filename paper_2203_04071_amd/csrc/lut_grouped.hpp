// Grouped convolution with few output channels per group, direct form (Sec. III-B "Convolution Layer": groups;
// the depthwise half of the separable convolution, eq. (1)): every output element is the sum of (Cin / groups) * kh * kw
// table entries T[x][w], each looked up on its own in the table image held in LDS.
//
// The rows kernel shares one activation load among the 8 or 16 output channels a lane accumulates; a depthwise layer has
// ONE output channel per input channel, so there is nothing to share and 7/8 of that kernel's lookups would be padding.
// Here a lane owns one output element at a time (consecutive lanes = consecutive pixels of one output plane, so the
// activation loads of a wave are adjacent bytes and its weight loads are one address), walks its taps, and moves on by
// the size of the grid; the table is staged once per workgroup and serves many planes.
// Padded taps are looked up with activation 0 like everywhere else (they are entries of the expanded input matrix).
#pragma once
#include "lut_rows.hpp"

namespace adapt {

struct GroupedParams {
    const int8_t *x;        // [N][Cin][H][W]
    const int8_t *w;        // [Cout][cg][kh][kw]
    int32_t *out;           // [N][Cout][Ho][Wo]
    const uint16_t *img;    // table image as in RowsParams
    int img_bytes;
    int Cin, H, W, Cout, Ho, Wo, kh, kw;
    int sh, sw, ph, pw, dh, dw;
    int cg, og;             // input / output channels per group
    int hoff, mask, row_bytes;
    int shift;              // < 0: out = acc;  >= 0: out += acc << shift (second half of a split table)
    size_t total;           // N * Cout * Ho * Wo
};

template <bool SIGNED>
__global__ __launch_bounds__(ROWS_THREADS) void lut_grouped_kernel(const GroupedParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    {   // stage the table image
        const uint4 *src = reinterpret_cast<const uint4 *>(p.img);
        uint4 *dst = reinterpret_cast<uint4 *>(smem);
        const int n16 = p.img_bytes >> 4;
        for (int i = threadIdx.x; i < n16; i += ROWS_THREADS) dst[i] = src[i];
    }
    __syncthreads();
    const size_t stride = (size_t)gridDim.x * ROWS_THREADS;
    const int HoWo = p.Ho * p.Wo, taps = p.kh * p.kw;
    const uint32_t zero2 = (uint32_t)p.hoff << 1;           // column of activation 0
    for (size_t o = (size_t)blockIdx.x * ROWS_THREADS + threadIdx.x; o < p.total; o += stride) {
        const size_t plane = o / HoWo;
        const int pix = (int)(o - plane * HoWo);
        const int oy = pix / p.Wo, ox = pix - oy * p.Wo;
        const int n = (int)(plane / p.Cout), co = (int)(plane - (size_t)n * p.Cout);
        const int grp = co / p.og;
        const int8_t *xg = p.x + ((size_t)n * p.Cin + (size_t)grp * p.cg) * p.H * p.W;
        const int8_t *wc = p.w + (size_t)co * p.cg * taps;
        const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
        uint32_t acc = 0;
        for (int ci = 0; ci < p.cg; ++ci) {
            const int8_t *xc = xg + (size_t)ci * p.H * p.W;
            const int8_t *wt = wc + ci * taps;
            for (int ky = 0; ky < p.kh; ++ky) {
                const int iy = iy0 + ky * p.dh;
                const bool yin = (unsigned)iy < (unsigned)p.H;
                for (int kx = 0; kx < p.kw; ++kx) {
                    const int ix = ix0 + kx * p.dw;
                    const bool in = yin && (unsigned)ix < (unsigned)p.W;
                    const uint32_t a2 = in ? (uint32_t)(((int)xc[iy * p.W + ix] + p.hoff) & p.mask) << 1 : zero2;
                    const uint32_t row = (uint32_t)(((int)wt[ky * p.kw + kx] + p.hoff) & p.mask) * (uint32_t)p.row_bytes;
                    acc += lds_entry<SIGNED>(smem, row + a2);
                }
            }
        }
        if (p.shift < 0) p.out[o] = (int32_t)acc;
        else p.out[o] = (int32_t)((uint32_t)p.out[o] + (acc << p.shift));
    }
}

}  // namespace adapt
