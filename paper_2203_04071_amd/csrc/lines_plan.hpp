// How a long-matrix product (derived tables streamed through LDS) is spread over the chip: which kernel, how many rows
// per lane, whether the inner dimension is split over workgroups, and the layout of the activation copy.  Host code only
// (no device calls), so that the decisions can be enumerated without a GPU.
#pragma once

namespace adapt_api {

enum LinesKernel {
    LK_GENERIC = 0,     // lut_lines_kernel: 128-byte lines, any padded channel count
    LK_FAST = 1,        // lut_lines_fast_kernel: 128-byte lines, channel-last copy
    LK_XMAJOR = 2,      // lut_lines_fast_kernel on the x-major copy (8 rows per lane)
    LK_QUAD = 3,        // lut_quad_kernel: 256-byte lines, sums on the matrix pipe, x-major copy
};

struct PlanIn {
    int M;              // rows of the product (transposed convolution: per phase)
    int tiles;          // tiles of 8 output channels x phases
    int k_cc, k_taps;   // the inner dimension as the 128-byte-line kernels walk it: steps of 8 per tap, taps
    int Wo;             // output width (a linear layer is one image row of M pixels: Wo = M)
    int sw;             // horizontal stride of the window
    int quad_steps;     // > 0: quad tables exist for this layer; their steps of 16 inner indices (taps x padded channels / 16)
    int cu;             // compute units
};

struct LinesPlan {
    int kernel;         // LinesKernel
    int R;              // rows per lane (LK_QUAD: per row slot; a workgroup owns 256 R rows, else 128 R)
    int ksplit;         // workgroups that share an output tile, each with a slice of the inner dimension
    int gps;            // slice length: groups of four steps (LK_QUAD: steps)
    int xmajor;         // layout of the activation copy
    int rows_per_wg() const { return (kernel == LK_QUAD ? 256 : 128) * R; }
};

// Quad kernel.  Rows per row slot R: the largest that still gives every compute unit a workgroup, because the table
// bytes streamed per multiply-accumulate fall with R.  When not even the smallest fills the chip, the inner dimension is
// split over up to 16 workgroups of at least four steps each (partial sums, added by reduce_partials_kernel).
// R rows are consecutive pixels of one image row: R = 8 and 4 take runs of four (Wo % 4 == 0), R = 2 pairs.
inline bool quad_rows_ok(int R, int M, int Wo) {
    if (R == 2) return M % 2 == 0 && Wo % 2 == 0;
    return M % R == 0 && Wo % 4 == 0;
}

inline LinesPlan plan_lines(const PlanIn &in) {
    const int M = in.M, cu = in.cu;
    if (in.quad_steps > 0 && in.sw == 1 && (quad_rows_ok(8, M, in.Wo) || quad_rows_ok(4, M, in.Wo) || quad_rows_ok(2, M, in.Wo))) {
        auto wgs = [&](int r) { return (long long)((M + 256 * r - 1) / (256 * r)) * in.tiles; };
        const int Rs[3] = {8, 4, 2};
        for (int R : Rs)
            if (quad_rows_ok(R, M, in.Wo) && wgs(R) >= cu) return LinesPlan{LK_QUAD, R, 1, in.quad_steps, 1};
        for (int R : Rs) {
            if (!quad_rows_ok(R, M, in.Wo)) continue;
            long long ks = (cu + wgs(R) - 1) / wgs(R);
            if (ks > in.quad_steps / 4) ks = in.quad_steps / 4;
            if (ks > 16) ks = 16;
            if (ks >= 2 && wgs(R) * ks * 4 >= 3LL * cu) {
                const int sps = (in.quad_steps + (int)ks - 1) / (int)ks;
                return LinesPlan{LK_QUAD, R, (in.quad_steps + sps - 1) / sps, sps, 1};
            }
        }
        for (int i = 2; i >= 0; --i)
            if (quad_rows_ok(Rs[i], M, in.Wo)) return LinesPlan{LK_QUAD, Rs[i], 1, in.quad_steps, 1};
    }
    // 128-byte-line kernels: rows per lane R (a workgroup handles 128 R rows) as large as still gives every compute unit
    // a workgroup.  When even R = 8 leaves three quarters of them idle and the inner dimension is long enough, keep
    // R = 8 and split the inner dimension over `ksplit` workgroups instead.
    auto wgs = [&](int r) { return (long long)((M + 128 * r - 1) / (128 * r)) * in.tiles; };
    LinesPlan pl{LK_GENERIC, 8, 1, 0, 0};
    const int groups = in.k_cc % 4 == 0 ? in.k_taps * in.k_cc / 4 : 0;     // the split needs the fast kernel
    bool split = false;
    if (wgs(8) * 4 <= cu && groups >= 8) {      // (with half the chip covered, 4 rows per lane does as well)
        int ks = (int)(cu / wgs(8));
        if (ks > groups / 4) ks = groups / 4;                   // at least four groups (16 steps) per slice
        if (ks > 16) ks = 16;
        if (ks >= 2) {
            pl.gps = (groups + ks - 1) / ks;
            pl.ksplit = (groups + pl.gps - 1) / pl.gps;
            split = true;
        }
    }
    if (!split) {
        while (pl.R > 2 && wgs(pl.R) < cu) pl.R /= 2;
        pl.gps = groups > 0 ? groups : 1;
    }
    pl.xmajor = (pl.R == 8 && in.Wo % 4 == 0 && M % 8 == 0 && in.sw == 1 && in.k_cc % 4 == 0) ? 1 : 0;
    pl.kernel = pl.xmajor ? LK_XMAJOR : (in.k_cc % 4 == 0 ? LK_FAST : LK_GENERIC);
    return pl;
}

}  // namespace adapt_api
