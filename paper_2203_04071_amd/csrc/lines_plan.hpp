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
    int bits;           // operand bits (table lines = 2^bits)
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

// Quad kernel.  The R = 8 or 4 rows of a row slot are consecutive pixels of one image row, in runs of four.
inline bool quad_rows_ok(int R, int M, int Wo) { return (R == 8 || R == 4) && M % R == 0 && Wo % 4 == 0; }

// Estimated duration, in clocks, of a quad launch with R rows per row slot; only differences between the candidates
// matter.  From measurements of whole layers on one MI355X (3 x 3 convolutions of 16 to 256 channels, 8-bit tables), per
// step of a workgroup: R = 8 about 4460 clocks when every compute unit has a workgroup and 3770 with half of them busy;
// R = 4 about 2780 - the path that fills LDS and registers (64 KB of table per step whatever R is, plus R x 4 KB of
// activations, at about 26 bytes per clock) bounds both, so the cost per multiply-accumulate falls as R grows, but so
// does the number of workgroups (two rows per row slot were measured too: slower everywhere).  Smaller tables (fewer
// bits) shrink the table part; the LDS reads (32 per lane and step at R = 8) then become the bound.
inline long long quad_step_clocks(int R, int bits, double busy) {
    if (bits >= 8) {
        if (R == 8) return (long long)(3080 + 1380 * busy);
        return (long long)(2280 + 500 * busy);
    }
    const long long lds = R == 8 ? 3040 : 1600;
    const long long fill = (long long)(((256LL << bits) + 4096LL * R) / 26.0);
    return lds > fill ? lds : fill;
}

inline long long quad_cost(int R, int M, int tiles, int steps, int bits, int cu) {
    const long long wgs = (long long)((M + 256 * R - 1) / (256 * R)) * tiles;
    const long long full = wgs / cu, rest = wgs % cu;
    long long c = full * steps * quad_step_clocks(R, bits, 1.0);
    if (rest) c += steps * quad_step_clocks(R, bits, (double)rest / cu);
    return c;
}

// The quad kernel takes a product when its tables exist, the window moves one pixel at a time, the inner dimension has
// at least QUAD_MIN_STEPS steps and some admissible R gives at least three quarters of the compute units a workgroup.
// Measured inside networks (tables arrive cold): 9-step 3 x 3 layers of 16 channels and an 8-step 1 x 1 layer of 128
// channels are 10 - 20 % faster on it than on the 128-byte-line kernels.  Layers that would cover half the compute units
// or less run on it with the inner dimension split over workgroups (the ResNet-style 64-channel 8 x 8 layers as 4 slices
// of 9 steps: 20 us with the kernel that adds the slices, against 27 us on the 128-byte-line kernels; the 32-channel
// layers as 2 slices: a little faster too).  A layer that fills the chip unsplit is never split: 8 rows per row slot
// x 2 slices measured the same as 4 rows unsplit at the benchmark layer, and slower inside the ResNet-style network.
constexpr int QUAD_MIN_STEPS = 4;
constexpr int QUAD_MIN_SLICE_STEPS = 8;

inline LinesPlan plan_lines(const PlanIn &in) {
    const int M = in.M, cu = in.cu;
    if (in.quad_steps >= QUAD_MIN_STEPS && in.sw == 1) {
        LinesPlan best{LK_QUAD, 0, 1, in.quad_steps, 1};
        long long best_cost = 0;
        const int Rs[2] = {8, 4};
        for (int R : Rs) {
            if (!quad_rows_ok(R, M, in.Wo)) continue;
            const long long wgs = (long long)((M + 256 * R - 1) / (256 * R)) * in.tiles;
            if (wgs * 4 < 3LL * cu) continue;
            const long long c = quad_cost(R, M, in.tiles, in.quad_steps, in.bits, cu);
            if (best.R == 0 || c < best_cost) { best.R = R; best_cost = c; }
        }
        if (best.R) return best;
        // No R fills three quarters of the chip.  With half of it or less at 4 rows per row slot, slices of the inner
        // dimension (at least QUAD_MIN_SLICE_STEPS steps each, at most 8 slices) go to workgroups of their own and a second
        // kernel adds the partial sums - if that fills the chip.
        if (quad_rows_ok(4, M, in.Wo)) {
            const long long wgs = (long long)((M + 1023) / 1024) * in.tiles;
            long long ks = cu / wgs;
            if (ks > in.quad_steps / QUAD_MIN_SLICE_STEPS) ks = in.quad_steps / QUAD_MIN_SLICE_STEPS;
            if (ks > 8) ks = 8;
            if (ks >= 2) {
                const int gps = (int)((in.quad_steps + ks - 1) / ks);
                ks = (in.quad_steps + gps - 1) / gps;
                if (ks >= 2 && wgs * ks * 4 >= 3LL * cu) {
                    best.R = 4; best.ksplit = (int)ks; best.gps = gps;
                    return best;
                }
            }
        }
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
