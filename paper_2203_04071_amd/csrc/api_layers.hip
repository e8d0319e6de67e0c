// C ABI, part 2: the table-lookup products (linear, convolution, transposed convolution), packed weights, whole-layer
// calls, chained layers and recurrent time steps.  All arithmetic of the path runs in the kernels included below;
// nothing here falls back to host computation.
#include <mutex>

#include "api_common.hpp"
#include "lut_lines.hpp"
#include "lut_quad.hpp"
#include "lines_plan.hpp"
#include "lut_rows.hpp"
#include "lut_grouped.hpp"

using namespace adapt_api;

namespace {

// Optional fp32 ends of a layer call.
struct LayerIO {
    const float *xf = nullptr;      // fp32 activations, quantised while the activation copy is made (the int8 pointer is unused)
    float s_x = 1.0f, Q = 127.0f;
    int deq = 0;                    // the output buffer receives fp32 y = float(acc) * s_out (+ bias[c]) (act 1: ReLU, 2: tanh)
    int act = 0;
    float s_out = 1.0f;
    const float *s_out_vec = nullptr;   // one output scale per channel instead of s_out
    const float *bias = nullptr;
    const float *resid = nullptr;       // fp32 tensor of the output's shape, added after the bias and before act
    adapt::ChainOut chain{};            // also write the output as the next convolution's quantised input copy (buf != nullptr)
    int chain_wo = 1;                   // width of the output (for the kernels that walk it element by element)
    // rescaling inside the product kernel needs a single table pass and an activation it knows
    bool fused(int storage) const { return deq && storage == 0 && act <= 1 && !chain.buf; }
};

int finish_inplace(int32_t *buf, size_t n, size_t channels, size_t inner, const LayerIO &io, hipStream_t s) {
    adapt::finish_inplace_kernel<<<ew_grid(n), adapt::EW_THREADS, 0, s>>>(buf, n, channels, inner, io.s_out, io.s_out_vec, io.bias, io.resid, io.act,
                                                                          io.chain, io.chain_wo);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

}  // namespace

struct adapt_weights {
    int kind;               // 0 linear, 1 conv2d, 2 transposed conv2d
    int bits, storage, device;
    int N, Cin, kh, kw;     // linear: Cin = K, kh = kw = 1
    int Cp, Cc, n_tiles;    // padded inner length (multiple of 8; linear: of 32), steps per tap, 8-channel tiles
    int pair_g;             // taps per group of four steps when taps are paired (see adapt::LinesParams), else 0
    size_t dt_bytes;        // per table-half (transposed convolution: all phases together)
    uint4 *dt_dev[2];
    // transposed convolution only
    int stride;
    bool phased;            // kh and kw are multiples of the stride: derived tables per phase exist
    int32_t *zsum_dev;      // [Cout][kh * kw] sums of T[0][w] over the input channels
    int8_t *w8_dev;         // copy of the weights for the geometries the phase form does not cover
    const adapt_lut *lut;   // the table handle (must outlive this handle), for those geometries
    mutable Workspace ws;   // padded activation copy of the latest call
    // convolutions: the geometry for which the workspace was prepared to receive its input copy from the layer before
    // (adapt_conv2d_chain_prepare): borders and padded channels zeroed, layout fixed
    mutable struct ChainIn {
        bool valid = false;
        int N = 0, H = 0, W = 0, sh = 0, sw = 0, ph = 0, pw = 0, dh = 0, dw = 0, xmajor = 0;
        // set by the layer that last wrote the copy: it applied ReLU before quantising, so every code is >= 0 and the
        // quad kernel needs only the first half of every table's lines
        bool nonneg = false;
    } chain_in;
    // linear layers only: row offsets [K][wofs_npad] for the whole-table kernel, which serves short activation matrices
    // transposed convolutions: the same for the gather form (wofs_dev, [kh kw Cin][wofs_npad]) and for the single-pixel
    // form, a linear layer with Cout kh kw outputs (wofs1_dev, [Cin][wofs1_npad])
    uint32_t *wofs_dev;
    int wofs_npad;
    uint32_t *wofs1_dev;
    int wofs1_npad;
    // The same derived tables in the quad order (lut_quad.hpp: 256-byte lines, entries as int8 digits of entry - dtq_c),
    // made at pack time for single-pass tables with 16 | padded channels; nullptr otherwise.
    uint4 *dtq_dev;
    int dtq_c;
    size_t dtq_bytes;       // transposed convolution: all phases together
    // linear [G Hs][Hs] handles (G = 4, 3 or 1 gates, even Hs, single-pass table) that can serve recurrent time steps:
    // row offsets with the columns in cell order (see adapt::RowsParams), made at pack time
    uint32_t *wofs_cell_dev;
    int cell_G;
};

/* ------------------------------------------------------------------ table-lookup matrix products */

// Scratch of the entry point that allocates nothing (adapt_approx_linear_noalloc): the row offsets of one call.  One
// array per GPU, part of the loaded code object, held until the process ends.  Host code never uses the array's name as
// an address: noalloc_scratch() asks the runtime for the device address once per device and hands that out.
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)4 << 20;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];

namespace {

int noalloc_scratch(void **out, const char *who) {
    static std::mutex mu;
    static void *ptr[64] = {};
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return fail(ADAPT_ERR_HIP, "%s: hipGetDevice failed", who);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void *p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));    // the current device's copy of the array
        if (e != hipSuccess || !p) return fail(ADAPT_ERR_HIP, "%s: hipGetSymbolAddress(scratch): %s", who, hipGetErrorString(e));
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return ADAPT_OK;
}

template <int NT, bool SIGNED>
int launch_rows_inst(const adapt::RowsParams &p, dim3 grid, size_t lds, hipStream_t s) {
    static std::atomic<size_t> configured{0};   // largest dynamic LDS size announced for this instantiation
    auto kern = adapt::lut_rows_kernel<NT, SIGNED>;
    if (lds > configured.load(std::memory_order_acquire)) {     // (two threads may both announce it: harmless)
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        size_t seen = configured.load(std::memory_order_relaxed);
        while (seen < lds && !configured.compare_exchange_weak(seen, lds, std::memory_order_release)) {}
    }
    kern<<<grid, adapt::ROWS_THREADS, lds, s>>>(p);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

struct Geometry {
    int mode;
    int M, N, Cin, taps, kw;
    int H, W, Wo, HoWo;
    int sh, sw, ph, pw, dh, dw;
    int kstride, img_stride;
    int wt;                 // GEMM mode only: the weights are stored [K][N] instead of [N][K]
    int groups;             // convolution only: 0 or 1 = ordinary; else N and Cin count one group's channels
};

// Run the rows kernel once per table image of the handle.
// prepacked: row offsets [K][prepacked_npad] made earlier by pack_row_offsets_kernel (prepacked_npad a multiple of 16),
// or nullptr to pack `w` into a stream-ordered temporary.
struct LstmStep {            // see adapt::RowsParams
    int kind = 1;            // 1: LSTM, 2: GRU, 3: plain cell
    int relu = 0;            // plain cell: ReLU instead of tanh
    int Hs;
    const int32_t *acc_ih;
    const float *bias;
    const float *bias_hh = nullptr;
    float *c, *h;
    const float *h_prev = nullptr;
    int8_t *qh_next;
    float s_ih, s_hh, s_h, Qh;
};

// pack_into: room for Ktot * (N rounded up to 16) * groups row offsets that the call may use instead of a stream-ordered
// temporary (then it allocates nothing)
int run_rows(const adapt_lut *lut, const int8_t *x, const int8_t *w, int32_t *out, const Geometry &g, hipStream_t s,
             const uint32_t *prepacked = nullptr, int prepacked_npad = 0, const LayerIO *io = nullptr,
             const LstmStep *lstm = nullptr, uint32_t *pack_into = nullptr) {
    const int bits = lut->bits;
    const long long Ktot = (long long)g.taps * g.Cin;
    const int ngroups = g.groups > 1 ? g.groups : 1;
    if (g.M == 0 || g.N == 0) return ADAPT_OK;
    if (Ktot == 0) {
        const size_t n = (size_t)g.M * g.N * ngroups;
        adapt::fill_u32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(reinterpret_cast<uint32_t *>(out), 0u, n);
        HIP_TRY(hipGetLastError());
        return ADAPT_OK;
    }
    // tile shape: prefer 16 outputs per lane; shrink the tile until the grid covers the chip
    const int cu = device_cus();
    int NT = 16, MT = 1024;
    auto wgs = [&](int nt, int mt) { return (long long)((g.M + mt - 1) / mt) * ((g.N + nt - 1) / nt) * ngroups; };
    while (MT > 64 && (MT / 2 >= g.M || (wgs(NT, MT) < cu && Ktot / (adapt::ROWS_THREADS / (MT / 2)) >= 16))) MT /= 2;
    if ((wgs(NT, MT) < cu && g.N > 8) || (ngroups > 1 && g.N <= 8)) NT = 8;
    if (lstm) { NT = lstm->kind == 2 ? 6 : (lstm->kind == 3 ? 2 : 8); MT = 64; }    // the cell epilogue sits in the split-K reduction: all gates of two units
    const int KS = adapt::ROWS_THREADS / MT;
    const int Npad = prepacked ? prepacked_npad : ((g.N + NT - 1) / NT) * NT;

    uint32_t *wofs = nullptr;
    int rc = ADAPT_OK;
    if (!prepacked) {
        if (pack_into) wofs = pack_into;
        else HIP_TRY(dbg_malloc_async((void **)&wofs, (size_t)Ktot * Npad * ngroups * sizeof(uint32_t), s));
        const size_t pack_n = (size_t)Ktot * Npad;
        adapt::pack_row_offsets_kernel<<<dim3((unsigned)((pack_n + 255) / 256), (unsigned)ngroups), 256, 0, s>>>(
            w, wofs, (int)Ktot, g.N, Npad, g.Cin, g.taps, g.wt ? (int)adapt::MODE_CONVT : g.mode, 1 << (bits - 1), (1 << bits) - 1,
            lut->rs * 2);
        hipError_t pe = hipGetLastError();
        if (pe != hipSuccess) rc = fail(ADAPT_ERR_HIP, "pack_row_offsets launch: %s", hipGetErrorString(pe));
    }

    adapt::RowsParams p;
    p.x = x; p.wofs = prepacked ? prepacked : wofs; p.out = out;
    p.img_bytes = lut->img_bytes;
    p.M = g.M; p.N = g.N; p.Npad = Npad; p.out_ch = g.N * ngroups; p.mode = g.mode; p.Cin = g.Cin; p.taps = g.taps; p.kw = g.kw;
    p.H = g.H; p.W = g.W; p.Wo = g.Wo; p.HoWo = g.HoWo;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw; p.dh = g.dh; p.dw = g.dw;
    p.kstride = g.kstride; p.img_stride = g.img_stride;
    p.hoff = 1 << (bits - 1); p.mask = (1 << bits) - 1;
    p.a_zero2 = (1 << (bits - 1)) * 2; p.a_skip2 = (1 << bits) * 2;
    p.MT = MT; p.KS = KS;
    const bool fuse = io && io->fused(lut->storage);
    p.deq = fuse ? 1 : 0; p.act = fuse ? io->act : 0; p.scale = fuse ? io->s_out : 1.0f; p.bias = fuse ? io->bias : nullptr;
    p.scales = fuse ? io->s_out_vec : nullptr;
    p.lstm = lstm ? lstm->kind : 0; p.Hs = 0; p.acc_ih = nullptr; p.c = p.h = nullptr; p.qh_next = nullptr;
    p.h_prev = nullptr; p.bias_hh = nullptr;
    p.s_ih = p.s_hh = p.s_h = p.Qh = 1.0f;
    if (lstm) {
        p.Hs = lstm->Hs; p.acc_ih = lstm->acc_ih; p.bias = lstm->bias; p.c = lstm->c; p.h = lstm->h; p.qh_next = lstm->qh_next;
        p.s_ih = lstm->s_ih; p.s_hh = lstm->s_hh; p.s_h = lstm->s_h; p.Qh = lstm->Qh;
        p.h_prev = lstm->h_prev; p.bias_hh = lstm->bias_hh;
        if (lstm->kind == 3) p.act = lstm->relu ? 1 : 0;
    }
    dim3 grid((unsigned)((g.M + MT - 1) / MT), (unsigned)(Npad / NT), (unsigned)ngroups);
    size_t lds = (size_t)lut->img_bytes;
    if (KS > 1 && (size_t)adapt::ROWS_THREADS * NT * 4 > lds) lds = (size_t)adapt::ROWS_THREADS * NT * 4;
    for (int half = 0; half <= lut->storage && rc == ADAPT_OK; ++half) {
        p.img = lut->img_dev[half];
        p.shift = half == 0 ? -1 : 16;
        const bool sgn = (lut->storage == 0) || half == 1;
        if (NT == 16) rc = sgn ? launch_rows_inst<16, true>(p, grid, lds, s) : launch_rows_inst<16, false>(p, grid, lds, s);
        else if (NT == 6) rc = launch_rows_inst<6, true>(p, grid, lds, s);      // (GRU step: single-pass tables only)
        else if (NT == 2) rc = launch_rows_inst<2, true>(p, grid, lds, s);      // (plain recurrent step, likewise)
        else rc = sgn ? launch_rows_inst<8, true>(p, grid, lds, s) : launch_rows_inst<8, false>(p, grid, lds, s);
    }
    if (wofs && !pack_into) {
        hipError_t fe = hipFreeAsync(wofs, s);
        if (rc == ADAPT_OK && fe != hipSuccess) rc = fail(ADAPT_ERR_HIP, "hipFreeAsync: %s", hipGetErrorString(fe));
    }
    if (rc == ADAPT_OK && io && io->deq && !fuse) {
        const size_t inner = g.mode == adapt::MODE_GEMM ? 1 : (size_t)g.HoWo;
        rc = finish_inplace(out, (size_t)g.M * g.N * ngroups, (size_t)g.N * ngroups, inner, *io, s);
    }
    return rc;
}


// Grouped convolution with fewer than 8 output channels per group (depthwise and its relatives): direct form
// io: whole-layer form (fp32 activations in, rescaled fp32 / chained output): only the tiled kernel has it, so the call is
// refused with ADAPT_ERR_UNSUPPORTED when the shape does not take that kernel
int run_grouped(const adapt_lut *lut, const int8_t *x, const int8_t *w, int32_t *out, int N, int Cin, int H, int W, int Cout, int Ho,
                int Wo, int kh, int kw, int sh, int sw, int ph, int pw, int dh, int dw, int groups, hipStream_t s,
                const LayerIO *io = nullptr) {
    adapt::GroupedParams p;
    p.x = x; p.w = w; p.out = out; p.img_bytes = lut->img_bytes;
    p.xf = io ? io->xf : nullptr; p.qscale = io ? io->s_x : 1.0f; p.qQ = io ? io->Q : 1.0f;
    p.deq = io ? io->deq : 0; p.act = io ? io->act : 0; p.scale = io ? io->s_out : 1.0f;
    p.scales = io ? io->s_out_vec : nullptr; p.bias = io ? io->bias : nullptr;
    p.chain = io ? io->chain : adapt::ChainOut{};
    p.Cin = Cin; p.H = H; p.W = W; p.Cout = Cout; p.Ho = Ho; p.Wo = Wo; p.kh = kh; p.kw = kw;
    p.sh = sh; p.sw = sw; p.ph = ph; p.pw = pw; p.dh = dh; p.dw = dw;
    p.cg = Cin / groups; p.og = Cout / groups;
    p.hoff = 1 << (lut->bits - 1); p.mask = (1 << lut->bits) - 1; p.row_bytes = lut->rs * 2;
    p.total = (size_t)N * Cout * Ho * Wo;
    if (!p.total) return ADAPT_OK;
    const int cu = device_cus();
    // tiled form: the input region of a tile and the tap words of its groups sit in LDS next to the table
    const int taps = kh * kw;
    long long Wr = (long long)(Wo - 1) * sw + (long long)(kw - 1) * dw + 1;
    // strips of four output pixels (see the kernel): filter widths and strides it is instantiated for; the region rows
    // then cover whole strips and are a multiple of 4 bytes wide
    int variant = 0;
    if (dw == 1 && (kw == 3 || kw == 5) && (sw == 1 || sw == 2) && lut->img_bytes % 4 == 0) {
        variant = (kw == 3 ? 1 : 2) + (sw == 2 ? 2 : 0);
        const long long Wo4 = (Wo + 3) / 4;
        Wr = ((4 * Wo4 - 1) * sw + kw + 3) / 4 * 4;
    }
    const long long rows_min = (long long)(kh - 1) * dh + 1;
    const long long cap = (long long)adapt::GROUPED_PF * adapt::ROWS_THREADS;
    if (variant && p.cg * rows_min * Wr > cap) {        // the wider rows do not fit: pixel by pixel
        variant = 0;
        Wr = (long long)(Wo - 1) * sw + (long long)(kw - 1) * dw + 1;
    }
    const long long wgroup = (long long)p.og * p.cg * taps;             // tap words of one group
    const size_t wl_bytes = (size_t)adapt::ROWS_THREADS * 4;
    const bool tiled = wgroup <= adapt::ROWS_THREADS && p.cg * rows_min * Wr <= cap &&
                       (size_t)lut->img_bytes + wl_bytes + (size_t)cap <= 160 * 1024;
    size_t blocks, lds;
    if (io && (!tiled || lut->storage != 0))
        return fail(ADAPT_ERR_UNSUPPORTED, "grouped layer call: this shape or table does not take the tiled kernel");
    if (tiled) {
        // rows per tile: as many as the region buffer holds for one group; then as many groups as still fit; both
        // reduced again while the tiles would not cover the chip twice
        long long ro = (cap / ((long long)p.cg * Wr) - rows_min) / sh + 1;
        if (ro > Ho) ro = Ho;
        auto rows_in = [&](long long r) { return (r - 1) * sh + rows_min; };
        long long gt = cap / ((long long)p.cg * rows_in(ro) * Wr);
        if (gt > adapt::ROWS_THREADS / wgroup) gt = adapt::ROWS_THREADS / wgroup;
        if (gt > groups) gt = groups;
        if (gt < 1) gt = 1;
        auto tiles = [&](long long r, long long g) { return (long long)N * ((groups + g - 1) / g) * ((Ho + r - 1) / r); };
        while (gt > 1 && tiles(ro, gt) < 2LL * cu) gt = (gt + 1) / 2;
        while (ro > 1 && tiles(ro, gt) < 2LL * cu) ro = (ro + 1) / 2;
        // a tile whose channels are whole quads writes the next layer's copy a word at a time
        const long long quad = p.og % 4 == 0 ? 1 : (p.og % 2 == 0 ? 2 : 4);
        if (p.chain.buf && gt > quad) gt -= gt % quad;
        if (tiles(ro, gt) > 0x7fffffffLL) return fail(ADAPT_ERR_UNSUPPORTED, "adapt_approx_conv2d: too many tiles");
        p.gt = (int)gt;
        {
            // work items of (channel slot, pixel): enough slots that a tile has work for every lane
            const long long chans = gt * p.og, npix = ro * Wo;
            long long cpl = npix >= adapt::ROWS_THREADS ? chans : chans * npix / adapt::ROWS_THREADS;
            if (cpl < 1) cpl = 1;
            if (p.chain.buf && chans % 4 == 0) cpl = cpl < 4 ? 4 : cpl / 4 * 4;
            p.cpl = (int)cpl;
        }
        p.chain4 = p.chain.buf && (gt * p.og) % 4 == 0 && p.chain.Cp % 4 == 0;
        p.ro = (int)ro; p.n_chunks = (int)((Ho + ro - 1) / ro);
        p.rows_in = (int)rows_in(ro); p.Wr = (int)Wr;
        p.tile_elems = (int)gt * p.cg * p.rows_in * p.Wr;
        p.wl_bytes = (int)wl_bytes;
        p.ntiles = (int)tiles(ro, gt);
        {
            const int K = p.cg * taps, Wo4 = (Wo + 3) / 4;
            p.d_plane_in = fast_div((uint32_t)(p.rows_in * p.Wr)); p.d_Wr = fast_div((uint32_t)p.Wr);
            p.d_ogK = fast_div((uint32_t)(p.og * K)); p.d_K = fast_div((uint32_t)K); p.d_taps = fast_div((uint32_t)taps);
            p.d_kw = fast_div((uint32_t)kw);
            p.d_npix = fast_div((uint32_t)(p.ro * Wo)); p.d_Wo = fast_div((uint32_t)Wo);
            p.d_nstrip = fast_div((uint32_t)(p.ro * Wo4)); p.d_Wo4 = fast_div((uint32_t)Wo4);
        }
        blocks = (size_t)p.ntiles < (size_t)cu ? (size_t)p.ntiles : (size_t)cu;
        lds = (size_t)lut->img_bytes + wl_bytes + (size_t)((p.tile_elems + 15) / 16 * 16);
    } else {
        // one workgroup per compute unit at most (the table image fills its LDS), fewer when there is little to do
        p.chain4 = 0; p.cpl = 1;
        p.d_plane_in = p.d_Wr = p.d_ogK = p.d_K = p.d_taps = p.d_kw = p.d_npix = p.d_Wo = p.d_nstrip = p.d_Wo4 = fast_div(1u);
        p.gt = p.ro = p.n_chunks = p.rows_in = p.Wr = p.tile_elems = p.wl_bytes = p.ntiles = 0;
        blocks = (p.total + adapt::ROWS_THREADS * 4 - 1) / (adapt::ROWS_THREADS * 4);
        if (blocks > (size_t)cu) blocks = (size_t)cu;
        lds = (size_t)lut->img_bytes;
    }
    if (!tiled) variant = 0;
    using kern_t = void (*)(const adapt::GroupedParams);
    static const kern_t tiled_kernels[5][2] = {
        {adapt::lut_grouped_tiled_kernel<false, 0, 1>, adapt::lut_grouped_tiled_kernel<true, 0, 1>},
        {adapt::lut_grouped_tiled_kernel<false, 3, 1>, adapt::lut_grouped_tiled_kernel<true, 3, 1>},
        {adapt::lut_grouped_tiled_kernel<false, 5, 1>, adapt::lut_grouped_tiled_kernel<true, 5, 1>},
        {adapt::lut_grouped_tiled_kernel<false, 3, 2>, adapt::lut_grouped_tiled_kernel<true, 3, 2>},
        {adapt::lut_grouped_tiled_kernel<false, 5, 2>, adapt::lut_grouped_tiled_kernel<true, 5, 2>},
    };
    static std::atomic<size_t> configured[6][2];
    for (int half = 0; half <= lut->storage; ++half) {
        p.img = lut->img_dev[half];
        p.shift = half == 0 ? -1 : 16;
        const bool sgn = (lut->storage == 0) || half == 1;
        const kern_t kern = tiled ? tiled_kernels[variant][sgn] : (sgn ? adapt::lut_grouped_kernel<true> : adapt::lut_grouped_kernel<false>);
        const int slot = tiled ? variant : 5;
        if (lds > configured[slot][sgn].load(std::memory_order_acquire)) {
            HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
            size_t seen = configured[slot][sgn].load(std::memory_order_relaxed);
            while (seen < lds && !configured[slot][sgn].compare_exchange_weak(seen, lds, std::memory_order_release)) {}
        }
        kern<<<(unsigned)blocks, adapt::ROWS_THREADS, lds, s>>>(p);
        HIP_TRY(hipGetLastError());
    }
    return ADAPT_OK;
}


/* ---- "lines" path: derived tables streamed through LDS (long matrices) ---- */

template <int R, bool SIGNED, bool REGULAR>
int launch_lines_inst(const adapt::LinesParams &p, unsigned grid, hipStream_t s) {
    adapt::lut_lines_kernel<R, SIGNED, REGULAR><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

template <int R, bool SIGNED, bool REGULAR>
int launch_lines_fast(const adapt::LinesParams &p, unsigned grid, hipStream_t s) {
    if constexpr (SIGNED) {
        if (p.pair_g) {     // tap pairing exists for single-pass (signed) tables only
            if (p.copy_lines == 256) adapt::lut_lines_fast_kernel<R, true, REGULAR, true, false, true><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
            else adapt::lut_lines_fast_kernel<R, true, REGULAR, false, false, true><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
            HIP_TRY(hipGetLastError());
            return ADAPT_OK;
        }
    }
    if (p.copy_lines == 256) adapt::lut_lines_fast_kernel<R, SIGNED, REGULAR, true, false><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
    else adapt::lut_lines_fast_kernel<R, SIGNED, REGULAR, false, false><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

// x-major activation copy: 8 regular rows per lane
template <bool SIGNED>
int launch_lines_xmajor(const adapt::LinesParams &p, unsigned grid, hipStream_t s) {
    if constexpr (SIGNED) {
        if (p.pair_g) {
            if (p.copy_lines == 256) adapt::lut_lines_fast_kernel<8, true, true, true, true, true><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
            else adapt::lut_lines_fast_kernel<8, true, true, false, true, true><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
            HIP_TRY(hipGetLastError());
            return ADAPT_OK;
        }
    }
    if (p.copy_lines == 256) adapt::lut_lines_fast_kernel<8, SIGNED, true, true, true><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
    else adapt::lut_lines_fast_kernel<8, SIGNED, true, false, true><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

// quad kernel (x-major copy, single-pass tables as int8 digits); extra: the instantiation whose epilogue also takes the
// border terms of a transposed convolution off, knows tanh and writes the next layer's input copy
template <int DOPS, int R>
int launch_quad_inst(const adapt::LinesParams &p, unsigned grid, bool extra, hipStream_t s) {
    if (extra) adapt::lut_quad_kernel<DOPS, R, true><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
    else adapt::lut_quad_kernel<DOPS, R, false><<<grid, adapt::LINES_THREADS, 0, s>>>(p);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

template <int R>
int launch_quad_r(const adapt::LinesParams &p, unsigned grid, bool extra, hipStream_t s) {
    if (p.copy_lines == 256) return launch_quad_inst<4, R>(p, grid, extra, s);
    if (p.copy_lines == 128) return launch_quad_inst<2, R>(p, grid, extra, s);
    return launch_quad_inst<1, R>(p, grid, extra, s);
}

int launch_quad(const adapt::LinesParams &p, unsigned grid, int R, bool extra, hipStream_t s) {
    if (R == 8) return launch_quad_r<8>(p, grid, extra, s);
    return launch_quad_r<4>(p, grid, extra, s);
}

template <int R>
int launch_lines_r(const adapt::LinesParams &p, unsigned grid, bool sgn, bool regular, hipStream_t s) {
    if (p.Cc % 4 == 0) {       // groups of four steps never straddle a filter tap: fully unrolled variant
        if (regular) return sgn ? launch_lines_fast<R, true, true>(p, grid, s) : launch_lines_fast<R, false, true>(p, grid, s);
        return sgn ? launch_lines_fast<R, true, false>(p, grid, s) : launch_lines_fast<R, false, false>(p, grid, s);
    }
    if (regular) return sgn ? launch_lines_inst<R, true, true>(p, grid, s) : launch_lines_inst<R, false, true>(p, grid, s);
    return sgn ? launch_lines_inst<R, true, false>(p, grid, s) : launch_lines_inst<R, false, false>(p, grid, s);
}

struct LinesShape {
    int kind;            // 0 linear, 1 conv2d
    int N, Cin, kh, kw;  // output channels, inner length per tap, taps
    int Cp, Cc, n_tiles;
    int pair_g;          // > 0: tap pairing, that many taps per group of four steps (see adapt::LinesParams)
    size_t dt_bytes;     // per table half
    // as the kernels see the inner dimension: steps per "tap" and number of "taps"
    int k_cc() const { return pair_g ? 4 : Cc; }
    int k_taps() const { return pair_g ? (kh * kw + pair_g - 1) / pair_g : kh * kw; }
};

// pairing: convolutions with 8 or 16 (padded) channels and a single-pass table pack 4 or 2 taps into a group of steps,
// which lets them run on the fast kernel
LinesShape lines_shape(int kind, int bits, int N, int Cin, int kh, int kw, bool may_pair = false) {
    LinesShape q;
    q.kind = kind; q.N = N; q.Cin = Cin; q.kh = kh; q.kw = kw;
    q.Cp = kind == 0 ? ((Cin + 31) / 32) * 32 : ((Cin + 7) / 8) * 8;
    q.Cc = q.Cp / 8;
    q.n_tiles = (N + 7) / 8;
    q.pair_g = (may_pair && kind == 1 && q.Cp <= 16) ? 32 / q.Cp : 0;
    q.dt_bytes = (size_t)q.n_tiles * q.k_taps() * q.k_cc() * ((size_t)adapt::LINE_BYTES << bits);
    return q;
}

int pack_lines(const adapt_lut *lut, const int8_t *w, const LinesShape &q, uint4 *const dt[2], hipStream_t s) {
    for (int half = 0; half <= lut->storage; ++half) {
        const size_t total = q.dt_bytes / 16;
        size_t blocks = (total + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        adapt::pack_line_tables_kernel<<<(unsigned)blocks, 256, 0, s>>>(lut->lut16_dev[half], w, dt[half], lut->bits, q.N, q.Cin,
                                                                       q.kh * q.kw, q.Cc, q.n_tiles, 0, q.pair_g, q.Cp / 4);
        HIP_TRY(hipGetLastError());
    }
    return ADAPT_OK;
}

struct LinesPhase {      // one stride-1 sub-convolution of a transposed convolution (plain layers: a single zero phase)
    int xt_off = 0;         // bytes into the activation copy
    int out_off = 0;        // elements into an output plane
    long long dt_off = 0;   // 16-byte units into the derived tables
};

struct LinesCall {       // per-call geometry of the activation side
    int M, HoWo, Wo;
    long long img_stride;
    int oy_stride, ox_stride, ky_stride, kx_stride;
    int xmajor, ch_stride;  // x-major activation copy (see pad_channels_last_kernel) and its bytes per channel step
    int out_plane, out_sy, out_sx;      // see adapt::LinesParams
    std::vector<LinesPhase> phases;
    LinesPlan plan;                     // from plan_product(): kernel, rows per lane, split of the inner dimension
    // Derived tables in the quad order (lut_quad.hpp) and the offset of their digit form; needed when the plan says LK_QUAD
    const uint4 *dt_quad = nullptr;
    int quad_c = 0;
    bool nonneg_in = false;             // every activation code is >= 0 (copy written by a ReLU epilogue)
    int32_t *partial = nullptr;         // room for the partial sums when the plan splits the inner dimension
    // transposed convolution: zero sums and geometry for taking the border terms off inside the kernel (see
    // adapt::LinesParams::zsum); run_lines reports through border_done whether it did
    const int32_t *zsum = nullptr;
    int cv_Ho = 0, cv_Wo = 0, cv_H = 0, cv_W = 0, cv_kh = 0, cv_kw = 0, cv_s = 1, cv_pad = 0, cv_Ly = 0, cv_Lx = 0;
    size_t out_elems = 0;               // elements of the whole output tensor
    size_t out_channels = 1, out_inner = 1;     // where the channel sits in a flat output index: (i / inner) % channels
};

// The plan of one product (see lines_plan.hpp).  M: rows (per phase); phases: 1, or stride^2 of a transposed convolution;
// Wo: output width (linear layers: M); sw: horizontal stride; quad_tables: the caller holds tables in the quad order.
LinesPlan plan_product(const LinesShape &q, int bits, int storage, int M, int phases, int Wo, int sw, bool quad_tables, int cu = 0) {
    PlanIn in;
    in.M = M; in.tiles = q.n_tiles * phases; in.k_cc = q.k_cc(); in.k_taps = q.k_taps(); in.Wo = Wo; in.sw = sw;
    in.quad_steps = (quad_tables && storage == 0 && q.Cp % adapt::QUAD_STEP == 0) ? q.kh * q.kw * (q.Cp / adapt::QUAD_STEP) : 0;
    in.bits = bits; in.cu = cu > 0 ? cu : device_cus();
    LinesPlan pl = plan_lines(in);
#ifdef ADAPT_TUNING_KNOBS
    if (const char *e = getenv("ADAPT_QUAD_PLAN")) {        // "R,ksplit": tuning experiments only (not compiled into the product)
        int R = 0, ks = 0;
        if (pl.kernel == LK_QUAD && sscanf(e, "%d,%d", &R, &ks) == 2 && quad_rows_ok(R, M, Wo) && ks >= 1 && ks <= in.quad_steps) {
            const int sps = (in.quad_steps + ks - 1) / ks;
            pl.R = R; pl.gps = sps; pl.ksplit = (in.quad_steps + sps - 1) / sps;
        }
    }
#endif
    return pl;
}

// bytes of partial sums a call needs from its workspace (0 without a split of the inner dimension): ksplit copies of
// the output for reduce_partials_kernel
size_t plan_partial_bytes(const LinesPlan &pl, size_t out_elems) {
    return pl.ksplit > 1 ? (size_t)pl.ksplit * out_elems * sizeof(int32_t) : 0;
}

// bytes of one phase's tables in the quad order
size_t quad_table_bytes(const LinesShape &q, int bits) {
    return (size_t)q.n_tiles * q.kh * q.kw * (q.Cp / adapt::QUAD_STEP) * ((size_t)adapt::QUAD_LINE_BYTES << bits);
}

// The kernel that adds split sums can run without an fp32 output buffer (only the next layer's copy is wanted) in its
// four-elements-per-thread form: rescaled output with a chained copy, everything in whole quads and 16-byte aligned.
static bool adding_kernel_without_output_ok(const LinesCall &c, const LayerIO *io) {
    if (!io || !io->chain.buf || !io->deq) return false;
    const int wo = io->chain_wo;
    return c.out_elems < 0x7fffffffull && c.out_elems % 4 == 0 && c.out_inner % 4 == 0 && wo > 0 && wo % 4 == 0 && c.partial &&
           ((reinterpret_cast<uintptr_t>(c.partial) | reinterpret_cast<uintptr_t>(io->resid)) & 15u) == 0;
}

int run_lines(int bits, int storage, const LinesShape &q, uint4 *const dt[2], const int8_t *xt, const LinesCall &c,
              int32_t *out, hipStream_t s, const LayerIO *io = nullptr, bool may_fuse = true, bool *border_done = nullptr,
              bool *finished = nullptr) {
    const int n_phases = (int)c.phases.size();
    const LinesPlan &pl = c.plan;
    const int R = pl.R;
    const bool quad = pl.kernel == LK_QUAD;
    const bool split = pl.ksplit > 1;
    const bool sums_elsewhere = split;      // partial sums in c.partial, added by reduce_partials_kernel
    if (sums_elsewhere && !c.partial) return fail(ADAPT_ERR_HIP, "lines path: no room for partial sums");
    adapt::LinesParams p;
    p.xt = xt;
    p.M = c.M; p.N = q.N; p.n_tiles = q.n_tiles;
    p.Cc = quad ? q.Cp / adapt::QUAD_STEP : q.k_cc(); p.taps = quad ? q.kh * q.kw : q.k_taps(); p.kw = q.kw; p.bits = bits;
    p.pair_g = quad ? 0 : q.pair_g; p.pair_cg = q.Cp / 4; p.taps_real = q.kh * q.kw;
    if (q.pair_g && storage != 0) return fail(ADAPT_ERR_HIP, "lines path: tap pairing with a two-pass table");
    p.HoWo = c.HoWo; p.Wo = c.Wo; p.img_stride = c.img_stride;
    p.oy_stride = c.oy_stride; p.ox_stride = c.ox_stride; p.ky_stride = c.ky_stride; p.kx_stride = c.kx_stride;
    p.ch_stride = c.ch_stride;
    p.out_plane = c.out_plane; p.out_sy = c.out_sy; p.out_sx = c.out_sx;
    p.m_tiles = (c.M + pl.rows_per_wg() - 1) / pl.rows_per_wg();
    p.d_HoWo = fast_div((uint32_t)p.HoWo); p.d_Wo = fast_div((uint32_t)p.Wo);
    p.d_ntiles = fast_div((uint32_t)p.n_tiles); p.d_mtiles = fast_div((uint32_t)p.m_tiles); p.d_phases = fast_div(1u);
    p.ksplit = pl.ksplit; p.gps = pl.gps; p.ks_out_stride = sums_elsewhere ? (long long)c.out_elems : 0;
    // digit tables: every real lookup of an output lacks the offset (sums wrap in 32 bits like everything else)
    // (the fast 128-byte-line kernels and the quad kernel copy only the lines that can be selected; the generic kernel copies all)
    p.copy_lines = c.nonneg_in ? (1 << bits) / 2 : (1 << bits);
    p.corr = quad ? (int)(uint32_t)((unsigned long long)((long long)q.kh * q.kw * q.Cin * (long long)c.quad_c)) : 0;
    // one base offset per lane is enough when the R rows of a lane are equally spaced in xt
    const bool regular = (c.M % R == 0) && (c.HoWo == 1 || c.Wo % R == 0);
    const bool xmajor = pl.kernel == LK_XMAJOR;
    if (c.xmajor != pl.xmajor) return fail(ADAPT_ERR_HIP, "lines path: the activation copy does not have the layout of the plan");
    // the quad kernel has an instantiation that takes the border terms of a transposed convolution off itself and
    // knows tanh; the kernel that adds split sums knows tanh too
    const bool border_in_kernel = c.zsum && !sums_elsewhere && quad;
    if (border_done) *border_done = border_in_kernel;
    const bool act_ok = io && (io->act <= 1 || (io->act == 2 && (sums_elsewhere || quad)));
    const bool fuse = (may_fuse || border_in_kernel) && io && io->deq && storage == 0 && act_ok;
    if (finished) *finished = fuse;
    const bool fuse_in_kernel = fuse && !sums_elsewhere;
    const bool chain_in_kernel = fuse_in_kernel && io->chain.buf;
    const bool extra = quad && (border_in_kernel || (fuse_in_kernel && io->act == 2) || chain_in_kernel);
    p.chain = chain_in_kernel ? io->chain : adapt::ChainOut{};
    // a caller that only wants the next layer's copy passes no output buffer; that works where the product kernel itself
    // finishes the sums and writes the copy (no partial sums, no separate finishing pass, residual aside)
    if (!out && !chain_in_kernel && !(sums_elsewhere && fuse && storage == 0 && adding_kernel_without_output_ok(c, io)))
        return fail(ADAPT_ERR_UNSUPPORTED, "this layer shape finishes its sums in a separate pass over the output: y_dev is needed");
    p.no_out = (!out && !sums_elsewhere) ? 1 : 0;       // (partial sums are always stored)
    p.zsum = border_in_kernel ? c.zsum : nullptr;
    p.cv_s = fast_div((uint32_t)c.cv_s);
    p.cv_Ho = c.cv_Ho; p.cv_Wo = c.cv_Wo; p.cv_H = c.cv_H; p.cv_W = c.cv_W; p.cv_kh = c.cv_kh; p.cv_kw = c.cv_kw;
    p.cv_pad = c.cv_pad; p.cv_Ly = c.cv_Ly; p.cv_Lx = c.cv_Lx;
    p.deq = fuse_in_kernel ? 1 : 0; p.act = fuse_in_kernel ? io->act : 0;
    p.scale = fuse_in_kernel ? io->s_out : 1.0f; p.bias = fuse_in_kernel ? io->bias : nullptr;
    p.scales = fuse_in_kernel ? io->s_out_vec : nullptr;
    p.resid = fuse_in_kernel ? io->resid : nullptr;
    const long long quad_phase_u4 = quad ? (long long)(quad_table_bytes(q, bits) / 16) : 0;
    int rc = ADAPT_OK;
    for (int half = 0; half <= storage && rc == ADAPT_OK; ++half) {
        p.dt = quad ? c.dt_quad : dt[half];
        p.out = sums_elsewhere ? c.partial : out;
        p.shift = (half == 0 || sums_elsewhere) ? -1 : 16;
        const bool sgn = storage == 0 || half == 1;
        for (int first = 0; first < n_phases && rc == ADAPT_OK; first += 4) {       // up to four phases per launch
            p.phases = n_phases - first < 4 ? n_phases - first : 4;
            for (int i = 0; i < 4; ++i) {
                const int fi = first + (i < p.phases ? i : 0);
                const LinesPhase &f = c.phases[fi];
                p.xt_off[i] = f.xt_off; p.out_off[i] = f.out_off; p.dt_off[i] = quad ? (long long)fi * quad_phase_u4 : f.dt_off;
            }
            const long long grid = (long long)p.m_tiles * q.n_tiles * p.phases * p.ksplit;
            if (grid > 0x7fffffffLL) return fail(ADAPT_ERR_UNSUPPORTED, "lines path: grid too large");
            p.d_phases = fast_div((uint32_t)p.phases);
            if (quad) rc = launch_quad(p, (unsigned)grid, R, extra, s);
            else if (xmajor) rc = sgn ? launch_lines_xmajor<true>(p, (unsigned)grid, s) : launch_lines_xmajor<false>(p, (unsigned)grid, s);
            else if (R == 8) rc = launch_lines_r<8>(p, (unsigned)grid, sgn, regular, s);
            else if (R == 4) rc = launch_lines_r<4>(p, (unsigned)grid, sgn, regular, s);
            else rc = launch_lines_r<2>(p, (unsigned)grid, sgn, regular, s);
        }
        if (sums_elsewhere && rc == ADAPT_OK) {
            const int wo = io ? io->chain_wo : 1;
            const bool chained = fuse && half == 0 && io->chain.buf;
            // four elements per thread where planes (and, with a chained copy, rows) are whole quads and everything is aligned
            const bool quads = fuse && half == 0 && c.out_elems < 0x7fffffffull && c.out_elems % 4 == 0 && c.out_inner % 4 == 0 &&
                               c.out_inner < 0x7fffffffull && c.out_channels < 0x7fffffffull && (!chained || wo % 4 == 0) &&
                               ((reinterpret_cast<uintptr_t>(c.partial) | reinterpret_cast<uintptr_t>(out) |
                                 reinterpret_cast<uintptr_t>(io->resid)) & 15u) == 0;
            if (!out && !(quads && chained))
                return fail(ADAPT_ERR_UNSUPPORTED, "this layer shape finishes its sums in a separate pass over the output: y_dev is needed");
            const size_t threads_needed = quads ? c.out_elems / 4 : c.out_elems;
            adapt::reduce_partials_kernel<<<ew_grid(threads_needed), adapt::EW_THREADS, 0, s>>>(
                c.partial, pl.ksplit, c.out_elems, out, c.out_elems, half == 0 ? -1 : 16, (fuse && half == 0) ? 1 : 0, c.out_channels,
                c.out_inner, fuse ? io->s_out : 1.0f, fuse ? io->s_out_vec : nullptr, fuse ? io->bias : nullptr, fuse ? io->resid : nullptr,
                fuse ? io->act : 0, (fuse && half == 0) ? io->chain : adapt::ChainOut{}, wo, fast_div((uint32_t)(quads ? c.out_inner : 1)),
                fast_div((uint32_t)(quads ? c.out_channels : 1)), fast_div((uint32_t)(quads && wo > 0 ? wo : 1)), quads ? 1 : 0);
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) rc = fail(ADAPT_ERR_HIP, "reduce_partials launch: %s", hipGetErrorString(e));
        }
    }
    return rc;
}

// Derived tables of a handle in the quad order (single-pass tables, 16 | padded channels), made when the handle is
// packed.  Entries are the int8 digits of entry - c with c = smallest entry + 32640 (see adapt::quad_entry).
int pack_quad(adapt_weights *h, hipStream_t s, const char *who) {
    if (h->storage != 0 || h->Cp % adapt::QUAD_STEP != 0 || h->Cp == 0) return ADAPT_OK;
    LinesShape q;
    q.kind = h->kind; q.N = h->N; q.Cin = h->Cin; q.Cp = h->Cp; q.n_tiles = h->n_tiles;
    const int phases = h->kind == 2 ? h->stride * h->stride : 1;
    q.kh = h->kind == 2 ? h->kh / h->stride : h->kh; q.kw = h->kind == 2 ? h->kw / h->stride : h->kw;
    const size_t bytes = quad_table_bytes(q, h->bits) * phases;
    if (bytes == 0) return ADAPT_OK;
    hipError_t e = dbg_malloc((void **)&h->dtq_dev, bytes);
    if (e != hipSuccess) return fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "%s: hipMalloc(%zu): %s", who, bytes, hipGetErrorString(e));
    h->dtq_bytes = bytes;
    h->dtq_c = h->lut->min_entry + 32640;
    const size_t total = bytes / 16;
    size_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (h->kind == 2)
        adapt::pack_quad_tables_convt_kernel<<<(unsigned)blocks, 256, 0, s>>>(h->lut->lut16_dev[0], h->w8_dev, h->dtq_dev, h->bits, h->N, h->Cin,
                                                                             h->kh, h->kw, h->stride, h->Cp, h->n_tiles, 1, h->dtq_c);
    else
        adapt::pack_quad_tables_kernel<<<(unsigned)blocks, 256, 0, s>>>(h->lut->lut16_dev[0], h->w8_dev, h->dtq_dev, h->bits, h->N, h->Cin,
                                                                       h->kh * h->kw, h->Cp, h->n_tiles, 0, 1, h->dtq_c);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

// zero-padded activation copy of a convolution's input (int8, or fp32 quantised on the way)
int launch_pad(const LayerIO *io, const int8_t *x, int bits, int8_t *xt, int N, int C, int H, int W, int ph, int pw, int Cp, int xmajor,
               hipStream_t s) {
    const size_t total = (size_t)N * (H + 2 * ph) * (W + 2 * pw) * (Cp / 4);
    size_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    if (!blocks) return ADAPT_OK;
    const adapt::FastDiv dwp = fast_div((uint32_t)(W + 2 * pw)), dc4 = fast_div((uint32_t)(Cp / 4)), dhp = fast_div((uint32_t)(H + 2 * ph));
    const int fast = total < 0x7fffffffull ? 1 : 0;
    if (fast && (size_t)N * C * H * W < 0x7fffffffull && total * 4 < 0x7fffffffull) {
        // several words per thread, all operands in flight together
        constexpr int U = 2;
        const unsigned mblocks = (unsigned)(((total + U - 1) / U + 255) / 256);
        if (io && io->xf)
            adapt::pad_channels_last_multi_kernel<adapt::SrcF32, U><<<mblocks, 256, 0, s>>>(
                adapt::SrcF32{io->xf, io->s_x, io->Q, (1u << bits) - 1u}, xt, C, H, W, ph, pw, Cp, xmajor, dwp, dc4, dhp, (uint32_t)total);
        else
            adapt::pad_channels_last_multi_kernel<adapt::SrcI8, U><<<mblocks, 256, 0, s>>>(adapt::SrcI8{x, (1u << bits) - 1u}, xt, C, H, W, ph, pw,
                                                                                           Cp, xmajor, dwp, dc4, dhp, (uint32_t)total);
        HIP_TRY(hipGetLastError());
        return ADAPT_OK;
    }
    if (io && io->xf)
        adapt::pad_channels_last_kernel<<<(unsigned)blocks, 256, 0, s>>>(adapt::SrcF32{io->xf, io->s_x, io->Q, (1u << bits) - 1u}, xt, N, C, H, W,
                                                                         ph, pw, Cp, xmajor, dwp, dc4, dhp, fast);
    else
        adapt::pad_channels_last_kernel<<<(unsigned)blocks, 256, 0, s>>>(adapt::SrcI8{x, (1u << bits) - 1u}, xt, N, C, H, W, ph, pw, Cp, xmajor,
                                                                         dwp, dc4, dhp, fast);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

// activation side of a linear layer: A itself when its rows are a multiple of 32 bytes, else a zero-padded copy
int lines_linear(int bits, int storage, const LinesShape &q, uint4 *const dt[2], const int8_t *a, int32_t *out, int M, hipStream_t s,
                 Workspace *ws, const LayerIO *io = nullptr, const adapt_weights *wh = nullptr) {
    const uint32_t amask = (1u << bits) - 1u;
    const adapt::SrcI8 src8{a, amask};
    const adapt::SrcF32 srcf{io ? io->xf : nullptr, io ? io->s_x : 1.0f, io ? io->Q : 1.0f, amask};
    const bool from_f32 = io && io->xf;
    const int K = q.Cin, Kp = q.Cp;
    int8_t *tmp = nullptr;
    const int8_t *xt = a;
    LinesCall c;
    c.M = M;
    c.phases.resize(1);
    c.out_elems = (size_t)M * q.N; c.out_channels = (size_t)q.N; c.out_inner = 1;
    c.plan = plan_product(q, bits, storage, M, 1, M, 1, wh && wh->dtq_dev);
    const size_t part_bytes = plan_partial_bytes(c.plan, c.out_elems);
    const size_t copy_bytes = (((size_t)M * Kp + 64 + 255) / 256) * 256;
    if (c.plan.xmajor) {
        // x-major copy: one image of one row of M pixels with K channels; a lane's 8 rows x 4 inner indices are 32
        // contiguous bytes instead of 8 words that are a whole matrix row apart
        int wrc = ws_get(ws, copy_bytes + part_bytes, s, (void **)&tmp);
        if (wrc) return wrc;
        dim3 grid((unsigned)((M + 63) / 64), (unsigned)((Kp / 4 + 15) / 16));
        if (from_f32) adapt::rows_to_xmajor_kernel<<<grid, 256, 0, s>>>(srcf, tmp, M, K, Kp);
        else adapt::rows_to_xmajor_kernel<<<grid, 256, 0, s>>>(src8, tmp, M, K, Kp);
        xt = tmp;
        c.HoWo = M; c.Wo = M; c.img_stride = 0;
        c.oy_stride = c.ky_stride = 0; c.ox_stride = c.kx_stride = 4;
        c.xmajor = 1; c.ch_stride = M;
        c.out_plane = 1; c.out_sy = 0; c.out_sx = q.N;
        if (c.plan.kernel == LK_QUAD) { c.dt_quad = wh->dtq_dev; c.quad_c = wh->dtq_c; }
    } else {
        if (Kp != K || from_f32 || part_bytes) {
            int wrc = ws_get(ws, copy_bytes + part_bytes, s, (void **)&tmp);
            if (wrc) return wrc;
        }
        if (Kp != K || from_f32) {
            const size_t total = (size_t)M * Kp;
            size_t blocks = (total + 255) / 256;
            if (blocks > 65536) blocks = 65536;
            if (from_f32) adapt::pad_rows_kernel<<<(unsigned)blocks, 256, 0, s>>>(srcf, tmp, M, K, Kp);
            else adapt::pad_rows_kernel<<<(unsigned)blocks, 256, 0, s>>>(src8, tmp, M, K, Kp);
            xt = tmp;
        }
        c.HoWo = 1; c.Wo = 1; c.img_stride = Kp;
        c.oy_stride = c.ox_stride = c.ky_stride = c.kx_stride = 0;
        c.xmajor = 0; c.ch_stride = 0;
        c.out_plane = 1; c.out_sy = 0; c.out_sx = 0;
    }
    if (part_bytes) c.partial = reinterpret_cast<int32_t *>(tmp + copy_bytes);
    bool finished = false;
    int rc = run_lines(bits, storage, q, dt, xt, c, out, s, io, true, nullptr, &finished);
    rc = ws_put(ws, tmp, s, rc);
    if (rc == ADAPT_OK && io && io->deq && !finished) rc = finish_inplace(out, (size_t)M * q.N, (size_t)q.N, 1, *io, s);
    return rc;
}

// activation side of a convolution: zero-padded channel-last copy of x
int lines_conv2d(int bits, int storage, const LinesShape &q, uint4 *const dt[2], const int8_t *x, int32_t *out, int N, int H,
                 int W, int Ho, int Wo, int sh, int sw, int ph, int pw, int dh, int dw, hipStream_t s, Workspace *ws,
                 const LayerIO *io = nullptr, const adapt_weights *wh = nullptr, bool input_ready = false) {
    const int Hp = H + 2 * ph, Wp = W + 2 * pw, Cp = q.Cp;
    const size_t xt_bytes = (size_t)N * Hp * Wp * Cp;
    // With 8 rows per lane that are 8 consecutive output pixels of a stride-1 convolution, the copy is laid
    // out so that these rows' activations are contiguous (one wide load per lane instead of one per row).
    const int M = N * Ho * Wo;
    const LinesPlan plan = plan_product(q, bits, storage, M, 1, Wo, sw, wh && wh->dtq_dev);
    const int xmajor = plan.xmajor;
    const size_t out_elems = (size_t)M * q.N;
    const size_t part_bytes = plan_partial_bytes(plan, out_elems);
    const size_t copy_bytes = ((xt_bytes + 64 + 255) / 256) * 256;
    int8_t *xt = nullptr;
    {
        if (input_ready) {      // the layer before wrote the copy (adapt_conv2d_chain_prepare fixed its place and layout)
            if (!ws || !ws->ptr || ws->bytes < copy_bytes + part_bytes || !wh || wh->chain_in.xmajor != xmajor)
                return fail(ADAPT_ERR_INVALID_ARGUMENT, "chained convolution: the input buffer was not prepared for this geometry");
            xt = static_cast<int8_t *>(ws->ptr);
        } else {
            if (wh && wh->chain_in.valid) {     // an ordinary call with another geometry ends the prepared state
                const auto &ci = wh->chain_in;
                if (ci.N != N || ci.H != H || ci.W != W || ci.sh != sh || ci.sw != sw || ci.ph != ph || ci.pw != pw || ci.dh != dh || ci.dw != dw)
                    wh->chain_in.valid = false;
            }
            int wrc = ws_get(ws, copy_bytes + part_bytes, s, (void **)&xt);
            if (wrc) return wrc;
            int prc = launch_pad(io, x, bits, xt, N, q.Cin, H, W, ph, pw, Cp, xmajor, s);
            if (prc) return ws_put(ws, xt, s, prc);
        }
    }
    LinesCall c;
    c.plan = plan;
    c.M = M; c.HoWo = Ho * Wo; c.Wo = Wo;
    c.img_stride = (long long)Hp * Wp * Cp;
    c.oy_stride = sh * Wp * Cp; c.ky_stride = dh * Wp * Cp;
    c.ox_stride = xmajor ? 4 * sw : sw * Cp;
    c.kx_stride = xmajor ? 4 * dw : dw * Cp;
    c.xmajor = xmajor; c.ch_stride = Wp;
    c.out_plane = Ho * Wo; c.out_sy = Wo; c.out_sx = 1;
    c.phases.resize(1);
    c.out_elems = out_elems; c.out_channels = (size_t)q.N; c.out_inner = (size_t)Ho * Wo;
    if (part_bytes) c.partial = reinterpret_cast<int32_t *>(xt + copy_bytes);
    if (plan.kernel == LK_QUAD) { c.dt_quad = wh->dtq_dev; c.quad_c = wh->dtq_c; }
    c.nonneg_in = input_ready && wh && wh->chain_in.nonneg;
    bool finished = false;
    int rc = run_lines(bits, storage, q, dt, xt, c, out, s, io, true, nullptr, &finished);
    rc = ws_put(ws, xt, s, rc);
    if (rc == ADAPT_OK && io && io->deq && !finished)
        rc = finish_inplace(out, (size_t)M * q.N, (size_t)q.N, (size_t)Ho * Wo, *io, s);
    return rc;
}

// Transposed convolution as stride * stride stride-1 convolutions (see pack_line_tables_convt_kernel).  Needs kernel
// sizes that are multiples of the stride, an output size that is one too, and more than one input pixel.
bool convt_phases_ok(int H, int W, int kh, int kw, int st, int pad) {
    return kh % st == 0 && kw % st == 0 && (2 * pad) % st == 0 && (long long)H * W > 1;
}

LinesShape convt_phase_shape(int bits, int Cout, int Cin, int kh, int kw, int st) {
    return lines_shape(1, bits, Cout, Cin, kh / st, kw / st);       // one phase; dt_bytes is per phase
}

int lines_conv_transpose2d(int bits, int storage, const LinesShape &q, uint4 *const dt[2], const int32_t *zsum, const int8_t *x,
                           int32_t *out, int N, int H, int W, int kh, int kw, int st, int pad, hipStream_t s, Workspace *ws,
                           const LayerIO *io = nullptr, const adapt_weights *wh = nullptr, bool input_ready = false) {
    const int Ty = q.kh, Tx = q.kw, Cp = q.Cp;
    const int Hp = H + 2 * (Ty - 1), Wp = W + 2 * (Tx - 1);
    const int Ho = (H - 1) * st - 2 * pad + kh, Wo = (W - 1) * st - 2 * pad + kw;
    const int Qy = Ho / st, Qx = Wo / st;
    const int M = N * Qy * Qx;
    const size_t xt_bytes = (size_t)N * Hp * Wp * Cp;
    const LinesPlan plan = plan_product(q, bits, storage, M, st * st, Qx, 1, wh && wh->dtq_dev);
    const int xmajor = plan.xmajor;
    const size_t out_elems = (size_t)N * q.N * Ho * Wo;
    const size_t part_bytes = plan_partial_bytes(plan, out_elems);
    const size_t copy_bytes = ((xt_bytes + 64 + 255) / 256) * 256;
    int8_t *xt = nullptr;
    if (input_ready) {          // the layer before wrote the copy (adapt_conv_transpose2d_chain_prepare fixed its place and layout)
        if (!ws || !ws->ptr || ws->bytes < copy_bytes + part_bytes || !wh || wh->chain_in.xmajor != xmajor)
            return fail(ADAPT_ERR_INVALID_ARGUMENT, "chained transposed convolution: the input buffer was not prepared for this geometry");
        xt = static_cast<int8_t *>(ws->ptr);
    } else {
        if (wh) wh->chain_in.valid = false;     // (an ordinary call overwrites a prepared copy)
        int wrc = ws_get(ws, copy_bytes + part_bytes, s, (void **)&xt);
        if (wrc) return wrc;
        int prc = launch_pad(io, x, bits, xt, N, q.Cin, H, W, Ty - 1, Tx - 1, Cp, xmajor, s);
        if (prc) return ws_put(ws, xt, s, prc);
    }
    LinesCall c;
    c.plan = plan;
    c.M = M; c.HoWo = Qy * Qx; c.Wo = Qx;
    c.img_stride = (long long)Hp * Wp * Cp;
    c.oy_stride = c.ky_stride = Wp * Cp;
    c.ox_stride = c.kx_stride = xmajor ? 4 : Cp;
    c.xmajor = xmajor; c.ch_stride = Wp;
    c.out_plane = Ho * Wo; c.out_sy = st * Wo; c.out_sx = st;
    const long long phase_u4 = (long long)(q.dt_bytes / 16);
    for (int ry = 0; ry < st; ++ry)
        for (int rx = 0; rx < st; ++rx) {
            // first window position of the phase: the smallest q with an output row s q + r - pad >= 0; in the
            // copy (padded by T - 1) the window of that output starts at row q
            const int qy0 = pad > ry ? (pad - ry + st - 1) / st : 0, qx0 = pad > rx ? (pad - rx + st - 1) / st : 0;
            LinesPhase f;
            f.xt_off = qy0 * Wp * Cp + qx0 * (xmajor ? 4 : Cp);
            f.out_off = (st * qy0 + ry - pad) * Wo + (st * qx0 + rx - pad);
            f.dt_off = (long long)(ry * st + rx) * phase_u4;
            c.phases.push_back(f);
        }
    // window taps over the zero border were looked up; the layer is defined over real pairs only
    const int Ly = kh - st - pad > 0 ? kh - st - pad : 0, Lx = kw - st - pad > 0 ? kw - st - pad : 0;
    const bool border = Ly > 0 || Lx > 0;       // then the sums are corrected before they can be rescaled
    c.out_elems = out_elems; c.out_channels = (size_t)q.N; c.out_inner = (size_t)Ho * Wo;
    if (part_bytes) c.partial = reinterpret_cast<int32_t *>(xt + copy_bytes);
    const bool quad = plan.kernel == LK_QUAD;
    if (quad) { c.dt_quad = wh->dtq_dev; c.quad_c = wh->dtq_c; }
    c.nonneg_in = input_ready && wh && wh->chain_in.nonneg;
    const bool chained = io && io->chain.buf;
    if ((border || chained) && out_elems < 0x7fffffffull) {     // the product kernel takes the border terms off where it can; its
        if (border) c.zsum = zsum;                              // chained copy needs the true output position of a phase's pixel
        c.cv_Ho = Ho; c.cv_Wo = Wo; c.cv_H = H; c.cv_W = W; c.cv_kh = kh; c.cv_kw = kw; c.cv_s = st; c.cv_pad = pad; c.cv_Ly = Ly; c.cv_Lx = Lx;
    }
    bool border_done = false, finished = false;
    // a chained copy is written by the quad kernel's epilogue or, for every other kernel, by the pass that rescales afterwards
    const bool chain_ok_in_kernel = !chained || (quad && part_bytes == 0 && out_elems < 0x7fffffffull);
    int rc = run_lines(bits, storage, q, dt, xt, c, out, s, io, !border && chain_ok_in_kernel, &border_done, &finished);
    rc = ws_put(ws, xt, s, rc);
    if (rc != ADAPT_OK) return rc;
    const size_t planes = (size_t)N * q.N;
    if (border_done) {      // sums corrected in the product kernel's epilogue (and rescaled there, if it could)
        if (io && io->deq && !finished) return finish_inplace(out, planes * Ho * Wo, (size_t)q.N, (size_t)Ho * Wo, *io, s);
        return ADAPT_OK;
    }
    const int nrows = 2 * Ly < Ho ? 2 * Ly : Ho, ncols = 2 * Lx < Wo ? 2 * Lx : Wo;
    const size_t work[2] = {planes * nrows * Wo, planes * (size_t)(Ho - nrows) * ncols};
    for (int region = 0; region < 2; ++region) {
        if (!work[region]) continue;
        size_t blocks = (work[region] + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        adapt::convt_border_fix_kernel<<<(unsigned)blocks, 256, 0, s>>>(out, zsum, (int)planes, q.N, Ho, Wo, H, W, kh, kw, st, pad, Ly,
                                                                       Lx, region);
        HIP_TRY(hipGetLastError());
    }
    if (io && io->deq && (border || !finished)) return finish_inplace(out, planes * Ho * Wo, (size_t)q.N, (size_t)Ho * Wo, *io, s);
    return ADAPT_OK;
}

// derived tables of all phases + zero sums into caller-provided buffers
int pack_convt(const adapt_lut *lut, const int8_t *w, const LinesShape &q, int kh, int kw, int st, uint4 *const dt[2], int32_t *zsum,
               hipStream_t s) {
    for (int half = 0; half <= lut->storage; ++half) {
        const size_t total = q.dt_bytes / 16 * st * st;
        size_t blocks = (total + 255) / 256;
        if (blocks > 65536) blocks = 65536;
        adapt::pack_line_tables_convt_kernel<<<(unsigned)blocks, 256, 0, s>>>(lut->lut16_dev[half], w, dt[half], lut->bits, q.N, q.Cin, kh,
                                                                             kw, st, q.Cc, q.n_tiles);
        HIP_TRY(hipGetLastError());
    }
    const int nz = q.N * kh * kw;
    adapt::convt_zero_sums_kernel<<<(unsigned)((nz + 255) / 256), 256, 0, s>>>(lut->lut16_dev[0], lut->storage ? lut->lut16_dev[1] : nullptr,
                                                                              w, zsum, lut->bits, q.N, q.Cin, kh * kw);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

// limits of the lines path: 32-bit byte offsets into the activation copy, and a sane table stream
bool lines_fits(long long xt_bytes, size_t dt_bytes, int storage) {
    return xt_bytes < 0x7fffff00LL && dt_bytes * (size_t)(storage + 1) <= ((size_t)4 << 30);
}

// one-shot use: pack into a stream-ordered temporary, run, release
template <typename F>
int with_temp_tables(const adapt_lut *lut, const int8_t *w, const LinesShape &q, hipStream_t s, F &&body) {
    uint4 *dt[2] = {nullptr, nullptr};
    int rc = ADAPT_OK;
    for (int half = 0; half <= lut->storage; ++half) {
        hipError_t e = dbg_malloc_async((void **)&dt[half], q.dt_bytes, s);
        if (e != hipSuccess) {
            rc = fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "hipMallocAsync(tables): %s", hipGetErrorString(e));
            break;
        }
    }
    if (rc == ADAPT_OK) rc = pack_lines(lut, w, q, dt, s);
    if (rc == ADAPT_OK) rc = body(dt);
    for (int half = 0; half < 2; ++half)
        if (dt[half]) (void)hipFreeAsync(dt[half], s);
    return rc;
}

// The lines path pays K*N*2^b table entries of packing and streams them once per 128*R rows:
// worth it from a few thousand rows on.
constexpr int LINES_MIN_ROWS = 4096;

int check_lut(const adapt_lut *lut, const char *who) {
    if (!lut) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: lut is NULL", who);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != lut->device)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: table handle belongs to device %d, current device is %d", who, lut->device, dev);
    return ADAPT_OK;
}

// transposed convolution on the rows kernel
int convt_rows(const adapt_lut *lut, const int8_t *x, const int8_t *w, int32_t *acc, int N, int Cin, int H, int W, int Cout, int kh,
               int kw, int stride, int pad, hipStream_t s, const adapt_weights *h = nullptr, const LayerIO *io = nullptr) {
    const int Ho = (H - 1) * stride - 2 * pad + kh, Wo = (W - 1) * stride - 2 * pad + kw;
    Geometry g{};
    if (H == 1 && W == 1 && pad == 0) {
        // one input pixel: output pixel (ky, kx) of channel co is the inner product of the input vector with
        // w[:, co, ky, kx] -- a linear layer with N = Cout kh kw whose weights are stored [K][N]
        g.mode = adapt::MODE_GEMM; g.M = N; g.N = Cout * kh * kw; g.Cin = Cin; g.taps = 1; g.kw = 1;
        g.H = 1; g.W = 1; g.Wo = 1; g.HoWo = 1; g.sh = g.sw = g.dh = g.dw = 1; g.ph = g.pw = 0;
        g.kstride = 1; g.img_stride = Cin; g.wt = 1;
        if (io && io->deq) {
            // here the output is [N][Cout][kh][kw] while the product's channel axis is Cout kh kw: rescale afterwards
            int rc = h ? run_rows(lut, x, w, acc, g, s, h->wofs1_dev, h->wofs1_npad) : run_rows(lut, x, w, acc, g, s);
            if (rc) return rc;
            return finish_inplace(acc, (size_t)N * Cout * kh * kw, (size_t)Cout, (size_t)kh * kw, *io, s);
        }
        return h ? run_rows(lut, x, w, acc, g, s, h->wofs1_dev, h->wofs1_npad) : run_rows(lut, x, w, acc, g, s);
    }
    g.mode = adapt::MODE_CONVT; g.M = N * Ho * Wo; g.N = Cout; g.Cin = Cin; g.taps = kh * kw; g.kw = kw;
    g.H = H; g.W = W; g.Wo = Wo; g.HoWo = Ho * Wo;
    g.sh = stride; g.sw = stride; g.ph = pad; g.pw = pad; g.dh = g.dw = 1;
    g.kstride = H * W; g.img_stride = Cin * H * W;
    return h ? run_rows(lut, x, w, acc, g, s, h->wofs_dev, h->wofs_npad, io) : run_rows(lut, x, w, acc, g, s, nullptr, 0, io);
}

// transposed convolution with plain weights: the cheapest form the geometry allows
int convt_any(const adapt_lut *lut, const int8_t *x, const int8_t *w, int32_t *acc, int N, int Cin, int H, int W, int Cout, int kh,
              int kw, int stride, int pad, hipStream_t s) {
    const int Ho = (H - 1) * stride - 2 * pad + kh, Wo = (W - 1) * stride - 2 * pad + kw;
    const long long M = (long long)N * Ho * Wo;
    if (convt_phases_ok(H, W, kh, kw, stride, pad) && M >= LINES_MIN_ROWS && Cin >= 4) {
        const LinesShape q = convt_phase_shape(lut->bits, Cout, Cin, kh, kw, stride);
        const long long xt_bytes = (long long)N * (H + 2LL * (q.kh - 1)) * (W + 2LL * (q.kw - 1)) * q.Cp;
        const size_t all = q.dt_bytes * stride * stride;
        if (lines_fits(xt_bytes, all, lut->storage)) {
            uint4 *dt[2] = {nullptr, nullptr};
            int32_t *zsum = nullptr;
            int rc = ADAPT_OK;
            hipError_t e = dbg_malloc_async((void **)&zsum, (size_t)Cout * kh * kw * sizeof(int32_t), s);
            for (int half = 0; half <= lut->storage && e == hipSuccess; ++half) e = dbg_malloc_async((void **)&dt[half], all, s);
            if (e != hipSuccess)
                rc = fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "hipMallocAsync(tables): %s", hipGetErrorString(e));
            if (rc == ADAPT_OK) rc = pack_convt(lut, w, q, kh, kw, stride, dt, zsum, s);
            if (rc == ADAPT_OK) rc = lines_conv_transpose2d(lut->bits, lut->storage, q, dt, zsum, x, acc, N, H, W, kh, kw, stride, pad, s, nullptr);
            for (int half = 0; half < 2; ++half)
                if (dt[half]) (void)hipFreeAsync(dt[half], s);
            if (zsum) (void)hipFreeAsync(zsum, s);
            return rc;
        }
    }
    return convt_rows(lut, x, w, acc, N, Cin, H, W, Cout, kh, kw, stride, pad, s);
}

}  // namespace

extern "C" {

int adapt_approx_linear(const adapt_lut *lut, const int8_t *a_dev, const int8_t *w_dev, int32_t *acc_dev, int M,
                        int K, int N, void *stream) {
    int rc = check_lut(lut, "adapt_approx_linear");
    if (rc) return rc;
    if (M < 0 || K < 0 || N < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_linear: negative dimension");
    if (M == 0 || N == 0) return ADAPT_OK;
    if (!acc_dev || (K > 0 && (!a_dev || !w_dev))) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_linear: NULL pointer");
    if ((long long)M * N > 0x7fffffffLL || (long long)M * K > 0x7fffffffLL || (long long)N * K > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "adapt_approx_linear: tensor with more than 2^31-1 elements");
    Geometry g{};
    g.mode = adapt::MODE_GEMM; g.M = M; g.N = N; g.Cin = K; g.taps = 1; g.kw = 1;
    g.H = 1; g.W = 1; g.Wo = 1; g.HoWo = 1; g.sh = g.sw = g.dh = g.dw = 1; g.ph = g.pw = 0;
    g.kstride = 1; g.img_stride = K;
    if (M >= LINES_MIN_ROWS && K >= 8) {
        const LinesShape q = lines_shape(0, lut->bits, N, K, 1, 1);
        if (lines_fits((long long)M * q.Cp, q.dt_bytes, lut->storage))
            return with_temp_tables(lut, w_dev, q, (hipStream_t)stream, [&](uint4 *const dt[2]) {
                return lines_linear(lut->bits, lut->storage, q, dt, a_dev, acc_dev, M, (hipStream_t)stream, nullptr);
            });
    }
    return run_rows(lut, a_dev, w_dev, acc_dev, g, (hipStream_t)stream);
}

int adapt_approx_linear_noalloc(const adapt_lut *lut, const int8_t *a_dev, const int8_t *w_dev, int32_t *acc_dev, int M, int K, int N,
                                void *stream) {
    const char *who = "adapt_approx_linear_noalloc";
    int rc = check_lut(lut, who);
    if (rc) return rc;
    if (M < 0 || K < 0 || N < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: negative dimension", who);
    if (M == 0 || N == 0) return ADAPT_OK;
    if (!acc_dev || (K > 0 && (!a_dev || !w_dev))) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if ((long long)M * N > 0x7fffffffLL || (long long)M * K > 0x7fffffffLL || (long long)N * K > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    const long long need = (long long)K * (((long long)N + 15) / 16 * 16) * (long long)sizeof(uint32_t);
    if (need > (long long)NOALLOC_SCRATCH_BYTES)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: K * (N rounded up to 16) * 4 = %lld bytes of row offsets exceed the %zu bytes of static scratch",
                    who, need, NOALLOC_SCRATCH_BYTES);
    void *scr = nullptr;
    if ((rc = noalloc_scratch(&scr, who))) return rc;
    Geometry g{};
    g.mode = adapt::MODE_GEMM; g.M = M; g.N = N; g.Cin = K; g.taps = 1; g.kw = 1;
    g.H = 1; g.W = 1; g.Wo = 1; g.HoWo = 1; g.sh = g.sw = g.dh = g.dw = 1; g.ph = g.pw = 0;
    g.kstride = 1; g.img_stride = K;
    return run_rows(lut, a_dev, w_dev, acc_dev, g, (hipStream_t)stream, nullptr, 0, nullptr, nullptr, static_cast<uint32_t *>(scr));
}

int adapt_approx_conv2d(const adapt_lut *lut, const int8_t *x_dev, const int8_t *w_dev, int32_t *acc_dev, int N,
                        int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w, int pad_h,
                        int pad_w, int dil_h, int dil_w, int groups, void *stream) {
    int rc = check_lut(lut, "adapt_approx_conv2d");
    if (rc) return rc;
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || kh < 1 || kw < 1 || stride_h < 1 || stride_w < 1 ||
        pad_h < 0 || pad_w < 0 || dil_h < 1 || dil_w < 1 || groups < 1)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv2d: bad dimension");
    if (Cin % groups || Cout % groups) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv2d: channels not divisible by groups");
    const long long Ho = ((long long)H + 2LL * pad_h - (long long)dil_h * (kh - 1) - 1) / stride_h + 1;
    const long long Wo = ((long long)W + 2LL * pad_w - (long long)dil_w * (kw - 1) - 1) / stride_w + 1;
    if ((long long)H + 2LL * pad_h - (long long)dil_h * (kh - 1) - 1 < 0 || (long long)W + 2LL * pad_w - (long long)dil_w * (kw - 1) - 1 < 0)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv2d: filter larger than padded input");
    if (N == 0) return ADAPT_OK;
    if (!x_dev || !w_dev || !acc_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv2d: NULL pointer");
    if ((long long)N * Cout * Ho * Wo > 0x7fffffffLL || (long long)N * Cin * H * W > 0x7fffffffLL ||
        (long long)N * Ho * Wo > 0x7fffffffLL || (long long)Cout * Cin * kh * kw > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "adapt_approx_conv2d: tensor with more than 2^31-1 elements");
    if (groups > 1 && Cout / groups < 8)
        return run_grouped(lut, x_dev, w_dev, acc_dev, N, Cin, H, W, Cout, (int)Ho, (int)Wo, kh, kw, stride_h, stride_w, pad_h, pad_w,
                           dil_h, dil_w, groups, (hipStream_t)stream);
    Geometry g{};
    g.mode = adapt::MODE_CONV; g.M = (int)(N * Ho * Wo); g.N = Cout / groups; g.Cin = Cin / groups; g.taps = kh * kw; g.kw = kw;
    g.H = H; g.W = W; g.Wo = (int)Wo; g.HoWo = (int)(Ho * Wo);
    g.sh = stride_h; g.sw = stride_w; g.ph = pad_h; g.pw = pad_w; g.dh = dil_h; g.dw = dil_w;
    g.kstride = H * W; g.img_stride = Cin * H * W; g.groups = groups;
    if (groups == 1 && g.M >= LINES_MIN_ROWS && Cin >= 4) {
        const LinesShape q = lines_shape(1, lut->bits, Cout, Cin, kh, kw, lut->storage == 0);
        const long long xt_bytes = (long long)N * (H + 2LL * pad_h) * (W + 2LL * pad_w) * q.Cp;
        if (lines_fits(xt_bytes, q.dt_bytes, lut->storage))
            return with_temp_tables(lut, w_dev, q, (hipStream_t)stream, [&](uint4 *const dt[2]) {
                return lines_conv2d(lut->bits, lut->storage, q, dt, x_dev, acc_dev, N, H, W, (int)Ho, (int)Wo, stride_h, stride_w,
                                    pad_h, pad_w, dil_h, dil_w, (hipStream_t)stream, nullptr);
            });
    }
    return run_rows(lut, x_dev, w_dev, acc_dev, g, (hipStream_t)stream);
}

int adapt_approx_conv_transpose2d(const adapt_lut *lut, const int8_t *x_dev, const int8_t *w_dev, int32_t *acc_dev,
                                  int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride, int pad,
                                  void *stream) {
    int rc = check_lut(lut, "adapt_approx_conv_transpose2d");
    if (rc) return rc;
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv_transpose2d: bad dimension");
    const long long Ho = ((long long)H - 1) * stride - 2LL * pad + kh, Wo = ((long long)W - 1) * stride - 2LL * pad + kw;
    if (Ho < 1 || Wo < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv_transpose2d: empty output");
    if (N == 0) return ADAPT_OK;
    if (!x_dev || !w_dev || !acc_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv_transpose2d: NULL pointer");
    if ((long long)N * Cout * Ho * Wo > 0x7fffffffLL || (long long)N * Cin * H * W > 0x7fffffffLL ||
        (long long)Cout * Cin * kh * kw > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "adapt_approx_conv_transpose2d: tensor with more than 2^31-1 elements");
    return convt_any(lut, x_dev, w_dev, acc_dev, N, Cin, H, W, Cout, kh, kw, stride, pad, (hipStream_t)stream);
}


/* ------------------------------------------------------------------ pre-packed weights */

// A linear handle [G Hs][Hs] with G = 4, 3 or 1, even Hs and a single-pass table can serve recurrent time steps
// (adapt_lstm_step_f32 / adapt_gru_step_f32 / adapt_rnn_step_f32): row offsets with the columns in cell order (see
// adapt::RowsParams), from the handle's copy of the weights.
static int pack_cell_offsets(adapt_weights *h, hipStream_t s, const char *who) {
    const int Hs = h->Cin;
    if (h->storage != 0 || Hs % 2 != 0 || h->N % Hs != 0) return ADAPT_OK;
    const int G = h->N / Hs;
    if (G != 4 && G != 3 && G != 1) return ADAPT_OK;
    const size_t n = (size_t)Hs * G * Hs;
    HIP_TRY(dbg_malloc((void **)&h->wofs_cell_dev, n * sizeof(uint32_t)));
    h->cell_G = G;
    adapt::pack_row_offsets_cell_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(h->w8_dev, h->wofs_cell_dev, Hs, G, 1 << (h->bits - 1),
                                                                                  (1 << h->bits) - 1, h->lut->rs * 2);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(ADAPT_ERR_HIP, "%s: pack launch: %s", who, hipGetErrorString(e));
    return ADAPT_OK;
}

static int weights_pack(adapt_weights **out, const adapt_lut *lut, const int8_t *w_dev, int kind, int N, int Cin, int kh,
                        int kw, void *stream, const char *who) {
    if (!out) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: out is NULL", who);
    *out = nullptr;
    int rc = check_lut(lut, who);
    if (rc) return rc;
    if (N < 1 || Cin < 1 || kh < 1 || kw < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    if (!w_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: w_dev is NULL", who);
    if ((long long)N * Cin * kh * kw > 0x7fffffffLL) return fail(ADAPT_ERR_UNSUPPORTED, "%s: more than 2^31-1 weights", who);
    const LinesShape q = lines_shape(kind, lut->bits, N, Cin, kh, kw, lut->storage == 0);
    if (q.dt_bytes * (size_t)(lut->storage + 1) > ((size_t)64 << 30))
        return fail(ADAPT_ERR_OUT_OF_MEMORY, "%s: packed tables would need %zu bytes", who, q.dt_bytes * (size_t)(lut->storage + 1));
    adapt_weights *h = new (std::nothrow) adapt_weights();
    if (!h) return fail(ADAPT_ERR_OUT_OF_MEMORY, "%s: host allocation failed", who);
    h->kind = kind; h->bits = lut->bits; h->storage = lut->storage; h->device = lut->device;
    h->N = N; h->Cin = Cin; h->kh = kh; h->kw = kw; h->Cp = q.Cp; h->Cc = q.Cc; h->n_tiles = q.n_tiles; h->pair_g = q.pair_g;
    h->dt_bytes = q.dt_bytes;
    h->dt_dev[0] = h->dt_dev[1] = nullptr;
    h->stride = 1; h->phased = false; h->zsum_dev = nullptr; h->w8_dev = nullptr; h->lut = lut;
    h->wofs_dev = nullptr; h->wofs_npad = 0; h->wofs1_dev = nullptr; h->wofs1_npad = 0; h->dtq_dev = nullptr; h->dtq_c = 0; h->dtq_bytes = 0; h->wofs_cell_dev = nullptr; h->cell_G = 0;
    {   // copy of the weights (for table orders made later)
        const size_t wbytes = (size_t)N * Cin * kh * kw;
        hipError_t e = dbg_malloc((void **)&h->w8_dev, wbytes);
        if (e == hipSuccess) e = hipMemcpyAsync(h->w8_dev, w_dev, wbytes, hipMemcpyDeviceToDevice, (hipStream_t)stream);
        if (e != hipSuccess) {
            if (h->w8_dev) (void)hipFree(h->w8_dev);
            delete h;
            return fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "%s: copy of the weights: %s", who, hipGetErrorString(e));
        }
    }
    if (kind == 0) {
        h->wofs_npad = ((N + 15) / 16) * 16;
        const size_t pack_n = (size_t)Cin * h->wofs_npad;
        hipError_t e = dbg_malloc((void **)&h->wofs_dev, pack_n * sizeof(uint32_t));
        if (e != hipSuccess) {
            delete h;
            return fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "%s: hipMalloc: %s", who, hipGetErrorString(e));
        }
        adapt::pack_row_offsets_kernel<<<(unsigned)((pack_n + 255) / 256), 256, 0, (hipStream_t)stream>>>(
            w_dev, h->wofs_dev, Cin, N, h->wofs_npad, Cin, 1, (int)adapt::MODE_GEMM, 1 << (lut->bits - 1), (1 << lut->bits) - 1, lut->rs * 2);
    }
    for (int half = 0; half <= lut->storage; ++half) {
        hipError_t e = dbg_malloc((void **)&h->dt_dev[half], q.dt_bytes);
        if (e != hipSuccess) {
            const size_t want = q.dt_bytes;
            adapt_weights_destroy(h);
            return fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "%s: hipMalloc(%zu): %s", who, want,
                        hipGetErrorString(e));
        }
    }
    rc = pack_lines(lut, w_dev, q, h->dt_dev, (hipStream_t)stream);
    if (rc == ADAPT_OK) rc = pack_quad(h, (hipStream_t)stream, who);
    if (rc == ADAPT_OK && kind == 0) rc = pack_cell_offsets(h, (hipStream_t)stream, who);
    if (rc != ADAPT_OK) {
        adapt_weights_destroy(h);
        return rc;
    }
    *out = h;
    return ADAPT_OK;
}

static LinesShape shape_of(const adapt_weights *h) {
    LinesShape q;
    q.kind = h->kind; q.N = h->N; q.Cin = h->Cin; q.kh = h->kh; q.kw = h->kw;
    q.Cp = h->Cp; q.Cc = h->Cc; q.n_tiles = h->n_tiles; q.dt_bytes = h->dt_bytes; q.pair_g = h->pair_g;
    return q;
}

static int check_weights(const adapt_weights *h, int kind, const char *who) {
    if (!h) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: weights handle is NULL", who);
    if (h->kind != kind) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: handle was packed for the other layer type", who);
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != h->device)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: handle belongs to device %d, current device is %d", who, h->device, dev);
    return ADAPT_OK;
}

int adapt_weights_pack_linear(adapt_weights **out, const adapt_lut *lut, const int8_t *w_dev, int K, int N, void *stream) {
    return weights_pack(out, lut, w_dev, 0, N, K, 1, 1, stream, "adapt_weights_pack_linear");
}

int adapt_weights_pack_conv2d(adapt_weights **out, const adapt_lut *lut, const int8_t *w_dev, int Cout, int Cin, int kh, int kw,
                              void *stream) {
    return weights_pack(out, lut, w_dev, 1, Cout, Cin, kh, kw, stream, "adapt_weights_pack_conv2d");
}

int adapt_weights_pack_conv_transpose2d(adapt_weights **out, const adapt_lut *lut, const int8_t *w_dev, int Cin, int Cout, int kh,
                                        int kw, int stride, void *stream) {
    const char *who = "adapt_weights_pack_conv_transpose2d";
    if (!out) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: out is NULL", who);
    *out = nullptr;
    int rc = check_lut(lut, who);
    if (rc) return rc;
    if (Cout < 1 || Cin < 1 || kh < 1 || kw < 1 || stride < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    if (!w_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: w_dev is NULL", who);
    if ((long long)Cout * Cin * kh * kw > 0x7fffffffLL) return fail(ADAPT_ERR_UNSUPPORTED, "%s: more than 2^31-1 weights", who);
    adapt_weights *h = new (std::nothrow) adapt_weights();
    if (!h) return fail(ADAPT_ERR_OUT_OF_MEMORY, "%s: host allocation failed", who);
    h->kind = 2; h->bits = lut->bits; h->storage = lut->storage; h->device = lut->device;
    h->N = Cout; h->Cin = Cin; h->kh = kh; h->kw = kw; h->stride = stride;
    h->Cp = h->Cc = h->n_tiles = 0; h->dt_bytes = 0; h->pair_g = 0;
    h->dt_dev[0] = h->dt_dev[1] = nullptr;
    h->zsum_dev = nullptr; h->w8_dev = nullptr; h->lut = lut;
    h->wofs_dev = nullptr; h->wofs_npad = 0; h->wofs1_dev = nullptr; h->wofs1_npad = 0; h->dtq_dev = nullptr; h->dtq_c = 0; h->dtq_bytes = 0; h->wofs_cell_dev = nullptr; h->cell_G = 0;
    h->phased = kh % stride == 0 && kw % stride == 0 && stride <= 8;
    const size_t wbytes = (size_t)Cout * Cin * kh * kw;
    hipError_t e = dbg_malloc((void **)&h->w8_dev, wbytes);
    if (e == hipSuccess) e = hipMemcpyAsync(h->w8_dev, w_dev, wbytes, hipMemcpyDeviceToDevice, (hipStream_t)stream);
    {   // row offsets for the whole-table kernel, both forms
        const int taps = kh * kw, hoff = 1 << (lut->bits - 1), mask = (1 << lut->bits) - 1;
        h->wofs_npad = ((Cout + 15) / 16) * 16;
        h->wofs1_npad = ((Cout * taps + 15) / 16) * 16;
        const size_t n0 = (size_t)taps * Cin * h->wofs_npad, n1 = (size_t)Cin * h->wofs1_npad;
        if (e == hipSuccess) e = dbg_malloc((void **)&h->wofs_dev, n0 * sizeof(uint32_t));
        if (e == hipSuccess) e = dbg_malloc((void **)&h->wofs1_dev, n1 * sizeof(uint32_t));
        if (e == hipSuccess) {
            adapt::pack_row_offsets_kernel<<<(unsigned)((n0 + 255) / 256), 256, 0, (hipStream_t)stream>>>(
                w_dev, h->wofs_dev, taps * Cin, Cout, h->wofs_npad, Cin, taps, (int)adapt::MODE_CONVT, hoff, mask, lut->rs * 2);
            adapt::pack_row_offsets_kernel<<<(unsigned)((n1 + 255) / 256), 256, 0, (hipStream_t)stream>>>(
                w_dev, h->wofs1_dev, Cin, Cout * taps, h->wofs1_npad, Cin, 1, (int)adapt::MODE_CONVT, hoff, mask, lut->rs * 2);
        }
    }
    if (e == hipSuccess && h->phased) {
        const LinesShape q = convt_phase_shape(lut->bits, Cout, Cin, kh, kw, stride);
        const size_t all = q.dt_bytes * stride * stride;
        if (all * (size_t)(lut->storage + 1) > ((size_t)64 << 30)) {
            h->phased = false;      // too large to hold: this handle keeps to the plain form
        } else {
            h->Cp = q.Cp; h->Cc = q.Cc; h->n_tiles = q.n_tiles; h->dt_bytes = all;
            e = dbg_malloc((void **)&h->zsum_dev, (size_t)Cout * kh * kw * sizeof(int32_t));
            for (int half = 0; half <= lut->storage && e == hipSuccess; ++half) e = dbg_malloc((void **)&h->dt_dev[half], all);
            if (e == hipSuccess) {
                rc = pack_convt(lut, w_dev, q, kh, kw, stride, h->dt_dev, h->zsum_dev, (hipStream_t)stream);
                if (rc == ADAPT_OK) rc = pack_quad(h, (hipStream_t)stream, who);
                if (rc != ADAPT_OK) {
                    adapt_weights_destroy(h);
                    return rc;
                }
            }
        }
    }
    if (e != hipSuccess) {
        adapt_weights_destroy(h);
        return fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "%s: %s", who, hipGetErrorString(e));
    }
    *out = h;
    return ADAPT_OK;
}

int adapt_weights_destroy(adapt_weights *h) {
    if (!h) return ADAPT_OK;
    for (int j = 0; j < 2; ++j)
        if (h->dt_dev[j]) (void)hipFree(h->dt_dev[j]);
    if (h->ws.ptr) (void)hipFree(h->ws.ptr);
    if (h->wofs_dev) (void)hipFree(h->wofs_dev);
    if (h->wofs1_dev) (void)hipFree(h->wofs1_dev);
    if (h->dtq_dev) (void)hipFree(h->dtq_dev);
    if (h->wofs_cell_dev) (void)hipFree(h->wofs_cell_dev);
    if (h->zsum_dev) (void)hipFree(h->zsum_dev);
    if (h->w8_dev) (void)hipFree(h->w8_dev);
    delete h;
    return ADAPT_OK;
}

int adapt_approx_conv_transpose2d_packed(const adapt_weights *h, const int8_t *x_dev, int32_t *acc_dev, int N, int H, int W, int pad,
                                         void *stream) {
    const char *who = "adapt_approx_conv_transpose2d_packed";
    int rc = check_weights(h, 2, who);
    if (rc) return rc;
    if (N < 0 || H < 1 || W < 1 || pad < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    const long long Ho = ((long long)H - 1) * h->stride - 2LL * pad + h->kh, Wo = ((long long)W - 1) * h->stride - 2LL * pad + h->kw;
    if (Ho < 1 || Wo < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: empty output", who);
    if (N == 0) return ADAPT_OK;
    if (!x_dev || !acc_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if ((long long)N * h->N * Ho * Wo > 0x7fffffffLL || (long long)N * h->Cin * H * W > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    if (h->phased && convt_phases_ok(H, W, h->kh, h->kw, h->stride, pad)) {
        LinesShape q = convt_phase_shape(h->bits, h->N, h->Cin, h->kh, h->kw, h->stride);
        const long long xt_bytes = (long long)N * (H + 2LL * (q.kh - 1)) * (W + 2LL * (q.kw - 1)) * q.Cp;
        if (xt_bytes < 0x7fffff00LL)
            return lines_conv_transpose2d(h->bits, h->storage, q, h->dt_dev, h->zsum_dev, x_dev, acc_dev, N, H, W, h->kh, h->kw,
                                          h->stride, pad, (hipStream_t)stream, &h->ws, nullptr, h);
    }
    // geometries outside the phase form (a single input pixel, output sizes that are no multiple of the stride)
    return convt_rows(h->lut, x_dev, h->w8_dev, acc_dev, N, h->Cin, H, W, h->N, h->kh, h->kw, h->stride, pad, (hipStream_t)stream, h);
}

int adapt_plan_packed(int kind, int bits, int storage, int Cout, int Cin, int kh, int kw, int stride, int rows, int Wo, int sw, int cu,
                      int *kernel, int *rows_per_workgroup, int *ksplit, int *steps, int *workgroups) {
    const char *who = "adapt_plan_packed";
    if (kind < 0 || kind > 2 || bits < 2 || bits > 8 || storage < 0 || storage > 1 || Cout < 1 || Cin < 1 || kh < 1 || kw < 1 || stride < 1 ||
        rows < 1 || Wo < 1 || sw < 1)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad argument", who);
    int k = 0, rpw = 0, ks = 1, st = 0, wg = 0;
    const bool phased = kind == 2 && kh % stride == 0 && kw % stride == 0;
    if (rows < LINES_MIN_ROWS && kind == 0) {
        k = -1;                                 // whole-table kernel (lut_rows_kernel)
    } else if (kind == 2 && !phased) {
        k = -1;
    } else {
        const LinesShape q = kind == 2 ? convt_phase_shape(bits, Cout, Cin, kh, kw, stride) : lines_shape(kind, bits, Cout, Cin, kh, kw, storage == 0);
        const int phases = kind == 2 ? stride * stride : 1;
        const bool quad_tables = storage == 0 && q.Cp % adapt::QUAD_STEP == 0;
        const LinesPlan pl = plan_product(q, bits, storage, rows, phases, Wo, sw, quad_tables, cu > 0 ? cu : 0);
        k = pl.kernel; rpw = pl.rows_per_wg(); ks = pl.ksplit;
        st = pl.kernel == LK_QUAD ? q.kh * q.kw * (q.Cp / adapt::QUAD_STEP) : q.k_taps() * q.k_cc();
        wg = ((rows + rpw - 1) / rpw) * q.n_tiles * phases * ks;
    }
    if (kernel) *kernel = k;
    if (rows_per_workgroup) *rows_per_workgroup = rpw;
    if (ksplit) *ksplit = ks;
    if (steps) *steps = st;
    if (workgroups) *workgroups = wg;
    return ADAPT_OK;
}

int adapt_approx_linear_packed(const adapt_weights *h, const int8_t *a_dev, int32_t *acc_dev, int M, void *stream) {
    int rc = check_weights(h, 0, "adapt_approx_linear_packed");
    if (rc) return rc;
    if (M < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_linear_packed: negative M");
    if (M == 0) return ADAPT_OK;
    if (!a_dev || !acc_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_linear_packed: NULL pointer");
    if ((long long)M * h->Cp >= 0x7fffff00LL || (long long)M * h->N > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "adapt_approx_linear_packed: tensor with more than 2^31-1 elements");
    if (M < LINES_MIN_ROWS) {       // too few rows to amortise streaming the derived tables: whole-table kernel
        Geometry g{};
        g.mode = adapt::MODE_GEMM; g.M = M; g.N = h->N; g.Cin = h->Cin; g.taps = 1; g.kw = 1;
        g.H = 1; g.W = 1; g.Wo = 1; g.HoWo = 1; g.sh = g.sw = g.dh = g.dw = 1; g.ph = g.pw = 0;
        g.kstride = 1; g.img_stride = h->Cin;
        return run_rows(h->lut, a_dev, nullptr, acc_dev, g, (hipStream_t)stream, h->wofs_dev, h->wofs_npad);
    }
    return lines_linear(h->bits, h->storage, shape_of(h), h->dt_dev, a_dev, acc_dev, M, (hipStream_t)stream, &h->ws, nullptr, h);
}

int adapt_approx_conv2d_packed(const adapt_weights *h, const int8_t *x_dev, int32_t *acc_dev, int N, int H, int W, int stride_h,
                               int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, void *stream) {
    int rc = check_weights(h, 1, "adapt_approx_conv2d_packed");
    if (rc) return rc;
    if (N < 0 || H < 1 || W < 1 || stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 || dil_h < 1 || dil_w < 1)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv2d_packed: bad dimension");
    const long long eh = (long long)H + 2LL * pad_h - (long long)dil_h * (h->kh - 1) - 1;
    const long long ew = (long long)W + 2LL * pad_w - (long long)dil_w * (h->kw - 1) - 1;
    if (eh < 0 || ew < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv2d_packed: filter larger than padded input");
    const long long Ho = eh / stride_h + 1, Wo = ew / stride_w + 1;
    if (N == 0) return ADAPT_OK;
    if (!x_dev || !acc_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv2d_packed: NULL pointer");
    const long long xt_bytes = (long long)N * (H + 2LL * pad_h) * (W + 2LL * pad_w) * h->Cp;
    if (xt_bytes >= 0x7fffff00LL || (long long)N * h->N * Ho * Wo > 0x7fffffffLL || (long long)N * Ho * Wo > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "adapt_approx_conv2d_packed: tensor with more than 2^31-1 elements");
    return lines_conv2d(h->bits, h->storage, shape_of(h), h->dt_dev, x_dev, acc_dev, N, H, W, (int)Ho, (int)Wo, stride_h, stride_w,
                        pad_h, pad_w, dil_h, dil_w, (hipStream_t)stream, &h->ws, nullptr, h);
}

/* ------------------------------------------------------------------ whole layers, fp32 in and out */

// y_optional: the caller chains into a next layer and may want nothing but that layer's input copy
static int layer_io(LayerIO *io, const adapt_weights *h, const float *x_dev, const float *y_dev, float s_x, float s_out,
                    const float *s_out_vec_dev, const float *bias_dev, int act, const char *who, bool y_optional = false) {
    if (!x_dev || (!y_dev && !y_optional)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if (!(s_x > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_x must be > 0", who);
    if (act < 0 || act > 2) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: act=%d not in {0, 1, 2}", who, act);
    io->xf = x_dev; io->s_x = s_x; io->Q = (float)((1 << (h->bits - 1)) - 1);
    io->deq = 1; io->act = act; io->s_out = s_out; io->s_out_vec = s_out_vec_dev; io->bias = bias_dev;
    return ADAPT_OK;
}

// int8 copy of fp32 activations in the handle's workspace, for the whole-table kernel
static int quantize_into_ws(const adapt_weights *h, const LayerIO &io, size_t n, hipStream_t s, int8_t **q) {
    int rc = ws_get(&h->ws, n + 64, s, (void **)q);
    if (rc) return rc;
    const int vec = (aligned16(io.xf) && aligned16(*q)) ? 1 : 0;
    adapt::quantize_kernel<<<ew_grid(n / 16 + 1), adapt::EW_THREADS, 0, s>>>(io.xf, *q, n, io.s_x, io.Q, vec);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_linear_layer_f32(const adapt_weights *h, const float *x_dev, float *y_dev, int M, float s_x, float s_out,
                           const float *s_out_vec_dev, const float *bias_dev, int act, void *stream) {
    const char *who = "adapt_linear_layer_f32";
    int rc = check_weights(h, 0, who);
    if (rc) return rc;
    if (M < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: negative M", who);
    if (M == 0) return ADAPT_OK;
    LayerIO io;
    if ((rc = layer_io(&io, h, x_dev, y_dev, s_x, s_out, s_out_vec_dev, bias_dev, act, who))) return rc;
    if ((long long)M * h->Cp >= 0x7fffff00LL || (long long)M * h->N > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    hipStream_t s = (hipStream_t)stream;
    int32_t *out = reinterpret_cast<int32_t *>(y_dev);
    if (M < LINES_MIN_ROWS) {
        int8_t *q = nullptr;
        if ((rc = quantize_into_ws(h, io, (size_t)M * h->Cin, s, &q))) return rc;
        Geometry g{};
        g.mode = adapt::MODE_GEMM; g.M = M; g.N = h->N; g.Cin = h->Cin; g.taps = 1; g.kw = 1;
        g.H = 1; g.W = 1; g.Wo = 1; g.HoWo = 1; g.sh = g.sw = g.dh = g.dw = 1; g.ph = g.pw = 0;
        g.kstride = 1; g.img_stride = h->Cin;
        return run_rows(h->lut, q, nullptr, out, g, s, h->wofs_dev, h->wofs_npad, &io);
    }
    return lines_linear(h->bits, h->storage, shape_of(h), h->dt_dev, nullptr, out, M, s, &h->ws, &io, h);
}

// geometry shared by the convolution layer calls
struct ConvGeo {
    long long Ho, Wo;
};

static int conv_geo(const adapt_weights *h, int N, int H, int W, int sh, int sw, int ph, int pw, int dh, int dw, ConvGeo *g, const char *who) {
    if (N < 0 || H < 1 || W < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    const long long eh = (long long)H + 2LL * ph - (long long)dh * (h->kh - 1) - 1;
    const long long ew = (long long)W + 2LL * pw - (long long)dw * (h->kw - 1) - 1;
    if (eh < 0 || ew < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: filter larger than padded input", who);
    g->Ho = eh / sh + 1; g->Wo = ew / sw + 1;
    const long long xt_bytes = (long long)N * (H + 2LL * ph) * (W + 2LL * pw) * h->Cp;
    if (xt_bytes >= 0x7fffff00LL || (long long)N * h->N * g->Ho * g->Wo > 0x7fffffffLL || (long long)N * g->Ho * g->Wo > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    return ADAPT_OK;
}

// x_dev == nullptr: the input copy is already in the handle's prepared workspace (written by the layer before);
// next != nullptr: also write the output as next's input copy, quantised with s_next
static int conv2d_layer(const adapt_weights *h, const float *x_dev, float *y_dev, int N, int H, int W, int stride_h, int stride_w,
                        int pad_h, int pad_w, int dil_h, int dil_w, float s_x, float s_out, const float *s_out_vec_dev,
                        const float *bias_dev, const float *residual_dev, int act, const adapt_weights *next, float s_next, void *stream,
                        const char *who) {
    int rc = check_weights(h, 1, who);
    if (rc) return rc;
    ConvGeo g;
    if ((rc = conv_geo(h, N, H, W, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, &g, who))) return rc;
    if (N == 0) return ADAPT_OK;
    const bool input_ready = x_dev == nullptr;
    if (input_ready) {
        const auto &ci = h->chain_in;
        if (!ci.valid || ci.N != N || ci.H != H || ci.W != W || ci.sh != stride_h || ci.sw != stride_w || ci.ph != pad_h || ci.pw != pad_w ||
            ci.dh != dil_h || ci.dw != dil_w)
            return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: x_dev is NULL but the handle was not prepared for this geometry", who);
    }
    LayerIO io;
    if ((rc = layer_io(&io, h, input_ready ? reinterpret_cast<const float *>(h) : x_dev, y_dev, s_x, s_out, s_out_vec_dev, bias_dev, act, who,
                       next != nullptr)))
        return rc;
    if (input_ready) io.xf = nullptr;
    io.resid = residual_dev;
    if (residual_dev && residual_dev == y_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: residual_dev must not alias y_dev", who);
    if (next) {
        if ((rc = check_weights(next, 1, who))) return rc;
        if (next == h) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: a layer cannot chain into itself (one workspace per handle)", who);
        const auto &ci = next->chain_in;
        if (!ci.valid || ci.N != N || ci.H != g.Ho || ci.W != g.Wo || next->Cin != h->N || !next->ws.ptr)
            return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: the next layer was not prepared for this layer's output", who);
        if (!(s_next > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_next must be > 0", who);
        io.chain.buf = static_cast<int8_t *>(next->ws.ptr);
        io.chain.xmajor = ci.xmajor; io.chain.Hp = ci.H + 2 * ci.ph; io.chain.Wp = ci.W + 2 * ci.pw; io.chain.Cp = next->Cp;
        io.chain.ph = ci.ph; io.chain.pw = ci.pw;
        io.chain.scale = s_next; io.chain.Q = (float)((1 << (next->bits - 1)) - 1); io.chain.mask = (1u << next->bits) - 1u;
        io.chain_wo = (int)g.Wo;
    }
    rc = lines_conv2d(h->bits, h->storage, shape_of(h), h->dt_dev, nullptr, reinterpret_cast<int32_t *>(y_dev), N, H, W, (int)g.Ho,
                      (int)g.Wo, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, (hipStream_t)stream, &h->ws, &io, h, input_ready);
    // (only a call that has written next's copy may say what the copy holds)
    if (rc == ADAPT_OK && next) next->chain_in.nonneg = act == 1;
    return rc;
}

int adapt_conv2d_layer_f32(const adapt_weights *h, const float *x_dev, float *y_dev, int N, int H, int W, int stride_h, int stride_w,
                           int pad_h, int pad_w, int dil_h, int dil_w, float s_x, float s_out, const float *s_out_vec_dev,
                           const float *bias_dev, const float *residual_dev, int act, void *stream) {
    const char *who = "adapt_conv2d_layer_f32";
    if (!x_dev && N > 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    return conv2d_layer(h, x_dev, y_dev, N, H, W, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, s_x, s_out, s_out_vec_dev, bias_dev,
                        residual_dev, act, nullptr, 1.0f, stream, who);
}

int adapt_conv2d_chain_prepare(const adapt_weights *h, int N, int H, int W, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h,
                               int dil_w, void *stream) {
    const char *who = "adapt_conv2d_chain_prepare";
    int rc = check_weights(h, 1, who);
    if (rc) return rc;
    ConvGeo g;
    if ((rc = conv_geo(h, N, H, W, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, &g, who))) return rc;
    h->chain_in.valid = false;
    if (N == 0) return ADAPT_OK;
    // the layout decisions of lines_conv2d
    const LinesShape q = shape_of(h);
    const int M = (int)(N * g.Ho * g.Wo);
    const LinesPlan plan = plan_product(q, h->bits, h->storage, M, 1, (int)g.Wo, stride_w, h->dtq_dev != nullptr);
    const int xmajor = plan.xmajor;
    const size_t xt_bytes = (size_t)N * (H + 2 * pad_h) * (W + 2 * pad_w) * q.Cp;
    const size_t copy_bytes = ((xt_bytes + 64 + 255) / 256) * 256;
    const size_t part_bytes = plan_partial_bytes(plan, (size_t)M * q.N);
    int8_t *xt = nullptr;
    if ((rc = ws_get(&h->ws, copy_bytes + part_bytes, (hipStream_t)stream, (void **)&xt))) return rc;
    adapt::fill_u32_kernel<<<ew_grid(copy_bytes / 4), 256, 0, (hipStream_t)stream>>>(reinterpret_cast<uint32_t *>(xt), 0u, copy_bytes / 4);
    HIP_TRY(hipGetLastError());
    auto &ci = h->chain_in;
    ci.N = N; ci.H = H; ci.W = W; ci.sh = stride_h; ci.sw = stride_w; ci.ph = pad_h; ci.pw = pad_w; ci.dh = dil_h; ci.dw = dil_w;
    ci.xmajor = xmajor; ci.nonneg = false; ci.valid = true;
    return ADAPT_OK;
}

int adapt_conv2d_layer_chain_f32(const adapt_weights *h, const float *x_dev, float *y_dev, int N, int H, int W, int stride_h,
                                 int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, float s_x, float s_out,
                                 const float *s_out_vec_dev, const float *bias_dev, const float *residual_dev, int act,
                                 const adapt_weights *next, float s_next, void *stream) {
    return conv2d_layer(h, x_dev, y_dev, N, H, W, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, s_x, s_out, s_out_vec_dev, bias_dev,
                        residual_dev, act, next, s_next, stream, "adapt_conv2d_layer_chain_f32");
}

int adapt_conv2d_grouped_layer_f32(const adapt_lut *lut, const float *x_dev, const int8_t *w_dev, float *y_dev, int N, int Cin, int H,
                                   int W, int Cout, int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h,
                                   int dil_w, int groups, float s_x, float s_out, const float *s_out_vec_dev, const float *bias_dev,
                                   int act, const adapt_weights *next, float s_next, void *stream) {
    const char *who = "adapt_conv2d_grouped_layer_f32";
    int rc = check_lut(lut, who);
    if (rc) return rc;
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || kh < 1 || kw < 1 || stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 ||
        dil_h < 1 || dil_w < 1 || groups < 1)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    if (Cin % groups || Cout % groups) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: channels not divisible by groups", who);
    if (act < 0 || act > 2) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: act=%d not in {0, 1, 2}", who, act);
    if (!(s_x > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_x must be > 0", who);
    const long long eh = (long long)H + 2LL * pad_h - (long long)dil_h * (kh - 1) - 1, ew = (long long)W + 2LL * pad_w - (long long)dil_w * (kw - 1) - 1;
    if (eh < 0 || ew < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: filter larger than padded input", who);
    const long long Ho = eh / stride_h + 1, Wo = ew / stride_w + 1;
    if (N == 0) return ADAPT_OK;
    if (!x_dev || !w_dev || (!y_dev && !next)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if ((long long)N * Cout * Ho * Wo > 0x7fffffffLL || (long long)N * Cin * H * W > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    const bool wide_groups = Cout / groups >= 8 || groups == 1;     // whole-table kernel over a group dimension instead of the tiled kernel
    if (wide_groups && !y_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: groups of 8 or more output channels need y_dev (the sums are finished in place)", who);
    if (wide_groups && ((long long)N * Ho * Wo > 0x7fffffffLL || (long long)Cout * (Cin / groups) * kh * kw > 0x7fffffffLL))
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    LayerIO io;
    io.xf = x_dev; io.s_x = s_x; io.Q = (float)((1 << (lut->bits - 1)) - 1);
    io.deq = 1; io.act = act; io.s_out = s_out; io.s_out_vec = s_out_vec_dev; io.bias = bias_dev;
    if (next) {
        if ((rc = check_weights(next, 1, who))) return rc;
        const auto &ci = next->chain_in;
        if (!ci.valid || ci.N != N || ci.H != Ho || ci.W != Wo || next->Cin != Cout || !next->ws.ptr)
            return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: the next layer was not prepared for this layer's output", who);
        if (!(s_next > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_next must be > 0", who);
        io.chain.buf = static_cast<int8_t *>(next->ws.ptr);
        io.chain.xmajor = ci.xmajor; io.chain.Hp = ci.H + 2 * ci.ph; io.chain.Wp = ci.W + 2 * ci.pw; io.chain.Cp = next->Cp;
        io.chain.ph = ci.ph; io.chain.pw = ci.pw;
        io.chain.scale = s_next; io.chain.Q = (float)((1 << (next->bits - 1)) - 1); io.chain.mask = (1u << next->bits) - 1u;
        io.chain_wo = (int)Wo;
    }
    if (wide_groups) {
        // quantise into a stream-ordered temporary, then the product of adapt_approx_conv2d with the layer's finishing
        // pass (inside the product kernel when it can, else in place afterwards, which also writes next's copy)
        hipStream_t s = (hipStream_t)stream;
        const size_t n = (size_t)N * Cin * H * W;
        int8_t *q8 = nullptr;
        HIP_TRY(dbg_malloc_async((void **)&q8, n + 64, s));
        adapt::quantize_kernel<<<ew_grid(n / 16 + 1), adapt::EW_THREADS, 0, s>>>(x_dev, q8, n, s_x, io.Q, (aligned16(x_dev) && aligned16(q8)) ? 1 : 0);
        hipError_t qe = hipGetLastError();
        rc = qe == hipSuccess ? ADAPT_OK : fail(ADAPT_ERR_HIP, "%s: quantise launch: %s", who, hipGetErrorString(qe));
        if (rc == ADAPT_OK) {
            Geometry g{};
            g.mode = adapt::MODE_CONV; g.M = (int)(N * Ho * Wo); g.N = Cout / groups; g.Cin = Cin / groups; g.taps = kh * kw; g.kw = kw;
            g.H = H; g.W = W; g.Wo = (int)Wo; g.HoWo = (int)(Ho * Wo);
            g.sh = stride_h; g.sw = stride_w; g.ph = pad_h; g.pw = pad_w; g.dh = dil_h; g.dw = dil_w;
            g.kstride = H * W; g.img_stride = Cin * H * W; g.groups = groups;
            io.xf = nullptr;
            rc = run_rows(lut, q8, w_dev, reinterpret_cast<int32_t *>(y_dev), g, s, nullptr, 0, &io);
        }
        hipError_t fe = hipFreeAsync(q8, s);
        if (rc == ADAPT_OK && fe != hipSuccess) rc = fail(ADAPT_ERR_HIP, "hipFreeAsync: %s", hipGetErrorString(fe));
    } else {
        rc = run_grouped(lut, nullptr, w_dev, reinterpret_cast<int32_t *>(y_dev), N, Cin, H, W, Cout, (int)Ho, (int)Wo, kh, kw, stride_h,
                         stride_w, pad_h, pad_w, dil_h, dil_w, groups, (hipStream_t)stream, &io);
    }
    if (rc == ADAPT_OK && next) next->chain_in.nonneg = act == 1;
    return rc;
}

int adapt_conv_transpose2d_layer_f32(const adapt_weights *h, const float *x_dev, float *y_dev, int N, int H, int W, int pad, float s_x,
                                     float s_out, const float *s_out_vec_dev, const float *bias_dev, int act, void *stream) {
    const char *who = "adapt_conv_transpose2d_layer_f32";
    int rc = check_weights(h, 2, who);
    if (rc) return rc;
    if (N < 0 || H < 1 || W < 1 || pad < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    const long long Ho = ((long long)H - 1) * h->stride - 2LL * pad + h->kh, Wo = ((long long)W - 1) * h->stride - 2LL * pad + h->kw;
    if (Ho < 1 || Wo < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: empty output", who);
    if (N == 0) return ADAPT_OK;
    LayerIO io;
    if ((rc = layer_io(&io, h, x_dev, y_dev, s_x, s_out, s_out_vec_dev, bias_dev, act, who))) return rc;
    if ((long long)N * h->N * Ho * Wo > 0x7fffffffLL || (long long)N * h->Cin * H * W > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    hipStream_t s = (hipStream_t)stream;
    int32_t *out = reinterpret_cast<int32_t *>(y_dev);
    if (h->phased && convt_phases_ok(H, W, h->kh, h->kw, h->stride, pad)) {
        LinesShape q = convt_phase_shape(h->bits, h->N, h->Cin, h->kh, h->kw, h->stride);
        const long long xt_bytes = (long long)N * (H + 2LL * (q.kh - 1)) * (W + 2LL * (q.kw - 1)) * q.Cp;
        if (xt_bytes < 0x7fffff00LL)
            return lines_conv_transpose2d(h->bits, h->storage, q, h->dt_dev, h->zsum_dev, nullptr, out, N, H, W, h->kh, h->kw, h->stride,
                                          pad, s, &h->ws, &io, h);
    }
    int8_t *q8 = nullptr;
    if ((rc = quantize_into_ws(h, io, (size_t)N * h->Cin * H * W, s, &q8))) return rc;
    return convt_rows(h->lut, q8, h->w8_dev, out, N, h->Cin, H, W, h->N, h->kh, h->kw, h->stride, pad, s, h, &io);
}

// geometry of the phase form of a transposed convolution layer call, or UNSUPPORTED
static int convt_chain_geo(const adapt_weights *h, int N, int H, int W, int pad, LinesShape *q, long long *Ho, long long *Wo, const char *who) {
    if (N < 0 || H < 1 || W < 1 || pad < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    *Ho = ((long long)H - 1) * h->stride - 2LL * pad + h->kh; *Wo = ((long long)W - 1) * h->stride - 2LL * pad + h->kw;
    if (*Ho < 1 || *Wo < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: empty output", who);
    if ((long long)N * h->N * *Ho * *Wo > 0x7fffffffLL || (long long)N * h->Cin * H * W > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    if (!(h->phased && convt_phases_ok(H, W, h->kh, h->kw, h->stride, pad)))
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: only geometries that take the phase form (filter a multiple of the stride, more than one input pixel)", who);
    *q = convt_phase_shape(h->bits, h->N, h->Cin, h->kh, h->kw, h->stride);
    const long long xt_bytes = (long long)N * (H + 2LL * (q->kh - 1)) * (W + 2LL * (q->kw - 1)) * q->Cp;
    if (xt_bytes >= 0x7fffff00LL) return fail(ADAPT_ERR_UNSUPPORTED, "%s: input copy of 2 GiB or more", who);
    return ADAPT_OK;
}

int adapt_conv_transpose2d_chain_prepare(const adapt_weights *h, int N, int H, int W, int pad, void *stream) {
    const char *who = "adapt_conv_transpose2d_chain_prepare";
    int rc = check_weights(h, 2, who);
    if (rc) return rc;
    h->chain_in.valid = false;
    LinesShape q;
    long long Ho, Wo;
    if ((rc = convt_chain_geo(h, N, H, W, pad, &q, &Ho, &Wo, who))) return rc;
    if (N == 0) return ADAPT_OK;
    // the layout decisions of lines_conv_transpose2d
    const int st = h->stride, Ty = q.kh, Tx = q.kw;
    const int Qy = (int)(Ho / st), Qx = (int)(Wo / st), M = N * Qy * Qx;
    const LinesPlan plan = plan_product(q, h->bits, h->storage, M, st * st, Qx, 1, h->dtq_dev != nullptr);
    const int xmajor = plan.xmajor;
    const size_t xt_bytes = (size_t)N * (H + 2 * (Ty - 1)) * (W + 2 * (Tx - 1)) * q.Cp;
    const size_t copy_bytes = ((xt_bytes + 64 + 255) / 256) * 256;
    const size_t part_bytes = plan_partial_bytes(plan, (size_t)N * q.N * Ho * Wo);
    int8_t *xt = nullptr;
    if ((rc = ws_get(&h->ws, copy_bytes + part_bytes, (hipStream_t)stream, (void **)&xt))) return rc;
    adapt::fill_u32_kernel<<<ew_grid(copy_bytes / 4), 256, 0, (hipStream_t)stream>>>(reinterpret_cast<uint32_t *>(xt), 0u, copy_bytes / 4);
    HIP_TRY(hipGetLastError());
    auto &ci = h->chain_in;
    ci.N = N; ci.H = H; ci.W = W; ci.sh = ci.sw = st; ci.ph = Ty - 1; ci.pw = Tx - 1; ci.dh = ci.dw = pad;     // (dh, dw: the layer's padding)
    ci.xmajor = xmajor; ci.nonneg = false; ci.valid = true;
    return ADAPT_OK;
}

int adapt_conv_transpose2d_layer_chain_f32(const adapt_weights *h, const float *x_dev, float *y_dev, int N, int H, int W, int pad, float s_x,
                                           float s_out, const float *s_out_vec_dev, const float *bias_dev, int act,
                                           const adapt_weights *next, float s_next, void *stream) {
    const char *who = "adapt_conv_transpose2d_layer_chain_f32";
    int rc = check_weights(h, 2, who);
    if (rc) return rc;
    const bool input_ready = x_dev == nullptr;
    LinesShape q;
    long long Ho = 0, Wo = 0;
    const bool phase_form = h->phased && H >= 1 && W >= 1 && pad >= 0 && convt_phases_ok(H, W, h->kh, h->kw, h->stride, pad);
    if (input_ready || phase_form) {
        if ((rc = convt_chain_geo(h, N, H, W, pad, &q, &Ho, &Wo, who))) return rc;
    } else {
        if (N < 0 || H < 1 || W < 1 || pad < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
        Ho = ((long long)H - 1) * h->stride - 2LL * pad + h->kh; Wo = ((long long)W - 1) * h->stride - 2LL * pad + h->kw;
        if (Ho < 1 || Wo < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: empty output", who);
        if ((long long)N * h->N * Ho * Wo > 0x7fffffffLL || (long long)N * h->Cin * H * W > 0x7fffffffLL)
            return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    }
    if (N == 0) return ADAPT_OK;
    if (input_ready) {
        const auto &ci = h->chain_in;
        if (!ci.valid || ci.N != N || ci.H != H || ci.W != W || ci.dh != pad || ci.sh != h->stride)
            return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: x_dev is NULL but the handle was not prepared for this geometry", who);
    }
    LayerIO io;
    if ((rc = layer_io(&io, h, input_ready ? reinterpret_cast<const float *>(h) : x_dev, y_dev, s_x, s_out, s_out_vec_dev, bias_dev, act, who,
                       next != nullptr)))
        return rc;
    if (input_ready) io.xf = nullptr;
    if (next) {
        if (!next || (next->kind != 1 && next->kind != 2)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: next is not a convolution handle", who);
        if ((rc = check_weights(next, next->kind, who))) return rc;
        if (next == h) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: a layer cannot chain into itself (one workspace per handle)", who);
        const auto &ci = next->chain_in;
        if (!ci.valid || ci.N != N || ci.H != Ho || ci.W != Wo || next->Cin != h->N || !next->ws.ptr)
            return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: the next layer was not prepared for this layer's output", who);
        if (!(s_next > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_next must be > 0", who);
        io.chain.buf = static_cast<int8_t *>(next->ws.ptr);
        io.chain.xmajor = ci.xmajor; io.chain.Hp = ci.H + 2 * ci.ph; io.chain.Wp = ci.W + 2 * ci.pw; io.chain.Cp = next->Cp;
        io.chain.ph = ci.ph; io.chain.pw = ci.pw;
        io.chain.scale = s_next; io.chain.Q = (float)((1 << (next->bits - 1)) - 1); io.chain.mask = (1u << next->bits) - 1u;
        io.chain_wo = (int)Wo;
    }
    hipStream_t s = (hipStream_t)stream;
    int32_t *out = reinterpret_cast<int32_t *>(y_dev);
    if (input_ready || phase_form) {
        rc = lines_conv_transpose2d(h->bits, h->storage, q, h->dt_dev, h->zsum_dev, nullptr, out, N, H, W, h->kh, h->kw, h->stride, pad, s,
                                    &h->ws, &io, h, input_ready);
    } else {
        if (!y_dev) return fail(ADAPT_ERR_UNSUPPORTED, "%s: this geometry finishes its sums in a separate pass over the output: y_dev is needed", who);
        int8_t *q8 = nullptr;
        if ((rc = quantize_into_ws(h, io, (size_t)N * h->Cin * H * W, s, &q8))) return rc;
        rc = convt_rows(h->lut, q8, h->w8_dev, out, N, h->Cin, H, W, h->N, h->kh, h->kw, h->stride, pad, s, h, &io);
    }
    if (rc == ADAPT_OK && next) next->chain_in.nonneg = act == 1;
    return rc;
}

/* ------------------------------------------------------------------ LSTM time step in one kernel */

int adapt_lstm_step_f32(const adapt_weights *h, const int8_t *qh_dev, const int32_t *acc_ih_dev, float s_ih, float s_hh, float s_h,
                        const float *bias_dev, float *c_dev, float *h_dev, int8_t *qh_next_dev, int B, int Hs, void *stream) {
    const char *who = "adapt_lstm_step_f32";
    int rc = check_weights(h, 0, who);
    if (rc) return rc;
    if (B < 1 || Hs < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    if (h->N != 4 * Hs || h->Cin != Hs) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: handle is not a packed [4 Hs][Hs] matrix", who);
    if (!(s_h > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_h must be > 0", who);
    if (!qh_dev || !acc_ih_dev || !c_dev || !h_dev || !qh_next_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if (qh_dev == qh_next_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: qh_next_dev must not alias qh_dev", who);
    if (h->storage != 0 || Hs % 2 != 0 || (long long)B * 4 * Hs > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: shape outside the fused kernel (Hs even, single-pass table)", who);
    hipStream_t s = (hipStream_t)stream;
    if (!h->wofs_cell_dev || h->cell_G != 4) return fail(ADAPT_ERR_UNSUPPORTED, "%s: the handle holds no cell-order offsets", who);
    Geometry g{};
    g.mode = adapt::MODE_GEMM; g.M = B; g.N = 4 * Hs; g.Cin = Hs; g.taps = 1; g.kw = 1;
    g.H = 1; g.W = 1; g.Wo = 1; g.HoWo = 1; g.sh = g.sw = g.dh = g.dw = 1; g.ph = g.pw = 0;
    g.kstride = 1; g.img_stride = Hs;
    LstmStep ls;
    ls.Hs = Hs; ls.acc_ih = acc_ih_dev; ls.bias = bias_dev; ls.c = c_dev; ls.h = h_dev; ls.qh_next = qh_next_dev;
    ls.s_ih = s_ih; ls.s_hh = s_hh; ls.s_h = s_h; ls.Qh = (float)((1 << (h->bits - 1)) - 1);
    return run_rows(h->lut, qh_dev, nullptr, nullptr, g, s, h->wofs_cell_dev, 4 * Hs, nullptr, &ls);
}

int adapt_gru_step_f32(const adapt_weights *h, const int8_t *qh_dev, const int32_t *acc_ih_dev, float s_ih, float s_hh, float s_h,
                       const float *b_ih_dev, const float *b_hh_dev, const float *h_prev_dev, float *h_dev, int8_t *qh_next_dev, int B,
                       int Hs, void *stream) {
    const char *who = "adapt_gru_step_f32";
    int rc = check_weights(h, 0, who);
    if (rc) return rc;
    if (B < 1 || Hs < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    if (h->N != 3 * Hs || h->Cin != Hs) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: handle is not a packed [3 Hs][Hs] matrix", who);
    if (!(s_h > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_h must be > 0", who);
    if (!qh_dev || !acc_ih_dev || !h_prev_dev || !h_dev || !qh_next_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if (qh_dev == qh_next_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: qh_next_dev must not alias qh_dev", who);
    if (h->storage != 0 || Hs % 2 != 0 || (long long)B * 3 * Hs > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: shape outside the fused kernel (Hs even, single-pass table)", who);
    hipStream_t s = (hipStream_t)stream;
    if (!h->wofs_cell_dev || h->cell_G != 3) return fail(ADAPT_ERR_UNSUPPORTED, "%s: the handle holds no cell-order offsets", who);
    Geometry g{};
    g.mode = adapt::MODE_GEMM; g.M = B; g.N = 3 * Hs; g.Cin = Hs; g.taps = 1; g.kw = 1;
    g.H = 1; g.W = 1; g.Wo = 1; g.HoWo = 1; g.sh = g.sw = g.dh = g.dw = 1; g.ph = g.pw = 0;
    g.kstride = 1; g.img_stride = Hs;
    LstmStep ls;
    ls.kind = 2;
    ls.Hs = Hs; ls.acc_ih = acc_ih_dev; ls.bias = b_ih_dev; ls.bias_hh = b_hh_dev; ls.c = nullptr; ls.h = h_dev; ls.h_prev = h_prev_dev;
    ls.qh_next = qh_next_dev;
    ls.s_ih = s_ih; ls.s_hh = s_hh; ls.s_h = s_h; ls.Qh = (float)((1 << (h->bits - 1)) - 1);
    return run_rows(h->lut, qh_dev, nullptr, nullptr, g, s, h->wofs_cell_dev, 3 * Hs, nullptr, &ls);
}

int adapt_rnn_step_f32(const adapt_weights *h, const int8_t *qh_dev, const int32_t *acc_ih_dev, float s_ih, float s_hh, float s_h,
                       const float *bias_dev, int relu, float *h_dev, int8_t *qh_next_dev, int B, int Hs, void *stream) {
    const char *who = "adapt_rnn_step_f32";
    int rc = check_weights(h, 0, who);
    if (rc) return rc;
    if (B < 1 || Hs < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    if (h->N != Hs || h->Cin != Hs) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: handle is not a packed [Hs][Hs] matrix", who);
    if (!(s_h > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_h must be > 0", who);
    if (!qh_dev || !acc_ih_dev || !h_dev || !qh_next_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if (qh_dev == qh_next_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: qh_next_dev must not alias qh_dev", who);
    if (h->storage != 0 || Hs % 2 != 0 || (long long)B * Hs > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: shape outside the fused kernel (Hs even, single-pass table)", who);
    hipStream_t s = (hipStream_t)stream;
    if (!h->wofs_cell_dev || h->cell_G != 1) return fail(ADAPT_ERR_UNSUPPORTED, "%s: the handle holds no cell-order offsets", who);
    Geometry g{};
    g.mode = adapt::MODE_GEMM; g.M = B; g.N = Hs; g.Cin = Hs; g.taps = 1; g.kw = 1;
    g.H = 1; g.W = 1; g.Wo = 1; g.HoWo = 1; g.sh = g.sw = g.dh = g.dw = 1; g.ph = g.pw = 0;
    g.kstride = 1; g.img_stride = Hs;
    LstmStep ls;
    ls.kind = 3; ls.relu = relu ? 1 : 0;
    ls.Hs = Hs; ls.acc_ih = acc_ih_dev; ls.bias = bias_dev; ls.c = nullptr; ls.h = h_dev; ls.qh_next = qh_next_dev;
    ls.s_ih = s_ih; ls.s_hh = s_hh; ls.s_h = s_h; ls.Qh = (float)((1 << (h->bits - 1)) - 1);
    return run_rows(h->lut, qh_dev, nullptr, nullptr, g, s, h->wofs_cell_dev, Hs, nullptr, &ls);
}

}  // extern "C"
