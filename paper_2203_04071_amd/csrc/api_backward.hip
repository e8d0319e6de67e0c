// C ABI, part 4: the backward pass of Sec. III-A's retraining (straight-through estimator) and the optimiser step.
#include "api_common.hpp"
#include "ste_backward.hpp"

using namespace adapt_api;

namespace {

// Shape of the gradient products' launch: 128 x 128 outputs per workgroup where that still occupies three quarters of
// the compute units, else 64 x 64; eight waves per workgroup instead of four (KS = 2) where there are fewer than two
// workgroups per compute unit.  Env ADAPT_STE_TILE = 64 / 128 and ADAPT_STE_KS = 1 / 2 force one (for measurements).
// `full`: whole tiles, 16-byte rows.
int ste_env(const char *name) {
    const char *e = getenv(name);
    return e ? atoi(e) : 0;
}
// Floats of partial sums a split product may need: it is split only below 256 tiles of 64 x 64, into at most
// 512 / tiles + 1 parts.
constexpr size_t STE_PARTIAL_FLOATS = (size_t)(512 + 256) * 64 * 64;

// partials != nullptr (STE_PARTIAL_FLOATS floats): a product with few output tiles and a long contraction is split
// over grid z into partial sums, which ste_reduce_masked_kernel adds in a fixed order.
void launch_ste_gemm(const adapt::SteParams &p_in, bool a_t, bool aligned, hipStream_t s, float *partials = nullptr) {
    static const int env_tile = ste_env("ADAPT_STE_TILE"), env_ks = ste_env("ADAPT_STE_KS");
    adapt::SteParams p = p_in;
    const int cus = device_cus();
    const long long t128 = (((long long)p.I + 127) / 128) * (((long long)p.J + 127) / 128);
    int tile = 4 * t128 >= 3 * cus ? 128 : 64;
    // whole 64-tiles where 128-tiles would be ragged: the unguarded 16-byte loads are worth more than the larger tile
    const bool whole_ok = aligned && p.R % adapt::STE_TR == 0 && p.lda % 4 == 0 && p.R > 0;
    if (tile == 128 && whole_ok && (p.I % 128 || p.J % 128) && p.I % 64 == 0 && p.J % 64 == 0) tile = 64;
    if (env_tile == 64 || env_tile == 128) tile = env_tile;
    dim3 grid((unsigned)((p.J + tile - 1) / tile), (unsigned)((p.I + tile - 1) / tile), 1);
    const int chunks = (p.R + adapt::STE_TR - 1) / adapt::STE_TR;
    const long long tiles = (long long)grid.x * grid.y;
    p.cps = chunks > 0 ? chunks : 1;
    int parts = 1;
    if (partials && p.im2col && tile == 64 && tiles < cus && chunks >= 8) {       // (the kernels split only in their unfolded-input form)
        int want = (int)((2 * cus + tiles - 1) / tiles);
        if (want > chunks / 4) want = chunks / 4;                   // at least four chunks per part
        if (want >= 2) {
            p.cps = (chunks + want - 1) / want;
            parts = (chunks + p.cps - 1) / p.cps;
        }
    }
    if (parts > 1) { grid.z = (unsigned)parts; p.c = partials; p.o = nullptr; }
    int ks = tiles * parts < 2 * cus ? 2 : 1;
    if (env_ks == 1 || env_ks == 2) ks = env_ks;
    const bool full = aligned && p.I % tile == 0 && p.J % tile == 0 && p.R % adapt::STE_TR == 0 && p.lda % 4 == 0 && p.R > 0;
#define STE_LAUNCH4(AT, T, F, U) \
    do { if (ks == 2) adapt::ste_gemm_kernel<AT, T, F, 2, U><<<grid, adapt::STE_THREADS * 2, 0, s>>>(p); \
         else adapt::ste_gemm_kernel<AT, T, F, 1, U><<<grid, adapt::STE_THREADS, 0, s>>>(p); } while (0)
#define STE_LAUNCH2(AT, T, U) do { if (full) STE_LAUNCH4(AT, T, true, U); else STE_LAUNCH4(AT, T, false, U); } while (0)
    if (a_t && p.im2col) { if (tile == 128) STE_LAUNCH2(true, 128, true); else STE_LAUNCH2(true, 64, true); }
    else if (a_t) { if (tile == 128) STE_LAUNCH2(true, 128, false); else STE_LAUNCH2(true, 64, false); }
    else { if (tile == 128) STE_LAUNCH2(false, 128, false); else STE_LAUNCH2(false, 64, false); }
#undef STE_LAUNCH2
#undef STE_LAUNCH4
    if (parts > 1) {
        const size_t n = (size_t)p.I * (size_t)p.J;
        const size_t blocks = (n + 255) / 256;
        adapt::ste_reduce_masked_kernel<<<(unsigned)(blocks < 4096 ? blocks : 4096), 256, 0, s>>>(partials, parts, n, p_in.o, p_in.so, p_in.Q,
                                                                                                  p_in.c);
    }
}

}  // namespace

extern "C" {

int adapt_ste_linear_backward_f32(const float *dy_dev, const float *x_dev, const float *w_dev, int M, int K, int N, float s_x,
                                  float s_w, int bits, float *dx_dev, float *dw_dev, float *db_dev, void *stream) {
    const char *who = "adapt_ste_linear_backward_f32";
    if (M < 0 || K < 0 || N < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: negative size", who);
    if (bits < 2 || bits > 16) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bits=%d not in [2,16]", who, bits);
    if (!(s_x > 0.0f) || !(s_w > 0.0f) || s_x > 3.0e38f || s_w > 3.0e38f)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: scales must be finite and > 0", who);
    const bool want_dx = dx_dev && M > 0 && K > 0, want_dw = dw_dev && N > 0 && K > 0, want_db = db_dev && N > 0;
    if ((want_dx || want_dw || want_db) && M > 0 && N > 0 && !dy_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL dy_dev", who);
    if ((want_dx || want_dw) && ((M > 0 && !x_dev) || (N > 0 && !w_dev))) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL x_dev / w_dev", who);
    for (const void *q : {(const void *)dy_dev, (const void *)x_dev, (const void *)w_dev, (const void *)dx_dev, (const void *)dw_dev, (const void *)db_dev})
        if (reinterpret_cast<uintptr_t>(q) & 3u) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: pointer not aligned to 4 bytes", who);
    if ((dx_dev && (dx_dev == x_dev || dx_dev == dy_dev || dx_dev == w_dev)) || (dw_dev && (dw_dev == w_dev || dw_dev == dy_dev || dw_dev == x_dev)))
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: a gradient must not alias an input", who);
    if (((long long)M + 63) / 64 > 65535 || ((long long)N + 63) / 64 > 65535)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: M and N are limited to %d", who, 65535 * 64);
    hipStream_t s = (hipStream_t)stream;
    const float Q = (float)((1 << (bits - 1)) - 1);
    if (want_dx) {          // dx [M][K] = inside(x) * dy [M][N] . fq(w) [N][K]
        adapt::SteParams p{};
        p.a = dy_dev; p.b = w_dev; p.o = x_dev; p.c = dx_dev;
        p.I = M; p.J = K; p.R = N; p.lda = N;
        p.sb = s_w; p.so = s_x; p.Q = Q;
        launch_ste_gemm(p, false, aligned16(dy_dev) && aligned16(w_dev), s);
        HIP_TRY(hipGetLastError());
    }
    if (want_dw) {          // dw [N][K] = inside(w) * dy^T [N][M] . fq(x) [M][K]
        adapt::SteParams p{};
        p.a = dy_dev; p.b = x_dev; p.o = w_dev; p.c = dw_dev;
        p.I = N; p.J = K; p.R = M; p.lda = N;
        p.sb = s_x; p.so = s_w; p.Q = Q;
        launch_ste_gemm(p, true, aligned16(dy_dev) && aligned16(x_dev), s);
        HIP_TRY(hipGetLastError());
    }
    if (want_db) {
        adapt::ste_colsum_kernel<<<(unsigned)((N + 31) / 32), adapt::STE_COLSUM_THREADS, 0, s>>>(dy_dev, db_dev, M, N);
        HIP_TRY(hipGetLastError());
    }
    return ADAPT_OK;
}

}  // extern "C"

namespace {
struct SteConvPlan {
    adapt::SteConvGeo g;
    long long M, K;
    size_t rows_bytes, col_bytes, wp_bytes, part_bytes, total;
};
int ste_conv_plan(SteConvPlan *pl, int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w,
                  int dil_h, int dil_w, bool want_dx, bool want_dw, const char *who) {
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || kh < 1 || kw < 1 || stride_h < 1 || stride_w < 1 || pad_h < 0 || pad_w < 0 ||
        dil_h < 1 || dil_w < 1)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    const long long Ho = ((long long)H + 2LL * pad_h - (long long)dil_h * (kh - 1) - 1) / stride_h + 1;
    const long long Wo = ((long long)W + 2LL * pad_w - (long long)dil_w * (kw - 1) - 1) / stride_w + 1;
    if ((long long)H + 2LL * pad_h < (long long)dil_h * (kh - 1) + 1 || (long long)W + 2LL * pad_w < (long long)dil_w * (kw - 1) + 1)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: the filter does not fit the padded image", who);
    pl->M = (long long)N * Ho * Wo;
    pl->K = (long long)Cin * kh * kw;
    if (pl->M > 65535LL * 64 || pl->K > 0x7fffffffLL || Ho > 0x7fffffffLL || Wo > 0x7fffffffLL || (long long)N * Cin * H * W > (1LL << 40))
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor too large (N Ho Wo is limited to %d)", who, 65535 * 64);
    if ((long long)H * W > 0x7fffffffLL || Ho * Wo > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: an image plane is limited to 2^31 - 1 pixels", who);
    adapt::SteConvGeo &g = pl->g;
    g = adapt::SteConvGeo{};
    g.N = N; g.C = Cin; g.H = H; g.W = W; g.O = Cout; g.kh = kh; g.kw = kw; g.sh = stride_h; g.sw = stride_w; g.ph = pad_h; g.pw = pad_w;
    g.dh = dil_h; g.dw = dil_w; g.Ho = (int)Ho; g.Wo = (int)Wo;
    g.dK = fast_div((uint32_t)pl->K); g.dkw = fast_div((uint32_t)kw); g.dkhkw = fast_div((uint32_t)(kh * kw)); g.dWo = fast_div((uint32_t)Wo);
    g.dHoWo = fast_div((uint32_t)(Ho * Wo)); g.dC = fast_div((uint32_t)Cin); g.dW = fast_div((uint32_t)W); g.dHW = fast_div((uint32_t)(H * W));
    g.dO = fast_div((uint32_t)Cout); g.dP = fast_div((uint32_t)(Ho * Wo)); g.dsh = fast_div((uint32_t)stride_h); g.dsw = fast_div((uint32_t)stride_w);
    auto up = [](size_t b) { return (b + 255) / 256 * 256; };
    pl->rows_bytes = up((size_t)pl->M * Cout * sizeof(float));
    pl->col_bytes = up((size_t)pl->M * (size_t)pl->K * sizeof(float));
    pl->part_bytes = up(STE_PARTIAL_FLOATS * sizeof(float));
    pl->wp_bytes = want_dx ? up((size_t)Cout * (size_t)pl->K * sizeof(float)) : 0;
    pl->total = pl->rows_bytes + (want_dx ? pl->col_bytes : 0) + pl->wp_bytes + pl->part_bytes;
    return ADAPT_OK;
}
}  // namespace

extern "C" {

int adapt_ste_conv2d_backward_workspace(int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w, int pad_h,
                                        int pad_w, int dil_h, int dil_w, int want_dx, int want_dw, size_t *bytes) {
    const char *who = "adapt_ste_conv2d_backward_workspace";
    if (!bytes) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    SteConvPlan pl;
    int rc = ste_conv_plan(&pl, N, Cin, H, W, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, want_dx != 0, want_dw != 0, who);
    if (rc) return rc;
    *bytes = pl.total;
    return ADAPT_OK;
}

int adapt_ste_conv2d_backward_f32(const float *dy_dev, const float *x_dev, const float *w_dev, int N, int Cin, int H, int W, int Cout,
                                  int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w, float s_x,
                                  float s_w, int bits, float *dx_dev, float *dw_dev, float *db_dev, void *workspace_dev,
                                  size_t workspace_bytes, void *stream) {
    const char *who = "adapt_ste_conv2d_backward_f32";
    if (bits < 2 || bits > 16) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bits=%d not in [2,16]", who, bits);
    if (!(s_x > 0.0f) || !(s_w > 0.0f) || s_x > 3.0e38f || s_w > 3.0e38f)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: scales must be finite and > 0", who);
    SteConvPlan pl;
    int rc = ste_conv_plan(&pl, N, Cin, H, W, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, dx_dev != nullptr,
                           dw_dev != nullptr, who);
    if (rc) return rc;
    if (pl.M > 0 && (!dy_dev || !x_dev || !w_dev)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    for (const void *q : {(const void *)dy_dev, (const void *)x_dev, (const void *)w_dev, (const void *)dx_dev, (const void *)dw_dev,
                          (const void *)db_dev})
        if (reinterpret_cast<uintptr_t>(q) & 3u) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: pointer not aligned to 4 bytes", who);
    if ((dx_dev && (dx_dev == x_dev || dx_dev == dy_dev || dx_dev == w_dev)) || (dw_dev && (dw_dev == w_dev || dw_dev == dy_dev || dw_dev == x_dev)))
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: a gradient must not alias an input", who);
    if (!dx_dev && !dw_dev && !db_dev) return ADAPT_OK;
    hipStream_t s = (hipStream_t)stream;
    const adapt::SteConvGeo &g = pl.g;
    const float Q = (float)((1 << (bits - 1)) - 1);
    const size_t w_elems = (size_t)Cout * (size_t)pl.K, x_elems = (size_t)N * Cin * H * W;
    if (pl.M == 0) {        // no samples: the weight and bias gradients are zero, there is no input gradient
        if (dw_dev) adapt::fill_u32_kernel<<<ew_grid(w_elems), 256, 0, s>>>(reinterpret_cast<uint32_t *>(dw_dev), 0u, w_elems);
        if (db_dev) adapt::fill_u32_kernel<<<ew_grid((size_t)Cout), 256, 0, s>>>(reinterpret_cast<uint32_t *>(db_dev), 0u, (size_t)Cout);
        HIP_TRY(hipGetLastError());
        return ADAPT_OK;
    }
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255u) || workspace_bytes < pl.total)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: workspace of %zu bytes, aligned to 256, needed (adapt_ste_conv2d_backward_workspace)", who,
                    pl.total);
    char *ws = static_cast<char *>(workspace_dev);
    float *rows = reinterpret_cast<float *>(ws);
    float *dcol = dx_dev ? reinterpret_cast<float *>(ws + pl.rows_bytes) : nullptr;
    float *partials = reinterpret_cast<float *>(ws + pl.total - pl.part_bytes);      // used by one kernel pair at a time (stream order)
    const int M = (int)pl.M, K = (int)pl.K, P = g.Ho * g.Wo;
    const size_t rows_n = (size_t)M * Cout, col_n = (size_t)M * K;     // (col_n: elements of dcol)
    if (rows_n < 0x7fffffffull) adapt::ste_rows_from_nchw_kernel<uint32_t><<<ew_grid(rows_n), 256, 0, s>>>(dy_dev, rows, g, rows_n);
    else adapt::ste_rows_from_nchw_kernel<size_t><<<ew_grid(rows_n), 256, 0, s>>>(dy_dev, rows, g, rows_n);
    HIP_TRY(hipGetLastError());
    if (dw_dev) {           // dw [Cout][K] = inside(w) * rows^T [Cout][M] . fq(col(x)) [M][K], col(x) read from x itself
        adapt::SteParams p{};
        p.a = rows; p.b = x_dev; p.o = w_dev; p.c = dw_dev;
        p.I = Cout; p.J = K; p.R = M; p.lda = Cout;
        p.sb = s_x; p.so = s_w; p.Q = Q;
        p.im2col = 1; p.g = g;
        launch_ste_gemm(p, true, true, s, partials);        // (both operands lie in the workspace)
        HIP_TRY(hipGetLastError());
    }
    if (dx_dev) {           // dcol [M][K] = rows [M][Cout] . fq(w) [Cout][K]; dx = inside(x) * the taps of dcol gathered onto the image
        adapt::SteParams p{};
        float *wp = reinterpret_cast<float *>(ws + pl.rows_bytes + pl.col_bytes);      // the weights with the channel last in each row
        adapt::ste_taps_first_kernel<<<ew_grid(w_elems), 256, 0, s>>>(w_dev, wp, Cout, Cin, kh * kw);
        HIP_TRY(hipGetLastError());
        p.a = rows; p.b = wp; p.o = nullptr; p.c = dcol;
        p.I = M; p.J = K; p.R = Cout; p.lda = Cout;
        p.sb = s_w; p.so = 1.0f; p.Q = Q;
        launch_ste_gemm(p, false, true, s);
        HIP_TRY(hipGetLastError());
        if (x_elems < 0x7fffffffull && col_n < 0x7fffffffull)
            adapt::ste_col2im_kernel<uint32_t><<<ew_grid(x_elems), 256, 0, s>>>(dcol, x_dev, dx_dev, g, s_x, Q, x_elems);
        else adapt::ste_col2im_kernel<size_t><<<ew_grid(x_elems), 256, 0, s>>>(dcol, x_dev, dx_dev, g, s_x, Q, x_elems);
        HIP_TRY(hipGetLastError());
    }
    if (db_dev) {
        const int Z = N < 16 ? N : 16;
        if ((size_t)Z * Cout <= STE_PARTIAL_FLOATS && Z > 1) {
            adapt::ste_bias_grad_nchw_kernel<<<dim3((unsigned)Cout, (unsigned)Z), 256, 0, s>>>(dy_dev, partials, N, Cout, P);
            adapt::ste_reduce_masked_kernel<<<(unsigned)((Cout + 255) / 256), 256, 0, s>>>(partials, Z, (size_t)Cout, nullptr, 1.0f, Q, db_dev);
        } else {
            adapt::ste_bias_grad_nchw_kernel<<<dim3((unsigned)Cout, 1), 256, 0, s>>>(dy_dev, db_dev, N, Cout, P);
        }
        HIP_TRY(hipGetLastError());
    }
    return ADAPT_OK;
}

int adapt_relu_backward_f32(const float *dy_dev, const float *y_dev, float *dx_dev, size_t n, void *stream) {
    if ((!dy_dev || !y_dev || !dx_dev) && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_relu_backward_f32: NULL pointer");
    if (!n) return ADAPT_OK;
    adapt::relu_backward_kernel<<<ew_grid(n), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(dy_dev, y_dev, dx_dev, n);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_sgd_step_f32(float *w_dev, const float *g_dev, size_t n, float lr, void *stream) {
    if ((!w_dev || !g_dev) && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_sgd_step_f32: NULL pointer");
    if (w_dev == g_dev && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_sgd_step_f32: w_dev and g_dev must differ");
    if (!n) return ADAPT_OK;
    adapt::sgd_kernel<<<ew_grid(n), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(w_dev, g_dev, n, lr);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

}  // extern "C"
