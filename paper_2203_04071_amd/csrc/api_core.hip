// C ABI, part 1: error text, table handles, quantiser / dequantiser, calibrators, the fp32 operations between layers.
#include "api_common.hpp"

namespace adapt_api {
thread_local char g_err[512] = "";
}
using namespace adapt_api;

extern "C" {

const char *adapt_last_error(void) { return g_err; }

int adapt_device_cu_count(void) {
    int dev = 0, cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return fail(ADAPT_ERR_HIP, "hipGetDevice failed");
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return fail(ADAPT_ERR_HIP, "hipDeviceGetAttribute failed");
    return cu;
}

int adapt_lut_create(adapt_lut **out, int bits, const int32_t *table_host) {
    if (!out) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut_create: out is NULL");
    *out = nullptr;
    if (!table_host) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut_create: table_host is NULL");
    if (bits < 2 || bits > 8) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut_create: bits=%d not in [2,8]", bits);
    const int n = 1 << bits;
    int32_t lo = table_host[0], hi = table_host[0];
    for (int i = 0; i < n * n; ++i) {
        if (table_host[i] < lo) lo = table_host[i];
        if (table_host[i] > hi) hi = table_host[i];
    }
    adapt_lut *l = new (std::nothrow) adapt_lut();
    if (!l) return fail(ADAPT_ERR_OUT_OF_MEMORY, "adapt_lut_create: host allocation failed");
    l->bits = bits;
    l->min_entry = lo;
    l->max_entry = hi;
    l->storage = (lo >= -32768 && hi <= 32767) ? 0 : 1;
    l->rs = n + 2;
    l->img_bytes = ((n * l->rs * 2 + 15) / 16) * 16;
    l->img_dev[0] = l->img_dev[1] = nullptr;
    l->lut16_dev[0] = l->lut16_dev[1] = nullptr;
    if (hipGetDevice(&l->device) != hipSuccess) {
        delete l;
        return fail(ADAPT_ERR_HIP, "adapt_lut_create: hipGetDevice failed");
    }
    // private image order: row = weight operand, column = activation operand, then a zero column
    std::vector<uint16_t> img((size_t)l->img_bytes / 2, 0);
    for (int half = 0; half <= l->storage; ++half) {
        for (int w = 0; w < n; ++w)
            for (int a = 0; a < n; ++a) {
                const uint32_t v = (uint32_t)table_host[(size_t)a * n + w];
                uint16_t e;
                if (l->storage == 0) e = (uint16_t)v;
                else e = half == 0 ? (uint16_t)(v & 0xffffu) : (uint16_t)(v >> 16);
                img[(size_t)w * l->rs + a] = e;
            }
        hipError_t e = dbg_malloc((void **)&l->img_dev[half], (size_t)l->img_bytes);
        if (e == hipSuccess) e = hipMemcpy(l->img_dev[half], img.data(), (size_t)l->img_bytes, hipMemcpyHostToDevice);
        // plain copy indexed by the two's-complement wrap of the operands: [a & mask][w & mask]
        std::vector<uint16_t> plain((size_t)n * n);
        const int hh = n >> 1;
        for (int a = -hh; a < hh; ++a)
            for (int w = -hh; w < hh; ++w)
                plain[(size_t)(a & (n - 1)) * n + (w & (n - 1))] = img[(size_t)(w + hh) * l->rs + (a + hh)];
        if (e == hipSuccess) e = dbg_malloc((void **)&l->lut16_dev[half], plain.size() * 2);
        if (e == hipSuccess) e = hipMemcpy(l->lut16_dev[half], plain.data(), plain.size() * 2, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            for (int j = 0; j < 2; ++j) {
                if (l->img_dev[j]) (void)hipFree(l->img_dev[j]);
                if (l->lut16_dev[j]) (void)hipFree(l->lut16_dev[j]);
            }
            delete l;
            return fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP,
                        "adapt_lut_create: device image: %s", hipGetErrorString(e));
        }
    }
    *out = l;
    return ADAPT_OK;
}

int adapt_lut_destroy(adapt_lut *lut) {
    if (!lut) return ADAPT_OK;
    for (int j = 0; j < 2; ++j) {
        if (lut->img_dev[j]) (void)hipFree(lut->img_dev[j]);
        if (lut->lut16_dev[j]) (void)hipFree(lut->lut16_dev[j]);
    }
    delete lut;
    return ADAPT_OK;
}

int adapt_lut_info(const adapt_lut *lut, int *bits, int *storage, int32_t *min_entry, int32_t *max_entry) {
    if (!lut) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut_info: lut is NULL");
    if (bits) *bits = lut->bits;
    if (storage) *storage = lut->storage;
    if (min_entry) *min_entry = lut->min_entry;
    if (max_entry) *max_entry = lut->max_entry;
    return ADAPT_OK;
}

/* ------------------------------------------------------------------ quantiser / dequantiser */

int adapt_absmax_f32(const float *x_dev, size_t n, float *amax_dev, void *stream) {
    if (!amax_dev || (!x_dev && n)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_absmax_f32: NULL pointer");
    hipStream_t s = (hipStream_t)stream;
    adapt::fill_u32_kernel<<<1, 64, 0, s>>>(reinterpret_cast<uint32_t *>(amax_dev), 0u, 1);
    if (n) {
        const int vec = aligned16(x_dev) ? 1 : 0;
        adapt::absmax_kernel<<<ew_grid(n / 8 + 1), adapt::EW_THREADS, 0, s>>>(x_dev, n, reinterpret_cast<uint32_t *>(amax_dev), vec);
    }
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_quantize_f32(const float *x_dev, int8_t *q_dev, size_t n, float scale, int bits, void *stream) {
    if ((!x_dev || !q_dev) && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_quantize_f32: NULL pointer");
    if (bits < 2 || bits > 8) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_quantize_f32: bits=%d not in [2,8]", bits);
    if (!(scale > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_quantize_f32: scale must be > 0");
    if (n == 0) return ADAPT_OK;
    const int vec = (aligned16(x_dev) && aligned16(q_dev)) ? 1 : 0;
    const float Q = (float)((1 << (bits - 1)) - 1);
    adapt::quantize_kernel<<<ew_grid(n / 16 + 1), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(x_dev, q_dev, n, scale, Q, vec);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_dequant_i32(const int32_t *acc_dev, float *y_dev, size_t outer, size_t channels, size_t inner,
                      float scale, const float *bias_dev, void *stream) {
    const size_t n = outer * channels * inner;
    if ((!acc_dev || !y_dev) && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_dequant_i32: NULL pointer");
    if (n == 0) return ADAPT_OK;
    const int vec = (aligned16(acc_dev) && aligned16(y_dev) && (!bias_dev || inner % 4 == 0)) ? 1 : 0;
    adapt::dequant_kernel<<<ew_grid(n / 4 + 1), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(acc_dev, y_dev, n, channels, inner, scale, bias_dev, vec);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}


/* ------------------------------------------------------------------ per-channel ranges, percentile calibrator */

int adapt_absmax_rows_f32(const float *x_dev, size_t rows, size_t cols, float *amax_dev, void *stream) {
    if (rows == 0) return ADAPT_OK;
    if (!amax_dev || (!x_dev && cols)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_absmax_rows_f32: NULL pointer");
    if (rows > 0x7fffffffULL) return fail(ADAPT_ERR_UNSUPPORTED, "adapt_absmax_rows_f32: more than 2^31-1 rows");
    adapt::absmax_rows_kernel<<<(unsigned)rows, adapt::EW_THREADS, 0, (hipStream_t)stream>>>(x_dev, cols, amax_dev);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_quantize_rows_f32(const float *x_dev, int8_t *q_dev, size_t rows, size_t cols, const float *scales_dev, int bits,
                            void *stream) {
    if (bits < 2 || bits > 8) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_quantize_rows_f32: bits=%d not in [2,8]", bits);
    if (rows == 0 || cols == 0) return ADAPT_OK;
    if (!x_dev || !q_dev || !scales_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_quantize_rows_f32: NULL pointer");
    adapt::quantize_rows_kernel<<<ew_grid(rows * cols), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(
        x_dev, q_dev, rows, cols, scales_dev, (float)((1 << (bits - 1)) - 1));
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_dequant_i32_per_channel(const int32_t *acc_dev, float *y_dev, size_t outer, size_t channels, size_t inner,
                                  const float *scales_dev, const float *bias_dev, void *stream) {
    const size_t n = outer * channels * inner;
    if (n == 0) return ADAPT_OK;
    if (!acc_dev || !y_dev || !scales_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_dequant_i32_per_channel: NULL pointer");
    adapt::dequant_pc_kernel<<<ew_grid(n), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(acc_dev, y_dev, n, channels, inner, scales_dev,
                                                                                        bias_dev);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_histogram_abs_f32(const float *x_dev, size_t n, float amax, int bins, uint32_t *counts_dev, void *stream) {
    if (bins < 1 || bins > 4096) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_histogram_abs_f32: bins=%d not in [1,4096]", bins);
    if (!(amax > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_histogram_abs_f32: amax must be > 0");
    if (!counts_dev || (!x_dev && n)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_histogram_abs_f32: NULL pointer");
    if (n == 0) return ADAPT_OK;
    const float width = amax / (float)bins;
    const int vec = (reinterpret_cast<uintptr_t>(x_dev) & 15u) == 0 ? 1 : 0;
    adapt::histogram_abs_kernel<<<ew_grid(n / 8 + 1), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(x_dev, n, width, bins, counts_dev, vec);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_percentile_from_histogram(const uint32_t *counts_dev, int bins, float amax, unsigned num, unsigned den, float *calib_max_dev,
                                    void *stream) {
    if (bins < 1 || bins > 4096) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_percentile_from_histogram: bins=%d not in [1,4096]", bins);
    if (!(amax > 0.0f) || den == 0 || num > den || den > (1u << 20))
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_percentile_from_histogram: need amax > 0 and 0 <= num <= den <= 2^20");
    if (!counts_dev || !calib_max_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_percentile_from_histogram: NULL pointer");
    adapt::percentile_kernel<<<1, 64, 0, (hipStream_t)stream>>>(counts_dev, bins, amax / (float)bins, num, den, calib_max_dev);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_mse_from_histogram(const uint32_t *counts_dev, int bins, float amax, int bits, float *calib_max_dev, void *stream) {
    if (bins < 1 || bins > 4096) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_mse_from_histogram: bins=%d not in [1,4096]", bins);
    if (!(amax > 0.0f) || bits < 2 || bits > 16) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_mse_from_histogram: need amax > 0 and 2 <= bits <= 16");
    if (!counts_dev || !calib_max_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_mse_from_histogram: NULL pointer");
    hipStream_t s = (hipStream_t)stream;
    double *err = nullptr;
    HIP_TRY(dbg_malloc_async((void **)&err, (size_t)bins * sizeof(double), s));
    const float width = amax / (float)bins;
    adapt::mse_candidates_kernel<<<(unsigned)((bins + 255) / 256), 256, 0, s>>>(counts_dev, bins, width, (float)((1 << (bits - 1)) - 1), err);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) {
        adapt::mse_pick_kernel<<<1, 64, 0, s>>>(err, bins, width, calib_max_dev);
        e = hipGetLastError();
    }
    hipError_t fe = hipFreeAsync(err, s);
    if (e != hipSuccess) return fail(ADAPT_ERR_HIP, "adapt_mse_from_histogram: %s", hipGetErrorString(e));
    if (fe != hipSuccess) return fail(ADAPT_ERR_HIP, "hipFreeAsync: %s", hipGetErrorString(fe));
    return ADAPT_OK;
}

int adapt_entropy_from_histogram(const uint32_t *counts_dev, int bins, float amax, int bits, float *calib_max_dev, void *stream) {
    if (bins < 1 || bins > 4096) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_entropy_from_histogram: bins=%d not in [1,4096]", bins);
    if (!(amax > 0.0f) || bits < 2 || bits > 16) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_entropy_from_histogram: need amax > 0 and 2 <= bits <= 16");
    if (!counts_dev || !calib_max_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_entropy_from_histogram: NULL pointer");
    hipStream_t s = (hipStream_t)stream;
    double *loss = nullptr;
    HIP_TRY(dbg_malloc_async((void **)&loss, (size_t)bins * sizeof(double), s));
    const float width = amax / (float)bins;
    adapt::entropy_candidates_kernel<<<(unsigned)((bins + 255) / 256), 256, 0, s>>>(counts_dev, bins, 1 << (bits - 1), loss);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) {
        adapt::mse_pick_kernel<<<1, 64, 0, s>>>(loss, bins, width, calib_max_dev);      // first smallest: calib_max = k * width
        e = hipGetLastError();
    }
    hipError_t fe = hipFreeAsync(loss, s);
    if (e != hipSuccess) return fail(ADAPT_ERR_HIP, "adapt_entropy_from_histogram: %s", hipGetErrorString(e));
    if (fe != hipSuccess) return fail(ADAPT_ERR_HIP, "hipFreeAsync: %s", hipGetErrorString(fe));
    return ADAPT_OK;
}

/* ------------------------------------------------------------------ fp32 operations between layers */

int adapt_relu_f32(const float *x_dev, float *y_dev, size_t n, void *stream) {
    if ((!x_dev || !y_dev) && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_relu_f32: NULL pointer");
    if (!n) return ADAPT_OK;
    const int vec = ((reinterpret_cast<uintptr_t>(x_dev) | reinterpret_cast<uintptr_t>(y_dev)) & 15u) == 0 ? 1 : 0;
    adapt::relu_kernel<<<ew_grid(n / 4 + 1), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(x_dev, y_dev, n, vec);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_add_f32(const float *a_dev, const float *b_dev, float *y_dev, size_t n, int relu, void *stream) {
    if ((!a_dev || !b_dev || !y_dev) && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_add_f32: NULL pointer");
    if (!n) return ADAPT_OK;
    const int vec = ((reinterpret_cast<uintptr_t>(a_dev) | reinterpret_cast<uintptr_t>(b_dev) | reinterpret_cast<uintptr_t>(y_dev)) & 15u) == 0 ? 1 : 0;
    adapt::add_kernel<<<ew_grid(n / 4 + 1), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(a_dev, b_dev, y_dev, n, relu, vec);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}


int adapt_avgpool_hw_f32(const float *x_dev, float *y_dev, size_t NC, size_t HW, void *stream) {
    if ((!x_dev || !y_dev) && NC) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_avgpool_hw_f32: NULL pointer");
    if (HW == 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_avgpool_hw_f32: HW is 0");
    if (!NC) return ADAPT_OK;
    if (HW == 64 && (reinterpret_cast<uintptr_t>(x_dev) & 15u) == 0 && (NC + 63) / 64 <= 0x7fffffffull)
        adapt::avgpool64_kernel<<<(unsigned)((NC + 63) / 64), 64, 0, (hipStream_t)stream>>>(x_dev, y_dev, NC);
    else
        adapt::avgpool_kernel<<<(unsigned)((NC + adapt::EW_THREADS - 1) / adapt::EW_THREADS), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(x_dev, y_dev, NC, HW);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_shortcut_a_f32(const float *x_dev, float *y_dev, int N, int Cin, int H, int W, int Cout, void *stream) {
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < Cin) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_shortcut_a_f32: bad dimension");
    if (N == 0) return ADAPT_OK;
    if (!x_dev || !y_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_shortcut_a_f32: NULL pointer");
    if (x_dev == y_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_shortcut_a_f32: in-place not possible");
    const size_t total = (size_t)N * Cout * ((H + 1) / 2) * ((W + 1) / 2);
    const int fast = total < 0x7fffffffull && (size_t)N * Cin * H * W < 0x7fffffffull ? 1 : 0;
    adapt::shortcut_a_kernel<<<ew_grid(total), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(
        x_dev, y_dev, N, Cin, H, W, Cout, fast_div((uint32_t)((W + 1) / 2)), fast_div((uint32_t)((H + 1) / 2)), fast_div((uint32_t)Cout), fast);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

static int unary(const float *x_dev, float *y_dev, size_t n, int op, void *stream, const char *who) {
    if ((!x_dev || !y_dev) && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if (!n) return ADAPT_OK;
    adapt::unary_kernel<<<ew_grid(n), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(x_dev, y_dev, n, op);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_tanh_f32(const float *x_dev, float *y_dev, size_t n, void *stream) { return unary(x_dev, y_dev, n, 0, stream, "adapt_tanh_f32"); }
int adapt_sigmoid_f32(const float *x_dev, float *y_dev, size_t n, void *stream) { return unary(x_dev, y_dev, n, 1, stream, "adapt_sigmoid_f32"); }

static int lstm_cell(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh, const float *bias_dev, float *c_dev,
                     float *h_dev, int8_t *qh_dev, float s_h, int bits, int B, int Hs, void *stream, const char *who) {
    if (B < 0 || Hs < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: negative dimension", who);
    const size_t n = (size_t)B * Hs;
    if (!n) return ADAPT_OK;
    if (!acc_ih_dev || !acc_hh_dev || !c_dev || !h_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    adapt::lstm_cell_kernel<<<(unsigned)((n + adapt::EW_THREADS - 1) / adapt::EW_THREADS), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(
        acc_ih_dev, acc_hh_dev, s_ih, s_hh, bias_dev, c_dev, h_dev, B, Hs, qh_dev, s_h, (float)((1 << (bits - 1)) - 1));
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_lstm_cell_f32(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh,
                        const float *bias_dev, float *c_dev, float *h_dev, int B, int Hs, void *stream) {
    return lstm_cell(acc_ih_dev, acc_hh_dev, s_ih, s_hh, bias_dev, c_dev, h_dev, nullptr, 1.0f, 8, B, Hs, stream, "adapt_lstm_cell_f32");
}

int adapt_lstm_cell_q_f32(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh, const float *bias_dev,
                          float *c_dev, float *h_dev, int8_t *qh_dev, float s_h, int bits, int B, int Hs, void *stream) {
    if (!qh_dev && (size_t)B * Hs) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lstm_cell_q_f32: NULL pointer");
    if (bits < 2 || bits > 8) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lstm_cell_q_f32: bits=%d not in [2,8]", bits);
    if (!(s_h > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lstm_cell_q_f32: scale must be > 0");
    return lstm_cell(acc_ih_dev, acc_hh_dev, s_ih, s_hh, bias_dev, c_dev, h_dev, qh_dev, s_h, bits, B, Hs, stream, "adapt_lstm_cell_q_f32");
}

static int cell_args(const char *who, const void *a, const void *b, const void *h, const int8_t *qh, float s_h, int bits, int B, int Hs,
                     size_t *n) {
    if (B < 0 || Hs < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: negative dimension", who);
    *n = (size_t)B * Hs;
    if (!*n) return ADAPT_OK;
    if (!a || !b || !h) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if (qh) {
        if (bits < 2 || bits > 8) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bits=%d not in [2,8]", who, bits);
        if (!(s_h > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: scale must be > 0", who);
    }
    return ADAPT_OK;
}

int adapt_gru_cell_f32(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh, const float *b_ih_dev,
                       const float *b_hh_dev, const float *h_prev_dev, float *h_dev, int8_t *qh_dev, float s_h, int bits, int B,
                       int Hs, void *stream) {
    size_t n = 0;
    int rc = cell_args("adapt_gru_cell_f32", acc_ih_dev, acc_hh_dev, h_dev, qh_dev, s_h, bits, B, Hs, &n);
    if (rc || !n) return rc;
    if (!h_prev_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_gru_cell_f32: NULL pointer");
    adapt::gru_cell_kernel<<<(unsigned)((n + adapt::EW_THREADS - 1) / adapt::EW_THREADS), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(
        acc_ih_dev, acc_hh_dev, s_ih, s_hh, b_ih_dev, b_hh_dev, h_prev_dev, h_dev, B, Hs, qh_dev, s_h,
        qh_dev ? (float)((1 << (bits - 1)) - 1) : 1.0f);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

int adapt_rnn_cell_f32(const int32_t *acc_ih_dev, const int32_t *acc_hh_dev, float s_ih, float s_hh, const float *bias_dev, int relu,
                       float *h_dev, int8_t *qh_dev, float s_h, int bits, int B, int Hs, void *stream) {
    size_t n = 0;
    int rc = cell_args("adapt_rnn_cell_f32", acc_ih_dev, acc_hh_dev, h_dev, qh_dev, s_h, bits, B, Hs, &n);
    if (rc || !n) return rc;
    adapt::rnn_cell_kernel<<<(unsigned)((n + adapt::EW_THREADS - 1) / adapt::EW_THREADS), adapt::EW_THREADS, 0, (hipStream_t)stream>>>(
        acc_ih_dev, acc_hh_dev, s_ih, s_hh, bias_dev, relu, h_dev, B, Hs, qh_dev, s_h, qh_dev ? (float)((1 << (bits - 1)) - 1) : 1.0f);
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}



}  // extern "C"
