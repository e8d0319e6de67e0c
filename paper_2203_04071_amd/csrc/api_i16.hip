// C ABI, part 3: operands wider than 8 bits (tables in device memory) and multipliers given as functions.
#include "api_common.hpp"
#include "lut_big.hpp"

using namespace adapt_api;

struct adapt_lut16 {
    int bits;               // 2..12
    int device;
    int32_t *t_dev;         // [w + H][a + H], 2^b x 2^b int32
};

extern "C" {

/* ------------------------------------------------------------------ operands wider than 8 bits, function multipliers */

int adapt_lut16_create(adapt_lut16 **out, int bits, const int32_t *table_host) {
    if (!out) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut16_create: out is NULL");
    *out = nullptr;
    if (!table_host) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut16_create: table_host is NULL");
    if (bits < 2 || bits > 12) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut16_create: bits=%d not in [2,12]", bits);
    const size_t bytes = ((size_t)1 << (2 * bits)) * sizeof(int32_t);
    adapt_lut16 *l = new (std::nothrow) adapt_lut16();
    if (!l) return fail(ADAPT_ERR_OUT_OF_MEMORY, "adapt_lut16_create: host allocation failed");
    l->bits = bits; l->t_dev = nullptr; l->device = 0;
    int32_t *tmp = nullptr;
    (void)hipGetDevice(&l->device);
    hipError_t e = dbg_malloc((void **)&l->t_dev, bytes);
    if (e == hipSuccess) e = dbg_malloc((void **)&tmp, bytes);
    if (e == hipSuccess) e = hipMemcpy(tmp, table_host, bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) {
        adapt::big_transpose_kernel<<<ew_grid(bytes / 4), 256, 0, nullptr>>>(tmp, l->t_dev, bits);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (tmp) (void)hipFree(tmp);
    if (e != hipSuccess) {
        if (l->t_dev) (void)hipFree(l->t_dev);
        delete l;
        (void)hipGetLastError();
        return fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "adapt_lut16_create: %s", hipGetErrorString(e));
    }
    *out = l;
    return ADAPT_OK;
}

static int func_args(const char *who, int kind, int param, int bits, int max_bits) {
    if (kind < 0 || kind > 2) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: kind=%d not in [0,2]", who, kind);
    if (bits < 2 || bits > max_bits) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bits=%d not in [2,%d]", who, bits, max_bits);
    if (param < 0 || param >= bits) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: param=%d not in [0,bits)", who, param);
    return ADAPT_OK;
}

int adapt_lut16_create_from_func(adapt_lut16 **out, int kind, int param, int bits) {
    if (!out) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut16_create_from_func: out is NULL");
    *out = nullptr;
    int rc = func_args("adapt_lut16_create_from_func", kind, param, bits, 12);
    if (rc) return rc;
    const size_t entries = (size_t)1 << (2 * bits);
    adapt_lut16 *l = new (std::nothrow) adapt_lut16();
    if (!l) return fail(ADAPT_ERR_OUT_OF_MEMORY, "adapt_lut16_create_from_func: host allocation failed");
    l->bits = bits; l->t_dev = nullptr; l->device = 0;
    (void)hipGetDevice(&l->device);
    hipError_t e = dbg_malloc((void **)&l->t_dev, entries * sizeof(int32_t));
    if (e == hipSuccess) {
        adapt::big_table_from_func_kernel<<<ew_grid(entries), 256, 0, nullptr>>>(l->t_dev, bits, kind, param);
        e = hipGetLastError();
    }
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        if (l->t_dev) (void)hipFree(l->t_dev);
        delete l;
        (void)hipGetLastError();
        return fail(e == hipErrorOutOfMemory ? ADAPT_ERR_OUT_OF_MEMORY : ADAPT_ERR_HIP, "adapt_lut16_create_from_func: %s",
                    hipGetErrorString(e));
    }
    *out = l;
    return ADAPT_OK;
}

int adapt_lut16_destroy(adapt_lut16 *lut) {
    if (!lut) return ADAPT_OK;
    if (lut->t_dev) (void)hipFree(lut->t_dev);
    delete lut;
    return ADAPT_OK;
}

int adapt_lut16_bits(const adapt_lut16 *lut) {
    if (!lut) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_lut16_bits: lut is NULL");
    return lut->bits;
}

int adapt_quantize_i16_f32(const float *x_dev, int16_t *q_dev, size_t n, float scale, int bits, void *stream) {
    if ((!x_dev || !q_dev) && n) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_quantize_i16_f32: NULL pointer");
    if (bits < 2 || bits > 16) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_quantize_i16_f32: bits=%d not in [2,16]", bits);
    if (!(scale > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_quantize_i16_f32: scale must be > 0");
    if (n == 0) return ADAPT_OK;
    adapt::quantize_i16_kernel<<<ew_grid(n), 256, 0, (hipStream_t)stream>>>(x_dev, q_dev, n, scale, (float)((1 << (bits - 1)) - 1));
    HIP_TRY(hipGetLastError());
    return ADAPT_OK;
}

}  // extern "C"

namespace {

// whole-layer form: the finishing pass of the product kernel
struct BigLayer {
    float s_out = 1.0f;
    const float *s_out_vec = nullptr, *bias = nullptr;
    int act = 0;
};

// table form: lut != nullptr; function form: lut == nullptr and (kind, param)
int run_big(const adapt_lut16 *lut, int kind, int param, const int16_t *x, const int16_t *w, int32_t *out, adapt::BigParams p, hipStream_t s,
            const BigLayer *layer = nullptr) {
    if (p.M == 0 || p.N == 0) return ADAPT_OK;
    p.deq = layer ? 1 : 0; p.act = layer ? layer->act : 0; p.scale = layer ? layer->s_out : 1.0f;
    p.scales = layer ? layer->s_out_vec : nullptr; p.bias = layer ? layer->bias : nullptr;
    const long long K = (long long)p.taps * p.Cin;
    const int NT = lut ? adapt::BIG_NT_TABLE : adapt::BIG_NT_FUNC, threads = lut ? adapt::BIG_THREADS_TABLE : adapt::BIG_THREADS_FUNC;
    p.Npad = (p.N + NT - 1) / NT * NT;
    if (K * p.Npad > 0x7fffffffLL) return fail(ADAPT_ERR_UNSUPPORTED, "weights with more than 2^31-1 packed words");
    const long long wgs = (long long)((p.M + threads - 1) / threads) * (p.Npad / NT);
    if (wgs > 0x7fffffffLL) return fail(ADAPT_ERR_UNSUPPORTED, "too many workgroups");
    int32_t *words = nullptr;
    HIP_TRY(dbg_malloc_async((void **)&words, (size_t)(K > 0 ? K : 1) * p.Npad * sizeof(int32_t), s));
    int rc = ADAPT_OK;
    if (K > 0) {
        const size_t n = (size_t)K * p.Npad;
        adapt::big_pack_weights_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(w, words, (int)K, p.N, p.Npad, p.Cin, p.taps,
                                                                                 lut ? lut->bits : 0);
        hipError_t pe = hipGetLastError();
        if (pe != hipSuccess) rc = fail(ADAPT_ERR_HIP, "big_pack_weights launch: %s", hipGetErrorString(pe));
    }
    p.x = x; p.words = words; p.out = out;
    const dim3 grid((unsigned)wgs);
    if (rc == ADAPT_OK) {
        constexpr int FN = adapt::BIG_NT_FUNC, FT = adapt::BIG_THREADS_FUNC;
        if (lut) {
            adapt::MulTable mt{lut->t_dev, 1 << (lut->bits - 1), (1 << lut->bits) - 1};
            adapt::big_rows_kernel<adapt::MulTable, adapt::BIG_NT_TABLE, adapt::BIG_THREADS_TABLE, true><<<grid, threads, 0, s>>>(p, mt);
        } else if (kind == adapt::FUNC_EXACT) {
            adapt::big_rows_kernel<adapt::MulFunc<adapt::FUNC_EXACT>, FN, FT, false><<<grid, threads, 0, s>>>(p, adapt::MulFunc<adapt::FUNC_EXACT>{param});
        } else if (kind == adapt::FUNC_TRUNC) {
            adapt::big_rows_kernel<adapt::MulFunc<adapt::FUNC_TRUNC>, FN, FT, false><<<grid, threads, 0, s>>>(p, adapt::MulFunc<adapt::FUNC_TRUNC>{param});
        } else {
            adapt::big_rows_kernel<adapt::MulFunc<adapt::FUNC_MITCHELL>, FN, FT, false><<<grid, threads, 0, s>>>(p, adapt::MulFunc<adapt::FUNC_MITCHELL>{param});
        }
        hipError_t le = hipGetLastError();
        if (le != hipSuccess) rc = fail(ADAPT_ERR_HIP, "big_rows launch: %s", hipGetErrorString(le));
    }
    hipError_t fe = hipFreeAsync(words, s);
    if (rc == ADAPT_OK && fe != hipSuccess) rc = fail(ADAPT_ERR_HIP, "hipFreeAsync: %s", hipGetErrorString(fe));
    return rc;
}

int big_linear(const char *who, const adapt_lut16 *lut, int kind, int param, const int16_t *a, const int16_t *w, int32_t *acc, int M,
               int K, int N, void *stream, const BigLayer *layer = nullptr) {
    if (M < 0 || K < 0 || N < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: negative dimension", who);
    if (M == 0 || N == 0) return ADAPT_OK;
    if (!acc || (K > 0 && (!a || !w))) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if ((long long)M * N > 0x7fffffffLL || (long long)M * K > 0x7fffffffLL || (long long)N * K > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    adapt::BigParams p{};
    p.M = M; p.N = N; p.conv = 0; p.Cin = K; p.taps = 1; p.kw = 1;
    p.H = p.W = p.Wo = p.HoWo = 1; p.sh = p.sw = p.dh = p.dw = 1; p.ph = p.pw = 0;
    p.kstride = 1; p.img_stride = K;
    return run_big(lut, kind, param, a, w, acc, p, (hipStream_t)stream, layer);
}

int big_conv2d(const char *who, const adapt_lut16 *lut, int kind, int param, const int16_t *x, const int16_t *w, int32_t *acc, int N,
               int Cin, int H, int W, int Cout, int kh, int kw, int sh, int sw, int ph, int pw, int dh, int dw, void *stream,
               const BigLayer *layer = nullptr) {
    if (N < 0 || Cin < 1 || H < 1 || W < 1 || Cout < 1 || kh < 1 || kw < 1 || sh < 1 || sw < 1 || ph < 0 || pw < 0 || dh < 1 || dw < 1)
        return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    const long long eh = (long long)H + 2LL * ph - (long long)dh * (kh - 1) - 1, ew = (long long)W + 2LL * pw - (long long)dw * (kw - 1) - 1;
    if (eh < 0 || ew < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: filter larger than padded input", who);
    const long long Ho = eh / sh + 1, Wo = ew / sw + 1;
    if (N == 0) return ADAPT_OK;
    if (!x || !w || !acc) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    if ((long long)N * Cout * Ho * Wo > 0x7fffffffLL || (long long)N * Cin * H * W > 0x7fffffffLL ||
        (long long)Cout * Cin * kh * kw > 0x7fffffffLL)
        return fail(ADAPT_ERR_UNSUPPORTED, "%s: tensor with more than 2^31-1 elements", who);
    adapt::BigParams p{};
    p.M = (int)(N * Ho * Wo); p.N = Cout; p.conv = 1; p.Cin = Cin; p.taps = kh * kw; p.kw = kw;
    p.H = H; p.W = W; p.Wo = (int)Wo; p.HoWo = (int)(Ho * Wo);
    p.sh = sh; p.sw = sw; p.ph = ph; p.pw = pw; p.dh = dh; p.dw = dw;
    p.kstride = H * W; p.img_stride = Cin * H * W;
    return run_big(lut, kind, param, x, w, acc, p, (hipStream_t)stream, layer);
}

}  // namespace

extern "C" {

int adapt_approx_linear_i16(const adapt_lut16 *lut, const int16_t *a_dev, const int16_t *w_dev, int32_t *acc_dev, int M, int K, int N,
                            void *stream) {
    if (!lut) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_linear_i16: lut is NULL");
    return big_linear("adapt_approx_linear_i16", lut, 0, 0, a_dev, w_dev, acc_dev, M, K, N, stream);
}

int adapt_approx_linear_func_i16(int kind, int param, int bits, const int16_t *a_dev, const int16_t *w_dev, int32_t *acc_dev, int M,
                                 int K, int N, void *stream) {
    int rc = func_args("adapt_approx_linear_func_i16", kind, param, bits, 16);
    if (rc) return rc;
    return big_linear("adapt_approx_linear_func_i16", nullptr, kind, param, a_dev, w_dev, acc_dev, M, K, N, stream);
}

int adapt_approx_conv2d_i16(const adapt_lut16 *lut, const int16_t *x_dev, const int16_t *w_dev, int32_t *acc_dev, int N, int Cin, int H,
                            int W, int Cout, int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w, int dil_h, int dil_w,
                            void *stream) {
    if (!lut) return fail(ADAPT_ERR_INVALID_ARGUMENT, "adapt_approx_conv2d_i16: lut is NULL");
    return big_conv2d("adapt_approx_conv2d_i16", lut, 0, 0, x_dev, w_dev, acc_dev, N, Cin, H, W, Cout, kh, kw, stride_h, stride_w, pad_h,
                      pad_w, dil_h, dil_w, stream);
}

int adapt_approx_conv2d_func_i16(int kind, int param, int bits, const int16_t *x_dev, const int16_t *w_dev, int32_t *acc_dev, int N,
                                 int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w,
                                 int dil_h, int dil_w, void *stream) {
    int rc = func_args("adapt_approx_conv2d_func_i16", kind, param, bits, 16);
    if (rc) return rc;
    return big_conv2d("adapt_approx_conv2d_func_i16", nullptr, kind, param, x_dev, w_dev, acc_dev, N, Cin, H, W, Cout, kh, kw, stride_h,
                      stride_w, pad_h, pad_w, dil_h, dil_w, stream);
}


/* ------------------------------------------------------------------ whole layers on operands of up to 16 bits */

}  // extern "C"

namespace {

// lut != NULL: table form (its bits); else the function (kind, param) at `bits`.  Quantises x into a stream-ordered
// temporary, then runs the product with the finishing pass in its epilogue.
template <class Product>
int i16_layer(const char *who, const adapt_lut16 *lut, int kind, int param, int bits, const float *x_dev, size_t n_in, float s_x, float s_out,
              const float *s_out_vec_dev, const float *bias_dev, int act, hipStream_t s, Product product) {
    if (lut) bits = lut->bits;
    else if (int rc = func_args(who, kind, param, bits, 16)) return rc;
    if (act < 0 || act > 2) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: act=%d not in {0, 1, 2}", who, act);
    if (!(s_x > 0.0f)) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: s_x must be > 0", who);
    BigLayer layer;
    layer.s_out = s_out; layer.s_out_vec = s_out_vec_dev; layer.bias = bias_dev; layer.act = act;
    if (n_in == 0) return product(nullptr, layer);      // (no inner dimension: the sums are 0, the finishing pass still runs)
    if (!x_dev) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: NULL pointer", who);
    int16_t *q = nullptr;
    HIP_TRY(dbg_malloc_async((void **)&q, n_in * sizeof(int16_t), s));
    adapt::quantize_i16_kernel<<<ew_grid(n_in), 256, 0, s>>>(x_dev, q, n_in, s_x, (float)((1 << (bits - 1)) - 1));
    hipError_t qe = hipGetLastError();
    int rc = qe == hipSuccess ? ADAPT_OK : fail(ADAPT_ERR_HIP, "%s: quantise launch: %s", who, hipGetErrorString(qe));
    if (rc == ADAPT_OK) rc = product(q, layer);
    hipError_t fe = hipFreeAsync(q, s);
    if (rc == ADAPT_OK && fe != hipSuccess) rc = fail(ADAPT_ERR_HIP, "hipFreeAsync: %s", hipGetErrorString(fe));
    return rc;
}

}  // namespace

extern "C" {

int adapt_linear_layer_i16_f32(const adapt_lut16 *lut, int kind, int param, int bits, const float *x_dev, const int16_t *w_dev, float *y_dev,
                               int M, int K, int N, float s_x, float s_out, const float *s_out_vec_dev, const float *bias_dev, int act,
                               void *stream) {
    const char *who = "adapt_linear_layer_i16_f32";
    if (M < 0 || K < 0 || N < 0) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: negative dimension", who);
    return i16_layer(who, lut, kind, param, bits, x_dev, (size_t)M * K, s_x, s_out, s_out_vec_dev, bias_dev, act, (hipStream_t)stream,
                     [&](const int16_t *q, const BigLayer &layer) {
                         return big_linear(who, lut, kind, param, q, w_dev, reinterpret_cast<int32_t *>(y_dev), M, K, N, stream, &layer);
                     });
}

int adapt_conv2d_layer_i16_f32(const adapt_lut16 *lut, int kind, int param, int bits, const float *x_dev, const int16_t *w_dev, float *y_dev,
                               int N, int Cin, int H, int W, int Cout, int kh, int kw, int stride_h, int stride_w, int pad_h, int pad_w,
                               int dil_h, int dil_w, float s_x, float s_out, const float *s_out_vec_dev, const float *bias_dev, int act,
                               void *stream) {
    const char *who = "adapt_conv2d_layer_i16_f32";
    if (N < 0 || Cin < 1 || H < 1 || W < 1) return fail(ADAPT_ERR_INVALID_ARGUMENT, "%s: bad dimension", who);
    return i16_layer(who, lut, kind, param, bits, x_dev, (size_t)N * Cin * H * W, s_x, s_out, s_out_vec_dev, bias_dev, act, (hipStream_t)stream,
                     [&](const int16_t *q, const BigLayer &layer) {
                         if (N == 0) return (int)ADAPT_OK;
                         return big_conv2d(who, lut, kind, param, q, w_dev, reinterpret_cast<int32_t *>(y_dev), N, Cin, H, W, Cout, kh, kw,
                                           stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, stream, &layer);
                     });
}

}  // extern "C"
