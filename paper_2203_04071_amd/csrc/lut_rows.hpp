// General table-lookup matrix-product kernel ("rows" kernel): the whole 2^b x 2^b multiplier table
// sits in LDS and every inner-product term is one 16-bit LDS read (Sec. IV of the paper: the inner
// multiplications are table look-ups; its AVX2 gather becomes a per-lane LDS gather here).
//
// Mapping (gfx950, 64-wide waves): lanes run along the rows of the expanded input matrix (batch x
// output pixels), because that is the long dimension of every layer shape; the weight of a term is
// wave-uniform, so the byte offset of its table row comes from a scalar load of a pre-packed
// offset array and the per-lane part of the address is just the activation.  The LDS image is
// stored weight-major, image[w][a], so that all lanes of one lookup fall into one row: at most
// 2^b/2 distinct bank words, identical activations broadcast.
//
// One kernel serves linear layers, convolutions (implicit expansion, padded taps are looked up with
// activation 0) and transposed convolutions in gather form (taps without a real input pixel read an
// all-zero extra column, so they add nothing).  Short matrices split K over the waves of a
// workgroup and reduce through LDS.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "elementwise.hpp"

namespace adapt {

constexpr int ROWS_THREADS = 1024;

enum { MODE_GEMM = 0, MODE_CONV = 1, MODE_CONVT = 2 };

struct RowsParams {
    const int8_t *x;        // activations: [M][K] or NCHW
    const uint32_t *wofs;   // [Ktot][Npad] byte offset of the table row of weight (k, n); k = tap * Cin + ci
    int32_t *out;           // [M][N] or NCHW
    const uint16_t *img;    // table image: 2^b rows (one per weight) of RS = 2^b + 2 entries
    int img_bytes;          // multiple of 16
    int M, N, Npad;
    int out_ch;             // channels of the output tensor: N, or groups * N for a grouped convolution (blockIdx.z = group:
                            // x advanced by Cin channels, wofs by one [Ktot][Npad] block, outputs by N channels per group)
    int mode;
    int Cin;                // inner length per tap (GEMM: K)
    int taps, kw;           // kh * kw (GEMM: 1)
    int H, W, Wo, HoWo;     // GEMM: HoWo = Wo = 1
    int sh, sw, ph, pw, dh, dw;
    int kstride;            // elements between consecutive ci of one row (GEMM 1, conv H * W)
    int img_stride;         // elements per image of x (GEMM: K)
    int hoff, mask;         // H = 2^(b-1), 2^b - 1
    int a_zero2, a_skip2;   // byte offset in a table row of activation 0 / of the all-zero column
    int MT, KS;             // rows per workgroup, K slices per workgroup; MT * KS == ROWS_THREADS
    int shift;              // < 0: out = acc;  >= 0: out += acc << shift (second half of a split table)
    // fused rescaling (single-pass tables only): deq != 0 stores fp32 y = float(acc) * scale, + bias[n] if bias, then
    // max(y, 0) if act == 1, each operation rounded separately, instead of the int32 sum
    int deq, act;
    float scale;
    const float *scales;    // one scale per output channel (then `scale` is unused), or nullptr
    const float *bias;
    // Recurrent time step (lstm = 1: LSTM, G = 4 gates; lstm = 2: GRU, G = 3; lstm = 3: plain cell, G = 1, `act` = 1 for
    // ReLU instead of tanh; linear layer with N = G Hs whose offsets
    // were packed in "cell order": packed column 2 G (u / 2) + 2 g + (u % 2) is gate g of hidden unit u, so the 2 G
    // columns of a workgroup are all gates of two units): the sums are not stored; the workgroup runs the cell for its
    // two units (the operations of lstm_cell_kernel / gru_cell_kernel) and writes (c,) h and the quantised h of the
    // next step.  LSTM: bias = b_ih + b_hh folded by the caller.  GRU: bias = b_ih, bias_hh = b_hh, h_prev read.
    int lstm, Hs;
    const int32_t *acc_ih;      // [M][G Hs]
    float *c, *h;               // [M][Hs]
    const float *h_prev;        // [M][Hs] (GRU; may be h)
    const float *bias_hh;       // [3 Hs] or nullptr (GRU)
    int8_t *qh_next;            // [M][Hs]
    float s_ih, s_hh, s_h, Qh;
};

__device__ __forceinline__ uint32_t finish_sum(const RowsParams &p, uint32_t v, int n) {
    if (!p.deq) return v;
    float y = (float)(int32_t)v * (p.scales ? p.scales[n] : p.scale);
    if (p.bias) y = y + p.bias[n];
    if (p.act == 1) y = y > 0.0f ? y : 0.0f;
    return __float_as_uint(y);
}

// weights -> byte offsets of their table rows, in the order the kernel walks K
// (blockIdx.y = group of a grouped convolution: its N filters follow the previous group's, its block of offsets too)
__global__ void pack_row_offsets_kernel(const int8_t *__restrict__ w, uint32_t *__restrict__ wofs, int Ktot,
                                        int N, int Npad, int Cin, int taps, int mode, int hoff, int mask,
                                        int row_bytes) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (size_t)Ktot * Npad) return;
    w += (size_t)blockIdx.y * N * Ktot;
    wofs += (size_t)blockIdx.y * Ktot * Npad;
    const int k = (int)(idx / Npad), n = (int)(idx % Npad);
    uint32_t v = 0;
    if (n < N) {
        const int t = k / Cin, ci = k - t * Cin;
        size_t wi;
        if (mode == MODE_CONVT) wi = ((size_t)ci * N + n) * taps + t;      // [Cin][Cout][kh][kw]
        else wi = ((size_t)n * Cin + ci) * taps + t;                       // [N][K] / [Cout][Cin][kh][kw]
        v = (uint32_t)(((int)w[wi] + hoff) & mask) * (uint32_t)row_bytes;
    }
    wofs[idx] = v;
}

// W_hh [G Hs][Hs] -> row offsets with the columns in cell order: packed column 2 G (u / 2) + 2 g + (u % 2) holds gate g
// of hidden unit u, i.e. weight row g * Hs + u.  Stored [pair of units][k][2 G]: the 2 G columns a workgroup needs are
// contiguous over k, so its scalar loads fetch whole cache lines that it uses completely (stored [k][column] every load
// touched a line of its own and used 24 or 32 bytes of it).
__global__ void pack_row_offsets_cell_kernel(const int8_t *__restrict__ w, uint32_t *__restrict__ wofs, int Hs, int G, int hoff,
                                             int mask, int row_bytes) {
    const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int N = G * Hs;
    if (idx >= (size_t)Hs * N) return;
    const int k = (int)(idx / N), cp = (int)(idx % N);
    const int pair = cp / (2 * G), within = cp - pair * 2 * G;
    const int u = pair * 2 + (within & 1), g = within >> 1;
    const size_t wi = ((size_t)g * Hs + u) * Hs + k;
    wofs[((size_t)pair * Hs + k) * (2 * G) + within] = (uint32_t)(((int)w[wi] + hoff) & mask) * (uint32_t)row_bytes;
}

template <bool SIGNED>
__device__ __forceinline__ uint32_t lds_entry(const unsigned char *smem, uint32_t off) {
    if (SIGNED) return (uint32_t)(int32_t) * reinterpret_cast<const int16_t *>(smem + off);
    return (uint32_t) * reinterpret_cast<const uint16_t *>(smem + off);
}

// Copy the table image (img_bytes, a multiple of 16) into LDS with ROWS_THREADS lanes; the caller synchronises the
// workgroup afterwards.  (LDS-direct loads issued back to back were measured slower than this plain loop: 2.5 us more
// per launch of the LSTM step.)
__device__ __forceinline__ void stage_table(unsigned char *smem, const uint16_t *img, int img_bytes, int tid) {
    const uint4 *src = reinterpret_cast<const uint4 *>(img);
    uint4 *dst = reinterpret_cast<uint4 *>(smem);
    const int n16 = img_bytes >> 4;
    for (int i = tid; i < n16; i += ROWS_THREADS) dst[i] = src[i];
}

template <int NT, bool SIGNED>
__global__ __launch_bounds__(ROWS_THREADS) void lut_rows_kernel(const RowsParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    stage_table(smem, p.img, p.img_bytes, tid);
    __syncthreads();

    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    // (MT and KS are powers of two, MT * KS = 1024: shifts instead of divisions, which cost tens of instructions each —
    // noticeable in a kernel that is launched once per time step)
    const int mt_log = __builtin_ctz((unsigned)p.MT), ks_log = 10 - mt_log;
    const int row_waves = p.MT >> 6;
    const int ks = wave >> (mt_log - 6);
    const int rb = wave - ks * row_waves;
    const int r_in_tile = rb * 64 + lane;
    const int m = blockIdx.x * p.MT + r_in_tile;
    const bool mvalid = m < p.M;
    const int mm = mvalid ? m : p.M - 1;
    const int n0 = blockIdx.y * NT;

    int img = mm, pix = 0, oy = 0, ox = 0;          // linear layer: HoWo = Wo = 1
    if (p.mode != MODE_GEMM) {
        img = mm / p.HoWo;
        pix = mm - img * p.HoWo;
        oy = pix / p.Wo;
        ox = pix - oy * p.Wo;
    }
    const int grp = blockIdx.z;
    const int8_t *xb = p.x + (size_t)img * p.img_stride + (size_t)grp * p.Cin * p.kstride;

    const int Ktot = p.taps * p.Cin;
    const uint32_t *wofs = p.wofs + (size_t)grp * Ktot * p.Npad;
    const int ch0 = grp * p.N;              // first output channel of the group
    const int kc = (Ktot + p.KS - 1) >> ks_log;
    int k = ks * kc;
    const int k_end = min(Ktot, k + kc);

    uint32_t acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = 0;

    // Linear layers whose rows are word-aligned: the activations of this lane's K slice are fetched as whole words, 32
    // inner indices at a time and one block ahead of their use, so that the loop never waits for a byte load.
    if (p.mode == MODE_GEMM && p.kstride == 1 && (p.Cin & 3) == 0 && (kc & 3) == 0 &&
        (reinterpret_cast<uintptr_t>(p.x) & 3u) == 0) {
        const uint32_t *xw = reinterpret_cast<const uint32_t *>(xb);       // row of this lane
        auto fetch = [&](uint32_t *dst, int kk) {
#pragma unroll
            for (int d = 0; d < 8; ++d) dst[d] = (kk + 4 * d < k_end) ? xw[(kk >> 2) + d] : 0u;
        };
        // TILED: offsets stored [column tile][k][NT] (cell order), so the loads of consecutive k are contiguous
        auto loop = [&](auto tiled_c) {
            constexpr bool TILED = decltype(tiled_c)::value;
            uint32_t cur[8], nxt[8];
            if (k < k_end) fetch(nxt, k);
            while (k < k_end) {
#pragma unroll
                for (int d = 0; d < 8; ++d) cur[d] = nxt[d];
                if (k + 32 < k_end) fetch(nxt, k + 32);
                const int cnt = min(32, k_end - k);
                const uint32_t *wblk = wofs + ((size_t)blockIdx.y * Ktot + k) * NT;      // (TILED)
                // a whole block of 32 runs without branches, so that the lookups of one word overlap the sums of the last
                auto block = [&](auto full_c) {
                    constexpr bool FULL = decltype(full_c)::value;
#pragma unroll
                    for (int d = 0; d < 8; ++d) {
                        if (FULL || 4 * d < cnt) {          // uniform in the wave
#pragma unroll
                            for (int bq = 0; bq < 4; ++bq) {
                                const int a = (int)(int8_t)(cur[d] >> (8 * bq));
                                const uint32_t a2 = (uint32_t)(((a + p.hoff) & p.mask) << 1);
                                const uint32_t *w1 = TILED ? wblk + (4 * d + bq) * NT : wofs + (size_t)(k + 4 * d + bq) * p.Npad + n0;
#pragma unroll
                                for (int n = 0; n < NT; ++n) acc[n] += lds_entry<SIGNED>(smem, w1[n] + a2);
                            }
                        }
                    }
                };
                if (cnt == 32) block(std::true_type{});
                else block(std::false_type{});
                k += cnt;
            }
        };
        if (p.lstm) loop(std::true_type{});
        else loop(std::false_type{});
    }

    while (k < k_end) {
        const int t = k / p.Cin;
        const int c0 = k - t * p.Cin;
        const int cnt = min(p.Cin - c0, k_end - k);
        int base = 0;
        bool valid = true;
        if (p.mode == MODE_CONV) {
            const int ky = t / p.kw, kx = t - ky * p.kw;
            const int iy = oy * p.sh - p.ph + ky * p.dh, ix = ox * p.sw - p.pw + kx * p.dw;
            valid = (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
            base = iy * p.W + ix;
        } else if (p.mode == MODE_CONVT) {
            const int ky = t / p.kw, kx = t - ky * p.kw;
            const int ty = oy + p.ph - ky, tx = ox + p.pw - kx;
            const int iy = ty / p.sh, ix = tx / p.sw;
            valid = ty >= 0 && tx >= 0 && iy * p.sh == ty && ix * p.sw == tx && iy < p.H && ix < p.W;
            base = iy * p.W + ix;
        }
        const int fill2 = (p.mode == MODE_CONVT) ? p.a_skip2 : p.a_zero2;
        const int8_t *xp = xb + (valid ? base : 0) + (size_t)c0 * p.kstride;
        // (cell order: offsets stored [column tile][k][NT], see pack_row_offsets_cell_kernel)
        const size_t wstep = p.lstm ? (size_t)NT : (size_t)p.Npad;
        const uint32_t *wr = p.lstm ? wofs + ((size_t)blockIdx.y * Ktot + k) * NT : wofs + (size_t)k * p.Npad + n0;
        int c = 0;
        for (; c + 4 <= cnt; c += 4) {
            uint32_t a2[4];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int a = xp[(size_t)(c + kk) * p.kstride];
                a2[kk] = valid ? (uint32_t)(((a + p.hoff) & p.mask) << 1) : (uint32_t)fill2;
            }
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const uint32_t *w4 = wr + (size_t)(c + kk) * wstep;
#pragma unroll
                for (int n = 0; n < NT; ++n) acc[n] += lds_entry<SIGNED>(smem, w4[n] + a2[kk]);
            }
        }
        for (; c < cnt; ++c) {
            const int a = xp[(size_t)c * p.kstride];
            const uint32_t a2 = valid ? (uint32_t)(((a + p.hoff) & p.mask) << 1) : (uint32_t)fill2;
            const uint32_t *w1 = wr + (size_t)c * wstep;
#pragma unroll
            for (int n = 0; n < NT; ++n) acc[n] += lds_entry<SIGNED>(smem, w1[n] + a2);
        }
        k += cnt;
    }

    // Time-step kernels: thread tid < 2 MT (MT = 64 there) runs the cell of (row tid % MT, unit tid / MT of the
    // workgroup's pair) after the reduction.  What the cell reads besides the sums — the step's input products, the
    // previous c or h — comes from memory not touched before in this step; it is requested here, when this wave has
    // finished its lookups, and arrives while the workgroup meets at the barriers and the sums are reduced.  (Requested
    // earlier, before or during the lookups, the same loads made the LSTM step slower every time it was tried.)
    constexpr int CELL_G = NT == 8 ? 4 : (NT == 6 ? 3 : 1);
    const int cell_e = tid >> mt_log, cell_r = tid - cell_e * p.MT, cell_m = blockIdx.x * p.MT + cell_r;
    const bool cell_thread = (NT == 8 || NT == 6 || NT == 2) && p.lstm != 0 && tid < 2 * p.MT && cell_m < p.M;
    int32_t cell_ih[4] = {0, 0, 0, 0};
    float cell_prev = 0.0f, cell_b[4] = {0.0f, 0.0f, 0.0f, 0.0f}, cell_b2[3] = {0.0f, 0.0f, 0.0f};
    asm volatile("" : : : "memory");        // (keeps the loads below from being moved up into the loops)
    if (cell_thread) {
        const int u = blockIdx.y * 2 + cell_e;
#pragma unroll
        for (int g = 0; g < CELL_G; ++g) cell_ih[g] = p.acc_ih[(size_t)cell_m * CELL_G * p.Hs + (size_t)g * p.Hs + u];
        if (NT == 8) cell_prev = p.c[(size_t)cell_m * p.Hs + u];
        else if (NT == 6) cell_prev = p.h_prev[(size_t)cell_m * p.Hs + u];
        if (p.bias) {
#pragma unroll
            for (int g = 0; g < CELL_G; ++g) cell_b[g] = p.bias[g * p.Hs + u];
        }
        if (NT == 6 && p.bias_hh) {
#pragma unroll
            for (int g = 0; g < 3; ++g) cell_b2[g] = p.bias_hh[g * p.Hs + u];
        }
    }

    if (p.KS == 1) {
        if (mvalid) {
            int32_t *o = p.out + (size_t)img * p.out_ch * p.HoWo + pix;
#pragma unroll
            for (int n = 0; n < NT; ++n) {
                if (n0 + n < p.N) {
                    int32_t *q = o + (size_t)(ch0 + n0 + n) * p.HoWo;
                    if (p.shift < 0) *q = (int32_t)finish_sum(p, acc[n], ch0 + n0 + n);
                    else *q = (int32_t)((uint32_t)*q + (acc[n] << p.shift));
                }
            }
        }
        return;
    }

    // K was split over the waves: reduce the partial sums through LDS (the table is no longer needed)
    __syncthreads();
    uint32_t *red = reinterpret_cast<uint32_t *>(smem);      // [KS][NT][MT]
#pragma unroll
    for (int n = 0; n < NT; ++n) red[((size_t)ks * NT + n) * p.MT + r_in_tile] = acc[n];
    __syncthreads();
    if (NT == 2 && p.lstm == 3) {
        // one thread per (row, unit of the pair): the sum, then the plain recurrent cell (the operations of rnn_cell_kernel)
        for (int o = tid; o < 2 * p.MT; o += ROWS_THREADS) {
            // (empty statements: without them the compiler converts the values requested above to fp32 right behind their
            // loads, i.e. waits for them before the barriers)
#pragma unroll
            for (int g = 0; g < CELL_G; ++g) asm volatile("" : "+v"(cell_ih[g]));
            asm volatile("" : "+v"(cell_prev));
            const int e = o >> mt_log, r = o - e * p.MT;
            const int m2 = blockIdx.x * p.MT + r;
            if (m2 >= p.M) continue;
            const int u = blockIdx.y * 2 + e;
            const size_t ci = (size_t)m2 * p.Hs + u;
            uint32_t s = 0;
            for (int j = 0; j < p.KS; ++j) s += red[((size_t)j * NT + e) * p.MT + r];
            const float uu = (float)cell_ih[0] * p.s_ih;
            const float vv = (float)(int32_t)s * p.s_hh;
            float t = uu + vv;
            t = t + (p.bias ? cell_b[0] : 0.0f);
            const float hn = p.act == 1 ? (t > 0.0f ? t : 0.0f) : tanh_spec(t);
            p.h[ci] = hn;
            p.qh_next[ci] = (int8_t)quant1(hn, p.s_h, p.Qh);
        }
        return;
    }
    if (NT == 6 && p.lstm == 2) {
        // one thread per (row, unit of the pair): the three gate sums, then the GRU cell
        for (int o = tid; o < 2 * p.MT; o += ROWS_THREADS) {
            // (empty statements: without them the compiler converts the values requested above to fp32 right behind their
            // loads, i.e. waits for them before the barriers)
#pragma unroll
            for (int g = 0; g < CELL_G; ++g) asm volatile("" : "+v"(cell_ih[g]));
            asm volatile("" : "+v"(cell_prev));
            const int e = o >> mt_log, r = o - e * p.MT;
            const int m2 = blockIdx.x * p.MT + r;
            if (m2 >= p.M) continue;
            const int u = blockIdx.y * 2 + e;
            const size_t ci = (size_t)m2 * p.Hs + u;
            float gi[3], gh[3];
#pragma unroll
            for (int g = 0; g < 3; ++g) {
                uint32_t s = 0;
                for (int j = 0; j < p.KS; ++j) s += red[((size_t)j * NT + g * 2 + e) * p.MT + r];
                float uu = (float)cell_ih[g] * p.s_ih;
                if (p.bias) uu = uu + cell_b[g];
                float vv = (float)(int32_t)s * p.s_hh;
                if (p.bias_hh) vv = vv + cell_b2[g];
                gi[g] = uu;
                gh[g] = vv;
            }
            const float rg = sigmoid_spec(gi[0] + gh[0]);
            const float zg = sigmoid_spec(gi[1] + gh[1]);
            const float rn = rg * gh[2];
            const float ng = tanh_spec(gi[2] + rn);
            const float omz = 1.0f - zg;
            const float t0 = omz * ng;
            const float t1 = zg * cell_prev;
            const float hn = t0 + t1;
            p.h[ci] = hn;
            p.qh_next[ci] = (int8_t)quant1(hn, p.s_h, p.Qh);
        }
        return;
    }
    if (NT == 8 && p.lstm == 1) {
        // one thread per (row, unit of the pair): the four gate sums, then the cell
        for (int o = tid; o < 2 * p.MT; o += ROWS_THREADS) {
            // (empty statements: without them the compiler converts the values requested above to fp32 right behind their
            // loads, i.e. waits for them before the barriers)
#pragma unroll
            for (int g = 0; g < CELL_G; ++g) asm volatile("" : "+v"(cell_ih[g]));
            asm volatile("" : "+v"(cell_prev));
            const int e = o >> mt_log, r = o - e * p.MT;
            const int m2 = blockIdx.x * p.MT + r;
            if (m2 >= p.M) continue;
            const int u = blockIdx.y * 2 + e;
            const size_t ci = (size_t)m2 * p.Hs + u;
            float pre[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                uint32_t s = 0;
                for (int j = 0; j < p.KS; ++j) s += red[((size_t)j * NT + g * 2 + e) * p.MT + r];
                const float uu = (float)cell_ih[g] * p.s_ih;
                const float vv = (float)(int32_t)s * p.s_hh;
                float t = uu + vv;
                t = t + (p.bias ? cell_b[g] : 0.0f);
                pre[g] = t;
            }
            const float ig = sigmoid_spec(pre[0]);
            const float fg = sigmoid_spec(pre[1]);
            const float gg = tanh_spec(pre[2]);
            const float og = sigmoid_spec(pre[3]);
            const float fc = fg * cell_prev;
            const float igg = ig * gg;
            const float cn = fc + igg;
            p.c[ci] = cn;
            const float hn = og * tanh_spec(cn);
            p.h[ci] = hn;
            p.qh_next[ci] = (int8_t)quant1(hn, p.s_h, p.Qh);
        }
        return;
    }
    for (int o = tid; o < NT * p.MT; o += ROWS_THREADS) {
        const int n = o >> mt_log, r = o - n * p.MT;
        const int m2 = blockIdx.x * p.MT + r;
        if (m2 >= p.M || n0 + n >= p.N) continue;
        uint32_t s = 0;
        for (int j = 0; j < p.KS; ++j) s += red[((size_t)j * NT + n) * p.MT + r];
        const int img2 = p.mode == MODE_GEMM ? m2 : m2 / p.HoWo, pix2 = m2 - img2 * p.HoWo;
        int32_t *q = p.out + (size_t)img2 * p.out_ch * p.HoWo + (size_t)(ch0 + n0 + n) * p.HoWo + pix2;
        if (p.shift < 0) *q = (int32_t)finish_sum(p, s, ch0 + n0 + n);
        else *q = (int32_t)((uint32_t)*q + (s << p.shift));
    }
}

}  // namespace adapt
