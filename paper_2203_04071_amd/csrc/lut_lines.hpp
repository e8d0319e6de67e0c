// "Lines" kernel: table-lookup matrix product for long matrices (many rows per weight).
//
// Idea (gfx950): a 16-bit LDS gather delivers one table entry per lane per bank cycle and suffers
// bank conflicts that depend on the activation statistics.  Because the weights of a layer are
// static, the entries a workgroup needs at inner step k, for its 8 output channels n and ALL
// activation values a, form a small derived table  D_k[a][n] = T[a][W[n][k]]  (Sec. III-C: the
// table is a 1:1 image of the multiplier, so re-ordering it changes nothing).  Stored activation-
// major, one lookup with the activation as line index returns the entries of 8 output channels in
// one 128-bit LDS read.  Eight inner steps (one per lane of an 8-lane group, "k-sub" j) share a
// 128-byte line, so the 8 lanes that serve one matrix row read 8 different 16-byte columns: reads
// are conflict-free by construction whatever the activations are.
//
// Derived tables are built once per layer by pack_line_tables_kernel (K*N*2^b entries) and
// streamed from L2 into a double-buffered LDS slot, one 2^b x 128 B table per step; a workgroup
// reuses each table for 128*R matrix rows.  Work per multiply-accumulate in the hot loop:
// 1/8 LDS read + 1 v_dot2 (unpack one 16-bit half and add) + 1/4 address op.
//
// Mapping: workgroup = 1024 lanes = 128 row slots x 8 k-subs; lane (rs, j) owns rows rs*R .. rs*R+R-1
// of the tile and inner indices ci in [j*Cc, (j+1)*Cc) of every filter tap; it keeps 8*R partial
// sums which are reduced over j at the end.  Activations come from a channel-last, zero-padded
// copy of the input (conv) or from the row-major activation matrix (linear), so the address of a
// lane's next activations is base_row + tap_offset + j*Cc + t with no bounds logic; a padded tap
// reads activation 0 and therefore adds T[0][w], as the definition of the layer demands.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "elementwise.hpp"

namespace adapt {

constexpr int LINES_THREADS = 1024;
constexpr int LINE_BYTES = 128;      // 8 k-subs x 8 channels x int16

typedef short short2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// A layer's output written a second time as the NEXT convolution's input copy: quantised with that layer's activation
// scale (the quantiser of Sec. III-A), as table line indices, at the element's place in the zero-padded x-major or
// channel-last copy (see pad_channels_last_kernel) whose borders and padded channels were zeroed beforehand.  The next
// layer then needs no copy kernel of its own.  buf == nullptr: nothing to do.
struct ChainOut {
    int8_t *buf;
    int xmajor, Hp, Wp, Cp, ph, pw;
    float scale, Q;
    uint32_t mask;
    // element (image, channel c, row oy, column ox) of the producing layer's fp32 output y
    __device__ __forceinline__ void put(int img, int c, int oy, int ox, float y) const {
        const uint32_t q = (uint32_t)quant1(y, scale, Q) & mask;
        // (a copy is smaller than 2^31 bytes: 32-bit offsets)
        const uint32_t row = (uint32_t)img * (uint32_t)Hp + (uint32_t)(oy + ph), col = (uint32_t)(ox + pw);
        const uint32_t a = xmajor ? ((row * (uint32_t)(Cp >> 2) + (uint32_t)(c >> 2)) * (uint32_t)Wp + col) * 4u + (uint32_t)(c & 3)
                                  : (row * (uint32_t)Wp + col) * (uint32_t)Cp + (uint32_t)c;
        buf[a] = (int8_t)q;
    }
    // the same for channels c .. c + 3 (c a multiple of 4, Cp a multiple of 4) of one pixel: they are one aligned word
    // of either copy
    __device__ __forceinline__ uint32_t code(float y) const { return (uint32_t)quant1(y, scale, Q) & mask; }
    __device__ __forceinline__ void put4(int img, int c, int oy, int ox, uint32_t codes) const {
        const uint32_t row = (uint32_t)img * (uint32_t)Hp + (uint32_t)(oy + ph), col = (uint32_t)(ox + pw);
        const uint32_t a = xmajor ? ((row * (uint32_t)(Cp >> 2) + (uint32_t)(c >> 2)) * (uint32_t)Wp + col) * 4u
                                  : (row * (uint32_t)Wp + col) * (uint32_t)Cp + (uint32_t)c;
        *reinterpret_cast<uint32_t *>(buf + a) = codes;
    }
};

// Epilogues of the x-major kernels: lane (hq, cq) of a group of 8 lanes (j = 2 cq + hq) holds four consecutive pixels of
// channel cq (and cq + 4) of its channel tile.  `mine` = its four codes of one of them (byte i = pixel i).  Returned:
// the codes of pixel cq in the four channels that the lanes (hq, 0..3) of the group hold, byte c = channel c — one
// aligned word of the next layer's copy instead of four single bytes.  All lanes of the group must call it.
__device__ __forceinline__ uint32_t chain_gather4(uint32_t mine, int lane, int hq, int cq) {
    const int base = (lane & ~7) + hq;
    uint32_t word = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        const uint32_t v = (uint32_t)__builtin_amdgcn_ds_bpermute((base + 2 * c) << 2, (int)mine);
        word |= ((v >> (8 * cq)) & 0xffu) << (8 * c);
    }
    return word;
}

struct LinesParams {
    const int8_t *xt;       // activations (see above)
    const uint4 *dt;        // derived tables [n_tiles][steps][2^b lines][8 columns] x 16 B
    int32_t *out;
    int M, N, n_tiles;
    int Cc, taps, kw;       // steps = taps * Cc
    int bits;
    int HoWo, Wo;           // linear: 1, 1
    long long img_stride;   // bytes of xt per image (linear: bytes per row); the whole of xt is < 2^31 bytes
    int oy_stride, ox_stride;   // bytes of xt per output row / column step (stride * padded width * Cp, stride * Cp)
    int ky_stride, kx_stride;   // bytes of xt per filter row / column (dilation * padded width * Cp, dilation * Cp)
    int shift;              // < 0: out = acc; >= 0: out += acc << shift
    int ch_stride;          // x-major activation copy only: bytes per channel step (padded width); else unused
    // Where row (img, a, b) of the M x N product goes: out[(img * N + n) * out_plane + out_off + a * out_sy + b * out_sx],
    // (a, b) = position in the HoWo / Wo grid.  Convolution: out_plane = HoWo, out_sy = Wo, out_sx = 1.
    int out_plane, out_sy, out_sx;
    // A transposed convolution with stride s is s * s ordinary stride-1 convolutions ("phases"), each with its own
    // derived tables, window origin in xt and interleaved output positions; up to 4 of them share one launch.
    // Workgroup order: n-tile fastest, then row tile, then phase.
    int phases, m_tiles;
    // Fused rescaling (single-pass tables only): when deq != 0 the output buffer receives fp32
    //   y = float(acc) * scale, then + bias[n] if bias, then max(y, 0) if act == 1
    // (the operations of dequant_kernel and relu_kernel, each rounded separately) instead of the int32 sums.
    int deq, act;
    float scale;
    const float *scales;    // one scale per output channel (then `scale` is unused), or nullptr
    const float *bias;
    const float *resid;     // residual input: fp32 tensor of the output's shape added after the bias, before act; or nullptr
    int xt_off[4];          // bytes into xt
    int out_off[4];         // elements into an output plane
    long long dt_off[4];    // 16-byte units into dt
    // Split of the inner dimension over workgroups (fast kernel only): workgroup slice ks handles the groups of four
    // steps [ks * gps, min(groups, (ks + 1) * gps)) and stores its partial sums at out + ks * ks_out_stride (elements);
    // reduce_partials_kernel adds the slices up.  ksplit == 1: no split.
    int ksplit, gps;
    long long ks_out_stride;
    // the divisions every lane (rows -> image, row, column) and every wave (workgroup id -> tiles) starts with, as
    // multiply-and-shift: they were 1 - 2 us of every launch
    FastDiv d_HoWo, d_Wo, d_ntiles, d_mtiles, d_phases;
    int no_out;             // 1: only the chained copy is wanted, the finished sums are not stored (out is then never dereferenced)
    int copy_lines;         // quad and fast kernels: lines of every table that are copied into LDS (all 2^bits, or the first half when
                            // the activations are known to be >= 0: their codes then never select the other half)
    int corr;               // quad kernel (digit tables): added to every finished sum, digit_c x real lookups (lut_quad.hpp); else 0
    // Tap pairing (fast kernel, PAIRED): layers with fewer than 32 (padded) channels per tap put pair_g = 32 / Cp taps
    // side by side in a group of four steps: k-sub j serves tap pair_g * group + j / pair_cg and the four channels
    // 4 * (j % pair_cg) + step of it (pair_cg = Cp / 4).  `taps` then counts groups and Cc is 4; taps_real is the
    // number of filter taps (taps beyond it are padding: all-zero tables).
    int pair_g, pair_cg, taps_real;
    // Transposed convolution with the border terms taken off in the epilogue (zsum != nullptr; single-pass tables, no
    // split of the inner dimension): the phase convolutions look up every window tap, also those over the zero border
    // of the padded copy, but the layer is defined over real (input, weight) pairs only; zsum[co][tap] = sum over the
    // input channels of T[0][w] is what such a tap added.  Output and input sizes, filter, stride, padding, and the
    // widths Ly / Lx of the output border in which some tap has no input pixel.
    ChainOut chain;     // (ordinary convolutions with fused rescaling only: out_sy = Wo, out_sx = 1)
    const int32_t *zsum;
    FastDiv cv_s;                       // division by the stride
    int cv_Ho, cv_Wo, cv_H, cv_W, cv_kh, cv_kw, cv_pad, cv_Ly, cv_Lx;
};

// what is stored for the finished sum v of output channel n (see LinesParams::deq)
// off: element offset of the output position (for the residual input)
// What the window taps WITHOUT an input pixel added to output pixel (oy, ox) of channel co of a transposed convolution
// (see LinesParams::zsum); zero away from the border.
__device__ __forceinline__ uint32_t convt_border_terms(const LinesParams &p, int co, int oy, int ox) {
    const int st = (int)p.cv_s.d;
    const int qy = (int)p.cv_s.div((uint32_t)(oy + p.cv_pad)), ry = oy + p.cv_pad - qy * st;
    const int qx = (int)p.cv_s.div((uint32_t)(ox + p.cv_pad)), rx = ox + p.cv_pad - qx * st;
    uint32_t extra = 0;
    for (int m = 0; m * st + ry < p.cv_kh; ++m) {
        const bool yin = qy - m >= 0 && qy - m < p.cv_H;
        for (int nn = 0; nn * st + rx < p.cv_kw; ++nn) {
            const bool xin = qx - nn >= 0 && qx - nn < p.cv_W;
            if (!(yin && xin)) extra += (uint32_t)p.zsum[(size_t)co * p.cv_kh * p.cv_kw + (ry + st * m) * p.cv_kw + (rx + st * nn)];
        }
    }
    return extra;
}

// The same for the four pixels (oy, ox + i * stride), i = 0 .. 3, of one phase: they share the row's taps and the column
// residue, so every zero sum is loaded once.
__device__ __forceinline__ void convt_border_terms4(const LinesParams &p, int co, int oy, int ox, uint32_t (&extra)[4]) {
    const int st = (int)p.cv_s.d;
    const int qy = (int)p.cv_s.div((uint32_t)(oy + p.cv_pad)), ry = oy + p.cv_pad - qy * st;
    const int qx = (int)p.cv_s.div((uint32_t)(ox + p.cv_pad)), rx = ox + p.cv_pad - qx * st;
    const int32_t *z = p.zsum + (size_t)co * p.cv_kh * p.cv_kw;
#pragma unroll
    for (int i = 0; i < 4; ++i) extra[i] = 0;
    for (int m = 0; m * st + ry < p.cv_kh; ++m) {
        const bool yin = qy - m >= 0 && qy - m < p.cv_H;
        for (int nn = 0; nn * st + rx < p.cv_kw; ++nn) {
            const int x0 = qx - nn;             // input column of pixel 0; pixel i has x0 + i
            if (yin && x0 >= 0 && x0 + 3 < p.cv_W) continue;
            const uint32_t zz = (uint32_t)z[(ry + st * m) * p.cv_kw + (rx + st * nn)];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (!(yin && (unsigned)(x0 + i) < (unsigned)p.cv_W)) extra[i] += zz;
        }
    }
}

// EXTRA: the instantiation also knows tanh; the plain one does not (eight inlined copies of that code in an epilogue
// cost the ordinary layers about a microsecond per launch)
template <bool EXTRA = false>
__device__ __forceinline__ uint32_t finish_sum(const LinesParams &p, uint32_t v, int n, size_t off) {
    if (!p.deq) return v;
    float y = (float)(int32_t)v * (p.scales ? p.scales[n] : p.scale);
    if (p.bias) y = y + p.bias[n];
    if (p.resid) y = y + p.resid[off];
    if (p.act == 1) y = y > 0.0f ? y : 0.0f;
    else if (EXTRA && p.act == 2) y = tanh_spec(y);
    return __float_as_uint(y);
}

// per-phase launch parameters without indexing the by-value argument block dynamically
template <typename T>
__device__ __forceinline__ T pick4(const T *v, int i) {
    return i == 0 ? v[0] : (i == 1 ? v[1] : (i == 2 ? v[2] : v[3]));
}

// Activation sources of the copy kernels: already quantised int8, or fp32 quantised on the fly with the quantiser of
// quantize_kernel (Sec. III-A), so that a layer needs no separate quantisation pass.  The copies hold table line
// indices (the kernels that extract a bit field do not care, the quad kernel relies on it).
// byte(): the operand as a table line index, i.e. its two's-complement bits below 2^b (mask = 2^b - 1)
// load() / code(): the two halves of byte(), for kernels that request several operands before they convert the first
struct SrcI8 {
    typedef int8_t raw_t;
    const int8_t *x;
    uint32_t mask;
    __device__ __forceinline__ uint32_t byte(size_t i) const { return (uint32_t)(uint8_t)x[i] & mask; }
    __device__ __forceinline__ raw_t load(uint32_t i) const { return x[i]; }
    __device__ __forceinline__ uint32_t code(raw_t v) const { return (uint32_t)(uint8_t)v & mask; }
};
struct SrcF32 {
    typedef float raw_t;
    const float *x;
    float scale, Q;
    uint32_t mask;
    __device__ __forceinline__ uint32_t byte(size_t i) const { return (uint32_t)quant1(x[i], scale, Q) & mask; }
    __device__ __forceinline__ raw_t load(uint32_t i) const { return x[i]; }
    __device__ __forceinline__ uint32_t code(raw_t v) const { return (uint32_t)quant1(v, scale, Q) & mask; }
};

// NCHW int8 -> zero-padded copy, Cp (a multiple of 8) channels per pixel, in one of two orders:
//   xmajor == 0: channel-last            [N][H + 2 ph][W + 2 pw][Cp]
//   xmajor == 1: groups of four channels [N][H + 2 ph][Cp / 4][W + 2 pw][4]  (the four channel bytes of
//                consecutive pixels are adjacent, so 4 rows x 4 channels of a lane are 16 contiguous bytes)
template <typename Src>
__global__ void pad_channels_last_kernel(const Src x, int8_t *__restrict__ xt, int N, int C, int H,
                                         int W, int ph, int pw, int Cp, int xmajor, FastDiv dwp, FastDiv dc4, FastDiv dhp,
                                         int fast) {
    const int Hp = H + 2 * ph, Wp = W + 2 * pw;
    const size_t total = (size_t)N * Hp * Wp * (Cp / 4);
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        // consecutive threads walk along x for a fixed group of 4 channels: reads coalesce per channel plane
        int xp, c4, yp, n;
        if (fast) {             // total < 2^31
            const uint32_t i32 = (uint32_t)i;
            const uint32_t r1 = dwp.div(i32);
            xp = (int)(i32 - r1 * dwp.d);
            const uint32_t r2 = dc4.div(r1);
            c4 = (int)(r1 - r2 * dc4.d);
            const uint32_t r3 = dhp.div(r2);
            yp = (int)(r2 - r3 * dhp.d);
            n = (int)r3;
        } else {
            xp = (int)(i % Wp);
            size_t r = i / Wp;
            c4 = (int)(r % (Cp / 4));
            r /= (Cp / 4);
            yp = (int)(r % Hp);
            n = (int)(r / Hp);
        }
        const int y = yp - ph, xx = xp - pw;
        uint32_t v = 0;
        if (y >= 0 && y < H && xx >= 0 && xx < W) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = c4 * 4 + q;
                if (c < C) v |= x.byte((((size_t)n * C + c) * H + y) * W + xx) << (8 * q);
            }
        }
        if (xmajor) *reinterpret_cast<uint32_t *>(xt + i * 4) = v;
        else *reinterpret_cast<uint32_t *>(xt + (((size_t)n * Hp + yp) * Wp + xp) * Cp + c4 * 4) = v;
    }
}

// The same copy for tensors of fewer than 2^31 elements on both sides, U output words per thread (word t, t + threads,
// ...): all 4 U operands are requested before the first is converted.  One word per thread makes 9 waves per SIMD at
// the benchmark layer, one more than fit at a time, so part of the copy waited for a second round of waves (one
// memory round trip each); with two words per thread everything is resident at once and in flight together
// (measured: 7.0 against 7.6 - 8.4 us; three words the same, six words no gain).
template <typename Src, int U>
__global__ __launch_bounds__(256) void pad_channels_last_multi_kernel(const Src x, int8_t *__restrict__ xt, int C, int H, int W, int ph,
                                                                      int pw, int Cp, int xmajor, FastDiv dwp, FastDiv dc4,
                                                                      FastDiv dhp, uint32_t total) {
    const uint32_t threads = gridDim.x * 256u, t = blockIdx.x * 256u + threadIdx.x;
    const uint32_t HW = (uint32_t)H * (uint32_t)W;
    typename Src::raw_t raw[U][4];
    uint32_t dst[U];
    bool live[U], have[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t i = t + (uint32_t)u * threads;
        live[u] = i < total;
        const uint32_t ii = live[u] ? i : 0u;
        const uint32_t r1 = dwp.div(ii), xp = ii - r1 * dwp.d;
        const uint32_t r2 = dc4.div(r1), c4 = r1 - r2 * dc4.d;
        const uint32_t n = dhp.div(r2), yp = r2 - n * dhp.d;
        const int y = (int)yp - ph, xx = (int)xp - pw;
        const bool inside = live[u] && y >= 0 && y < H && xx >= 0 && xx < W;
        const uint32_t src = ((n * (uint32_t)C + c4 * 4u) * (uint32_t)H + (uint32_t)(inside ? y : 0)) * (uint32_t)W + (uint32_t)(inside ? xx : 0);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            have[u][q] = inside && (int)(c4 * 4u) + q < C;
            raw[u][q] = x.load(have[u][q] ? src + (uint32_t)q * HW : 0u);
        }
        dst[u] = xmajor ? ii * 4u : ((n * dhp.d + yp) * dwp.d + xp) * (uint32_t)Cp + c4 * 4u;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        uint32_t v = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) v |= (have[u][q] ? x.code(raw[u][q]) : 0u) << (8 * q);
        if (live[u]) *reinterpret_cast<uint32_t *>(xt + dst[u]) = v;
    }
}

// [M][K] int8 -> [M][Kp] with zero fill, Kp a multiple of 32
template <typename Src>
__global__ void pad_rows_kernel(const Src a, int8_t *__restrict__ at, int M, int K, int Kp) {
    const size_t total = (size_t)M * Kp;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int k = (int)(i % Kp);
        const size_t m = i / Kp;
        at[i] = k < K ? (int8_t)a.byte(m * K + k) : (int8_t)0;
    }
}

// [M][K] int8 -> [Kp / 4][M][4]: for four consecutive inner indices the bytes of consecutive rows are adjacent (the
// x-major order above with one image of one row), zero fill beyond K.  One workgroup of 256 threads moves a tile of
// 64 rows x 64 inner indices through LDS so that both the reads (along K) and the writes (along M) coalesce.
template <typename Src>
__global__ __launch_bounds__(256) void rows_to_xmajor_kernel(const Src a, int8_t *__restrict__ at, int M, int K, int Kp) {
    __shared__ uint32_t tile[16][65];
    const int m0 = blockIdx.x * 64, c0 = blockIdx.y * 16;      // c counts groups of four inner indices
    const int tid = threadIdx.x;
    const bool fast = std::is_same<Src, SrcI8>::value && (K % 4 == 0) && ((reinterpret_cast<uintptr_t>(a.x) & 3u) == 0);
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int ml = pass * 16 + tid / 16, c = tid % 16;
        const int m = m0 + ml, k = (c0 + c) * 4;
        uint32_t v = 0;
        if (m < M) {
            if (fast) {
                if (k < K) v = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const int8_t *>(a.x) + (size_t)m * K + k) & (a.mask * 0x01010101u);
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (k + q < K) v |= a.byte((size_t)m * K + k + q) << (8 * q);
            }
        }
        tile[c][ml] = v;
    }
    __syncthreads();
#pragma unroll
    for (int pass = 0; pass < 4; ++pass) {
        const int c = pass * 4 + tid / 64, ml = tid % 64;
        const int m = m0 + ml;
        if (m < M && (c0 + c) * 4 < Kp) *reinterpret_cast<uint32_t *>(at + ((size_t)(c0 + c) * M + m) * 4) = tile[c][ml];
    }
}

// Derived tables.  lut16: [2^b][2^b] 16-bit entries, index [a & mask][w & mask] (two's-complement
// wrap of the signed operands, so activation 0 is line 0).  One thread writes the 8 channel entries
// of (n-tile, step, line a, k-sub j).  wmode 0: w[n][K] / [Cout][Cin][taps]; wmode 1: [Cin][Cout][taps].
// pair_g > 0: tap pairing (see LinesParams): step = 4 * group + t, k-sub j holds tap pair_g * group + j / pair_cg,
// channel 4 * (j % pair_cg) + t; `steps` is then 4 * number of groups, else taps * Cc.
__global__ void pack_line_tables_kernel(const uint16_t *__restrict__ lut16, const int8_t *__restrict__ w,
                                        uint4 *__restrict__ dt, int bits, int N, int Cin, int taps, int Cc,
                                        int n_tiles, int wmode, int pair_g, int pair_cg) {
    const int lines = 1 << bits, mask = lines - 1;
    const size_t per_table = (size_t)lines * 8;
    const size_t steps = pair_g > 0 ? (size_t)((taps + pair_g - 1) / pair_g) * 4 : (size_t)taps * Cc;
    const size_t total = (size_t)n_tiles * steps * per_table;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int j = (int)(i & 7);
        const int a = (int)((i >> 3) & mask);
        const size_t ts = i / per_table;
        const int step = (int)(ts % steps);
        const int nt = (int)(ts / steps);
        int tap, ci;
        if (pair_g > 0) {
            tap = pair_g * (step >> 2) + j / pair_cg;
            ci = 4 * (j % pair_cg) + (step & 3);
        } else {
            tap = step / Cc;
            ci = j * Cc + (step - tap * Cc);
        }
        uint32_t e[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int n = nt * 8 + c;
            uint32_t v = 0;
            if (n < N && ci < Cin && tap < taps) {
                const size_t wi = wmode == 0 ? ((size_t)n * Cin + ci) * taps + tap : ((size_t)ci * N + n) * taps + tap;
                v = lut16[(size_t)a * lines + ((int)w[wi] & mask)];
            }
            e[c] = v;
        }
        dt[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
}

// Derived tables of the s * s phases of a transposed convolution with stride s (kh and kw multiples of s).
// Output rows with (oy + pad) % s == ry only meet the filter rows ky = ry + s m, m = 0..Ty-1 (Ty = kh / s), and
// input rows iy = (oy + pad) / s - m: an ordinary stride-1 convolution over the input whose window row m'
// (top to bottom) carries filter row ky = ry + s (Ty - 1 - m'); likewise for columns.
// w is [Cin][Cout][kh][kw]; layout [phase = ry * s + rx][n_tile][step = (m' * Tx + n') * Cc + t][line][k-sub].
__global__ void pack_line_tables_convt_kernel(const uint16_t *__restrict__ lut16, const int8_t *__restrict__ w,
                                              uint4 *__restrict__ dt, int bits, int N, int Cin, int kh, int kw, int s,
                                              int Cc, int n_tiles) {
    const int lines = 1 << bits, mask = lines - 1;
    const int Ty = kh / s, Tx = kw / s;
    const size_t per_table = (size_t)lines * 8;
    const size_t steps = (size_t)Ty * Tx * Cc;
    const size_t per_phase = (size_t)n_tiles * steps * per_table;
    const size_t total = per_phase * s * s;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int phase = (int)(i / per_phase);
        const size_t ip = i - (size_t)phase * per_phase;
        const int ry = phase / s, rx = phase - ry * s;
        const int j = (int)(ip & 7);
        const int a = (int)((ip >> 3) & mask);
        const size_t ts = ip / per_table;
        const int step = (int)(ts % steps);
        const int nt = (int)(ts / steps);
        const int tap = step / Cc, t = step - tap * Cc;
        const int mw = tap / Tx, nw = tap - mw * Tx;
        const int ky = ry + s * (Ty - 1 - mw), kx = rx + s * (Tx - 1 - nw);
        const int ci = j * Cc + t;
        uint32_t e[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int n = nt * 8 + c;
            uint32_t v = 0;
            if (n < N && ci < Cin) {
                const size_t wi = (((size_t)ci * N + n) * kh + ky) * kw + kx;
                v = lut16[(size_t)a * lines + ((int)w[wi] & mask)];
            }
            e[c] = v;
        }
        dt[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
}

// zsum[co][ky * kw + kx] = sum over ci of T[0][w[ci][co][ky][kx]] (int32, wrap-around): what one window tap that
// lies over the zero border of the padded input copy adds to an output of channel co.
// lut_lo / lut_hi: 16-bit tables [a & mask][w & mask]; lut_hi == nullptr: lut_lo holds signed entries.
__global__ void convt_zero_sums_kernel(const uint16_t *__restrict__ lut_lo, const uint16_t *__restrict__ lut_hi,
                                       const int8_t *__restrict__ w, int32_t *__restrict__ zsum, int bits, int N, int Cin,
                                       int taps) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * taps) return;
    const int co = idx / taps, tap = idx - co * taps;
    const int mask = (1 << bits) - 1;
    uint32_t sum = 0;
    for (int ci = 0; ci < Cin; ++ci) {
        const int wv = (int)w[((size_t)ci * N + co) * taps + tap] & mask;      // row of activation 0 is row 0
        if (lut_hi) sum += (uint32_t)lut_lo[wv] + ((uint32_t)(int32_t)(int16_t)lut_hi[wv] << 16);
        else sum += (uint32_t)(int32_t)(int16_t)lut_lo[wv];
    }
    zsum[idx] = (int32_t)sum;
}

// The phase convolutions look up every window tap, also those over the zero border; the transposed convolution is
// defined over real (input, weight) pairs only, so for every output pixel near the border the sums of the taps without
// an input pixel are taken off again.  region 0: the first/last Ly output rows (all columns); region 1: the first/last
// Lx columns of the remaining rows.  One thread per (image, channel, pixel of the region).
__global__ void convt_border_fix_kernel(int32_t *__restrict__ out, const int32_t *__restrict__ zsum, int planes, int Cout,
                                        int Ho, int Wo, int H, int W, int kh, int kw, int s, int pad, int Ly, int Lx,
                                        int region) {
    const int nrows = 2 * Ly < Ho ? 2 * Ly : Ho;        // rows of region 0
    const int ncols = 2 * Lx < Wo ? 2 * Lx : Wo;
    const int rr = region == 0 ? nrows : Ho - nrows;
    const int rc = region == 0 ? Wo : ncols;
    const size_t total = (size_t)planes * rr * rc;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int c = (int)(i % rc);
        const size_t t = i / rc;
        const int r = (int)(t % rr);
        const int plane = (int)(t / rr);
        int oy, ox;
        if (region == 0) {
            oy = (nrows == Ho || r < Ly) ? r : Ho - (nrows - r);
            ox = c;
        } else {
            oy = Ly + r;
            ox = (ncols == Wo || c < Lx) ? c : Wo - (ncols - c);
        }
        const int co = plane % Cout;
        const int qy = (oy + pad) / s, ry = (oy + pad) - qy * s;
        const int qx = (ox + pad) / s, rx = (ox + pad) - qx * s;
        uint32_t extra = 0;
        for (int m = 0; m * s + ry < kh; ++m) {
            const bool yin = qy - m >= 0 && qy - m < H;
            for (int n = 0; n * s + rx < kw; ++n) {
                const bool xin = qx - n >= 0 && qx - n < W;
                if (!(yin && xin)) extra += (uint32_t)zsum[(size_t)co * kh * kw + (ry + s * m) * kw + (rx + s * n)];
            }
        }
        int32_t *q = out + ((size_t)plane * Ho + oy) * Wo + ox;
        *q = (int32_t)((uint32_t)*q - extra);
    }
}

// In-place rescaling of a buffer of int32 sums into fp32 for the cases the product kernels cannot rescale themselves
// (two-pass tables, transposed convolutions whose border terms are taken off afterwards, tanh outputs):
// y = float(acc) * scale, + bias[c], then act (0 none, 1 max(y, 0), 2 tanh as in unary_kernel).
// (chain: see ChainOut; chain_wo = width of the output, for the element's row and column)
__global__ __launch_bounds__(EW_THREADS) void finish_inplace_kernel(int32_t *__restrict__ buf, size_t n, size_t channels, size_t inner,
                                                                    float scale, const float *__restrict__ scales,
                                                                    const float *__restrict__ bias, const float *__restrict__ resid,
                                                                    int act, ChainOut chain, int chain_wo) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) {
        const size_t ch = (i / inner) % channels;
        float y = (float)buf[i] * (scales ? scales[ch] : scale);
        if (bias) y = y + bias[ch];
        if (resid) y = y + resid[i];
        if (act == 1) y = y > 0.0f ? y : 0.0f;
        else if (act == 2) y = tanh_spec(y);
        reinterpret_cast<float *>(buf)[i] = y;
        if (chain.buf) {
            const size_t pix = i % inner;
            chain.put((int)(i / (inner * channels)), (int)ch, (int)(pix / chain_wo), (int)(pix % chain_wo), y);
        }
    }
}

// out[i] = sum over the ks slices of part[k * stride + i]; then either stored (shift < 0; deq != 0: rescaled as in
// finish_inplace_kernel) or added to out[i] after a left shift (second half of a two-pass table)
__global__ __launch_bounds__(EW_THREADS) void reduce_partials_kernel(const int32_t *__restrict__ part, int ks, size_t stride_elems,
                                                                     int32_t *__restrict__ out, size_t n, int shift, int deq,
                                                                     size_t channels, size_t inner, float scale,
                                                                     const float *__restrict__ scales,
                                                                     const float *__restrict__ bias, const float *__restrict__ resid,
                                                                     int act, ChainOut chain, int chain_wo, FastDiv d_inner,
                                                                     FastDiv d_ch, FastDiv d_wo, int quads) {
    const size_t stride = (size_t)gridDim.x * EW_THREADS;
    if (quads) {
        // rescaled output, fewer than 2^31 elements, planes and rows that are multiples of four elements, 16-byte aligned
        // buffers: four consecutive elements per thread (one channel, one row), index arithmetic in 32 bits by
        // multiply-and-shift (the general loop below spends most of its time in 64-bit divisions)
        const uint32_t n4 = (uint32_t)(n >> 2), stride4 = (uint32_t)(stride_elems >> 2);
        const uint4 *part4 = reinterpret_cast<const uint4 *>(part);
        const uint32_t inner32 = (uint32_t)inner, ch32 = (uint32_t)channels;
        for (uint32_t q = blockIdx.x * EW_THREADS + threadIdx.x; q < n4; q += (uint32_t)stride) {
            uint4 v = part4[q];
            for (int k = 1; k < ks; ++k) {
                const uint4 t = part4[(size_t)k * stride4 + q];
                v.x += t.x; v.y += t.y; v.z += t.z; v.w += t.w;
            }
            const uint32_t i = q * 4u;
            const uint32_t plane = d_inner.div(i), img = d_ch.div(plane);
            const uint32_t ch = plane - img * ch32, pix = i - plane * inner32;
            const float sc = scales ? scales[ch] : scale;
            float y[4] = {(float)(int32_t)v.x * sc, (float)(int32_t)v.y * sc, (float)(int32_t)v.z * sc, (float)(int32_t)v.w * sc};
            if (bias) {
                const float b = bias[ch];
#pragma unroll
                for (int e = 0; e < 4; ++e) y[e] = y[e] + b;
            }
            if (resid) {
                const float4 r = reinterpret_cast<const float4 *>(resid)[q];
                y[0] = y[0] + r.x; y[1] = y[1] + r.y; y[2] = y[2] + r.z; y[3] = y[3] + r.w;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (act == 1) y[e] = y[e] > 0.0f ? y[e] : 0.0f;
                else if (act == 2) y[e] = tanh_spec(y[e]);
            }
            if (out) reinterpret_cast<float4 *>(out)[q] = make_float4(y[0], y[1], y[2], y[3]);      // (nullptr: only the copy is wanted)
            if (chain.buf) {
                const uint32_t oy = d_wo.div(pix), ox = pix - oy * (uint32_t)chain_wo;
#pragma unroll
                for (int e = 0; e < 4; ++e) chain.put((int)img, (int)ch, (int)oy, (int)ox + e, y[e]);
            }
        }
        return;
    }
    for (size_t i = (size_t)blockIdx.x * EW_THREADS + threadIdx.x; i < n; i += stride) {
        uint32_t v = 0;
        for (int k = 0; k < ks; ++k) v += (uint32_t)part[(size_t)k * stride_elems + i];
        if (shift >= 0) {
            out[i] = (int32_t)((uint32_t)out[i] + (v << shift));
        } else if (deq) {
            const size_t ch = (i / inner) % channels;
            float y = (float)(int32_t)v * (scales ? scales[ch] : scale);
            if (bias) y = y + bias[ch];
            if (resid) y = y + resid[i];
            if (act == 1) y = y > 0.0f ? y : 0.0f;
            else if (act == 2) y = tanh_spec(y);
            reinterpret_cast<float *>(out)[i] = y;
            if (chain.buf) {
                const size_t pix = i % inner;
                chain.put((int)(i / (inner * channels)), (int)ch, (int)(pix / chain_wo), (int)(pix % chain_wo), y);
            }
        } else {
            out[i] = (int32_t)v;
        }
    }
}

template <bool SIGNED>
__device__ __forceinline__ void accum8(uint32_t *acc, const uint4 v) {
    const uint32_t r[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        if (SIGNED) {
            const short2_t s = __builtin_bit_cast(short2_t, r[q]);
            acc[2 * q] = (uint32_t)__builtin_amdgcn_sdot2(s, short2_t{1, 0}, (int)acc[2 * q], false);
            acc[2 * q + 1] = (uint32_t)__builtin_amdgcn_sdot2(s, short2_t{0, 1}, (int)acc[2 * q + 1], false);
        } else {
            const ushort2_t s = __builtin_bit_cast(ushort2_t, r[q]);
            acc[2 * q] = __builtin_amdgcn_udot2(s, ushort2_t{1, 0}, acc[2 * q], false);
            acc[2 * q + 1] = __builtin_amdgcn_udot2(s, ushort2_t{0, 1}, acc[2 * q + 1], false);
        }
    }
}

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef const __attribute__((address_space(1))) void *global_void_ptr;

constexpr int TABLE_U4_MAX = 256 * 8;    // 16-byte units of one 8-bit table (32 KB)

// s_waitcnt immediates below use the gfx9 encoding: vmcnt in bits 3:0, expcnt (left at 7) in 6:4, lgkmcnt(0) in 11:8

// Asynchronous copy of one derived table (table_u4 16-byte units) from global memory straight into
// an LDS buffer (no registers in between): lane l of a wave writes the 16 bytes at M0 + 16 l.
// Written in assembly so that the compiler neither counts these operations nor guards later LDS
// reads against them; the kernel orders them itself with wait_and_barrier().
__device__ __forceinline__ void table_dma(const uint4 *src, uint4 *dst, int table_u4, int wave, int lane) {
    const int u0 = wave * 64;
    if (u0 < table_u4) {
        if (u0 + lane < table_u4) {
            const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_void_ptr)(dst + u0);
            const uint32_t voff = (uint32_t)(u0 + lane) * 16u;
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                         :
                         : "v"(voff), "s"(src), "s"(lds_addr)
                         : "memory", "m0");
        }
    }
    const int u1 = u0 + LINES_THREADS;
    if (u1 < table_u4) {
        const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_void_ptr)(dst + u1);
        const uint32_t voff = (uint32_t)(u1 + lane) * 16u;
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                     :
                     : "v"(voff), "s"(src), "s"(lds_addr)
                     : "memory", "m0");
    }
}

// wait until at most `keep` of this wave's most recent memory operations are outstanding (memory
// operations of one wave complete in order), and all of its LDS reads have returned
__device__ __forceinline__ void wait_vm(int keep) {
    switch (keep < 0 ? 0 : (keep > 10 ? 10 : keep)) {      // rounding down only waits longer
        case 0: __builtin_amdgcn_s_waitcnt(0x0070); break;
        case 1: __builtin_amdgcn_s_waitcnt(0x0071); break;
        case 2: __builtin_amdgcn_s_waitcnt(0x0072); break;
        case 3: __builtin_amdgcn_s_waitcnt(0x0073); break;
        case 4: __builtin_amdgcn_s_waitcnt(0x0074); break;
        case 5: __builtin_amdgcn_s_waitcnt(0x0075); break;
        case 6: __builtin_amdgcn_s_waitcnt(0x0076); break;
        case 7: __builtin_amdgcn_s_waitcnt(0x0077); break;
        case 8: __builtin_amdgcn_s_waitcnt(0x0078); break;
        case 9: __builtin_amdgcn_s_waitcnt(0x0079); break;
        default: __builtin_amdgcn_s_waitcnt(0x007a); break;
    }
}

template <bool SIGNED>
__device__ __forceinline__ void accum8(uint32_t *acc, const u32x4_t v) {
    accum8<SIGNED>(acc, make_uint4(v.x, v.y, v.z, v.w));
}

// Sum of an R x 8 block of partial sums (acc[row * 8 + channel]) over the 8 k-sub lanes (j = 0..7) of a row slot,
// as a reduce-scatter in three exchanges: in each, a lane keeps the half of its values that it will store, hands
// the other half to its partner and adds what the partner hands over.  Partners: 7 - j (splits on channel bit 1),
// j ^ 1 (splits on the half of the rows), j ^ 2 (channel bit 0).  Lane j ends with w[i][t] = the complete sum of row
// (R / 2) * (j & 1) + i, channel (j >> 1) + 4 * t.  (Two thirds of the operations of summing everything everywhere
// and then selecting, and few enough live registers that nothing spills.)
template <int R>
__device__ __forceinline__ void reduce_scatter(const uint32_t *acc, int j, uint32_t (&w)[R / 2][2]) {
    static_assert(R % 2 == 0, "rows are split in two halves");
    const bool k0 = j & 1, k1 = j & 2, k2 = j & 4;
    uint32_t s1[R][4];                      // [row][channel bit 0 + 2 * channel bit 2], channel bit 1 == k2
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const uint32_t lo = acc[i * 8 + (cc & 1) + 4 * (cc >> 1)], hi = acc[i * 8 + (cc & 1) + 4 * (cc >> 1) + 2];
            const uint32_t keep = k2 ? hi : lo, give = k2 ? lo : hi;
            s1[i][cc] = keep + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)give, 0x141, 0xF, 0xF, true);   // row_half_mirror
        }
    uint32_t s2[R / 2][4];                  // [row of half k0][as above]
#pragma unroll
    for (int i = 0; i < R / 2; ++i)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            const uint32_t keep = k0 ? s1[i + R / 2][cc] : s1[i][cc], give = k0 ? s1[i][cc] : s1[i + R / 2][cc];
            s2[i][cc] = keep + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)give, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
        }
#pragma unroll
    for (int i = 0; i < R / 2; ++i)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint32_t keep = k1 ? s2[i][2 * t + 1] : s2[i][2 * t], give = k1 ? s2[i][2 * t] : s2[i][2 * t + 1];
            w[i][t] = keep + (uint32_t)__builtin_amdgcn_update_dpp(0, (int)give, 0x4E, 0xF, 0xF, true);      // quad_perm [2,3,0,1]
        }
}

// R: rows per lane.  SIGNED: entries are int16 (else uint16 low halves of a wide table).
// REGULAR: the R rows of every lane are equally spaced in xt (linear layers; convolutions whose
// output width is a multiple of R), so one base offset per lane suffices.
template <int R, bool SIGNED, bool REGULAR>
__global__ __launch_bounds__(LINES_THREADS) void lut_lines_kernel(const LinesParams p) {
    // three table buffers: read one, the next one is complete, the third is being filled
    __shared__ uint4 tbl[3 * TABLE_U4_MAX];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = tid & 7;
    const int rs = tid >> 3;
    const int wg = (int)p.d_ntiles.div(blockIdx.x);     // consecutive workgroup ids land on different XCDs:
    const int nt = blockIdx.x - wg * p.n_tiles;         // n-tile == id mod n_tiles keeps one table stream per XCD L2
    const int ph = (int)p.d_mtiles.div((uint32_t)wg);
    const int mt = wg - ph * p.m_tiles;
    const int8_t *const xt = p.xt + pick4(p.xt_off, ph);
    const int out_off = pick4(p.out_off, ph);
    const int lines = 1 << p.bits;
    const int table_u4 = lines * 8;
    const int steps = p.taps * p.Cc;
    const uint4 *dt = p.dt + pick4(p.dt_off, ph) + (size_t)nt * steps * table_u4;
    // memory operations per table copy issued by this wave (uniform in the wave)
    const int dma_ops = (wave * 64 < table_u4 ? 1 : 0) + (wave * 64 + LINES_THREADS < table_u4 ? 1 : 0);

    // byte offset in xt of (row origin + first inner index of this lane's k-sub).  REGULAR (M is a
    // multiple of R): a lane whose rows lie beyond the matrix reads the last R rows instead.
    uint32_t base[REGULAR ? 1 : R];
    uint32_t row_step = 0;          // REGULAR: distance between consecutive rows of a lane
    {
        int r0 = mt * (128 * R) + rs * R;
        if (REGULAR && r0 > p.M - R) r0 = p.M - R;
#pragma unroll
        for (int i = 0; i < (REGULAR ? 1 : R); ++i) {
            int r = r0 + i;
            if (r >= p.M) r = p.M - 1;
            const int img = (int)p.d_HoWo.div((uint32_t)r), pix = r - img * p.HoWo;
            const int oy = (int)p.d_Wo.div((uint32_t)pix), ox = pix - oy * p.Wo;
            base[i] = (uint32_t)((long long)img * p.img_stride + (long long)oy * p.oy_stride + (long long)ox * p.ox_stride + j * p.Cc);
        }
        if (REGULAR) row_step = p.HoWo == 1 ? (uint32_t)p.img_stride : (uint32_t)p.ox_stride;
    }

    uint32_t acc[R * 8];
#pragma unroll
    for (int q = 0; q < R * 8; ++q) acc[q] = 0;

    // Activation loads are issued with inline assembly so that the compiler does not count them: it
    // would otherwise wait for ALL outstanding memory operations (table copies included) before the
    // first use.  They are issued before the step's table copy, and every step ends with a wait that
    // leaves at most that copy outstanding, so after wait_and_barrier() they have landed; the
    // registers are passed through that wait so no use can be scheduled ahead of it.
    auto load_acts = [&](uint32_t *aw, int tap, int t4) {
        const int ky = tap / p.kw, kx = tap - ky * p.kw;
        const int8_t *xrow = xt + (ky * p.ky_stride + kx * p.kx_stride) + t4;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            if (REGULAR) {
                const int8_t *srow = xrow + (size_t)i * row_step;
                asm volatile("global_load_dword %0, %1, %2" : "=v"(aw[i]) : "v"(base[0]), "s"(srow));
            } else {
                asm volatile("global_load_dword %0, %1, %2" : "=v"(aw[i]) : "v"(base[i]), "s"(xrow));
            }
        }
    };
    auto tie = [&](uint32_t *aw) {
#pragma unroll
        for (int i = 0; i < R; ++i) asm volatile("" : "+v"(aw[i]));
    };

    // prologue: tables of steps 0 and 1, activations of the first group
    table_dma(dt, tbl, table_u4, wave, lane);
    if (steps > 1) table_dma(dt + table_u4, tbl + TABLE_U4_MAX, table_u4, wave, lane);
    uint32_t aw[R], awn[R];
    load_acts(aw, 0, 0);
    wait_vm(0);
    __builtin_amdgcn_s_barrier();
    tie(aw);

    const uint32_t colbase = (uint32_t)j * 16;
    const uint32_t ubits = (uint32_t)p.bits;
    int tap = 0, t = 0;                     // position of the current step

    // Order of this wave's memory operations: per step the table copy (dma_ops operations) first,
    // then, in the first step of a group of four, the R activation loads of the NEXT group.
    const bool fetch_first = ((wave >> 2) & 1) != 0;     // waves w and w + 4 share a SIMD
    uint4 rv[R];
    int rd = 0, wr = 2;                     // buffer read in this step / buffer the table of step + 2 goes to
    bool prev_loaded = false;               // did the previous step issue activation loads?
    int ops_since_acts = 0;                 // table-copy operations issued after the latest activation loads
    for (int step = 0; step < steps; ++step) {
        // the table of step + 2 goes to the buffer that was read in step - 1
        const bool more = step + 2 < steps;
        if (more) {
            table_dma(dt + (size_t)(step + 2) * table_u4, tbl + wr * TABLE_U4_MAX, table_u4, wave, lane);
            ops_since_acts += dma_ops;
        }
        // activations of the next group of four steps are requested one group ahead
        bool loaded = false;
        if ((t & 3) == 0) {
            int ntap = tap, nt4 = t + 4;
            if (nt4 >= p.Cc) { nt4 = 0; ++ntap; }
            if (ntap < p.taps) { load_acts(awn, ntap, nt4); loaded = true; ops_since_acts = 0; }
        }
        // Half of the waves of each SIMD add up the entries they fetched in the PREVIOUS step before
        // fetching this step's, the other half fetch first and add afterwards: while one half keeps
        // the vector ALU busy the other half keeps the LDS busy, although all meet at every barrier.
        if (!fetch_first && step > 0) {
#pragma unroll
            for (int i = 0; i < R; ++i) accum8<SIGNED>(acc + i * 8, rv[i]);
        }
        const unsigned char *cur = reinterpret_cast<const unsigned char *>(tbl + rd * TABLE_U4_MAX) + colbase;
        const uint32_t sh = (uint32_t)(t & 3) * 8u;
#pragma unroll
        for (int i = 0; i < R; ++i) {
            const uint32_t a = __builtin_amdgcn_ubfe(aw[i], sh, ubits);
            rv[i] = *reinterpret_cast<const uint4 *>(cur + (a << 7));
        }
        if (fetch_first) {
#pragma unroll
            for (int i = 0; i < R; ++i) accum8<SIGNED>(acc + i * 8, rv[i]);
        }
        ++t;
        if (t == p.Cc) { t = 0; ++tap; }
        const bool group_end = (t & 3) == 0;
        // The table of step + 1 (copied during step - 1, before that step's activation loads) must have
        // landed: everything issued after it may stay in flight.  At the end of a group the next
        // activations must have landed too.
        int keep = (more ? dma_ops : 0) + ((prev_loaded || loaded) ? R : 0);
        if (group_end && ops_since_acts < keep) keep = ops_since_acts;
        wait_vm(keep);
        __builtin_amdgcn_s_barrier();
        tie(awn);
        prev_loaded = loaded;
        rd = rd == 2 ? 0 : rd + 1;
        wr = wr == 2 ? 0 : wr + 1;
        if (group_end) {
#pragma unroll
            for (int i = 0; i < R; ++i) aw[i] = awn[i];
        }
    }

    if (!fetch_first && steps > 0) {
#pragma unroll
        for (int i = 0; i < R; ++i) accum8<SIGNED>(acc + i * 8, rv[i]);
    }

    // lane j stores rows (R / 2) * (j & 1) .. + R / 2 - 1 of channels (j >> 1) and (j >> 1) + 4
    uint32_t w[R / 2][2];
    reduce_scatter<R>(acc, j, w);
#pragma unroll
    for (int i = 0; i < R / 2; ++i) {
        const int r = mt * (128 * R) + rs * R + (R / 2) * (j & 1) + i;
        if (r >= p.M) continue;
        const int img = (int)p.d_HoWo.div((uint32_t)r), pix = r - img * p.HoWo;
        const int a = (int)p.d_Wo.div((uint32_t)pix), b = pix - a * p.Wo;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int n = nt * 8 + (j >> 1) + 4 * t;
            if (n >= p.N) continue;
            int32_t *q = p.out + ((size_t)img * p.N + n) * p.out_plane + out_off + a * p.out_sy + b * p.out_sx;
            if (p.shift < 0) {
                const uint32_t f = finish_sum(p, w[i][t], n, (size_t)(q - p.out));
                if (!p.no_out) *q = (int32_t)f;
                if (p.chain.buf) p.chain.put(img, n, a, b, __uint_as_float(f));
            } else {
                *q = (int32_t)((uint32_t)*q + (w[i][t] << p.shift));
            }
        }
    }
}


// The two halves of the inner loop of the fast kernel, in assembly so that their order is exactly
// the one written (the compiler would hoist the LDS reads of the next step above the additions of
// this one and run out of registers).
//
// The compiler takes the result of an asm statement to be complete when the statement ends, but the
// LDS reads and global loads issued here land later.  Nothing it generates may touch such a register
// before the wait that covers it, or a copy / spill would move stale data.  So these registers are
// read-write operands of every statement that uses them (one live range, nothing to copy), the loop
// body contains no control flow at all (the same operations are issued in every group; past the end of
// the matrix they fetch valid but unused data), and a final wait retires everything before the compiler
// takes over again.  paper_2203_04071_amd/isa_check.py verifies the generated code.
//
// row_add: wait until at most WAITN younger LDS reads are outstanding (then v has landed), then add
// its eight 16-bit entries to eight accumulators: v_dot2 with the constant (1, 0) / (0, 1) extends one
// half of a register and adds it in a single instruction.
template <bool SIGNED, int WAITN>
__device__ __forceinline__ void row_add(uint32_t *a, u32x4_t &v) {
    if constexpr (SIGNED) {
        asm volatile("s_waitcnt lgkmcnt(%[wn])\n\t"
                     "v_dot2c_i32_i16 %0, 1, %[x]\n\tv_dot2c_i32_i16 %1, 0x10000, %[x]\n\t"
                     "v_dot2c_i32_i16 %2, 1, %[y]\n\tv_dot2c_i32_i16 %3, 0x10000, %[y]\n\t"
                     "v_dot2c_i32_i16 %4, 1, %[z]\n\tv_dot2c_i32_i16 %5, 0x10000, %[z]\n\t"
                     "v_dot2c_i32_i16 %6, 1, %[w]\n\tv_dot2c_i32_i16 %7, 0x10000, %[w]"
                     : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])
                     : [x] "v"(v.x), [y] "v"(v.y), [z] "v"(v.z), [w] "v"(v.w), [wn] "n"(WAITN));
    } else {
        const uint32_t c_lo = 0x00000001u, c_hi = 0x00010000u;
        asm volatile("s_waitcnt lgkmcnt(%[wn])\n\t"
                     "v_dot2_u32_u16 %0, %[x], %[lo], %0\n\tv_dot2_u32_u16 %1, %[x], %[hi], %1\n\t"
                     "v_dot2_u32_u16 %2, %[y], %[lo], %2\n\tv_dot2_u32_u16 %3, %[y], %[hi], %3\n\t"
                     "v_dot2_u32_u16 %4, %[z], %[lo], %4\n\tv_dot2_u32_u16 %5, %[z], %[hi], %5\n\t"
                     "v_dot2_u32_u16 %6, %[w], %[lo], %6\n\tv_dot2_u32_u16 %7, %[w], %[hi], %7"
                     : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]), "+v"(a[4]), "+v"(a[5]), "+v"(a[6]), "+v"(a[7])
                     : [x] "v"(v.x), [y] "v"(v.y), [z] "v"(v.z), [w] "v"(v.w), [wn] "n"(WAITN), [lo] "v"(c_lo), [hi] "v"(c_hi));
    }
}

// row_fetch: activation = `bits`-wide field at bit SHIFT of word; read the 16 bytes of this lane's
// column in that activation's line.  col = LDS address of the column in line 0 of table buffer 0 or 2,
// OFF = 0 or 32768 selects the buffer after it.
template <int SHIFT, int OFF>
__device__ __forceinline__ void row_fetch(u32x4_t &v, uint32_t word, uint32_t bits, uint32_t col) {
    uint32_t tmp;
    asm volatile("v_bfe_u32 %[t], %[wd], %[sh], %[bits]\n\t"
                 "v_lshl_add_u32 %[t], %[t], 7, %[col]\n\t"
                 "ds_read_b128 %[v], %[t] offset:%[off]"
                 : [v] "+v"(v), [t] "=&v"(tmp)
                 : [wd] "v"(word), [sh] "n"(SHIFT), [bits] "s"(bits), [col] "v"(col), [off] "n"(OFF));
}

// ---------------------------------------------------------------------------------------------
// Fast variant of the kernel above for the common case: the inner length per tap is a multiple of
// 32 (Cc % 4 == 0), so groups of four steps never straddle a tap.  Four steps are unrolled; with four
// table buffers every buffer index and every wait count is a compile-time constant.
//
// Software pipeline.  A lane's R rows are handled in two halves that share R/2 register quadruples.
// In step s a wave first adds the entries of rows 0..R/2-1 (fetched during step s - 1) and, as each
// quadruple becomes free, fetches into it the entries of a row of the second half from table s; then
// it adds those and refills the quadruples with the first-half rows of step s + 1 from table s + 1.
// Every LDS read thus has half a step to return, reads stay in flight across the barrier, and a wave
// arrives at the barrier as soon as its vector-ALU work is done.  Table s + 3 is copied while step s
// runs (into the buffer of table s - 1, which nobody reads any more).
//
// Invariant after the barrier that ends step s: tables s + 1 and s + 2 are complete and visible to
// all waves.  To keep it, before that barrier every wave waits for ITS part of table s + 2 (issued in
// step s - 1).  Order of a wave's memory operations, per group g of four steps (D = copy operations
// per table, A(g+1) = the R activation loads of the next group):
//     u=0: D(4g+3) A(g+1)   u=1: D(4g+4)   u=2: D(4g+5)   u=3: D(4g+6)
// Operations of one wave complete in order, so "table s + 2 has landed" means "at most as many
// operations in flight as were issued after it": D + A at the end of u = 0 and u = 1, D at the end of
// u = 2 (which also guarantees A(g+1), needed by the fetches of u = 3) and of u = 3.  The last two
// groups issue fewer operations and simply wait for everything.
// ---------------------------------------------------------------------------------------------
template <int R, bool SIGNED, bool REGULAR, bool TWO_OPS, bool XMAJOR, bool PAIRED = false>
__global__ __launch_bounds__(LINES_THREADS) void lut_lines_fast_kernel(const LinesParams p) {
    __shared__ uint4 tbl[4 * TABLE_U4_MAX];          // 128 KB
    constexpr int D = TWO_OPS ? 2 : 1;
    // s_waitcnt immediates: vmcnt(n), expcnt and lgkmcnt left at their maxima (no wait)
    constexpr int A = XMAJOR ? 2 : R;                // memory operations per group of activation loads
    constexpr int WAIT_DA = 0x0F70 | (D + A);
    constexpr int WAIT_D = 0x0F70 | D;
    constexpr int WAIT_ALL = 0x0F70;
    static_assert(D + A < 16, "vmcnt immediate");
    static_assert(!XMAJOR || (REGULAR && R == 8), "x-major activations: 8 rows per lane in two runs of 4 pixels");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = tid & 7;
    const int rs = tid >> 3;
    const int wg = (int)p.d_ntiles.div(blockIdx.x);
    const int nt = blockIdx.x - wg * p.n_tiles;
    const int pk = (int)p.d_mtiles.div((uint32_t)wg);
    const int mt = wg - pk * p.m_tiles;
    const int ks = (int)p.d_phases.div((uint32_t)pk);   // slice of the inner dimension
    const int ph = pk - ks * p.phases;
    const int8_t *const xt = p.xt + pick4(p.xt_off, ph);
    const int out_off = pick4(p.out_off, ph);
    int32_t *const outp = p.out + (size_t)ks * p.ks_out_stride;
    const int lines = 1 << p.bits;
    const int table_u4 = lines * 8;
    const int steps_all = p.taps * p.Cc;
    const int g_begin = ks * p.gps;
    const int groups = min(steps_all >> 2, g_begin + p.gps) - g_begin;      // groups of this slice (>= 1)
    const int steps = groups << 2;
    const uint32_t table_bytes = (uint32_t)table_u4 * 16u;
    const unsigned char *dt = reinterpret_cast<const unsigned char *>(p.dt + pick4(p.dt_off, ph) + (size_t)nt * steps_all * table_u4) +
                              (size_t)(g_begin << 2) * table_bytes;

    // table copy geometry: 8-bit tables take two operations of 64 lanes per wave, smaller tables one
    // operation of table_u4 / 16 lanes per wave
    // (copy_lines: all lines of a table, or the first half when every activation code is known to be >= 0)
    const int lanes_act = TWO_OPS ? 64 : ((p.copy_lines * 8) >> 4);
    const uint64_t dma_mask = ~0ull >> (64 - lanes_act);       // 1 <= lanes_act <= 64
    const uint32_t dma_voff = (uint32_t)(wave * lanes_act + lane) * 16u;
    const uint32_t lds_tbl = (uint32_t)(uintptr_t)(lds_void_ptr)tbl;
    const uint32_t lds_wave = lds_tbl + (uint32_t)(wave * lanes_act) * 16u;
    // table min(step, steps - 1) -> buffer `buf`.  Past the last table the copy is repeated into a buffer nobody reads any
    // more, so that every group issues the same operations and the wait counts below hold to the end.
    auto dma = [&](int step_, int buf) {
        const int step = step_ < steps ? step_ : steps - 1;
        const unsigned char *src = dt + (size_t)(unsigned)step * table_bytes;
        const uint32_t m0v = lds_wave + (uint32_t)buf * (TABLE_U4_MAX * 16u);
        if constexpr (TWO_OPS) {
            asm volatile("s_mov_b32 m0, %[ma]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[vo], %[sa]\n\t"
                         "s_mov_b32 m0, %[mb]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[vo], %[sb]"
                         :
                         : [vo] "v"(dma_voff), [sa] "s"(src), [sb] "s"(src + 16384), [ma] "s"(m0v), [mb] "s"(m0v + 16384u)
                         : "memory", "m0");
        } else {
            uint64_t save;
            asm volatile("s_mov_b64 %[sv], exec\n\ts_mov_b64 exec, %[mk]\n\t"
                         "s_mov_b32 m0, %[ma]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[vo], %[sa]\n\t"
                         "s_mov_b64 exec, %[sv]"
                         : [sv] "=&s"(save)
                         : [vo] "v"(dma_voff), [sa] "s"(src), [ma] "s"(m0v), [mk] "s"(dma_mask)
                         : "memory", "m0");
        }
    };

    // XMAJOR: the 8 rows of a lane are two runs of 4 consecutive output pixels (each inside one image row), one base each
    constexpr int NB = XMAJOR ? 2 : (REGULAR ? 1 : R);
    uint32_t base[NB];
    uint32_t row_step = 0;
    // position of row r: image, output row a, output column b; the run after an x-major run of 4 pixels follows
    // without further divisions (Wo and HoWo are multiples of 4 there)
    auto row_pos = [&](int r, int &img, int &a, int &b) {
        img = (int)p.d_HoWo.div((uint32_t)r);
        const int pix = r - img * p.HoWo;
        a = (int)p.d_Wo.div((uint32_t)pix);
        b = pix - a * p.Wo;
    };
    auto next_run = [&](int &img, int &a, int &b) {
        b += 4;
        if (b == p.Wo) { b = 0; ++a; }
        if (a * p.Wo == p.HoWo) { a = 0; ++img; }
    };
    // first inner index of this lane's k-sub inside a tap, as a byte offset: PAIRED channel group j % pair_cg, else
    // the j-th run of Cc channels
    const int ksub_ch = PAIRED ? 4 * (j % p.pair_cg) : j * p.Cc;
    const int ksub_off = XMAJOR ? ksub_ch * p.ch_stride : ksub_ch;
    {
        int r0 = mt * (128 * R) + rs * R;
        if (REGULAR && r0 > p.M - R) r0 = p.M - R;
        if constexpr (XMAJOR) {
            int img, a, b;
            row_pos(r0, img, a, b);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                base[i] = (uint32_t)((long long)img * p.img_stride + (long long)a * p.oy_stride + (long long)b * p.ox_stride + ksub_off);
                next_run(img, a, b);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NB; ++i) {
                int r = r0 + i;
                if (r >= p.M) r = p.M - 1;
                int img, a, b;
                row_pos(r, img, a, b);
                base[i] = (uint32_t)((long long)img * p.img_stride + (long long)a * p.oy_stride + (long long)b * p.ox_stride + ksub_off);
            }
        }
        if (REGULAR) row_step = p.HoWo == 1 ? (uint32_t)p.img_stride : (uint32_t)p.ox_stride;
    }
    // Activations of a group of four steps, one register per row (one byte per step).  XMAJOR: two 16-byte loads
    // into two register quadruples; else one 4-byte load per row.  Nothing is issued when on == 0.
    struct Acts {
        u32x4_t q[XMAJOR ? 2 : 1];
        uint32_t w[XMAJOR ? 1 : R];
        __device__ __forceinline__ uint32_t row(int i) const { return XMAJOR ? q[i / 4][i % 4] : w[i]; }
    };
    // lane_off: per-lane part of the tap offset (PAIRED; else 0)
    auto load_acts = [&](Acts &a, const int8_t *xrow, uint32_t lane_off) {
        if constexpr (XMAJOR) {     // 4 consecutive pixels x 4 channel bytes are 16 contiguous bytes
            const uint32_t b0 = base[0] + lane_off, b1 = base[NB - 1] + lane_off;
            asm volatile("global_load_dwordx4 %[a0], %[b0], %[xr]\n\tglobal_load_dwordx4 %[a1], %[b1], %[xr]"
                         : [a0] "+v"(a.q[0]), [a1] "+v"(a.q[1])
                         : [b0] "v"(b0), [b1] "v"(b1), [xr] "s"(xrow));
        } else {
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const int8_t *srow = REGULAR ? xrow + (size_t)i * row_step : xrow;
                const uint32_t b0 = base[REGULAR ? 0 : i] + lane_off;
                asm volatile("global_load_dword %[a0], %[b0], %[xr]" : [a0] "+v"(a.w[i]) : [b0] "v"(b0), [xr] "s"(srow));
            }
        }
    };
    // end of a step: wait until at most the given number of this wave's memory operations are outstanding, then meet
    // the other waves
    auto step_end = [&](auto imm) {
        asm volatile("s_waitcnt %[im]\n\ts_barrier" : : [im] "n"(decltype(imm)::value) : "memory");
    };
    // aw = awn at the end of a group, as a statement of its own: left to the compiler, the copy could be scheduled
    // ahead of the wait that covers the loads into awn (it believes awn complete since the load statement)
    auto take_next = [&](Acts &dst, const Acts &src) {
        if constexpr (XMAJOR) {
            uint32_t t[8];
            asm volatile("v_mov_b32 %0, %8\n\tv_mov_b32 %1, %9\n\tv_mov_b32 %2, %10\n\tv_mov_b32 %3, %11\n\t"
                         "v_mov_b32 %4, %12\n\tv_mov_b32 %5, %13\n\tv_mov_b32 %6, %14\n\tv_mov_b32 %7, %15"
                         : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]), "=&v"(t[7])
                         : "v"(src.q[0].x), "v"(src.q[0].y), "v"(src.q[0].z), "v"(src.q[0].w), "v"(src.q[1].x), "v"(src.q[1].y),
                           "v"(src.q[1].z), "v"(src.q[1].w));
            dst.q[0] = u32x4_t{t[0], t[1], t[2], t[3]};
            dst.q[1] = u32x4_t{t[4], t[5], t[6], t[7]};
        } else {
#pragma unroll
            for (int i = 0; i < R; ++i) asm volatile("v_mov_b32 %0, %1" : "=v"(dst.w[i]) : "v"(src.w[i]));
        }
    };

    uint32_t acc[R * 8];
#pragma unroll
    for (int q = 0; q < R * 8; ++q) acc[q] = 0;

    // position of the NEXT group's activations (starts at this slice's first group).  Unpaired: all lanes are in the
    // same tap, (kx, t4) and the offsets are uniform.  PAIRED: a lane's tap is pair_g * group + j / pair_cg, so its
    // filter position and offset live in vector registers and advance by pair_g taps per group; taps past the last
    // one (padding, all-zero tables) read offset 0.
    const int tap0 = PAIRED ? 0 : (g_begin << 2) / p.Cc;
    const int ky0 = tap0 / p.kw;
    int kx = tap0 - ky0 * p.kw, t4 = PAIRED ? 0 : (g_begin << 2) - tap0 * p.Cc;
    int t4off = XMAJOR ? t4 * p.ch_stride : t4;                 // byte offset of inner index t4 within a tap
    uint32_t rowoff = (uint32_t)(ky0 * p.ky_stride);            // ky * ky_stride
    uint32_t tapoff = rowoff + (uint32_t)(kx * p.kx_stride);    // + kx * kx_stride; both advance by additions
    int ltap = 0, lkx = 0;
    uint32_t loff = 0;
    if constexpr (PAIRED) {
        ltap = p.pair_g * g_begin + j / p.pair_cg;
        const int lky = ltap / p.kw;
        lkx = ltap - lky * p.kw;
        loff = (uint32_t)(lky * p.ky_stride + lkx * p.kx_stride);
    }
    auto lane_off = [&]() -> uint32_t { return PAIRED ? (ltap < p.taps_real ? loff : 0u) : 0u; };
    auto advance_group = [&]() {
        if constexpr (PAIRED) {
            // pair_g (2 or 4) single-tap steps, written without branches
            const uint32_t wrap = (uint32_t)(p.ky_stride - p.kw * p.kx_stride);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool on = q < p.pair_g;
                lkx += on ? 1 : 0;
                loff += on ? (uint32_t)p.kx_stride : 0u;
                const bool w = lkx == p.kw;
                loff += w ? wrap : 0u;
                lkx = w ? 0 : lkx;
            }
            ltap += p.pair_g;
            return;
        }
        t4 += 4;
        t4off += XMAJOR ? 4 * p.ch_stride : 4;
        if (t4 == p.Cc) {
            t4 = 0;
            t4off = 0;
            ++kx;
            tapoff += (uint32_t)p.kx_stride;
            if (kx == p.kw) { kx = 0; rowoff += (uint32_t)p.ky_stride; tapoff = rowoff; }
        }
    };

    Acts aw, awn;
#pragma unroll
    for (int q = 0; q < (XMAJOR ? 2 : 1); ++q) { aw.q[q] = u32x4_t{0, 0, 0, 0}; awn.q[q] = u32x4_t{0, 0, 0, 0}; }
#pragma unroll
    for (int i = 0; i < (XMAJOR ? 1 : R); ++i) { aw.w[i] = 0; awn.w[i] = 0; }
    constexpr int H = R / 2;                // rows per half
    constexpr int WN = H - 1;               // younger LDS reads that may be in flight when a row is added
    u32x4_t rv[H];
#pragma unroll
    for (int i = 0; i < H; ++i) rv[i] = u32x4_t{0, 0, 0, 0};
    const uint32_t ubits = (uint32_t)p.bits;
    // LDS address of this lane's column in table buffers 0 and 2 (buffers 1 and 3 lie 32768 bytes after them)
    const uint32_t cb0 = lds_tbl + (uint32_t)j * 16u;
    const uint32_t cb2 = cb0 + 2u * (TABLE_U4_MAX * 16u);

    // prologue: tables of steps 0..2, activations of group 0
    dma(0, 0);
    dma(1, 1);
    dma(2, 2);
    load_acts(aw, PAIRED ? xt : xt + tapoff + t4off, lane_off());
    step_end(std::integral_constant<int, WAIT_ALL>{});
    advance_group();
    // first-half entries of step 0
#pragma unroll
    for (int i = 0; i < H; ++i) row_fetch<0, 0>(rv[i], aw.row(i), ubits, cb0);

    for (int g = 0; g < groups; ++g) {
        const int s0 = g << 2;
        // u = 0: table buffers 0 (this step) and 1 (next step); activations of the next group (after the last group:
        // those of the first one again, unused)
        dma(s0 + 3, 3);
        load_acts(awn, (!PAIRED && g + 1 < groups) ? xt + tapoff + t4off : xt, g + 1 < groups ? lane_off() : 0u);
#pragma unroll
        for (int i = 0; i < H; ++i) { row_add<SIGNED, WN>(acc + i * 8, rv[i]); row_fetch<0, 0>(rv[i], aw.row(H + i), ubits, cb0); }
#pragma unroll
        for (int i = 0; i < H; ++i) { row_add<SIGNED, WN>(acc + (H + i) * 8, rv[i]); row_fetch<8, 32768>(rv[i], aw.row(i), ubits, cb0); }
        step_end(std::integral_constant<int, WAIT_DA>{});
        // u = 1: buffers 1 and 2
        dma(s0 + 4, 0);
#pragma unroll
        for (int i = 0; i < H; ++i) { row_add<SIGNED, WN>(acc + i * 8, rv[i]); row_fetch<8, 32768>(rv[i], aw.row(H + i), ubits, cb0); }
#pragma unroll
        for (int i = 0; i < H; ++i) { row_add<SIGNED, WN>(acc + (H + i) * 8, rv[i]); row_fetch<16, 0>(rv[i], aw.row(i), ubits, cb2); }
        step_end(std::integral_constant<int, WAIT_DA>{});
        // u = 2: buffers 2 and 3
        dma(s0 + 5, 1);
#pragma unroll
        for (int i = 0; i < H; ++i) { row_add<SIGNED, WN>(acc + i * 8, rv[i]); row_fetch<16, 0>(rv[i], aw.row(H + i), ubits, cb2); }
#pragma unroll
        for (int i = 0; i < H; ++i) { row_add<SIGNED, WN>(acc + (H + i) * 8, rv[i]); row_fetch<24, 32768>(rv[i], aw.row(i), ubits, cb2); }
        step_end(std::integral_constant<int, WAIT_D>{});
        // u = 3: buffers 3 and 0; the second-half fetches are the first rows of the next group's first step (awn has
        // landed: the wait that ended u = 2 covers it; after the last group they read a stale table and are discarded)
        dma(s0 + 6, 2);
#pragma unroll
        for (int i = 0; i < H; ++i) { row_add<SIGNED, WN>(acc + i * 8, rv[i]); row_fetch<24, 32768>(rv[i], aw.row(H + i), ubits, cb2); }
#pragma unroll
        for (int i = 0; i < H; ++i) { row_add<SIGNED, WN>(acc + (H + i) * 8, rv[i]); row_fetch<0, 0>(rv[i], awn.row(i), ubits, cb0); }
        step_end(std::integral_constant<int, WAIT_D>{});
        take_next(aw, awn);
        advance_group();
    }
    // retire the reads and copies issued past the end before the compiler may reuse their registers
    if constexpr (H == 4)
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" : "+v"(rv[0]), "+v"(rv[1]), "+v"(rv[2]), "+v"(rv[3]) : : "memory");
    else if constexpr (H == 2)
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" : "+v"(rv[0]), "+v"(rv[1]) : : "memory");
    else
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" : "+v"(rv[0]) : : "memory");

    // lane j stores rows (R / 2) * (j & 1) .. + R / 2 - 1 of channels (j >> 1) and (j >> 1) + 4; in the x-major form (R = 8)
    // the rows are 4 consecutive pixels, so the two lanes of a pair write 32 adjacent bytes and the 8 row slots of
    // a wave a whole 256-byte stretch of one channel in one instruction
    uint32_t w[R / 2][2];
    reduce_scatter<R>(acc, j, w);
    const int r0 = mt * (128 * R) + rs * R + (R / 2) * (j & 1);
    if constexpr (XMAJOR) {
        static_assert(!XMAJOR || R == 8, "runs of 4 pixels");
        if (r0 + 4 > p.M) return;           // M is a multiple of 8 here
        int img, a0, b0;
        row_pos(r0, img, a0, b0);
        uint32_t codes[2] = {0u, 0u};       // chained copy: this lane's four codes per channel tile half (byte i = pixel i)
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int n = nt * 8 + (j >> 1) + 4 * t;
            if (n >= p.N) continue;
            int32_t *q0 = outp + ((size_t)img * p.N + n) * p.out_plane + out_off + a0 * p.out_sy + b0 * p.out_sx;
            const int sx = p.out_sx;
            uint32_t f[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) f[i] = p.shift < 0 ? finish_sum(p, w[i][t], n, (size_t)(q0 + i * sx - outp)) : w[i][t];
            if (p.chain.buf) {
                if (nt * 8 + 4 * t + 3 < p.N) {     // the whole channel quad exists: exchanged below, stored as words
#pragma unroll
                    for (int i = 0; i < 4; ++i) codes[t] |= p.chain.code(__uint_as_float(f[i])) << (8 * i);
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) p.chain.put(img, n, a0, b0 + i, __uint_as_float(f[i]));
                }
            }
            if (p.no_out) {
                // only the chained copy is wanted
            } else if (p.shift < 0 && sx == 1 && (reinterpret_cast<uintptr_t>(q0) & 15u) == 0) {
                *reinterpret_cast<uint4 *>(q0) = make_uint4(f[0], f[1], f[2], f[3]);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (p.shift < 0) q0[i * sx] = (int32_t)f[i];
                    else q0[i * sx] = (int32_t)((uint32_t)q0[i * sx] + (f[i] << p.shift));
                }
            }
        }
        if (p.chain.buf) {      // the four lanes that hold one pixel run's four channels trade bytes: words instead of bytes
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint32_t word = chain_gather4(codes[t], lane, j & 1, j >> 1);
                if (nt * 8 + 4 * t + 3 < p.N) p.chain.put4(img, nt * 8 + 4 * t, a0, b0 + (j >> 1), word);
            }
        }
    } else {
        int img0 = 0, pix0 = 0;
        if (REGULAR) { img0 = (int)p.d_HoWo.div((uint32_t)r0); pix0 = r0 - img0 * p.HoWo; }
#pragma unroll
        for (int i = 0; i < R / 2; ++i) {
            const int r = r0 + i;
            if (r >= p.M) continue;
            int img, pix;
            if (REGULAR && p.HoWo > 1) { img = img0; pix = pix0 + i; }      // consecutive pixels of one output row
            else { img = (int)p.d_HoWo.div((uint32_t)r); pix = r - img * p.HoWo; }
            const int a = (int)p.d_Wo.div((uint32_t)pix), b = pix - a * p.Wo;
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int n = nt * 8 + (j >> 1) + 4 * t;
                if (n >= p.N) continue;
                int32_t *q = outp + ((size_t)img * p.N + n) * p.out_plane + out_off + a * p.out_sy + b * p.out_sx;
                if (p.shift < 0) {
                    const uint32_t f = finish_sum(p, w[i][t], n, (size_t)(q - outp));
                    if (!p.no_out) *q = (int32_t)f;
                    if (p.chain.buf) p.chain.put(img, n, a, b, __uint_as_float(f));
                } else {
                    *q = (int32_t)((uint32_t)*q + (w[i][t] << p.shift));
                }
            }
        }
    }
}

}  // namespace adapt
