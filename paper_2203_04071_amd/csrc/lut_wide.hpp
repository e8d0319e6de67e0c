// "Wide lines" kernel: the derived-table product (see lut_lines.hpp) with 256-byte table lines.
//
// Same idea and the same derived tables D_k[a][n] = T[a][W[n][k]] as the lines kernels, re-ordered so that one
// table line holds the entries of SIXTEEN inner indices (16 slots x 8 channels x int16 = 256 bytes):
//   * the LDS address of a lookup is (activation << 8) | (slot << 4) | (buffer << 16): byte-aligned fields, so ONE
//     v_perm_b32 builds it from the activation word (the 128-byte lines need a bit-field extract and a shift-add);
//   * the 16 lanes that read one line cover all 64 LDS banks (128-byte lines leave every read on half of them and
//     collide whenever two activations have the same parity);
//   * a step covers 16 inner indices, so there is one barrier per 16 instead of per 8.
// A step's table is 2^b x 256 bytes (64 KB for 8-bit operands); two buffers: while step s is read from one, the table
// of step s + 1 is copied into the other (it has a whole step to land, so every step simply ends with vmcnt(0)).
//
// Mapping: 1024 lanes = 128 row slots x 8 k-subs; lane (rs, j) owns rows rs*8 .. rs*8+7 (two runs of 4 output pixels,
// x-major activation copy) and, in every step, the two slots 2j and 2j+1.  A group = 2 steps = 32 consecutive inner
// indices (channels) of one filter tap; the lane's activation word of a group holds channels 4j .. 4j+3 of it: bytes
// 0, 1 belong to the first step (slots 2j, 2j+1), bytes 2, 3 to the second.  Row slots of odd index read their two
// slots in the opposite order, so that the 64 lanes of one read instruction spread over all 16 slots.
// The activation copy must hold table line indices (activation & (2^b - 1)), which the copy kernels write.
//
// Only the shape the big layers have is covered: 8 rows per lane from an x-major copy, single-pass (signed) tables,
// 32 | channels per tap.  Everything else stays on the lines kernels.
#pragma once
#include "lut_lines.hpp"

namespace adapt {

constexpr int WIDE_LINE_BYTES = 256;
constexpr int WIDE_BUF_BYTES = 65536;

// Derived tables in the wide order: [n_tile][wide step = 2 * group + h][line a][slot t] x 16 bytes, slot t of step h of
// a group holding inner index 32 * group + 4 * (t / 2) + 2 * h + (t % 2)  (group counts 32-index blocks over all taps:
// tap = group / (Cp / 32)).  wmode as in pack_line_tables_kernel.
// digit form (digits != 0): an entry e is stored as the two int8 digits of e - digit_c = d0 - 128 d1 (low byte d0, high
// byte d1; |e - digit_c| stays within [-16384, 16511], which the caller has checked), so that an int8 matrix
// instruction with the weights (1, -128) rebuilds it; padded channels hold the digits of 0 and the kernel adds
// digit_c times the number of real lookups at the end.
__device__ __forceinline__ uint32_t wide_entry(uint32_t v16, int digits, int digit_c) {
    if (!digits) return v16;
    const int e = (int)(int16_t)v16 - digit_c;
    int t = 127 - e;                                    // d1 = floor((127 - e) / 128), at most 127
    int d1 = t >= 0 ? t >> 7 : -((-t + 127) >> 7);
    if (d1 > 127) d1 = 127;
    const int d0 = e + 128 * d1;
    return (uint32_t)(d0 & 0xff) | ((uint32_t)(d1 & 0xff) << 8);
}

__global__ void pack_wide_tables_kernel(const uint16_t *__restrict__ lut16, const int8_t *__restrict__ w,
                                        uint4 *__restrict__ dt, int bits, int N, int Cin, int taps, int Cp, int n_tiles,
                                        int wmode, int digits, int digit_c) {
    const int lines = 1 << bits, mask = lines - 1;
    const size_t per_table = (size_t)lines * 16;
    const int gpt = Cp / 32;                        // groups per tap
    const size_t wsteps = (size_t)taps * gpt * 2;
    const size_t total = (size_t)n_tiles * wsteps * per_table;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int t = (int)(i & 15);
        const int a = (int)((i >> 4) & mask);
        const size_t ts = i / per_table;
        const int ws = (int)(ts % wsteps);
        const int nt = (int)(ts / wsteps);
        const int group = ws >> 1, h = ws & 1;
        const int tap = group / gpt;
        const int ci = (group - tap * gpt) * 32 + 4 * (t >> 1) + 2 * h + (t & 1);
        uint32_t e[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int n = nt * 8 + c;
            uint32_t v = 0;
            if (n < N && ci < Cin) {
                const size_t wi = wmode == 0 ? ((size_t)n * Cin + ci) * taps + tap : ((size_t)ci * N + n) * taps + tap;
                v = wide_entry(lut16[(size_t)a * lines + ((int)w[wi] & mask)], digits, digit_c);
            }
            e[c] = v;
        }
        dt[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
}

// Transposed convolution: the phase blocks of pack_line_tables_convt_kernel in the wide order.
__global__ void pack_wide_tables_convt_kernel(const uint16_t *__restrict__ lut16, const int8_t *__restrict__ w,
                                              uint4 *__restrict__ dt, int bits, int N, int Cin, int kh, int kw, int s, int Cp,
                                              int n_tiles, int digits, int digit_c) {
    const int lines = 1 << bits, mask = lines - 1;
    const int Ty = kh / s, Tx = kw / s, gpt = Cp / 32;
    const size_t per_table = (size_t)lines * 16;
    const size_t wsteps = (size_t)Ty * Tx * gpt * 2;
    const size_t per_phase = (size_t)n_tiles * wsteps * per_table;
    const size_t total = per_phase * s * s;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int phase = (int)(i / per_phase);
        const size_t ip = i - (size_t)phase * per_phase;
        const int ry = phase / s, rx = phase - ry * s;
        const int t = (int)(ip & 15);
        const int a = (int)((ip >> 4) & mask);
        const size_t ts = ip / per_table;
        const int ws = (int)(ts % wsteps);
        const int nt = (int)(ts / wsteps);
        const int group = ws >> 1, h = ws & 1;
        const int tap = group / gpt;
        const int ci = (group - tap * gpt) * 32 + 4 * (t >> 1) + 2 * h + (t & 1);
        const int mw = tap / Tx, nw = tap - mw * Tx;
        const int ky = ry + s * (Ty - 1 - mw), kx = rx + s * (Tx - 1 - nw);
        uint32_t e[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int n = nt * 8 + c;
            uint32_t v = 0;
            if (n < N && ci < Cin) {
                const size_t wi = (((size_t)ci * N + n) * kh + ky) * kw + kx;
                v = wide_entry(lut16[(size_t)a * lines + ((int)w[wi] & mask)], digits, digit_c);
            }
            e[c] = v;
        }
        dt[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
}

// address = permute(activation word, column word, selector); read the 16 bytes there
__device__ __forceinline__ void wide_fetch(u32x4_t &v, uint32_t word, uint32_t colw, uint32_t sel) {
    uint32_t tmp;
    asm volatile("v_perm_b32 %[t], %[wd], %[cw], %[sl]\n\t"
                 "ds_read_b128 %[v], %[t]"
                 : [v] "+v"(v), [t] "=&v"(tmp)
                 : [wd] "v"(word), [cw] "v"(colw), [sl] "v"(sel));
}

// Digit tables (MF instantiations): the eight entries a lane has read are widened and added by the matrix pipe instead
// of eight vector instructions.  v_mfma_i32_16x16x64_i8 computes D[i][j] += sum_k A[i][k] B[k][j]; lane l holds column
// j = l % 16 of B for the 16 k of block l / 16, and afterwards rows 4 (l / 16) .. + 3 of column j of D.  With B = the 16
// bytes the lane has read and an A that is zero outside the diagonal blocks (row 4 q + c only has weights in block q:
// 1 and -128 on the two digit bytes of entry c, or of entry 4 + c for the second instruction), every lane gets the
// four sums of ITS OWN entries back in its own registers.  The vector pipe keeps the address arithmetic, which runs
// in the shadow of the matrix instructions (the dot instructions of the other form share the matrix pipe).
typedef int i32x4_t __attribute__((ext_vector_type(4)));

__device__ __forceinline__ i32x4_t wide_mf_weights(int lane, int half) {
    const int i = lane & 15, q = lane >> 4;
    i32x4_t a = {0, 0, 0, 0};
    if ((i >> 2) == q) {
        const int e = (i & 3) + half * 4;
        const uint32_t wt = (e & 1) ? 0x80010000u : 0x00008001u;
        if ((e >> 1) == 0) a.x = (int)wt;
        else if ((e >> 1) == 1) a.y = (int)wt;
        else if ((e >> 1) == 2) a.z = (int)wt;
        else a.w = (int)wt;
    }
    return a;
}

template <int WAITN>
__device__ __forceinline__ void row_add_mf(i32x4_t &d0, i32x4_t &d1, u32x4_t &v, const i32x4_t &a0, const i32x4_t &a1) {
    asm volatile("s_waitcnt lgkmcnt(%[wn])\n\t"
                 "v_mfma_i32_16x16x64_i8 %[d0], %[a0], %[v], %[d0]\n\t"
                 "v_mfma_i32_16x16x64_i8 %[d1], %[a1], %[v], %[d1]"
                 : [d0] "+v"(d0), [d1] "+v"(d1)
                 : [v] "v"(v), [a0] "v"(a0), [a1] "v"(a1), [wn] "n"(WAITN));
}

// DOPS: table copy operations per wave and step = 2^b * 256 B / (16 waves * 1 KB): 4 / 2 / 1 for b = 8 / 7 / <= 6
// (smaller tables: one operation with fewer lanes).
template <int DOPS, bool EXTRA = false, bool MF = false>
__global__ __launch_bounds__(LINES_THREADS) void lut_lines_wide_kernel(const LinesParams p) {
    __shared__ __attribute__((aligned(256))) uint4 tbl[2 * (WIDE_BUF_BYTES / 16)];      // 128 KB
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int j = tid & 7;
    const int rs = tid >> 3;
    const int wg = (int)p.d_ntiles.div(blockIdx.x);
    const int nt = blockIdx.x - wg * p.n_tiles;
    const int pk = (int)p.d_mtiles.div((uint32_t)wg);
    const int mt = wg - pk * p.m_tiles;
    const int ks = (int)p.d_phases.div((uint32_t)pk);
    const int ph = pk - ks * p.phases;
    const int8_t *const xt = p.xt + pick4(p.xt_off, ph);
    const int out_off = pick4(p.out_off, ph);
    int32_t *const outp = p.out + (size_t)ks * p.ks_out_stride;
    const int lines = 1 << p.bits;
    const uint32_t table_bytes = (uint32_t)lines * WIDE_LINE_BYTES;
    const int groups_all = (p.taps * p.Cc) >> 2;            // groups of 32 inner indices
    const int g_begin = ks * p.gps;
    const int groups = min(groups_all, g_begin + p.gps) - g_begin;
    const int wsteps = groups * 2;
    const unsigned char *dt = reinterpret_cast<const unsigned char *>(p.dt) + ((size_t)pick4(p.dt_off, ph) << 4) +
                              ((size_t)nt * groups_all + g_begin) * 2 * table_bytes;
    const uint32_t lds_tbl = (uint32_t)(uintptr_t)(lds_void_ptr)tbl;
    if ((lds_tbl & 0xffffu) != 0) return;       // the address arithmetic below needs the buffers at multiples of 64 KB

    // table copy: operation o of wave w moves the 1 KB chunk (o * 16 + w); tables below 16 KB use part of the lanes
    const int lanes_act = DOPS > 1 ? 64 : min(64, (int)(table_bytes >> 8));     // table_bytes / 16 waves / 16 B
    const uint64_t dma_mask = ~0ull >> (64 - lanes_act);
    const uint32_t dma_voff = (uint32_t)(wave * lanes_act + lane) * 16u;
    auto dma = [&](int step_, int buf) {
        const int step = step_ < wsteps ? step_ : wsteps - 1;
        const unsigned char *src = dt + (size_t)(unsigned)step * table_bytes;
        const uint32_t m0v = lds_tbl + (uint32_t)buf * WIDE_BUF_BYTES + (uint32_t)(wave * lanes_act) * 16u;
        uint64_t save;
#pragma unroll
        for (int o = 0; o < DOPS; ++o) {
            asm volatile("s_mov_b64 %[sv], exec\n\ts_mov_b64 exec, %[mk]\n\t"
                         "s_mov_b32 m0, %[ma]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[vo], %[sa]\n\t"
                         "s_mov_b64 exec, %[sv]"
                         : [sv] "=&s"(save)
                         : [vo] "v"(dma_voff), [sa] "s"(src + o * 16384), [ma] "s"(m0v + (uint32_t)o * 16384u), [mk] "s"(dma_mask)
                         : "memory", "m0");
        }
    };

    // activation side: exactly the x-major addressing of lut_lines_fast_kernel, with 32 consecutive channels per group
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
    uint32_t base[2];
    {
        int r0 = mt * 1024 + rs * 8;
        if (r0 > p.M - 8) r0 = p.M - 8;
        int img, a, b;
        row_pos(r0, img, a, b);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            base[i] = (uint32_t)((long long)img * p.img_stride + (long long)a * p.oy_stride + (long long)b * p.ox_stride +
                                 4 * j * p.ch_stride);
            next_run(img, a, b);
        }
    }
    struct Acts {
        u32x4_t q[2];
        __device__ __forceinline__ uint32_t row(int i) const { return q[i / 4][i % 4]; }
    };
    auto load_acts = [&](Acts &a, const int8_t *xrow) {
        asm volatile("global_load_dwordx4 %[a0], %[b0], %[xr]\n\tglobal_load_dwordx4 %[a1], %[b1], %[xr]"
                     : [a0] "+v"(a.q[0]), [a1] "+v"(a.q[1])
                     : [b0] "v"(base[0]), [b1] "v"(base[1]), [xr] "s"(xrow));
    };
    auto step_end = [&]() { asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" : : : "memory"); };
    auto take_next = [&](Acts &dst, const Acts &src) {
        uint32_t t[8];
        asm volatile("v_mov_b32 %0, %8\n\tv_mov_b32 %1, %9\n\tv_mov_b32 %2, %10\n\tv_mov_b32 %3, %11\n\t"
                     "v_mov_b32 %4, %12\n\tv_mov_b32 %5, %13\n\tv_mov_b32 %6, %14\n\tv_mov_b32 %7, %15"
                     : "=&v"(t[0]), "=&v"(t[1]), "=&v"(t[2]), "=&v"(t[3]), "=&v"(t[4]), "=&v"(t[5]), "=&v"(t[6]), "=&v"(t[7])
                     : "v"(src.q[0].x), "v"(src.q[0].y), "v"(src.q[0].z), "v"(src.q[0].w), "v"(src.q[1].x), "v"(src.q[1].y),
                       "v"(src.q[1].z), "v"(src.q[1].w));
        dst.q[0] = u32x4_t{t[0], t[1], t[2], t[3]};
        dst.q[1] = u32x4_t{t[4], t[5], t[6], t[7]};
    };

    // position of the next group's activations: groups per tap = Cc / 4, 32 channels = 8 channel groups of the copy each
    const int gpt = p.Cc >> 2;
    const int tap0 = g_begin / gpt;
    const int ky0 = tap0 / p.kw;
    int kx = tap0 - ky0 * p.kw, gi = g_begin - tap0 * gpt;
    uint32_t choff = (uint32_t)(gi * 32 * p.ch_stride);
    uint32_t rowoff = (uint32_t)(ky0 * p.ky_stride);
    uint32_t tapoff = rowoff + (uint32_t)(kx * p.kx_stride);
    auto advance_group = [&]() {
        ++gi;
        choff += (uint32_t)(32 * p.ch_stride);
        if (gi == gpt) {
            gi = 0;
            choff = 0;
            ++kx;
            tapoff += (uint32_t)p.kx_stride;
            if (kx == p.kw) { kx = 0; rowoff += (uint32_t)p.ky_stride; tapoff = rowoff; }
        }
    };

    uint32_t acc[64];
#pragma unroll
    for (int q = 0; q < 64; ++q) acc[q] = 0;
    Acts aw, awn;
#pragma unroll
    for (int q = 0; q < 2; ++q) { aw.q[q] = u32x4_t{0, 0, 0, 0}; awn.q[q] = u32x4_t{0, 0, 0, 0}; }
    u32x4_t rv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rv[i] = u32x4_t{0, 0, 0, 0};

    // Address pieces.  Column word for read r (0, 1) in buffer u (0, 1): byte 0 = slot * 16, byte 2 = buffer (the buffers
    // sit at LDS addresses that are multiples of 64 KB).  Selector: result byte 0 = column byte 0, byte 1 = activation
    // byte 2 h + e, byte 2 = column byte 2, byte 3 = 0; in v_perm_b32 the bytes of the first source are numbered 4..7,
    // those of the second 0..3, and 0x0c gives zero.  Odd row slots take their slots in the opposite order.
    const uint32_t e0 = (uint32_t)(rs & 1);
    uint32_t colw[2][2], sel[2][2];
#pragma unroll
    for (int u = 0; u < 2; ++u)
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const uint32_t e = e0 ^ (uint32_t)r;
            colw[u][r] = (((uint32_t)(2 * j) + e) << 4) | ((lds_tbl >> 16) + (uint32_t)u) << 16;
            sel[u][r] = 0x0c020000u | ((4u + 2u * (uint32_t)u + e) << 8);
        }

    // digit tables: sums of row i in accm[2 i] (channels 0..3) and accm[2 i + 1] (channels 4..7)
    i32x4_t accm[MF ? 16 : 1];
#pragma unroll
    for (int q = 0; q < (MF ? 16 : 1); ++q) accm[q] = i32x4_t{0, 0, 0, 0};
    const i32x4_t mfa0 = wide_mf_weights(lane, 0), mfa1 = wide_mf_weights(lane, 1);
    auto add_row = [&](auto rowc, auto waitc, u32x4_t &v) {
        constexpr int row = decltype(rowc)::value, WN = decltype(waitc)::value;
        if constexpr (MF) row_add_mf<WN>(accm[2 * row], accm[2 * row + 1], v, mfa0, mfa1);
        else row_add<true, WN>(acc + row * 8, v);
    };

    // one step: 16 row-reads (read r = 0: rows 0..7, then r = 1: rows 0..7), four in flight
    auto run_step = [&](auto uc) {
        constexpr int u = decltype(uc)::value;
#pragma unroll
        for (int q = 0; q < 4; ++q) wide_fetch(rv[q], aw.row(q), colw[u][0], sel[u][0]);
        auto body = [&](auto qc) {
            constexpr int q = decltype(qc)::value;
            add_row(std::integral_constant<int, (q & 7)>{}, std::integral_constant<int, 3>{}, rv[q & 3]);
            constexpr int qn = q + 4;
            wide_fetch(rv[q & 3], aw.row(qn & 7), colw[u][qn >> 3], sel[u][qn >> 3]);
        };
        body(std::integral_constant<int, 0>{}); body(std::integral_constant<int, 1>{}); body(std::integral_constant<int, 2>{});
        body(std::integral_constant<int, 3>{}); body(std::integral_constant<int, 4>{}); body(std::integral_constant<int, 5>{});
        body(std::integral_constant<int, 6>{}); body(std::integral_constant<int, 7>{}); body(std::integral_constant<int, 8>{});
        body(std::integral_constant<int, 9>{}); body(std::integral_constant<int, 10>{}); body(std::integral_constant<int, 11>{});
        add_row(std::integral_constant<int, 4>{}, std::integral_constant<int, 3>{}, rv[0]);
        add_row(std::integral_constant<int, 5>{}, std::integral_constant<int, 2>{}, rv[1]);
        add_row(std::integral_constant<int, 6>{}, std::integral_constant<int, 1>{}, rv[2]);
        add_row(std::integral_constant<int, 7>{}, std::integral_constant<int, 0>{}, rv[3]);
    };

    // prologue: table of step 0, activations of the first group
    dma(0, 0);
    load_acts(aw, xt + tapoff + choff);
    step_end();
    advance_group();

    for (int g = 0; g < groups; ++g) {
        // first step of the group: buffer 0; the table of the second step goes to buffer 1, the next group's
        // activations are requested (after the last group: the first one's again, unused)
        dma(2 * g + 1, 1);
        load_acts(awn, g + 1 < groups ? xt + tapoff + choff : xt);
        run_step(std::integral_constant<int, 0>{});
        step_end();
        // second step: buffer 1; the table of the next group's first step goes to buffer 0
        dma(2 * g + 2, 0);
        run_step(std::integral_constant<int, 1>{});
        step_end();
        take_next(aw, awn);
        advance_group();
    }

    // Lane j ends with run (j & 1) of channels (j >> 1) and (j >> 1) + 4: the two lanes of a pair write 32 adjacent
    // bytes, and the 8 row slots of a wave a whole 256-byte stretch of one channel in one instruction.
    if constexpr (MF) {
        // the last matrix instructions have to leave the pipe before a vector instruction reads their registers
        asm volatile("s_nop 15\n\ts_nop 15" : : : "memory");
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[q * 4 + 0] = (uint32_t)accm[q].x; acc[q * 4 + 1] = (uint32_t)accm[q].y;
            acc[q * 4 + 2] = (uint32_t)accm[q].z; acc[q * 4 + 3] = (uint32_t)accm[q].w;
        }
    }
    const int r0 = mt * 1024 + rs * 8;
    if (r0 + 8 > p.M) return;               // M is a multiple of 8 here; no barrier follows
    const int hq = j & 1, cq = j >> 1;
    uint32_t w[4][2];
    reduce_scatter<8>(acc, j, w);
    if (MF && ks == 0) {                    // digit tables: the offset of the entries, once per output
#pragma unroll
        for (int i = 0; i < 4; ++i) { w[i][0] += (uint32_t)p.corr; w[i][1] += (uint32_t)p.corr; }
    }
    int img, a0, b0;
    row_pos(r0 + 4 * hq, img, a0, b0);
    // transposed convolution (EXTRA instantiation, zsum given): the phase's output pixels of this run of 4 are
    // (oy, ox + i * out_sx); the taps that lay over the zero border are taken off for the few runs that touch the border
    int oy = 0, ox = 0;
    bool near_border = false;
    const bool true_pos = EXTRA && p.cv_Wo > 0 && (p.zsum || p.chain.buf);      // (cv_Wo > 0: a transposed convolution)
    if (true_pos) {
        const int oy0 = out_off / p.cv_Wo, ox0 = out_off - oy0 * p.cv_Wo;       // uniform: once per workgroup
        oy = oy0 + a0 * (p.out_sy / p.cv_Wo);
        ox = ox0 + b0 * p.out_sx;
        if (p.zsum) near_border = oy < p.cv_Ly || oy >= p.cv_Ho - p.cv_Ly || ox < p.cv_Lx || ox + 3 * p.out_sx >= p.cv_Wo - p.cv_Lx;
    }
    uint32_t codes[2] = {0u, 0u};           // chained copy: this lane's four codes per channel tile half (byte i = pixel i)
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int n = nt * 8 + 4 * t + cq;
        if (n >= p.N) continue;
        if (EXTRA && near_border) {
#pragma unroll
            for (int i = 0; i < 4; ++i) w[i][t] -= convt_border_terms(p, n, oy, ox + i * p.out_sx);
        }
        int32_t *q0 = outp + ((size_t)img * p.N + n) * p.out_plane + out_off + a0 * p.out_sy + b0 * p.out_sx;
        const int sx = p.out_sx;
        uint32_t f[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) f[i] = p.shift < 0 ? finish_sum<EXTRA>(p, w[i][t], n, (size_t)(q0 + i * sx - outp)) : w[i][t];
        if (EXTRA && p.chain.buf) {
            if (nt * 8 + 4 * t + 3 < p.N) {         // the whole channel quad exists: exchanged below, stored as words
#pragma unroll
                for (int i = 0; i < 4; ++i) codes[t] |= p.chain.code(__uint_as_float(f[i])) << (8 * i);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (true_pos) p.chain.put(img, n, oy, ox + i * p.out_sx, __uint_as_float(f[i]));   // a phase's pixels of the output
                    else p.chain.put(img, n, a0, b0 + i, __uint_as_float(f[i]));
                }
            }
        }
        if (p.shift < 0 && sx == 1 && (reinterpret_cast<uintptr_t>(q0) & 15u) == 0) {
            *reinterpret_cast<uint4 *>(q0) = make_uint4(f[0], f[1], f[2], f[3]);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (p.shift < 0) q0[i * sx] = (int32_t)f[i];
                else q0[i * sx] = (int32_t)((uint32_t)q0[i * sx] + (f[i] << p.shift));
            }
        }
    }
    if (EXTRA && p.chain.buf) {     // the four lanes that hold one pixel run's four channels trade bytes: words instead of bytes
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint32_t word = chain_gather4(codes[t], lane, hq, cq);
            if (nt * 8 + 4 * t + 3 < p.N) {
                if (true_pos) p.chain.put4(img, nt * 8 + 4 * t, oy, ox + cq * p.out_sx, word);
                else p.chain.put4(img, nt * 8 + 4 * t, a0, b0 + cq, word);
            }
        }
    }
}

}  // namespace adapt
