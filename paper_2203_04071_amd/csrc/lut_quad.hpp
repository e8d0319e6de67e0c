// "Quad" kernel: the derived-table product (see lut_lines.hpp) in which the matrix pipe adds the table entries AND sums
// them over the four lanes that share an output row.
//
// Derived tables D_k[a][n] = T[a][W[n][k]] as in the lines kernels, in 256-byte lines: line a of a step's table holds,
// for the step's 16 inner indices ("slots", slot s = channel 16 * block + s of one filter tap) the entries of the 8
// output channels of the tile.  An entry e is stored as two int8 digits of e - c = d0 - 256 d1 (c = smallest entry +
// 32640, so that every 16-bit table fits), byte 2 ch = d0, byte 2 ch + 1 = d1 of channel ch.
//
// Mapping.  A wave = 16 row slots x 4 k-subs: lane l serves row slot l % 16 and k-sub q = l / 16.  In every step the
// four k-subs of a row slot take four slots each (one aligned group of four channels = one activation word), for each
// of the R rows of the slot: 4 R reads of 16 bytes per lane and step.  v_mfma_i32_16x16x64_i8 computes
// D[i][j] += sum_k A[i][k] B[k][j] with lane l holding column j = l % 16 of B for the 16 k of block l / 16: with B = the
// 16 bytes a lane has just read, column j collects the reads of the four k-subs of row slot j, and with
//     A[ch][.]     = (+1 on byte 2 ch, -128 on byte 2 ch + 1) of every block,        ch = 0..7
//     A[8 + ch][.] = (-128 on byte 2 ch + 1) of every block
// D[ch][j] + D[8 + ch][j] is the sum of the entries of channel ch over those four reads.  One matrix instruction thus
// widens, adds and reduces 64 x 8 entries; the vector pipe is left with one byte permute per read (the LDS address).
// Lane l ends with rows 4 (l / 16) .. + 3 of column l % 16 of D: lanes l and l ^ 32 hold the two parts of channels
// 4 (q % 2) .. + 3 and exchange them once, in the epilogue.
//
// LDS: line address = buffer << 16 | activation << 8 | slot << 4, built by one v_perm_b32 from the activation word.  The 16
// lanes of a k-sub (16 row slots) read 16 different slots in every instruction - row slot r takes channel group
// (q + r % 4) % 4 and, in read t, byte (t + r / 4) % 4 of it - so a read instruction is free of bank conflicts whatever
// the activations are.  Two 64 KB buffers: while step s is read from one, the table of step s + 1 is copied
// into the other by LDS-direct loads (no register round trip); a step ends when the wave's part of that copy has landed
// (a counted wait that leaves the newer activation loads in flight) and a barrier.
//
// What a step streams.  Steps run block by block (16 channels), the taps of a block one after the other.  Only the lines
// that can be selected are copied (LinesParams::copy_lines: all, or the first half behind a ReLU).  Every table is new
// to the L2 that serves it, so the workgroups that share a table touch it two steps ahead (one plain load per wave) and
// start their copies at different chunks.  With the phases of a transposed convolution, the workgroups of one row
// tile's phases run next to each other on one XCD, so that the L2 merges the interleaved pixels they write.
//
// Activations come from the x-major zero-padded copy (see pad_channels_last_kernel), which holds table line indices:
// the R pixels x 4 channels of a lane and step are R / 4 loads of 16 bytes.
#pragma once
#include "lut_lines.hpp"

namespace adapt {

constexpr int QUAD_LINE_BYTES = 256;
constexpr int QUAD_BUF_BYTES = 65536;
constexpr int QUAD_STEP = 16;           // inner indices per step
constexpr int QUAD_ROW_SLOTS = 256;     // per workgroup: 16 waves x 16
#ifndef ADAPT_QUAD_PF_DIST
#define ADAPT_QUAD_PF_DIST 2
#endif
constexpr int QUAD_PF_DIST = ADAPT_QUAD_PF_DIST;    // the L2 prefetch runs this many steps ahead of the table being copied

// the two int8 digits of entry v16 (16 bits of a table, signed or the unsigned low half of a wide one) minus digit_c
__device__ __forceinline__ uint32_t quad_entry(uint32_t v16, int sgn, int digit_c) {
    const int e = (sgn ? (int)(int16_t)v16 : (int)v16) - digit_c;      // in [-32640, 32895]
    const int d0 = ((e + 128) & 0xff) - 128;
    const int d1 = -((e - d0) >> 8);                                    // exact: e - d0 is a multiple of 256
    return (uint32_t)(d0 & 0xff) | ((uint32_t)(d1 & 0xff) << 8);
}

// Derived tables in the quad order: [n_tile][step = block * taps + tap][line a][slot s] x 16 bytes (block = 16 padded
// input channels).  The taps of one block are consecutive steps: a workgroup then reads the same 16 channels of its
// pixels (shifted by a pixel or a row) in consecutive steps, so the activation lines it needs are still in the
// nearest caches, and the tables can stream through L2 without pushing them out.
// wmode 0: w[n][K] / [Cout][Cin][taps]; wmode 1: [Cin][Cout][taps].  Padded channels and output channels hold the
// digits of 0 (they add nothing; the kernel adds digit_c once per REAL lookup at the end).
static __global__ void pack_quad_tables_kernel(const uint16_t *__restrict__ lut16, const int8_t *__restrict__ w, uint4 *__restrict__ dt,
                                               int bits, int N, int Cin, int taps, int Cp, int n_tiles, int wmode, int sgn,
                                               int digit_c) {
    const int lines = 1 << bits, mask = lines - 1;
    const size_t per_table = (size_t)lines * 16;
    const size_t steps = (size_t)taps * (Cp / QUAD_STEP);
    const size_t total = (size_t)n_tiles * steps * per_table;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int s = (int)(i & 15);
        const int a = (int)((i >> 4) & mask);
        const size_t ts = i / per_table;
        const int step = (int)(ts % steps);
        const int nt = (int)(ts / steps);
        const int blk = step / taps, tap = step - blk * taps;
        const int ci = blk * QUAD_STEP + s;
        uint32_t e[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int n = nt * 8 + c;
            uint32_t v = 0;
            if (n < N && ci < Cin) {
                const size_t wi = wmode == 0 ? ((size_t)n * Cin + ci) * taps + tap : ((size_t)ci * N + n) * taps + tap;
                v = quad_entry(lut16[(size_t)a * lines + ((int)w[wi] & mask)], sgn, digit_c);
            }
            e[c] = v;
        }
        dt[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
}

// Transposed convolution: the phase blocks of pack_line_tables_convt_kernel in the quad order,
// [phase = ry * s + rx][n_tile][step = block * (Ty Tx) + (m' * Tx + n')][line][slot].
static __global__ void pack_quad_tables_convt_kernel(const uint16_t *__restrict__ lut16, const int8_t *__restrict__ w,
                                                     uint4 *__restrict__ dt, int bits, int N, int Cin, int kh, int kw, int s, int Cp,
                                                     int n_tiles, int sgn, int digit_c) {
    const int lines = 1 << bits, mask = lines - 1;
    const int Ty = kh / s, Tx = kw / s, bpt = Cp / QUAD_STEP;
    const size_t per_table = (size_t)lines * 16;
    const size_t steps = (size_t)Ty * Tx * bpt;
    const size_t per_phase = (size_t)n_tiles * steps * per_table;
    const size_t total = per_phase * s * s;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const int phase = (int)(i / per_phase);
        const size_t ip = i - (size_t)phase * per_phase;
        const int ry = phase / s, rx = phase - ry * s;
        const int sl = (int)(ip & 15);
        const int a = (int)((ip >> 4) & mask);
        const size_t ts = ip / per_table;
        const int step = (int)(ts % steps);
        const int nt = (int)(ts / steps);
        const int blk = step / (Ty * Tx), tap = step - blk * (Ty * Tx);
        const int ci = blk * QUAD_STEP + sl;
        const int mw = tap / Tx, nw = tap - mw * Tx;
        const int ky = ry + s * (Ty - 1 - mw), kx = rx + s * (Tx - 1 - nw);
        uint32_t e[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const int n = nt * 8 + c;
            uint32_t v = 0;
            if (n < N && ci < Cin) {
                const size_t wi = (((size_t)ci * N + n) * kh + ky) * kw + kx;
                v = quad_entry(lut16[(size_t)a * lines + ((int)w[wi] & mask)], sgn, digit_c);
            }
            e[c] = v;
        }
        dt[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16), e[6] | (e[7] << 16));
    }
}

typedef int i32x4_t __attribute__((ext_vector_type(4)));

// A operand of the matrix instruction (see the head of this file): lane l holds row l % 16, the same for every block
__device__ __forceinline__ i32x4_t quad_mf_weights(int lane) {
    const int i = lane & 15, ch = i & 7;
    const uint32_t lo = i < 8 ? 0x00008001u : 0x00008000u, hi = i < 8 ? 0x80010000u : 0x80000000u;
    const uint32_t wt = (ch & 1) ? hi : lo;
    i32x4_t a = {0, 0, 0, 0};
    if ((ch >> 1) == 0) a.x = (int)wt;
    else if ((ch >> 1) == 1) a.y = (int)wt;
    else if ((ch >> 1) == 2) a.z = (int)wt;
    else a.w = (int)wt;
    return a;
}

// address = permute(activation word, column word, selector); read the 16 bytes there
__device__ __forceinline__ void quad_fetch(u32x4_t &v, uint32_t word, uint32_t colw, uint32_t sel) {
    uint32_t tmp;
    asm volatile("v_perm_b32 %[t], %[wd], %[cw], %[sl]\n\t"
                 "ds_read_b128 %[v], %[t]"
                 : [v] "+v"(v), [t] "=&v"(tmp)
                 : [wd] "v"(word), [cw] "v"(colw), [sl] "v"(sel));
}

template <int WAITN>
__device__ __forceinline__ void quad_add(i32x4_t &d, u32x4_t &v, const i32x4_t &a) {
    asm volatile("s_waitcnt lgkmcnt(%[wn])\n\t"
                 "v_mfma_i32_16x16x64_i8 %[d], %[a], %[v], %[d]"
                 : [d] "+v"(d)
                 : [v] "v"(v), [a] "v"(a), [wn] "n"(WAITN));
}

// DOPS: table copy operations per wave and step = copied lines * 256 B / (16 waves * 1 KB): 4 / 2 / 1 for 256 / 128 /
// <= 64 lines (fewer: one operation with fewer lanes).  R: rows (consecutive output pixels) per row slot, 8 or 4: a
// workgroup owns 256 R rows.  EXTRA: the epilogue also knows tanh, the border terms of a transposed convolution and the
// next layer's quantised input copy.
// Launch parameters as for the lines kernels, with these readings: Cc = steps per tap (padded channels / 16);
// gps = steps per slice of the inner dimension (ksplit > 1).
template <int DOPS, int R, bool EXTRA>
__global__ __launch_bounds__(LINES_THREADS) void lut_quad_kernel(const LinesParams p) {
    static_assert(R == 8 || R == 4, "rows per row slot");
    // 128 KB; the alignment makes the LDS layout put the buffers at multiples of 64 KB, which the address arithmetic
    // below relies on (the buffer number sits in bits 16 and up of a line address)
    __shared__ __attribute__((aligned(QUAD_BUF_BYTES))) uint4 tbl[2 * (QUAD_BUF_BYTES / 16)];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int q = lane >> 4;                    // k-sub
    const int rl = lane & 15;                   // row slot inside the wave
    const int rs = wave * 16 + rl;              // row slot inside the workgroup
    const int wg = (int)p.d_ntiles.div(blockIdx.x);
    const int nt = blockIdx.x - wg * p.n_tiles;
    // Consecutive workgroup numbers go to consecutive XCDs.  With 8 n-tiles (or a multiple) an n-tile stays on one XCD;
    // with 4 / 2 / 1 n-tiles every 2nd / 4th / 8th workgroup `wg` of an n-tile shares its XCD (xcd_span).  The phases of
    // a transposed convolution vary fastest AMONG THE WORKGROUPS OF ONE XCD: the stride^2 workgroups that write the
    // interleaved pixels of the same output lines then run at about the same time behind the same L2, which merges
    // their partial lines.  `rest` numbers the workgroups of one n-tile and phase (row tile and slice of the inner
    // dimension).
    int xcd_span = (p.n_tiles < 8 && 8 % p.n_tiles == 0) ? 8 / p.n_tiles : 1;
    if ((p.m_tiles * p.ksplit) % xcd_span) xcd_span = 1;
    const int wx = wg & (xcd_span - 1), wy = wg / xcd_span;
    const int wz = (int)p.d_phases.div((uint32_t)wy);
    const int ph = wy - wz * p.phases;
    const int rest = wz * xcd_span + wx;
    const int ks = (int)p.d_mtiles.div((uint32_t)rest);
    const int mt = rest - ks * p.m_tiles;
    const int8_t *const xt = p.xt + pick4(p.xt_off, ph);
    const int out_off = pick4(p.out_off, ph);
    int32_t *const outp = p.out + (size_t)ks * p.ks_out_stride;
    const int lines = 1 << p.bits;
    const uint32_t table_bytes = (uint32_t)lines * QUAD_LINE_BYTES;          // distance between the tables of two steps
    const uint32_t copy_bytes = (uint32_t)p.copy_lines * QUAD_LINE_BYTES;    // what a step brings into LDS (DOPS covers it)
    const int steps_all = p.taps * p.Cc;
    const int s_begin = ks * p.gps;
    const int nsteps = min(steps_all, s_begin + p.gps) - s_begin;
    const unsigned char *dt = reinterpret_cast<const unsigned char *>(p.dt) + ((size_t)pick4(p.dt_off, ph) << 4) +
                              ((size_t)nt * steps_all + s_begin) * table_bytes;
    const uint32_t lds_tbl = (uint32_t)(uintptr_t)(lds_void_ptr)tbl;

    // table copy: operation o of wave w moves the 1 KB chunk (o * 16 + w); tables below 16 KB use part of the lanes
    const int lanes_act = DOPS > 1 ? 64 : min(64, (int)(copy_bytes >> 8));      // copy_bytes / 16 waves / 16 B
    const uint64_t dma_mask = ~0ull >> (64 - lanes_act);
    const uint32_t dma_voff = (uint32_t)lane * 16u;
    // (8-bit tables: workgroup number `rest` (of an n-tile and phase) starts two chunks further on than its predecessor, so that the workgroups
    // that stream one table do not all ask L2 for the same lines at the same moment)
    const uint32_t dma_rot = DOPS == 4 ? (uint32_t)rest * 2u : 0u;
    auto dma = [&](int step_, int buf) {
        const int step = step_ < nsteps ? step_ : nsteps - 1;       // past the end: a valid table, never read
        const unsigned char *src = dt + (size_t)(unsigned)step * table_bytes;
        const uint32_t m0v = lds_tbl + (uint32_t)buf * QUAD_BUF_BYTES;
        uint64_t save;
#pragma unroll
        for (int o = 0; o < DOPS; ++o) {
            const uint32_t chunk = DOPS == 4 ? ((uint32_t)(o * 16 + wave) + dma_rot) & 63u : (uint32_t)(o * 16 + wave);
            const uint32_t at = DOPS > 1 ? chunk * 1024u : (uint32_t)(wave * lanes_act) * 16u;
            asm volatile("s_mov_b64 %[sv], exec\n\ts_mov_b64 exec, %[mk]\n\t"
                         "s_mov_b32 m0, %[ma]\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %[vo], %[sa]\n\t"
                         "s_mov_b64 exec, %[sv]"
                         : [sv] "=&s"(save)
                         : [vo] "v"(dma_voff), [sa] "s"(src + at), [ma] "s"(m0v + at), [mk] "s"(dma_mask)
                         : "memory", "m0");
        }
    };

    // L2 prefetch.  The workgroups with the same n-tile stream the same tables at about the same time, and every table
    // is new to the L2 they share (consecutive workgroup numbers go to consecutive XCDs, so with 8 n-tiles, or a multiple,
    // one n-tile stays on one XCD; with 4 / 2 / 1 n-tiles every 2nd / 4th / 8th of its workgroups does).  Left alone, the
    // first copy of every step would wait for device memory.  So each of up to 32 such workgroups touches its share of
    // the 128-byte lines of the table QUAD_PF_DIST steps ahead with one plain load per wave (a few active addresses,
    // result never used): the copy operations one step later then hit in L2.
    const int pf_span = (p.n_tiles < 8 && 8 % p.n_tiles == 0) ? 8 / p.n_tiles : 1;     // (as xcd_span, without its fallback)
    // (`rest` numbers the workgroups of one n-tile and phase; 32 workgroups of an XCD run at a time, the phases among them)
    const int pf_peers = max(1, min(32 / p.phases, (int)(gridDim.x / (unsigned)(p.n_tiles * p.phases)) / pf_span));
    const int pf_share = 1 << (31 - __builtin_clz((unsigned)pf_peers));         // a power of two
    const int pf_lines = (int)(copy_bytes >> 7);
    const int pf_per_wg = (pf_lines + pf_share - 1) / pf_share;
    const int pf_per_wave = (pf_per_wg + 15) >> 4;                              // <= 32 (512 lines, one workgroup)
    const uint32_t pf_voff =
        128u * (uint32_t)min(((rest / pf_span) & (pf_share - 1)) * pf_per_wg + wave * pf_per_wave + min(lane, pf_per_wave - 1), pf_lines - 1);
    uint32_t pf_sink = 0;
    // (tables of one copy operation - 16 KB or less - are not prefetched: the extra load per wave and step costs more
    // there than the copies' wait for memory, 3 % of a step)
    constexpr int NP = DOPS >= 2 ? 1 : 0;
    auto prefetch = [&](int step_) {
        if constexpr (NP == 0) return;
        const int step = step_ < nsteps ? step_ : nsteps - 1;
        asm volatile("global_load_dword %[d], %[vo], %[sa]" : [d] "+v"(pf_sink) : [vo] "v"(pf_voff), [sa] "s"(dt + (size_t)(unsigned)step * table_bytes));
    };

    // activation side: x-major addressing (as lut_lines_fast_kernel), 16 consecutive channels per step
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
    const int g = (q + (rl & 3)) & 3;           // this lane's channel group (of four) inside every step
    constexpr int NL = R == 8 ? 2 : 1;          // loads per lane and step
    uint32_t base[NL];
    int r0 = mt * (QUAD_ROW_SLOTS * R) + rs * R;
    const bool live = r0 + R <= p.M;            // (M is a multiple of R)
    if (!live) r0 = p.M - R;
    {
        int img, a, b;
        row_pos(r0, img, a, b);
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            base[i] = (uint32_t)((long long)img * p.img_stride + (long long)a * p.oy_stride + (long long)b * p.ox_stride +
                                 4 * g * p.ch_stride);
            next_run(img, a, b);
        }
    }
    typedef u32x4_t ld_t;                   // what one load returns: four pixels x four channels
    struct Acts {
        ld_t v[NL];
        __device__ __forceinline__ uint32_t row(int i) const { return v[i / 4][i % 4]; }
    };
    auto load_acts = [&](Acts &a, const int8_t *xrow) {
        if constexpr (R == 8)
            asm volatile("global_load_dwordx4 %[a0], %[b0], %[xr]\n\tglobal_load_dwordx4 %[a1], %[b1], %[xr]"
                         : [a0] "+v"(a.v[0]), [a1] "+v"(a.v[1])
                         : [b0] "v"(base[0]), [b1] "v"(base[1]), [xr] "s"(xrow));
        else
            asm volatile("global_load_dwordx4 %[a0], %[b0], %[xr]" : [a0] "+v"(a.v[0]) : [b0] "v"(base[0]), [xr] "s"(xrow));
    };
    // End of a step: this wave's part of the next table has landed (its copy operations were issued BEFORE the step's
    // activation loads, and a wave's memory operations retire in order, so all but the newest NL are done); the
    // activation loads stay in flight across the barrier and are waited for where the next step first needs them.
    // Per step a wave issues, in this order: DOPS copy operations, NL activation loads, NP prefetch loads.
    auto step_end = [&]() { asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" : : "n"(NL + NP) : "memory"); };
    // Start of a step, after its copy operations and loads have been issued: the activations requested one step ago
    // (the oldest NL of the 2 (NL + NP) + DOPS operations in flight) have arrived.
    auto acts_ready = [&]() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(DOPS + NL + 2 * NP) : "memory"); };

    // position of a step's activations: step = block * taps + tap (Cc blocks of 16 channels = 4 channel groups of the copy)
    int bi = s_begin / p.taps;
    const int tap0 = s_begin - bi * p.taps;
    const int kh = p.taps / p.kw;
    int ky = tap0 / p.kw, kx = tap0 - ky * p.kw;
    uint32_t choff = (uint32_t)(bi * QUAD_STEP * p.ch_stride);
    uint32_t rowoff = (uint32_t)(ky * p.ky_stride);
    uint32_t tapoff = rowoff + (uint32_t)(kx * p.kx_stride);
    auto advance_step = [&]() {
        ++kx;
        tapoff += (uint32_t)p.kx_stride;
        if (kx == p.kw) {
            kx = 0;
            ++ky;
            rowoff += (uint32_t)p.ky_stride;
            if (ky == kh) { ky = 0; rowoff = 0; choff += (uint32_t)(QUAD_STEP * p.ch_stride); }
            tapoff = rowoff;
        }
    };

    i32x4_t acc[R];
#pragma unroll
    for (int i = 0; i < R; ++i) acc[i] = i32x4_t{0, 0, 0, 0};
    Acts actA, actB;
#pragma unroll
    for (int i = 0; i < NL; ++i) { actA.v[i] = ld_t{}; actB.v[i] = ld_t{}; }
    u32x4_t rv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rv[i] = u32x4_t{0, 0, 0, 0};

    // Address pieces.  Column word for read t in buffer u: byte 0 = slot * 16, byte 2 = buffer.  Selector: result byte 0 =
    // column byte 0, byte 1 = activation byte e, byte 2 = column byte 2, byte 3 = 0; in v_perm_b32 the bytes of the first
    // source are numbered 4..7, those of the second 0..3, and 0x0c gives zero.
    uint32_t colw[2][4], sel[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const uint32_t e = (uint32_t)((t + (rl >> 2)) & 3);
        sel[t] = 0x0c020000u | ((4u + e) << 8);
#pragma unroll
        for (int u = 0; u < 2; ++u) colw[u][t] = ((4u * (uint32_t)g + e) << 4) | ((lds_tbl >> 16) + (uint32_t)u) << 16;
    }
    const i32x4_t mfa = quad_mf_weights(lane);

    // one step: 4 R reads (read t of rows 0..R-1, t = 0..3), four in flight
    auto run_step = [&](auto uc, const Acts &aw) {
        constexpr int u = decltype(uc)::value;
        constexpr int NR = 4 * R;
#pragma unroll
        for (int n = 0; n < 4; ++n) quad_fetch(rv[n], aw.row(n % R), colw[u][n / R], sel[n / R]);
#pragma unroll
        for (int n = 0; n < NR - 4; ++n) {
            quad_add<3>(acc[n % R], rv[n & 3], mfa);
            quad_fetch(rv[n & 3], aw.row((n + 4) % R), colw[u][(n + 4) / R], sel[(n + 4) / R]);
        }
        quad_add<3>(acc[(NR - 4) % R], rv[0], mfa);
        quad_add<2>(acc[(NR - 3) % R], rv[1], mfa);
        quad_add<1>(acc[(NR - 2) % R], rv[2], mfa);
        quad_add<0>(acc[(NR - 1) % R], rv[3], mfa);
    };

    // prologue: table of step 0, activations of step 0
#pragma unroll
    for (int d = 1; d <= QUAD_PF_DIST; ++d) prefetch(d);
    dma(0, 0);
    load_acts(actA, xt + tapoff + choff);
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" : : : "memory");
    advance_step();

    int s = 0;
    for (; s + 1 < nsteps; s += 2) {
        // even step: buffer 0; the table of the next step goes to buffer 1 and its activations are requested
        dma(s + 1, 1);
        load_acts(actB, xt + tapoff + choff);
        prefetch(s + 1 + QUAD_PF_DIST);
        advance_step();
        acts_ready();
        run_step(std::integral_constant<int, 0>{}, actA);
        step_end();
        // odd step: buffer 1; the next step's table goes to buffer 0 (after the last step: the last one again, unused,
        // and the first activations again)
        dma(s + 2, 0);
        load_acts(actA, s + 2 < nsteps ? xt + tapoff + choff : xt);
        prefetch(s + 2 + QUAD_PF_DIST);
        advance_step();
        acts_ready();
        run_step(std::integral_constant<int, 1>{}, actB);
        step_end();
    }
    asm volatile("s_waitcnt vmcnt(0)" : : : "memory");                      // retire what is still in flight
    asm volatile("" : : "v"(pf_sink));
    if (s < nsteps) run_step(std::integral_constant<int, 0>{}, actA);      // odd number of steps: the last one

    // the last matrix instructions have to leave the pipe before a vector instruction reads their registers
    // (every accumulator passes through an asm statement behind the waiting one, so that no read of it can be scheduled
    // ahead of the wait)
    asm volatile("s_nop 15\n\ts_nop 15" : : : "memory");
#pragma unroll
    for (int i = 0; i < R; ++i) asm volatile("" : "+v"(acc[i]));
    // Lanes l and l ^ 32 hold the two parts (rows ch and 8 + ch of D) of the sums of channels 4 (q % 2) .. + 3 of the row
    // slot's R pixels.  Lane q < 2 finishes the first two of these channels, lane q >= 2 the other two, each for all R
    // pixels: every lane hands its partner the parts the partner will finish and adds what it is handed.  A lane then
    // stores runs of four consecutive pixels (16 bytes) and the 16 lanes of a k-sub a whole 256-byte stretch of one
    // channel in one instruction.
    constexpr int NRUN = R / 4;             // runs of four pixels
    const int hi = q >> 1;
    const int cb = nt * 8 + 4 * (q & 1);    // first channel of the quad that the two lanes share
    uint32_t w[R][2];
#pragma unroll
    for (int i = 0; i < R; ++i) {
        const int part[4] = {acc[i].x, acc[i].y, acc[i].z, acc[i].w};
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
            const int keep = hi ? part[2 + cc] : part[cc], give = hi ? part[cc] : part[2 + cc];
            w[i][cc] = (uint32_t)keep + (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, give);
            if (ks == 0) w[i][cc] += (uint32_t)p.corr;      // the offset of the digit form, once per output
        }
    }
    if (!live) return;                      // no barrier follows
    const bool true_pos = EXTRA && p.cv_Wo > 0 && (p.zsum || p.chain.buf);      // (cv_Wo > 0: a transposed convolution)
    const int sx = p.out_sx;
    const bool quad_ok = cb + 3 < p.N;      // the whole channel quad exists: a chained copy takes it as one word per pixel
#pragma unroll
    for (int run = 0; run < NRUN; ++run) {
        int img, a0, b0;
        row_pos(r0 + 4 * run, img, a0, b0); // (a run lies in one image row: Wo is a multiple of 4)
        // transposed convolution (EXTRA instantiation, zsum given): the phase's output pixels are (oy, ox + i * out_sx);
        // the taps that lay over the zero border are taken off for the few runs that touch the border
        int oy = 0, ox = 0;
        bool near_border = false;
        if (true_pos) {
            const int oy0 = out_off / p.cv_Wo, ox0 = out_off - oy0 * p.cv_Wo;   // uniform: once per workgroup
            oy = oy0 + a0 * (p.out_sy / p.cv_Wo);
            ox = ox0 + b0 * p.out_sx;
            if (p.zsum) near_border = oy < p.cv_Ly || oy >= p.cv_Ho - p.cv_Ly || ox < p.cv_Lx || ox + 3 * p.out_sx >= p.cv_Wo - p.cv_Lx;
        }
        uint32_t pk[4] = {0u, 0u, 0u, 0u};  // chained copy: this lane's two codes per pixel (byte cc = channel 2 hi + cc)
#pragma unroll
        for (int cc = 0; cc < 2; ++cc) {
            const int n = cb + 2 * hi + cc;
            if (n >= p.N) continue;
            uint32_t v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = w[4 * run + i][cc];
            if (EXTRA && near_border) {     // (out_sx is the stride there)
                uint32_t extra[4];
                convt_border_terms4(p, n, oy, ox, extra);
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] -= extra[i];
            }
            int32_t *q0 = outp + ((size_t)img * p.N + n) * p.out_plane + out_off + a0 * p.out_sy + b0 * p.out_sx;
            uint32_t f[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) f[i] = finish_sum<EXTRA>(p, v[i], n, (size_t)(q0 + i * sx - outp));
            if (EXTRA && p.chain.buf) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if (quad_ok) pk[i] |= p.chain.code(__uint_as_float(f[i])) << (8 * cc);
                    else if (true_pos) p.chain.put(img, n, oy, ox + i * p.out_sx, __uint_as_float(f[i]));
                    else p.chain.put(img, n, a0, b0 + i, __uint_as_float(f[i]));
                }
            }
            if (EXTRA && p.no_out) {
                // only the chained copy is wanted
            } else if (sx == 1 && (reinterpret_cast<uintptr_t>(q0) & 15u) == 0) {
                *reinterpret_cast<uint4 *>(q0) = make_uint4(f[0], f[1], f[2], f[3]);
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i) q0[i * sx] = (int32_t)f[i];
            }
        }
        if (EXTRA && p.chain.buf) {
            // The two lanes hold the two halves of every pixel's channel quad.  Each hands the other the pixels it will
            // not write (lane hi = 0 writes pixels 0 and 1, lane hi = 1 pixels 2 and 3) and stores whole words.  Both
            // lanes of a pair are live together, so the exchange is uniform.
            const uint32_t give = hi ? (pk[0] | (pk[1] << 16)) : (pk[2] | (pk[3] << 16));
            const uint32_t got = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, (int)give);
            if (quad_ok) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const uint32_t theirs = (got >> (16 * i)) & 0xffffu, mine = pk[2 * hi + i];
                    const uint32_t word = hi ? (theirs | (mine << 16)) : (mine | (theirs << 16));
                    const int px = 2 * hi + i;
                    if (true_pos) p.chain.put4(img, cb, oy, ox + px * p.out_sx, word);
                    else p.chain.put4(img, cb, a0, b0 + px, word);
                }
            }
        }
    }
}

}  // namespace adapt
