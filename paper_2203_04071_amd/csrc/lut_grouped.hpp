// Grouped convolution with few output channels per group, direct form (Sec. III-B "Convolution Layer": groups;
// the depthwise half of the separable convolution, eq. (1)): every output element is the sum of (Cin / groups) * kh * kw
// table entries T[x][w], each looked up on its own in the table image held in LDS.
//
// The rows kernel shares one activation load among the 8 or 16 output channels a lane accumulates; a depthwise layer has
// ONE output channel per input channel, so there is nothing to share and 7/8 of that kernel's lookups would be padding.
// Here a lane owns one output element at a time (consecutive lanes = consecutive pixels of one output plane, so the
// activation loads of a wave are adjacent bytes and its weight loads are one address), walks its taps, and moves on by
// the size of the grid; the table is staged once per workgroup and serves many planes.
// Padded taps are looked up with activation 0 like everywhere else (they are entries of the expanded input matrix).
#pragma once
#include "lut_lines.hpp"
#include "lut_rows.hpp"

namespace adapt {

struct GroupedParams {
    const int8_t *x;        // [N][Cin][H][W]
    const int8_t *w;        // [Cout][cg][kh][kw]
    int32_t *out;           // [N][Cout][Ho][Wo]
    const uint16_t *img;    // table image as in RowsParams
    int img_bytes;
    int Cin, H, W, Cout, Ho, Wo, kh, kw;
    int sh, sw, ph, pw, dh, dw;
    int cg, og;             // input / output channels per group
    int hoff, mask, row_bytes;
    int shift;              // < 0: out = acc;  >= 0: out += acc << shift (second half of a split table)
    size_t total;           // N * Cout * Ho * Wo
    // tiled kernel only: a tile = (image, block of `gt` consecutive groups, chunk of `ro` output rows)
    int gt;                 // groups per tile (the last block of an image may hold fewer)
    int ro, n_chunks;       // output rows per tile, tiles per plane
    int rows_in, Wr;        // rows / width of the input region of a tile: (ro-1) sh + (kh-1) dh + 1, (Wo-1) sw + (kw-1) dw + 1
    int tile_elems;         // gt * cg * rows_in * Wr  (<= GROUPED_PF * ROWS_THREADS)
    int wl_bytes;           // LDS bytes of the gt * og * cg * kh * kw (<= ROWS_THREADS) tap words (multiple of 16)
    int ntiles;             // N * ceil(groups / gt) * n_chunks
    // whole-layer form (tiled kernel, single-pass tables): xf != nullptr reads fp32 activations and quantises them while
    // the tile is written (the quantiser of Sec. III-A with scale qscale); deq != 0 turns the sums into fp32
    // y = float(acc) * scale (or scales[co]), + bias[co], then ReLU (act 1) or tanh (act 2), stored at `out` unless that is
    // nullptr; chain: y also becomes the next convolution's quantised input copy (see ChainOut)
    const float *xf;
    float qscale, qQ;
    int deq, act;
    float scale;
    const float *scales, *bias;
    ChainOut chain;
    // divisors of the per-lane set-up of the tiled kernel (two dozen integer divisions per lane were 5 us of every launch)
    FastDiv d_plane_in, d_Wr, d_ogK, d_K, d_taps, d_kw, d_npix, d_Wo, d_nstrip, d_Wo4;
    int cpl;                // output channels per work item of the tiled kernel (a multiple of 4 when chain4)
    int chain4;             // every tile starts at a channel that is a multiple of 4 and the copy's rows are whole words
};

constexpr int GROUPED_CHUNK = 9;

template <bool SIGNED>
__global__ __launch_bounds__(ROWS_THREADS) void lut_grouped_kernel(const GroupedParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    stage_table(smem, p.img, p.img_bytes, threadIdx.x);
    __syncthreads();
    const size_t stride = (size_t)gridDim.x * ROWS_THREADS;
    const int HoWo = p.Ho * p.Wo, taps = p.kh * p.kw;
    const uint32_t zero2 = (uint32_t)p.hoff << 1;           // column of activation 0
    for (size_t o = (size_t)blockIdx.x * ROWS_THREADS + threadIdx.x; o < p.total; o += stride) {
        const size_t plane = o / HoWo;
        const int pix = (int)(o - plane * HoWo);
        const int oy = pix / p.Wo, ox = pix - oy * p.Wo;
        const int n = (int)(plane / p.Cout), co = (int)(plane - (size_t)n * p.Cout);
        const int grp = co / p.og;
        const int8_t *xg = p.x + ((size_t)n * p.Cin + (size_t)grp * p.cg) * p.H * p.W;
        const int8_t *wc = p.w + (size_t)co * p.cg * taps;
        const int iy0 = oy * p.sh - p.ph, ix0 = ox * p.sw - p.pw;
        // taps in blocks of GROUPED_CHUNK: all loads of a block are issued before its first lookup (addresses of
        // padded or surplus taps are clamped to element 0 and their values replaced, so no load is conditional)
        const int K = p.cg * taps;
        uint32_t acc = 0;
        int ci = 0, ky = 0, kx = 0;
        for (int k0 = 0; k0 < K; k0 += GROUPED_CHUNK) {
            uint32_t a2[GROUPED_CHUNK], row[GROUPED_CHUNK];
#pragma unroll
            for (int u = 0; u < GROUPED_CHUNK; ++u) {
                const bool live = k0 + u < K;
                const int iy = iy0 + ky * p.dh, ix = ix0 + kx * p.dw;
                const bool in = live && (unsigned)iy < (unsigned)p.H && (unsigned)ix < (unsigned)p.W;
                const int a = xg[in ? ((size_t)ci * p.H + iy) * p.W + ix : 0];
                const int wv = wc[live ? k0 + u : 0];
                a2[u] = in ? (uint32_t)((a + p.hoff) & p.mask) << 1 : zero2;
                row[u] = (uint32_t)((wv + p.hoff) & p.mask) * (uint32_t)p.row_bytes;
                if (++kx == p.kw) {
                    kx = 0;
                    if (++ky == p.kh) { ky = 0; ++ci; }
                }
            }
#pragma unroll
            for (int u = 0; u < GROUPED_CHUNK; ++u)
                if (k0 + u < K) acc += lds_entry<SIGNED>(smem, row[u] + a2[u]);
        }
        if (p.shift < 0) p.out[o] = (int32_t)acc;
        else p.out[o] = (int32_t)((uint32_t)p.out[o] + (acc << p.shift));
    }
}

// The same sums with the input region of a tile staged in LDS next to the table (160 KB per compute unit: 129 KB of
// table leave room for a few KB of activations): a workgroup walks tiles = (image, block of `gt` consecutive groups,
// chunk of output rows); for each it writes the zero-padded input region of the block's channels (as table column
// indices; padding = the column of activation 0) and one word per filter tap (row offset of its weight | offset of the
// tap inside the region << 18) into LDS, then every lane sums the taps of its output pixels from LDS alone.  One global
// byte load per INPUT element instead of one per tap, and the next tile's elements are in flight (held in registers)
// while this tile is summed.  Only one workgroup fits a compute unit, so nothing else hides latency: tiles are made as
// large as the region buffer allows (several planes of a depthwise layer), and everything that does not depend on the
// tile (which region elements a lane fetches, which pixels it sums, the tap offsets) is computed once per lane — the
// tile loop has no division and no per-tap index arithmetic (uniform index arithmetic lands on the one scalar unit
// that the 16 waves of the workgroup share, which is what bounded the first version of this kernel).
constexpr int GROUPED_PF = 8;               // input elements a lane prefetches per tile (region <= 8 KB)
constexpr int GROUPED_TOFF_SHIFT = 18;      // row offsets stay below 2^18 (255 rows of 516 bytes), tap offsets below 2^14

//
// KW > 0 (filter width KW, horizontal stride SW, no horizontal dilation; region rows a multiple of 4 bytes wide): a work
// item is a strip of FOUR adjacent output pixels of one channel.  The 3 SW + KW activation bytes that a filter row
// needs for the strip are read as aligned words, once, and the filter row's tap words once, so an item issues one LDS
// read per lookup plus a handful per filter row instead of three per lookup — the kernel is bound by the number of
// LDS instructions.  When the layer also writes the next layer's input copy, the four lanes of a quad hold the same
// strip of four consecutive channels and exchange their codes, so that each stores one pixel's four channels as a word.
template <bool SIGNED, int KW, int SW>
__global__ __launch_bounds__(ROWS_THREADS) void lut_grouped_tiled_kernel(const GroupedParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    uint32_t *wl = reinterpret_cast<uint32_t *>(smem + p.img_bytes);        // [gt * og][cg][taps] words of the tile's groups
    unsigned char *tl = smem + p.img_bytes + p.wl_bytes;                     // [gt * cg][rows_in][Wr] column indices
    const int groups = p.Cin / p.cg, taps = p.kh * p.kw, K = p.cg * taps;
    const int plane_in = p.rows_in * p.Wr;
    const int ngb = (groups + p.gt - 1) / p.gt;                              // blocks of groups per image

    // tile-invariant per-lane facts
    int el_r[GROUPED_PF], el_x[GROUPED_PF], el_off[GROUPED_PF];    // region element idx = tid + u * 1024: row, column, source offset
#pragma unroll
    for (int u = 0; u < GROUPED_PF; ++u) {
        const int idx = tid + u * ROWS_THREADS;
        const int c = (int)p.d_plane_in.div((uint32_t)idx), rem = idx - c * plane_in;
        const int r = (int)p.d_Wr.div((uint32_t)rem), xx = rem - r * p.Wr;
        el_r[u] = r;
        el_x[u] = xx - p.pw;
        el_off[u] = (c * p.H + r) * p.W + xx - p.pw;
    }
    uint32_t my_toff = 0;                       // tap offset of word tid (word = (group in block, oc, ci, ky, kx))
    if (tid < p.gt * p.og * K) {
        const int gi = (int)p.d_ogK.div((uint32_t)tid), k = tid - (int)p.d_K.div((uint32_t)tid) * K;
        const int ci = (int)p.d_taps.div((uint32_t)k), tp = k - ci * taps;
        const int ky = (int)p.d_kw.div((uint32_t)tp), kx = tp - ky * p.kw;
        my_toff = (uint32_t)(((gi * p.cg + ci) * p.rows_in + ky * p.dh) * p.Wr + kx * p.dw) << GROUPED_TOFF_SHIFT;
    }
    // work items of a tile: (slot of cpl consecutive output channels, output row, output column), column fastest; lane
    // tid takes items tid, tid + 1024, ...: its first item and the step, decomposed once
    const int npix = p.ro * p.Wo;
    const int it0_s = (int)p.d_npix.div((uint32_t)tid), it0_r = (int)p.d_Wo.div((uint32_t)(tid - it0_s * npix));
    const int it0_x = tid - it0_s * npix - it0_r * p.Wo;
    const int d_s = (int)p.d_npix.div(ROWS_THREADS), d_r = (int)p.d_Wo.div((uint32_t)(ROWS_THREADS - d_s * npix));
    const int d_x = ROWS_THREADS - d_s * npix - d_r * p.Wo;

    // strips (KW > 0): items (slot, row, strip of 4 columns), strip fastest; with the quad exchange the 4 lanes of a quad
    // share an item and differ in the channel (slot = 4 channels), otherwise slot = channel
    const int q4 = KW > 0 && p.chain4 ? 1 : 0, cl = q4 ? tid & 3 : 0;
    const int Wo4 = (p.Wo + 3) >> 2, nstrip = p.ro * Wo4;
    const int s_tid = q4 ? tid >> 2 : tid, s_step = q4 ? ROWS_THREADS >> 2 : ROWS_THREADS;
    const int st0_s = (int)p.d_nstrip.div((uint32_t)s_tid), st0_r = (int)p.d_Wo4.div((uint32_t)(s_tid - st0_s * nstrip));
    const int st0_x = s_tid - st0_s * nstrip - st0_r * Wo4;
    const int sd_s = (int)p.d_nstrip.div((uint32_t)s_step), sd_r = (int)p.d_Wo4.div((uint32_t)(s_step - sd_s * nstrip));
    const int sd_x = s_step - sd_s * nstrip - sd_r * Wo4;
    const bool vec_out = (p.Wo & 3) == 0 && (reinterpret_cast<uintptr_t>(p.out) & 15u) == 0;                                   // 4 outputs of a strip = one aligned 16-byte store

    // Prefetch: the byte loads are issued from inline assembly and retired by an explicit wait just before their values
    // are written to LDS, one tile later.  (Issued by the compiler they would be waited for at the first instruction
    // that touches the value, and it places the byte extension right behind the load.)  The registers are written and
    // consumed inside one loop iteration, so nothing carries them around the back edge;
    // paper_2203_04071_amd/isa_check.py verifies that the generated code does not touch them in between.
    int pre[GROUPED_PF];
    uint32_t pre_in = 0;                        // bit u: element u lies inside the image
    int wpre = 0;
    auto prefetch = [&](int n, int gb, int chunk) {
        const int gcount = min(p.gt, groups - gb * p.gt);
        const int elems = gcount * p.cg * plane_in, words = gcount * p.og * K;
        const int iy_start = chunk * p.ro * p.sh - p.ph;
        const int8_t *xg = p.x + ((size_t)n * p.Cin + (size_t)gb * p.gt * p.cg) * p.H * p.W;
        const int shift_off = iy_start * p.W;
        pre_in = 0;
#pragma unroll
        for (int u = 0; u < GROUPED_PF; ++u) {
            const bool in = tid + u * ROWS_THREADS < elems && (unsigned)(iy_start + el_r[u]) < (unsigned)p.H &&
                            (unsigned)el_x[u] < (unsigned)p.W;
            if (p.xf) {         // (uniform)
                const float *src = p.xf + ((size_t)n * p.Cin + (size_t)gb * p.gt * p.cg) * p.H * p.W + (in ? el_off[u] + shift_off : 0);
                asm volatile("global_load_dword %0, %1, off" : "=v"(pre[u]) : "v"(src) : "memory");
            } else {
                const int8_t *src = xg + (in ? el_off[u] + shift_off : 0);
                asm volatile("global_load_sbyte %0, %1, off" : "=v"(pre[u]) : "v"(src) : "memory");
            }
            pre_in |= in ? 1u << u : 0u;
        }
        const int8_t *wsrc = p.w + (tid < words ? (size_t)gb * p.gt * p.og * K + tid : 0);
        asm volatile("global_load_sbyte %0, %1, off" : "=v"(wpre) : "v"(wsrc) : "memory");
    };
    auto land = [&]() {                         // retire the prefetch, write the tile (all of the buffer: surplus = activation 0)
        static_assert(GROUPED_PF == 8, "the wait names eight registers");
        asm volatile("s_waitcnt vmcnt(0)"
                     : "+v"(pre[0]), "+v"(pre[1]), "+v"(pre[2]), "+v"(pre[3]), "+v"(pre[4]), "+v"(pre[5]), "+v"(pre[6]),
                       "+v"(pre[7]), "+v"(wpre)
                     :
                     : "memory");
#pragma unroll
        for (int u = 0; u < GROUPED_PF; ++u)
            if (tid + u * ROWS_THREADS < p.tile_elems) {
                const int a = p.xf ? quant1(__int_as_float(pre[u]), p.qscale, p.qQ) : pre[u];
                tl[tid + u * ROWS_THREADS] = (unsigned char)((pre_in >> u) & 1u ? ((a + p.hoff) & p.mask) : p.hoff);
            }
        if (tid < p.gt * p.og * K) wl[tid] = ((uint32_t)((wpre + p.hoff) & p.mask) * (uint32_t)p.row_bytes) | my_toff;
    };

    // tile -> (image, block of groups, chunk) once; afterwards the three counters advance by the decomposed grid size
    // (a scalar division costs tens of scalar instructions, and the scalar unit is shared by all waves of the workgroup)
    int tile = blockIdx.x;
    int chunk = tile % p.n_chunks, gb = (tile / p.n_chunks) % ngb, n = (tile / p.n_chunks) / ngb;
    const int g_chunk = (int)gridDim.x % p.n_chunks, g_gb = ((int)gridDim.x / p.n_chunks) % ngb,
              g_n = ((int)gridDim.x / p.n_chunks) / ngb;
    auto advance = [&](int &nn, int &gg, int &cc) {
        cc += g_chunk;
        if (cc >= p.n_chunks) { cc -= p.n_chunks; ++gg; }
        gg += g_gb;
        if (gg >= ngb) { gg -= ngb; ++nn; }
        nn += g_n;
    };
    if (tile >= p.ntiles) return;               // (never: the grid is at most ntiles)
    prefetch(n, gb, chunk);                     // in flight while the table is staged
    stage_table(smem, p.img, p.img_bytes, tid);
    land();
    __syncthreads();                            // table and first tile staged
    for (; tile < p.ntiles; tile += gridDim.x) {
        int n2 = n, gb2 = gb, chunk2 = chunk;
        advance(n2, gb2, chunk2);
        const bool more = tile + (int)gridDim.x < p.ntiles;
        if (more) prefetch(n2, gb2, chunk2);    // lands while this tile is summed

        const int row0 = chunk * p.ro;
        const int ocs = min(p.gt, groups - gb * p.gt) * p.og;               // output channels of this tile
        if constexpr (KW > 0) {
            constexpr int NW = (3 * SW + KW + 3) / 4;                       // words of activations per filter row
            constexpr uint32_t ROWM = (1u << GROUPED_TOFF_SHIFT) - 1u;
            const int nslots = q4 ? (ocs + 3) >> 2 : ocs;
            int sl = st0_s, r = st0_r, x4 = st0_x;
            while (sl < nslots) {
                if (row0 + r < p.Ho) {                                      // (the same for the lanes of a quad)
                    const int oc_own = q4 ? sl * 4 + cl : sl;
                    const int oc = min(oc_own, ocs - 1);                    // a lane beyond the last channel repeats it, stores nothing
                    const bool own = oc_own < ocs;
                    const uint32_t *wr = wl + oc * K;
                    const unsigned char *tb = tl + (r * p.sh) * p.Wr + x4 * (4 * SW);
                    uint32_t acc[4] = {0u, 0u, 0u, 0u};
                    const int frows = p.cg * p.kh;
                    for (int t = 0; t < frows; ++t) {
                        uint32_t e[KW], sg[NW];
#pragma unroll
                        for (int kx = 0; kx < KW; ++kx) e[kx] = wr[t * KW + kx];
                        const uint32_t *sp = reinterpret_cast<const uint32_t *>(tb + (e[0] >> GROUPED_TOFF_SHIFT));
#pragma unroll
                        for (int i = 0; i < NW; ++i) sg[i] = sp[i];
#pragma unroll
                        for (int kx = 0; kx < KW; ++kx)
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int idx = j * SW + kx;
                                const uint32_t a2 = ((sg[idx >> 2] >> (8 * (idx & 3))) & 0xffu) << 1;
                                acc[j] += lds_entry<SIGNED>(smem, (e[kx] & ROWM) + a2);
                            }
                    }
                    const int co = gb * p.gt * p.og + oc, oy = row0 + r, ox = x4 * 4;
                    int32_t *q = p.out + (((size_t)n * p.Cout + co) * p.Ho + oy) * p.Wo + ox;
                    if (p.deq) {
                        const float sc = p.scales ? p.scales[co] : p.scale;
                        float y[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            y[j] = (float)(int32_t)acc[j] * sc;
                            if (p.bias) y[j] = y[j] + p.bias[co];
                            if (p.act == 1) y[j] = y[j] > 0.0f ? y[j] : 0.0f;
                            else if (p.act == 2) y[j] = tanh_spec(y[j]);
                        }
                        if (p.out && own) {
                            if (vec_out) {
                                *reinterpret_cast<float4 *>(q) = make_float4(y[0], y[1], y[2], y[3]);
                            } else {
#pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    if (ox + j < p.Wo) reinterpret_cast<float *>(q)[j] = y[j];
                            }
                        }
                        if (q4) {
                            uint32_t mine = 0;                              // byte j: code of pixel ox + j in this lane's channel
#pragma unroll
                            for (int j = 0; j < 4; ++j) mine |= p.chain.code(y[j]) << (8 * j);
                            // lane cl of the quad collects pixel ox + cl: byte l = the code lane l holds for that pixel
                            const uint32_t v0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mine, 0x00, 0xf, 0xf, false);
                            const uint32_t v1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mine, 0x55, 0xf, 0xf, false);
                            const uint32_t v2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mine, 0xaa, 0xf, 0xf, false);
                            const uint32_t v3 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)mine, 0xff, 0xf, 0xf, false);
                            const int s8 = cl * 8;
                            const uint32_t word = ((v0 >> s8) & 0xffu) | (((v1 >> s8) & 0xffu) << 8) | (((v2 >> s8) & 0xffu) << 16) |
                                                  (((v3 >> s8) & 0xffu) << 24);
                            if (sl * 4 + 3 < ocs) {
                                if (ox + cl < p.Wo) p.chain.put4(n, gb * p.gt * p.og + sl * 4, oy, ox + cl, word);
                            } else if (own) {
#pragma unroll
                                for (int j = 0; j < 4; ++j)
                                    if (ox + j < p.Wo) p.chain.put(n, co, oy, ox + j, y[j]);
                            }
                        } else if (p.chain.buf) {
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                if (ox + j < p.Wo) p.chain.put(n, co, oy, ox + j, y[j]);
                        }
                    } else if (own && vec_out && p.shift < 0) {
                        *reinterpret_cast<uint4 *>(q) = make_uint4(acc[0], acc[1], acc[2], acc[3]);
                    } else if (own) {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (ox + j < p.Wo) q[j] = p.shift < 0 ? (int32_t)acc[j] : (int32_t)((uint32_t)q[j] + (acc[j] << p.shift));
                    }
                }
                x4 += sd_x;
                if (x4 >= Wo4) { x4 -= Wo4; ++r; }
                r += sd_r;
                if (r >= p.ro) { r -= p.ro; ++sl; }
                sl += sd_s;
            }
        } else {
        const int nslots = (ocs + p.cpl - 1) / p.cpl;
        int sl = it0_s, r = it0_r, ox = it0_x;
        while (sl < nslots) {
            if (row0 + r < p.Ho) {
                const int oc0 = sl * p.cpl, oc1 = min(ocs, oc0 + p.cpl);
                const unsigned char *tb = tl + (r * p.sh) * p.Wr + ox * p.sw;
                int32_t *q = p.out + (((size_t)n * p.Cout + (size_t)gb * p.gt * p.og + oc0) * p.Ho + row0 + r) * p.Wo + ox;
                uint32_t codes = 0;
                for (int oc = oc0; oc < oc1; ++oc) {
                    const uint32_t *wr = wl + oc * K;
                    uint32_t acc = 0;
                    int k = 0;
                    for (; k + GROUPED_CHUNK <= K; k += GROUPED_CHUNK) {
                        uint32_t e[GROUPED_CHUNK], a2[GROUPED_CHUNK];
#pragma unroll
                        for (int u = 0; u < GROUPED_CHUNK; ++u) e[u] = wr[k + u];
#pragma unroll
                        for (int u = 0; u < GROUPED_CHUNK; ++u) a2[u] = (uint32_t)tb[e[u] >> GROUPED_TOFF_SHIFT] << 1;
#pragma unroll
                        for (int u = 0; u < GROUPED_CHUNK; ++u)
                            acc += lds_entry<SIGNED>(smem, (e[u] & ((1u << GROUPED_TOFF_SHIFT) - 1u)) + a2[u]);
                    }
                    for (; k < K; ++k) {
                        const uint32_t e = wr[k];
                        acc += lds_entry<SIGNED>(smem, (e & ((1u << GROUPED_TOFF_SHIFT) - 1u)) + ((uint32_t)tb[e >> GROUPED_TOFF_SHIFT] << 1));
                    }
                    if (p.deq) {
                        const int co = gb * p.gt * p.og + oc;
                        float y = (float)(int32_t)acc * (p.scales ? p.scales[co] : p.scale);
                        if (p.bias) y = y + p.bias[co];
                        if (p.act == 1) y = y > 0.0f ? y : 0.0f;
                        else if (p.act == 2) y = tanh_spec(y);
                        if (p.out) *reinterpret_cast<float *>(q) = y;
                        if (p.chain.buf) {
                            if (p.chain4 && (oc | 3) < ocs) {       // four channels of this pixel make one word of the copy
                                codes |= p.chain.code(y) << ((oc & 3) * 8);
                                if ((oc & 3) == 3) {
                                    p.chain.put4(n, co - 3, row0 + r, ox, codes);
                                    codes = 0;
                                }
                            } else {
                                p.chain.put(n, co, row0 + r, ox, y);
                            }
                        }
                    } else if (p.shift < 0) {
                        *q = (int32_t)acc;
                    } else {
                        *q = (int32_t)((uint32_t)*q + (acc << p.shift));
                    }
                    q += (size_t)p.Ho * p.Wo;
                }
            }
            ox += d_x;
            if (ox >= p.Wo) { ox -= p.Wo; ++r; }
            r += d_r;
            if (r >= p.ro) { r -= p.ro; ++sl; }
            sl += d_s;
        }
        }
        __syncthreads();                        // everyone has finished reading this tile
        if (more) land();
        __syncthreads();
        n = n2; gb = gb2; chunk = chunk2;
    }
}

}  // namespace adapt
