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

template <bool SIGNED>
__global__ __launch_bounds__(ROWS_THREADS) void lut_grouped_tiled_kernel(const GroupedParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x;
    stage_table(smem, p.img, p.img_bytes, tid);
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
        const int c = idx / plane_in, rem = idx - c * plane_in;
        const int r = rem / p.Wr, xx = rem - r * p.Wr;
        el_r[u] = r;
        el_x[u] = xx - p.pw;
        el_off[u] = (c * p.H + r) * p.W + xx - p.pw;
    }
    uint32_t my_toff = 0;                       // tap offset of word tid (word = (group in block, oc, ci, ky, kx))
    if (tid < p.gt * p.og * K) {
        const int gi = tid / (p.og * K), k = tid % K, ci = k / taps, tp = k - ci * taps;
        const int ky = tp / p.kw, kx = tp - ky * p.kw;
        my_toff = (uint32_t)(((gi * p.cg + ci) * p.rows_in + ky * p.dh) * p.Wr + kx * p.dw) << GROUPED_TOFF_SHIFT;
    }
    const int pix0_r = tid / p.Wo, pix0_x = tid - pix0_r * p.Wo;            // first output pixel of this lane in a tile
    const int step_r = ROWS_THREADS / p.Wo, step_x = ROWS_THREADS - step_r * p.Wo;
    const int npix = p.ro * p.Wo;

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
            const int8_t *src = xg + (in ? el_off[u] + shift_off : 0);
            asm volatile("global_load_sbyte %0, %1, off" : "=v"(pre[u]) : "v"(src) : "memory");
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
            if (tid + u * ROWS_THREADS < p.tile_elems)
                tl[tid + u * ROWS_THREADS] = (unsigned char)((pre_in >> u) & 1u ? ((pre[u] + p.hoff) & p.mask) : p.hoff);
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
    prefetch(n, gb, chunk);
    land();
    __syncthreads();                            // table and first tile staged
    for (; tile < p.ntiles; tile += gridDim.x) {
        int n2 = n, gb2 = gb, chunk2 = chunk;
        advance(n2, gb2, chunk2);
        const bool more = tile + (int)gridDim.x < p.ntiles;
        if (more) prefetch(n2, gb2, chunk2);    // lands while this tile is summed

        const int row0 = chunk * p.ro;
        const int ocs = min(p.gt, groups - gb * p.gt) * p.og;               // output channels of this tile
        int r = pix0_r, ox = pix0_x;
        for (int pp = tid; pp < npix; pp += ROWS_THREADS) {
            if (row0 + r < p.Ho) {
                const unsigned char *tb = tl + (r * p.sh) * p.Wr + ox * p.sw;
                int32_t *q = p.out + (((size_t)n * p.Cout + (size_t)gb * p.gt * p.og) * p.Ho + row0 + r) * p.Wo + ox;
                for (int oc = 0; oc < ocs; ++oc) {
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
                    if (p.shift < 0) *q = (int32_t)acc;
                    else *q = (int32_t)((uint32_t)*q + (acc << p.shift));
                    q += (size_t)p.Ho * p.Wo;
                }
            }
            r += step_r; ox += step_x;
            if (ox >= p.Wo) { ox -= p.Wo; ++r; }
        }
        __syncthreads();                        // everyone has finished reading this tile
        if (more) land();
        __syncthreads();
        n = n2; gb = gb2; chunk = chunk2;
    }
}

}  // namespace adapt
