// Ceiling probes for the benchmark (NOT part of the product library: built into libadapt_probes.so, which only bench.py
// loads).  Each probe is a small kernel that exercises ONE resource the table-lookup kernels depend on, in the access
// pattern those kernels use, with 16 waves on every compute unit; bench.py runs them right before its timed region and
// prices the product kernel's work against what they measure:
//   0  16-bit LDS gathers, conflict-free (64 lanes -> 64 consecutive words): the "one lookup per bank-lane and clock" rate
//   1  16-bit LDS gathers inside one 8-bit table row with Gaussian activations (what the whole-table kernel does)
//   2  16-byte LDS reads, the 16 lanes of a quarter-wave on the 16 slots of a 256-byte line, random lines (quad kernel)
//   3  L2 -> LDS copies of 64 KB tables by LDS-direct loads, one table stream per XCD-resident group of workgroups
//   4  v_mfma_i32_16x16x64_i8 on independent accumulators
//   5  2, 3 and 4 together in the proportions of one quad-kernel step (4 rows per row slot), with its barrier
//   6  16-bit LDS gathers inside one 256-byte row of a 7-bit table, uniform activations (the recurrent time step)
//   7  the same with two copies of the table, the second rotated by 16 banks, even lanes on one and odd lanes on the other
//   8  8-bit LDS gathers inside one 128-byte row (a 7-bit table of one-byte entries: one word per bank)
//   9  the row held in a register across the wave and gathered with ds_bpermute_b32: per lookup one conflict-free
//      ds_read_b32 (the row) + one ds_bpermute_b32 (the gather)
// extern "C" adapt_probe_run(which, iters, &ms, &units): runs probe `which` on the current device (default stream,
// synchronous, best of three launches), returns the kernel time in ms and the units one launch processed (lookups for 0
// and 1, bytes for 2 and 3, matrix instructions for 4, steps x workgroups for 5).  Returns 0, or -1 on a HIP error.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <random>
#include <vector>

namespace {

constexpr int THREADS = 1024;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void *lds_ptr;

// 8 addresses per lane (host-made), 8 reads in flight per iteration
template <int WIDTH>
__global__ __launch_bounds__(THREADS) void lds_read_probe(const uint32_t *__restrict__ addrs, int iters, uint32_t *out) {
    __shared__ __attribute__((aligned(65536))) uint32_t smem[32768];      // 128 KB
    for (int i = threadIdx.x; i < 32768; i += THREADS) smem[i] = (uint32_t)i * 2654435761u;
    __syncthreads();
    const uint32_t base = (uint32_t)(uintptr_t)(lds_ptr)smem;
    uint32_t a[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) a[j] = base + addrs[(size_t)j * THREADS + threadIdx.x];
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
        if (WIDTH == 1) {
            uint32_t r0, r1, r2, r3, r4, r5, r6, r7;
            asm volatile("ds_read_i8 %0, %8\n ds_read_i8 %1, %9\n ds_read_i8 %2, %10\n ds_read_i8 %3, %11\n"
                         "ds_read_i8 %4, %12\n ds_read_i8 %5, %13\n ds_read_i8 %6, %14\n ds_read_i8 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)\n"
                         : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                         : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
            acc += r0 + r1 + r2 + r3 + r4 + r5 + r6 + r7;
        } else if (WIDTH == 2) {
            uint32_t r0, r1, r2, r3, r4, r5, r6, r7;
            asm volatile("ds_read_u16 %0, %8\n ds_read_u16 %1, %9\n ds_read_u16 %2, %10\n ds_read_u16 %3, %11\n"
                         "ds_read_u16 %4, %12\n ds_read_u16 %5, %13\n ds_read_u16 %6, %14\n ds_read_u16 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)\n"
                         : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                         : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
            acc += r0 + r1 + r2 + r3 + r4 + r5 + r6 + r7;
        } else {
            u32x4_t r0, r1, r2, r3, r4, r5, r6, r7;
            asm volatile("ds_read_b128 %0, %8\n ds_read_b128 %1, %9\n ds_read_b128 %2, %10\n ds_read_b128 %3, %11\n"
                         "ds_read_b128 %4, %12\n ds_read_b128 %5, %13\n ds_read_b128 %6, %14\n ds_read_b128 %7, %15\n"
                         "s_waitcnt lgkmcnt(0)\n"
                         : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                         : "v"(a[0]), "v"(a[1]), "v"(a[2]), "v"(a[3]), "v"(a[4]), "v"(a[5]), "v"(a[6]), "v"(a[7]));
            const u32x4_t s = r0 + r1 + r2 + r3 + r4 + r5 + r6 + r7;
            acc += s.x + s.y + s.z + s.w;
        }
    }
    out[(size_t)blockIdx.x * THREADS + threadIdx.x] = acc;
}

// Row in a register, gather by ds_bpermute_b32: per lookup the row of the (wave-uniform) weight is read with lane l
// taking word l (conflict-free), then every lane fetches word (activation / 2) of it from the lane that holds it.
__global__ __launch_bounds__(THREADS) void bpermute_probe(const uint32_t *__restrict__ addrs, int iters, uint32_t *out) {
    __shared__ __attribute__((aligned(65536))) uint32_t smem[32768];
    for (int i = threadIdx.x; i < 32768; i += THREADS) smem[i] = (uint32_t)i * 2654435761u;
    __syncthreads();
    const uint32_t base = (uint32_t)(uintptr_t)(lds_ptr)smem, lane = threadIdx.x & 63;
    uint32_t rowaddr[8], sel[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const uint32_t a = addrs[(size_t)j * THREADS + threadIdx.x];      // row * 256 + entry * 2
        rowaddr[j] = base + (a & ~255u) + lane * 4;
        sel[j] = ((a & 255u) >> 2) << 2;                                    // lane that holds the entry's word, times 4
    }
    uint32_t acc = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            uint32_t row, got;
            asm volatile("ds_read_b32 %0, %2\n\ts_waitcnt lgkmcnt(0)\n\tds_bpermute_b32 %1, %3, %0\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(row), "=&v"(got)
                         : "v"(rowaddr[j]), "v"(sel[j]));
            acc += got;
        }
    }
    out[(size_t)blockIdx.x * THREADS + threadIdx.x] = acc;
}

// One step of the combined probe / the copy probe.  COPY: a 64 KB table into the other buffer (4 operations per wave);
// READS: 16 reads of 16 bytes per lane; MFMA: one matrix instruction per read (or 16 without reads).
template <bool COPY, bool READS, bool MFMA>
__global__ __launch_bounds__(THREADS) void step_probe(const unsigned char *__restrict__ tables, int tables_per_stream, int steps,
                                                      const uint32_t *__restrict__ addrs, uint32_t *out) {
    __shared__ __attribute__((aligned(65536))) uint4 tbl[2 * 4096];       // two 64 KB buffers
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lds = (uint32_t)(uintptr_t)(lds_ptr)tbl;
    // the workgroups that share an XCD (every eighth) walk the same table stream, as the n-tiles of a layer do
    const unsigned char *stream = tables + (size_t)(blockIdx.x % 8) * (size_t)tables_per_stream * 65536;
    uint32_t a[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) a[j] = lds + addrs[(size_t)(j & 7) * THREADS + tid] + (uint32_t)(j >> 3) * 4096u;
    i32x4_t acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i] = i32x4_t{0, 0, 0, 0};
    const i32x4_t wt = {0x00008001, (int)0x80010000u, 0x00008001, (int)0x80010000u};
    u32x4_t rv[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) rv[i] = u32x4_t{1, 2, 3, 4};
    if (!COPY) {
        for (int i = tid; i < 2 * 4096; i += THREADS) tbl[i] = make_uint4(i, i + 1, i + 2, i + 3);
        __syncthreads();
    }
    const uint32_t voff = (uint32_t)(wave * 64 + lane) * 16u;
    for (int s = 0; s < steps; ++s) {
        const uint32_t bufofs = (uint32_t)(s & 1) * 65536u;
        if (COPY) {
            const unsigned char *src = stream + (size_t)(s % tables_per_stream) * 65536;
            const uint32_t m0v = lds + (65536u - bufofs) + (uint32_t)wave * 1024u;
#pragma unroll
            for (int o = 0; o < 4; ++o)
                asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                             :
                             : "v"(voff), "s"(src + o * 16384), "s"(m0v + (uint32_t)o * 16384u)
                             : "memory", "m0");
        }
        if (READS) {
#pragma unroll
            for (int n = 0; n < 4; ++n) asm volatile("ds_read_b128 %0, %1" : "+v"(rv[n]) : "v"(a[n] ^ bufofs));
#pragma unroll
            for (int n = 0; n < 12; ++n) {
                if (MFMA) asm volatile("s_waitcnt lgkmcnt(3)\n\tv_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+v"(acc[n & 3]) : "v"(wt), "v"(rv[n & 3]));
                else asm volatile("s_waitcnt lgkmcnt(3)\n\tv_xor_b32 %0, %0, %1" : "+v"(acc[n & 3].x) : "v"(rv[n & 3].x));
                asm volatile("ds_read_b128 %0, %1" : "+v"(rv[n & 3]) : "v"(a[n + 4] ^ bufofs));
            }
#pragma unroll
            for (int n = 12; n < 16; ++n) {
                if (MFMA) asm volatile("s_waitcnt lgkmcnt(0)\n\tv_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+v"(acc[n & 3]) : "v"(wt), "v"(rv[n & 3]));
                else asm volatile("s_waitcnt lgkmcnt(0)\n\tv_xor_b32 %0, %0, %1" : "+v"(acc[n & 3].x) : "v"(rv[n & 3].x));
            }
        } else if (MFMA) {
#pragma unroll
            for (int n = 0; n < 16; ++n) asm volatile("v_mfma_i32_16x16x64_i8 %0, %1, %2, %0" : "+v"(acc[n & 3]) : "v"(wt), "v"(rv[n & 3]));
        }
        if (COPY) asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" : : : "memory");
    }
    asm volatile("s_nop 15\n\ts_nop 15" : : : "memory");
#pragma unroll
    for (int i = 0; i < 4; ++i) asm volatile("" : "+v"(acc[i]));
    out[(size_t)blockIdx.x * THREADS + tid] = (uint32_t)(acc[0].x + acc[1].y + acc[2].z + acc[3].w) + rv[0].x;
}

struct Buffers {
    int device = -1, cus = 0;
    uint32_t *addrs = nullptr, *out = nullptr;
    unsigned char *tables = nullptr;
    static constexpr int TABLES_PER_STREAM = 36;        // the benchmark layer's 36 steps
};
Buffers g;

bool setup() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return false;
    if (g.device == dev) return true;
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) return false;
    g.cus = prop.multiProcessorCount;
    if (hipMalloc(&g.addrs, sizeof(uint32_t) * 8 * THREADS) != hipSuccess) return false;
    if (hipMalloc(&g.out, sizeof(uint32_t) * THREADS * (size_t)g.cus) != hipSuccess) return false;
    const size_t tb = (size_t)8 * Buffers::TABLES_PER_STREAM * 65536;
    if (hipMalloc(&g.tables, tb) != hipSuccess) return false;
    if (hipMemset(g.tables, 1, tb) != hipSuccess) return false;
    g.device = dev;
    return true;
}

// lane -> byte offset patterns (8 per lane)
std::vector<uint32_t> pattern(int which) {
    std::vector<uint32_t> a((size_t)8 * THREADS);
    std::mt19937 rng(12345u + (unsigned)which);
    std::normal_distribution<double> gauss(0.0, 24.4);      // quantised N(0, 1) activations under a max-abs scale of 127 / 5.2
    for (int j = 0; j < 8; ++j)
        for (int w = 0; w < THREADS / 64; ++w) {
            const uint32_t row = rng() % 256;
            for (int l = 0; l < 64; ++l) {
                uint32_t v;
                if (which == 0) v = row * 512 + (uint32_t)l * 4;                           // 64 consecutive words
                else if (which == 1) {                                                     // Gaussian column of one 512-byte row
                    int q = (int)std::lrint(gauss(rng));
                    q = q < -128 ? -128 : (q > 127 ? 127 : q);
                    v = row * 512 + (uint32_t)(q + 128) * 2;
                } else if (which == 6 || which == 9) v = (row % 128) * 256 + (rng() % 128) * 2;      // 7-bit row, uniform entry
                else if (which == 7) {                                                     // two copies, odd lanes on the rotated one
                    const uint32_t e2 = (rng() % 128) * 2;
                    v = (l & 1) ? 32768 + (row % 128) * 256 + ((e2 + 64) & 255) : (row % 128) * 256 + e2;
                } else if (which == 8) v = (row % 128) * 128 + (rng() % 128);              // one-byte entries
                else v = (rng() % 16) * 256 + (uint32_t)(l % 16) * 16;                   // slot = lane % 16 of a random line (first 4 KB; + 4096 j' in the kernel)
                a[(size_t)j * THREADS + w * 64 + l] = v;
            }
        }
    if (which >= 2 && which <= 5)     // spread the lines over the whole 64 KB buffer: line = random
        for (auto &v : a) v = (v & 0xff) | ((rng() % 240) << 8);
    return a;
}

}  // namespace

extern "C" int adapt_probe_cu_count(void) { return setup() ? g.cus : -1; }

extern "C" int adapt_probe_run(int which, int iters, float *ms_out, double *units_out) {
    if (!setup() || which < 0 || which > 9 || iters < 1 || !ms_out || !units_out) return -1;
    const std::vector<uint32_t> a = pattern(which < 2 || which > 5 ? which : 2);
    if (hipMemcpy(g.addrs, a.data(), a.size() * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess) return -1;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return -1;
    float best = 1e30f;
    const dim3 grid((unsigned)g.cus), block(THREADS);
    const int tps = Buffers::TABLES_PER_STREAM;
    for (int rep = 0; rep < 3; ++rep) {
        (void)hipEventRecord(e0, nullptr);
        switch (which) {
            case 0: case 1: case 6: case 7: lds_read_probe<2><<<grid, block>>>(g.addrs, iters, g.out); break;
            case 8: lds_read_probe<1><<<grid, block>>>(g.addrs, iters, g.out); break;
            case 9: bpermute_probe<<<grid, block>>>(g.addrs, iters, g.out); break;
            case 2: lds_read_probe<16><<<grid, block>>>(g.addrs, iters, g.out); break;
            case 3: step_probe<true, false, false><<<grid, block>>>(g.tables, tps, iters, g.addrs, g.out); break;
            case 4: step_probe<false, false, true><<<grid, block>>>(g.tables, tps, iters, g.addrs, g.out); break;
            default: step_probe<true, true, true><<<grid, block>>>(g.tables, tps, iters, g.addrs, g.out); break;
        }
        (void)hipEventRecord(e1, nullptr);
        if (hipEventSynchronize(e1) != hipSuccess || hipGetLastError() != hipSuccess) return -1;
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, e0, e1);
        if (ms < best) best = ms;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *ms_out = best;
    const double wgs = (double)g.cus;
    switch (which) {
        case 0: case 1: case 6: case 7: case 8: case 9: *units_out = wgs * THREADS * 8.0 * iters; break;     // lookups
        case 2: *units_out = wgs * THREADS * 8.0 * iters * 16.0; break;             // bytes read from LDS
        case 3: *units_out = wgs * 65536.0 * iters; break;                          // bytes copied into LDS
        case 4: *units_out = wgs * 16.0 * 16.0 * iters; break;                      // matrix instructions (16 waves x 16 per step)
        default: *units_out = wgs * iters; break;                                   // steps
    }
    return 0;
}
