// Memory-system probe for the box the library runs on: what a plain streaming
// kernel with the library's tile structure (128-bit accesses, one contiguous
// 1 KiB run per wave access, all loads of a tile issued up front) achieves for
// R read streams and W write streams, with plain or non-temporal accesses.
// It gives the practical ceiling the update kernels are compared against:
// the DC-ASGD push is a 4-read/3-write stream, the pull a copy, the worker
// kernel 3 reads and 1 write.
//
// usage: membw_probe [floats per stream, default 25557032] [shapes | stagger | sustain | issue]
// Allocates (4 + 4) buffers of that many floats; prints GB/s per pattern.
// With "shapes" it prints instead, for the 4-read/3-write pattern with
// non-temporal accesses, what other ways of laying the same work over waves
// and time achieve: longer contiguous runs per wave, lanes that own
// consecutive groups, persistent blocks that have the next tile's loads in
// flight while the current tile is stored, the library's shape with the number
// of resident blocks per compute unit capped by a claim of LDS that the kernel
// never touches (a cap of 8 claims nothing: the hardware's own limit of
// resident waves applies), and launches whose waves issue
// their loads and their stores in alternating windows of the chip-wide
// 100 MHz clock (every wait is on that free-running counter, never on another
// wave, and gives up after a fixed number of polls).
// With "stagger" it shifts the seven streams of that pattern against each other
// by multiples of a step, to see whether their relative placement matters;
// with "sustain" it repeats that launch for about two seconds and prints the rate
// over time; with "issue" it measures no memory at all but the rate at which
// the vector ALUs take instructions of a few kinds (the other roof of the
// kernels that do much arithmetic per byte).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

typedef float f32x4 __attribute__((ext_vector_type(4)));

#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            std::exit(1);                                                             \
        }                                                                             \
    } while (0)

template <bool NT> __device__ __forceinline__ f32x4 ld(const f32x4* p) {
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT> __device__ __forceinline__ void st(f32x4* p, f32x4 v) {
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

struct Streams {
    const f32x4* r[4];
    f32x4* w[4];
};

template <int R, int W, int ITEMS, bool LNT, bool SNT>
__global__ void __launch_bounds__(512) stream_kernel(Streams a, size_t n4, float k) {
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        const size_t first = t * tile_quads + threadIdx.x;
        f32x4 v[ITEMS][R > 0 ? R : 1];
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const size_t q = first + (size_t)j * blockDim.x;
#pragma unroll
            for (int s = 0; s < R; ++s) v[j][s] = q < n4 ? ld<LNT>(a.r[s] + q) : f32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const size_t q = first + (size_t)j * blockDim.x;
            f32x4 acc = f32x4{k, k, k, k};
#pragma unroll
            for (int s = 0; s < R; ++s) acc = acc * k + v[j][s];
            if (W == 0) {                      // keep the loads alive without writing
                if (acc.x == 123.456f && q < n4) a.w[0][q] = acc;
            }
#pragma unroll
            for (int s = 0; s < W; ++s)
                if (q < n4) st<SNT>(a.w[s] + q, acc);
        }
    }
}

template <int R, int W, int ITEMS, bool LNT, bool SNT>
static float median_ms(Streams a, size_t n4, int threads, int reps) {
    const size_t tile_quads = (size_t)threads * ITEMS;
    const unsigned grid = (unsigned)((n4 + tile_quads - 1) / tile_quads);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int i = 0; i < 3; ++i)
        hipLaunchKernelGGL((stream_kernel<R, W, ITEMS, LNT, SNT>), dim3(grid), dim3(threads), 0, 0, a, n4, 0.5f);
    std::vector<float> ts;
    for (int i = 0; i < reps; ++i) {
        CHECK(hipEventRecord(e0));
        hipLaunchKernelGGL((stream_kernel<R, W, ITEMS, LNT, SNT>), dim3(grid), dim3(threads), 0, 0, a, n4, 0.5f);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        ts.push_back(ms);
    }
    CHECK(hipGetLastError());
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    std::sort(ts.begin(), ts.end());
    return ts[ts.size() / 2];
}

// best of three launch shapes for one access policy
template <int R, int W, bool LNT, bool SNT>
static double best_gbs(Streams a, size_t n4) {
    const double bytes = (double)(R + W) * (double)n4 * 16.0;
    float t = median_ms<R, W, 1, LNT, SNT>(a, n4, 256, 15);
    t = std::min(t, median_ms<R, W, 2, LNT, SNT>(a, n4, 256, 15));
    t = std::min(t, median_ms<R, W, 2, LNT, SNT>(a, n4, 512, 15));
    return bytes / t / 1e6;
}

template <int R, int W> static void pattern(const char* name, Streams a, size_t n4) {
    std::printf("%-22s plain %5.0f | loads nt %5.0f | stores nt %5.0f | both nt %5.0f   GB/s\n", name,
                best_gbs<R, W, false, false>(a, n4), best_gbs<R, W, true, false>(a, n4),
                best_gbs<R, W, false, true>(a, n4), best_gbs<R, W, true, true>(a, n4));
    std::fflush(stdout);
}

// ---- other shapes of the 4-read/3-write stream ---------------------------------
// LAYOUT 0: lane l of a tile touches groups l, l + blockDim, ... (the library's);
//        1: wave v of the block owns ITEMS consecutive runs of 64 groups (ITEMS KiB
//           contiguous per wave and stream);
//        2: lane l owns ITEMS consecutive groups (a wave access strides by ITEMS).
template <int ITEMS, int LAYOUT>
__device__ __forceinline__ size_t quad_of(size_t tile, int j) {
    const size_t base = tile * ((size_t)blockDim.x * ITEMS);
    if constexpr (LAYOUT == 0) return base + (size_t)j * blockDim.x + threadIdx.x;
    else if constexpr (LAYOUT == 1)
        return base + ((size_t)(threadIdx.x >> 6) * ITEMS + j) * 64 + (threadIdx.x & 63);
    else return base + (size_t)threadIdx.x * ITEMS + j;
}

template <int ITEMS, int LAYOUT>
__device__ __forceinline__ void load_tile(const Streams& a, size_t tile, size_t n4, f32x4 (&v)[ITEMS][4]) {
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const size_t q = quad_of<ITEMS, LAYOUT>(tile, j);
#pragma unroll
        for (int s = 0; s < 4; ++s) v[j][s] = q < n4 ? ld<true>(a.r[s] + q) : f32x4{0, 0, 0, 0};
    }
}

template <int ITEMS, int LAYOUT>
__device__ __forceinline__ void store_tile(const Streams& a, size_t tile, size_t n4, float k,
                                           const f32x4 (&v)[ITEMS][4]) {
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const size_t q = quad_of<ITEMS, LAYOUT>(tile, j);
        f32x4 acc = f32x4{k, k, k, k};
#pragma unroll
        for (int s = 0; s < 4; ++s) acc = acc * k + v[j][s];
#pragma unroll
        for (int s = 0; s < 3; ++s)
            if (q < n4) st<true>(a.w[s] + q, acc);
    }
}

// one block per tile, or (capped grid) blocks that walk tiles
template <int ITEMS, int LAYOUT>
__global__ void __launch_bounds__(512) shape_kernel(Streams a, size_t n4, float k) {
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        f32x4 v[ITEMS][4];
        load_tile<ITEMS, LAYOUT>(a, t, n4, v);
        store_tile<ITEMS, LAYOUT>(a, t, n4, k, v);
    }
}

// persistent blocks, the loads of the next tile issued before the stores of this one
template <int ITEMS, int LAYOUT>
__global__ void __launch_bounds__(512) ahead_kernel(Streams a, size_t n4, float k) {
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    size_t t = blockIdx.x;
    if (t >= ntiles) return;
    f32x4 cur[ITEMS][4], nxt[ITEMS][4];
    load_tile<ITEMS, LAYOUT>(a, t, n4, cur);
    for (;;) {
        const size_t tn = t + gridDim.x;
        const bool more = tn < ntiles;
        if (more) load_tile<ITEMS, LAYOUT>(a, tn, n4, nxt);
        store_tile<ITEMS, LAYOUT>(a, t, n4, k, cur);
        if (!more) break;
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
#pragma unroll
            for (int s = 0; s < 4; ++s) cur[j][s] = nxt[j][s];
        t = tn;
    }
}

// Wait until the chip-wide constant-rate counter (100 MHz) is inside the window
// [lo, hi) of its period (a power of two, given as a mask), polling at most
// `polls` times: the counter runs by itself, nothing another wave does is
// waited for, and the loop ends after `polls` rounds whatever it reads.
__device__ __forceinline__ void wait_window(uint32_t mask, uint32_t lo, uint32_t hi, int polls) {
    for (int i = 0; i < polls; ++i) {
        const uint32_t ph = (uint32_t)__builtin_amdgcn_s_memrealtime() & mask;
        if (ph >= lo && ph < hi) return;
        __builtin_amdgcn_s_sleep(4);
    }
}

// loads are issued in the first `split` ticks of every period, stores in the rest
template <int ITEMS>
__global__ void __launch_bounds__(512) windowed_kernel(Streams a, size_t n4, float k, uint32_t mask,
                                                       uint32_t split, int polls) {
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    for (size_t t = blockIdx.x; t < ntiles; t += gridDim.x) {
        f32x4 v[ITEMS][4];
        wait_window(mask, 0u, split, polls);
        load_tile<ITEMS, 0>(a, t, n4, v);
        // the stores below depend on the loads, so the wave first waits for its data
        f32x4 keep = v[0][0];
#pragma unroll
        for (int j = 0; j < ITEMS; ++j)
#pragma unroll
            for (int s = 0; s < 4; ++s) keep = keep + v[j][s];
        if (keep.x == 123.456f) k += 1.0f;       // uses every loaded value before the wait
        wait_window(mask, split, mask + 1u, polls);
        store_tile<ITEMS, 0>(a, t, n4, k, v);
    }
}

// R read streams and 7 - R write streams over eight buffers (reads take the first R,
// writes the last 7 - R, so no buffer is both): how the rate depends on the share of
// writes when the number of streams stays the same.
struct Eight { f32x4* p[8]; };

template <int R>
__global__ void __launch_bounds__(256) share_kernel(Eight a, size_t n4, float k) {
    constexpr int W = 7 - R;
    const size_t q0 = (size_t)blockIdx.x * (blockDim.x * 2) + threadIdx.x;
    f32x4 v[2][R > 0 ? R : 1];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const size_t q = q0 + (size_t)j * blockDim.x;
#pragma unroll
        for (int s = 0; s < R; ++s) v[j][s] = q < n4 ? ld<true>(a.p[s] + q) : f32x4{0, 0, 0, 0};
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const size_t q = q0 + (size_t)j * blockDim.x;
        f32x4 acc = f32x4{k, k, k, k};
#pragma unroll
        for (int s = 0; s < R; ++s) acc = acc * k + v[j][s];
        if (W == 0) {
            if (acc.x == 123.456f && q < n4) a.p[7][q] = acc;
        }
#pragma unroll
        for (int s = 0; s < W; ++s)
            if (q < n4) st<true>(a.p[8 - W + s] + q, acc);
    }
}

// The push's bytes over fewer streams: two of the four read streams and two of the
// three write streams are one stream each of twice the width, interleaved in runs of
// 1 KiB (what w and MeanSquare would be if they shared one array), so that a wave
// reads 2 KiB + 1 KiB + 1 KiB and writes 2 KiB + 1 KiB, all fully coalesced.
template <bool MERGED>
__global__ void __launch_bounds__(256) merged_kernel(const f32x4* a2, const f32x4* r1, const f32x4* r2,
                                                     const f32x4* r3, f32x4* w2, f32x4* w1, f32x4* w0,
                                                     size_t n4, float k) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const size_t q = (size_t)blockIdx.x * (blockDim.x * 2) + (size_t)j * blockDim.x + threadIdx.x;
        if (q >= n4) continue;
        const size_t run = q >> 6, lane = q & 63;
        f32x4 x0, x1;
        if (MERGED) {
            x0 = ld<true>(a2 + (2 * run) * 64 + lane);
            x1 = ld<true>(a2 + (2 * run + 1) * 64 + lane);
        } else {
            x0 = ld<true>(a2 + q);
            x1 = ld<true>(r3 + q);
        }
        const f32x4 x2 = ld<true>(r1 + q), x3 = ld<true>(r2 + q);
        const f32x4 acc = ((x0 * k + x1) * k + x2) * k + x3;
        if (MERGED) {
            st<true>(w2 + (2 * run) * 64 + lane, acc);
            st<true>(w2 + (2 * run + 1) * 64 + lane, acc);
        } else {
            st<true>(w2 + q, acc);
            st<true>(w0 + q, acc);
        }
        st<true>(w1 + q, acc);
    }
}

template <class Launch> static float median_of(Launch&& launch, int reps) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    for (int i = 0; i < 3; ++i) launch();
    std::vector<float> ts;
    for (int i = 0; i < reps; ++i) {
        CHECK(hipEventRecord(e0));
        launch();
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        ts.push_back(ms);
    }
    CHECK(hipGetLastError());
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    std::sort(ts.begin(), ts.end());
    return ts[ts.size() / 2];
}

template <int ITEMS, int LAYOUT>
static void shape_row(const char* name, Streams a, size_t n4, int threads, int cap_per_cu, int cus) {
    const double bytes = 7.0 * (double)n4 * 16.0;
    const size_t tile_quads = (size_t)threads * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    unsigned grid = (unsigned)ntiles;
    if (cap_per_cu > 0 && (size_t)cap_per_cu * cus < ntiles) grid = (unsigned)(cap_per_cu * cus);
    const float t = median_of([&] {
        hipLaunchKernelGGL((shape_kernel<ITEMS, LAYOUT>), dim3(grid), dim3(threads), 0, 0, a, n4, 0.5f);
    }, 11);
    std::printf("%-44s threads %3d items %d grid %7u  %6.1f us  %5.0f GB/s\n", name, threads, ITEMS, grid,
                t * 1e3, bytes / t / 1e6);
    std::fflush(stdout);
}

template <int ITEMS, int LAYOUT>
static void ahead_row(const char* name, Streams a, size_t n4, int threads, int per_cu, int cus) {
    const double bytes = 7.0 * (double)n4 * 16.0;
    const unsigned grid = (unsigned)(per_cu * cus);
    const float t = median_of([&] {
        hipLaunchKernelGGL((ahead_kernel<ITEMS, LAYOUT>), dim3(grid), dim3(threads), 0, 0, a, n4, 0.5f);
    }, 11);
    std::printf("%-44s threads %3d items %d grid %7u  %6.1f us  %5.0f GB/s\n", name, threads, ITEMS, grid,
                t * 1e3, bytes / t / 1e6);
    std::fflush(stdout);
}

template <int ITEMS>
static void windowed_row(Streams a, size_t n4, int threads, uint32_t period, uint32_t split) {
    const double bytes = 7.0 * (double)n4 * 16.0;
    const size_t tile_quads = (size_t)threads * ITEMS;
    const unsigned grid = (unsigned)((n4 + tile_quads - 1) / tile_quads);
    // 4 x 64 cycles per poll: 2000 polls outlast four of the longest periods used here
    const float t = median_of([&] {
        hipLaunchKernelGGL((windowed_kernel<ITEMS>), dim3(grid), dim3(threads), 0, 0, a, n4, 0.5f,
                           period - 1u, split, 2000);
    }, 11);
    std::printf("loads/stores in clock windows: period %5.2f us, loads in the first %5.2f us; threads %3d items %d"
                "  %6.1f us  %5.0f GB/s\n", period * 0.01, split * 0.01, threads, ITEMS, t * 1e3,
                bytes / t / 1e6);
    std::fflush(stdout);
}

template <int R> static void share_row(Eight e, size_t n4) {
    const double bytes = 7.0 * (double)n4 * 16.0;
    const unsigned grid = (unsigned)((n4 + 511) / 512);
    // settle first: a mix inherits the state the previous one left for tens of launches
    for (int i = 0; i < 60; ++i)
        hipLaunchKernelGGL((share_kernel<R>), dim3(grid), dim3(256), 0, 0, e, n4, 0.5f);
    const float t = median_of([&] {
        hipLaunchKernelGGL((share_kernel<R>), dim3(grid), dim3(256), 0, 0, e, n4, 0.5f);
    }, 41);
    std::printf("%d read + %d write streams (%2.0f %% of the bytes written)   %6.1f us  %5.0f GB/s\n", R, 7 - R,
                100.0 * (7 - R) / 7.0, t * 1e3, bytes / t / 1e6);
    std::fflush(stdout);
}

template <int ITEMS> static void occupancy_rows(Streams a, size_t n4) {
    CHECK(hipFuncSetAttribute(reinterpret_cast<const void*>(&shape_kernel<ITEMS, 0>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, 163840));
    const double bytes = 7.0 * (double)n4 * 16.0;
    for (int threads : {64, 128, 256, 512})
        for (unsigned per_cu : {8u, 4u, 2u, 1u}) {
            const unsigned lds = per_cu >= 8 ? 0u : (163840u / per_cu) & ~1023u;
            const size_t tile = (size_t)threads * ITEMS;
            const unsigned grid = (unsigned)((n4 + tile - 1) / tile);
            for (int i = 0; i < 20; ++i)
                hipLaunchKernelGGL((shape_kernel<ITEMS, 0>), dim3(grid), dim3(threads), lds, 0, a, n4, 0.5f);
            const float t = median_of([&] {
                hipLaunchKernelGGL((shape_kernel<ITEMS, 0>), dim3(grid), dim3(threads), lds, 0, a, n4, 0.5f);
            }, 21);
            std::printf("library shape, %3d threads x %d groups, at most %u blocks per CU (%6u bytes of LDS claimed)"
                        "  %6.1f us  %5.0f GB/s\n", threads, ITEMS, per_cu, lds, t * 1e3, bytes / t / 1e6);
            std::fflush(stdout);
        }
}

static void shapes(Streams a, size_t n4) {
    int dev = 0, cus = 0;
    CHECK(hipGetDevice(&dev));
    CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    std::printf("4 reads + 3 writes, all non-temporal, %d compute units; median of 11 launches\n", cus);
    shape_row<2, 0>("library shape (1 KiB per wave access)", a, n4, 256, 0, cus);
    shape_row<4, 0>("library shape", a, n4, 256, 0, cus);
    shape_row<2, 1>("wave owns 2 KiB per stream", a, n4, 256, 0, cus);
    shape_row<4, 1>("wave owns 4 KiB per stream", a, n4, 256, 0, cus);
    shape_row<8, 1>("wave owns 8 KiB per stream", a, n4, 256, 0, cus);
    shape_row<4, 1>("wave owns 4 KiB per stream", a, n4, 64, 0, cus);
    shape_row<8, 1>("wave owns 8 KiB per stream", a, n4, 64, 0, cus);
    shape_row<2, 2>("lane owns 2 consecutive groups", a, n4, 256, 0, cus);
    shape_row<4, 2>("lane owns 4 consecutive groups", a, n4, 256, 0, cus);
    shape_row<8, 2>("lane owns 8 consecutive groups", a, n4, 256, 0, cus);
    shape_row<2, 0>("library shape, blocks walk tiles, 8 per CU", a, n4, 256, 8, cus);
    shape_row<4, 1>("wave owns 4 KiB, blocks walk tiles, 8 per CU", a, n4, 256, 8, cus);
    ahead_row<2, 0>("next tile's loads before this tile's stores, 4 per CU", a, n4, 256, 4, cus);
    ahead_row<2, 0>("next tile's loads before this tile's stores, 8 per CU", a, n4, 256, 8, cus);
    ahead_row<1, 0>("next tile's loads before this tile's stores, 8 per CU", a, n4, 256, 8, cus);
    ahead_row<4, 1>("the same, wave owns 4 KiB, 4 per CU", a, n4, 256, 4, cus);
    ahead_row<2, 0>("next tile's loads before this tile's stores, 16 per CU", a, n4, 128, 16, cus);
    {
        // n4 is rounded down to whole runs of 64 groups for this comparison
        const size_t m4 = n4 & ~(size_t)63;
        f32x4 *wide_r = nullptr, *wide_w = nullptr;
        CHECK(hipMalloc((void**)&wide_r, 2 * m4 * 16));
        CHECK(hipMalloc((void**)&wide_w, 2 * m4 * 16));
        CHECK(hipMemset(wide_r, 0, 2 * m4 * 16));
        CHECK(hipMemset(wide_w, 0, 2 * m4 * 16));
        const double bytes = 7.0 * (double)m4 * 16.0;
        const unsigned grid = (unsigned)((m4 + 511) / 512);
        for (int merged = 0; merged < 2; ++merged) {
            for (int i = 0; i < 40; ++i)
                hipLaunchKernelGGL((merged_kernel<false>), dim3(grid), dim3(256), 0, 0, a.r[0], a.r[1], a.r[2],
                                   a.r[3], a.w[0], a.w[1], a.w[2], m4, 0.5f);
            const float t = median_of([&] {
                if (merged)
                    hipLaunchKernelGGL((merged_kernel<true>), dim3(grid), dim3(256), 0, 0,
                                       (const f32x4*)wide_r, a.r[1], a.r[2], a.r[3], wide_w, a.w[1], a.w[2], m4,
                                       0.5f);
                else
                    hipLaunchKernelGGL((merged_kernel<false>), dim3(grid), dim3(256), 0, 0, a.r[0], a.r[1],
                                       a.r[2], a.r[3], a.w[0], a.w[1], a.w[2], m4, 0.5f);
            }, 41);
            std::printf("%-60s  %6.1f us  %5.0f GB/s\n",
                        merged ? "the same bytes as 3 read + 2 write streams (two pairs share an array, 1 KiB runs)"
                               : "4 read + 3 write streams, one group per lane and pass", t * 1e3,
                        bytes / t / 1e6);
            std::fflush(stdout);
        }
        CHECK(hipFree(wide_r));
        CHECK(hipFree(wide_w));
    }
    // fewer resident blocks per compute unit (dynamic LDS the kernel never touches caps them)
    occupancy_rows<2>(a, n4);
    occupancy_rows<4>(a, n4);
    occupancy_rows<8>(a, n4);
    Eight e;
    for (int i = 0; i < 4; ++i) { e.p[i] = const_cast<f32x4*>(a.r[i]); e.p[4 + i] = a.w[i]; }
    std::printf("seven streams, 256 threads x 2 groups, all non-temporal, by share of writes:\n");
    share_row<7>(e, n4); share_row<6>(e, n4); share_row<5>(e, n4); share_row<4>(e, n4);
    share_row<3>(e, n4); share_row<2>(e, n4); share_row<1>(e, n4); share_row<0>(e, n4);
    for (uint32_t period : {256u, 512u, 1024u, 2048u, 4096u})
        for (uint32_t num : {4u, 5u}) {          // loads get 4/8 or 5/8 of the period
            windowed_row<2>(a, n4, 256, period, period * num / 8);
            windowed_row<1>(a, n4, 256, period, period * num / 8);
        }
}

// The 4-read/3-write library shape with stream s moved up by s * step bytes: do the
// seven accesses a lane issues at one offset meet in the same channel or bank?
static void stagger(size_t n, size_t n4) {
    const size_t slack = (size_t)8 << 20;                 // room for the largest shift of the last stream
    char* raw[7];
    for (int i = 0; i < 7; ++i) {
        CHECK(hipMalloc((void**)&raw[i], n4 * 16 + slack));
        CHECK(hipMemset(raw[i], 0, n4 * 16 + slack));
    }
    CHECK(hipDeviceSynchronize());
    std::printf("4 reads + 3 writes, library shape (256 threads x 2 groups), streams of %zu floats;\n"
                "stream s starts s * step bytes into its own allocation; median of 11 launches\n", n);
    const size_t steps[] = {0, 256, 1024, 4096, 4096 + 256, 16384, 65536, 65536 + 4096, 262144, 1 << 20,
                            (1 << 20) + 4096 + 256, 0};
    for (size_t step : steps) {
        Streams a;
        for (int i = 0; i < 4; ++i) a.r[i] = reinterpret_cast<const f32x4*>(raw[i] + (size_t)i * step);
        for (int i = 0; i < 3; ++i) a.w[i] = reinterpret_cast<f32x4*>(raw[4 + i] + (size_t)(4 + i) * step);
        a.w[3] = a.w[2];
        const double bytes = 7.0 * (double)n4 * 16.0;
        const unsigned grid = (unsigned)((n4 + 511) / 512);
        const float t = median_of([&] {
            hipLaunchKernelGGL((shape_kernel<2, 0>), dim3(grid), dim3(256), 0, 0, a, n4, 0.5f);
        }, 11);
        std::printf("step %8zu bytes   %6.1f us  %5.0f GB/s   (first allocation at %p, spacing of allocations %zd)\n",
                    step, t * 1e3, bytes / t / 1e6, (void*)raw[0], (ptrdiff_t)(raw[1] - raw[0]));
        std::fflush(stdout);
    }
    for (int i = 0; i < 7; ++i) CHECK(hipFree(raw[i]));
}

// The same launch over and over for about two seconds, timed in chunks: does the
// rate settle, drift or step while the chip stays busy?
static void sustain(Streams a, size_t n4) {
    const double bytes = 7.0 * (double)n4 * 16.0;
    const unsigned grid = (unsigned)((n4 + 511) / 512);
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    const int chunk = n4 > 20000000 ? 40 : 200;
    std::printf("4 reads + 3 writes, library shape, back to back; GB/s per chunk of %d launches:\n", chunk);
    double elapsed = 0.0;
    for (int c = 0; c < 60 && elapsed < 2500.0; ++c) {
        CHECK(hipEventRecord(e0));
        for (int i = 0; i < chunk; ++i)
            hipLaunchKernelGGL((shape_kernel<2, 0>), dim3(grid), dim3(256), 0, 0, a, n4, 0.5f);
        CHECK(hipEventRecord(e1));
        CHECK(hipEventSynchronize(e1));
        float ms;
        CHECK(hipEventElapsedTime(&ms, e0, e1));
        elapsed += ms;
        std::printf("%5.0f", bytes * chunk / ms / 1e6);
        if (c % 12 == 11) std::printf("   (%.0f ms)\n", elapsed);
    }
    std::printf("\n");
    CHECK(hipGetLastError());
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
}

// ---- issue rate of the vector ALU -------------------------------------------
// What "bound by arithmetic" can mean on this chip: eight independent chains per
// lane of one instruction kind, nothing else in the loop but its counter.
// Reported per kind and per number of resident waves: lane-instructions per
// second over the whole chip, and the cycles of the device-reported clock that
// one SIMD spends per wave instruction.
enum IssueOp { OP_FMA, OP_MUL, OP_ADD, OP_MAD64, OP_MULLO, OP_RSQ, OP_SQRT, OP_RCP, OP_MULHI, OP_ADDU,
               OP_XOR, OP_AND, OP_SHIFT, OP_MINU, OP_SELECT, OP_MOVE, OP_CONVERT };

template <int OP>
__global__ void __launch_bounds__(256) issue_kernel(float* out, float a, float b, uint32_t ua, int iters) {
    float x[8];
    uint32_t u[8];
    uint64_t l[8];
    const uint64_t mask = 0x5555555555555555ull * (uint64_t)(ua | 1u);   // lanes of a select, in scalar registers
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        x[i] = a + 0.125f * (float)i + 1e-3f * (float)threadIdx.x;
        u[i] = ua * (uint32_t)(i + 1) + threadIdx.x;
        l[i] = ((uint64_t)u[i] << 32) | (uint32_t)(threadIdx.x + i);
    }
#pragma unroll 8
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (OP == OP_FMA) x[i] = __builtin_fmaf(x[i], a, b);
            if constexpr (OP == OP_MUL) x[i] = x[i] * a;
            if constexpr (OP == OP_ADD) x[i] = x[i] + b;
            if constexpr (OP == OP_MAD64) l[i] = (uint64_t)(uint32_t)l[i] * (uint64_t)ua + l[i];
            if constexpr (OP == OP_MULLO) u[i] = u[i] * u[i];
            if constexpr (OP == OP_MULHI) u[i] = __umulhi(u[i], u[i]);
            if constexpr (OP == OP_ADDU) u[i] = u[i] + u[(i + 1) & 7];
            // kinds the compiler would fold or fuse are written out (register operands only)
            if constexpr (OP == OP_XOR) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(u[i]) : "v"(ua));
            if constexpr (OP == OP_AND) asm volatile("v_and_b32 %0, %0, %1" : "+v"(u[i]) : "v"(ua));
            if constexpr (OP == OP_SHIFT) asm volatile("v_lshrrev_b32 %0, 1, %0" : "+v"(u[i]));
            if constexpr (OP == OP_MINU) asm volatile("v_min_u32 %0, %0, %1" : "+v"(u[i]) : "v"(ua));
            if constexpr (OP == OP_SELECT)
                asm volatile("v_cndmask_b32_e64 %0, %0, %1, %2" : "+v"(u[i]) : "v"(ua), "s"(mask));
            if constexpr (OP == OP_MOVE) asm volatile("v_mov_b32 %0, %1" : "=v"(u[i]) : "v"(ua));
            if constexpr (OP == OP_CONVERT) asm volatile("v_cvt_f32_u32 %0, %0" : "+v"(u[i]));
            if constexpr (OP == OP_RSQ) x[i] = __builtin_amdgcn_rsqf(x[i]);
            if constexpr (OP == OP_SQRT) x[i] = __builtin_amdgcn_sqrtf(x[i]);
            if constexpr (OP == OP_RCP) x[i] = __builtin_amdgcn_rcpf(x[i]);
        }
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) sum += x[i] + (float)u[i] + (float)(uint32_t)(l[i] >> 32) + (float)(uint32_t)l[i];
    out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

template <int OP> static void issue_rows(const char* name, float* out, int cus, double clock_hz) {
    const int iters = 20000;
    for (int per_cu : {1, 2, 4, 8}) {                // 256-thread blocks: that many waves per SIMD
        const unsigned grid = (unsigned)(cus * per_cu);
        const float t = median_of([&] {
            hipLaunchKernelGGL((issue_kernel<OP>), dim3(grid), dim3(256), 0, 0, out, 1.0000001f, 1e-9f,
                               2654435761u, iters);
        }, 9);
        const double wave_instr = (double)grid * 4.0 * iters * 8.0;
        std::printf("%-34s %d waves per SIMD  %8.1f us  %6.2f T lane-instr/s  %5.2f cycles per wave instruction and SIMD\n",
                    name, per_cu, t * 1e3, wave_instr * 64.0 / (t * 1e-3) / 1e12,
                    (double)cus * 4.0 * clock_hz * (t * 1e-3) / wave_instr);
        std::fflush(stdout);
    }
}

static void issue() {
    int dev = 0, cus = 0, khz = 0;
    CHECK(hipGetDevice(&dev));
    CHECK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    CHECK(hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev));
    float* out;
    CHECK(hipMalloc(&out, (size_t)cus * 8 * 256 * sizeof(float)));
    std::printf("%d compute units, device-reported clock %.2f GHz; 8 independent chains per lane, 20000 x 8 instructions per lane\n",
                cus, khz / 1e6);
    const double hz = khz * 1e3;
    issue_rows<OP_FMA>("v_fma_f32", out, cus, hz);
    issue_rows<OP_MUL>("v_mul_f32", out, cus, hz);
    issue_rows<OP_ADD>("v_add_f32", out, cus, hz);
    issue_rows<OP_MAD64>("v_mad_u64_u32", out, cus, hz);
    issue_rows<OP_MULLO>("v_mul_lo_u32", out, cus, hz);
    issue_rows<OP_MULHI>("v_mul_hi_u32", out, cus, hz);
    issue_rows<OP_ADDU>("v_add_u32", out, cus, hz);
    issue_rows<OP_XOR>("v_xor_b32", out, cus, hz);
    issue_rows<OP_AND>("v_and_b32", out, cus, hz);
    issue_rows<OP_SHIFT>("v_lshrrev_b32", out, cus, hz);
    issue_rows<OP_MINU>("v_min_u32", out, cus, hz);
    issue_rows<OP_SELECT>("v_cndmask_b32 (mask in SGPRs)", out, cus, hz);
    issue_rows<OP_MOVE>("v_mov_b32", out, cus, hz);
    issue_rows<OP_CONVERT>("v_cvt_f32_u32", out, cus, hz);
    issue_rows<OP_RSQ>("v_rsq_f32", out, cus, hz);
    issue_rows<OP_SQRT>("v_sqrt_f32", out, cus, hz);
    issue_rows<OP_RCP>("v_rcp_f32", out, cus, hz);
    CHECK(hipFree(out));
}

int main(int argc, char** argv) {
    const size_t n = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 25557032ull;
    if (n < 4 || n > (1ull << 32)) {
        std::printf("floats per stream must be in [4, 2^32]\n");
        return 2;
    }
    const size_t n4 = n / 4;
    if (argc > 2 && std::string(argv[2]) == "stagger") {
        stagger(n, n4);
        return 0;
    }
    if (argc > 2 && std::string(argv[2]) == "issue") {
        issue();
        return 0;
    }
    Streams a;
    for (int i = 0; i < 4; ++i) {
        void* p;
        CHECK(hipMalloc(&p, n4 * 16));
        CHECK(hipMemset(p, 0, n4 * 16));
        a.r[i] = static_cast<const f32x4*>(p);
        CHECK(hipMalloc(&p, n4 * 16));
        CHECK(hipMemset(p, 0, n4 * 16));
        a.w[i] = static_cast<f32x4*>(p);
    }
    CHECK(hipDeviceSynchronize());
    if (argc > 2 && std::string(argv[2]) == "sustain") {
        sustain(a, n4);
        return 0;
    }
    if (argc > 2 && std::string(argv[2]) == "shapes") {
        std::printf("streams of %zu floats (%.1f MB each)\n", n, n4 * 16 / 1e6);
        shapes(a, n4);
        return 0;
    }
    std::printf("streams of %zu floats (%.1f MB each); median of 15 launches, best of 3 launch shapes\n", n,
                n4 * 16 / 1e6);
    pattern<1, 0>("1 read", a, n4);
    pattern<0, 1>("1 write", a, n4);
    pattern<1, 1>("copy (pull)", a, n4);
    pattern<3, 1>("3 read 1 write (worker)", a, n4);
    pattern<4, 3>("4 read 3 write (push)", a, n4);
    return 0;
}
