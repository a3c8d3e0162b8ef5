// Memory-system probe for the box the library runs on: what a plain streaming
// kernel with the library's tile structure (128-bit accesses, one contiguous
// 1 KiB run per wave access, all loads of a tile issued up front) achieves for
// R read streams and W write streams, with plain or non-temporal accesses.
// It gives the practical ceiling the update kernels are compared against:
// the DC-ASGD push is a 4-read/3-write stream, the pull a copy, the worker
// kernel 3 reads and 1 write.
//
// usage: membw_probe [floats per stream, default 25557032]
// Allocates (4 + 4) buffers of that many floats; prints GB/s per pattern.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstdlib>
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

int main(int argc, char** argv) {
    const size_t n = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 25557032ull;
    if (n < 4 || n > (1ull << 32)) {
        std::printf("floats per stream must be in [4, 2^32]\n");
        return 2;
    }
    const size_t n4 = n / 4;
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
    std::printf("streams of %zu floats (%.1f MB each); median of 15 launches, best of 3 launch shapes\n", n,
                n4 * 16 / 1e6);
    pattern<1, 0>("1 read", a, n4);
    pattern<0, 1>("1 write", a, n4);
    pattern<1, 1>("copy (pull)", a, n4);
    pattern<3, 1>("3 read 1 write (worker)", a, n4);
    pattern<4, 3>("4 read 3 write (push)", a, n4);
    return 0;
}
