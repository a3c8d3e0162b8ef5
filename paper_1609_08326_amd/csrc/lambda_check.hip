// Stand-alone checker for the short forms of sqrt and divide used by the
// adaptive-lambda kernels (root_rn_midrange / quotient_rn_midrange): compares
// them with the IEEE operations (correctly rounded sqrt and division as the
// compiler expands them) over their whole domain.
//
//   lambda_check roots                 every radicand in [2^-64, 2^64)
//   lambda_check quotients FIRST COUNT every radicand of two binades ([1, 4):
//                                      all significands, both exponent parities)
//                                      against numerators 1 + k*2^-23 for
//                                      k = FIRST .. FIRST+COUNT-1  (COUNT <= 2^23)
//   lambda_check sampled N SEED        N random (radicand, numerator) pairs over
//                                      the whole admitted range, both signs
//   lambda_check predicate N SEED      N random groups of four radicands (edges of
//                                      the window and the excluded pattern included):
//                                      the four-at-once admission test against
//                                      four single ones, and the wave-wide vote
//                                      against a vote over the single tests
//   lambda_check table N SEED FILE     N random (radicand, numerator) pairs over the
//                                      whole positive finite range (denormals included):
//                                      writes N records of six 32-bit words to FILE -
//                                      radicand, numerator, the device's IEEE sqrt and
//                                      quotient numerator/sqrt, and the short forms'
//                                      root and quotient (the IEEE values again where
//                                      the pair is not admitted) - so that a host
//                                      program can compare all four with its own CPU's
//                                      IEEE operations
//   lambda_check radius                the noise generator's radius sqrt(-2 ln u) in its short
//                                      form against the form with the general divide and
//                                      square root, on all 2^24 values of u
// Prints the number of cases and of mismatches, the first few mismatches, and
// exits non-zero if there is any.
#include <hip/hip_runtime.h>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "dcasgd_kernels.hip.h"

using namespace dcasgd;

#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); std::exit(2); } } while (0)

struct Report {
    unsigned long long mismatches;
    unsigned long long skipped;   // radicands the kernels do not take the short path for
    unsigned long long admitted_waves;   // predicate mode: waves whose vote was "all admitted"
    uint32_t first[8][4];   // radicand bits, numerator bits, got, expected
};

__device__ void note(Report* rep, uint32_t x, uint32_t a, float got, float want) {
    const unsigned long long slot = atomicAdd(&rep->mismatches, 1ull);
    if (slot < 8) {
        rep->first[slot][0] = x;
        rep->first[slot][1] = a;
        rep->first[slot][2] = __float_as_uint(got);
        rep->first[slot][3] = __float_as_uint(want);
    }
}

// every input of the noise radius: k = word >> 8 in [0, 2^24)
__global__ void check_radius(Report* rep) {
    const uint32_t k = blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= (1u << 24)) return;
    const uint32_t word = (k << 8) | (k & 0xFFu);      // the low byte does not enter
    const float want = radius_from_word_as<false>(word);
    const float got = radius_from_word_as<true>(word);
    if (__float_as_uint(got) != __float_as_uint(want)) note(rep, word, 0u, got, want);
}

// radicand bits first .. first+count-1
__global__ void check_roots(uint32_t first, uint32_t count, Report* rep) {
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += gridDim.x * blockDim.x) {
        const float x = __uint_as_float(first + i);
        if (!in_midrange(x)) { atomicAdd(&rep->skipped, 1ull); continue; }
        float y;
        const float got = root_rn_midrange(x, y);
        const float want = __builtin_sqrtf(x);
        if (__float_as_uint(got) != __float_as_uint(want)) note(rep, first + i, 0u, got, want);
    }
}

// thread <-> radicand in [1, 4); loop over numerators in [1, 2)
__global__ void check_quotients(uint32_t k_first, uint32_t k_count, Report* rep) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;      // < 2^24
    const uint32_t xb = 0x3F800000u + i;
    if (!in_midrange(__uint_as_float(xb))) { atomicAdd(&rep->skipped, (unsigned long long)k_count); return; }
    float y;
    const float root = root_rn_midrange(__uint_as_float(xb), y);
    for (uint32_t k = 0; k < k_count; ++k) {
        const uint32_t ab = 0x3F800000u + k_first + k;
        const float a = __uint_as_float(ab);
        const float got = quotient_rn_midrange(a, root, y);
        const float want = a / root;
        if (__float_as_uint(got) != __float_as_uint(want)) note(rep, xb, ab, got, want);
    }
}

__device__ uint32_t mix(uint32_t v) {          // any well-mixing hash will do here
    v ^= v >> 16; v *= 0x7FEB352Du; v ^= v >> 15; v *= 0x846CA68Bu; v ^= v >> 16;
    return v;
}

// radicands over [2^-64, 2^64), numerators over +-[2^-40, 2^40]
__global__ void check_sampled(unsigned long long n, uint32_t seed, Report* rep) {
    for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (unsigned long long)gridDim.x * blockDim.x) {
        const uint32_t u = mix((uint32_t)i ^ seed), v = mix(u + 0x9E3779B9u + (uint32_t)(i >> 32));
        const uint32_t xb = 0x1F800000u + (u & 0x3FFFFFFFu);
        const uint32_t mag = 0x2B800000u + (v % 0x28000001u);      // 2^-40 .. 2^40
        const uint32_t ab = mag | (v & 0x80000000u);
        if (!in_midrange(__uint_as_float(xb))) { atomicAdd(&rep->skipped, 1ull); continue; }
        float y;
        const float root = root_rn_midrange(__uint_as_float(xb), y);
        const float a = __uint_as_float(ab);
        const float got = quotient_rn_midrange(a, root, y);
        const float want = a / __builtin_sqrtf(__uint_as_float(xb));
        if (__float_as_uint(got) != __float_as_uint(want)) note(rep, xb, ab, got, want);
    }
}

// the four-at-once form of the admission test against four single tests
__global__ void check_predicate(unsigned long long n, uint32_t seed, Report* rep) {
    for (unsigned long long i = (unsigned long long)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (unsigned long long)gridDim.x * blockDim.x) {
        float x[4];
        bool each = true;
        uint32_t u = mix((uint32_t)i ^ seed) + (uint32_t)(i >> 32);
        // Per wave (64 consecutive cases): a third of the waves draw freely, a third
        // hold admitted radicands only, a third admitted ones except one value of
        // one lane - so that the wave-wide vote is exercised on both answers.
        const uint32_t wave_draw = mix((uint32_t)(i >> 6) * 0x9E3779B9u + seed);
        const uint32_t kind = wave_draw % 3u;
        const bool odd_one = kind == 2u && (uint32_t)(i & 63u) == ((wave_draw >> 8) & 63u);
        for (int c = 0; c < 4; ++c) {
            u = mix(u + 0x9E3779B9u);
            uint32_t b = u;
            if (kind != 0u) b = 0x1F800000u + (u & 0x3FFFFFFFu);                        // inside the window
            const bool steer = kind == 0u || (odd_one && (uint32_t)c == ((wave_draw >> 16) & 3u));
            // steer a share of the draws onto the interesting values
            if (steer && (u & 0x300u) == 0x100u)                                      // the patterns and
                b = (b & 0xFF000000u) | (0x007FFFFCu + ((u >> 10) & 3u) + ((u >> 12) & 1u));   // their neighbours
            if (steer && (u & 0x300u) == 0x200u) b = 0x1F800000u + (b & 3u) - 2u;       // lower edge
            if (steer && (u & 0x300u) == 0x300u) b = 0x5F800000u + (b & 3u) - 2u;       // upper edge
            x[c] = __uint_as_float(b);
            each = each && in_midrange(x[c]);
        }
        if (quad_in_midrange(x) != each) note(rep, __float_as_uint(x[0]), __float_as_uint(x[1]), 0.f, 0.f);
        // and the wave-wide vote the kernels take against a vote over the single tests
        const bool wave_wants = __builtin_amdgcn_ballot_w64(!each) == 0;
        if (wave_wants && (i & 63u) == 0) atomicAdd(&rep->admitted_waves, 1ull);
        if (wave_all_in_midrange(x) != wave_wants)
            note(rep, __float_as_uint(x[2]), __float_as_uint(x[3]), 1.f, wave_wants ? 1.f : 0.f);
    }
}

__global__ void fill_table(uint32_t n, uint32_t seed, uint32_t* out) {
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
        const uint32_t u = mix(i ^ seed), v = mix(u + 0x9E3779B9u);
        uint32_t xb = u & 0x7FFFFFFFu;                        // positive
        if ((xb >> 23) == 0xFFu) xb -= 0x00800000u;           // finite
        if ((u >> 31) != 0u && (i & 7u) == 0u) xb &= 0x007FFFFFu;   // a share of denormals
        uint32_t ab = v;
        if (((ab >> 23) & 0xFFu) == 0xFFu) ab -= 0x00800000u;
        const float x = __uint_as_float(xb), a = __uint_as_float(ab);
        const float root = __builtin_sqrtf(x);
        const float quot = a / root;
        float sroot = root, squot = quot;
        const float mag = __builtin_fabsf(a);
        if (in_midrange(x) && mag >= 0x1p-40f && mag <= 0x1p40f) {
            float y;
            sroot = root_rn_midrange(x, y);
            squot = quotient_rn_midrange(a, sroot, y);
        }
        uint32_t* rec = out + 6ull * i;
        rec[0] = xb; rec[1] = ab;
        rec[2] = __float_as_uint(root); rec[3] = __float_as_uint(quot);
        rec[4] = __float_as_uint(sroot); rec[5] = __float_as_uint(squot);
    }
}

static int finish(const char* what, unsigned long long cases, Report* dev) {
    Report host;
    CHECK(hipDeviceSynchronize());
    CHECK(hipMemcpy(&host, dev, sizeof(host), hipMemcpyDeviceToHost));
    std::printf("%s: %llu cases (%llu of them not admitted to the short path, skipped), "
                "%llu mismatches\n", what, cases, host.skipped, host.mismatches);
    for (unsigned long long i = 0; i < host.mismatches && i < 8; ++i)
        std::printf("  radicand 0x%08x numerator 0x%08x got 0x%08x expected 0x%08x\n",
                    host.first[i][0], host.first[i][1], host.first[i][2], host.first[i][3]);
    std::fflush(stdout);
    return host.mismatches ? 1 : 0;
}

int main(int argc, char** argv) {
    if (argc < 2) { std::fprintf(stderr, "usage: see the header of lambda_check.hip\n"); return 2; }
    Report* rep = nullptr;
    CHECK(hipMalloc(&rep, sizeof(Report)));
    CHECK(hipMemset(rep, 0, sizeof(Report)));
    if (!std::strcmp(argv[1], "roots")) {
        const uint32_t first = 0x1F800000u, total = 0x40000000u, step = 1u << 26;
        for (uint32_t done = 0; done < total; done += step) {
            hipLaunchKernelGGL(check_roots, dim3(4096), dim3(256), 0, 0, first + done, step, rep);
            CHECK(hipGetLastError());
            CHECK(hipDeviceSynchronize());
        }
        return finish("roots", total, rep);
    }
    if (!std::strcmp(argv[1], "radius")) {
        hipLaunchKernelGGL(check_radius, dim3((1u << 24) / 256), dim3(256), 0, 0, rep);
        CHECK(hipGetLastError());
        CHECK(hipDeviceSynchronize());
        return finish("radius", 1ull << 24, rep);
    }
    if (!std::strcmp(argv[1], "quotients") && argc >= 4) {
        const unsigned long long k_first = std::strtoull(argv[2], nullptr, 0);
        const unsigned long long k_count = std::strtoull(argv[3], nullptr, 0);
        if (k_first + k_count > (1ull << 23) || k_count == 0) { std::fprintf(stderr, "bad range\n"); return 2; }
        const uint32_t per_launch = 1u << 11;      // 2^24 radicands x 2^11 numerators per launch
        unsigned long long done = 0;
        int launches = 0;
        while (done < k_count) {
            const uint32_t now = (uint32_t)((k_count - done < per_launch) ? k_count - done : per_launch);
            hipLaunchKernelGGL(check_quotients, dim3((1u << 24) / 256), dim3(256), 0, 0,
                               (uint32_t)(k_first + done), now, rep);
            CHECK(hipGetLastError());
            CHECK(hipDeviceSynchronize());
            done += now;
            if (++launches % 64 == 0) {
                Report host;
                CHECK(hipMemcpy(&host, rep, sizeof(host), hipMemcpyDeviceToHost));
                std::printf("  numerators %llu of %llu done, %llu mismatches so far\n", done, k_count,
                            host.mismatches);
                std::fflush(stdout);
            }
        }
        return finish("quotients", (1ull << 24) * k_count, rep);
    }
    if (!std::strcmp(argv[1], "sampled") && argc >= 4) {
        const unsigned long long n = std::strtoull(argv[2], nullptr, 0);
        const uint32_t seed = (uint32_t)std::strtoull(argv[3], nullptr, 0);
        hipLaunchKernelGGL(check_sampled, dim3(8192), dim3(256), 0, 0, n, seed, rep);
        CHECK(hipGetLastError());
        return finish("sampled", n, rep);
    }
    if (!std::strcmp(argv[1], "predicate") && argc >= 4) {
        const unsigned long long n = std::strtoull(argv[2], nullptr, 0);
        const uint32_t seed = (uint32_t)std::strtoull(argv[3], nullptr, 0);
        hipLaunchKernelGGL(check_predicate, dim3(8192), dim3(256), 0, 0, n, seed, rep);
        CHECK(hipGetLastError());
        const int rc = finish("predicate", n, rep);
        Report host;
        CHECK(hipMemcpy(&host, rep, sizeof(host), hipMemcpyDeviceToHost));
        std::printf("predicate: %llu of %llu waves voted that all their radicands are admitted\n",
                    host.admitted_waves, (n + 63) / 64);
        return rc;
    }
    if (!std::strcmp(argv[1], "table") && argc >= 5) {
        const unsigned long long n = std::strtoull(argv[2], nullptr, 0);
        const uint32_t seed = (uint32_t)std::strtoull(argv[3], nullptr, 0);
        if (n == 0 || n > (1ull << 26)) { std::fprintf(stderr, "N must be in [1, 2^26]\n"); return 2; }
        uint32_t* dev = nullptr;
        CHECK(hipMalloc(&dev, n * 24));
        hipLaunchKernelGGL(fill_table, dim3(4096), dim3(256), 0, 0, (uint32_t)n, seed, dev);
        CHECK(hipGetLastError());
        CHECK(hipDeviceSynchronize());
        std::vector<uint32_t> host(n * 6);
        CHECK(hipMemcpy(host.data(), dev, n * 24, hipMemcpyDeviceToHost));
        std::FILE* f = std::fopen(argv[4], "wb");
        if (!f || std::fwrite(host.data(), 24, n, f) != n || std::fclose(f) != 0) {
            std::fprintf(stderr, "cannot write %s\n", argv[4]);
            return 2;
        }
        std::printf("table: %llu records written to %s\n", n, argv[4]);
        return 0;
    }
    std::fprintf(stderr, "usage: see the header of lambda_check.hip\n");
    return 2;
}
