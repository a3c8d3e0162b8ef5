// Host side of the C ABI declared in include/dcasgd.h: argument validation,
// bookkeeping of Algorithm 2's counter t and of which backups are current,
// and kernel launches.  No allocator is called here; the one device array the
// library owns is the static workspace declared below.
#include "../../include/dcasgd.h"

#include <algorithm>
#include <cmath>
#include <mutex>
#include <new>
#include <type_traits>
#include <vector>

#include <hip/hip_ext.h>

#include "dcasgd_kernels.hip.h"

using namespace dcasgd;

// Scratch of dcasgd_sync_fold_ordered_static, the entry point for callers that
// cannot allocate: one FoldWorkspace (256.5 KB) that every GPU the library
// runs on holds until the process ends.  In host code the array's name is only
// a stand-in; the device address is looked up once per GPU (scratch_on_current_
// device) and that pointer is what kernels receive.
static __device__ __align__(256) unsigned char scratch[sizeof(FoldWorkspace)];

namespace {
constexpr int kMaxDevices = 64;
void* scratch_address[kMaxDevices] = {};   // device address of `scratch`, per GPU, once known
std::mutex scratch_lock;

// Address of this GPU's copy of `scratch`; nullptr if the runtime cannot tell.
void* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> guard(scratch_lock);
    if (!scratch_address[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        scratch_address[dev] = p;
    }
    return scratch_address[dev];
}
}  // namespace

// Launches that can be timed between two dcasgd_timing_read calls; further
// ones run untimed, so an unread handle does not pile up events.
#define DCASGD_MAX_TIMED 65536
#ifndef DCASGD_FOLD_KC
#define DCASGD_FOLD_KC 4      // gradients of a fold a lane loads before it starts on them
#endif
#ifndef DCASGD_RUN_PAIRS_BELOW
#define DCASGD_RUN_PAIRS_BELOW (1 << 17)   // float4 groups below which the event loop gives a group two lanes
                                           // (fewer than two waves per SIMD otherwise; measured equal at 2^17)
#endif
#ifndef DCASGD_NORM_ITEMS
#define DCASGD_NORM_ITEMS 4   // float4 groups a lane of the norm kernel has in flight
#endif

struct dcasgd_server {
    size_t d = 0;
    int M = 0;
    Hyper hp{};
    bool adaptive = false, grad_bf16 = false, pull_on_push = false;
    bool bak_bf16 = false;            // backup rows hold bfloat16 snapshots
    float* w = nullptr;
    void* bak = nullptr;
    size_t bak_stride = 0;            // in elements of the backup format
    float* ms = nullptr;
    bool bound = false, ready = false;
    hipStream_t stream = nullptr;     // stream of the most recent call that changed w (init, push*, fold*)
    uint64_t t = 0;                   // pushes applied (Algorithm 2's t)
    std::vector<uint64_t> fresh_at;   // t at which w_bak(m) was last set to w
    int threads = 256, max_blocks = 0;
    int items = 1;                    // float4 groups per lane of the worker-fused push
    int push_items = 2;               // ... of the push and pull kernels (both set by size in dcasgd_create)
    int batch_threads = 64;           // the queue kernel does 16x the work per lane: one wave per block
    int streaming = 2;                // 0 plain, 1 gradient+backup non-temporal, 2 everything, 3 worker too
    int norm_blocks = 0;              // grid of the norm kernel, set by dcasgd_init
    int last_error = DCASGD_OK;
    uint32_t* ctr = nullptr;          // optional device-resident copy of t (low 32 bits)
    // optional per-launch timing of the server-update kernels
    bool timing = false;
    std::vector<hipEvent_t> timing_events;   // start, stop, start, stop, ...
    size_t timing_used = 0;                  // events handed out since the last read
};

namespace {

inline int fail(dcasgd_t h, int code) {
    if (h) h->last_error = code;
    return code;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

inline bool overlaps(const void* a, size_t abytes, const void* b, size_t bbytes) {
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + bbytes && b0 < a0 + abytes;
}

inline bool valid_threads(int t) { return t >= 64 && t <= 512 && t % 64 == 0; }
inline bool valid_items(int i) { return i == 1 || i == 2 || i == 4; }

template <class F> inline void with_bool(bool v, F&& f) {
    if (v) f(std::true_type{}); else f(std::false_type{});
}
template <class F> inline void with_level(int v, F&& f) {
    switch (v) {
        case 0: f(std::integral_constant<int, 0>{}); break;
        case 1: f(std::integral_constant<int, 1>{}); break;
        default: f(std::integral_constant<int, 2>{}); break;
    }
}
// Load-group size of the queue kernel by queue length: a kernel built for
// groups of 16 holds 32 float4 registers of loads per lane whatever the queue
// brings; shorter queues (and the pieces a queue with repeated workers is cut
// into) run the kernel built for groups of 8, 4, 2, 1.  (A third kernel built
// for groups of at most 4 keeps more waves resident and measured 2 % slower on
// pieces of about four entries.)
template <class F> inline void with_group(int K, F&& f) {
    if (K >= 16) f(std::integral_constant<int, 16>{});
    else f(std::integral_constant<int, 8>{});
}
template <class F> inline void with_items(int v, F&& f) {
    switch (v) {
        case 1: f(std::integral_constant<int, 1>{}); break;
        case 2: f(std::integral_constant<int, 2>{}); break;
        default: f(std::integral_constant<int, 4>{}); break;
    }
}

// blocks needed so that every tile of `per_block` float4 groups is covered
inline unsigned grid_for(size_t n4, size_t per_block, int max_blocks) {
    size_t tiles = (n4 + per_block - 1) / per_block;
    if (tiles == 0) tiles = 1;                       // the ragged tail still needs block 0
    if (max_blocks > 0 && tiles > (size_t)max_blocks) tiles = (size_t)max_blocks;
    if (tiles > 0x7FFFFFFFull) tiles = 0x7FFFFFFFull; // blocks loop over tiles anyway
    return (unsigned)tiles;
}

// Two events of their own for the next timed launch (created on demand, reused).
inline bool next_event_pair(dcasgd_t h, hipEvent_t* start, hipEvent_t* stop) {
    if (h->timing_used >= 2 * (size_t)DCASGD_MAX_TIMED) return false;   // unread backlog full
    while (h->timing_events.size() < h->timing_used + 2) {
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return false;
        h->timing_events.push_back(e);
    }
    *start = h->timing_events[h->timing_used];
    *stop = h->timing_events[h->timing_used + 1];
    h->timing_used += 2;
    return true;
}

// Launch of a server-update kernel.  With timing on, the launch itself carries
// a start and a stop event (hipExtLaunchKernelGGL), so the pair brackets the
// kernel's execution and nothing else; no extra packet goes into the stream.
#define DCASGD_LAUNCH(h, kern, grid, block, s, ...)                                          \
    do {                                                                                       \
        hipEvent_t ev0_ = nullptr, ev1_ = nullptr;                                             \
        if ((h)->timing && next_event_pair((h), &ev0_, &ev1_))                                 \
            hipExtLaunchKernelGGL(kern, dim3(grid), dim3(block), 0, s, ev0_, ev1_, 0,          \
                                  __VA_ARGS__);                                                \
        else                                                                                   \
            hipLaunchKernelGGL(kern, dim3(grid), dim3(block), 0, s, __VA_ARGS__);              \
    } while (0)

// keep the device-resident push counter in step with t after n applied pushes
inline void advance_counter(dcasgd_t h, uint32_t n, hipStream_t s) {
    if (h->ctr) hipLaunchKernelGGL(counter_add_kernel, dim3(1), dim3(64), 0, s, h->ctr, n);
}

inline int launched(dcasgd_t h) {
    return hipGetLastError() == hipSuccess ? DCASGD_OK : fail(h, DCASGD_EHIP);
}

inline size_t grad_bytes(const dcasgd_server* h) { return h->d * (h->grad_bf16 ? 2 : 4); }
inline size_t bak_elem(const dcasgd_server* h) { return h->bak_bf16 ? 2 : 4; }
inline size_t bak_bytes(const dcasgd_server* h) {
    return (size_t)h->M * h->bak_stride * bak_elem(h);
}
inline void* bak_row(const dcasgd_server* h, int worker) {
    return static_cast<char*>(h->bak) + (size_t)worker * h->bak_stride * bak_elem(h);
}

int check_grad(dcasgd_t h, const void* grad) {
    if (!grad) return DCASGD_EINVAL;
    if (!aligned(grad, h->grad_bf16 ? 8 : 16)) return DCASGD_EALIGN;
    const size_t gb = grad_bytes(h);
    if (overlaps(grad, gb, h->w, h->d * 4) ||
        overlaps(grad, gb, h->bak, bak_bytes(h)) ||
        (h->ms && overlaps(grad, gb, h->ms, h->d * 4)) ||
        (h->hp.vel && overlaps(grad, gb, h->hp.vel, h->d * 4)))
        return DCASGD_EINVAL;
    return DCASGD_OK;
}

void launch_pull(dcasgd_t h, int worker, hipStream_t s) {
    const size_t n4 = h->d / 4;
    void* row = bak_row(h, worker);
    const unsigned grid = grid_for(n4, (size_t)h->threads * h->push_items, h->max_blocks);
    with_items(h->push_items, [&](auto IT) {
        with_bool(h->streaming != 0, [&](auto NT) {
          with_bool(h->bak_bf16, [&](auto BB) {
            DCASGD_LAUNCH(h, (pull_kernel<decltype(IT)::value, decltype(NT)::value,
                                          decltype(BB)::value>), grid,
                          h->threads, s, static_cast<const float*>(h->w), row, n4, h->d);
          });
        });
    });
}

void launch_push(dcasgd_t h, int worker, const void* grad, bool fuse_pull, hipStream_t s) {
    const size_t n4 = h->d / 4;
    void* row = bak_row(h, worker);
    const unsigned grid = grid_for(n4, (size_t)h->threads * h->push_items, h->max_blocks);
    with_bool(h->adaptive, [&](auto AD) {
     with_bool(h->hp.vel != nullptr, [&](auto MO) {
      with_bool(h->grad_bf16, [&](auto BF) {
        with_bool(fuse_pull, [&](auto PL) {
          with_items(h->push_items, [&](auto IT) {
            if (h->bak_bf16) {
                // bfloat16 backups come in the fully streaming form only
                DCASGD_LAUNCH(h, (push_kernel<decltype(AD)::value, decltype(MO)::value,
                                              decltype(BF)::value, decltype(PL)::value,
                                              decltype(IT)::value, 2, true>),
                              grid, h->threads, s, h->hp, h->w, h->ms, row, grad, n4, h->d);
                return;
            }
            with_level(h->streaming, [&](auto NT) {
                DCASGD_LAUNCH(h, (push_kernel<decltype(AD)::value, decltype(MO)::value,
                                              decltype(BF)::value, decltype(PL)::value,
                                              decltype(IT)::value, decltype(NT)::value, false>),
                              grid, h->threads, s, h->hp, h->w, h->ms, row, grad, n4, h->d);
            });
          });
        });
      });
     });
    });
}

// Grid of the norm kernel.  A pure read stream is fastest with few, long-lived
// blocks: two per compute unit measured best on MI355X (one 102 MB vector in
// 15 us).  Asked once per handle, in dcasgd_init, so that the fold calls
// themselves make no device queries.
bool size_norm_grid(dcasgd_t h) {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
        cus < 1) {
        (void)hipGetLastError();
        return false;
    }
    h->norm_blocks = 2 * cus < FOLD_WS_BLOCKS ? 2 * cus : FOLD_WS_BLOCKS;
    return true;
}

// entries [k0, k1) of a queue; their workers are pairwise distinct
void launch_batch(dcasgd_t h, const int* workers, const void* const* grads, int k0, int k1,
                  hipStream_t s) {
    BatchArgs a{};
    a.K = k1 - k0;
    for (int k = k0; k < k1; ++k) {
        a.grad[k - k0] = grads[k];
        a.bak[k - k0] = bak_row(h, workers[k]);
    }
    const size_t n4 = h->d / 4;
    const int threads = h->batch_threads;
    const unsigned grid = grid_for(n4, (size_t)threads, h->max_blocks);
    with_bool(h->adaptive, [&](auto AD) {
     with_bool(h->hp.vel != nullptr, [&](auto MO) {
      with_bool(h->grad_bf16, [&](auto BF) {
        with_bool(h->streaming != 0, [&](auto NT) {
          with_bool(h->bak_bf16, [&](auto BB) {
            with_group(a.K, [&](auto KC) {
              DCASGD_LAUNCH(h, (push_batch_kernel<decltype(AD)::value, decltype(MO)::value,
                                                  decltype(BF)::value, decltype(KC)::value,
                                                  decltype(NT)::value, decltype(BB)::value>),
                            grid, threads, s, h->hp, h->w, h->ms, a, n4, h->d);
            });
          });
        });
      });
     });
    });
}

}  // namespace

extern "C" {

dcasgd_t dcasgd_create(size_t d, int M, float eta, float lambda0, int mode, float ema_m,
                       float eps) {
    const int variant = mode & 0xF;
    const int flags = mode & ~0xF;
    if (d == 0 || M <= 0) return nullptr;
    if (variant != DCASGD_MODE_C && variant != DCASGD_MODE_A) return nullptr;
    if (flags & ~(DCASGD_GRAD_BF16 | DCASGD_PULL_ON_PUSH | DCASGD_BAK_BF16)) return nullptr;
    if (!std::isfinite(eta) || !std::isfinite(lambda0) || !std::isfinite(ema_m) ||
        !std::isfinite(eps))
        return nullptr;
    if (variant == DCASGD_MODE_A && (!(ema_m >= 0.0f && ema_m < 1.0f) || eps < 0.0f))
        return nullptr;
    dcasgd_server* h = new (std::nothrow) dcasgd_server;
    if (!h) return nullptr;
    h->d = d;
    h->M = M;
    h->hp.eta = eta;
    h->hp.lambda0 = lambda0;
    h->hp.ema_m = ema_m;
    h->hp.one_minus_m = 1.0f - ema_m;
    h->hp.eps = eps;
    const float mag = std::fabs(lambda0);
    h->hp.lambda_midrange = (mag >= 0x1p-40f && mag <= 0x1p40f) ? 1 : 0;
    h->adaptive = variant == DCASGD_MODE_A;
    h->grad_bf16 = (flags & DCASGD_GRAD_BF16) != 0;
    h->pull_on_push = (flags & DCASGD_PULL_ON_PUSH) != 0;
    h->bak_bf16 = (flags & DCASGD_BAK_BF16) != 0;
    h->fresh_at.assign((size_t)M, 0);
    // four float4 groups per lane once the vectors dwarf the last-level cache (measured:
    // 2 % faster than two at 550 MB per vector, 0-2 % slower at 100 MB)
    h->push_items = d >= ((size_t)1 << 26) ? 4 : 2;
    // the worker-fused push (three times the registers per group): one group per lane
    // while the vectors are of the last-level cache's order, four once they dwarf it
    // (measured: 131 / 135 / 137 us for 1 / 2 / 4 at 100 MB vectors, 822 / 786 / 754 us
    // at 550 MB)
    h->items = d >= ((size_t)1 << 26) ? 4 : 1;
    return h;
}

int dcasgd_destroy(dcasgd_t h) {
    if (!h) return DCASGD_EINVAL;
    for (hipEvent_t e : h->timing_events) (void)hipEventDestroy(e);
    delete h;
    return DCASGD_OK;
}

int dcasgd_bind(dcasgd_t h, float* w, void* bak, size_t bak_stride, float* ms) {
    if (!h) return DCASGD_EINVAL;
    if (!w || !bak || (h->adaptive && !ms)) return fail(h, DCASGD_EINVAL);
    if (bak_stride < h->d) return fail(h, DCASGD_EINVAL);
    // every row must start on a 16-byte boundary: 4 floats or 8 bfloat16 values
    if (!aligned(w, 16) || !aligned(bak, 16) || (ms && !aligned(ms, 16)) ||
        bak_stride % (h->bak_bf16 ? 8 : 4) != 0)
        return fail(h, DCASGD_EALIGN);
    const size_t vb = h->d * 4, bb = (size_t)h->M * bak_stride * bak_elem(h);
    if (overlaps(w, vb, bak, bb) || (ms && (overlaps(ms, vb, bak, bb) || overlaps(ms, vb, w, vb))))
        return fail(h, DCASGD_EINVAL);
    h->w = w;
    h->bak = bak;
    h->bak_stride = bak_stride;
    h->ms = ms;
    h->hp.mu = 0.0f;          // a velocity vector belongs to the state it was set up for
    h->hp.vel = nullptr;
    h->ctr = nullptr;
    h->bound = true;
    h->ready = false;
    return DCASGD_OK;
}

int dcasgd_init(dcasgd_t h, void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->bound) return fail(h, DCASGD_ESTATE);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // set-up work of dcasgd_sync_fold_ordered_static is done here, so that the
    // call itself is nothing but launches (a failed lookup is retried there)
    (void)scratch_on_current_device();
    (void)size_norm_grid(h);
    for (int m = 0; m < h->M; ++m) launch_pull(h, m, s);
    if (h->ms) {
        const size_t n4 = h->d / 4;
        const unsigned grid = grid_for(n4, 512, 4096);
        hipLaunchKernelGGL(fill_kernel, dim3(grid), dim3(512), 0, s, h->ms, 0.0f, n4, h->d);
    }
    if (h->ctr) hipLaunchKernelGGL(counter_set_kernel, dim3(1), dim3(64), 0, s, h->ctr, 0u);
    h->stream = s;
    h->t = 0;
    h->fresh_at.assign((size_t)h->M, 0);
    const int rc = launched(h);
    h->ready = rc == DCASGD_OK;       // a handle whose initial copies did not launch stays unusable
    return rc;
}

int dcasgd_push(dcasgd_t h, int worker, const void* grad, void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    if (worker < 0 || worker >= h->M) return fail(h, DCASGD_EINVAL);
    if (int rc = check_grad(h, grad)) return fail(h, rc);
    hipStream_t s = static_cast<hipStream_t>(stream);
    launch_push(h, worker, grad, h->pull_on_push, s);
    advance_counter(h, 1, s);
    h->stream = s;
    h->t += 1;
    if (h->pull_on_push) h->fresh_at[(size_t)worker] = h->t;
    return launched(h);
}

int dcasgd_push_batch(dcasgd_t h, const int* workers, const void* const* grads, int K,
                      void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    if (!workers || !grads || K < 1 || K > DCASGD_MAX_K) return fail(h, DCASGD_EINVAL);
    for (int k = 0; k < K; ++k) {
        if (workers[k] < 0 || workers[k] >= h->M) return fail(h, DCASGD_EINVAL);
        if (int rc = check_grad(h, grads[k])) return fail(h, rc);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    // cut the queue wherever a worker shows up a second time within a launch
    int begin = 0;
    while (begin < K) {
        int end = begin + 1;
        for (; end < K; ++end) {
            bool seen = false;
            for (int k = begin; k < end; ++k) seen = seen || workers[k] == workers[end];
            if (seen) break;
        }
        launch_batch(h, workers, grads, begin, end, s);
        begin = end;
    }
    advance_counter(h, (uint32_t)K, s);
    h->stream = s;
    for (int k = 0; k < K; ++k) {
        h->t += 1;
        h->fresh_at[(size_t)workers[k]] = h->t;
    }
    return launched(h);
}

// what the worker-fused calls ask of the synthetic loss besides a valid worker
static int check_synth_loss(dcasgd_t h, const float* hdiag, const float* wstar, float sigma) {
    if (!hdiag || !wstar || !std::isfinite(sigma)) return DCASGD_EINVAL;
    if (h->d > ((size_t)1 << 34)) return DCASGD_EINVAL;    // the counter holds i/4 in 32 bits
    if (!aligned(hdiag, 16) || !aligned(wstar, 16)) return DCASGD_EALIGN;
    const size_t vb = h->d * 4, bb = bak_bytes(h);
    const void* loss[2] = {hdiag, wstar};
    for (const void* p : loss)
        if (overlaps(p, vb, h->w, vb) || overlaps(p, vb, h->bak, bb) ||
            (h->ms && overlaps(p, vb, h->ms, vb)) ||
            (h->hp.vel && overlaps(p, vb, h->hp.vel, vb)))
            return DCASGD_EINVAL;
    return DCASGD_OK;
}

int dcasgd_push_synth(dcasgd_t h, int worker, const float* hdiag, const float* wstar, float sigma,
                      uint64_t seed, void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    if (worker < 0 || worker >= h->M || h->t > 0xFFFFFFFFull) return fail(h, DCASGD_EINVAL);
    if (int rc = check_synth_loss(h, hdiag, wstar, sigma)) return fail(h, rc);
    const size_t n4 = h->d / 4;
    void* row = bak_row(h, worker);
    const unsigned grid = grid_for(n4, (size_t)h->threads * h->items, h->max_blocks);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    // with a device-resident counter the kernel reads the push index itself
    const uint32_t push_idx = h->ctr ? 0u : (uint32_t)h->t;
    hipStream_t s = static_cast<hipStream_t>(stream);
    with_bool(h->adaptive, [&](auto AD) {
     with_bool(h->hp.vel != nullptr, [&](auto MO) {
      with_bool(h->grad_bf16, [&](auto BF) {
        with_bool(h->pull_on_push, [&](auto PL) {
          with_items(h->items, [&](auto IT) {
            with_bool(h->bak_bf16, [&](auto BB) {
              DCASGD_LAUNCH(h, (push_synth_kernel<decltype(AD)::value, decltype(MO)::value,
                                                  decltype(BF)::value, decltype(PL)::value,
                                                  decltype(IT)::value, decltype(BB)::value>),
                            grid, h->threads, s, h->hp, h->w, h->ms, row, hdiag, wstar, sigma, k0,
                            k1, push_idx, h->ctr, n4, h->d);
            });
          });
        });
      });
     });
    });
    advance_counter(h, 1, s);
    h->stream = s;
    h->t += 1;
    if (h->pull_on_push) h->fresh_at[(size_t)worker] = h->t;
    return launched(h);
}

int dcasgd_run_synth(dcasgd_t h, const int* workers, size_t T, const float* hdiag,
                     const float* wstar, float sigma, uint64_t seed, void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    if (!workers && T > 0) return fail(h, DCASGD_EINVAL);
    for (size_t e = 0; e < T; ++e)
        if (workers[e] < 0 || workers[e] >= h->M) return fail(h, DCASGD_EINVAL);
    if (h->t + T > 0xFFFFFFFFull) return fail(h, DCASGD_EINVAL);
    if (int rc = check_synth_loss(h, hdiag, wstar, sigma)) return fail(h, rc);
    if (T == 0) return DCASGD_OK;
    if (h->M > 65536) {
        // the block kernel names workers in 16 bits: beyond that, arrival by arrival
        for (size_t e = 0; e < T; ++e)
            if (int rc = dcasgd_push_synth(h, workers[e], hdiag, wstar, sigma, seed, stream)) return rc;
        return DCASGD_OK;
    }
    // Blocks of up to RUN_BLOCK arrivals per launch; one float4 group per lane
    // and pass, since a lane stays with its group for the whole block.  Short
    // vectors (fewer groups than give every SIMD a few waves) are cut finer:
    // two lanes per group.
    const size_t n4 = h->d / 4;
    const bool pairs = n4 < (size_t)DCASGD_RUN_PAIRS_BELOW;
    const size_t lanes = pairs ? 2 * n4 : n4;
    const int threads = lanes >= ((size_t)1 << 20) ? 256 : 64;
    // one more block when d is not a multiple of four: it does that tail and nothing else
    const unsigned grid = grid_for(lanes, (size_t)threads, h->max_blocks) + (h->d % 4 ? 1u : 0u);
    const size_t row_bytes = h->bak_stride * bak_elem(h);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (size_t e0 = 0; e0 < T; e0 += RUN_BLOCK) {
        const int A = (int)std::min<size_t>(RUN_BLOCK, T - e0);
        Arrivals arr{};
        for (int e = 0; e < A; ++e) arr.worker[e] = (uint16_t)workers[e0 + e];
        const uint32_t push_idx = h->ctr ? 0u : (uint32_t)h->t;
        with_bool(h->adaptive, [&](auto AD) {
         with_bool(h->hp.vel != nullptr, [&](auto MO) {
          with_bool(h->grad_bf16, [&](auto BF) {
            with_bool(h->pull_on_push, [&](auto PL) {
              with_bool(h->bak_bf16, [&](auto BB) {
                with_bool(h->streaming != 0, [&](auto NT) {
                  if (pairs)
                      DCASGD_LAUNCH(h, (run_synth_pairs_kernel<decltype(AD)::value, decltype(MO)::value,
                                                               decltype(BF)::value, decltype(PL)::value,
                                                               decltype(BB)::value, decltype(NT)::value>),
                                    grid, threads, s, h->hp, h->w, h->ms, h->bak, row_bytes, hdiag,
                                    wstar, sigma, k0, k1, push_idx, h->ctr, arr, A, n4, h->d);
                  else
                      DCASGD_LAUNCH(h, (run_synth_kernel<decltype(AD)::value, decltype(MO)::value,
                                                         decltype(BF)::value, decltype(PL)::value,
                                                         decltype(BB)::value, decltype(NT)::value>),
                                    grid, threads, s, h->hp, h->w, h->ms, h->bak, row_bytes, hdiag,
                                    wstar, sigma, k0, k1, push_idx, h->ctr, arr, A, n4, h->d);
                });
              });
            });
          });
         });
        });
        advance_counter(h, (uint32_t)A, s);
        h->stream = s;
        for (int e = 0; e < A; ++e) {
            h->t += 1;
            if (h->pull_on_push) h->fresh_at[(size_t)workers[e0 + e]] = h->t;
        }
        if (int rc = launched(h)) return rc;
    }
    return DCASGD_OK;
}

// Both fold entry points: with a workspace the gradients are first ranked by
// norm on the device and folded in that order, without one the caller's order
// stands.
static int fold_impl(dcasgd_t h, const void* const* grads, int J, int J_total, float eta_hat,
                     FoldWorkspace* ws, bool ordered, const float* kept, void* stream,
                     bool apply = true, bool untimed = false) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    // untimed: launches carry no events even while timing is on (events are
    // created on demand, which is an allocation)
    struct TimingOff {
        dcasgd_t h; bool was;
        TimingOff(dcasgd_t h_, bool off) : h(h_), was(h_->timing) { if (off) h->timing = false; }
        ~TimingOff() { h->timing = was; }
    } timing_guard(h, untimed);
    if (!grads || J < 1 || J > DCASGD_MAX_K || J_total < J || !std::isfinite(eta_hat))
        return fail(h, DCASGD_EINVAL);
    if (kept) {
        // the kept w_t may be a backup row (a pull is the natural way to keep it), but
        // nothing the fold writes and none of its gradients
        if (h->bak_bf16 && overlaps(kept, h->d * 4, h->bak, bak_bytes(h))) return fail(h, DCASGD_EINVAL);
        if (!aligned(kept, 16)) return fail(h, DCASGD_EALIGN);
        if (overlaps(kept, h->d * 4, h->w, h->d * 4) ||
            (h->ms && overlaps(kept, h->d * 4, h->ms, h->d * 4)) ||
            (h->hp.vel && overlaps(kept, h->d * 4, h->hp.vel, h->d * 4)))
            return fail(h, DCASGD_EINVAL);
        for (int j = 0; j < J; ++j)
            if (grads[j] && overlaps(kept, h->d * 4, grads[j], grad_bytes(h)))
                return fail(h, DCASGD_EINVAL);
    }
    FoldArgs a{};
    a.J = J;
    for (int j = 0; j < J; ++j) {
        if (int rc = check_grad(h, grads[j])) return fail(h, rc);
        a.grad[j] = grads[j];
    }
    if (ordered) {
        if (!ws) return fail(h, DCASGD_EINVAL);
        if (!aligned(ws, 256)) return fail(h, DCASGD_EALIGN);
        const size_t wb = sizeof(FoldWorkspace);
        if (overlaps(ws, wb, h->w, h->d * 4) ||
            overlaps(ws, wb, h->bak, bak_bytes(h)) ||
            (h->ms && overlaps(ws, wb, h->ms, h->d * 4)) ||
            (h->hp.vel && overlaps(ws, wb, h->hp.vel, h->d * 4)) ||
            (h->ctr && overlaps(ws, wb, h->ctr, 4)))
            return fail(h, DCASGD_EINVAL);
        for (int j = 0; j < J; ++j)
            if (overlaps(ws, wb, grads[j], grad_bytes(h))) return fail(h, DCASGD_EINVAL);
    }
    Hyper hp = h->hp;
    hp.eta = eta_hat / (float)J_total;      // per-gradient step, formed once in binary32
    const size_t n4 = h->d / 4;
    const int threads = h->batch_threads;
    const unsigned grid = grid_for(n4, (size_t)threads, h->max_blocks);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (ordered) {
        if (h->norm_blocks == 0 && !size_norm_grid(h)) return fail(h, DCASGD_EHIP);
        const int cap = (h->max_blocks > 0 && h->max_blocks < h->norm_blocks) ? h->max_blocks
                                                                              : h->norm_blocks;
        const unsigned nblocks = grid_for(n4, 256 * DCASGD_NORM_ITEMS, cap);
        with_bool(h->grad_bf16, [&](auto BF) {
          with_bool(h->streaming != 0, [&](auto NT) {
            DCASGD_LAUNCH(h, (grad_sqnorm_kernel<decltype(BF)::value, decltype(NT)::value,
                                                  DCASGD_NORM_ITEMS>),
                          nblocks, 256, s, a, ws, n4, h->d);
          });
        });
        DCASGD_LAUNCH(h, fold_order_kernel, 1, 1024, s, a, ws, (int)nblocks);
        if (!apply)                        // norms and ranking only: the model is not touched,
            return launched(h);            // and the stream a later pull uses stays what it was
    }
    with_bool(h->adaptive, [&](auto AD) {
     with_bool(h->hp.vel != nullptr, [&](auto MO) {
      with_bool(h->grad_bf16, [&](auto BF) {
        with_bool(h->streaming != 0, [&](auto NT) {
          if (kept) {
            DCASGD_LAUNCH(h, (sync_fold_kernel<decltype(AD)::value, decltype(MO)::value,
                                               decltype(BF)::value, DCASGD_FOLD_KC,
                                               decltype(NT)::value, false, true>),
                          grid, threads, s, hp, h->w, h->ms, a,
                          static_cast<const FoldWorkspace*>(nullptr), kept, n4, h->d);
            return;
          }
          with_bool(ordered, [&](auto OR) {
            DCASGD_LAUNCH(h, (sync_fold_kernel<decltype(AD)::value, decltype(MO)::value,
                                               decltype(BF)::value, DCASGD_FOLD_KC,
                                               decltype(NT)::value, decltype(OR)::value, false>),
                          grid, threads, s, hp, h->w, h->ms, a,
                          static_cast<const FoldWorkspace*>(ws),
                          static_cast<const float*>(nullptr), n4, h->d);
          });
        });
      });
     });
    });
    advance_counter(h, (uint32_t)J, s);
    h->stream = s;
    h->t += (uint64_t)J;
    return launched(h);
}

int dcasgd_sync_fold(dcasgd_t h, const void* const* grads, int J, float eta_hat, void* stream) {
    return fold_impl(h, grads, J, J, eta_hat, nullptr, false, nullptr, stream);
}

int dcasgd_grad_sqnorms(dcasgd_t h, const void* const* grads, int J, void* workspace,
                        void* stream) {
    return fold_impl(h, grads, J, J, 0.0f, static_cast<FoldWorkspace*>(workspace), true, nullptr,
                     stream, false);
}

int dcasgd_sync_fold_part(dcasgd_t h, const void* const* grads, int J, int J_total, float eta_hat,
                          const float* kept_w, void* stream) {
    if (h && !kept_w) return fail(h, DCASGD_EINVAL);
    return fold_impl(h, grads, J, J_total, eta_hat, nullptr, false, kept_w, stream);
}

int dcasgd_sync_fold_ordered(dcasgd_t h, const void* const* grads, int J, float eta_hat,
                             void* workspace, void* stream) {
    static_assert(sizeof(FoldWorkspace) == DCASGD_FOLD_WS_BYTES, "header and kernels agree");
    return fold_impl(h, grads, J, J, eta_hat, static_cast<FoldWorkspace*>(workspace), true, nullptr,
                     stream);
}

int dcasgd_sync_fold_ordered_static(dcasgd_t h, const void* const* grads, int J, float eta_hat,
                                    void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    // the scratch holds one workspace: room for DCASGD_MAX_K gradients, any d
    if (J > DCASGD_MAX_K) return fail(h, DCASGD_EINVAL);
    void* ws = scratch_on_current_device();
    if (!ws) return fail(h, DCASGD_EHIP);
    return fold_impl(h, grads, J, J, eta_hat, static_cast<FoldWorkspace*>(ws), true, nullptr,
                     stream, true, true);
}

const float* dcasgd_pull(dcasgd_t h, int worker) {
    if (!h) return nullptr;
    if (!h->ready) { fail(h, DCASGD_ESTATE); return nullptr; }
    if (worker < 0 || worker >= h->M) { fail(h, DCASGD_EINVAL); return nullptr; }
    const float* row = static_cast<const float*>(bak_row(h, worker));
    if (h->fresh_at[(size_t)worker] == h->t) return row;   // already equal to w
    launch_pull(h, worker, h->stream);
    h->fresh_at[(size_t)worker] = h->t;
    if (launched(h) != DCASGD_OK) return nullptr;
    return row;
}

uint64_t dcasgd_step(dcasgd_t h) { return h ? h->t : 0; }

int dcasgd_last_error(dcasgd_t h) { return h ? h->last_error : DCASGD_EINVAL; }

const char* dcasgd_strerror(int code) {
    switch (code) {
        case DCASGD_OK:     return "ok";
        case DCASGD_EINVAL: return "invalid argument";
        case DCASGD_EALIGN: return "pointer or stride not aligned";
        case DCASGD_ESTATE: return "handle not bound/initialised";
        case DCASGD_EHIP:   return "HIP runtime error at launch";
        default:            return "unknown status";
    }
}

int dcasgd_set_momentum(dcasgd_t h, float mu, float* vel, void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->bound) return fail(h, DCASGD_ESTATE);
    if (!std::isfinite(mu)) return fail(h, DCASGD_EINVAL);
    if (mu == 0.0f || !vel) {                 // plain update again
        h->hp.mu = 0.0f;
        h->hp.vel = nullptr;
        return DCASGD_OK;
    }
    if (!aligned(vel, 16)) return fail(h, DCASGD_EALIGN);
    const size_t vb = h->d * 4;
    if (overlaps(vel, vb, h->w, vb) ||
        overlaps(vel, vb, h->bak, bak_bytes(h)) ||
        (h->ms && overlaps(vel, vb, h->ms, vb)))
        return fail(h, DCASGD_EINVAL);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const size_t n4 = h->d / 4;
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(n4, 512, 4096)), dim3(512), 0, s, vel, 0.0f, n4,
                       h->d);
    h->hp.mu = mu;
    h->hp.vel = vel;
    return launched(h);
}

int dcasgd_bind_counter(dcasgd_t h, uint32_t* counter, void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    if (!counter) {
        h->ctr = nullptr;
        return DCASGD_OK;
    }
    if (!aligned(counter, 4)) return fail(h, DCASGD_EALIGN);
    const size_t vb = h->d * 4;
    if (overlaps(counter, 4, h->w, vb) ||
        overlaps(counter, 4, h->bak, bak_bytes(h)) ||
        (h->ms && overlaps(counter, 4, h->ms, vb)) ||
        (h->hp.vel && overlaps(counter, 4, h->hp.vel, vb)))
        return fail(h, DCASGD_EINVAL);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(counter_set_kernel, dim3(1), dim3(64), 0, s, counter, (uint32_t)h->t);
    h->ctr = counter;
    return launched(h);
}

int dcasgd_set_step(dcasgd_t h, uint64_t t) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    h->t = t;
    // which backups equal w is unknown after launches the host did not see
    h->fresh_at.assign((size_t)h->M, ~(uint64_t)0);
    return DCASGD_OK;
}

int dcasgd_worker_grad(dcasgd_t h, int worker, const float* hdiag, const float* wstar, float sigma,
                       uint64_t seed, uint32_t offset, void* grad_out, void* stream) {
    if (!h) return DCASGD_EINVAL;
    if (!h->ready) return fail(h, DCASGD_ESTATE);
    if (worker < 0 || worker >= h->M || !hdiag || !wstar || !std::isfinite(sigma))
        return fail(h, DCASGD_EINVAL);
    if (h->d > ((size_t)1 << 34) || h->t + offset > 0xFFFFFFFFull) return fail(h, DCASGD_EINVAL);
    if (int rc = check_grad(h, grad_out)) return fail(h, rc);
    if (!aligned(hdiag, 16) || !aligned(wstar, 16)) return fail(h, DCASGD_EALIGN);
    const size_t vb = h->d * 4, gb = grad_bytes(h);
    if (overlaps(grad_out, gb, hdiag, vb) || overlaps(grad_out, gb, wstar, vb))
        return fail(h, DCASGD_EINVAL);
    const void* snap = bak_row(h, worker);
    const size_t n4 = h->d / 4;
    const unsigned grid = grid_for(n4, 256, 0);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const uint32_t t_arg = h->ctr ? offset : (uint32_t)h->t + offset;
    hipStream_t s = static_cast<hipStream_t>(stream);
    with_bool(h->grad_bf16, [&](auto BF) {
      with_bool(h->bak_bf16, [&](auto BB) {
        with_bool(h->streaming >= 3, [&](auto SN) {
          hipLaunchKernelGGL((synth_grad_kernel<decltype(BF)::value, 1, decltype(BB)::value,
                                                decltype(SN)::value>),
                             dim3(grid), dim3(256), 0, s, snap, hdiag, wstar, sigma, k0, k1, t_arg,
                             static_cast<const uint32_t*>(h->ctr), grad_out, n4, h->d);
        });
      });
    });
    return launched(h);
}

int dcasgd_timing(dcasgd_t h, int enable) {
    if (!h) return DCASGD_EINVAL;
    // Unread pairs may still belong to launches in flight: wait for the last
    // one before its events are handed out again (launches on one handle are
    // issued in order, so the last stop event is the last to complete).
    if (h->timing_used >= 2 &&
        hipEventSynchronize(h->timing_events[h->timing_used - 1]) != hipSuccess)
        return fail(h, DCASGD_EHIP);
    h->timing = enable != 0;
    h->timing_used = 0;
    return DCASGD_OK;
}

int dcasgd_timing_read(dcasgd_t h, double* total_ms, uint64_t* launches) {
    if (!h) return DCASGD_EINVAL;
    if (!total_ms || !launches) return fail(h, DCASGD_EINVAL);
    double sum = 0.0;
    const size_t n = h->timing_used;
    if (n >= 2 && hipEventSynchronize(h->timing_events[n - 1]) != hipSuccess)
        return fail(h, DCASGD_EHIP);
    for (size_t i = 0; i + 1 < n; i += 2) {
        float ms = 0.0f;
        if (hipEventSynchronize(h->timing_events[i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, h->timing_events[i], h->timing_events[i + 1]) != hipSuccess)
            return fail(h, DCASGD_EHIP);
        sum += ms;
    }
    *total_ms = sum;
    *launches = n / 2;
    h->timing_used = 0;
    return DCASGD_OK;
}

int dcasgd_timing_read_each(dcasgd_t h, float* each_ms, size_t capacity, uint64_t* launches) {
    if (!h) return DCASGD_EINVAL;
    if (!launches || (capacity > 0 && !each_ms)) return fail(h, DCASGD_EINVAL);
    const size_t n = h->timing_used / 2;
    for (size_t i = 0; i < n; ++i) {
        float ms = 0.0f;
        if (hipEventSynchronize(h->timing_events[2 * i + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, h->timing_events[2 * i], h->timing_events[2 * i + 1]) !=
                hipSuccess)
            return fail(h, DCASGD_EHIP);
        if (i < capacity) each_ms[i] = ms;
    }
    *launches = n;
    h->timing_used = 0;
    return DCASGD_OK;
}

int dcasgd_set_eta(dcasgd_t h, float eta) {
    if (!h) return DCASGD_EINVAL;
    if (!std::isfinite(eta)) return fail(h, DCASGD_EINVAL);
    h->hp.eta = eta;       // passed by value with every launch: later pushes use it
    return DCASGD_OK;
}

int dcasgd_set_lambda(dcasgd_t h, float lambda0) {
    if (!h) return DCASGD_EINVAL;
    if (!std::isfinite(lambda0)) return fail(h, DCASGD_EINVAL);
    h->hp.lambda0 = lambda0;   // passed by value with every launch, like eta
    const float mag = std::fabs(lambda0);
    h->hp.lambda_midrange = (mag >= 0x1p-40f && mag <= 0x1p40f) ? 1 : 0;
    return DCASGD_OK;
}

int dcasgd_set_launch(dcasgd_t h, int threads, int items, int max_blocks, int streaming) {
    if (!h) return DCASGD_EINVAL;
    if (threads > 0 && !valid_threads(threads)) return fail(h, DCASGD_EINVAL);
    if (items > 0 && !valid_items(items)) return fail(h, DCASGD_EINVAL);
    if (max_blocks < 0 || streaming < 0 || streaming > 3) return fail(h, DCASGD_EINVAL);
    if (threads > 0) {
        h->threads = threads;
        h->batch_threads = threads > 256 ? 256 : threads;
    }
    if (items > 0) h->items = h->push_items = items;
    h->max_blocks = max_blocks;
    h->streaming = streaming;
    return DCASGD_OK;
}

int dcasgd_synth_grad(const void* snap, const float* hdiag, const float* wstar, float sigma,
                      uint64_t seed, uint32_t push_idx, void* grad_out, int formats, size_t d,
                      void* stream, int threads, int items) {
    if (formats & ~7) return DCASGD_EINVAL;
    const bool as_bf16 = (formats & 1) != 0, snap_bf16 = (formats & 2) != 0;
    const bool uncached = (formats & 4) != 0;
    if (!snap || !hdiag || !wstar || !grad_out || d == 0) return DCASGD_EINVAL;
    if (d > ((size_t)1 << 34)) return DCASGD_EINVAL;    // the counter holds i/4 in 32 bits
    if (!std::isfinite(sigma)) return DCASGD_EINVAL;
    if (threads <= 0) threads = 256;
    if (items <= 0) items = 1;
    if (!valid_threads(threads) || !valid_items(items)) return DCASGD_EINVAL;
    if (!aligned(snap, snap_bf16 ? 8 : 16) || !aligned(hdiag, 16) || !aligned(wstar, 16) ||
        !aligned(grad_out, as_bf16 ? 8 : 16))
        return DCASGD_EALIGN;
    const size_t ob = d * (as_bf16 ? 2 : 4);
    if (overlaps(grad_out, ob, snap, d * (snap_bf16 ? 2 : 4)) || overlaps(grad_out, ob, hdiag, d * 4) ||
        overlaps(grad_out, ob, wstar, d * 4))
        return DCASGD_EINVAL;
    const size_t n4 = d / 4;
    const unsigned grid = grid_for(n4, (size_t)threads * items, 0);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    hipStream_t s = static_cast<hipStream_t>(stream);
    with_bool(as_bf16, [&](auto BF) {
        with_items(items, [&](auto IT) {
          with_bool(snap_bf16, [&](auto BB) {
            with_bool(uncached, [&](auto SN) {
              hipLaunchKernelGGL((synth_grad_kernel<decltype(BF)::value, decltype(IT)::value,
                                                    decltype(BB)::value, decltype(SN)::value>),
                                 dim3(grid), dim3(threads), 0, s, snap, hdiag, wstar, sigma, k0, k1,
                                 push_idx, static_cast<const uint32_t*>(nullptr), grad_out, n4, d);
            });
          });
        });
    });
    return hipGetLastError() == hipSuccess ? DCASGD_OK : DCASGD_EHIP;
}

}  // extern "C"
