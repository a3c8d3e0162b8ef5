// Device code of the DC-ASGD server update for gfx950 (CDNA4, wave64).
//
// Everything here is elementwise streaming work: each parameter is read,
// updated and written once per push, with no reuse inside a launch.  The
// kernels are therefore built around 128-bit global loads and stores issued
// up front (ITEMS independent float4 groups per lane), non-temporal hints
// (gradients and backups are not touched again for a whole cycle of pushes;
// measured on MI355X, streaming loads and stores are also the faster choice
// for w and MeanSquare), and enough resident wavefronts to keep HBM busy.
// There is no LDS use and no MFMA: no operand is shared between lanes.
//
// Arithmetic contract (matches the header of the C ABI): binary32, one rounding
// per operation, no contraction, correctly rounded sqrt and division.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#pragma clang fp contract(off)

#ifndef DCASGD_SHORT_RADIUS
#define DCASGD_SHORT_RADIUS true    // false: the noise radius through the general sqrt and divide
#endif

namespace dcasgd {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t u16x4 __attribute__((ext_vector_type(4)));

struct Hyper {
    float eta;
    float lambda0;
    float ema_m;         // m of Eq. 18
    float one_minus_m;   // 1 - m, formed once on the host in binary32
    float eps;
    int lambda_midrange; // |lambda0| in [2^-40, 2^40]: the short sqrt/divide may be used
    float mu;            // momentum coefficient (used only when vel is set)
    float* vel;          // velocity vector, or nullptr: plain update
};

// ---- memory helpers ---------------------------------------------------------
template <bool NT>
__device__ __forceinline__ f32x4 load4(const float* base, size_t quad) {
    const f32x4* p = reinterpret_cast<const f32x4*>(base) + quad;
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}

template <bool NT>
__device__ __forceinline__ void store4(float* base, size_t quad, f32x4 v) {
    f32x4* p = reinterpret_cast<f32x4*>(base) + quad;
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

__device__ __forceinline__ float widen_bf16(uint16_t h) {
    return __uint_as_float(static_cast<uint32_t>(h) << 16);
}

// binary32 -> bfloat16 bits, round to nearest, ties to even (finite inputs)
__device__ __forceinline__ uint16_t narrow_bf16(float x) {
    const uint32_t b = __float_as_uint(x);
    return static_cast<uint16_t>((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

// Four gradient elements of group `quad`, float32 or bfloat16 in memory.
template <bool BF16, bool NT>
__device__ __forceinline__ f32x4 load_grad4(const void* grad, size_t quad) {
    if constexpr (BF16) {
        const u16x4* p = reinterpret_cast<const u16x4*>(grad) + quad;
        u16x4 r;
        if constexpr (NT) r = __builtin_nontemporal_load(p);
        else r = *p;
        f32x4 g;
        g.x = widen_bf16(r.x); g.y = widen_bf16(r.y);
        g.z = widen_bf16(r.z); g.w = widen_bf16(r.w);
        return g;
    } else {
        return load4<NT>(reinterpret_cast<const float*>(grad), quad);
    }
}

template <bool BF16>
__device__ __forceinline__ float load_grad1(const void* grad, size_t i) {
    if constexpr (BF16) return widen_bf16(reinterpret_cast<const uint16_t*>(grad)[i]);
    else return reinterpret_cast<const float*>(grad)[i];
}

// Backup rows hold binary32 or, with BB, bfloat16 snapshots: what a pull hands
// to the worker is round-to-nearest-even of w, and that same number is what
// the next push of that worker is compensated against.
template <bool BB, bool NT>
__device__ __forceinline__ f32x4 load_bak4(const void* bak, size_t quad) {
    return load_grad4<BB, NT>(bak, quad);
}
template <bool BB>
__device__ __forceinline__ float load_bak1(const void* bak, size_t i) {
    return load_grad1<BB>(bak, i);
}
template <bool BB, bool NT>
__device__ __forceinline__ void store_bak4(void* bak, size_t quad, f32x4 v) {
    if constexpr (BB) {
        u16x4 r;
        r.x = narrow_bf16(v.x); r.y = narrow_bf16(v.y);
        r.z = narrow_bf16(v.z); r.w = narrow_bf16(v.w);
        u16x4* p = reinterpret_cast<u16x4*>(bak) + quad;
        if constexpr (NT) __builtin_nontemporal_store(r, p);
        else *p = r;
    } else {
        store4<NT>(reinterpret_cast<float*>(bak), quad, v);
    }
}
template <bool BB>
__device__ __forceinline__ void store_bak1(void* bak, size_t i, float v) {
    if constexpr (BB) reinterpret_cast<uint16_t*>(bak)[i] = narrow_bf16(v);
    else reinterpret_cast<float*>(bak)[i] = v;
}

// Velocity of a float4 group.  MOM is a compile-time switch: the plain kernels
// carry no velocity registers and no extra traffic.
template <bool MOM>
__device__ __forceinline__ f32x4 load_vel4(const Hyper& hp, size_t quad) {
    if constexpr (MOM) return load4<true>(hp.vel, quad);
    else return f32x4{0.f, 0.f, 0.f, 0.f};
}
template <bool MOM>
__device__ __forceinline__ void store_vel4(const Hyper& hp, size_t quad, f32x4 v) {
    if constexpr (MOM) store4<true>(hp.vel, quad, v);
}
template <bool MOM>
__device__ __forceinline__ float load_vel1(const Hyper& hp, size_t i) {
    if constexpr (MOM) return hp.vel[i];
    else return 0.f;
}
template <bool MOM>
__device__ __forceinline__ void store_vel1(const Hyper& hp, size_t i, float v) {
    if constexpr (MOM) hp.vel[i] = v;
}

// w <- w - eta*gdc, or with momentum v <- mu*v + gdc; w <- w - eta*v.
template <bool MOM>
__device__ __forceinline__ void take_step(const Hyper& hp, float gdc, float& w, float& v) {
    float dir = gdc;
    if constexpr (MOM) {
        const float carried = hp.mu * v;
        v = carried + gdc;
        dir = v;
    }
    const float step = hp.eta * dir;
    w = w - step;
}

// ---- the update rule ----------------------------------------------------------
// Eq. 4.1 applied to one parameter; in the adaptive variant Eq. 18 refreshes
// MeanSquare first and lambda is lambda0 / sqrt(MeanSquare + eps).
template <bool ADAPTIVE, bool MOM>
__device__ __forceinline__ void apply_push(const Hyper& hp, float g, float b,
                                           float& w, float& ms, float& v) {
    const float gsq = g * g;
    float lam = hp.lambda0;
    if constexpr (ADAPTIVE) {
        const float keep = hp.ema_m * ms;
        const float add = hp.one_minus_m * gsq;
        ms = keep + add;
        const float under = ms + hp.eps;
        const float root = __builtin_sqrtf(under);
        lam = hp.lambda0 / root;
    }
    const float drift = w - b;            // how far the model moved since the pull
    const float curv = lam * gsq;         // diagonal Hessian estimate
    const float comp = curv * drift;
    const float gdc = g + comp;           // delay-compensated gradient
    take_step<MOM>(hp, gdc, w, v);
}

// lambda0 / sqrt(x) as two correctly rounded operations, without the exponent
// rescaling and special-value fix-ups of the general expansions.  While
// operands and results stay far from both ends of the exponent range the
// rescaling is the identity, so these give the same bits in ten instructions
// instead of about thirty, and with ONE transcendental (half-rate)
// instruction: the hardware estimate y of 1/sqrt(x) serves both steps.
// Root: s = x*y (within a few ulps of sqrt(x)), its exact residual x - s*s,
// and one Newton step with h = y/2.
// Quotient: the same y, within two ulps of 1/root, is sharpened by one Newton
// step and seeds a*y; one residual correction follows.  (With the
// unsharpened y and two corrections about two quotients in a billion come
// out one ulp off.)
// Both are checked against the IEEE operations by the stand-alone checker next
// to this file: every admitted radicand for the root; every pair of root and
// numerator significands, 1.4e14 cases, for the quotient; no mismatch.
__device__ __forceinline__ float root_rn_midrange(float x, float& y) {
    y = __builtin_amdgcn_rsqf(x);
    const float s = x * y;
    const float h = 0.5f * y;
    const float r = __builtin_fmaf(-s, s, x);
    return __builtin_fmaf(r, h, s);
}

// a / b for b = root_rn_midrange(x, y)
__device__ __forceinline__ float quotient_rn_midrange(float a, float b, float y) {
    const float e = __builtin_fmaf(-b, y, 1.0f);
    y = __builtin_fmaf(e, y, y);
    const float q = a * y;
    const float r = __builtin_fmaf(-b, q, a);
    return __builtin_fmaf(r, y, q);
}

// Radicands the short forms are used for: 2^-64 <= x < 2^64 (so not zero,
// denormal, negative, inf or NaN), except the two per pair of binades whose
// root has an all-ones significand (significand 0x7FFFFE or 0x7FFFFF with an
// even exponent field).  That root is the classical exception of division by
// iteration: 1/root lies a hair above the midpoint of two neighbours, a
// reciprocal sharpened by Newton steps still rounds to the lower one, and for
// a power-of-two numerator the corrected quotient lands exactly on the
// midpoint.  Those radicands take the general expansion instead.
__device__ __forceinline__ bool in_midrange(float x) {
    const uint32_t u = __float_as_uint(x);
    return (u - 0x1F800000u) < 0x40000000u && (u & 0x00FFFFFEu) != 0x007FFFFEu;
}

// in_midrange for four radicands at once, with the four answers folded by
// integer max/min instead of four compares each.  The range test needs no
// subtraction: as unsigned words, every admitted radicand lies in
// [0x1F800000, 0x5F800000) and every other one (zero, denormal, negative, inf,
// NaN) outside, so the smallest and the largest word decide.  The significand
// patterns are hit iff (word + 0x00800002) << 8 is 0 or 0x100 (the low 24 bits
// wrap to 0 and 1 exactly for 0x7FFFFE and 0x7FFFFF; one add-shift
// instruction), so the smallest of those four decides.
__device__ __forceinline__ bool quad_in_midrange(const float (&x)[4]) {
    uint32_t u[4], pat[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        u[c] = __float_as_uint(x[c]);
        pat[c] = (u[c] + 0x00800002u) << 8;
    }
    const uint32_t top = max(max(u[0], u[1]), max(u[2], u[3]));
    const uint32_t bottom = min(min(u[0], u[1]), min(u[2], u[3]));
    const uint32_t near = min(min(pat[0], pat[1]), min(pat[2], pat[3]));
    return bottom >= 0x1F800000u && top < 0x5F800000u && near > 0x100u;
}

// The wave-wide vote the kernels take: true iff every active lane's four
// radicands are admitted.  Same three tests as quad_in_midrange, each voted on
// its own so that the compare results are joined as wave masks on the scalar
// side and no per-lane boolean has to be materialised.
__device__ __forceinline__ bool wave_all_in_midrange(const float (&x)[4]) {
    uint32_t u[4], pat[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        u[c] = __float_as_uint(x[c]);
        pat[c] = (u[c] + 0x00800002u) << 8;
    }
    const uint32_t top = max(max(u[0], u[1]), max(u[2], u[3]));
    const uint32_t bottom = min(min(u[0], u[1]), min(u[2], u[3]));
    const uint32_t near = min(min(pat[0], pat[1]), min(pat[2], pat[3]));
    const uint64_t low = __builtin_amdgcn_ballot_w64(bottom < 0x1F800000u);
    const uint64_t high = __builtin_amdgcn_ballot_w64(top >= 0x5F800000u);
    const uint64_t hit = __builtin_amdgcn_ballot_w64(near <= 0x100u);
    return (low | high | hit) == 0;
}

// Four parameters at once.  The adaptive lambda needs sqrt and a divide per
// parameter; when every lane of the wave has all four radicands in the middle
// of the exponent range (any realistic MeanSquare + eps) the short forms above
// are used, otherwise the general ones: the result is the same bits either way.
template <bool ADAPTIVE, bool MOM>
__device__ __forceinline__ void apply_push4(const Hyper& hp, const f32x4& g, const f32x4& b,
                                            f32x4& w, f32x4& ms, f32x4& v) {
    if constexpr (!ADAPTIVE) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            float wc = w[c], mc = ms[c], vc = v[c];
            apply_push<false, MOM>(hp, g[c], b[c], wc, mc, vc);
            w[c] = wc;
            v[c] = vc;
        }
    } else {
        float gsq[4], under[4], lam[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            gsq[c] = g[c] * g[c];
            const float keep = hp.ema_m * ms[c];
            const float add = hp.one_minus_m * gsq[c];
            ms[c] = keep + add;
            under[c] = ms[c] + hp.eps;
        }
        if (wave_all_in_midrange(under) && hp.lambda_midrange != 0) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                float y;
                const float root = root_rn_midrange(under[c], y);
                lam[c] = quotient_rn_midrange(hp.lambda0, root, y);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c) lam[c] = hp.lambda0 / __builtin_sqrtf(under[c]);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const float drift = w[c] - b[c];
            const float curv = lam[c] * gsq[c];
            const float comp = curv * drift;
            const float gdc = g[c] + comp;
            float wc = w[c], vc = v[c];
            take_step<MOM>(hp, gdc, wc, vc);
            w[c] = wc;
            v[c] = vc;
        }
    }
}

// Which float4 group of a tile a lane handles in its j-th access: lane l touches
// groups l, l + blockDim.x, ..., so a wave-wide access is one contiguous 1 KiB
// run and a block covers a contiguous tile.  (Making the ITEMS runs of a wave
// adjacent - a wave walking ITEMS KiB of every stream - measured the same at
// 100 MB vectors and 3 % slower at 550 MB ones.)
template <int ITEMS>
__device__ __forceinline__ size_t tile_quad(size_t tile_first, int j) {
    return tile_first + (size_t)j * blockDim.x + threadIdx.x;
}

// ---- push (optionally fused with the pusher's pull) ----------------------------
// Work is cut into tiles of blockDim.x * ITEMS float4 groups; which groups a
// lane touches is tile_quad's choice; every wave-wide access is one contiguous
// 1 KiB run.  Blocks walk tiles with stride gridDim.x.
// NT: 0 = plain accesses, 1 = gradient and backup traffic non-temporal,
// 2 = w and MeanSquare non-temporal as well (state too large to be re-read
// from any cache before the next push).  (Level 3 of the launch settings is
// level 2 here plus a worker kernel that leaves nothing cached either.)
template <bool ADAPTIVE, bool MOM, bool BF16, bool PULL, int ITEMS, int NT, bool BB, bool CHECKED>
__device__ __forceinline__ void push_tile(const Hyper& hp, float* __restrict__ w,
                                          float* __restrict__ ms, void* __restrict__ bak,
                                          const void* __restrict__ grad, size_t first,
                                          size_t n4) {
    f32x4 W[ITEMS], B[ITEMS], G[ITEMS], S[ITEMS], V[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const size_t q = tile_quad<ITEMS>(first, j);
        if (!CHECKED || q < n4) {
            V[j] = load_vel4<MOM>(hp, q);
            G[j] = load_grad4<BF16, (NT >= 1)>(grad, q);
            B[j] = load_bak4<BB, (NT >= 1)>(bak, q);
            W[j] = load4<(NT >= 2)>(w, q);
            if constexpr (ADAPTIVE) S[j] = load4<(NT >= 2)>(ms, q);
            else S[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        } else {
            G[j] = B[j] = W[j] = S[j] = V[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const size_t q = tile_quad<ITEMS>(first, j);
        apply_push4<ADAPTIVE, MOM>(hp, G[j], B[j], W[j], S[j], V[j]);
        if (!CHECKED || q < n4) {
            store_vel4<MOM>(hp, q, V[j]);
            store4<(NT >= 2)>(w, q, W[j]);
            if constexpr (ADAPTIVE) store4<(NT >= 2)>(ms, q, S[j]);
            if constexpr (PULL) store_bak4<BB, (NT >= 1)>(bak, q, W[j]);
        }
    }
}

template <bool ADAPTIVE, bool MOM, bool BF16, bool PULL, int ITEMS, int NT, bool BB>
__global__ void __launch_bounds__(512)
push_kernel(Hyper hp, float* __restrict__ w, float* __restrict__ ms, void* __restrict__ bak,
            const void* __restrict__ grad, size_t n4, size_t d) {
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t first = tile * tile_quads;            // first group of the tile
        if ((tile + 1) * tile_quads <= n4)
            push_tile<ADAPTIVE, MOM, BF16, PULL, ITEMS, NT, BB, false>(hp, w, ms, bak, grad, first, n4);
        else
            push_tile<ADAPTIVE, MOM, BF16, PULL, ITEMS, NT, BB, true>(hp, w, ms, bak, grad, first, n4);
    }
    // up to three parameters beyond the last full group of four
    if (blockIdx.x == 0) {
        const size_t i = 4 * n4 + threadIdx.x;
        if (i < d) {
            float wi = w[i];
            float si = 0.f;
            if constexpr (ADAPTIVE) si = ms[i];
            float vi = load_vel1<MOM>(hp, i);
            apply_push<ADAPTIVE, MOM>(hp, load_grad1<BF16>(grad, i), load_bak1<BB>(bak, i), wi, si, vi);
            w[i] = wi;
            if constexpr (ADAPTIVE) ms[i] = si;
            if constexpr (PULL) store_bak1<BB>(bak, i, wi);
            store_vel1<MOM>(hp, i, vi);
        }
    }
}

// ---- K queued pushes in one pass (push; pull; push; pull; ...) -------------------
struct BatchArgs {
    const void* grad[16];   // grad[k]: gradient of queue entry k
    void* bak[16];          // bak[k]: backup row of the worker of entry k (all distinct)
    int K;
};

// w and ms stay in registers across the queue; entry k reads its gradient and
// its worker's backup, updates, and overwrites that backup with the new w.
// Entries are taken in groups: all 2*GROUP loads of a group are issued before
// its first update, so a full queue of 16 has 32 128-bit loads in flight per
// lane from the start (measured on MI355X: 897 us per queue of 16 at 25.6 M
// parameters against 914 us for groups of four with the next group's loads
// issued ahead, 919 us for plain groups of eight).  Shorter queues fall
// through to groups of 8, 4, 2, 1.
template <bool BF16, int GROUP, bool NT, bool BB>
__device__ __forceinline__ void batch_load(const BatchArgs& a, int k0, size_t q,
                                           f32x4 (&G)[GROUP], f32x4 (&B)[GROUP]) {
#pragma unroll
    for (int kk = 0; kk < GROUP; ++kk) {
        G[kk] = load_grad4<BF16, NT>(a.grad[k0 + kk], q);
        B[kk] = load_bak4<BB, NT>(a.bak[k0 + kk], q);
    }
}

template <bool ADAPTIVE, bool MOM, bool BF16, int GROUP, bool NT, bool BB>
__device__ __forceinline__ void batch_group(const Hyper& hp, const BatchArgs& a, int k0, size_t q,
                                            f32x4& W, f32x4& S, f32x4& V) {
    f32x4 G[GROUP], B[GROUP];
    batch_load<BF16, GROUP, NT, BB>(a, k0, q, G, B);
#pragma unroll
    for (int kk = 0; kk < GROUP; ++kk) {
        apply_push4<ADAPTIVE, MOM>(hp, G[kk], B[kk], W, S, V);
        store_bak4<BB, NT>(a.bak[k0 + kk], q, W);
    }
}

template <bool ADAPTIVE, bool MOM, bool BF16, int KC, bool NT, bool BB, bool CHECKED>
__device__ __forceinline__ void batch_quad(const Hyper& hp, float* __restrict__ w,
                                           float* __restrict__ ms, const BatchArgs& a,
                                           size_t q, size_t n4) {
    if (CHECKED && q >= n4) return;
    f32x4 W = load4<false>(w, q);
    f32x4 S = f32x4{0.f, 0.f, 0.f, 0.f};
    if constexpr (ADAPTIVE) S = load4<false>(ms, q);
    f32x4 V = load_vel4<MOM>(hp, q);
    int k = 0;
    for (; a.K - k >= KC; k += KC) batch_group<ADAPTIVE, MOM, BF16, KC, NT, BB>(hp, a, k, q, W, S, V);
    if constexpr (KC > 8)
        if (a.K - k >= 8) { batch_group<ADAPTIVE, MOM, BF16, 8, NT, BB>(hp, a, k, q, W, S, V); k += 8; }
    if constexpr (KC > 4)
        if (a.K - k >= 4) { batch_group<ADAPTIVE, MOM, BF16, 4, NT, BB>(hp, a, k, q, W, S, V); k += 4; }
    if constexpr (KC > 2)
        if (a.K - k >= 2) { batch_group<ADAPTIVE, MOM, BF16, 2, NT, BB>(hp, a, k, q, W, S, V); k += 2; }
    if constexpr (KC > 1)
        if (a.K - k >= 1) { batch_group<ADAPTIVE, MOM, BF16, 1, NT, BB>(hp, a, k, q, W, S, V); k += 1; }
    store4<false>(w, q, W);
    if constexpr (ADAPTIVE) store4<false>(ms, q, S);
    store_vel4<MOM>(hp, q, V);
}

template <bool ADAPTIVE, bool MOM, bool BF16, int KC, bool NT, bool BB>
__global__ void __launch_bounds__(256)
push_batch_kernel(Hyper hp, float* __restrict__ w, float* __restrict__ ms, BatchArgs a,
                  size_t n4, size_t d) {
    const size_t ntiles = (n4 + blockDim.x - 1) / blockDim.x;
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t q = tile * blockDim.x + threadIdx.x;
        if ((tile + 1) * blockDim.x <= n4)
            batch_quad<ADAPTIVE, MOM, BF16, KC, NT, BB, false>(hp, w, ms, a, q, n4);
        else
            batch_quad<ADAPTIVE, MOM, BF16, KC, NT, BB, true>(hp, w, ms, a, q, n4);
    }
    if (blockIdx.x == 0) {
        const size_t i = 4 * n4 + threadIdx.x;
        if (i < d) {
            float wi = w[i];
            float si = 0.f;
            if constexpr (ADAPTIVE) si = ms[i];
            float vi = load_vel1<MOM>(hp, i);
            for (int k = 0; k < a.K; ++k) {
                apply_push<ADAPTIVE, MOM>(hp, load_grad1<BF16>(a.grad[k], i),
                                          load_bak1<BB>(a.bak[k], i), wi, si, vi);
                store_bak1<BB>(a.bak[k], i, wi);
            }
            w[i] = wi;
            if constexpr (ADAPTIVE) ms[i] = si;
            store_vel1<MOM>(hp, i, vi);
        }
    }
}

// ---- synchronous delay-compensated fold (supplement, large mini-batch SSGD) ------
// J gradients taken at the same model w_t are applied one after the other;
// entry j is compensated for the distance the running model has moved from
// w_t.  Per parameter w_t is simply the value loaded on entry, so it stays in
// a register: the only traffic is w, MeanSquare and the J gradients.  hp.eta
// holds the per-gradient step eta_hat / J.
struct FoldArgs {
    const void* grad[16];
    int J;
};

// Workspace of the ordered fold (device memory, caller-owned).  The first
// launch leaves one partial sum of squares per block and gradient in
// `partial`; the second adds them up in a fixed order (so the result does not
// depend on scheduling), ranks the gradients and leaves the squared norms, the
// permutation and the gradient pointers in fold order.
constexpr int FOLD_WS_BLOCKS = 2048;
struct FoldWorkspace {
    double sqnorm[16];          // |g_j|^2 in the caller's numbering
    int perm[16];               // perm[r] = caller's index of the r-th gradient folded
    int reserved0[16];
    const void* ordered[16];    // grad[perm[r]]
    double reserved1[16];
    double partial[16][FOLD_WS_BLOCKS];
};
static_assert(sizeof(FoldWorkspace) == 512 + 16 * FOLD_WS_BLOCKS * 8, "documented layout");

// gp: the J gradient pointers in fold order, either the launch arguments
// themselves or the list the ordering kernel left in device memory.
// kept: w_t of a fold that is delivered in parts (the caller's copy), or nullptr
// when the fold starts here and w_t is simply the value of w on entry.
template <bool ADAPTIVE, bool MOM, bool BF16, int KC, bool NT, bool ANCH, bool CHECKED>
__device__ __forceinline__ void fold_quad(const Hyper& hp, float* __restrict__ w,
                                          float* __restrict__ ms, const void* const* gp, int J,
                                          const float* __restrict__ kept, size_t q, size_t n4) {
    if (CHECKED && q >= n4) return;
    f32x4 W = load4<false>(w, q);
    f32x4 anchor = W;
    if constexpr (ANCH) anchor = load4<NT>(kept, q);
    f32x4 S = f32x4{0.f, 0.f, 0.f, 0.f};
    if constexpr (ADAPTIVE) S = load4<false>(ms, q);
    f32x4 V = load_vel4<MOM>(hp, q);
    // groups of KC gradients, the next group's loads issued before this group is worked on
    const int full = (J / KC) * KC;
    f32x4 G[KC], N[KC];
    if (full > 0) {
#pragma unroll
        for (int jj = 0; jj < KC; ++jj) G[jj] = load_grad4<BF16, NT>(gp[jj], q);
    }
    for (int j0 = 0; j0 < full; j0 += KC) {
        if (j0 + KC < full) {
#pragma unroll
            for (int jj = 0; jj < KC; ++jj) N[jj] = load_grad4<BF16, NT>(gp[j0 + KC + jj], q);
        }
#pragma unroll
        for (int jj = 0; jj < KC; ++jj) apply_push4<ADAPTIVE, MOM>(hp, G[jj], anchor, W, S, V);
#pragma unroll
        for (int jj = 0; jj < KC; ++jj) G[jj] = N[jj];
    }
    for (int j = full; j < J; ++j) {
        const f32x4 g = load_grad4<BF16, NT>(gp[j], q);
        apply_push4<ADAPTIVE, MOM>(hp, g, anchor, W, S, V);
    }
    store4<false>(w, q, W);
    if constexpr (ADAPTIVE) store4<false>(ms, q, S);
    store_vel4<MOM>(hp, q, V);
}

template <bool ADAPTIVE, bool MOM, bool BF16, int KC, bool NT, bool ORD, bool ANCH>
__global__ void __launch_bounds__(256)
sync_fold_kernel(Hyper hp, float* __restrict__ w, float* __restrict__ ms, FoldArgs a,
                 const FoldWorkspace* __restrict__ ws, const float* __restrict__ kept, size_t n4,
                 size_t d) {
    const void* const* gp = a.grad;
    if constexpr (ORD) gp = ws->ordered;
    const size_t ntiles = (n4 + blockDim.x - 1) / blockDim.x;
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t q = tile * blockDim.x + threadIdx.x;
        if ((tile + 1) * blockDim.x <= n4)
            fold_quad<ADAPTIVE, MOM, BF16, KC, NT, ANCH, false>(hp, w, ms, gp, a.J, kept, q, n4);
        else
            fold_quad<ADAPTIVE, MOM, BF16, KC, NT, ANCH, true>(hp, w, ms, gp, a.J, kept, q, n4);
    }
    if (blockIdx.x == 0) {
        const size_t i = 4 * n4 + threadIdx.x;
        if (i < d) {
            float wi = w[i];
            float anchor = wi;
            if constexpr (ANCH) anchor = kept[i];
            float si = 0.f;
            if constexpr (ADAPTIVE) si = ms[i];
            float vi = load_vel1<MOM>(hp, i);
            for (int j = 0; j < a.J; ++j)
                apply_push<ADAPTIVE, MOM>(hp, load_grad1<BF16>(gp[j], i), anchor, wi, si, vi);
            w[i] = wi;
            if constexpr (ADAPTIVE) ms[i] = si;
            store_vel1<MOM>(hp, i, vi);
        }
    }
}

// ---- fold order (supplement: fold in increasing distance from w_t) ----------------
// Distance read as the gradient's own norm.  First launch: the gradients are
// walked one after the other, so that at any moment the whole chip streams
// through one contiguous vector; a lane keeps one binary64 accumulator (the
// square of a binary32 value is exact in binary64, so the only roundings are
// those of the additions) and has ITEMS tiles in flight.  After each gradient
// the wave adds up its lanes; at the end the block adds up its waves and
// writes its J partial sums.  Every step has a fixed order.  Pure read
// traffic: J gradients, once.
template <bool BF16, bool NT, int ITEMS>
__device__ __forceinline__ double lane_sum_of_squares(const void* __restrict__ g, size_t n4) {
    double s = 0.0;
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t first = tile * tile_quads + threadIdx.x;
        f32x4 G[ITEMS];
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const size_t q = first + (size_t)k * blockDim.x;
            G[k] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (q < n4) G[k] = load_grad4<BF16, NT>(g, q);
        }
#pragma unroll
        for (int k = 0; k < ITEMS; ++k) {
            const double x = (double)G[k].x, y = (double)G[k].y;
            const double z = (double)G[k].z, u = (double)G[k].w;
            s = __builtin_fma(x, x, s);
            s = __builtin_fma(y, y, s);
            s = __builtin_fma(z, z, s);
            s = __builtin_fma(u, u, s);
        }
    }
    return s;
}

template <bool BF16, bool NT, int ITEMS>
__global__ void __launch_bounds__(256)
grad_sqnorm_kernel(FoldArgs a, FoldWorkspace* __restrict__ ws, size_t n4, size_t d) {
    __shared__ double wave_sum[4][16];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int j = 0; j < a.J; ++j) {
        const void* g = a.grad[j];
        double s = lane_sum_of_squares<BF16, NT, ITEMS>(g, n4);
        if (blockIdx.x == 0) {
            const size_t i = 4 * n4 + threadIdx.x;
            if (i < d) {
                const double x = (double)load_grad1<BF16>(g, i);
                s = __builtin_fma(x, x, s);
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
        if (lane == 0) wave_sum[wave][j] = s;
    }
    __syncthreads();
    if ((int)threadIdx.x < a.J) {
        double s = wave_sum[0][threadIdx.x];
        for (int v = 1; v < (int)(blockDim.x >> 6); ++v) s += wave_sum[v][threadIdx.x];
        ws->partial[threadIdx.x][blockIdx.x] = s;
    }
}

// Second launch, one block of 16 waves: wave j adds the per-block partial sums
// of gradient j (lane l takes blocks l, l+64, ... in that order, then the
// lanes are added up), after which the gradients are ranked by (squared norm,
// index) with a NaN counted as +infinity, so that the ranks always form a
// permutation; rank r receives caller's index perm[r] and its pointer.
__global__ void __launch_bounds__(1024)
fold_order_kernel(FoldArgs a, FoldWorkspace* __restrict__ ws, int nblocks) {
    __shared__ double key[16];
    const int lane = threadIdx.x & 63, j = threadIdx.x >> 6;
    if (j < a.J) {
        double s = 0.0;
        for (int b = lane; b < nblocks; b += 64) s += ws->partial[j][b];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
        if (lane == 0) {
            ws->sqnorm[j] = s;
            key[j] = (s != s) ? __builtin_huge_val() : s;
        }
    }
    __syncthreads();
    const int t = threadIdx.x;
    if (t < a.J) {
        const double mine = key[t];
        int rank = 0;
        for (int k = 0; k < a.J; ++k) {
            const double other = key[k];
            rank += (other < mine || (other == mine && k < t)) ? 1 : 0;
        }
        ws->perm[rank] = t;
        ws->ordered[rank] = a.grad[t];
    }
}

// ---- pull: w_bak(m) <- w ---------------------------------------------------------
template <int ITEMS, bool NT, bool BB>
__global__ void __launch_bounds__(512)
pull_kernel(const float* __restrict__ w, void* __restrict__ bak, size_t n4, size_t d) {
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t first = tile * tile_quads + threadIdx.x;
        f32x4 V[ITEMS];
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const size_t q = first + (size_t)j * blockDim.x;
            if (q < n4) V[j] = load4<false>(w, q);
        }
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const size_t q = first + (size_t)j * blockDim.x;
            if (q < n4) store_bak4<BB, NT>(bak, q, V[j]);
        }
    }
    if (blockIdx.x == 0) {
        const size_t i = 4 * n4 + threadIdx.x;
        if (i < d) store_bak1<BB>(bak, i, w[i]);
    }
}

// ---- fill (MeanSquare <- 0 at initialisation) -----------------------------------
__global__ void __launch_bounds__(512)
fill_kernel(float* __restrict__ dst, float value, size_t n4, size_t d) {
    const f32x4 v = f32x4{value, value, value, value};
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < n4;
         q += (size_t)gridDim.x * blockDim.x)
        store4<false>(dst, q, v);
    if (blockIdx.x == 0) {
        const size_t i = 4 * n4 + threadIdx.x;
        if (i < d) dst[i] = value;
    }
}

// ---- synthetic worker: counter-based noise ------------------------------------
// Philox4x32 with ten rounds (Salmon et al., SC'11): each round multiplies
// words 0 and 2 by fixed odd constants, mixes the high halves with the other
// two words and the round key, and the key advances by a Weyl step.
struct Words4 { uint32_t a, b, c, d; };

__device__ __forceinline__ Words4 philox10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                           uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p02 = (uint64_t)c0 * 0xD2511F53ull;
        const uint64_t p20 = (uint64_t)c2 * 0xCD9E8D57ull;
        const uint32_t y0 = (uint32_t)(p20 >> 32) ^ c1 ^ k0;
        const uint32_t y2 = (uint32_t)(p02 >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)p20;
        c3 = (uint32_t)p02;
        c0 = y0;
        c2 = y2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Words4{c0, c1, c2, c3};
}

// sqrt(-2 ln u) for u = ((word >> 8) + 1) / 2^24, with ln through the atanh
// series on the mantissa folded into (sqrt(1/2), sqrt(2)].  The definition
// asks for a correctly rounded division and square root.  SHORT = false takes
// the compiler's general expansions (exponent rescaling, special values: 11
// and 15 instructions).  SHORT = true takes six and seven: the operands of
// this function are confined - the divisor lies in (1.7, 2.42), the radicand
// is zero or lies in [2^-23, 34) - so a reciprocal or reciprocal-square-root
// estimate, one Newton step and one residual correction suffice, and since
// the function has only 2^24 distinct inputs the claim "same bits" is checked
// on every one of them (lambda_check radius).
template <bool SHORT>
__device__ __forceinline__ float radius_from_word_as(uint32_t word) {
    const float u = (float)((word >> 8) + 1u) * 0x1p-24f;
    const uint32_t ub = __float_as_uint(u);
    int ex = (int)(ub >> 23) - 127;
    float mant = __uint_as_float((ub & 0x007FFFFFu) | 0x3F800000u);
    const bool fold = mant > 1.41421354f;
    const float halved = mant * 0.5f;
    mant = fold ? halved : mant;
    ex = fold ? ex + 1 : ex;
    const float num = mant - 1.0f;
    const float den = mant + 1.0f;
    float s;
    if constexpr (SHORT) {
        float y = __builtin_amdgcn_rcpf(den);
        const float e = __builtin_fmaf(-den, y, 1.0f);
        y = __builtin_fmaf(e, y, y);
        const float q = num * y;
        const float r = __builtin_fmaf(-den, q, num);
        s = __builtin_fmaf(r, y, q);
    } else {
        s = num / den;
    }
    const float ss = s * s;
    float acc = 0.11111111f;
    acc = acc * ss; acc = acc + 0.14285715f;
    acc = acc * ss; acc = acc + 0.2f;
    acc = acc * ss; acc = acc + 0.33333334f;
    acc = acc * ss; acc = acc + 1.0f;
    const float s2x = 2.0f * s;
    const float lnm = s2x * acc;
    const float lne = (float)ex * 0.69314718f;
    const float lnu = lne + lnm;
    const float arg = -2.0f * lnu;
    if constexpr (SHORT) {
        const float y = __builtin_amdgcn_rsqf(arg);
        const float t = arg * y;
        const float h = 0.5f * y;
        const float r = __builtin_fmaf(-t, t, arg);
        const float root = __builtin_fmaf(r, h, t);
        return arg == 0.0f ? arg : root;      // u = 1: the radicand is -0, and so is its root
    } else {
        return __builtin_sqrtf(arg);
    }
}
__device__ __forceinline__ float radius_from_word(uint32_t word) {
    return radius_from_word_as<DCASGD_SHORT_RADIUS>(word);
}

// (cos, sin) of 2*pi*j/2^24, j = word >> 8: fold to [0, pi/4], Taylor
// polynomials, then undo the fold by octant.
__device__ __forceinline__ void circle_from_word(uint32_t word, float& co, float& si) {
    const uint32_t j = word >> 8;
    const uint32_t quad = j >> 22;
    const uint32_t frac = j & 0x3FFFFFu;
    const bool mirror = frac > 0x200000u;
    const uint32_t folded = mirror ? 0x400000u - frac : frac;
    const float x = (float)folded * 0x1.921fb6p-22f;
    const float xx = x * x;
    float ps = 2.7557319e-6f;
    ps = ps * xx; ps = ps - 1.9841270e-4f;
    ps = ps * xx; ps = ps + 8.3333333e-3f;
    ps = ps * xx; ps = ps - 0.16666667f;
    ps = ps * xx; ps = ps + 1.0f;
    const float sin_x = x * ps;
    float pc = -2.7557319e-7f;
    pc = pc * xx; pc = pc + 2.4801587e-5f;
    pc = pc * xx; pc = pc - 1.3888889e-3f;
    pc = pc * xx; pc = pc + 4.1666668e-2f;
    pc = pc * xx; pc = pc - 0.5f;
    pc = pc * xx;
    const float cos_x = pc + 1.0f;
    const float sa = mirror ? cos_x : sin_x;   // sine of the first-quadrant angle
    const float ca = mirror ? sin_x : cos_x;
    // rotate by quad * 90 degrees
    const float c_even = (quad & 2u) ? -ca : ca;
    const float s_even = (quad & 2u) ? -sa : sa;
    const float c_odd = (quad & 2u) ? sa : -sa;
    const float s_odd = (quad & 2u) ? -ca : ca;
    co = (quad & 1u) ? c_odd : c_even;
    si = (quad & 1u) ? s_odd : s_even;
}

__device__ __forceinline__ f32x4 normals_for_quad(uint32_t k0, uint32_t k1, uint32_t t,
                                                  uint32_t quad_index) {
    const Words4 x = philox10(quad_index, t, 0u, 0u, k0, k1);
    float c, s;
    f32x4 z;
    const float r0 = radius_from_word(x.a);
    circle_from_word(x.b, c, s);
    z.x = r0 * c; z.y = r0 * s;
    const float r1 = radius_from_word(x.c);
    circle_from_word(x.d, c, s);
    z.z = r1 * c; z.w = r1 * s;
    return z;
}

__device__ __forceinline__ float synth_one(float snap, float h, float wstar, float sigma, float z) {
    const float off = snap - wstar;
    const float pull_back = h * off;
    const float noise = sigma * z;
    return pull_back + noise;
}

// The push index that keys the noise: a launch argument, or - when the server
// keeps its push counter in device memory - that counter plus the argument,
// read when the kernel runs, so a captured launch sequence can be replayed
// and still draws fresh noise.
__device__ __forceinline__ uint32_t push_index(uint32_t t_arg, const uint32_t* ctr) {
    return ctr ? *ctr + t_arg : t_arg;
}

// The device-side push counter: set, and advance after pushes (one lane).
__global__ void counter_set_kernel(uint32_t* ctr, uint32_t value) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *ctr = value;
}
__global__ void counter_add_kernel(uint32_t* ctr, uint32_t n) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *ctr = *ctr + n;
}

// g = h * (snap - wstar) + sigma * z, four parameters per Philox counter.
// SNT: snapshot read and gradient write non-temporal as well, so that the
// launch leaves nothing behind in the last-level cache for the push that
// follows (the default keeps both cacheable on purpose, see below).
template <bool BF16, int ITEMS, bool BB, bool SNT>
__global__ void __launch_bounds__(512)
synth_grad_kernel(const void* __restrict__ snap, const float* __restrict__ hdiag,
                  const float* __restrict__ wstar, float sigma, uint32_t k0, uint32_t k1,
                  uint32_t t_arg, const uint32_t* __restrict__ ctr, void* __restrict__ out,
                  size_t n4, size_t d) {
    const uint32_t t = push_index(t_arg, ctr);
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t first = tile * tile_quads + threadIdx.x;
        f32x4 A[ITEMS], H[ITEMS], O[ITEMS];
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const size_t q = first + (size_t)j * blockDim.x;
            if (q < n4) {
                // the snapshot is read again by the push that follows: leave it
                // cacheable; the loss vectors stream through once per arrival
                A[j] = load_bak4<BB, SNT>(snap, q);
                H[j] = load4<true>(hdiag, q);
                O[j] = load4<true>(wstar, q);
            } else {
                A[j] = H[j] = O[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
#pragma unroll
        for (int j = 0; j < ITEMS; ++j) {
            const size_t q = first + (size_t)j * blockDim.x;
            if (q < n4) {
                const f32x4 z = normals_for_quad(k0, k1, t, (uint32_t)q);
                f32x4 g;
                g.x = synth_one(A[j].x, H[j].x, O[j].x, sigma, z.x);
                g.y = synth_one(A[j].y, H[j].y, O[j].y, sigma, z.y);
                g.z = synth_one(A[j].z, H[j].z, O[j].z, sigma, z.z);
                g.w = synth_one(A[j].w, H[j].w, O[j].w, sigma, z.w);
                if constexpr (BF16) {
                    u16x4 pk;
                    pk.x = narrow_bf16(g.x); pk.y = narrow_bf16(g.y);
                    pk.z = narrow_bf16(g.z); pk.w = narrow_bf16(g.w);
                    if constexpr (SNT) __builtin_nontemporal_store(pk, reinterpret_cast<u16x4*>(out) + q);
                    else reinterpret_cast<u16x4*>(out)[q] = pk;
                } else {
                    store4<SNT>(reinterpret_cast<float*>(out), q, g);
                }
            }
        }
    }
    // ragged tail: the last, partial group of four shares one counter
    if (blockIdx.x == 0 && threadIdx.x == 0 && 4 * n4 < d) {
        const f32x4 z = normals_for_quad(k0, k1, t, (uint32_t)n4);
        const float zz[4] = {z.x, z.y, z.z, z.w};
        for (size_t i = 4 * n4; i < d; ++i) {
            const float g = synth_one(load_bak1<BB>(snap, i), hdiag[i], wstar[i], sigma, zz[i - 4 * n4]);
            if constexpr (BF16) reinterpret_cast<uint16_t*>(out)[i] = narrow_bf16(g);
            else reinterpret_cast<float*>(out)[i] = g;
        }
    }
}

// ---- synthetic worker fused into the push (and the pusher's pull) ----------------
// For the synthetic workload the arriving gradient is a function of the
// pusher's own backup, which the push reads anyway: compute it in registers
// instead of writing it to HBM and reading it back.  Per parameter: read
// backup, h, wstar, w, MeanSquare (20 B), write w, MeanSquare, backup (12 B).
// The arithmetic is the worker kernel's followed by the push kernel's, so the
// results are the same bits as the two separate launches.
template <bool BF16>
__device__ __forceinline__ float synth_delivered(float snap, float h, float wstar, float sigma,
                                                 float z) {
    const float g = synth_one(snap, h, wstar, sigma, z);
    if constexpr (BF16) return widen_bf16(narrow_bf16(g));
    else return g;
}

template <bool ADAPTIVE, bool MOM, bool BF16, bool PULL, int ITEMS, bool BB, bool CHECKED>
__device__ __forceinline__ void push_synth_tile(const Hyper& hp, float* __restrict__ w,
                                                float* __restrict__ ms, void* __restrict__ bak,
                                                const float* __restrict__ hdiag,
                                                const float* __restrict__ wstar, float sigma,
                                                uint32_t k0, uint32_t k1, uint32_t t,
                                                size_t first, size_t n4) {
    f32x4 W[ITEMS], B[ITEMS], H[ITEMS], O[ITEMS], S[ITEMS], V[ITEMS];
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const size_t q = first + (size_t)j * blockDim.x;
        if (!CHECKED || q < n4) {
            V[j] = load_vel4<MOM>(hp, q);
            B[j] = load_bak4<BB, true>(bak, q);
            H[j] = load4<true>(hdiag, q);
            O[j] = load4<true>(wstar, q);
            W[j] = load4<true>(w, q);
            if constexpr (ADAPTIVE) S[j] = load4<true>(ms, q);
            else S[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        } else {
            B[j] = H[j] = O[j] = W[j] = S[j] = V[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
    }
#pragma unroll
    for (int j = 0; j < ITEMS; ++j) {
        const size_t q = first + (size_t)j * blockDim.x;
        if (!CHECKED || q < n4) {
            const f32x4 z = normals_for_quad(k0, k1, t, (uint32_t)q);
            f32x4 g;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                g[c] = synth_delivered<BF16>(B[j][c], H[j][c], O[j][c], sigma, z[c]);
            apply_push4<ADAPTIVE, MOM>(hp, g, B[j], W[j], S[j], V[j]);
            store_vel4<MOM>(hp, q, V[j]);
            store4<true>(w, q, W[j]);
            if constexpr (ADAPTIVE) store4<true>(ms, q, S[j]);
            if constexpr (PULL) store_bak4<BB, true>(bak, q, W[j]);
        }
    }
}

template <bool ADAPTIVE, bool MOM, bool BF16, bool PULL, int ITEMS, bool BB>
__global__ void __launch_bounds__(512)
push_synth_kernel(Hyper hp, float* __restrict__ w, float* __restrict__ ms,
                  void* __restrict__ bak, const float* __restrict__ hdiag,
                  const float* __restrict__ wstar, float sigma, uint32_t k0, uint32_t k1,
                  uint32_t t_arg, const uint32_t* __restrict__ ctr, size_t n4, size_t d) {
    const uint32_t t = push_index(t_arg, ctr);
    const size_t tile_quads = (size_t)blockDim.x * ITEMS;
    const size_t ntiles = (n4 + tile_quads - 1) / tile_quads;
    for (size_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const size_t first = tile * tile_quads + threadIdx.x;
        if ((tile + 1) * tile_quads <= n4)
            push_synth_tile<ADAPTIVE, MOM, BF16, PULL, ITEMS, BB, false>(
                hp, w, ms, bak, hdiag, wstar, sigma, k0, k1, t, first, n4);
        else
            push_synth_tile<ADAPTIVE, MOM, BF16, PULL, ITEMS, BB, true>(
                hp, w, ms, bak, hdiag, wstar, sigma, k0, k1, t, first, n4);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && 4 * n4 < d) {
        const f32x4 z = normals_for_quad(k0, k1, t, (uint32_t)n4);
        for (size_t i = 4 * n4; i < d; ++i) {
            const float b = load_bak1<BB>(bak, i);
            const float g = synth_delivered<BF16>(b, hdiag[i], wstar[i], sigma, z[i - 4 * n4]);
            float wi = w[i];
            float si = 0.f;
            if constexpr (ADAPTIVE) si = ms[i];
            float vi = load_vel1<MOM>(hp, i);
            apply_push<ADAPTIVE, MOM>(hp, g, b, wi, si, vi);
            w[i] = wi;
            if constexpr (ADAPTIVE) ms[i] = si;
            if constexpr (PULL) store_bak1<BB>(bak, i, wi);
            store_vel1<MOM>(hp, i, vi);
        }
    }
}

// ---- a block of arrivals of the synthetic workload in one pass ------------------
// Algorithms 1 and 2 act on every parameter by itself, and for the synthetic
// workload the arriving gradient is a function of state the lane already holds.
// So a lane can keep its four parameters of w, MeanSquare, h and wstar in
// registers over a whole block of arrivals and apply them one after the other
// exactly as the arrival-by-arrival launches would (same operations in the
// same order, hence the same bits); per arrival only the pusher's backup row
// moves: 4 bytes read and, with the fused pull, 4 written per parameter
// instead of 32.  The next arrival's backup is requested before the current
// one is worked on; a worker that arrives twice in a row finds its backup in
// registers, and one that returns later reads what this same lane stored
// earlier in the launch (program order of one lane on one address).
constexpr int RUN_BLOCK = 64;                 // arrivals per launch
struct Arrivals { uint16_t worker[RUN_BLOCK]; };

// The d mod 4 last parameters of a block of arrivals: one lane per parameter,
// each forming only the normal it needs from the shared counter of the partial
// group (word pair a,b for the first two parameters, c,d for the third; cosine
// for even positions, sine for odd ones - what normals_for_quad hands out).
template <bool ADAPTIVE, bool MOM, bool BF16, bool PULL, bool BB>
__device__ __forceinline__ void run_synth_tail(const Hyper& hp, float* __restrict__ w,
                                               float* __restrict__ ms, void* bak, size_t row_bytes,
                                               const float* __restrict__ hdiag,
                                               const float* __restrict__ wstar, float sigma,
                                               uint32_t k0, uint32_t k1, uint32_t t0,
                                               const Arrivals& arr, int A, size_t n4, size_t d) {
    const size_t i = 4 * n4 + threadIdx.x;
    if (i >= d) return;
    const bool second_pair = threadIdx.x >= 2, odd = (threadIdx.x & 1) != 0;
    float wi = w[i];
    float si = 0.f;
    if constexpr (ADAPTIVE) si = ms[i];
    float vi = load_vel1<MOM>(hp, i);
    const float hi = hdiag[i], oi = wstar[i];
    for (int e = 0; e < A; ++e) {
        void* row = static_cast<char*>(bak) + arr.worker[e] * row_bytes;
        const Words4 x = philox10((uint32_t)n4, t0 + (uint32_t)e, 0u, 0u, k0, k1);
        const float r = radius_from_word(second_pair ? x.c : x.a);
        float co, sn;
        circle_from_word(second_pair ? x.d : x.b, co, sn);
        const float z = r * (odd ? sn : co);
        const float b = load_bak1<BB>(row, i);
        const float g = synth_delivered<BF16>(b, hi, oi, sigma, z);
        apply_push<ADAPTIVE, MOM>(hp, g, b, wi, si, vi);
        if constexpr (PULL) store_bak1<BB>(row, i, wi);
    }
    w[i] = wi;
    if constexpr (ADAPTIVE) ms[i] = si;
    store_vel1<MOM>(hp, i, vi);
}

template <bool ADAPTIVE, bool MOM, bool BF16, bool PULL, bool BB, bool NT>
__global__ void __launch_bounds__(256)
run_synth_kernel(Hyper hp, float* __restrict__ w, float* __restrict__ ms, void* bak,
                 size_t row_bytes, const float* __restrict__ hdiag,
                 const float* __restrict__ wstar, float sigma, uint32_t k0, uint32_t k1,
                 uint32_t t_arg, const uint32_t* __restrict__ ctr, Arrivals arr, int A,
                 size_t n4, size_t d) {
    const uint32_t t0 = push_index(t_arg, ctr);
    // the d mod 4 last parameters are a whole block of arrivals of scalar work: they get a
    // block of their own (the last one), so that no lane has two shares
    const bool has_tail = 4 * n4 < d;
    const size_t main_blocks = gridDim.x - (has_tail ? 1u : 0u);
    const bool tail_block = has_tail && blockIdx.x == main_blocks;
    const size_t stride = main_blocks * blockDim.x;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; !tail_block && q < n4; q += stride) {
        f32x4 W = load4<NT>(w, q);
        f32x4 S = f32x4{0.f, 0.f, 0.f, 0.f};
        if constexpr (ADAPTIVE) S = load4<NT>(ms, q);
        const f32x4 H = load4<NT>(hdiag, q);
        const f32x4 O = load4<NT>(wstar, q);
        f32x4 V = load_vel4<MOM>(hp, q);
        f32x4 B = load_bak4<BB, NT>(static_cast<char*>(bak) + arr.worker[0] * row_bytes, q);
        for (int e = 0; e < A; ++e) {
            void* row = static_cast<char*>(bak) + arr.worker[e] * row_bytes;
            const bool more = e + 1 < A;
            const bool again = more && arr.worker[e + 1] == arr.worker[e];
            f32x4 Bn = B;
            if (more && !again)
                Bn = load_bak4<BB, NT>(static_cast<char*>(bak) + arr.worker[e + 1] * row_bytes, q);
            const f32x4 z = normals_for_quad(k0, k1, t0 + (uint32_t)e, (uint32_t)q);
            f32x4 g;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                g[c] = synth_delivered<BF16>(B[c], H[c], O[c], sigma, z[c]);
            apply_push4<ADAPTIVE, MOM>(hp, g, B, W, S, V);
            if constexpr (PULL) {
                store_bak4<BB, NT>(row, q, W);
                if (again) {
                    // what a load of the row just stored would return
                    if constexpr (BB) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) Bn[c] = widen_bf16(narrow_bf16(W[c]));
                    } else {
                        Bn = W;
                    }
                }
            }
            B = Bn;
        }
        store_vel4<MOM>(hp, q, V);
        store4<NT>(w, q, W);
        if constexpr (ADAPTIVE) store4<NT>(ms, q, S);
    }
    if (tail_block)
        run_synth_tail<ADAPTIVE, MOM, BF16, PULL, BB>(hp, w, ms, bak, row_bytes, hdiag, wstar, sigma,
                                                      k0, k1, t0, arr, A, n4, d);
}

// The same loop for vectors too short to give every SIMD several waves at four
// parameters per lane (the 1 MB configurations: one wave per SIMD, and the
// dependent chains of Philox, Box-Muller and Eq. 18 leave it idle most of the
// time).  Here two lanes share a group of four: both draw the group's Philox
// words, each forms one of its two normal pairs and updates two parameters.
// Twice the waves for about 1.15 times the instructions; the arithmetic per
// parameter is unchanged, so the bits are.
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

template <bool NT>
__device__ __forceinline__ f32x2 load2(const float* base, size_t pair) {
    const f32x2* p = reinterpret_cast<const f32x2*>(base) + pair;
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT>
__device__ __forceinline__ void store2(float* base, size_t pair, f32x2 v) {
    f32x2* p = reinterpret_cast<f32x2*>(base) + pair;
    if constexpr (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}
template <bool BB, bool NT>
__device__ __forceinline__ f32x2 load_bak2(const void* bak, size_t pair) {
    if constexpr (BB) {
        const u16x2* p = reinterpret_cast<const u16x2*>(bak) + pair;
        u16x2 r;
        if constexpr (NT) r = __builtin_nontemporal_load(p);
        else r = *p;
        return f32x2{widen_bf16(r.x), widen_bf16(r.y)};
    } else {
        return load2<NT>(reinterpret_cast<const float*>(bak), pair);
    }
}
template <bool BB, bool NT>
__device__ __forceinline__ void store_bak2(void* bak, size_t pair, f32x2 v) {
    if constexpr (BB) {
        const u16x2 r = {narrow_bf16(v.x), narrow_bf16(v.y)};
        u16x2* p = reinterpret_cast<u16x2*>(bak) + pair;
        if constexpr (NT) __builtin_nontemporal_store(r, p);
        else *p = r;
    } else {
        store2<NT>(reinterpret_cast<float*>(bak), pair, v);
    }
}

// a pair seen by the four-wide update: both halves hold the same two values, so
// the duplicate arithmetic is one computation to the compiler
__device__ __forceinline__ f32x4 twice(f32x2 a) { return f32x4{a.x, a.y, a.x, a.y}; }

template <bool ADAPTIVE, bool MOM, bool BF16, bool PULL, bool BB, bool NT>
__global__ void __launch_bounds__(256)
run_synth_pairs_kernel(Hyper hp, float* __restrict__ w, float* __restrict__ ms, void* bak,
                       size_t row_bytes, const float* __restrict__ hdiag,
                       const float* __restrict__ wstar, float sigma, uint32_t k0, uint32_t k1,
                       uint32_t t_arg, const uint32_t* __restrict__ ctr, Arrivals arr, int A,
                       size_t n4, size_t d) {
    const uint32_t t0 = push_index(t_arg, ctr);
    const bool has_tail = 4 * n4 < d;                  // the last block does the d mod 4 tail only
    const size_t main_blocks = gridDim.x - (has_tail ? 1u : 0u);
    const bool tail_block = has_tail && blockIdx.x == main_blocks;
    const size_t stride = main_blocks * blockDim.x;
    const size_t npairs = 2 * n4;                      // pair p holds parameters 2p, 2p+1 of group p/2
    for (size_t p = (size_t)blockIdx.x * blockDim.x + threadIdx.x; !tail_block && p < npairs; p += stride) {
        const bool upper = (p & 1) != 0;
        // the lane's state is two values per vector; they are doubled for the four-wide
        // update inside each iteration, never across iterations (loop-carried copies
        // would be updated twice)
        f32x2 W = load2<NT>(w, p);
        f32x2 S = f32x2{0.f, 0.f};
        if constexpr (ADAPTIVE) S = load2<NT>(ms, p);
        const f32x2 H = load2<NT>(hdiag, p);
        const f32x2 O = load2<NT>(wstar, p);
        f32x2 V = f32x2{0.f, 0.f};
        if constexpr (MOM) V = load2<true>(hp.vel, p);
        f32x2 B = load_bak2<BB, NT>(static_cast<char*>(bak) + arr.worker[0] * row_bytes, p);
        for (int e = 0; e < A; ++e) {
            void* row = static_cast<char*>(bak) + arr.worker[e] * row_bytes;
            const bool more = e + 1 < A;
            const bool again = more && arr.worker[e + 1] == arr.worker[e];
            f32x2 Bn = B;
            if (more && !again)
                Bn = load_bak2<BB, NT>(static_cast<char*>(bak) + arr.worker[e + 1] * row_bytes, p);
            const Words4 x = philox10((uint32_t)(p >> 1), t0 + (uint32_t)e, 0u, 0u, k0, k1);
            const float r = radius_from_word(upper ? x.c : x.a);
            float co, si;
            circle_from_word(upper ? x.d : x.b, co, si);
            const f32x2 z = {r * co, r * si};
            f32x2 g;
            g.x = synth_delivered<BF16>(B.x, H.x, O.x, sigma, z.x);
            g.y = synth_delivered<BF16>(B.y, H.y, O.y, sigma, z.y);
            f32x4 W4 = twice(W), S4 = twice(S), V4 = twice(V);
            apply_push4<ADAPTIVE, MOM>(hp, twice(g), twice(B), W4, S4, V4);
            W = f32x2{W4.x, W4.y};
            S = f32x2{S4.x, S4.y};
            V = f32x2{V4.x, V4.y};
            if constexpr (PULL) {
                store_bak2<BB, NT>(row, p, W);
                if (again) {
                    if constexpr (BB) Bn = f32x2{widen_bf16(narrow_bf16(W.x)), widen_bf16(narrow_bf16(W.y))};
                    else Bn = W;
                }
            }
            B = Bn;
        }
        if constexpr (MOM) store2<true>(hp.vel, p, V);
        store2<NT>(w, p, W);
        if constexpr (ADAPTIVE) store2<NT>(ms, p, S);
    }
    if (tail_block)
        run_synth_tail<ADAPTIVE, MOM, BF16, PULL, BB>(hp, w, ms, bak, row_bytes, hdiag, wstar, sigma,
                                                      k0, k1, t0, arr, A, n4, d);
}

}  // namespace dcasgd
