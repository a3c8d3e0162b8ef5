// DC-ASGD parameter-server oracle: plain, sequential, slow, CPU only.
//
// THIS FILE IS TEST INFRASTRUCTURE. It is the yardstick the GPU library is
// compared against; nothing in the product path may include, link or call it,
// and it shares no code with the HIP sources.
//
// What it computes (Zheng et al., "Asynchronous Stochastic Gradient Descent
// with Delay Compensation"):
//   * the server of Algorithm 2: state w, w_bak(m) for m = 1..M (all started
//     at w_0) and the push counter t;
//   * the "receive g_m" branch, i.e. the update rule of Eq. 4.1 with a
//     constant lambda (DC-ASGD-c, Section 6) or with lambda_t = lambda_0 /
//     sqrt(MeanSquare(t) + eps) where MeanSquare follows Eq. 18 (DC-ASGD-a);
//   * the "pull request" branch: w_bak(m) <- w_t;
//   * the synchronous variant of the supplement ("Large Mini-batch Synchronous
//     SGD with Delay-Compensated Gradient"): J gradients taken at the same
//     model w_t are applied one after the other with step eta_hat/J, each
//     compensated for the distance the running model has already moved from
//     w_t;
//   * a stand-in for the worker of Algorithm 1 ("compute gradient"): the
//     gradient of a diagonal quadratic loss at the worker's snapshot plus
//     seeded Gaussian noise. This part is not from the paper; it is the
//     synthetic workload the benchmark configurations define.
//
// Arithmetic: IEEE-754 binary32, one rounding per written operation, no fused
// multiply-add, denormals kept. Build with
//   g++ -std=c++17 -O2 -ffp-contract=off -fno-fast-math
// Every float expression below is deliberately split into single operations so
// that the order of roundings can be read off the source.
//
// Readings taken where the paper is silent (each is listed again in the
// design notes of the repository):
//   * MeanSquare(t) is refreshed with the arriving gradient first and
//     lambda_t is formed from the refreshed value (both carry index t in
//     Eq. 18); MeanSquare(0) = 0; one MeanSquare vector per server;
//     g^2 is elementwise.
//   * (1 - m) of Eq. 18 is formed once, in binary32.
//   * the compensation term is grouped (lambda * g*g) * (w - w_bak): the
//     diagonal Hessian estimate lambda g.g of Section 4 is formed first.
//   * in the synchronous fold the order of the J gradients is the caller's;
//     the supplement suggests ordering by the distance from w_t, read here as
//     ascending gradient norm (a helper computes the squared norms); lambda
//     may be the adaptive one, MeanSquare then advances once per gradient;
//     eta_hat/J is formed once in binary32.
//   * bfloat16 snapshots (optional, not from the paper): the value handed to
//     the worker and the value kept as w_bak(m) are the same rounded number.
//   * momentum: the paper names momentum variants (footnote, Section 6)
//     without a formula.  Implemented as a proposal, the classical heavy
//     ball on the compensated gradient: v <- mu*v + g_dc, w <- w - eta*v, one
//     velocity vector per server.  The pins fix that this rule is what is
//     computed; whether it is the authors' rule is unpinned.
//
// Pins (see tests/test_oracle_*.py): lambda = 0 gives ASGD (Eq. 2.2); M = 1
// gives sequential SGD; exact-rational hand trace; closed forms for a
// constant gradient; Philox known answers and a second implementation on a
// million counters; Box-Muller against libm in double and bit for bit against
// a second implementation on numpy float32 arrays; bf16 rounding against a
// library conversion; the state finite after every push of the benchmark
// configurations; and single planted mistakes in a copy of this file, each of
// which must fail a pin.
// Parity unpinned (nothing in the paper fixes them; the pins only fix what is
// computed): that ascending gradient norm is the fold order the supplement's
// closing remark means; that heavy ball on the compensated gradient is the
// authors' momentum rule; what bfloat16 snapshots do to the accuracy of a
// real network; whether delay compensation helps on real networks at all
// (the paper's evidence is CIFAR-10 / ImageNet accuracy).

#include <cmath>
#include <cstddef>
#include <cstdint>
#include <cstring>
#include <thread>
#include <vector>
#include <xmmintrin.h>

namespace {

inline uint32_t bits_of(float x) { uint32_t u; std::memcpy(&u, &x, 4); return u; }
inline float float_of(uint32_t u) { float x; std::memcpy(&x, &u, 4); return x; }

// ---------------------------------------------------------------------------
// Philox4x32-10, the counter-based generator of Salmon, Moraes, Dror and Shaw
// (SC'11). Ten rounds; the key is bumped by the Weyl constants between rounds.
// ---------------------------------------------------------------------------
void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    const uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u;
    const uint32_t WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += WEYL_A; k1 += WEYL_B; }
        const uint64_t pa = (uint64_t)MUL_A * c0;
        const uint64_t pb = (uint64_t)MUL_B * c2;
        const uint32_t n0 = (uint32_t)(pb >> 32) ^ c1 ^ k0;
        const uint32_t n1 = (uint32_t)pb;
        const uint32_t n2 = (uint32_t)(pa >> 32) ^ c3 ^ k1;
        const uint32_t n3 = (uint32_t)pa;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// ---------------------------------------------------------------------------
// Two standard normals from two 32-bit words by the Box-Muller transform,
// written with + - * / sqrt only so that any IEEE machine gives the same bits.
//   u in (0,1] from the top 24 bits of xa, angle 2*pi*j/2^24 from the top 24
//   bits of xb;  z0 = sqrt(-2 ln u) cos(angle), z1 = sqrt(-2 ln u) sin(angle).
// ln u: u = 2^e * mt with mt in (sqrt(1/2), sqrt(2)], ln mt = 2 atanh(s),
//   s = (mt-1)/(mt+1), odd series through s^9.
// sin/cos: the angle is folded to x in [0, pi/4]; Taylor polynomials through
//   x^9 (sin) and x^10 (cos); the octant decides swap and signs.
// ---------------------------------------------------------------------------
void normal_pair(uint32_t xa, uint32_t xb, float* z0, float* z1) {
    // radius
    const uint32_t k = (xa >> 8) + 1u;                    // 1 .. 2^24
    const float u = (float)k * 0x1p-24f;                  // exact, in (0,1]
    const uint32_t ub = bits_of(u);
    int e = (int)(ub >> 23) - 127;
    float mt = float_of((ub & 0x007FFFFFu) | 0x3F800000u);  // [1,2)
    if (mt > 1.41421354f) { mt = mt * 0.5f; e = e + 1; }
    const float f = mt - 1.0f;
    const float mp = mt + 1.0f;
    const float s = f / mp;
    const float s2 = s * s;
    float p = 0.11111111f;           // 1/9
    p = p * s2;  p = p + 0.14285715f;  // 1/7
    p = p * s2;  p = p + 0.2f;         // 1/5
    p = p * s2;  p = p + 0.33333334f;  // 1/3
    p = p * s2;  p = p + 1.0f;
    const float twos = 2.0f * s;
    const float lm = twos * p;
    const float el = (float)e * 0.69314718f;
    const float lnu = el + lm;                            // <= 0
    const float m2l = -2.0f * lnu;
    const float r = std::sqrt(m2l);

    // angle
    const uint32_t j = xb >> 8;                           // 0 .. 2^24-1
    const uint32_t quadrant = j >> 22;
    uint32_t rr = j & 0x3FFFFFu;
    const bool swap = rr > 0x200000u;
    if (swap) rr = 0x400000u - rr;
    const float x = (float)rr * 0x1.921fb6p-22f;          // rr * (pi/2) / 2^22
    const float x2 = x * x;
    float sp = 2.7557319e-6f;          //  1/9!
    sp = sp * x2;  sp = sp - 1.9841270e-4f;   // -1/7!
    sp = sp * x2;  sp = sp + 8.3333333e-3f;   //  1/5!
    sp = sp * x2;  sp = sp - 0.16666667f;     // -1/3!
    sp = sp * x2;  sp = sp + 1.0f;
    float sn = x * sp;
    float cp = -2.7557319e-7f;         // -1/10!
    cp = cp * x2;  cp = cp + 2.4801587e-5f;   //  1/8!
    cp = cp * x2;  cp = cp - 1.3888889e-3f;   // -1/6!
    cp = cp * x2;  cp = cp + 4.1666668e-2f;   //  1/4!
    cp = cp * x2;  cp = cp - 0.5f;            // -1/2!
    cp = cp * x2;
    float cs = cp + 1.0f;
    if (swap) { const float tmp = sn; sn = cs; cs = tmp; }
    float C, S;
    switch (quadrant) {
        case 0:  C = cs;  S = sn;  break;
        case 1:  C = -sn; S = cs;  break;
        case 2:  C = -cs; S = -sn; break;
        default: C = sn;  S = -cs; break;
    }
    *z0 = r * C;
    *z1 = r * S;
}

// The four normals that belong to elements 4q .. 4q+3 at push index t.
// Counter (q, t, 0, tag), key (seed low word, seed high word).
void normal_quad(uint64_t seed, uint32_t t, uint32_t q, uint32_t tag, float z[4]) {
    const uint32_t ctr[4] = {q, t, 0u, tag};
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t x[4];
    philox4x32_10(ctr, key, x);
    normal_pair(x[0], x[1], &z[0], &z[1]);
    normal_pair(x[2], x[3], &z[2], &z[3]);
}

// binary32 -> bfloat16, round to nearest, ties to even (finite inputs).
inline uint16_t bf16_rne(float x) {
    const uint32_t b = bits_of(x);
    const uint32_t bias = 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)((b + bias) >> 16);
}
inline float bf16_widen(uint16_t h) { return float_of((uint32_t)h << 16); }

// ---------------------------------------------------------------------------
// Server state of Algorithm 2.
// ---------------------------------------------------------------------------
struct Server {
    size_t n = 0;          // number of parameters held
    int M = 0;             // number of workers
    float eta = 0, lambda0 = 0;
    int adaptive = 0;      // 0: DC-ASGD-c, 1: DC-ASGD-a
    float ema_m = 0, one_minus_m = 0, eps = 0;
    int momentum = 0;      // 1: heavy-ball momentum on the compensated gradient
    float mu = 0;
    uint64_t t = 0;        // pushes applied so far
    std::vector<float> w, ms, vel;
    std::vector<std::vector<float>> bak;
    int bak_bf16 = 0;      // 1: a pull hands out (and the server keeps) w rounded to bfloat16
};

// The delay-compensated gradient of Eq. 4.1 with lambda_t = lambda_0, one element.
inline float compensated_const(const Server& sv, float g, float b, float w) {
    const float diff = w - b;
    const float g2 = g * g;
    const float c1 = sv.lambda0 * g2;
    const float c2 = c1 * diff;
    const float gd = g + c2;
    return gd;
}

// Eq. 18, then the delay-compensated gradient with
// lambda_t = lambda_0 / sqrt(MeanSquare + eps).
inline float compensated_adaptive(const Server& sv, float g, float b, float w, float* ms) {
    const float g2 = g * g;
    const float t1 = sv.ema_m * *ms;
    const float t2 = sv.one_minus_m * g2;
    *ms = t1 + t2;
    const float den = *ms + sv.eps;
    const float rt = std::sqrt(den);
    const float lam = sv.lambda0 / rt;
    const float diff = w - b;
    const float c1 = lam * g2;
    const float c2 = c1 * diff;
    const float gd = g + c2;
    return gd;
}

// One arriving gradient element: w <- w - eta * gd (Algorithm 2), or, with
// momentum (the paper only mentions momentum variants in a footnote of
// Section 6; the rule here is the classical heavy ball applied to the
// compensated gradient): v <- mu*v + gd; w <- w - eta*v.
inline void push_elem(Server& sv, float eta, float g, float b, size_t i) {
    const float gd = sv.adaptive ? compensated_adaptive(sv, g, b, sv.w[i], &sv.ms[i])
                                 : compensated_const(sv, g, b, sv.w[i]);
    if (sv.momentum) {
        const float mv = sv.mu * sv.vel[i];
        sv.vel[i] = mv + gd;
        const float st = eta * sv.vel[i];
        sv.w[i] = sv.w[i] - st;
    } else {
        const float st = eta * gd;
        sv.w[i] = sv.w[i] - st;
    }
}

// Algorithm 2, "receive g_m", elements [lo, hi). g is indexed like w.
void push_range(Server& sv, int m, const float* g, size_t lo, size_t hi) {
    const float* b = sv.bak[m].data();
    for (size_t i = lo; i < hi; ++i) push_elem(sv, sv.eta, g[i], b[i], i);
}

// Algorithm 2, "pull request": w_bak(m) <- w_t, elements [lo, hi).
// With bfloat16 snapshots the worker receives round-to-nearest-even(w) and the
// server keeps exactly that value as w_bak(m): the gradient that comes back was
// taken at the rounded point, so w - w_bak(m) is still the true displacement
// from where the gradient was computed.  bak holds the widened value.
void pull_range(Server& sv, int m, size_t lo, size_t hi) {
    for (size_t i = lo; i < hi; ++i) {
        float v = sv.w[i];
        if (sv.bak_bf16) v = bf16_widen(bf16_rne(v));
        sv.bak[m][i] = v;
    }
}

// Supplement, last section: fold J gradients g[0..J) (each n floats, all taken
// at the model held on entry, w_t) into the model:
//   wt^{j+1} = wt^j - (eta_hat/J) * (g_j + lambda g_j.g_j.(wt^j - w_t)),  wt^0 = w_t.
// This is the push rule with the learning rate eta_hat/J and with w_t in the
// role of the backup for every j.
void sync_fold(Server& sv, const float* const* g, int J, float eta_hat) {
    const float step = eta_hat / (float)J;  // per-gradient learning rate
    for (size_t i = 0; i < sv.n; ++i) {
        const float anchor = sv.w[i];       // w_t
        for (int j = 0; j < J; ++j) push_elem(sv, step, g[j][i], anchor, i);
    }
}

// Stand-in worker (Algorithm 1, "compute gradient") for elements [lo, hi):
//   g_i = h_i * (snapshot_i - wstar_i) + sigma * z(seed, t, global index of i)
// optionally rounded to bfloat16 and widened again. gidx maps local element
// to its index in the full parameter vector (nullptr: identity); only the
// noise depends on it.
void synth_grad_range(const float* snap, const float* hdiag, const float* wstar,
                      float sigma, uint64_t seed, uint32_t t, const uint64_t* gidx,
                      int as_bf16, float* g, size_t lo, size_t hi) {
    float z[4] = {0, 0, 0, 0};
    uint64_t have_q = ~(uint64_t)0;      // block of four whose normals are in z
    for (size_t i = lo; i < hi; ++i) {
        const uint64_t gi = gidx ? gidx[i] : (uint64_t)i;
        if ((gi >> 2) != have_q) {
            have_q = gi >> 2;
            normal_quad(seed, t, (uint32_t)have_q, 0u, z);
        }
        const float dd = snap[i] - wstar[i];
        const float p = hdiag[i] * dd;
        const float nz = sigma * z[gi & 3u];
        float gv = p + nz;
        if (as_bf16) gv = bf16_widen(bf16_rne(gv));
        g[i] = gv;
    }
}

// One simulated arrival sequence, elements [lo, hi): for every event the
// worker's gradient is taken at its backup (which is what it last pulled),
// pushed, and the worker pulls again (Algorithm 1 is one such cycle).
void run_range(Server& sv, const int* order, size_t T, uint64_t t0,
               const float* hdiag, const float* wstar, float sigma, uint64_t seed,
               const uint64_t* gidx, int as_bf16, float* gbuf, size_t lo, size_t hi) {
    for (size_t e = 0; e < T; ++e) {
        const int m = order[e];
        synth_grad_range(sv.bak[m].data(), hdiag, wstar, sigma, seed,
                         (uint32_t)(t0 + e), gidx, as_bf16, gbuf, lo, hi);
        push_range(sv, m, gbuf, lo, hi);
        pull_range(sv, m, lo, hi);
    }
}

// The same sequence with a look at the state after every push: returns the
// index of the first event after whose push some w, MeanSquare or velocity
// value of [lo, hi) is not finite, or T if there is none.  (A non-finite
// backup can only come from a non-finite w.)  No arithmetic of its own.
size_t run_range_checked(Server& sv, const int* order, size_t T, uint64_t t0,
                         const float* hdiag, const float* wstar, float sigma, uint64_t seed,
                         const uint64_t* gidx, int as_bf16, float* gbuf, size_t lo, size_t hi) {
    size_t first_bad = T;
    for (size_t e = 0; e < T; ++e) {
        const int m = order[e];
        synth_grad_range(sv.bak[m].data(), hdiag, wstar, sigma, seed,
                         (uint32_t)(t0 + e), gidx, as_bf16, gbuf, lo, hi);
        push_range(sv, m, gbuf, lo, hi);
        if (first_bad == T) {
            bool finite = true;
            for (size_t i = lo; i < hi && finite; ++i) {
                finite = std::isfinite(sv.w[i]);
                if (finite && !sv.ms.empty()) finite = std::isfinite(sv.ms[i]);
                if (finite && !sv.vel.empty()) finite = std::isfinite(sv.vel[i]);
            }
            if (!finite) first_bad = e;
        }
        pull_range(sv, m, lo, hi);
    }
    return first_bad;
}

// Denormals must be kept: clear flush-to-zero / denormals-are-zero for the
// duration of a call in case the embedding process switched them on.
struct KeepDenormals {
    unsigned saved;
    KeepDenormals() : saved(_mm_getcsr()) { _mm_setcsr(saved & ~0x8040u); }
    ~KeepDenormals() { _mm_setcsr(saved); }
};

}  // namespace

// ---------------------------------------------------------------------------
// C interface (for ctypes). Every pointer is host memory owned by the caller
// unless stated otherwise. No argument checking beyond the obvious: this is a
// test oracle, callers are the tests.
// ---------------------------------------------------------------------------
extern "C" {

void oracle_philox4x32_10(const uint32_t* ctr, const uint32_t* key, uint32_t* out) {
    philox4x32_10(ctr, key, out);
}

void oracle_normal_pair(uint32_t xa, uint32_t xb, float* z) {
    KeepDenormals guard;
    normal_pair(xa, xb, &z[0], &z[1]);
}

// The same two calls over arrays (n counters with their keys; n word pairs):
// plain loops, so that tests can compare millions of cases.
void oracle_philox4x32_10_many(const uint32_t* ctr, const uint32_t* key, uint32_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) philox4x32_10(ctr + 4 * i, key + 2 * i, out + 4 * i);
}

void oracle_normal_pairs(const uint32_t* xa, const uint32_t* xb, float* z, size_t n) {
    KeepDenormals guard;
    for (size_t i = 0; i < n; ++i) normal_pair(xa[i], xb[i], &z[2 * i], &z[2 * i + 1]);
}

void oracle_normal_quad(uint64_t seed, uint32_t t, uint32_t q, uint32_t tag, float* z) {
    KeepDenormals guard;
    normal_quad(seed, t, q, tag, z);
}

void oracle_bf16_rne(const float* x, uint16_t* out, size_t n) {
    for (size_t i = 0; i < n; ++i) out[i] = bf16_rne(x[i]);
}

// mode: 0 = DC-ASGD-c, 1 = DC-ASGD-a. w0 has n floats; every backup starts as
// a copy of it, MeanSquare starts at zero, t at zero.
void* oracle_create(size_t n, int M, float eta, float lambda0, int mode,
                    float ema_m, float eps, const float* w0) {
    if (n == 0 || M <= 0 || (mode != 0 && mode != 1) || !w0) return nullptr;
    Server* sv = new Server;
    sv->n = n; sv->M = M; sv->eta = eta; sv->lambda0 = lambda0;
    sv->adaptive = mode; sv->ema_m = ema_m; sv->eps = eps;
    sv->one_minus_m = 1.0f - ema_m;
    sv->w.assign(w0, w0 + n);
    sv->ms.assign(n, 0.0f);
    sv->bak.assign(M, sv->w);
    return sv;
}

void oracle_destroy(void* h) { delete static_cast<Server*>(h); }

uint64_t oracle_step(void* h) { return static_cast<Server*>(h)->t; }

// Switch heavy-ball momentum on (velocity restarts at zero) or off (mu == 0).
void oracle_set_momentum(void* h, float mu) {
    Server& sv = *static_cast<Server*>(h);
    sv.mu = mu;
    sv.momentum = mu != 0.0f;
    sv.vel.assign(sv.momentum ? sv.n : 0, 0.0f);
}
void oracle_get_vel(void* h, float* out) {
    Server& sv = *static_cast<Server*>(h);
    if (sv.momentum) std::memcpy(out, sv.vel.data(), sv.n * sizeof(float));
}

// Snapshot storage variant (not from the paper, which only notes that the
// backups cost memory): bfloat16 backups.  Switching it on rounds the backups
// held at that moment, as if each worker had pulled in the new format.
void oracle_set_backup_bf16(void* h, int on) {
    Server& sv = *static_cast<Server*>(h);
    sv.bak_bf16 = on ? 1 : 0;
    if (!on) return;
    for (int m = 0; m < sv.M; ++m)
        for (size_t i = 0; i < sv.n; ++i) sv.bak[m][i] = bf16_widen(bf16_rne(sv.bak[m][i]));
}

// Learning-rate schedule (Section 6 divides eta by ten at fixed epochs).
void oracle_set_eta(void* h, float eta) { static_cast<Server*>(h)->eta = eta; }

// Algorithm 2 takes a time-indexed lambda_t as input: lambda (DC-ASGD-c) or
// lambda_0 (DC-ASGD-a) may be changed between pushes.
void oracle_set_lambda(void* h, float lambda0) { static_cast<Server*>(h)->lambda0 = lambda0; }

// Algorithm 2 "receive g_m": g has n floats (already widened if it travelled
// as bf16).
int oracle_push(void* h, int worker, const float* g) {
    Server& sv = *static_cast<Server*>(h);
    if (worker < 0 || worker >= sv.M) return -1;
    KeepDenormals guard;
    push_range(sv, worker, g, 0, sv.n);
    sv.t += 1;
    return 0;
}

// Algorithm 2 "pull request".
int oracle_pull(void* h, int worker) {
    Server& sv = *static_cast<Server*>(h);
    if (worker < 0 || worker >= sv.M) return -1;
    pull_range(sv, worker, 0, sv.n);
    return 0;
}

void oracle_get_w(void* h, float* out) {
    Server& sv = *static_cast<Server*>(h);
    std::memcpy(out, sv.w.data(), sv.n * sizeof(float));
}
void oracle_get_ms(void* h, float* out) {
    Server& sv = *static_cast<Server*>(h);
    std::memcpy(out, sv.ms.data(), sv.n * sizeof(float));
}
int oracle_get_bak(void* h, int worker, float* out) {
    Server& sv = *static_cast<Server*>(h);
    if (worker < 0 || worker >= sv.M) return -1;
    std::memcpy(out, sv.bak[worker].data(), sv.n * sizeof(float));
    return 0;
}
void oracle_set_ms(void* h, const float* in) {
    Server& sv = *static_cast<Server*>(h);
    sv.ms.assign(in, in + sv.n);
}

// Squared Euclidean norms of J gradients (g: J*n floats).  With a common step
// the distance |wt - w_t| that gradient j alone would produce is proportional
// to |g_j|, which is the quantity the supplement proposes to order the fold
// by (smallest first).  The value meant is the real number sum g_i^2: each
// square is exact in the 64-bit significand of long double and the running
// sum is kept there, so the double returned is the true value to within a few
// units of 2^-53 even for tens of millions of terms.
void oracle_grad_sqnorms(const float* g, int J, size_t n, double* out) {
    static_assert(sizeof(long double) > sizeof(double), "needs an extended accumulator");
    for (int j = 0; j < J; ++j) {
        long double acc = 0.0L;
        for (size_t i = 0; i < n; ++i) {
            const long double x = (long double)g[(size_t)j * n + i];
            acc += x * x;
        }
        out[j] = (double)acc;
    }
}

// Synchronous delay-compensated fold of J gradients (g: J*n floats, gradient
// j at g + j*n), all taken at the current model.  t advances by J.
int oracle_sync_fold(void* h, const float* g, int J, float eta_hat) {
    Server& sv = *static_cast<Server*>(h);
    if (J < 1 || !g) return -1;
    KeepDenormals guard;
    std::vector<const float*> rows((size_t)J);
    for (int j = 0; j < J; ++j) rows[(size_t)j] = g + (size_t)j * sv.n;
    sync_fold(sv, rows.data(), J, eta_hat);
    sv.t += (uint64_t)J;
    return 0;
}

// The same fold delivered in parts (more same-snapshot gradients than one call
// takes): Jc of the J_total gradients, compensated against the model the whole
// fold started from, which the caller kept in `anchor` (n floats).  The step is
// eta_hat / J_total, formed once in binary32 as in the undivided fold.
int oracle_sync_fold_part(void* h, const float* g, int Jc, int J_total, float eta_hat,
                          const float* anchor) {
    Server& sv = *static_cast<Server*>(h);
    if (Jc < 1 || J_total < Jc || !g || !anchor) return -1;
    KeepDenormals guard;
    const float step = eta_hat / (float)J_total;
    for (size_t i = 0; i < sv.n; ++i)
        for (int j = 0; j < Jc; ++j) push_elem(sv, step, g[(size_t)j * sv.n + i], anchor[i], i);
    sv.t += (uint64_t)Jc;
    return 0;
}

// Synthetic worker gradient taken at an arbitrary snapshot (n floats each).
void oracle_synth_grad(const float* snap, const float* hdiag, const float* wstar,
                       float sigma, uint64_t seed, uint32_t push_idx,
                       const uint64_t* gidx, int as_bf16, float* g_out, size_t n) {
    KeepDenormals guard;
    synth_grad_range(snap, hdiag, wstar, sigma, seed, push_idx, gidx, as_bf16, g_out, 0, n);
}

// The event loop: T arrivals, order[e] = worker of arrival e. The noise of
// arrival e is keyed by the server's push counter (t before the push).
// nthreads > 1 splits the elements into contiguous chunks, one sequential
// loop per chunk; elements never interact, so the result is the same bits.
int oracle_run(void* h, const int* order, size_t T, const float* hdiag,
               const float* wstar, float sigma, uint64_t seed,
               const uint64_t* gidx, int as_bf16, int nthreads) {
    Server& sv = *static_cast<Server*>(h);
    for (size_t e = 0; e < T; ++e)
        if (order[e] < 0 || order[e] >= sv.M) return -1;
    if (nthreads < 1) nthreads = 1;
    std::vector<float> gbuf(sv.n);
    const uint64_t t0 = sv.t;
    auto body = [&](size_t lo, size_t hi) {
        KeepDenormals guard;
        run_range(sv, order, T, t0, hdiag, wstar, sigma, seed, gidx, as_bf16,
                  gbuf.data(), lo, hi);
    };
    if (nthreads == 1) {
        body(0, sv.n);
    } else {
        std::vector<std::thread> pool;
        const size_t chunk = (sv.n + nthreads - 1) / nthreads;
        for (int k = 0; k < nthreads; ++k) {
            const size_t lo = (size_t)k * chunk;
            const size_t hi = lo + chunk < sv.n ? lo + chunk : sv.n;
            if (lo < hi) pool.emplace_back(body, lo, hi);
        }
        for (auto& th : pool) th.join();
    }
    sv.t += T;
    return 0;
}

// oracle_run that also reports when the state stopped being finite: *first_bad
// receives the index of the first arrival after whose push some element of w,
// MeanSquare or the velocity is inf or NaN, or -1 if every state stayed finite.
int oracle_run_checked(void* h, const int* order, size_t T, const float* hdiag,
                       const float* wstar, float sigma, uint64_t seed,
                       const uint64_t* gidx, int as_bf16, int nthreads, long long* first_bad) {
    Server& sv = *static_cast<Server*>(h);
    for (size_t e = 0; e < T; ++e)
        if (order[e] < 0 || order[e] >= sv.M) return -1;
    if (nthreads < 1) nthreads = 1;
    std::vector<float> gbuf(sv.n);
    std::vector<size_t> bad((size_t)nthreads, T);
    const uint64_t t0 = sv.t;
    const size_t chunk = (sv.n + nthreads - 1) / nthreads;
    std::vector<std::thread> pool;
    for (int k = 0; k < nthreads; ++k) {
        const size_t lo = (size_t)k * chunk;
        const size_t hi = lo + chunk < sv.n ? lo + chunk : sv.n;
        if (lo >= hi) continue;
        pool.emplace_back([&, k, lo, hi] {
            KeepDenormals guard;
            bad[(size_t)k] = run_range_checked(sv, order, T, t0, hdiag, wstar, sigma, seed, gidx,
                                               as_bf16, gbuf.data(), lo, hi);
        });
    }
    for (auto& th : pool) th.join();
    size_t first = T;
    for (size_t b : bad) first = b < first ? b : first;
    *first_bad = first == T ? -1 : (long long)first;
    sv.t += T;
    return 0;
}

}  // extern "C"
