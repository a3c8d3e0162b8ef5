/*
 * dcasgd.h - C ABI of the MI355X (gfx950) DC-ASGD parameter-server update.
 *
 * The library implements the server side of "Asynchronous Stochastic Gradient
 * Descent with Delay Compensation" (Zheng et al.): Algorithm 2 with the update
 * rule of Eq. 4.1, with a constant lambda (DC-ASGD-c) or the adaptive lambda
 * of Eq. 18 (DC-ASGD-a).  Every step runs in hand-written HIP kernels; the
 * library calls no device allocator and owns nothing but the small handle
 * and one static 256.5 KB device array (see dcasgd_sync_fold_ordered_static).
 *
 * Conventions
 *   - "device pointer": memory of the GPU that is current when the call is
 *     made, owned by the caller and kept alive until the stream has passed the
 *     call.  "host pointer": ordinary process memory, read during the call.
 *   - stream: a hipStream_t passed as void* (NULL = the default stream).  All
 *     work is enqueued on it and returns immediately; calls on one handle must
 *     be issued from one thread at a time and are ordered by the stream.
 *   - State vectors are float32.  w, ms and every backup row must be 16-byte
 *     aligned; bak_stride (in elements) must be a multiple of 4 and >= d.
 *   - No call throws or aborts.  int-returning calls return DCASGD_OK or a
 *     negative DCASGD_E* code; pointer-returning calls return NULL and leave
 *     the code in dcasgd_last_error().  Arguments are validated on the host
 *     before anything is launched; a rejected call launches nothing.
 *   - Arithmetic: IEEE binary32, one rounding per operation, no fused
 *     multiply-add, correctly rounded sqrt and division, denormals kept; the
 *     operation order is the one written next to each entry point.
 */
#ifndef DCASGD_H
#define DCASGD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dcasgd_server* dcasgd_t;

/* mode argument of dcasgd_create: one variant, optionally OR-ed with flags */
enum {
    DCASGD_MODE_C       = 0,       /* lambda_t = lambda0 (Section 6, "DC-ASGD-c")          */
    DCASGD_MODE_A       = 1,       /* lambda_t = lambda0/sqrt(MeanSquare(t)+eps), Eq. 18   */
    DCASGD_GRAD_BF16    = 1 << 4,  /* pushed gradients are bfloat16 (2 bytes per element)  */
    DCASGD_PULL_ON_PUSH = 1 << 5,  /* every push also refreshes the pusher's backup        */
    DCASGD_BAK_BF16     = 1 << 6   /* snapshots are handed out and kept as bfloat16        */
};

enum {
    DCASGD_OK      =  0,
    DCASGD_EINVAL  = -1,  /* bad handle, worker id, K, mode, hyper-parameter, NULL pointer, overlap */
    DCASGD_EALIGN  = -2,  /* a pointer or stride breaks the alignment rules above                   */
    DCASGD_ESTATE  = -3,  /* call needs dcasgd_bind / dcasgd_init first                             */
    DCASGD_EHIP    = -4   /* the HIP runtime reported an error at launch                            */
};

#define DCASGD_MAX_K 16   /* longest queue one dcasgd_push_batch call accepts */

/*
 * Create a server for d parameters and M workers (Algorithm 2, "Input").
 * eta: learning rate; lambda0: lambda of Eq. 4.1 (MODE_C) or lambda_0 of
 * Eq. 18 (MODE_A); ema_m: the constant m of Eq. 18, in [0,1) (ignored in
 * MODE_C); eps: the epsilon under the square root (>= 0).
 * Returns NULL if d == 0, M <= 0, the mode is unknown, ema_m is outside
 * [0,1), or a hyper-parameter is not finite.  No GPU call is made.
 */
dcasgd_t dcasgd_create(size_t d, int M, float eta, float lambda0, int mode,
                       float ema_m, float eps);

/* Free the handle (host memory only).  Bound device memory stays the caller's. */
int dcasgd_destroy(dcasgd_t h);

/*
 * Attach caller-owned device memory: w[d] (global model), bak (M rows of
 * bak_stride elements; row m is w_bak(m) of Algorithm 2), ms[d] (MeanSquare of
 * Eq. 18; may be NULL in MODE_C).  The ranges must not overlap.
 * Backup elements are float32, bak_stride a multiple of 4.  With
 * DCASGD_BAK_BF16 (a storage variant, not from the paper, which only remarks
 * that the backups cost memory) they are bfloat16 and bak_stride is a multiple
 * of 8: a pull stores round-to-nearest-even of w, the worker receives that
 * rounded snapshot, and the next push of that worker is compensated against
 * the very same number, so w - w_bak(m) is still the displacement from the
 * point the gradient was taken at.  Half the backup memory and pull traffic;
 * set_launch's streaming level is not honoured by the single-push kernel then.
 */
int dcasgd_bind(dcasgd_t h, float* w, void* bak, size_t bak_stride, float* ms);

/*
 * Algorithm 2, "Initialize": w_bak(m) <- w for every m, MeanSquare <- 0,
 * t <- 0.  w must already hold w_0.  Enqueued on stream.
 */
int dcasgd_init(dcasgd_t h, void* stream);

/*
 * Algorithm 2, "receive g_m": apply one pushed gradient (device pointer, d
 * elements, float32 or bfloat16 per DCASGD_GRAD_BF16, 16-byte aligned;
 * 8-byte for bfloat16).  Per element, in this order (b = w_bak(worker)):
 *   MODE_A only: g2 = g*g; t1 = ema_m*ms; t2 = (1-ema_m)*g2; ms = t1+t2;
 *                den = ms+eps; rt = sqrt(den); lam = lambda0/rt
 *   diff = w-b; g2 = g*g; c1 = lam*g2 (lambda0*g2 in MODE_C); c2 = c1*diff;
 *   gd = g+c2; st = eta*gd; w = w-st                                (Eq. 4.1)
 * then t <- t+1.  With DCASGD_PULL_ON_PUSH the same pass also stores
 * w_bak(worker) <- w (the pull that follows a push in Algorithm 1).
 */
int dcasgd_push(dcasgd_t h, int worker, const void* grad, void* stream);

/*
 * A queue of K pushes, 1 <= K <= DCASGD_MAX_K, defined as
 *   for k in 0..K-1: push(workers[k], grads[k]); pull(workers[k])
 * and computed in one pass per element with w and ms held in registers.
 * workers and grads are host arrays of K entries (grads[k]: device pointer
 * as for dcasgd_push).  A queue that repeats a worker is legal: it is split
 * into consecutive launches at each repeat so that the later push sees the
 * refreshed backup.  Mind what that means for the caller: Eq. 4.1 compensates
 * for w - w_bak(m), the distance from the point the gradient was taken at, so
 * the second gradient of a repeated worker has to have been formed from the
 * snapshot its first entry's pull left - which does not exist yet when one
 * call delivers both.  With one gradient in flight per worker (Algorithm 1)
 * such a queue cannot arise; a caller who does have one delivers it as two
 * calls, forming the later gradient in between.  Handing over a gradient
 * taken at the old snapshot is not detected and is compensated too little.
 */
int dcasgd_push_batch(dcasgd_t h, const int* workers, const void* const* grads,
                      int K, void* stream);

/*
 * Synchronous variant of the supplement ("Large Mini-batch Synchronous SGD
 * with Delay-Compensated Gradient"): J gradients (1 <= J <= DCASGD_MAX_K, host
 * array of device pointers as for dcasgd_push), all taken at the current
 * model w_t, are folded into w one after the other in the given order:
 *   wt^{j+1} = wt^j - (eta_hat/J) * (g_j + lambda g_j*g_j*(wt^j - w_t)),  wt^0 = w_t
 * i.e. the push rule above with eta = eta_hat/J (formed once in binary32) and
 * b = w_t for every j; in MODE_A MeanSquare advances once per gradient.  One
 * pass per element with w_t, w and ms in registers; backups are not touched;
 * t advances by J.  The order is the caller's; dcasgd_sync_fold_ordered below
 * applies the supplement's order heuristic.
 */
int dcasgd_sync_fold(dcasgd_t h, const void* const* grads, int J, float eta_hat, void* stream);

/*
 * The same fold with the order the supplement suggests at the end of that
 * section: the gradients whose running model stays closest to w_t go first,
 * taken here as ascending Euclidean norm of g_j (ties: the caller's order; a
 * gradient whose norm is NaN goes last).  Three launches on the stream: the
 * squared norms (binary64 accumulation of the exact squares, a fixed
 * summation tree, so a repeated call gives the same bits), the ranking, and
 * the fold of dcasgd_sync_fold over the ranked list; no host round trip.
 * workspace: device memory, DCASGD_FOLD_WS_BYTES bytes, 256-byte aligned,
 * caller-owned, overlapping none of the server's vectors or the gradients;
 * contents on entry are irrelevant.  After the call has run it holds, from its
 * start: 16 doubles, |g_j|^2 in the caller's numbering (entries < J valid);
 * at byte 128: 16 int32, perm[r] = caller's index of the r-th gradient folded.
 * Two calls that share a workspace must not overlap in time.
 */
#define DCASGD_FOLD_WS_BYTES 262656
int dcasgd_sync_fold_ordered(dcasgd_t h, const void* const* grads, int J, float eta_hat,
                             void* workspace, void* stream);

/*
 * dcasgd_sync_fold_ordered for callers that cannot allocate device memory and
 * so have no workspace to hand over: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same three launches, same
 * result bits; the workspace is a static array inside the library (262656
 * bytes on every GPU the library runs on, held until the process ends), whose
 * address is looked up once per GPU in dcasgd_init (or on the first call on a
 * GPU that saw no dcasgd_init).  The call itself allocates nothing, creates
 * no events (its launches are not timed even while dcasgd_timing is on) and
 * records no memset.  Limit: J <= DCASGD_MAX_K gradients, any d; a larger J is
 * refused with DCASGD_EINVAL, a failed address lookup with DCASGD_EHIP.
 * Nothing in the array needs clearing between calls (every slot that is read
 * was written earlier in the same call), but all calls on one GPU - from any
 * handle or thread - share it: two that overlap in time race, so keep them on
 * one stream or order them yourself.  The norms and the ranking stay inside
 * the library; callers who want to read them use dcasgd_sync_fold_ordered.
 */
int dcasgd_sync_fold_ordered_static(dcasgd_t h, const void* const* grads, int J, float eta_hat,
                                    void* stream);

/*
 * Only the first two launches of dcasgd_sync_fold_ordered: the squared norms of
 * J gradients and their ranking are left in the workspace (same layout), the
 * model is not touched and t does not advance.  For callers that rank more
 * gradients than one fold call takes and deliver them with dcasgd_sync_fold_part.
 */
int dcasgd_grad_sqnorms(dcasgd_t h, const void* const* grads, int J, void* workspace,
                        void* stream);

/*
 * The same fold delivered in parts, for more same-snapshot gradients than one
 * call takes (large mini-batch SSGD runs on many workers): J of the J_total
 * gradients are applied with the step eta_hat/J_total and compensated against
 * kept_w, the model the whole fold started from (w_t), which the caller kept:
 * device pointer, d floats, 16-byte aligned, not w, ms or the velocity; a
 * float32 backup row qualifies, so dcasgd_pull of a spare worker before the
 * first part is one way to keep it.  Parts applied in sequence leave the bits
 * of the undivided fold.  t advances by J.
 */
int dcasgd_sync_fold_part(dcasgd_t h, const void* const* grads, int J, int J_total,
                          float eta_hat, const float* kept_w, void* stream);

/*
 * Algorithm 2, "pull request": w_bak(worker) <- w, and returns the device
 * pointer of that backup row, which is what "send w_t back to worker m" hands
 * over.  The call has no stream argument: the copy is enqueued on the stream
 * of the most recent call on this handle that changed w - dcasgd_init,
 * dcasgd_push, dcasgd_push_batch, dcasgd_push_synth, dcasgd_run_synth or one
 * of the dcasgd_sync_fold* calls - and on no other (dcasgd_worker_grad,
 * dcasgd_grad_sqnorms, dcasgd_set_momentum and dcasgd_bind_counter leave it
 * alone), so the snapshot is ordered after that update.  A reader of the row
 * on another stream (a worker kernel, say) has to order itself against that
 * stream.  If the row already equals w by the host's bookkeeping (nothing was
 * pushed since it was last refreshed) nothing is launched; after launches the
 * host did not see (graph replays) dcasgd_set_step resets that bookkeeping.
 * NULL on error.  With DCASGD_BAK_BF16 the row holds bfloat16 values and the
 * pointer is to be cast accordingly.
 */
const float* dcasgd_pull(dcasgd_t h, int worker);

/* Number of pushes applied so far (the t of Algorithm 2). */
uint64_t dcasgd_step(dcasgd_t h);

/* Code of the most recent failed call on this handle (DCASGD_OK if none). */
int dcasgd_last_error(dcasgd_t h);

/* Static, human-readable text for a status code. */
const char* dcasgd_strerror(int code);

/*
 * Momentum variant.  Section 6 mentions momentum variants in a footnote and
 * gives no formula; this is the classical heavy ball applied to the
 * delay-compensated gradient g_dc of Eq. 4.1, one velocity per server:
 *   mv = mu*v; v = mv+g_dc; st = eta*v; w = w-st
 * It applies to every later dcasgd_push, dcasgd_push_batch, dcasgd_push_synth
 * and dcasgd_sync_fold.  vel: device pointer, d floats, 16-byte aligned, not
 * overlapping the bound state, owned by the caller; it is zeroed on stream.
 * mu == 0 or vel == NULL switches back to the plain update.  Needs
 * dcasgd_bind first.
 */
int dcasgd_set_momentum(dcasgd_t h, float mu, float* vel, void* stream);

/*
 * Launch-bound use (small models): keep a copy of the push counter t in
 * device memory so that sequences of launches can be captured into a HIP
 * graph and replayed.  counter: device pointer to one uint32, 4-byte aligned,
 * owned by the caller, not overlapping the state; it is set to t on stream.
 * From then on every push-type call also enqueues a one-lane kernel that
 * advances it (by 1, K or J), and worker gradients formed through the handle
 * (dcasgd_worker_grad, dcasgd_push_synth) read the push index that keys their
 * noise from it when they run instead of taking it as a launch argument -
 * a replayed graph therefore keeps drawing fresh noise.  NULL unbinds.
 * Replays advance the device counter but not the host's t: call
 * dcasgd_set_step afterwards with the number of pushes really applied (it
 * also forgets which backups are current, so the next dcasgd_pull copies).
 */
int dcasgd_bind_counter(dcasgd_t h, uint32_t* counter, void* stream);
int dcasgd_set_step(dcasgd_t h, uint64_t t);

/*
 * Synthetic worker through the handle: the gradient of worker's current
 * backup, as dcasgd_synth_grad would form it with push_idx = t + offset
 * (t read from the device counter if one is bound), written to grad_out in
 * the handle's gradient type.  offset lets a queue of K gradients be formed
 * before the K pushes are applied.
 */
int dcasgd_worker_grad(dcasgd_t h, int worker, const float* hdiag, const float* wstar,
                       float sigma, uint64_t seed, uint32_t offset, void* grad_out, void* stream);

/*
 * Per-launch timing of the server-update kernels (push, pull, push_batch,
 * push_synth, sync_fold, and run_synth: one launch per block of up to 64
 * arrivals).  While enabled, every such launch carries its own
 * start and stop HIP events, attached to the kernel itself, so their distance
 * is the kernel's execution time with no dispatch gap in it.  Events are host
 * objects created on demand and reused.  Do not enable it around launches
 * that are being captured into a HIP graph.
 * dcasgd_timing(h, enable) waits for the timed launches still in flight,
 * then switches it and forgets unread launches;
 * dcasgd_timing_read waits for the last timed launch, returns the summed
 * kernel time in milliseconds and the number of launches since the last read
 * (host pointers), and starts a new interval.  At most 65536 launches are
 * timed between two reads; later ones run untimed and are not counted in
 * *launches, so a reader who knows how many launches it issued can tell.
 */
int dcasgd_timing(dcasgd_t h, int enable);
int dcasgd_timing_read(dcasgd_t h, double* total_ms, uint64_t* launches);
/* The same read, launch by launch: each_ms[i] (host array of `capacity` floats)
 * receives the duration of the i-th timed launch since the last read, in launch
 * order, for i < min(*launches, capacity). */
int dcasgd_timing_read_each(dcasgd_t h, float* each_ms, size_t capacity, uint64_t* launches);

/*
 * Change the learning rate for all later pushes (the experiments of Section 6
 * divide it by ten at fixed epochs).  Pushes already enqueued keep the value
 * they were launched with.  eta must be finite.
 */
int dcasgd_set_eta(dcasgd_t h, float eta);

/*
 * Algorithm 2 lists a time-indexed lambda_t as its input: change lambda
 * (MODE_C) or lambda_0 of Eq. 18 (MODE_A) for all later pushes.  Must be finite.
 */
int dcasgd_set_lambda(dcasgd_t h, float lambda0);

/*
 * Launch shape used by this handle's kernels.  threads: 64..512, a multiple
 * of 64; items: float4 groups per thread, one of 1, 2, 4; max_blocks: 0 = one
 * block per tile, otherwise blocks loop over tiles; streaming: 0 = plain
 * accesses, 1 = gradient reads and backup reads/writes non-temporal, 2 = w
 * and MeanSquare accesses non-temporal as well, 3 = level 2 and in addition
 * dcasgd_worker_grad reads its snapshot and writes its gradient non-temporally
 * (at levels 0-2 it leaves both cacheable, so that a push that follows soon
 * finds them in the last-level cache when they fit; level 3 is the setting
 * that measures the update against HBM alone).  A zero/negative threads or
 * items keeps the current value.  Defaults: 256 threads (64 for the queue
 * kernel); items by size (push and pull kernels: 2, the worker-fused push:
 * 1, and 4 for both from d = 2^26 parameters on); one block per tile;
 * streaming 2.  dcasgd_run_synth honours max_blocks and streaming (plain at
 * level 0, non-temporal otherwise) but chooses its own shape: one float4 group
 * per lane (two lanes per group for vectors shorter than 2^17 groups, which
 * would otherwise leave most of the chip idle), 64 threads per block below
 * 2^20 lanes and 256 from there on, and a block of its own for the d mod 4
 * last parameters.
 */
int dcasgd_set_launch(dcasgd_t h, int threads, int items, int max_blocks, int streaming);

/*
 * Stand-in for Algorithm 1's "compute gradient" on a synthetic diagonal
 * quadratic (not from the paper): for i < d
 *   dd = snap[i]-wstar[i]; p = hdiag[i]*dd; nz = sigma*z_i; g = p+nz
 * where z_i is a standard normal drawn from Philox4x32-10 (key = seed,
 * counter = (i/4, push_idx, 0, 0), four normals per counter by Box-Muller in
 * +,-,*,/,sqrt only).  formats: bit 0 set = grad_out is bfloat16[d] (round to
 * nearest even), else float32[d]; bit 1 set = snap is bfloat16[d] (a backup
 * row of a DCASGD_BAK_BF16 server), else float32[d]; bit 2 set = the snapshot
 * read and the gradient write are non-temporal (nothing of this launch is
 * meant to stay in the last-level cache), else cacheable.  All pointers are device
 * pointers, 16-byte aligned (8-byte for a bfloat16 vector).  threads/items as
 * in dcasgd_set_launch (0 = defaults).
 */
int dcasgd_synth_grad(const void* snap, const float* hdiag, const float* wstar,
                      float sigma, uint64_t seed, uint32_t push_idx,
                      void* grad_out, int formats, size_t d, void* stream,
                      int threads, int items);

/*
 * Synthetic workload only: worker and push in one pass.  Equivalent to
 *   dcasgd_synth_grad(w_bak(worker), hdiag, wstar, sigma, seed, push_idx = t, g, ...);
 *   dcasgd_push(h, worker, g, stream);
 * (same bits, gradient rounded to bfloat16 in between if DCASGD_GRAD_BF16)
 * but the gradient stays in registers: 32 bytes of traffic per parameter
 * instead of 16 + 28.  hdiag, wstar: device pointers, d floats, 16-byte
 * aligned, not overlapping the bound state.  Honours DCASGD_PULL_ON_PUSH.
 */
int dcasgd_push_synth(dcasgd_t h, int worker, const float* hdiag, const float* wstar,
                      float sigma, uint64_t seed, void* stream);

/*
 * The event loop of Algorithms 1 and 2 for the synthetic workload, driven from
 * native code: the state the call leaves is, bit for bit, that of
 *   for e < T: dcasgd_push_synth(h, workers[e], hdiag, wstar, sigma, seed, stream)
 * i.e. worker workers[e] delivers the gradient of its snapshot, the server
 * applies it and (with DCASGD_PULL_ON_PUSH) hands the new model back.
 * workers: host array, read before the call returns.  The whole list and the
 * other arguments are validated before the first launch.  Both algorithms act
 * on each parameter by itself, so the arrivals are not launched one by one:
 * one launch covers up to 64 consecutive arrivals, each lane keeps its
 * parameters of w, MeanSquare, hdiag and wstar in registers over them, and per
 * arrival only the pusher's backup row is read and (with the fused pull)
 * written - about 8 bytes per parameter and arrival instead of 32, and one
 * launch per 64 arrivals, which is what matters for small models.  A worker
 * may appear any number of times.  t advances by T; with a bound counter the
 * noise is keyed at execution time as for dcasgd_push_synth.  (More than
 * 65536 workers: arrival-by-arrival launches.)
 */
int dcasgd_run_synth(dcasgd_t h, const int* workers, size_t T, const float* hdiag,
                     const float* wstar, float sigma, uint64_t seed, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* DCASGD_H */
