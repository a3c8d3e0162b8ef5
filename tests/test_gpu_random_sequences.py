"""Differential test of the whole C ABI as a state machine: a seeded random
sequence of calls (pushes, queues with and without repeated workers, pulls,
folds in the caller's order and ranked by norm (caller's and static workspace), worker-fused pushes, blocks
of arrivals through the native event loop, worker gradient + push, step-size and momentum changes) is applied to the library and,
call by call, to the oracle; every vector of the server state must agree bit
for bit at checkpoints and at the end."""
import sys

import numpy as np
import pytest

import oracle
from paper_1609_08326_amd import workloads as W

from gpu_harness import assert_same_bits

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check_state(sv, ref, M, d, tag):
    import torch
    torch.cuda.synchronize()
    assert sv.t == ref.t, tag
    if sv.counter is not None:
        assert int(sv.counter.item()) == ref.t, tag
    assert_same_bits(sv.w.cpu().numpy(), ref.w(), tag + " w")
    if sv.ms is not None:
        assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), tag + " ms")
    if sv.vel is not None:
        assert_same_bits(sv.vel.cpu().numpy(), ref.vel(), tag + " velocity")
    for m in range(M):
        assert_same_bits(sv.bak[m, :d].float().cpu().numpy(), ref.bak(m), tag + " bak[%d]" % m)


@pytest.mark.parametrize("seed", list(range(12)))
def test_random_call_sequence(seed):
    import torch
    from paper_1609_08326_amd import binding as B
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([1, 6, 255, 4099, 20011, 65536 + 3]))
    M = int(rng.integers(1, 7))
    mode = W.MODE_A if seed % 2 else W.MODE_C
    bf16 = bool(seed % 3 == 2)
    fused_pull = bool(rng.integers(0, 2))
    bak16 = bool(seed % 4 == 3 or seed == 8)          # snapshots kept as bfloat16
    lam0 = 2.0 if mode == W.MODE_A else 0.04
    wl = W.Workload("seq", d=d, M=M, T=1, mode=mode, eta=0.05, lambda0=lam0, ema_m=0.95, eps=1e-7,
                    h_lo=1e-3, h_hi=1.0, wstar_sigma=1.0, sigma=0.01, order="iid", seed=77 + seed,
                    grad_bf16=bf16)
    say("sequence seed=%d d=%d M=%d mode=%d bf16=%s pull_on_push=%s bak16=%s"
        % (seed, d, M, mode, bf16, fused_pull, bak16))
    hd_h, ws_h, w0 = wl.hdiag(), wl.wstar(), wl.w0()
    hd, ws = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    sv = B.Server(torch.from_numpy(w0).cuda(), M, wl.eta, lam0, mode, wl.ema_m, wl.eps,
                  grad_bf16=bf16, pull_on_push=fused_pull, bak_bf16=bak16)
    ref = oracle.Server(w0, M, wl.eta, lam0, mode, wl.ema_m, wl.eps)
    if bak16:
        ref.set_backup_bf16()
    if seed % 4 == 1:
        sv.bind_counter()                     # the device-resident copy of t must keep up
    fws = B.Server.fold_workspace()
    gdt = torch.bfloat16 if bf16 else torch.float32
    gscratch = torch.empty(d, dtype=gdt, device="cuda")

    def gradients(n):
        """n random gradients: host float32 values (already bf16-representable if the
        server takes bf16) and the device buffers holding them."""
        scale = rng.uniform(0.02, 0.5, (n, 1))
        g = (scale * rng.standard_normal((n, d))).astype(np.float32)
        gt = torch.from_numpy(g).to(gdt)
        return gt.float().numpy(), [gt[j].contiguous().cuda() for j in range(n)]

    ops = ["push", "batch", "batch_repeat", "pull", "fold", "fold_ranked", "push_synth",
           "worker_then_push", "eta", "momentum", "lambda", "fold_parts", "fold_static"]
    weights = np.array([4, 2, 1, 2, 1, 1, 2, 1, 1, 1, 1, 1, 1], dtype=float)
    trace = []
    loop_rng = np.random.default_rng(5000 + seed)
    lam_now = lam0
    for step in range(90):
        op = str(rng.choice(ops, p=weights / weights.sum()))
        trace.append(op)
        if op == "push":
            m = int(rng.integers(0, M))
            g, dev = gradients(1)
            sv.push(m, dev[0])
            ref.push(m, g[0])
            if fused_pull:
                ref.pull(m)
        elif op in ("batch", "batch_repeat"):
            K = int(rng.integers(1, 17))
            if op == "batch":
                K = min(K, M)
                ms_ = [int(x) for x in rng.permutation(M)[:K]]
            else:
                ms_ = [int(x) for x in rng.integers(0, M, K)]
            g, dev = gradients(K)
            sv.push_batch(ms_, dev)
            for k, m in enumerate(ms_):
                ref.push(m, g[k])
                ref.pull(m)
        elif op == "pull":
            m = int(rng.integers(0, M))
            sv.pull(m)
            ref.pull(m)
        elif op in ("fold", "fold_ranked"):
            J = int(rng.integers(1, 17))
            g, dev = gradients(J)
            eta_hat = float(np.float32(0.05 * J))
            if op == "fold":
                sv.sync_fold(dev, eta_hat)
                ref.sync_fold(g, eta_hat)
            else:
                sv.sync_fold(dev, eta_hat, workspace=fws)
                torch.cuda.synchronize()
                perm = B.Server.fold_order(fws, J)[1]
                want = np.argsort(oracle.grad_sqnorms(g), kind="stable")
                assert perm.tolist() == want.tolist(), (step, perm, want)
                ref.sync_fold(g[want], eta_hat)
        elif op == "fold_static":
            # the ranked fold with the library's static workspace: the order is not handed
            # out, it shows in the folded model
            J = int(rng.integers(1, 17))
            g, dev = gradients(J)
            eta_hat = float(np.float32(0.05 * J))
            sv.sync_fold_ordered_static(dev, eta_hat)
            ref.sync_fold(g[np.argsort(oracle.grad_sqnorms(g), kind="stable")], eta_hat)
        elif op == "fold_parts":
            J = int(rng.integers(17, 41))
            g, dev = gradients(J)
            eta_hat = float(np.float32(0.02 * J))
            kept = sv.w.clone()
            for lo in range(0, J, 16):
                sv.sync_fold_part(dev[lo:lo + 16], J, eta_hat, kept)
            ref.sync_fold(g, eta_hat)
        elif op == "push_synth":
            if not fused_pull:
                continue                      # the fused launch always refreshes the backup
            m = int(rng.integers(0, M))
            sv.push_synth(m, hd, ws, wl.sigma, wl.seed)
            ref.run(np.array([m], dtype=np.int32), hd_h, ws_h, wl.sigma, wl.seed, as_bf16=bf16)
        elif op == "worker_then_push":
            m = int(rng.integers(0, M))
            if sv.counter is not None:
                sv.worker_grad(m, hd, ws, wl.sigma, wl.seed, gscratch)
            else:
                B.synth_grad(sv.snapshot(m), hd, ws, wl.sigma, wl.seed, sv.t, gscratch)
            sv.push(m, gscratch)
            g = oracle.synth_grad(ref.bak(m), hd_h, ws_h, wl.sigma, wl.seed, ref.t, as_bf16=bf16)
            ref.push(m, g)
            if fused_pull:
                ref.pull(m)
        elif op == "eta":
            eta = float(np.float32(rng.choice([0.1, 0.05, 0.01, 0.002])))
            sv.set_eta(eta)
            ref.set_eta(eta)
        elif op == "lambda":
            # includes 0 (plain ASGD for a stretch) and values outside the short-form window
            lam = float(np.float32(rng.choice([0.0, 0.01, 0.04, 1.0, 2.0, 2.0 ** -45, -0.5])))
            sv.set_lambda(lam)
            ref.set_lambda(lam)
            lam_now = lam
        elif op == "momentum":
            mu = float(np.float32(rng.choice([0.0, 0.5, 0.9])))
            torch.cuda.synchronize()          # the old velocity buffer is released here
            sv.set_momentum(mu)
            ref.set_momentum(mu)
        if loop_rng.random() < 0.15 and lam_now >= 0.0:
            # a block of arrivals through the native event loop (its own generator, so the
            # calls above stay what they were before this one existed; not while lambda is
            # negative: dozens of anti-compensated delayed steps in a row diverge)
            trace.append("run_synth")
            block = loop_rng.integers(0, M, int(loop_rng.integers(1, 70))).astype(np.int32)
            sv.run_synth(block, hd, ws, wl.sigma, wl.seed)
            if fused_pull:
                ref.run(block, hd_h, ws_h, wl.sigma, wl.seed, as_bf16=bf16)
            else:
                for m in block:           # no pull: every gradient is taken at the standing backup
                    ref.push(int(m), oracle.synth_grad(ref.bak(int(m)), hd_h, ws_h, wl.sigma,
                                                       wl.seed, ref.t, as_bf16=bf16))
        if step % 23 == 22:
            check_state(sv, ref, M, d, "seed %d after %d calls (%s)" % (seed, step + 1, trace[-5:]))
    check_state(sv, ref, M, d, "seed %d at the end" % seed)
    assert np.all(np.isfinite(ref.w()))
