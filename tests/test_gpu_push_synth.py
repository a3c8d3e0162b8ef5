"""GPU parity for the worker+push fusion (synthetic workload only): the fused
launch must leave the same bits as the oracle's event loop, which is also
what the separate worker and push launches produce."""
import sys

import numpy as np
import pytest

import oracle
from paper_1609_08326_amd import workloads as W

from gpu_harness import DeviceRun, assert_same_bits, oracle_run

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def run_fused(wl, fused_pull=True, launch=None):
    import torch
    from paper_1609_08326_amd import binding as B
    hd_h, ws_h, order = wl.hdiag(), wl.wstar(), wl.arrivals()
    hd, ws = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    sv = B.Server(torch.from_numpy(wl.w0()).cuda(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m,
                  wl.eps, grad_bf16=wl.grad_bf16, pull_on_push=fused_pull)
    if launch:
        sv.set_launch(**launch)
    for m in order:
        sv.push_synth(int(m), hd, ws, wl.sigma, wl.seed)
        if not fused_pull:
            sv.pull(int(m))
    torch.cuda.synchronize()
    assert sv.t == len(order)
    return sv, hd_h, ws_h, order


def check(sv, ref, wl, idx=None):
    sel = (lambda a: a) if idx is None else (lambda a: a[idx.astype(np.int64)])
    assert_same_bits(sel(sv.w.cpu().numpy()), ref.w(), "w")
    if sv.ms is not None:
        assert_same_bits(sel(sv.ms.cpu().numpy()), ref.ms(), "ms")
    bak = sv.bak[:, : wl.d].cpu().numpy()
    for m in range(wl.M):
        assert_same_bits(sel(bak[m]), ref.bak(m), "bak[%d]" % m)


@pytest.mark.parametrize("mode", [W.MODE_C, W.MODE_A])
@pytest.mark.parametrize("bf16", [False, True])
def test_push_synth_small_sizes(mode, bf16):
    for d in (1, 3, 4, 6, 1023, 2048 + 1, 50001):
        for fused_pull, launch in ((True, None), (False, dict(threads=64, items=4)),
                                   (True, dict(threads=512, items=1, max_blocks=2))):
            wl = W.Workload("small", d=d, M=3, T=20, mode=mode, eta=0.1,
                            lambda0=2.0 if mode == W.MODE_A else 0.04, ema_m=0.95, eps=1e-7,
                            h_lo=1e-3, h_hi=1.0, wstar_sigma=1.0, sigma=0.01, order="iid",
                            grad_bf16=bf16, seed=91)
            say("push_synth d=%d mode=%d bf16=%s pull=%s launch=%s" % (d, mode, bf16, fused_pull, launch))
            sv, hd_h, ws_h, order = run_fused(wl, fused_pull, launch)
            ref = oracle_run(wl, hd_h, ws_h, order, nthreads=1)
            check(sv, ref, wl)


@pytest.mark.parametrize("cfg", [2, 4])
def test_push_synth_full_size_sampled(cfg):
    wl = W.CONFIGS[cfg]
    if cfg == 4:
        wl = wl.replace(T=24)
    say("push_synth full size %s" % wl.name)
    sv, hd_h, ws_h, order = run_fused(wl)
    idx = wl.sample_indices(100_000, edge=4096)
    ref = oracle_run(wl, hd_h, ws_h, order, idx=idx, nthreads=16)
    check(sv, ref, wl, idx=idx)


def test_push_synth_equals_separate_launches():
    wl = W.CONFIGS[1].replace(T=60)
    sv, _, _, _ = run_fused(wl)
    plain = DeviceRun(wl)
    assert_same_bits(sv.w.cpu().numpy(), plain.w, "fused vs separate w")
    assert_same_bits(sv.ms.cpu().numpy(), plain.ms, "fused vs separate ms")
    assert_same_bits(sv.bak[:, : wl.d].cpu().numpy().ravel(), plain.bak.ravel(), "fused vs separate bak")


def test_vector_longer_than_4_gib():
    """d = 2^30 + 3: byte offsets inside one vector pass 2^32, the float4 group
    index passes 2^28.  Worker-fused pushes and a separate worker + push, checked
    on a sample that includes both ends of the vector."""
    import torch
    from paper_1609_08326_amd import binding as B
    wl = W.CONFIGS[2].replace(name="huge", d=(1 << 30) + 3, M=1, T=3)
    say("huge vector d=%d" % wl.d)
    hd_h, ws_h = wl.hdiag(), wl.wstar()
    hd, ws = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    sv = B.Server(torch.zeros(wl.d, device="cuda"), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m,
                  wl.eps, pull_on_push=True)
    sv.push_synth(0, hd, ws, wl.sigma, wl.seed)
    sv.push_synth(0, hd, ws, wl.sigma, wl.seed)
    g = torch.empty(wl.d, device="cuda")
    B.synth_grad(sv.snapshot(0), hd, ws, wl.sigma, wl.seed, 2, g)
    sv.push(0, g)
    torch.cuda.synchronize()
    idx = wl.sample_indices(100_000, edge=4096)
    ii = torch.from_numpy(idx.astype(np.int64)).cuda()
    ref = oracle_run(wl, hd_h, ws_h, np.zeros(3, dtype=np.int32), idx=idx, nthreads=16)
    assert_same_bits(sv.w[ii].cpu().numpy(), ref.w(), "huge w")
    assert_same_bits(sv.ms[ii].cpu().numpy(), ref.ms(), "huge ms")
    assert_same_bits(sv.bak[0][ii].cpu().numpy(), ref.bak(0), "huge bak")
    # nothing beyond the sample is left untouched: w moved everywhere h is not tiny
    assert int((sv.w == 0).sum().item()) < wl.d // 1000


def test_native_event_loop_matches_oracle_and_validates_first():
    import torch
    from paper_1609_08326_amd import binding as B
    wl = W.CONFIGS[1].replace(T=120)
    hd_h, ws_h, order = wl.hdiag(), wl.wstar(), wl.arrivals()
    hd, ws = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    sv = B.Server(torch.from_numpy(wl.w0()).cuda(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m,
                  wl.eps, pull_on_push=True)
    bad = [int(m) for m in order[:10]] + [wl.M]
    with pytest.raises(B.DcasgdError):
        sv.run_synth(bad, hd, ws, wl.sigma, wl.seed)
    torch.cuda.synchronize()
    assert sv.t == 0                                   # nothing was launched for the bad list
    sv.run_synth(order[:50], hd, ws, wl.sigma, wl.seed)
    sv.run_synth([], hd, ws, wl.sigma, wl.seed)
    sv.run_synth(order[50:], hd, ws, wl.sigma, wl.seed)
    torch.cuda.synchronize()
    ref = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    ref.run(order, hd_h, ws_h, wl.sigma, wl.seed, nthreads=8)
    assert sv.t == ref.t == len(order)
    assert_same_bits(sv.w.cpu().numpy(), ref.w(), "native loop w")
    assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), "native loop ms")
    for m in range(wl.M):
        assert_same_bits(sv.bak[m, : wl.d].cpu().numpy(), ref.bak(m), "native loop bak[%d]" % m)


# ---- the event loop that keeps a lane's parameters in registers over a block of arrivals ----

def run_blocks(wl, order, fused_pull=True, bak_bf16=False, momentum=0.0, pieces=None, launch=None):
    """dcasgd_run_synth over `order`, delivered in the given pieces (list lengths)."""
    import torch
    from paper_1609_08326_amd import binding as B
    hd_h, ws_h = wl.hdiag(), wl.wstar()
    hd, ws = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    sv = B.Server(torch.from_numpy(wl.w0()).cuda(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m,
                  wl.eps, grad_bf16=wl.grad_bf16, pull_on_push=fused_pull, bak_bf16=bak_bf16)
    if momentum:
        sv.set_momentum(momentum)
    if launch:
        sv.set_launch(**launch)
    at = 0
    for n in (pieces or [len(order)]):
        sv.run_synth(order[at:at + n], hd, ws, wl.sigma, wl.seed)
        at += n
    assert at == len(order)
    torch.cuda.synchronize()
    assert sv.t == len(order)
    return sv, hd_h, ws_h


def check_blocks(sv, ref, wl, idx=None, bak_bf16=False):
    import torch
    sel = (lambda a: a) if idx is None else (lambda a: a[idx.astype(np.int64)])
    assert_same_bits(sel(sv.w.cpu().numpy()), ref.w(), "w")
    if sv.ms is not None:
        assert_same_bits(sel(sv.ms.cpu().numpy()), ref.ms(), "ms")
    rows = sv.bak[:, : wl.d]
    if bak_bf16:
        rows = rows.to(torch.float32)          # exact widening; the oracle holds the rounded values
    rows = rows.cpu().numpy()
    for m in range(wl.M):
        assert_same_bits(sel(rows[m]), ref.bak(m), "bak[%d]" % m)
    if sv.vel is not None:
        assert_same_bits(sel(sv.vel.cpu().numpy()), ref.vel(), "velocity")


def small(d, M, T, mode, order="iid", bf16=False, seed=17):
    return W.Workload("blocks", d=d, M=M, T=T, mode=mode, eta=0.1,
                      lambda0=2.0 if mode == W.MODE_A else 0.04, ema_m=0.95, eps=1e-7,
                      h_lo=1e-3, h_hi=1.0, wstar_sigma=1.0, sigma=0.01, order=order,
                      grad_bf16=bf16, seed=seed)


@pytest.mark.parametrize("mode", [W.MODE_C, W.MODE_A])
@pytest.mark.parametrize("bf16", [False, True])
def test_blocks_of_arrivals_small_sizes(mode, bf16):
    """150 arrivals = launches of 64, 64 and 22; M = 3 makes workers return at once and later."""
    for d in (1, 3, 4, 6, 1023, 2048 + 1, 50001):
        wl = small(d, 3, 150, mode, bf16=bf16)
        order = wl.arrivals()
        assert np.any(order[1:] == order[:-1]) and len(set(order.tolist())) == 3
        say("run_synth blocks d=%d mode=%d bf16=%s" % (d, mode, bf16))
        sv, hd_h, ws_h = run_blocks(wl, order)
        ref = oracle_run(wl, hd_h, ws_h, order, nthreads=1)
        check_blocks(sv, ref, wl)


@pytest.mark.parametrize("bak_bf16", [False, True])
@pytest.mark.parametrize("momentum", [0.0, 0.5])
def test_blocks_of_arrivals_with_rounded_snapshots_and_momentum(bak_bf16, momentum):
    for mode in (W.MODE_C, W.MODE_A):
        for d in (7, 4096 + 2, 30011):
            wl = small(d, 4, 131, mode, seed=23).replace(eta=0.03)   # momentum needs the smaller step
            order = wl.arrivals()
            say("run_synth blocks d=%d mode=%d bak_bf16=%s momentum=%s" % (d, mode, bak_bf16, momentum))
            sv, hd_h, ws_h = run_blocks(wl, order, bak_bf16=bak_bf16, momentum=momentum,
                                        pieces=[1, 63, 64, 3])
            ref = oracle_run(wl, hd_h, ws_h, order, nthreads=1, momentum=momentum, bak_bf16=bak_bf16)
            check_blocks(sv, ref, wl, bak_bf16=bak_bf16)


def test_blocks_of_arrivals_special_orders():
    """One worker only (every backup comes from registers), round robin (no worker twice in
    a row), and a launch grid smaller than the vector (lanes walk several groups)."""
    for M, order_kind, launch in ((1, "iid", None), (4, "round_robin", None),
                                  (5, "iid", dict(max_blocks=3))):
        for mode in (W.MODE_C, W.MODE_A):
            wl = small(20011, M, 140, mode, order=order_kind, seed=29).replace(eta=0.05)
            order = wl.arrivals()
            say("run_synth blocks M=%d order=%s launch=%s mode=%d" % (M, order_kind, launch, mode))
            sv, hd_h, ws_h = run_blocks(wl, order, launch=launch)
            ref = oracle_run(wl, hd_h, ws_h, order, nthreads=1)
            check_blocks(sv, ref, wl)


def test_blocks_of_arrivals_without_the_fused_pull_equal_single_launches():
    """No pull on push: backups stay where the explicit pulls left them, so a block of
    arrivals is a block of plain delayed-gradient steps; checked against the same arrivals
    delivered one launch each."""
    import torch
    for mode in (W.MODE_C, W.MODE_A):
        wl = small(30011, 3, 100, mode, seed=31)
        order = wl.arrivals()
        sv, _, _ = run_blocks(wl, order, fused_pull=False)
        one, _, _, _ = run_fused(wl.replace(T=0), fused_pull=False)
        hd = torch.from_numpy(wl.hdiag()).cuda()
        ws = torch.from_numpy(wl.wstar()).cuda()
        for m in order:
            one.push_synth(int(m), hd, ws, wl.sigma, wl.seed)
        torch.cuda.synchronize()
        assert_same_bits(sv.w.cpu().numpy(), one.w.cpu().numpy(), "no-pull blocks w")
        if mode == W.MODE_A:
            assert_same_bits(sv.ms.cpu().numpy(), one.ms.cpu().numpy(), "no-pull blocks ms")
        assert_same_bits(sv.bak[:, : wl.d].cpu().numpy().ravel(),
                         one.bak[:, : wl.d].cpu().numpy().ravel(), "no-pull blocks bak")
        # and against the oracle: pushes only, no pull in between
        ref = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
        hd_h, ws_h = wl.hdiag(), wl.wstar()
        for t, m in enumerate(order):
            ref.push(int(m), oracle.synth_grad(ref.bak(int(m)), hd_h, ws_h, wl.sigma, wl.seed, t))
        assert_same_bits(sv.w.cpu().numpy(), ref.w(), "no-pull blocks w vs oracle")


@pytest.mark.parametrize("cfg", [2, 4])
def test_blocks_of_arrivals_full_size(cfg):
    """Configuration 2: every element through all 200 arrivals; configuration 4: a sample of
    100 k elements (both ends of the vector included) through 24 arrivals."""
    wl = W.CONFIGS[cfg]
    if cfg == 4:
        wl = wl.replace(T=24)
    order = wl.arrivals()
    say("run_synth blocks full size %s" % wl.name)
    sv, hd_h, ws_h = run_blocks(wl, order)
    idx = wl.sample_indices(100_000, edge=4096) if cfg == 4 else None
    ref = oracle_run(wl, hd_h, ws_h, order, idx=idx, nthreads=16)
    check_blocks(sv, ref, wl, idx=idx)


def test_more_workers_than_the_block_kernel_names_fall_back_to_single_launches():
    """The block kernel names a worker in 16 bits; a server with more workers than that gets
    the same arrivals launched one by one (tiny vectors, so 70000 backups are a few megabytes)."""
    wl = small(6, 70000, 0, W.MODE_A, seed=37)
    order = np.array([69999, 0, 65536, 69999, 69999, 65535, 1, 0, 65536, 3], dtype=np.int32)
    sv, hd_h, ws_h = run_blocks(wl, order)
    ref = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    ref.run(order, hd_h, ws_h, wl.sigma, wl.seed)
    assert_same_bits(sv.w.cpu().numpy(), ref.w(), "many workers w")
    assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), "many workers ms")
    rows = sv.bak[:, : wl.d].cpu().numpy()
    for m in sorted(set(order.tolist())) + [2, 40000]:
        assert_same_bits(rows[m], ref.bak(m), "many workers bak[%d]" % m)


@pytest.mark.parametrize("mode", [W.MODE_C, W.MODE_A])
def test_blocks_of_arrivals_both_lane_layouts_every_element(mode):
    """Vectors shorter than 2^17 groups of four get two lanes per group, longer ones one lane per
    group: one size on each side of the switch, and one just past it with a ragged tail, every
    element compared."""
    for d in ((1 << 19) - 4, 1 << 19, (1 << 19) + 7):
        wl = small(d, 5, 100, mode, seed=41).replace(eta=0.05)
        order = wl.arrivals()
        say("run_synth blocks d=%d mode=%d" % (d, mode))
        sv, hd_h, ws_h = run_blocks(wl, order)
        ref = oracle_run(wl, hd_h, ws_h, order, nthreads=16)
        check_blocks(sv, ref, wl)
