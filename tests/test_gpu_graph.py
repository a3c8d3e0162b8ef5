"""Launch-bound use: with the push counter kept in device memory a block of
arrivals (worker gradient + push, or the fused launch) is captured into a HIP
graph once and replayed; every replay must land on the oracle's bits, i.e. the
noise keeps advancing although the launch arguments are frozen."""
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


def workload(d=60013, M=4, mode=W.MODE_A):
    return W.Workload("graph", d=d, M=M, T=8, mode=mode, eta=0.05,
                      lambda0=2.0 if mode == W.MODE_A else 0.04, ema_m=0.95, eps=1e-7,
                      h_lo=1e-3, h_hi=1.0, wstar_sigma=1.0, sigma=0.01, order="iid", seed=404)


def check(sv, ref, wl, tag):
    assert_same_bits(sv.w.cpu().numpy(), ref.w(), tag + " w")
    if sv.ms is not None:
        assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), tag + " ms")
    for m in range(wl.M):
        assert_same_bits(sv.bak[m, : wl.d].cpu().numpy(), ref.bak(m), tag + " bak[%d]" % m)


@pytest.mark.parametrize("streaming", [2, 3])
def test_counter_bound_eager_path_matches_oracle(streaming):
    """(streaming 3: the worker kernel issued through the handle leaves nothing cached;
    a cache policy changes no bit.)"""
    import torch
    from paper_1609_08326_amd import binding as B
    wl = workload()
    hd_h, ws_h, order = wl.hdiag(), wl.wstar(), wl.arrivals()
    hd, ws = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    sv = B.Server(torch.from_numpy(wl.w0()).cuda(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m,
                  wl.eps, pull_on_push=True)
    sv.set_launch(streaming=streaming)
    g = torch.empty(wl.d, device="cuda")
    sv.push_synth(int(order[0]), hd, ws, wl.sigma, wl.seed)       # t = 1 before binding
    sv.bind_counter()
    for m in order[1:5]:
        sv.worker_grad(int(m), hd, ws, wl.sigma, wl.seed, g)
        sv.push(int(m), g)
    sv.push_synth(int(order[5]), hd, ws, wl.sigma, wl.seed)
    sv.run_synth(order[6:], hd, ws, wl.sigma, wl.seed)            # the block kernel reads the counter too
    torch.cuda.synchronize()
    assert int(sv.counter.item()) == sv.t == len(order)
    ref = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    ref.run(order, hd_h, ws_h, wl.sigma, wl.seed)
    check(sv, ref, wl, "eager with device counter")


@pytest.mark.parametrize("fused_worker", [False, True, "one launch for the block"])
@pytest.mark.parametrize("mode", [W.MODE_C, W.MODE_A])
def test_replayed_block_of_arrivals_keeps_matching_the_oracle(fused_worker, mode):
    import torch
    from paper_1609_08326_amd import binding as B
    wl = workload(mode=mode)
    hd_h, ws_h, block = wl.hdiag(), wl.wstar(), wl.arrivals()
    say("graph replay fused_worker=%s mode=%d block=%s" % (fused_worker, mode, block.tolist()))
    hd, ws = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    w = torch.from_numpy(wl.w0()).cuda()
    g = torch.empty(wl.d, device="cuda")
    side = torch.cuda.Stream()
    torch.cuda.synchronize()

    def one_block(sv):
        if fused_worker == "one launch for the block":
            sv.run_synth(block, hd, ws, wl.sigma, wl.seed)
            return
        for m in block:
            if fused_worker:
                sv.push_synth(int(m), hd, ws, wl.sigma, wl.seed)
            else:
                sv.worker_grad(int(m), hd, ws, wl.sigma, wl.seed, g)
                sv.push(int(m), g)

    with torch.cuda.stream(side):
        sv = B.Server(w, wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps, pull_on_push=True)
        sv.bind_counter()
        one_block(sv)                                   # eager: arrivals 0 .. 7
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_block(sv)                                   # captured, not run
    ref = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    ref.run(block, hd_h, ws_h, wl.sigma, wl.seed)
    other = torch.zeros(1 << 18, device="cuda")
    replays = 4
    for r in range(replays):
        graph.replay()
        torch.cuda.synchronize()
        ref.run(block, hd_h, ws_h, wl.sigma, wl.seed)   # the oracle's t keeps counting
        check(sv, ref, wl, "replay %d" % r)
        assert int(sv.counter.item()) == ref.t
        other.add_(1.0)                                 # unrelated eager work between replays
        torch.cuda.synchronize()
    # the host did not see the replays: resynchronise, then carry on eagerly
    assert sv.t == 2 * len(block)
    sv.set_step(ref.t)
    assert sv.t == ref.t
    with torch.cuda.stream(side):
        m = int(block[0])
        row = sv.pull(m)                                # must really copy after a resync
        one_block(sv)
    side.synchronize()
    ref.run(block, hd_h, ws_h, wl.sigma, wl.seed)
    check(sv, ref, wl, "eager after resync")
    assert row.data_ptr() == sv.bak[m].data_ptr()


def test_counter_calls_reject_bad_arguments():
    import torch
    from paper_1609_08326_amd import binding as B
    lib = B.load()
    sv = B.Server(torch.zeros(1000, device="cuda"), 2, 0.1, 0.04, B.MODE_C)
    c = torch.zeros(4, dtype=torch.int32, device="cuda")
    hd = torch.ones(1000, device="cuda")
    g = torch.ones(1000, device="cuda")
    s = int(torch.cuda.current_stream().cuda_stream)
    assert lib.dcasgd_bind_counter(sv._h, c.data_ptr() + 2, s) == B.EALIGN
    assert lib.dcasgd_bind_counter(sv._h, sv.w.data_ptr(), s) == B.EINVAL
    assert lib.dcasgd_bind_counter(sv._h, c.data_ptr(), s) == B.OK
    assert lib.dcasgd_bind_counter(sv._h, None, s) == B.OK
    assert lib.dcasgd_worker_grad(sv._h, 2, hd.data_ptr(), hd.data_ptr(), 0.1, 1, 0, g.data_ptr(), s) == B.EINVAL
    assert lib.dcasgd_worker_grad(sv._h, 0, hd.data_ptr(), hd.data_ptr(), 0.1, 1, 0, hd.data_ptr(), s) == B.EINVAL
    assert lib.dcasgd_worker_grad(sv._h, 0, hd.data_ptr(), hd.data_ptr(), 0.1, 1, 0, sv.w.data_ptr(), s) == B.EINVAL
    torch.cuda.synchronize()
    assert sv.t == 0
