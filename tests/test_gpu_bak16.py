"""GPU parity for bfloat16 snapshots (DCASGD_BAK_BF16): every entry point that
reads or writes a backup row, against the oracle's bfloat16-snapshot mode, bit
for bit through the C ABI."""
import sys

import numpy as np
import pytest

import oracle
from paper_1609_08326_amd import workloads as W

from gpu_harness import DeviceRun, assert_same_bits, compare, oracle_run

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def small(d, M=3, T=24, mode=W.MODE_A, bf16=False, order="iid", K=1, seed=78):
    return W.Workload("small16", d=d, M=M, T=T, mode=mode, eta=0.1,
                      lambda0=2.0 if mode == W.MODE_A else 0.04, ema_m=0.95, eps=1e-7,
                      h_lo=1e-3, h_hi=1.0, wstar_sigma=1.0, sigma=0.01, order=order, K=K,
                      grad_bf16=bf16, seed=seed)


@pytest.mark.parametrize("mode", [W.MODE_C, W.MODE_A])
@pytest.mark.parametrize("bf16", [False, True])
@pytest.mark.parametrize("fused", [True, False])
def test_small_sizes_every_tail(mode, bf16, fused):
    for d in (1, 3, 4, 5, 7, 8, 9, 255, 256, 1023, 1025, 2048 + 3, 40000 + 1):
        for launch in (None, dict(threads=64, items=1), dict(threads=128, items=4),
                       dict(threads=512, items=2, max_blocks=3)):
            wl = small(d, mode=mode, bf16=bf16)
            say("bak16 d=%d mode=%d bf16=%s fused=%s launch=%s" % (d, mode, bf16, fused, launch))
            run = DeviceRun(wl, fused=fused, launch=launch, bak_bf16=True)
            ref = oracle_run(wl, run.hdiag_host, run.wstar_host, run.arrivals, nthreads=1,
                             bak_bf16=True)
            compare(run, ref, tag="bak16 d=%d" % d)


@pytest.mark.parametrize("mode", [W.MODE_C, W.MODE_A])
def test_queue_with_bfloat16_backups(mode):
    for d in (3, 257, 4096 + 2, 70001):
        for K in (1, 5, 16):
            wl = small(d, M=16, T=3 * K, mode=mode, order="queues", K=K)
            say("bak16 batch d=%d K=%d mode=%d" % (d, K, mode))
            run = DeviceRun(wl, batched=True, bak_bf16=True)
            ref = oracle_run(wl, run.hdiag_host, run.wstar_host, run.arrivals, nthreads=1,
                             bak_bf16=True)
            compare(run, ref, tag="bak16 batched d=%d K=%d" % (d, K))
    wl = small(5003, M=4, T=32, order="iid", K=8, seed=5)
    run = DeviceRun(wl, batched=True, bak_bf16=True)          # queues that repeat a worker
    ref = oracle_run(wl, run.hdiag_host, run.wstar_host, run.arrivals, nthreads=1, bak_bf16=True)
    compare(run, ref, tag="bak16 repeats")


def test_momentum_with_bfloat16_backups():
    wl = small(20011, M=4, T=30)
    run = DeviceRun(wl, momentum=0.9, bak_bf16=True)
    ref = oracle_run(wl, run.hdiag_host, run.wstar_host, run.arrivals, nthreads=1, momentum=0.9,
                     bak_bf16=True)
    compare(run, ref, tag="bak16 momentum")


@pytest.mark.parametrize("mode", [W.MODE_C, W.MODE_A])
@pytest.mark.parametrize("bf16", [False, True])
def test_worker_fused_push_and_worker_grad(mode, bf16):
    import torch
    from paper_1609_08326_amd import binding as B
    for d in (1, 6, 1027, 50001):
        wl = small(d, M=3, T=14, mode=mode, bf16=bf16)
        hd_h, ws_h, order = wl.hdiag(), wl.wstar(), wl.arrivals()
        hd, ws = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
        say("bak16 push_synth d=%d mode=%d bf16=%s" % (d, mode, bf16))
        sv = B.Server(torch.from_numpy(wl.w0()).cuda(), wl.M, wl.eta, wl.lambda0, wl.mode,
                      wl.ema_m, wl.eps, grad_bf16=bf16, pull_on_push=True, bak_bf16=True)
        g = torch.empty(d, dtype=sv.grad_dtype, device="cuda")
        for i, m in enumerate(order):
            if i % 2:
                sv.push_synth(int(m), hd, ws, wl.sigma, wl.seed)
            else:
                sv.worker_grad(int(m), hd, ws, wl.sigma, wl.seed, g)
                sv.push(int(m), g)
        torch.cuda.synchronize()
        ref = oracle.Server(wl.w0(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
        ref.set_backup_bf16()
        ref.run(order, hd_h, ws_h, wl.sigma, wl.seed, as_bf16=bf16)
        assert_same_bits(sv.w.cpu().numpy(), ref.w(), "bak16 push_synth w")
        for m in range(wl.M):
            assert_same_bits(sv.bak[m, :d].float().cpu().numpy(), ref.bak(m), "bak16 bak[%d]" % m)


def test_pull_returns_the_rounded_model_and_rows_are_bfloat16():
    import torch
    from paper_1609_08326_amd import binding as B
    rng = np.random.default_rng(11)
    d = 30011
    w0 = (rng.standard_normal(d) * np.exp(rng.uniform(-30, 30, d))).astype(np.float32)
    sv = B.Server(torch.from_numpy(w0).cuda(), 2, 0.1, 0.04, B.MODE_C, bak_bf16=True)
    assert sv.bak.dtype == torch.bfloat16 and sv.bak.element_size() == 2
    torch.cuda.synchronize()
    want = torch.from_numpy(w0).to(torch.bfloat16)
    assert torch.equal(sv.bak[0, :d].cpu(), want) and torch.equal(sv.bak[1, :d].cpu(), want)
    g = torch.from_numpy(rng.standard_normal(d).astype(np.float32)).cuda()
    sv.push(1, g)
    row = sv.pull(1)
    torch.cuda.synchronize()
    assert row.dtype == torch.bfloat16
    assert torch.equal(row.cpu(), sv.w.cpu().to(torch.bfloat16))
    assert torch.equal(sv.bak[0, :d].cpu(), want)


def test_bind_checks_the_stride_for_the_format():
    import torch
    from paper_1609_08326_amd import binding as B
    lib = B.load()
    h = lib.dcasgd_create(100, 2, 0.1, 0.04, B.MODE_C | B.BAK_BF16, 0.0, 0.0)
    w = torch.zeros(100, device="cuda")
    bak = torch.zeros((2, 128), dtype=torch.bfloat16, device="cuda")
    assert lib.dcasgd_bind(h, w.data_ptr(), bak.data_ptr(), 100, None) == B.EALIGN   # 100 % 8 != 0
    assert lib.dcasgd_bind(h, w.data_ptr(), bak.data_ptr(), 96, None) == B.EINVAL    # shorter than d
    assert lib.dcasgd_bind(h, w.data_ptr(), bak.data_ptr(), 104, None) == B.OK
    lib.dcasgd_destroy(h)
    assert not lib.dcasgd_create(100, 2, 0.1, 0.04, B.MODE_C | (1 << 7), 0.0, 0.0)


@pytest.mark.parametrize("cfg", [2, 4])
def test_config_full_size_sampled(cfg):
    """The benchmark's configurations 2 and 4 with bfloat16 snapshots, full size,
    default launch shape; the oracle follows a seeded sample through every push."""
    wl = W.CONFIGS[cfg]
    say("bak16 full-size sampled config %s" % wl.name)
    run = DeviceRun(wl, bak_bf16=True)
    idx = wl.sample_indices(150_000, edge=4096)
    ref = oracle_run(wl, run.hdiag_host, run.wstar_host, run.arrivals, idx=idx, nthreads=16,
                     bak_bf16=True)
    compare(run, ref, idx=idx, tag="bak16 " + wl.name)
    assert np.all(np.isfinite(run.w))
