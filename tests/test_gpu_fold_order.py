"""GPU parity for the ordered synchronous fold (supplement, closing remark of
the large mini-batch section: fold in increasing distance from w_t, read as
ascending gradient norm).  The squared norms are compared with the oracle's
within the bound derived below, the permutation and the folded model bit for
bit, through the C ABI."""
import ctypes as C
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


def norm_tolerance(d):
    """Relative bound on |device - oracle| for a sum of d non-negative exact squares.
    Device: a lane adds 16 terms per tile of 1024 groups it visits (two blocks per
    compute unit share the tiles: at most 13 tiles, 208 additions, at the sizes
    used here), then 6 shuffle steps, 3 wave sums, and in the second launch up to
    32 partials per lane and 6 more shuffle steps: under 256 binary64 roundings on
    any path, each on a partial sum below the total.  Oracle: d roundings at 2^-64."""
    return 256 * 2.0 ** -53 + d * 2.0 ** -64


def device_rows(g, bf16):
    import torch
    if bf16:
        gt = torch.from_numpy(g).to(torch.bfloat16)
        return gt.float().numpy(), [gt[j].contiguous().cuda() for j in range(g.shape[0])]
    return g, [torch.from_numpy(g[j]).cuda() for j in range(g.shape[0])]


def check_order(ws, g_host, J, d, tag):
    """Norms within the bound, the permutation equal to the oracle's stable sort."""
    from paper_1609_08326_amd import binding as B
    sq, perm = B.Server.fold_order(ws, J)
    want = oracle.grad_sqnorms(g_host)
    tol = norm_tolerance(d)
    assert np.all(np.abs(sq - want) <= tol * want), (tag, sq, want)
    order = np.argsort(want, kind="stable")
    gaps = np.diff(want[order])
    exact_tie = gaps == 0.0
    assert np.all(exact_tie | (gaps > 4 * tol * want[order][1:])), "test input: order not separated"
    assert perm.tolist() == order.tolist(), (tag, perm, order)
    return order


@pytest.mark.parametrize("mode", [W.MODE_C, W.MODE_A])
@pytest.mark.parametrize("bf16", [False, True])
def test_ordered_fold_small_sizes(mode, bf16):
    import torch
    from paper_1609_08326_amd import binding as B
    rng = np.random.default_rng(29)
    lam0 = 2.0 if mode == W.MODE_A else 0.04
    ws = B.Server.fold_workspace()
    ws.fill_(float("nan"))                       # contents on entry must not matter
    for d in (1, 3, 4, 257, 4096 + 2, 70001):
        for J in (1, 2, 5, 16):
            say("ordered fold d=%d J=%d mode=%d bf16=%s" % (d, J, mode, bf16))
            w0 = rng.standard_normal(d).astype(np.float32)
            sv = B.Server(torch.from_numpy(w0).cuda(), 2, 0.1, lam0, mode, 0.95, 1e-7,
                          grad_bf16=bf16)
            ref = oracle.Server(w0, 2, 0.1, lam0, mode, 0.95, 1e-7)
            for rnd in range(3):
                scale = rng.permutation(J).astype(np.float32)[:, None] * 0.07 + 0.05
                g = (scale * rng.standard_normal((J, d))).astype(np.float32)
                g, dev = device_rows(g, bf16)
                sv.sync_fold(dev, 0.1 * J, workspace=ws)
                torch.cuda.synchronize()
                order = check_order(ws, g, J, d, "d=%d J=%d round %d" % (d, J, rnd))
                ref.sync_fold(g[order], 0.1 * J)
            assert sv.t == ref.t == 3 * J
            assert_same_bits(sv.w.cpu().numpy(), ref.w(), "ordered fold w d=%d J=%d" % (d, J))
            if mode == W.MODE_A:
                assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), "ordered fold ms d=%d J=%d" % (d, J))


def test_ordered_fold_more_tiles_than_partial_slots():
    """Past 2048 tiles of 256 groups every block walks several tiles; with a
    smaller block cap the same gradients must give the same order."""
    import torch
    from paper_1609_08326_amd import binding as B
    rng = np.random.default_rng(31)
    d, J = 2_400_003, 5
    w0 = rng.standard_normal(d).astype(np.float32)
    scale = np.array([0.9, 0.2, 0.5, 0.1, 0.7], dtype=np.float32)[:, None]
    g = (scale * rng.standard_normal((J, d))).astype(np.float32)
    _, dev = device_rows(g, False)
    ws = B.Server.fold_workspace()
    results = []
    for max_blocks in (0, 300):
        say("ordered fold d=%d J=%d max_blocks=%d" % (d, J, max_blocks))
        sv = B.Server(torch.from_numpy(w0).cuda(), 1, 0.1, 2.0, W.MODE_A, 0.95, 1e-7)
        sv.set_launch(256, 2, max_blocks)
        sv.sync_fold(dev, 0.5, workspace=ws)
        torch.cuda.synchronize()
        order = check_order(ws, g, J, d, "max_blocks=%d" % max_blocks)
        results.append(sv.w.cpu().numpy())
        if max_blocks == 0:
            first = B.Server.fold_order(ws, J)[0]
            sv2 = B.Server(torch.from_numpy(w0).cuda(), 1, 0.1, 2.0, W.MODE_A, 0.95, 1e-7)
            sv2.sync_fold(dev, 0.5, workspace=ws)
            torch.cuda.synchronize()
            again = B.Server.fold_order(ws, J)[0]
            assert first.tobytes() == again.tobytes(), "the summation order is fixed"
    ref = oracle.Server(w0, 1, 0.1, 2.0, W.MODE_A, 0.95, 1e-7)
    ref.sync_fold(g[order], 0.5)
    for got in results:
        assert_same_bits(got, ref.w(), "ordered fold, several tiles per block")


def test_ties_keep_the_callers_order_and_nan_goes_last():
    import torch
    from paper_1609_08326_amd import binding as B
    rng = np.random.default_rng(37)
    d = 10007
    a = rng.standard_normal(d).astype(np.float32)
    b = (0.5 * rng.standard_normal(d)).astype(np.float32)
    g = np.stack([a, b, a, b, a])
    _, dev = device_rows(g, False)                   # five separate buffers
    w0 = rng.standard_normal(d).astype(np.float32)
    ws = B.Server.fold_workspace()
    sv = B.Server(torch.from_numpy(w0).cuda(), 1, 0.1, 0.04, W.MODE_C)
    sv.sync_fold(dev, 0.5, workspace=ws)
    torch.cuda.synchronize()
    sq, perm = B.Server.fold_order(ws, 5)
    assert sq[0] == sq[2] == sq[4] and sq[1] == sq[3]
    assert perm.tolist() == [1, 3, 0, 2, 4]
    ref = oracle.Server(w0, 1, 0.1, 0.04, W.MODE_C)
    ref.sync_fold(g[[1, 3, 0, 2, 4]], 0.5)
    assert_same_bits(sv.w.cpu().numpy(), ref.w(), "ties")
    # a gradient that holds a NaN sorts after everything else; the list stays a permutation
    bad = a.copy()
    bad[123] = np.nan
    huge = np.full(d, 3e38, dtype=np.float32)        # squares overflow binary32, not binary64
    g2 = np.stack([bad, a, huge, b])
    _, dev2 = device_rows(g2, False)
    sv = B.Server(torch.from_numpy(w0).cuda(), 1, 0.1, 0.04, W.MODE_C)
    sv.sync_fold(dev2, 0.4, workspace=ws)
    torch.cuda.synchronize()
    sq, perm = B.Server.fold_order(ws, 4)
    assert np.isnan(sq[0]) and np.isfinite(sq[2]) and sq[2] > 1e80
    assert perm.tolist() == [3, 1, 2, 0]


def test_workspace_is_checked():
    import torch
    from paper_1609_08326_amd import binding as B
    lib = B.load()
    d = B.FOLD_WS_BYTES // 4 + 1024                  # w is large enough to be mistaken for one
    sv = B.Server(torch.zeros(d, device="cuda"), 1, 0.1, 0.04, B.MODE_C)
    g = torch.ones(d, device="cuda")
    ga = (C.c_void_p * 1)(g.data_ptr())
    ws = B.Server.fold_workspace()
    s = int(torch.cuda.current_stream().cuda_stream)
    assert lib.dcasgd_sync_fold_ordered(sv._h, ga, 1, 0.1, None, s) == B.EINVAL
    assert lib.dcasgd_sync_fold_ordered(sv._h, ga, 1, 0.1, ws.data_ptr() + 8, s) == B.EALIGN
    assert lib.dcasgd_sync_fold_ordered(sv._h, ga, 1, 0.1, sv.w.data_ptr(), s) == B.EINVAL
    assert lib.dcasgd_sync_fold_ordered(sv._h, ga, 1, 0.1, g.data_ptr(), s) == B.EINVAL
    assert lib.dcasgd_sync_fold_ordered(sv._h, ga, 0, 0.1, ws.data_ptr(), s) == B.EINVAL
    assert lib.dcasgd_sync_fold_ordered(sv._h, ga, 17, 0.1, ws.data_ptr(), s) == B.EINVAL
    torch.cuda.synchronize()
    assert sv.t == 0 and float(sv.w.abs().max()) == 0.0
    assert lib.dcasgd_sync_fold_ordered(sv._h, ga, 1, 0.1, ws.data_ptr(), s) == B.OK
    torch.cuda.synchronize()
    assert sv.t == 1


def test_ordered_fold_full_size():
    """The benchmark's fold workload (ResNet-50 size, J = 16): the whole vector
    against the oracle, one fold."""
    import torch
    from paper_1609_08326_amd import binding as B
    wl = W.get("fold")
    say("ordered fold full size %s d=%d J=%d" % (wl.name, wl.d, wl.K))
    hd_h, ws_h, w0 = wl.hdiag(), wl.wstar(), wl.w0()
    hd, wst = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    sv = B.Server(torch.from_numpy(w0).cuda(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    gbuf = [torch.empty(wl.d, device="cuda") for _ in range(wl.K)]
    for j in range(wl.K):
        B.synth_grad(sv.w, hd, wst, wl.sigma, wl.seed, j, gbuf[j])
    ws = B.Server.fold_workspace()
    sv.sync_fold(gbuf, wl.eta * wl.K, workspace=ws)
    torch.cuda.synchronize()
    say("  device done; oracle gradients")
    g = np.stack([oracle.synth_grad(w0, hd_h, ws_h, wl.sigma, wl.seed, j) for j in range(wl.K)])
    order = check_order(ws, g, wl.K, wl.d, "full size")
    say("  order %s; oracle fold" % order.tolist())
    ref = oracle.Server(w0, wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
    ref.sync_fold(g[order], wl.eta * wl.K)
    assert_same_bits(sv.w.cpu().numpy(), ref.w(), "ordered fold w (full)")
    assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), "ordered fold ms (full)")


def test_ordered_fold_replays_from_a_captured_graph():
    """Norms, ranking and fold are three plain launches with no host round trip and no
    memset, so a round of J worker gradients plus the ordered fold can be captured into a
    HIP graph; every replay must land on the oracle's bits (with eager work in between)."""
    import torch
    from paper_1609_08326_amd import binding as B
    wl = W.get("fold").replace(d=300007, K=6)
    hd_h, ws_h, w0 = wl.hdiag(), wl.wstar(), wl.w0()
    hd, wst = torch.from_numpy(hd_h).cuda(), torch.from_numpy(ws_h).cuda()
    side = torch.cuda.Stream()
    gbuf = [torch.empty(wl.d, device="cuda") for _ in range(wl.K)]
    fws = B.Server.fold_workspace()
    torch.cuda.synchronize()

    def one_round(sv):
        for j in range(wl.K):
            B.synth_grad(sv.w, hd, wst, wl.sigma, wl.seed, j, gbuf[j])
        sv.sync_fold(gbuf, wl.eta * wl.K, workspace=fws)

    ref = oracle.Server(w0, wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)

    def one_round_ref():
        w_t = ref.w()
        g = np.stack([oracle.synth_grad(w_t, hd_h, ws_h, wl.sigma, wl.seed, j) for j in range(wl.K)])
        order = np.argsort(oracle.grad_sqnorms(g), kind="stable")
        ref.sync_fold(g[order], wl.eta * wl.K)
        return order

    with torch.cuda.stream(side):
        sv = B.Server(torch.from_numpy(w0).cuda(), wl.M, wl.eta, wl.lambda0, wl.mode, wl.ema_m, wl.eps)
        one_round(sv)                                   # eager warm-up round
    side.synchronize()
    one_round_ref()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        one_round(sv)                                   # captured, not run
    other = torch.zeros(1 << 18, device="cuda")
    for r in range(3):
        say("ordered fold graph replay %d" % r)
        graph.replay()
        torch.cuda.synchronize()
        order = one_round_ref()
        perm = B.Server.fold_order(fws, wl.K)[1]
        assert perm.tolist() == order.tolist(), (r, perm, order)
        assert_same_bits(sv.w.cpu().numpy(), ref.w(), "replay %d w" % r)
        assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), "replay %d ms" % r)
        other.add_(1.0)
        torch.cuda.synchronize()


def test_ranking_forty_gradients_and_folding_them_in_parts():
    """More gradients than one call takes: norms chunk by chunk (the model untouched),
    one ranking on the host, then the fold in parts in that order; norms within the bound,
    order and model equal to the oracle's."""
    import torch
    from paper_1609_08326_amd import binding as B
    rng = np.random.default_rng(47)
    d, J = 50003, 40
    w0 = rng.standard_normal(d).astype(np.float32)
    scale = (rng.permutation(J).astype(np.float32)[:, None] * 0.02 + 0.05)
    g = (scale * rng.standard_normal((J, d))).astype(np.float32)
    _, dev = device_rows(g, False)
    sv = B.Server(torch.from_numpy(w0).cuda(), 1, 0.1, 2.0, W.MODE_A, 0.95, 1e-7)
    ws = B.Server.fold_workspace()
    sq = []
    for lo in range(0, J, 16):
        sv.grad_sqnorms(dev[lo:lo + 16], ws)
        torch.cuda.synchronize()
        sq.append(B.Server.fold_order(ws, len(dev[lo:lo + 16]))[0])
    sq = np.concatenate(sq)
    assert sv.t == 0
    assert_same_bits(sv.w.cpu().numpy(), w0, "norms leave the model alone")
    want = oracle.grad_sqnorms(g)
    assert np.all(np.abs(sq - want) <= norm_tolerance(d) * want)
    order = np.argsort(sq, kind="stable")
    assert order.tolist() == np.argsort(want, kind="stable").tolist()
    kept = sv.w.clone()
    ranked = [dev[int(j)] for j in order]
    for lo in range(0, J, 16):
        sv.sync_fold_part(ranked[lo:lo + 16], J, 2.0, kept)
    torch.cuda.synchronize()
    ref = oracle.Server(w0, 1, 0.1, 2.0, W.MODE_A, 0.95, 1e-7)
    ref.sync_fold(g[order], 2.0)
    assert sv.t == ref.t == J
    assert_same_bits(sv.w.cpu().numpy(), ref.w(), "ranked fold of forty, w")
    assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), "ranked fold of forty, ms")
