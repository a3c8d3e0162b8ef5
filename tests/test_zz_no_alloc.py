"""The entry point that allocates nothing (dcasgd_sync_fold_ordered_static: the
ordered fold with the library's own static workspace) against the existing
entry point that takes the caller's workspace (dcasgd_sync_fold_ordered), through
the C ABI, bit for bit, on two calls in a row, the second on a smaller input:
the static array keeps the first call's contents and must not let them leak
into the second."""
import ctypes as C
import sys

import numpy as np
import pytest

import oracle

from gpu_harness import assert_same_bits

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def folded(B, torch, w0, grads, eta_hat, static):
    """State after one ordered fold of `grads` into a fresh adaptive server."""
    sv = B.Server(torch.from_numpy(w0).cuda(), 1, 0.1, 2.0, B.MODE_A, 0.95, 1e-7)
    dev = [torch.from_numpy(g).cuda() for g in grads]
    if static:
        sv.sync_fold_ordered_static(dev, eta_hat)
    else:
        ws = B.Server.fold_workspace()
        ws.fill_(float("nan"))
        sv.sync_fold(dev, eta_hat, workspace=ws)
    torch.cuda.synchronize()
    assert sv.t == len(grads)
    return sv.w.cpu().numpy(), sv.ms.cpu().numpy()


def test_static_workspace_fold_equals_the_callers_workspace_fold_twice_in_a_row():
    import torch
    from paper_1609_08326_amd import binding as B
    rng = np.random.default_rng(41)
    # first call: many tiles, a ragged tail, the longest list; second: smaller d, shorter list
    for d, J in ((1_300_003, 16), (70_001, 5)):
        say("static-workspace fold d=%d J=%d" % (d, J))
        w0 = rng.standard_normal(d).astype(np.float32)
        # norms well apart and not in the caller's order, so the ranking decides the bits
        scale = (rng.permutation(J).astype(np.float32) * 0.11 + 0.05)[:, None]
        g = (scale * rng.standard_normal((J, d))).astype(np.float32)
        w_ref, ms_ref = folded(B, torch, w0, g, 0.1 * J, static=False)
        w_got, ms_got = folded(B, torch, w0, g, 0.1 * J, static=True)
        assert_same_bits(w_got, w_ref, "static-workspace fold w d=%d J=%d" % (d, J))
        assert_same_bits(ms_got, ms_ref, "static-workspace fold ms d=%d J=%d" % (d, J))
        # the order matters for these inputs: the caller's order gives other bits
        sv = B.Server(torch.from_numpy(w0).cuda(), 1, 0.1, 2.0, B.MODE_A, 0.95, 1e-7)
        sv.sync_fold([torch.from_numpy(x).cuda() for x in g], 0.1 * J)
        torch.cuda.synchronize()
        assert not np.array_equal(sv.w.cpu().numpy().view(np.uint32), w_ref.view(np.uint32))


def test_static_workspace_fold_refuses_a_list_longer_than_its_limit():
    import torch
    from paper_1609_08326_amd import binding as B
    lib = B.load()
    d = 4099
    sv = B.Server(torch.zeros(d, device="cuda"), 1, 0.1, 2.0, B.MODE_A, 0.95, 1e-7)
    g = [torch.ones(d, device="cuda") for _ in range(B.MAX_K + 1)]
    ga = (C.c_void_p * len(g))(*[x.data_ptr() for x in g])
    before = sv.w.clone()
    rc = lib.dcasgd_sync_fold_ordered_static(sv._h, ga, len(g), 0.1, None)
    torch.cuda.synchronize()
    assert rc == B.EINVAL and sv.t == 0
    assert torch.equal(sv.w, before), "a refused call launches nothing"
    assert lib.dcasgd_sync_fold_ordered_static(sv._h, ga, 0, 0.1, None) == B.EINVAL
    assert lib.dcasgd_sync_fold_ordered_static(None, ga, 1, 0.1, None) == B.EINVAL


def test_static_workspace_fold_replays_from_a_captured_graph():
    """What the entry point is for: captured into a HIP graph (nothing in the call
    allocates, queries the device or records a memset) and replayed, with eager work and
    synchronisation between the replays; every replay is checked against the oracle's
    fold of the same gradients in ascending-norm order."""
    import torch
    from paper_1609_08326_amd import binding as B
    rng = np.random.default_rng(43)
    d, J = 300_007, 6
    w0 = rng.standard_normal(d).astype(np.float32)
    scale = (rng.permutation(J).astype(np.float32) * 0.02 + 0.01)[:, None]
    g = (scale * rng.standard_normal((J, d))).astype(np.float32)
    order = np.argsort(oracle.grad_sqnorms(g), kind="stable")
    side = torch.cuda.Stream()
    dev = [torch.from_numpy(x).cuda() for x in g]
    other = torch.zeros(1 << 20, device="cuda")
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        sv = B.Server(torch.from_numpy(w0).cuda(), 1, 0.1, 2.0, B.MODE_A, 0.95, 1e-7)
        sv.sync_fold_ordered_static(dev, 0.05 * J)          # eager once on the capture stream
    side.synchronize()
    ref = oracle.Server(w0, 1, 0.1, 2.0, oracle.MODE_A, 0.95, 1e-7)
    ref.sync_fold(g[order], 0.05 * J)
    assert_same_bits(sv.w.cpu().numpy(), ref.w(), "eager w")
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sv.sync_fold_ordered_static(dev, 0.05 * J)
    for r in range(3):
        say("static-workspace fold, graph replay %d" % r)
        graph.replay()
        torch.cuda.synchronize()
        ref.sync_fold(g[order], 0.05 * J)
        assert_same_bits(sv.w.cpu().numpy(), ref.w(), "replay %d w" % r)
        assert_same_bits(sv.ms.cpu().numpy(), ref.ms(), "replay %d ms" % r)
        other.add_(1.0)                                      # unrelated eager work between replays
        torch.cuda.synchronize()
