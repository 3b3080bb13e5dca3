"""The entry point that allocates nothing (pmpd_learned_forward_static) against the entry point it is a
variant of (pmpd_learned_forward), through the C ABI: same inputs, outputs compared bit for bit, on two
calls in a row of which the second is smaller (so that it runs on a work area that still holds the
first call's contents), and once more after the work area was used by a larger call again."""
import ctypes

import numpy as np
import pytest

import pmpd_synth as synth

pytestmark = pytest.mark.gpu


def _outputs(torch, net):
    return (torch.full((net.n_classes,), float("nan"), dtype=torch.float32, device="cuda"),
            torch.full((1,), -7, dtype=torch.int32, device="cuda"),
            torch.full((net.d_v,), float("nan"), dtype=torch.float32, device="cuda"))


def test_static_work_area_reproduces_the_workspace_entry_point():
    import torch

    import paper_2410_13461_amd as pmpd
    from paper_2410_13461_amd import binding

    assert torch.cuda.is_available()
    d, hidden, n_cls = 1024, 64, 5
    calls = [(777, 3000), (778, 130), (779, 5)]  # (seed, T): large, then smaller, then tiny
    nets, caches = [], []
    for seed, T in calls:
        Kh, Vh, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(seed, T, d, d, hidden, n_cls)
        nets.append(pmpd.LearnedScheduler(q, W1, b1, W2, b2))
        caches.append((torch.from_numpy(Kh).cuda(), torch.from_numpy(Vh).cuda()))
    # what the existing entry point gives, each call on a fresh workspace of its own
    want = []
    for net, (K, V) in zip(nets, caches):
        p, c, o = _outputs(torch, net)
        net.forward(K, V, p, c, o)
        torch.cuda.synchronize()
        want.append((p.clone(), c.clone(), o.clone()))
        assert torch.isfinite(p).all() and torch.isfinite(o).all() and 0 <= int(c.item()) < n_cls
    # the same calls through the static work area, back to back on one stream, no synchronisation between them
    got = [_outputs(torch, net) for net in nets]
    for net, (K, V), (p, c, o) in zip(nets, caches, got):
        print(f"[no-alloc] T={K.shape[0]}", flush=True)
        net.forward_static(K, V, p, c, o)
    torch.cuda.synchronize()
    for (seed, T), w, g in zip(calls, want, got):
        for name, a, b in zip(("probs", "cls", "context"), w, g):
            assert torch.equal(a, b), f"T={T}: {name} differs from pmpd_learned_forward"
    # larger again after the small ones, then the first case once more: still the same bits
    for idx in (0, 2, 0):
        p, c, o = _outputs(torch, nets[idx])
        nets[idx].forward_static(*caches[idx], p, c, o)
        torch.cuda.synchronize()
        assert torch.equal(p, want[idx][0]) and torch.equal(c, want[idx][1]) and torch.equal(o, want[idx][2])


def test_static_work_area_refuses_what_does_not_fit():
    import torch

    import paper_2410_13461_amd as pmpd
    from paper_2410_13461_amd import binding

    d_v, T = 65536, 4096  # 128 partial rows of 65536 floats = 32 MiB of work area
    net = pmpd.LearnedScheduler(np.zeros(64, np.float32), np.zeros((4, d_v), np.float32), np.zeros(4, np.float32),
                                np.zeros((3, 4), np.float32), np.zeros(3, np.float32))
    assert net.workspace_size(T) > (4 << 20)
    K = torch.zeros((T, 64), dtype=torch.float16, device="cuda")
    V = torch.zeros((T, d_v), dtype=torch.float16, device="cuda")
    p, c, o = _outputs(torch, net)
    with pytest.raises(pmpd.PMPDError, match="use pmpd_learned_forward") as e:
        net.forward_static(K, V, p, c, o)
    assert e.value.status == -5
    assert torch.isnan(p).all()  # nothing was launched
