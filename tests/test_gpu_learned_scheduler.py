"""Forward pass of the learned scheduler on the GPU against the fp64 oracle.

Tolerances (fp32 arithmetic against fp64): a score carries an absolute error of about
sqrt(D_k) * 2^-24 * |q||K_t| / sqrt(D_k), well below 1e-5 for the inputs here; softmax turns an absolute
score error d into a relative weight error d, so O is held to 2e-5 * sum_t p_t |V_t| per column and the
class probabilities to 1e-4 absolute (the small network multiplies the error of O by at most the row sums of
|W1| and |W2|, about 20 together for the seeded parameters).  Trained parameters are not public: the
scheduler's *quality* is unpinned, its arithmetic is what these tests hold."""
import numpy as np
import pytest

import oracle
import pmpd_synth as synth

pytestmark = pytest.mark.gpu

O_TOL = 2e-5
P_TOL = 1e-4


@pytest.fixture(scope="module")
def pmpd():
    import torch

    assert torch.cuda.is_available()
    import paper_2410_13461_amd as lib

    return lib


def _run(pmpd, K, V, q, W1, b1, W2, b2):
    import torch

    net = pmpd.LearnedScheduler(q, W1, b1, W2, b2)
    probs, cls, ctx = net.forward(torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda())
    torch.cuda.synchronize()
    return probs.cpu().numpy(), int(cls.item()), ctx.cpu().numpy()


def _compare(K, V, q, W1, b1, W2, b2, probs, cls, ctx):
    O_ref, p_ref, c_ref = oracle.learned_scheduler(q, K, V, W1, b1, W2, b2)
    T, Dk = K.shape
    sc = K.astype(np.float64) @ q.astype(np.float64) / np.sqrt(Dk)
    w = np.exp(sc - sc.max())
    w /= w.sum()
    budget = w @ np.abs(V.astype(np.float64))
    assert np.all(np.isfinite(ctx)) and np.all(np.isfinite(probs))
    assert np.all(np.abs(ctx - O_ref) <= O_TOL * budget + 1e-30)
    assert np.all(np.abs(probs - p_ref) <= P_TOL)
    assert abs(float(probs.sum()) - 1.0) <= 1e-5
    # the decision is taken on the kernel's own fp32 probabilities: first index of the largest
    assert cls == int(np.argmax(probs))
    top2 = np.sort(p_ref)[-2:]
    if top2[1] - top2[0] > 2 * P_TOL:
        assert cls == c_ref


@pytest.mark.parametrize("T,d_k,d_v,hidden,n_classes,sharp", [
    (1, 8, 8, 1, 2, 1.0),            # one token: O = V[0]
    (5, 16, 24, 3, 3, 1.0),          # below every tile size
    (67, 136, 520, 37, 5, 1.0),      # ragged everything: 65 value chunks -> two column blocks, odd hidden
    (512, 4096, 4096, 256, 5, 1.0),  # 7B-shaped cache of a 512-token prompt
    (1029, 1024, 2048, 64, 9, 3.0),  # more rows than chunks (9 rows per chunk, ragged last chunk), peaky softmax
    (2048, 4096, 4096, 256, 5, 0.2), # long prompt, flat softmax
    (300, 16384, 8, 5, 2, 0.5),      # widest key the kernel takes, narrowest value
])
def test_forward_matches_oracle(pmpd, T, d_k, d_v, hidden, n_classes, sharp):
    K, V, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(21, T, d_k, d_v, hidden, n_classes, sharpness=sharp)
    probs, cls, ctx = _run(pmpd, K, V, q, W1, b1, W2, b2)
    _compare(K, V, q, W1, b1, W2, b2, probs, cls, ctx)


def test_degenerate_cases(pmpd):
    K, V, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(22, 40, 64, 128, 16, 4)
    # zero query: uniform attention, O is the mean of the value rows
    probs, cls, ctx = _run(pmpd, K, V, 0 * q, W1, b1, W2, b2)
    assert np.allclose(ctx, V.astype(np.float64).mean(axis=0), rtol=0, atol=2e-6)
    _compare(K, V, 0 * q, W1, b1, W2, b2, probs, cls, ctx)
    # one key far ahead of the rest (score gap of hundreds): exp underflows for the others, no NaN
    K2 = K.copy()
    K2[7] = (60.0 * q / np.linalg.norm(q)).astype(np.float16)
    probs, cls, ctx = _run(pmpd, K2, V, 8 * q, W1, b1, W2, b2)
    assert np.array_equal(ctx, V[7].astype(np.float32))
    _compare(K2, V, 8 * q, W1, b1, W2, b2, probs, cls, ctx)
    # all hidden units off (large negative bias): the head sees zeros, probabilities = softmax(b2)
    probs, cls, ctx = _run(pmpd, K, V, q, W1, b1 - 1e4, W2, b2)
    e = np.exp(b2.astype(np.float64))
    assert np.all(np.abs(probs - e / e.sum()) <= 1e-6) and cls == int(np.argmax(probs))
    # equal logits: the first class wins
    probs, cls, ctx = _run(pmpd, K, V, q, W1, b1, 0 * W2, 0 * b2 + 0.25)
    assert cls == 0 and np.all(probs == probs[0])


def test_result_does_not_depend_on_what_the_workspace_held_and_repeats_bit_exactly(pmpd):
    import torch

    K, V, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(23, 777, 512, 1024, 48, 6)
    net = pmpd.LearnedScheduler(q, W1, b1, W2, b2)
    dK, dV = torch.from_numpy(K).cuda(), torch.from_numpy(V).cuda()
    p1, c1, o1 = net.forward(dK, dV)
    torch.cuda.synchronize()
    p1, c1, o1 = p1.clone(), c1.clone(), o1.clone()
    net._ws.fill_(0xFF)  # NaN patterns everywhere
    p2, c2, o2 = net.forward(dK, dV)
    torch.cuda.synchronize()
    assert torch.equal(p1, p2) and torch.equal(c1, c2) and torch.equal(o1, o2)
    # a shorter prompt right after a longer one reuses the same workspace
    p3, c3, o3 = net.forward(dK[:100].contiguous(), dV[:100].contiguous())
    torch.cuda.synchronize()
    _compare(K[:100], V[:100], q, W1, b1, W2, b2, p3.cpu().numpy(), int(c3.item()), o3.cpu().numpy())


def test_class_to_schedule_to_decode_run(pmpd):
    """The predicted class picks the switch point of a two-precision schedule that then drives decode steps."""
    import torch

    K, V, q, W1, b1, W2, b2 = synth.draw_learned_scheduler(24, 96, 256, 256, 32, 5)
    probs, cls, _ = _run(pmpd, K, V, q, W1, b1, W2, b2)
    OL, N = 64, 5
    sch = pmpd.schedule_from_class(3, 2, cls, OL, N)
    point = oracle.schedule_grid(OL, N)[cls]
    assert [sch.bits(k) for k in range(OL)] == [3 if k < point else 2 for k in range(OL)]
    assert abs(sch.avg_bits(OL) - oracle.schedule_avg_bits([3, 2], [0, point], OL)) < 1e-12
    out_f, in_f = 128, 256
    q4, s, a = synth.draw_weights(24, 0, 0, out_f, in_f)
    planes, sm = pmpd.pack(q4, s, a)
    st = pmpd.Stack([pmpd.upload_layer(planes, sm, out_f, in_f)])
    xs = np.stack([synth.draw_x(24, k, 0, 0, in_f)[0] for k in range(OL)])
    y = torch.zeros(OL, out_f, dtype=torch.float32, device="cuda")
    pmpd.decode_run(st, sch, 0, OL, torch.from_numpy(xs).cuda(), in_f, y, out_f)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    for k in (0, max(point - 1, 0), min(point, OL - 1), OL - 1):
        b = 3 if k < point else 2
        y_ref, t = oracle.linear(q4, s, a, b, xs[k])
        assert np.all(np.abs(yh[k] - y_ref[0]) <= 2e-3 * t[0])
        assert np.linalg.norm(yh[k] - y_ref[0]) <= 1e-3 * np.linalg.norm(y_ref[0])
