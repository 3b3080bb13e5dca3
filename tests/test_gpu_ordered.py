"""The dependency-ordered step (one cooperative launch, every tile waiting in the kernel for the outputs
it reads): every layer against the oracle on the inputs it really got, x = fp16(gain * y[source]) for
chained layers."""
import numpy as np
import pytest

import oracle
import pmpd_synth as synth

pytestmark = pytest.mark.gpu

REL_L2 = 1e-3
ABS_FACTOR = 2e-3


@pytest.fixture(scope="module")
def pmpd():
    import torch

    assert torch.cuda.is_available()
    import paper_2410_13461_amd as lib

    return lib


def _chain_of(shape):
    """(q,k,v) -> o -> (up,gate) -> down per block; o reads q, up/gate read o, down reads up, the next
    block reads down.  Gains keep the activations near unit scale (random weights, no norm layers)."""
    stages, sources, gains = [], [], []
    for blk in range(shape.n_blocks):
        base = 7 * blk
        prev_down = base - 7 + 5 if blk else -1
        for pi in range(7):  # q k v o up down gate
            if pi in (0, 1, 2):
                stages.append(4 * blk); sources.append(prev_down)
            elif pi == 3:
                stages.append(4 * blk + 1); sources.append(base + 0)
            elif pi in (4, 6):
                stages.append(4 * blk + 2); sources.append(base + 3)
            else:
                stages.append(4 * blk + 3); sources.append(base + 4)
            gains.append(0.5 if sources[-1] >= 0 else 1.0)
    return stages, sources, gains


def _build(pmpd, shape, seed):
    layers, raw = [], []
    for (blk, pi, nm, o, i) in shape.layers():
        q4, s, a = synth.draw_weights(seed, blk, pi, o, i, random_min=(pi % 2 == 1))
        raw.append((q4, s, a))
        planes, sm = pmpd.pack(q4, s, a)
        layers.append(pmpd.upload_layer(planes, sm, o, i))
    return layers, raw


@pytest.mark.parametrize("b", [4, 3, 2])
@pytest.mark.parametrize("shape", [synth.StackShape("tiny", 3, 256, 640),      # every layer in one K-part: plain y
                                   synth.StackShape("mid", 2, 2048, 5632)],    # 2 to 6 K-parts: fixed-point sums
                         ids=["one-part", "k-parts"])
def test_ordered_step_matches_oracle_layer_by_layer(pmpd, b, shape):
    import torch

    print(f"[ordered] b={b} {shape.name}", flush=True)
    layers, raw = _build(pmpd, shape, seed=21)
    stack = pmpd.Stack(layers)
    stages, sources, gains = _chain_of(shape)
    ordered = pmpd.Ordered(stack, stages, sources, gains)
    ordered.set_spin_limit(200000)
    y = torch.full((stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    for rep in range(3):  # the sums are reset by every step; fresh inputs, so a stale y of the last step shows
        xs = [synth.draw_x(21, rep, blk, pi, i)[0] for (blk, pi, nm, o, i) in shape.layers()]
        x = torch.from_numpy(np.concatenate(xs)).cuda()
        ordered.step(b, x, y)
        torch.cuda.synchronize()
        assert not ordered.timed_out()
        yh = y.cpu().numpy()
        for li, (q4, s, a) in enumerate(raw):
            if sources[li] < 0:
                xin = xs[li]
            else:
                so = stack.y_offsets[sources[li]]
                src = yh[so:so + q4.shape[1]]
                xin = (src * np.float32(gains[li])).astype(np.float16)  # fp32 product, round to nearest even
            o = stack.y_offsets[li]
            y_ref, t = oracle.linear(q4, s, a, b, xin)
            got = yh[o:o + q4.shape[0]].astype(np.float64)
            assert np.all(np.isfinite(got)), f"layer {li}"
            err = np.abs(got - y_ref[0])
            assert np.all(err <= ABS_FACTOR * t[0] + 1e-30), f"layer {li} b={b}: {err.max():.3e}"
            den = np.linalg.norm(y_ref[0])
            assert den == 0 or np.linalg.norm(got - y_ref[0]) / den <= REL_L2, f"layer {li} b={b}"
    # the K-parts meet by integer atomic adds: the order of arrival must not show in a single bit
    y_again = torch.zeros_like(y)
    for _ in range(3):
        ordered.step(b, x, y_again)
        torch.cuda.synchronize()
        assert torch.equal(y_again, y)
    # without chaining the same object reproduces the one-launch step
    free = pmpd.Ordered(stack, stages, [-1] * len(stages), [1.0] * len(stages))
    y1 = torch.zeros_like(y)
    y2 = torch.zeros_like(y)
    free.step(b, x, y1)
    pmpd.decode_step(stack, b, x, y2)
    torch.cuda.synchronize()
    assert not free.timed_out()
    # two summation orders of the same fp32 arithmetic: far inside the parity bar, relative to sum |w||x|
    y1h, y2h = y1.cpu().numpy().astype(np.float64), y2.cpu().numpy().astype(np.float64)
    for li, (q4, s, a) in enumerate(raw):
        o = stack.y_offsets[li]
        _, t = oracle.linear(q4, s, a, b, xs[li])
        assert np.all(np.abs(y1h[o:o + q4.shape[0]] - y2h[o:o + q4.shape[0]]) <= 1e-4 * t[0] + 1e-30), f"layer {li}"
    ordered.close(); free.close(); stack.close()


@pytest.mark.parametrize("b", [4, 2])
def test_ordered_longest_rows_meet_in_many_parts(pmpd, b):
    """Rows of 32768 features (the largest the library takes) are split into 29 K-parts, close to what the
    count bits of a sum hold; a ragged layer (192 rows) reads them."""
    import torch

    print(f"[ordered] longest rows b={b}", flush=True)
    dims = [(128, 32768), (192, 128)]
    raw, layers = [], []
    for li, (o, i) in enumerate(dims):
        q4, s, a = synth.draw_weights(31, li, 0, o, i, random_min=True)
        raw.append((q4, s, a))
        planes, sm = pmpd.pack(q4, s, a)
        layers.append(pmpd.upload_layer(planes, sm, o, i))
    stack = pmpd.Stack(layers)
    gain = 1.0 / 16.0
    ordered = pmpd.Ordered(stack, [0, 1], [-1, 0], [1.0, gain])
    ordered.set_spin_limit(200000)
    xs = [synth.draw_x(31, 0, li, 0, i)[0] for li, (o, i) in enumerate(dims)]
    x = torch.from_numpy(np.concatenate(xs)).cuda()
    y = torch.full((stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    ordered.step(b, x, y)
    torch.cuda.synchronize()
    assert not ordered.timed_out()
    yh = y.cpu().numpy()
    o0, o1 = stack.y_offsets
    for li, xin in ((0, xs[0]), (1, (yh[o0:o0 + 128] * np.float32(gain)).astype(np.float16))):
        q4, s, a = raw[li]
        y_ref, t = oracle.linear(q4, s, a, b, xin)
        got = yh[stack.y_offsets[li]:stack.y_offsets[li] + q4.shape[0]].astype(np.float64)
        assert np.all(np.abs(got - y_ref[0]) <= ABS_FACTOR * t[0] + 1e-30), f"layer {li}"
        assert np.linalg.norm(got - y_ref[0]) / np.linalg.norm(y_ref[0]) <= REL_L2, f"layer {li}"
    ordered.close(); stack.close()


def test_ordered_stage_with_more_tiles_than_workgroups(pmpd):
    """70400 output rows are 1100 tiles, more than the chip holds workgroups at once: the stage runs in
    two rounds of the grid.  The wide layer reads a narrow one of the stage before."""
    import torch

    print("[ordered] stage of 1100 tiles", flush=True)
    dims = [(256, 128), (70400, 256)]
    raw, layers = [], []
    for li, (o, i) in enumerate(dims):
        q4, s, a = synth.draw_weights(32, li, 0, o, i, random_min=True)
        raw.append((q4, s, a))
        planes, sm = pmpd.pack(q4, s, a)
        layers.append(pmpd.upload_layer(planes, sm, o, i))
    stack = pmpd.Stack(layers)
    gain = 0.25
    ordered = pmpd.Ordered(stack, [0, 1], [-1, 0], [1.0, gain])
    ordered.set_spin_limit(200000)
    xs = [synth.draw_x(32, 0, li, 0, i)[0] for li, (o, i) in enumerate(dims)]
    x = torch.from_numpy(np.concatenate(xs)).cuda()
    y = torch.full((stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    for b in (4, 2):
        ordered.step(b, x, y)
        torch.cuda.synchronize()
        assert not ordered.timed_out()
        yh = y.cpu().numpy()
        o0 = stack.y_offsets[0]
        for li, xin in ((0, xs[0]), (1, (yh[o0:o0 + 256] * np.float32(gain)).astype(np.float16))):
            q4, s, a = raw[li]
            y_ref, t = oracle.linear(q4, s, a, b, xin)
            got = yh[stack.y_offsets[li]:stack.y_offsets[li] + q4.shape[0]].astype(np.float64)
            assert np.all(np.abs(got - y_ref[0]) <= ABS_FACTOR * t[0] + 1e-30), f"layer {li} b={b}"
            assert np.linalg.norm(got - y_ref[0]) / np.linalg.norm(y_ref[0]) <= REL_L2, f"layer {li} b={b}"
    ordered.close(); stack.close()


def test_ordered_values_out_of_range_do_not_stall(pmpd):
    """A gain that drives the chained activations to infinity: the K-parts are clamped before they are
    added, so the counts in the sums stay intact and no tile waits for ever."""
    import torch

    shape = synth.StackShape("mid", 1, 2048, 5632)
    layers, raw = _build(pmpd, shape, seed=24)
    stack = pmpd.Stack(layers)
    stages, sources, gains = _chain_of(shape)
    ordered = pmpd.Ordered(stack, stages, sources, [1.0 if k < 0 else 6.0e4 for k in sources])
    ordered.set_spin_limit(200000)
    xs = [synth.draw_x(24, 0, blk, pi, i)[0] for (blk, pi, nm, o, i) in shape.layers()]
    x = torch.from_numpy(np.concatenate(xs)).cuda()
    y = torch.zeros(stack.y_elems, dtype=torch.float32, device="cuda")
    ordered.step(4, x, y)
    torch.cuda.synchronize()
    assert not ordered.timed_out()
    # the layers in front of the blow-up stayed in range and are still right: q, k, v read the external x, and o reads
    # q through the same huge gain only from the second link on (q itself is an ordinary output)
    yh = y.cpu().numpy()
    for li in (0, 1, 2):
        q4, s, a = raw[li]
        y_ref, t = oracle.linear(q4, s, a, 4, xs[li])
        got = yh[stack.y_offsets[li]:stack.y_offsets[li] + q4.shape[0]].astype(np.float64)
        assert np.all(np.abs(got - y_ref[0]) <= ABS_FACTOR * t[0]), f"layer {li}"
        assert np.linalg.norm(got - y_ref[0]) / np.linalg.norm(y_ref[0]) <= REL_L2, f"layer {li}"
    ordered.close(); stack.close()


def _check_chain(stack, raw, sources, gains, xs, yh, b):
    """Every layer of a chained step against the oracle on the inputs it really got."""
    for li, (q4, s, a) in enumerate(raw):
        if sources[li] < 0:
            xin = xs[li]
        else:
            so = stack.y_offsets[sources[li]]
            xin = (yh[so:so + q4.shape[1]] * np.float32(gains[li])).astype(np.float16)
        y_ref, t = oracle.linear(q4, s, a, b, xin)
        got = yh[stack.y_offsets[li]:stack.y_offsets[li] + q4.shape[0]].astype(np.float64)
        assert np.all(np.abs(got - y_ref[0]) <= ABS_FACTOR * t[0] + 1e-30), f"layer {li}"
        den = np.linalg.norm(y_ref[0])
        assert den == 0 or np.linalg.norm(got - y_ref[0]) / den <= REL_L2, f"layer {li}"


def test_ordered_wait_is_bounded_and_reported(pmpd):
    """With a limit of one poll a wait may run out.  Whether it does depends on timing (a consumer that finds its
    inputs complete at the first look never waits), so the flag's value is not asserted.  What must hold either
    way: the step ends (the synchronisation returns), every output is a finite number, the layers that wait for
    nothing (stage 0 reads the external x) are right, reading the flag clears it, and the same object, given its
    normal limit back, then runs a step that is right in every layer and reports no time-out."""
    import torch

    shape = synth.StackShape("tiny", 2, 256, 640)
    layers, raw = _build(pmpd, shape, seed=22)
    stack = pmpd.Stack(layers)
    stages, sources, gains = _chain_of(shape)
    ordered = pmpd.Ordered(stack, stages, sources, gains)
    ordered.set_spin_limit(1)
    xs = [synth.draw_x(22, 0, blk, pi, i)[0] for (blk, pi, nm, o, i) in shape.layers()]
    x = torch.from_numpy(np.concatenate(xs)).cuda()
    y = torch.full((stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    ordered.step(4, x, y)
    torch.cuda.synchronize()  # returns: the waits are bounded
    flag = ordered.timed_out()
    print(f"[ordered] a wait ran out with a limit of one poll: {flag}", flush=True)
    assert isinstance(flag, bool)
    assert not ordered.timed_out()  # reading the flag clears it
    yh = y.cpu().numpy()
    assert np.all(np.isfinite(yh))  # every row was written, whatever its inputs were
    for li in (0, 1, 2):
        q4, s, a = raw[li]
        y_ref, t = oracle.linear(q4, s, a, 4, xs[li])
        got = yh[stack.y_offsets[li]:stack.y_offsets[li] + q4.shape[0]].astype(np.float64)
        assert np.all(np.abs(got - y_ref[0]) <= ABS_FACTOR * t[0]), f"layer {li}"
    if not flag:  # nothing ran out: the whole chain must then be right
        _check_chain(stack, raw, sources, gains, xs, yh, 4)
    ordered.set_spin_limit(200000)
    y.fill_(float("nan"))
    ordered.step(4, x, y)
    torch.cuda.synchronize()
    assert not ordered.timed_out()
    _check_chain(stack, raw, sources, gains, xs, y.cpu().numpy(), 4)
    ordered.close(); stack.close()


def test_ordered_refuses_rows_too_long_for_the_part_count(pmpd):
    """A row is split into at most 31 K-parts of at most 32 groups (the count field of a sum word has five bits):
    126976 input features.  A longer row is refused when the object is created, not run."""
    import torch

    out_f, in_f = 64, 993 * 128
    pb, sb = pmpd.packed_size(out_f, in_f)
    planes = [torch.zeros(pb // 4, dtype=torch.int32, device="cuda") for _ in range(4)]
    layer = pmpd.PackedLayer(out_f, in_f, planes, torch.zeros(sb // 4, dtype=torch.int32, device="cuda"))
    stack = pmpd.Stack([layer])
    with pytest.raises(pmpd.PMPDError, match="cannot be split") as e:
        pmpd.Ordered(stack, [0], [-1], [1.0])
    assert e.value.status == -1
    stack.close()


def test_ordered_rejects_bad_chains(pmpd):
    shape = synth.StackShape("tiny", 1, 256, 640)
    layers, raw = _build(pmpd, shape, seed=23)
    stack = pmpd.Stack(layers)
    n = len(layers)
    ok_stage = [0, 0, 0, 1, 2, 3, 2]
    with pytest.raises(pmpd.PMPDError):  # source in the same stage
        pmpd.Ordered(stack, [0] * n, [-1, 0, -1, -1, -1, -1, -1], [1.0] * n)
    with pytest.raises(pmpd.PMPDError):  # 640 outputs feeding 256 inputs
        pmpd.Ordered(stack, ok_stage, [-1, -1, -1, 4, -1, -1, -1], [1.0] * n)
    with pytest.raises(pmpd.PMPDError):  # not a layer
        pmpd.Ordered(stack, ok_stage, [-1, -1, -1, 99, -1, -1, -1], [1.0] * n)
    with pytest.raises(pmpd.PMPDError):  # gain not finite
        pmpd.Ordered(stack, ok_stage, [-1, -1, -1, 0, -1, -1, -1], [1.0, 1.0, 1.0, float("inf"), 1.0, 1.0, 1.0])
    with pytest.raises(pmpd.PMPDError):  # one entry per layer
        pmpd.Ordered(stack, [0], [-1], [1.0])
    stack.close()
