"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Bars: pack/unpack bit-exact (checked on the CPU side);
linear layers  ||y - y*||_2 / ||y*||_2 <= 1e-3  and  |y[r] - y*[r]| <= 2e-3 * sum_i |W[r][i]||x[i]|."""
import sys

import numpy as np
import pytest

import oracle
import pmpd_synth as synth

pytestmark = pytest.mark.gpu

REL_L2 = 1e-3
ABS_FACTOR = 2e-3


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def assert_parity(y_gpu: np.ndarray, y_ref: np.ndarray, budget: np.ndarray, what: str):
    y_gpu = np.asarray(y_gpu, dtype=np.float64).reshape(y_ref.shape)
    assert np.all(np.isfinite(y_gpu)), f"{what}: non-finite output"
    err = np.abs(y_gpu - y_ref)
    bound = ABS_FACTOR * budget
    worst = np.argmax(err - bound)
    assert np.all(err <= bound), (
        f"{what}: |dy|={err.flat[worst]:.3e} > {bound.flat[worst]:.3e} at flat index {worst}")
    denom = np.linalg.norm(y_ref)
    if denom > 0:
        rel = np.linalg.norm(y_gpu - y_ref) / denom
        assert rel <= REL_L2, f"{what}: relative L2 error {rel:.3e}"
    else:
        assert np.all(y_gpu == 0)


@pytest.fixture(scope="module")
def pmpd():
    import torch

    assert torch.cuda.is_available()
    import paper_2410_13461_amd as lib

    return lib


def _device_layer(pmpd, q4, s, a):
    planes, sm = pmpd.pack(q4, s, a)
    return pmpd.upload_layer(planes, sm, q4.shape[0], q4.shape[1])


def _run_gemv(pmpd, layer, b, x_np):
    import torch

    x = torch.from_numpy(x_np).cuda()
    y = pmpd.gemv(layer, b, x)
    torch.cuda.synchronize()
    return y.cpu().numpy()


# shapes: several row tiles, ragged tails (out not a multiple of 64), K long enough for every
# split-K launch shape, and the non-power-of-two rows of the Llama MLPs (11008 = 86 groups).
SHAPES = [(64, 128), (100, 384), (257, 1408), (512, 4096), (200, 11008), (4096, 256), (130, 2048)]


@pytest.mark.parametrize("b", [4, 3, 2])
@pytest.mark.parametrize("out_f,in_f", SHAPES)
def test_gemv_matches_oracle(pmpd, b, out_f, in_f):
    _say(f"[gemv] out={out_f} in={in_f} b={b}")
    q4, s, a = synth.draw_weights(100, out_f, in_f, out_f, in_f, random_min=True)
    x = synth.draw_x(100, 0, out_f, in_f, in_f)[0]
    layer = _device_layer(pmpd, q4, s, a)
    y = _run_gemv(pmpd, layer, b, x)
    y_ref, t = oracle.linear(q4, s, a, b, x)
    assert_parity(y, y_ref[0], t[0], f"gemv {out_f}x{in_f} b={b}")


@pytest.mark.parametrize("b", [4, 3, 2])
def test_gemv_config0_full_layer(pmpd, b):
    """The 4096x4096 single-layer workload, seed 0, a = -8 s."""
    _say(f"[gemv cfg0] b={b}")
    q4, s, a = synth.draw_weights(0, 0, 0, 4096, 4096)
    x = synth.draw_x(0, 0, 0, 0, 4096)[0]
    layer = _device_layer(pmpd, q4, s, a)
    y = _run_gemv(pmpd, layer, b, x)
    y_ref, t = oracle.linear(q4, s, a, b, x)
    assert_parity(y, y_ref[0], t[0], f"cfg0 b={b}")
    # same launch twice: bit-identical (fixed reduction order, no atomics)
    y2 = _run_gemv(pmpd, layer, b, x)
    assert np.array_equal(y, y2)


@pytest.mark.parametrize("b", [4, 3, 2])
def test_gemv_ignores_planes_below_b(pmpd, b):
    """Planes b..3 live in separately allocated, poisoned buffers (or are absent)."""
    import torch

    _say(f"[gemv prefix] b={b}")
    out_f, in_f = 192, 1024
    q4, s, a = synth.draw_weights(7, 1, 1, out_f, in_f, random_min=True)
    x = synth.draw_x(7, 0, 1, 1, in_f)[0]
    planes, sm = pmpd.pack(q4, s, a)
    y_ref, t = oracle.linear(q4, s, a, b, x)
    rng = np.random.default_rng(3)
    poisoned = [p if k < b else rng.integers(0, 2 ** 32, size=p.size, dtype=np.uint32) for k, p in enumerate(planes)]
    y_poison = _run_gemv(pmpd, pmpd.upload_layer(poisoned, sm, out_f, in_f), b, x)
    absent = [p if k < b else None for k, p in enumerate(planes)]
    y_absent = _run_gemv(pmpd, pmpd.upload_layer(absent, sm, out_f, in_f), b, x)
    y_clean = _run_gemv(pmpd, pmpd.upload_layer(planes, sm, out_f, in_f), b, x)
    assert np.array_equal(y_poison, y_clean)
    assert np.array_equal(y_absent, y_clean)
    assert_parity(y_clean, y_ref[0], t[0], f"prefix b={b}")


@pytest.mark.parametrize("b", [4, 3, 2])
def test_gemv_adversarial_inputs(pmpd, b):
    _say(f"[gemv adversarial] b={b}")
    out_f, in_f = 128, 1024
    rng = np.random.default_rng(11)
    q_rand, s, a = synth.draw_weights(8, 2, 2, out_f, in_f, random_min=True)
    x_rand = synth.draw_x(8, 0, 2, 2, in_f)[0]
    G = in_f // 128
    cases = {}
    # codes: all zero, all fifteen, one plane only, alternating
    for name, q in (("zeros", np.zeros_like(q_rand)), ("fifteens", np.full_like(q_rand, 15)),
                    ("msb-only", np.full_like(q_rand, 8)), ("lsb-only", np.full_like(q_rand, 1)),
                    ("alternating", (np.arange(in_f, dtype=np.uint8) % 2 * 15)[None, :].repeat(out_f, 0))):
        cases["codes-" + name] = (q, s, a, x_rand)
    # scales at the ends of their range, minima far from -8 s
    s_ext = np.where(rng.random((out_f, G)) < 0.5, 1e-3, 1e-2).astype(np.float16)
    cases["scale-extremes"] = (q_rand, s_ext, a, x_rand)
    a_zero = np.zeros_like(a)
    cases["min-zero"] = (q_rand, s, a_zero, x_rand)
    # activations: zeros, ones, one-hot, one huge entry, tiny entries, single sign
    x_hot = np.zeros(in_f, dtype=np.float16); x_hot[517] = 1
    x_huge = x_rand.copy(); x_huge[300] = np.float16(30000.0)
    cases["x-zero"] = (q_rand, s, a, np.zeros(in_f, dtype=np.float16))
    cases["x-ones"] = (q_rand, s, a, np.ones(in_f, dtype=np.float16))
    cases["x-one-hot"] = (q_rand, s, a, x_hot)
    cases["x-huge-entry"] = (q_rand, s, a, x_huge)
    cases["x-tiny"] = (q_rand, s, a, (x_rand.astype(np.float32) * 1e-4).astype(np.float16))
    cases["x-positive"] = (q_rand, s, a, np.abs(x_rand))
    for name, (q, sv, av, xv) in cases.items():
        layer = _device_layer(pmpd, q, sv, av)
        y = _run_gemv(pmpd, layer, b, xv)
        y_ref, t = oracle.linear(q, sv, av, b, xv)
        assert_parity(y, y_ref[0], t[0], f"{name} b={b}")
    # one-hot activations must return the dequantised column exactly (one weight, no rounding)
    W = oracle.dequant(q_rand, s, a, b)
    y = _run_gemv(pmpd, _device_layer(pmpd, q_rand, s, a), b, x_hot)
    assert np.allclose(y, W[:, 517], rtol=2e-6, atol=0)


@pytest.mark.parametrize("b", [4, 3, 2])
@pytest.mark.parametrize("m", [1, 2, 3, 4, 8])
def test_gemm_skinny_matches_oracle(pmpd, b, m):
    import torch

    _say(f"[gemm] m={m} b={b}")
    for (out_f, in_f) in ((200, 2048), (128, 5632)):
        q4, s, a = synth.draw_weights(9, out_f, m, out_f, in_f, random_min=True)
        X = synth.draw_x(9, 0, out_f, m, in_f, m=m)
        layer = _device_layer(pmpd, q4, s, a)
        Y = pmpd.gemm(layer, b, torch.from_numpy(X).cuda())
        torch.cuda.synchronize()
        y_ref, t = oracle.linear(q4, s, a, b, X)
        assert_parity(Y.cpu().numpy(), y_ref, t, f"gemm {out_f}x{in_f} m={m} b={b}")


@pytest.mark.parametrize("b", [4, 3, 2])
@pytest.mark.parametrize("m", [9, 13, 16])
def test_gemm_one_token_block_matches_oracle(pmpd, b, m):
    """9 to 16 rows of X on a single layer: the fp16 kernel with the codes as subnormals.  Ragged row counts (one
    row tile, four and a bit), one group, an odd number of groups above one chunk of eight, and a row long enough
    for several chunks."""
    import torch

    _say(f"[gemm, one token block] m={m} b={b}")
    for (out_f, in_f) in ((200, 512), (70, 2432), (64, 128), (330, 5632)):
        q4, s, a = synth.draw_weights(14, out_f, m, out_f, in_f, random_min=True)
        X = synth.draw_x(14, 0, out_f, m, in_f, m=m)
        layer = _device_layer(pmpd, q4, s, a)
        Y = torch.full((m, out_f), float("nan"), dtype=torch.float32, device="cuda")
        pmpd.gemm(layer, b, torch.from_numpy(X).cuda(), Y)
        torch.cuda.synchronize()
        y_ref, t = oracle.linear(q4, s, a, b, X)
        assert_parity(Y.cpu().numpy(), y_ref, t, f"gemm {out_f}x{in_f} m={m} b={b}")


@pytest.mark.parametrize("b", [4, 3, 2])
# the prefill tile is 256 tokens x 4 row tiles of 64, groups taken two at a time: token counts around one and two
# tiles, ragged row counts (multiples of 4 and not), 1, 2, 3, 5 and 11 groups
@pytest.mark.parametrize("m,out_f,in_f", [(16, 200, 512), (100, 130, 2048), (512, 256, 1408), (129, 320, 5120),
                                          (257, 64, 128), (300, 192, 256), (256, 70, 384), (255, 64, 640), (513, 260, 256)])
def test_gemm_prefill_matches_oracle(pmpd, b, m, out_f, in_f):
    """m > 16 takes the prefill kernel (m = 16 the fp16 kernel of one token block): ragged M and N tiles, several
    K steps, all bit-widths."""
    import torch

    _say(f"[prefill gemm] m={m} out={out_f} in={in_f} b={b}")
    q4, s, a = synth.draw_weights(12, out_f, m, out_f, in_f, random_min=True)
    X = synth.draw_x(12, 0, out_f, m, in_f, m=m)
    layer = _device_layer(pmpd, q4, s, a)
    Y = torch.full((m, out_f), float("nan"), dtype=torch.float32, device="cuda")
    pmpd.gemm(layer, b, torch.from_numpy(X).cuda(), Y)
    torch.cuda.synchronize()
    y_ref, t = oracle.linear(q4, s, a, b, X)
    assert_parity(Y.cpu().numpy(), y_ref, t, f"prefill gemm m={m} {out_f}x{in_f} b={b}")


def test_gemm_prefill_into_a_y_that_is_not_16_byte_aligned(pmpd):
    """The prefill kernel stores 16 bytes per lane where Y allows it; a Y that starts 4 bytes off takes the scalar stores."""
    import torch

    m, out_f, in_f, b = 40, 128, 512, 4
    _say(f"[prefill gemm, unaligned Y] m={m} out={out_f} in={in_f} b={b}")
    q4, s, a = synth.draw_weights(14, out_f, m, out_f, in_f, random_min=True)
    X = synth.draw_x(14, 0, out_f, m, in_f, m=m)
    layer = _device_layer(pmpd, q4, s, a)
    buf = torch.full((m * out_f + 1,), float("nan"), dtype=torch.float32, device="cuda")
    Y = buf[1:].view(m, out_f)
    assert Y.data_ptr() % 16 == 4
    pmpd.gemm(layer, b, torch.from_numpy(X).cuda(), Y)
    torch.cuda.synchronize()
    y_ref, t = oracle.linear(q4, s, a, b, X)
    assert_parity(Y.cpu().numpy(), y_ref, t, "prefill gemm, unaligned Y")
    assert torch.isnan(buf[0]).item()  # the word before Y is untouched


@pytest.mark.parametrize("b", [4, 2])
def test_prefill_step_over_stack_matches_oracle(pmpd, b):
    import torch

    m = 70
    _say(f"[prefill_step] b={b} m={m}")
    shape, layers, raw = _small_stack(pmpd, seed=8)
    stack = pmpd.Stack(layers)
    Xs = [synth.draw_x(8, 0, blk, pi, i, m=m) for (blk, pi, nm, o, i) in shape.layers()]
    X = torch.from_numpy(np.concatenate([x.reshape(-1) for x in Xs])).cuda()
    Y = torch.full((m * stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    pmpd.prefill_step(stack, b, X, m, Y)
    torch.cuda.synchronize()
    Y = Y.cpu().numpy()
    for li, (q4, s, a) in enumerate(raw):
        o = m * stack.y_offsets[li]
        y_ref, t = oracle.linear(q4, s, a, b, Xs[li])
        got = Y[o:o + m * q4.shape[0]].reshape(m, q4.shape[0])
        assert_parity(got, y_ref, t, f"prefill_step layer {li} b={b}")
    stack.close()


@pytest.mark.parametrize("m", [40, 300])
def test_prefill_step_walks_many_short_items_per_workgroup(pmpd, m):
    """The prefill grid is one round of the chip and a workgroup walks through its items as one sequence of groups,
    with its loads up to three groups ahead.  Here every workgroup gets several items of one, two or three groups
    (more items than compute units, rows of 128, 256 and 384 columns, a ragged last tile), so the loads run ahead
    through up to three items at once; m = 300 also splits the tokens into two blocks."""
    import torch

    b = 4
    _say(f"[prefill_step, many short items] m={m}")
    dims = [(1000 + 8 * k, 128 * (1 + k % 3)) for k in range(45)]  # 16 to 22 row tiles: 4 to 6 items each
    dims = dims + [(2048, 128 * (1 + (k + 1) % 3)) for k in range(36)]  # 8 items each: 516 items in all
    layers, raw, Xs = [], [], []
    for li, (o, i) in enumerate(dims):
        q4, s_, a = synth.draw_weights(21, li, 0, o, i, random_min=(li % 2 == 1))
        raw.append((q4, s_, a))
        layers.append(_device_layer(pmpd, q4, s_, a))
        Xs.append(synth.draw_x(21, 0, li, 0, i, m=m))
    stack = pmpd.Stack(layers)
    X = torch.from_numpy(np.concatenate([x.reshape(-1) for x in Xs])).cuda()
    Y = torch.full((m * stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    pmpd.prefill_step(stack, b, X, m, Y)
    torch.cuda.synchronize()
    Y = Y.cpu().numpy()
    for li, (q4, s_, a) in enumerate(raw):
        o = m * stack.y_offsets[li]
        y_ref, t = oracle.linear(q4, s_, a, b, Xs[li])
        got = Y[o:o + m * q4.shape[0]].reshape(m, q4.shape[0])
        assert_parity(got, y_ref, t, f"prefill_step, short items, layer {li} ({q4.shape[0]} x {q4.shape[1]}) m={m}")
    stack.close()


@pytest.mark.parametrize("b", [4, 3, 2])
@pytest.mark.parametrize("m", [1, 2, 3, 4, 5, 8, 9, 12, 13, 16])
def test_batch_step_over_stack_matches_oracle(pmpd, b, m):
    import torch

    _say(f"[batch_step] b={b} m={m}")
    shape, layers, raw = _small_stack(pmpd, seed=9)
    stack = pmpd.Stack(layers)
    Xs = [synth.draw_x(9, 0, blk, pi, i, m=m) for (blk, pi, nm, o, i) in shape.layers()]
    X = torch.from_numpy(np.concatenate([x.reshape(-1) for x in Xs])).cuda()
    Y = torch.full((m * stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    pmpd.batch_step(stack, b, X, m, Y)
    torch.cuda.synchronize()
    Y = Y.cpu().numpy()
    for li, (q4, s, a) in enumerate(raw):
        o = m * stack.y_offsets[li]
        y_ref, t = oracle.linear(q4, s, a, b, Xs[li])
        assert_parity(Y[o:o + m * q4.shape[0]].reshape(m, q4.shape[0]), y_ref, t, f"batch_step layer {li} m={m} b={b}")
    stack.close()


@pytest.mark.parametrize("b", [4, 3, 2])
@pytest.mark.parametrize("m", [3, 7, 11, 16])
def test_batch_step_long_rows_and_adversarial_vectors(pmpd, b, m):
    """Rows long enough for several K-chunks of the batch kernels' activation images (86 and 33 groups, ragged
    row counts), and one vector of each awkward kind among ordinary ones: a huge entry among small ones, tiny
    values, subnormals, zeros, ones, a single sign, a one-hot vector.  Both batch kernels are met: the int8 one
    at 3 vectors (and at 7 for b = 3, 2), the fp16 one at 11 and 16 (and at 7 for b = 4)."""
    import torch

    _say(f"[batch_step long/adversarial] b={b} m={m}")
    shapes = [(130, 11008), (70, 4224), (64, 128)]
    raw = [synth.draw_weights(31, k, 0, o, i, random_min=(k == 1)) for k, (o, i) in enumerate(shapes)]
    layers = [_device_layer(pmpd, *w) for w in raw]
    stack = pmpd.Stack(layers)
    Xs = []
    for k, (o, i) in enumerate(shapes):
        X = synth.draw_x(31, 0, k, 0, i, m=m).copy()
        kinds = [
            lambda v: np.where(np.arange(i) == i // 3, np.float16(30000.0), (v.astype(np.float32) * 0.01).astype(np.float16)),
            lambda v: (v.astype(np.float32) * 1e-4).astype(np.float16),
            lambda v: (v.astype(np.float32) * 3e-7).astype(np.float16),          # fp16 subnormals
            lambda v: np.zeros(i, dtype=np.float16),
            lambda v: np.ones(i, dtype=np.float16),
            lambda v: np.abs(v),
            lambda v: (np.arange(i) == 5 * i // 7).astype(np.float16),
        ]
        for j in range(m):
            if j % 2 == 1 or m == 3:
                X[j] = kinds[(j // 2 + k) % len(kinds)](X[j])
        Xs.append(X)
    X = torch.from_numpy(np.concatenate([x.reshape(-1) for x in Xs])).cuda()
    Y = torch.full((m * stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    pmpd.batch_step(stack, b, X, m, Y)
    torch.cuda.synchronize()
    Y = Y.cpu().numpy()
    for li, (q4, s, a) in enumerate(raw):
        o = m * stack.y_offsets[li]
        y_ref, t = oracle.linear(q4, s, a, b, Xs[li])
        assert_parity(Y[o:o + m * q4.shape[0]].reshape(m, q4.shape[0]), y_ref, t, f"batch_step long layer {li} m={m} b={b}")
    stack.close()


@pytest.mark.parametrize("seed", list(range(8)))
def test_batch_step_random_shapes(pmpd, seed):
    """Stacks of layers with random row counts (1 to 400: below one tile, ragged, several workgroups) and 1 to 40
    groups (below, at and above one K-chunk of either batch kernel, odd and even), at a random batch of 3 to 16 and
    every bit-width."""
    import torch

    rng = np.random.default_rng(1000 + seed)
    m = int(rng.integers(3, 17))
    dims = [(int(rng.integers(1, 401)), 128 * int(rng.integers(1, 41))) for _ in range(5)]
    _say(f"[batch_step random] seed={seed} m={m} dims={dims}")
    raw = [synth.draw_weights(40 + seed, k, 0, o, i, random_min=(k % 2 == 0)) for k, (o, i) in enumerate(dims)]
    layers = [_device_layer(pmpd, *w) for w in raw]
    stack = pmpd.Stack(layers)
    Xs = [synth.draw_x(40 + seed, 0, k, 0, i, m=m) for k, (o, i) in enumerate(dims)]
    X = torch.from_numpy(np.concatenate([x.reshape(-1) for x in Xs])).cuda()
    for b in (4, 3, 2):
        Y = torch.full((m * stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
        pmpd.batch_step(stack, b, X, m, Y)
        torch.cuda.synchronize()
        Yh = Y.cpu().numpy()
        for li, (q4, s_, a) in enumerate(raw):
            o = m * stack.y_offsets[li]
            y_ref, t = oracle.linear(q4, s_, a, b, Xs[li])
            assert_parity(Yh[o:o + m * q4.shape[0]].reshape(m, q4.shape[0]), y_ref, t, f"batch_step random seed={seed} layer {li} {dims[li]} m={m} b={b}")
    stack.close()


def _small_stack(pmpd, seed=5):
    """A two-block stack with Llama-like proportions (hidden 256, intermediate 640, ragged)."""
    shape = synth.StackShape("tiny", 2, 256, 640)
    layers, raw = [], []
    for li, (blk, pi, nm, o, i) in enumerate(shape.layers()):
        q4, s, a = synth.draw_weights(seed, blk, pi, o, i, random_min=(pi % 2 == 1))
        raw.append((q4, s, a))
        layers.append(_device_layer(pmpd, q4, s, a))
    return shape, layers, raw


@pytest.mark.parametrize("b", [4, 3, 2])
def test_decode_step_matches_oracle_and_single_layer_calls(pmpd, b):
    import torch

    _say(f"[decode_step] b={b}")
    shape, layers, raw = _small_stack(pmpd)
    stack = pmpd.Stack(layers)
    xs = [synth.draw_x(5, 0, blk, pi, i)[0] for (blk, pi, nm, o, i) in shape.layers()]
    x = torch.from_numpy(np.concatenate(xs)).cuda()
    y = torch.full((stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    pmpd.decode_step(stack, b, x, y)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    for li, (q4, s, a) in enumerate(raw):
        o = stack.y_offsets[li]
        y_ref, t = oracle.linear(q4, s, a, b, xs[li])
        assert_parity(y[o:o + q4.shape[0]], y_ref[0], t[0], f"decode_step layer {li} b={b}")
    stack.close()


@pytest.mark.parametrize("variant", list(range(5)))
def test_every_stack_kernel_variant_matches_oracle(pmpd, variant):
    """Each launch shape of the one-launch decode step (selected per bit-width by default, forced
    here through the stack's setter and read back) gives the same answers."""
    import torch

    _say(f"[decode_step variant] {variant}")
    shape, layers, raw = _small_stack(pmpd, seed=10)
    stack = pmpd.Stack(layers)
    for b in (4, 3, 2):
        assert stack.variant(b) in range(5)
        stack.set_variant(b, variant)
        assert stack.variant(b) == variant
    xs = [synth.draw_x(10, 0, blk, pi, i)[0] for (blk, pi, nm, o, i) in shape.layers()]
    x = torch.from_numpy(np.concatenate(xs)).cuda()
    for b in (4, 3, 2):
        y = torch.full((stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
        pmpd.decode_step(stack, b, x, y)
        torch.cuda.synchronize()
        yh = y.cpu().numpy()
        for li, (q4, s, a) in enumerate(raw):
            o = stack.y_offsets[li]
            y_ref, t = oracle.linear(q4, s, a, b, xs[li])
            assert_parity(yh[o:o + q4.shape[0]], y_ref[0], t[0], f"variant {variant} layer {li} b={b}")
    stack.close()


def test_decode_run_follows_the_schedule(pmpd):
    import torch

    _say("[decode_run]")
    shape, layers, raw = _small_stack(pmpd, seed=6)
    stack = pmpd.Stack(layers)
    P, st, n_steps = (4, 3, 2), (0, 2, 5), 8
    sch = pmpd.Schedule(P, st, n_steps)
    xs = np.stack([np.concatenate([synth.draw_x(6, k, blk, pi, i)[0] for (blk, pi, nm, o, i) in shape.layers()])
                   for k in range(n_steps)])
    x = torch.from_numpy(xs).cuda()
    y = torch.zeros((n_steps, stack.y_elems), dtype=torch.float32, device="cuda")
    pmpd.decode_run(stack, sch, 0, n_steps, x, stack.x_elems, y, stack.y_elems)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    for k in range(n_steps):
        b = oracle.schedule_bits(P, st, k)
        assert sch.bits(k) == b
        for li, (q4, s, a) in enumerate(raw):
            xo, yo = stack.x_offsets[li], stack.y_offsets[li]
            y_ref, t = oracle.linear(q4, s, a, b, xs[k, xo:xo + q4.shape[1]])
            assert_parity(y[k, yo:yo + q4.shape[0]], y_ref[0], t[0], f"decode_run step {k} layer {li} b={b}")
    # a run that starts in the middle picks up the schedule at that step
    y2 = torch.zeros((3, stack.y_elems), dtype=torch.float32, device="cuda")
    pmpd.decode_run(stack, sch, 4, 3, x[4:], stack.x_elems, y2, stack.y_elems)
    torch.cuda.synchronize()
    assert np.array_equal(y2.cpu().numpy(), y[4:7])
    # an empty run launches nothing and leaves the output alone
    y3 = torch.full((stack.y_elems,), 3.0, dtype=torch.float32, device="cuda")
    pmpd.decode_run(stack, sch, 2, 0, x, stack.x_elems, y3, stack.y_elems)
    torch.cuda.synchronize()
    assert bool((y3 == 3.0).all())
    # steps past the schedule's horizon stay at the last precision reached
    y4 = torch.zeros((2, stack.y_elems), dtype=torch.float32, device="cuda")
    pmpd.decode_run(stack, sch, n_steps - 1, 2, x[n_steps - 2:], stack.x_elems, y4, stack.y_elems)
    torch.cuda.synchronize()
    assert sch.bits(n_steps + 5) == 2
    y4 = y4.cpu().numpy()
    for j, krow in enumerate((n_steps - 2, n_steps - 1)):
        for li, (q4, s, a) in enumerate(raw):
            xo, yo = stack.x_offsets[li], stack.y_offsets[li]
            y_ref, t = oracle.linear(q4, s, a, 2, xs[krow, xo:xo + q4.shape[1]])
            assert_parity(y4[j, yo:yo + q4.shape[0]], y_ref[0], t[0], f"decode_run past the horizon, row {j} layer {li}")
    stack.close()


def test_gpu_error_paths_do_not_launch(pmpd):
    import torch

    q4, s, a = synth.draw_weights(1, 0, 0, 64, 128)
    layer = _device_layer(pmpd, q4, s, a)
    x = torch.zeros(128, dtype=torch.float16, device="cuda")
    with pytest.raises(pmpd.PMPDError):
        pmpd.gemv(layer, 5, x)
    with pytest.raises(pmpd.PMPDError):
        pmpd.gemv(layer, 4, x[1:])  # misaligned view
    torch.cuda.synchronize()


def test_read_stream_runs_and_reports_its_bytes(pmpd):
    import torch

    buf = torch.zeros(160 * 1024 * 1024 // 4, dtype=torch.int32, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    n = pmpd.read_stream(buf, sink)
    torch.cuda.synchronize()
    assert n == 128 * 1024 * 1024  # rounded down to a multiple of 128 MiB
    assert int(sink.item()) == 0
    with pytest.raises(pmpd.PMPDError):
        pmpd.read_stream(buf[: 1024 * 1024], sink)  # too small


def test_steps_replay_from_a_captured_graph(pmpd):
    """A decode step, a batch step and a scheduled run captured in a HIP graph (through torch) replay to the eager
    result every time, with eager work of the same library between the replays; new activations written into the
    captured input buffer are picked up."""
    import torch

    _say("[graph replay]")
    shape, layers, raw = _small_stack(pmpd, seed=12)
    stack = pmpd.Stack(layers)
    m = 5
    x1 = torch.from_numpy(np.concatenate([synth.draw_x(12, 0, blk, pi, i)[0] for (blk, pi, nm, o, i) in shape.layers()])).cuda()
    xm = torch.from_numpy(np.concatenate([synth.draw_x(12, 1, blk, pi, i, m=m).reshape(-1) for (blk, pi, nm, o, i) in shape.layers()])).cuda()
    sch = pmpd.Schedule((4, 2), (0, 1), 2)
    y1 = torch.zeros(stack.y_elems, dtype=torch.float32, device="cuda")
    ym = torch.zeros(m * stack.y_elems, dtype=torch.float32, device="cuda")
    yr = torch.zeros((2, stack.y_elems), dtype=torch.float32, device="cuda")

    def work():
        pmpd.decode_step(stack, 3, x1, y1)
        pmpd.batch_step(stack, 4, xm, m, ym)
        pmpd.decode_run(stack, sch, 0, 2, x1, 0, yr, stack.y_elems)

    def eager_reference():
        work()
        torch.cuda.synchronize()
        return y1.clone(), ym.clone(), yr.clone()

    ref = eager_reference()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        work()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=side):
            work()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    for rep in range(4):
        if rep == 2:  # new activations in the captured buffers
            x1.copy_(torch.from_numpy(np.concatenate([synth.draw_x(13, 0, blk, pi, i)[0] for (blk, pi, nm, o, i) in shape.layers()])).cuda())
            ref = eager_reference()
        for t in (y1, ym, yr):
            t.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(y1, ref[0]) and torch.equal(ym, ref[1]) and torch.equal(yr, ref[2]), f"replay {rep}"
        # eager work between the replays
        pmpd.decode_step(stack, 2, x1, y1)
        torch.cuda.synchronize()
    stack.close()
