"""Full-size workloads, built exactly as bench.py builds them (same builder, same seed, every block) and run
through the calls bench.py times, so that the launch shape under test is the launch shape that is timed.
Outputs are checked on sampled rows of EVERY layer, which the CPU oracle computes one by one from the logical
weights kept for those rows (same tolerances as the element-wise parity tests); the 512-token prefill is
also checked on every output of three whole layers."""
import sys
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import oracle
import pmpd_synth as synth

pytestmark = pytest.mark.gpu

REL_L2 = 1e-3
ABS_FACTOR = 2e-3

# The launch shape pmpd_decode_step picks per bit-width (b = 4, 3, 2) for each benchmark stack (0: four tiles per
# workgroup, whole K per wave; 2: two tiles, K split in two).
EXPECTED_VARIANTS = {"7b": (0, 0, 2), "13b": (0, 0, 2), "mobile": (2, 0, 0)}


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _rows_for(blk, pi, out_f):
    """Rows kept per layer: first, last, both sides of the first tile boundary and of the last one, six random."""
    rng = np.random.default_rng(1000 * blk + pi)
    last_tile = (out_f - 1) // 64 * 64
    fixed = [0, 63, 64, last_tile - 1, last_tile, out_f - 1]
    rest = rng.choice(out_f, size=6, replace=False)
    return np.unique(np.concatenate([fixed, rest])).astype(np.int64)


def _check(got, y_ref, t, what):
    got = np.asarray(got, dtype=np.float64).reshape(y_ref.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - y_ref)
    assert np.all(err <= ABS_FACTOR * t), f"{what}: max-abs bound violated ({err.max():.3e})"
    rel = np.linalg.norm(got - y_ref) / np.linalg.norm(y_ref)
    assert rel <= REL_L2, f"{what}: relative L2 {rel:.3e}"


def _check_sampled_layers(shape, stack, kept, b, x_of_layer, y_host, m, what, layers=None):
    """Sampled rows of every layer (or of `layers`) of a step's output against the oracle.
    x_of_layer(li) -> fp16 [m, in]; y_host: the step's whole output in the stack's layout."""
    n = 0
    for (blk, pi), (rows, q4r, sr, ar) in kept.items():
        li = blk * 7 + pi
        if layers is not None and li not in layers:
            continue
        o = shape.proj_shapes()[pi][1]
        yo = m * stack.y_offsets[li]
        got = y_host[yo:yo + m * o].reshape(m, o)[:, rows]
        y_ref, t = oracle.linear(q4r, sr, ar, b, x_of_layer(li))
        _check(got, y_ref, t, f"{what} layer ({blk},{pi}) b={b}")
        n += 1
    return n


def _assert_variants(stack, name):
    got = tuple(stack.variant(b) for b in (4, 3, 2))
    assert got == EXPECTED_VARIANTS[name], f"{name} stack runs launch shapes {got}, the documented ones are {EXPECTED_VARIANTS[name]}"


@pytest.fixture(scope="module")
def pmpd():
    import torch

    assert torch.cuda.is_available()
    import paper_2410_13461_amd as lib

    return lib


# ------------------------------------------------------------------ 7B-shaped stack ----
@pytest.fixture(scope="module")
def stack7b(pmpd):
    """The Llama-7B-shaped stack exactly as bench.py builds it (seed 0, 32 blocks), a few rows of every layer kept."""
    from paper_2410_13461_amd import workload

    _say("[full-size] building the 7B-shaped stack (32 blocks)")
    stack, layers, kept = workload.build_stack(synth.LLAMA_7B, seed=0, keep_rows=_rows_for)
    assert len(layers) == 224 and len(kept) == 224
    yield stack, layers, kept
    stack.close()


def _x_slices(shape, stack, x):
    return lambda li: x[stack.x_offsets[li]:stack.x_offsets[li] + shape.proj_shapes()[li % 7][2]]


@pytest.mark.parametrize("b", [4, 3, 2])
def test_7b_decode_step_every_layer(pmpd, stack7b, b):
    import torch
    from paper_2410_13461_amd import workload

    stack, layers, kept = stack7b
    _say(f"[full-size 7B decode step] b={b}")
    _assert_variants(stack, "7b")
    x = workload.draw_step_activations(synth.LLAMA_7B, 0, 7)
    x_dev = torch.from_numpy(x).cuda()
    y_dev = torch.full((stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    pmpd.decode_step(stack, b, x_dev, y_dev)
    torch.cuda.synchronize()
    y = y_dev.cpu().numpy()
    assert np.all(np.isfinite(y))  # every row of every layer was written
    assert _check_sampled_layers(synth.LLAMA_7B, stack, kept, b, _x_slices(synth.LLAMA_7B, stack, x), y, 1, "7B") == 224


def test_7b_progressive_schedule_256_steps(pmpd, stack7b):
    """64 steps at 4 bits, 96 at 3, 96 at 2, fresh activations per step; every layer checked at the phase boundaries."""
    import torch
    from paper_2410_13461_amd import workload

    stack, layers, kept = stack7b
    P, st, n_steps = synth.SCHEDULE_7B_256
    sch = pmpd.Schedule(P, st, n_steps)
    assert sch.avg_bits(n_steps) == 2.875
    _say("[full-size 7B schedule] 256 steps")
    # only the checked steps get seeded activations of their own; the others reuse step 1's buffer
    check_steps = [0, 63, 64, 159, 160, 255]
    xs = {k: workload.draw_step_activations(synth.LLAMA_7B, 0, k) for k in check_steps + [1]}
    x_all = torch.empty((n_steps, stack.x_elems), dtype=torch.float16, device="cuda")
    filler = torch.from_numpy(xs[1]).cuda()
    for k in range(n_steps):
        x_all[k] = torch.from_numpy(xs[k]).cuda() if k in xs else filler
    y_all = torch.zeros((n_steps, stack.y_elems), dtype=torch.float32, device="cuda")
    pmpd.decode_run(stack, sch, 0, n_steps, x_all, stack.x_elems, y_all, stack.y_elems)
    torch.cuda.synchronize()
    for k in check_steps:
        b = oracle.schedule_bits(P, st, k)
        y = y_all[k].cpu().numpy()
        n = _check_sampled_layers(synth.LLAMA_7B, stack, kept, b, _x_slices(synth.LLAMA_7B, stack, xs[k]), y, 1, f"schedule step {k}")
        assert n == 224
    # steps of one phase that share activations give identical results; across a switch they differ
    assert torch.equal(y_all[2], y_all[3])
    assert not torch.equal(y_all[65], y_all[1])


# ------------------------------------------------------------- mobile-scale stack ----
@pytest.fixture(scope="module")
def stack_mobile(pmpd):
    """The mobile-scale stack as `bench.py --workload mobile` builds its first copy (seed 0, 22 blocks)."""
    from paper_2410_13461_amd import workload

    _say("[full-size] building the mobile-scale stack (22 blocks)")
    stack, layers, kept = workload.build_stack(synth.MOBILE, seed=0, keep_rows=_rows_for)
    assert len(layers) == 154
    yield stack, layers, kept
    stack.close()


def _draw_batch(shape, seed, m, n_blocks, workers=8):
    """Per-layer activations [m, in] of one batched step, and their concatenation in the stack's layout."""
    jobs = [(blk, pi, i) for blk in range(n_blocks) for pi, (nm, o, i) in enumerate(shape.proj_shapes())]
    with ThreadPoolExecutor(max_workers=workers) as pool:
        Xs = list(pool.map(lambda j: synth.draw_x(seed, 0, j[0], j[1], j[2], m=m), jobs))
    return Xs


@pytest.mark.parametrize("m", [1, 2, 3, 4, 8, 16])
def test_mobile_stack_batches_every_layer(pmpd, stack_mobile, m):
    """The 22-block stack at batch 1, 2, 3, 4, 8, 16 and every bit-width through pmpd_batch_step, the call the
    benchmark times: sampled rows of all 154 layers, every vector of the batch."""
    import torch

    shape = synth.MOBILE
    stack, layers, kept = stack_mobile
    _say(f"[full-size mobile] m={m}")
    _assert_variants(stack, "mobile")
    Xs = _draw_batch(shape, 3, m, shape.n_blocks)
    X = torch.from_numpy(np.concatenate([x.reshape(-1) for x in Xs])).cuda()
    Y = torch.empty(m * stack.y_elems, dtype=torch.float32, device="cuda")
    for b in (4, 3, 2):
        Y.fill_(float("nan"))
        pmpd.batch_step(stack, b, X, m, Y)
        torch.cuda.synchronize()
        Yh = Y.cpu().numpy()
        assert np.all(np.isfinite(Yh))
        assert _check_sampled_layers(shape, stack, kept, b, lambda li: Xs[li], Yh, m, f"mobile m={m}") == 154
    if m <= 8:  # the single-layer entry point takes its own path for these batches: three shapes of the last block
        for pi in (0, 4, 5):
            li = 21 * 7 + pi
            rows, q4r, sr, ar = kept[(21, pi)]
            for b in (4, 3, 2):
                G = pmpd.gemm(layers[li], b, torch.from_numpy(Xs[li]).cuda())
                torch.cuda.synchronize()
                y_ref, t = oracle.linear(q4r, sr, ar, b, Xs[li])
                _check(G.cpu().numpy()[:, rows], y_ref, t, f"mobile gemm layer (21,{pi}) m={m} b={b}")


# ------------------------------------------------------------------ 13B-shaped stack ----
FULL_13B = ((0, 0), (20, 4), (39, 5))  # whole layers kept for the prefill: q 5120x5120, up 13824x5120, down 5120x13824


@pytest.fixture(scope="module")
def stack13b(pmpd):
    """The 13B-shaped stack as `bench.py --workload 13b` builds it (seed 0, 40 blocks)."""
    from paper_2410_13461_amd import workload

    _say("[full-size] building the 13B-shaped stack (40 blocks)")
    stack, layers, kept = workload.build_stack(synth.LLAMA_13B, seed=0, keep_host=set(FULL_13B), keep_rows=_rows_for)
    assert len(layers) == 280
    full = {k: kept.pop(k) for k in FULL_13B}
    for (blk, pi), (q4, s, a) in full.items():  # the whole layers also serve as sampled ones
        rows = _rows_for(blk, pi, q4.shape[0])
        kept[(blk, pi)] = (rows, q4[rows].copy(), s[rows].copy(), a[rows].copy())
    yield stack, layers, kept, full
    stack.close()


def test_13b_prefill_512_tokens_full_stack(pmpd, stack13b):
    """512-token prefill at b = 4 over all 280 layers in one call (the call and the size the benchmark times):
    every output of three whole layers, and sampled rows x sampled tokens of every other layer."""
    import torch

    shape = synth.LLAMA_13B
    stack, layers, kept, full = stack13b
    m = 512
    _say("[full-size 13B prefill] drawing 512 tokens for 280 layers")
    Xs = _draw_batch(shape, 4, m, shape.n_blocks, workers=16)
    X_dev = torch.empty(m * stack.x_elems, dtype=torch.float16, device="cuda")
    for li, x in enumerate(Xs):
        xo = m * stack.x_offsets[li]
        X_dev[xo:xo + x.size] = torch.from_numpy(x.reshape(-1)).cuda()
    Y_dev = torch.full((m * stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    _say("[full-size 13B prefill] running")
    pmpd.prefill_step(stack, 4, X_dev, m, Y_dev)
    torch.cuda.synchronize()
    assert bool(torch.isfinite(Y_dev).all())  # every output of every layer was written
    toks = np.array([0, 1, 15, 16, 127, 128, 255, 256, 300, 511])
    for (blk, pi), (rows, q4r, sr, ar) in kept.items():
        li = blk * 7 + pi
        o = shape.proj_shapes()[pi][1]
        yo = m * stack.y_offsets[li]
        got = Y_dev[yo:yo + m * o].view(m, o)[torch.from_numpy(toks).cuda()][:, torch.from_numpy(rows).cuda()].cpu().numpy()
        y_ref, t = oracle.linear(q4r, sr, ar, 4, Xs[li][toks])
        _check(got, y_ref, t, f"13B prefill layer ({blk},{pi})")
    for (blk, pi), (q4, s, a) in full.items():
        _say(f"[full-size 13B prefill] whole layer ({blk},{pi})")
        li = blk * 7 + pi
        o = q4.shape[0]
        yo = m * stack.y_offsets[li]
        got = Y_dev[yo:yo + m * o].view(m, o).cpu().numpy()
        y_ref, t = oracle.linear_dense(q4, s, a, 4, Xs[li])
        _check(got, y_ref, t, f"13B prefill whole layer ({blk},{pi})")


def test_13b_decode_128_steps_full_stack(pmpd, stack13b):
    """128 decode steps over all 280 layers, 3 bits for steps 0..47 and 2 bits from step 48; every layer checked at
    steps 0, 47, 48 and 127."""
    import torch
    from paper_2410_13461_amd import workload

    shape = synth.LLAMA_13B
    stack, layers, kept, full = stack13b
    _assert_variants(stack, "13b")
    P, st, n_steps = synth.SCHEDULE_13B_128
    sch = pmpd.Schedule(P, st, n_steps)
    assert sch.avg_bits(n_steps) == 2.375
    check_steps = [0, 47, 48, 127]
    _say("[full-size 13B decode] 128 steps")
    xs = {k: workload.draw_step_activations(shape, 4, k) for k in check_steps}
    x_all = torch.zeros((n_steps, stack.x_elems), dtype=torch.float16, device="cuda")
    for k in check_steps:
        x_all[k] = torch.from_numpy(xs[k]).cuda()
    y_all = torch.zeros((n_steps, stack.y_elems), dtype=torch.float32, device="cuda")
    pmpd.decode_run(stack, sch, 0, n_steps, x_all, stack.x_elems, y_all, stack.y_elems)
    torch.cuda.synchronize()
    for k in check_steps:
        b = oracle.schedule_bits(P, st, k)
        assert b == (3 if k < 48 else 2)
        y = y_all[k].cpu().numpy()
        assert _check_sampled_layers(shape, stack, kept, b, _x_slices(shape, stack, xs[k]), y, 1, f"13B step {k}") == 280
    # b = 4 on the same stack (the prefill precision, one token): launch shape 0 over 108-group rows
    y = torch.full((stack.y_elems,), float("nan"), dtype=torch.float32, device="cuda")
    pmpd.decode_step(stack, 4, x_all[0], y)
    torch.cuda.synchronize()
    assert _check_sampled_layers(shape, stack, kept, 4, _x_slices(shape, stack, xs[0]), y.cpu().numpy(), 1, "13B b=4") == 280
