"""The unquantised fp16 matrix-vector reference (the denominator of the paper's Table-3-style speedups)
against the fp64 definition, single layers and a ragged list of layers in one launch."""
import numpy as np
import pytest

import oracle
import pmpd_synth as synth

pytestmark = pytest.mark.gpu

# fp16 x fp16 products are exact in fp32; only the fp32 accumulation rounds: about in * 2^-24 relative to
# sum |w||x| in the worst case, far inside the bar the quantised path is held to.
REL_L2 = 1e-5
ABS_FACTOR = 1e-5


@pytest.fixture(scope="module")
def pmpd():
    import torch

    assert torch.cuda.is_available()
    import paper_2410_13461_amd as lib

    return lib


def _check(y_gpu, y_ref, budget):
    y_gpu = np.asarray(y_gpu, dtype=np.float64)
    assert np.all(np.isfinite(y_gpu))
    rel = np.linalg.norm(y_gpu - y_ref) / max(np.linalg.norm(y_ref), 1e-30)
    assert rel <= REL_L2, rel
    assert np.all(np.abs(y_gpu - y_ref) <= ABS_FACTOR * budget + 1e-30)


@pytest.mark.parametrize("out_f,in_f", [(1, 128), (3, 256), (33, 384), (64, 4096), (100, 11008), (517, 5120),
                                         (4096, 4096), (40, 32768)])
def test_fp16_gemv_matches_the_definition(pmpd, out_f, in_f):
    import torch

    W = synth.draw_fp16_weights(11, 0, 0, out_f, in_f)
    x = synth.draw_x(11, 0, 0, 0, in_f)[0]
    y_ref, t = oracle.linear_fp16(W, x)
    y = pmpd.fp16_gemv(torch.from_numpy(W).cuda(), torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    _check(y.cpu().numpy(), y_ref[0], t[0])


def test_fp16_gemv_special_values(pmpd):
    """Integer weights and inputs: every partial sum is exact in fp32, so the result is the integer itself."""
    import torch

    out_f, in_f = 70, 1408
    W = (np.arange(out_f)[:, None] % 7 - 3 + (np.arange(in_f)[None, :] % 5)).astype(np.float16)
    x = ((np.arange(in_f) % 9) - 4).astype(np.float16)
    y = pmpd.fp16_gemv(torch.from_numpy(W).cuda(), torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    exact = W.astype(np.int64) @ x.astype(np.int64)
    assert np.array_equal(y.cpu().numpy().astype(np.int64), exact)
    assert np.array_equal(y.cpu().numpy(), exact.astype(np.float32))


def test_fp16_stack_one_launch_ragged_layers(pmpd):
    import torch

    shapes = [(64, 256), (1, 128), (97, 1408), (300, 512), (32, 128), (2050, 2048)]
    Ws = [synth.draw_fp16_weights(5, k, 0, o, i) for k, (o, i) in enumerate(shapes)]
    xs = [synth.draw_x(5, 0, k, 0, i)[0] for k, (o, i) in enumerate(shapes)]
    dW = [torch.from_numpy(W).cuda() for W in Ws]
    st = pmpd.Fp16Stack(dW)
    x = torch.from_numpy(np.concatenate(xs)).cuda()
    y = torch.full((st.y_elems + 5,), -7.0, dtype=torch.float32, device="cuda")
    pmpd.fp16_step(st, x, y)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    assert np.all(yh[st.y_elems:] == -7.0)  # nothing written past the last layer's rows
    for k, (o, i) in enumerate(shapes):
        y_ref, t = oracle.linear_fp16(Ws[k], xs[k])
        _check(yh[st.y_offsets[k]:st.y_offsets[k] + o], y_ref[0], t[0])
    # a second step with other activations overwrites every output
    xs2 = [synth.draw_x(6, 1, k, 0, i)[0] for k, (o, i) in enumerate(shapes)]
    pmpd.fp16_step(st, torch.from_numpy(np.concatenate(xs2)).cuda(), y)
    torch.cuda.synchronize()
    yh = y.cpu().numpy()
    for k, (o, i) in enumerate(shapes):
        y_ref, t = oracle.linear_fp16(Ws[k], xs2[k])
        _check(yh[st.y_offsets[k]:st.y_offsets[k] + o], y_ref[0], t[0])
    st.close()


def test_fp16_reference_of_dequantised_weights_agrees_with_the_quantised_path(pmpd):
    """W_4 rounded to fp16 and run through the fp16 kernel lands within fp16 rounding of the 4-bit pass:
    the two kernels compute the same layer."""
    import torch

    out_f, in_f = 256, 1024
    q4, s, a = synth.draw_weights(3, 0, 0, out_f, in_f)
    x = synth.draw_x(3, 0, 0, 0, in_f)[0]
    W16 = oracle.dequant(q4, s, a, 4).astype(np.float16)
    y16 = pmpd.fp16_gemv(torch.from_numpy(W16).cuda(), torch.from_numpy(x).cuda()).cpu().numpy()
    planes, sm = pmpd.pack(q4, s, a)
    lay = pmpd.upload_layer(planes, sm, out_f, in_f)
    yq = pmpd.gemv(lay, 4, torch.from_numpy(x).cuda()).cpu().numpy()
    _, t = oracle.linear(q4, s, a, 4, x)
    assert np.all(np.abs(y16.astype(np.float64) - yq) <= 2.0 ** -10 * t[0])
