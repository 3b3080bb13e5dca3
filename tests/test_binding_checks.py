"""CPU-only tests of what the Python binding refuses before anything reaches the C ABI.

The library gets bare addresses, so a host tensor, another element type, a strided view or a
buffer shorter than the call touches would become a wild access inside a kernel: the binding
checks those four things for every tensor argument and raises before any launch."""
import types

import numpy as np
import pytest
import torch

import paper_2410_13461_amd as pmpd
from paper_2410_13461_amd import binding


def test_dev_ptr_refuses_host_dtype_stride_and_size():
    x = torch.zeros(256, dtype=torch.float16)
    with pytest.raises(pmpd.PMPDError, match="device memory"):
        binding._dev_ptr(x, "float16", 256, "x")
    with pytest.raises(pmpd.PMPDError, match="expected a torch tensor"):
        binding._dev_ptr(np.zeros(4, dtype=np.float16), "float16", 4, "x")


class _FakeCuda(torch.Tensor):
    """A host tensor whose is_cuda says True, so that the later checks can be reached without a GPU.
    Nothing is ever launched with it: every case below must raise first."""

    @staticmethod
    def __new__(cls, t):
        return torch.Tensor._make_subclass(cls, t)

    @property
    def is_cuda(self):
        return True


def test_dev_ptr_checks_after_the_device_check():
    x = _FakeCuda(torch.zeros(256, dtype=torch.float32))
    with pytest.raises(pmpd.PMPDError, match="dtype"):
        binding._dev_ptr(x, "float16", 256, "x")
    x = _FakeCuda(torch.zeros(512, dtype=torch.float16)[::2])
    with pytest.raises(pmpd.PMPDError, match="not contiguous"):
        binding._dev_ptr(x, "float16", 256, "x")
    x = _FakeCuda(torch.zeros(255, dtype=torch.float16))
    with pytest.raises(pmpd.PMPDError, match="needs 256") as e:
        binding._dev_ptr(x, "float16", 256, "x")
    assert e.value.status == -5
    ok = _FakeCuda(torch.zeros(256, dtype=torch.float16))
    assert binding._dev_ptr(ok, "float16", 256, "x").value == ok.data_ptr()
    assert binding._dev_ptr(ok, "any", 1, "x").value == ok.data_ptr()


def _host_layer(out_f=64, in_f=128):
    pb, sb = pmpd.packed_size(out_f, in_f)
    planes = [torch.zeros(pb // 4, dtype=torch.int32) for _ in range(4)]
    return pmpd.PackedLayer(out_f, in_f, planes, torch.zeros(sb // 4, dtype=torch.int32))


def test_gemv_and_gemm_refuse_host_tensors_before_any_launch():
    lay = _host_layer()
    with pytest.raises(pmpd.PMPDError, match="gemv x"):
        pmpd.gemv(lay, 4, torch.zeros(128, dtype=torch.float16))
    with pytest.raises(pmpd.PMPDError, match="gemm X"):
        pmpd.gemm(lay, 4, torch.zeros((2, 128), dtype=torch.float16))
    with pytest.raises(pmpd.PMPDError, match=r"expected \[m, 128\]"):
        pmpd.gemm(lay, 4, _FakeCuda(torch.zeros((2, 256), dtype=torch.float16)))
    # activations that pass: the layer's own tensors are checked next (host memory here)
    with pytest.raises(pmpd.PMPDError, match=r"planes\[0\]"):
        pmpd.gemv(lay, 4, _FakeCuda(torch.zeros(128, dtype=torch.float16)), _FakeCuda(torch.zeros(64)))
    short = _host_layer()
    short.planes[0] = _FakeCuda(torch.zeros(8, dtype=torch.int32))
    with pytest.raises(pmpd.PMPDError, match=r"planes\[0\].*needs 256"):
        short.struct()


def _fake_stack(x_elems=1024, y_elems=512):
    st = pmpd.Stack.__new__(pmpd.Stack)
    st.x_elems, st.y_elems, st._h = x_elems, y_elems, None
    return st


@pytest.mark.parametrize("call", ["decode_step", "batch_step", "prefill_step", "decode_run", "ordered"])
def test_stack_calls_refuse_short_or_wrong_buffers(call):
    st = _fake_stack()
    good_x = _FakeCuda(torch.zeros(4 * 1024, dtype=torch.float16))
    good_y = _FakeCuda(torch.zeros(4 * 512, dtype=torch.float32))
    bad = [
        (torch.zeros(4 * 1024, dtype=torch.float16), good_y, "device memory"),
        (_FakeCuda(torch.zeros(4 * 1024, dtype=torch.float32)), good_y, "dtype"),
        (good_x, _FakeCuda(torch.zeros(4 * 512, dtype=torch.float16)), "dtype"),
        (_FakeCuda(torch.zeros(100, dtype=torch.float16)), good_y, "needs"),
        (good_x, _FakeCuda(torch.zeros(100, dtype=torch.float32)), "needs"),
    ]
    for x, y, what in bad:
        with pytest.raises(pmpd.PMPDError, match=what):
            if call == "decode_step":
                pmpd.decode_step(st, 4, x, y)
            elif call == "batch_step":
                pmpd.batch_step(st, 4, x, 4, y)
            elif call == "prefill_step":
                pmpd.prefill_step(st, 4, x, 4, y)
            elif call == "decode_run":
                sch = types.SimpleNamespace(_h=None)
                pmpd.decode_run(st, sch, 0, 4, x, 1024, y, 512)
            else:
                o = pmpd.Ordered.__new__(pmpd.Ordered)
                o.stack, o._h = st, None
                o.step(4, x, y)


def test_batch_sizes_scale_the_required_length():
    st = _fake_stack()
    x = _FakeCuda(torch.zeros(2 * 1024, dtype=torch.float16))
    y = _FakeCuda(torch.zeros(4 * 512, dtype=torch.float32))
    with pytest.raises(pmpd.PMPDError, match="needs 4096"):
        pmpd.batch_step(st, 4, x, 4, y)
    with pytest.raises(pmpd.PMPDError, match="needs 4096"):
        pmpd.decode_run(st, types.SimpleNamespace(_h=None), 0, 4, x, 1024, y, 512)


def test_fp16_and_learned_wrappers_refuse_host_tensors():
    W = torch.zeros((64, 128), dtype=torch.float16)
    with pytest.raises(pmpd.PMPDError, match="fp16_gemv W"):
        pmpd.fp16_gemv(W, torch.zeros(128, dtype=torch.float16))
    with pytest.raises(pmpd.PMPDError, match="fp16_gemv x"):
        pmpd.fp16_gemv(_FakeCuda(W), torch.zeros(128, dtype=torch.float16))
    with pytest.raises(pmpd.PMPDError, match="Fp16Stack weight"):
        pmpd.Fp16Stack([W])
    net = pmpd.LearnedScheduler.__new__(pmpd.LearnedScheduler)
    net.d_k, net.d_v, net.hidden, net.n_classes = 64, 64, 8, 3
    with pytest.raises(pmpd.PMPDError, match="learned scheduler K"):
        net.forward(torch.zeros((16, 64), dtype=torch.float16), torch.zeros((16, 64), dtype=torch.float16))
    with pytest.raises(pmpd.PMPDError, match="do not fit"):
        net.forward(_FakeCuda(torch.zeros((16, 32), dtype=torch.float16)), _FakeCuda(torch.zeros((16, 64), dtype=torch.float16)))
    with pytest.raises(pmpd.PMPDError, match="read_stream buf"):
        pmpd.read_stream(torch.zeros(1 << 20, dtype=torch.int32), torch.zeros(1, dtype=torch.int32))
