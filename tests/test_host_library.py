"""CPU-side tests of the native library: exported symbols, storage format against the
oracle's independent implementation, argument validation, and the schedule."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import pmpd_synth as synth
import paper_2410_13461_amd as pmpd
from paper_2410_13461_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "pmpd.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(pmpd_[a-z_0-9]+)\s*\(", header))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(pmpd.lib_path())
    missing = [n for n in sorted(declared) if not hasattr(lib, n)]
    assert not missing, f"declared but not exported: {missing}"
    assert set(binding.EXPORTS) == declared
    assert set(pmpd.exported_symbols()) == declared


def test_packed_size():
    assert pmpd.packed_size(4096, 4096) == (4096 * 4096 // 8, 4096 * 32 * 4)
    assert pmpd.packed_size(65, 128) == (128 * 128 // 8, 128 * 4)
    for bad in [(0, 128, 128), (64, 100, 128), (64, 128, 64), (-1, 128, 128), (64, 0, 128)]:
        with pytest.raises(pmpd.PMPDError) as e:
            pmpd.packed_size(*bad)
        assert e.value.status == -1


@pytest.mark.parametrize("out_f,in_f", [(64, 128), (100, 384), (257, 1408)])
def test_pack_is_byte_exact_with_the_oracle(out_f, in_f):
    q4, s, a = synth.draw_weights(21, 0, 0, out_f, in_f, random_min=True)
    planes, sm = pmpd.pack(q4, s, a)
    oplanes, osm = oracle.pack(q4, s, a)
    for k in range(4):
        assert np.array_equal(planes[k], oplanes[k]), f"plane {k} differs"
    assert np.array_equal(sm, osm)


@pytest.mark.parametrize("out_f,in_f", [(70, 256), (64, 128)])
def test_unpack_round_trip_prefix_and_cross_check(out_f, in_f):
    q4, s, a = synth.draw_weights(22, 0, 0, out_f, in_f)
    planes, sm = pmpd.pack(q4, s, a)
    rng = np.random.default_rng(5)
    for b in (4, 3, 2, 1):
        want = q4 >> (4 - b)
        assert np.array_equal(pmpd.unpack(planes, b, out_f, in_f), want)
        # lower planes poisoned or absent: same answer
        junk = list(planes[:b]) + [rng.integers(0, 2 ** 32, size=planes[0].size, dtype=np.uint32) for _ in range(4 - b)]
        assert np.array_equal(pmpd.unpack(junk, b, out_f, in_f), want)
        assert np.array_equal(pmpd.unpack(list(planes[:b]) + [None] * (4 - b), b, out_f, in_f), want)
        # each side unpacks what the other packed
        assert np.array_equal(oracle.unpack(planes, b, out_f, in_f), want)
        oplanes, _ = oracle.pack(q4, s, a)
        assert np.array_equal(pmpd.unpack(oplanes, b, out_f, in_f), want)


def test_pack_rejects_bad_input():
    q4, s, a = synth.draw_weights(1, 0, 0, 64, 128)
    bad = q4.copy()
    bad[0, 0] = 31
    with pytest.raises(pmpd.PMPDError) as e:
        pmpd.pack(bad, s, a)
    assert e.value.status == -1
    with pytest.raises(pmpd.PMPDError):
        pmpd.pack(q4, s[:, :0], a)
    with pytest.raises(pmpd.PMPDError):
        pmpd.pack(q4[:, :100], s, a)


def _host_layer(out_f=64, in_f=128):
    """A layer struct with fake (never dereferenced) aligned addresses for validation tests."""
    lay = binding._Layer(out_f, in_f, 128, 0)
    for k in range(4):
        lay.planes[k] = 0x10000 + 0x1000 * k
    lay.scale_min = 0x20000
    return lay


def test_gemv_argument_validation_needs_no_gpu():
    L = binding._load()
    x, y = ctypes.c_void_p(0x30000), ctypes.c_void_p(0x40000)

    def call(lay, b, xx=x, yy=y):
        return L.pmpd_gemv(ctypes.byref(lay), b, xx, yy, None)

    assert call(_host_layer(), 5) == -1
    assert call(_host_layer(), 1) == -1
    assert b"bit-width" in L.pmpd_last_error()
    assert call(_host_layer(in_f=100), 4) == -1
    assert call(_host_layer(out_f=0), 4) == -1
    lay = _host_layer()
    lay.group_size = 64
    assert call(lay, 4) == -1
    lay = _host_layer()
    lay.reserved = 7
    assert call(lay, 4) == -1
    lay = _host_layer()
    lay.planes[2] = None
    assert call(lay, 3) == -1  # b=3 needs planes 0..2
    lay = _host_layer()
    lay.planes[1] = 0x10008
    assert call(lay, 4) == -2
    lay = _host_layer()
    lay.scale_min = 0x20002
    assert call(lay, 4) == -2
    assert call(_host_layer(), 4, xx=ctypes.c_void_p(0x30008)) == -2
    assert call(_host_layer(), 4, yy=ctypes.c_void_p(0x40002)) == -2
    assert call(_host_layer(), 4, xx=None) == -1
    assert L.pmpd_gemv(None, 4, x, y, None) == -1
    assert L.pmpd_gemm(ctypes.byref(_host_layer()), 4, x, 0, y, None) == -1
    assert L.pmpd_gemm(ctypes.byref(_host_layer()), 4, x, 65537, y, None) == -1
    assert L.pmpd_batch_step(None, 4, x, 2, y, None) == -1
    assert L.pmpd_batch_step(ctypes.c_void_p(0x1234), 4, x, 2, ctypes.c_void_p(0x40002), None) == -2
    assert L.pmpd_prefill_step(None, 4, x, 16, y, None) == -1
    assert L.pmpd_prefill_step(ctypes.c_void_p(0x1234), 4, x, 0, y, None) == -1
    assert L.pmpd_prefill_step(ctypes.c_void_p(0x1234), 1, x, 16, y, None) == -1
    assert L.pmpd_decode_step(None, 4, x, y, None) == -1
    assert L.pmpd_decode_step(ctypes.c_void_p(0x1234), 7, x, y, None) == -1
    assert L.pmpd_strerror(-2) == b"misaligned buffer"
    assert L.pmpd_strerror(0) == b"ok"


def test_stack_argument_validation_needs_no_gpu():
    L = binding._load()
    arr = (binding._Layer * 2)(_host_layer(), _host_layer(128, 256))
    need = ctypes.c_size_t()
    assert L.pmpd_stack_workspace_size(arr, 2, ctypes.byref(need)) == 0
    assert need.value >= 2 * 72 + 8 and need.value % 256 == 0
    assert L.pmpd_stack_workspace_size(arr, 0, ctypes.byref(need)) == -1
    assert L.pmpd_stack_workspace_size(None, 2, ctypes.byref(need)) == -1
    xo = (ctypes.c_int64 * 2)(0, 128)
    yo = (ctypes.c_int64 * 2)(0, 64)
    h = ctypes.c_void_p()
    assert L.pmpd_stack_create(arr, 2, xo, yo, None, 4096, ctypes.byref(h)) == -1
    assert L.pmpd_stack_create(arr, 2, xo, yo, ctypes.c_void_p(0x50010), 4096, ctypes.byref(h)) == -2
    bad_xo = (ctypes.c_int64 * 2)(0, 100)
    assert L.pmpd_stack_create(arr, 2, bad_xo, yo, ctypes.c_void_p(0x50000), 4096, ctypes.byref(h)) == -2
    assert L.pmpd_stack_create(arr, 2, xo, yo, ctypes.c_void_p(0x50000), 16, ctypes.byref(h)) == -5


# ------------------------------------------------------------------ schedule ----
def test_schedule_matches_oracle_and_closed_forms():
    for (P, st, OL) in (synth.SCHEDULE_7B_256, synth.SCHEDULE_13B_128, ((4, 3, 2), (0, 10, 10), 32),
                        ((3, 2), (0, 0), 50), ((4, 3, 2), (0, 5, 256), 256), ((4,), (0,), 8)):
        sch = pmpd.Schedule(P, st, OL)
        for k in range(OL):
            assert sch.bits(k) == oracle.schedule_bits(P, st, k)
        for n in (1, OL // 2, OL):
            assert sch.avg_bits(n) == pytest.approx(oracle.schedule_avg_bits(P, st, n), abs=1e-15)
        sch.close()
    sch = pmpd.Schedule(*synth.SCHEDULE_7B_256)
    assert sch.avg_bits(256) == 2.875
    assert [sch.bits(k) for k in (0, 63, 64, 159, 160, 255, 1000)] == [4, 4, 3, 3, 2, 2, 2]
    sch = pmpd.Schedule(*synth.SCHEDULE_13B_128)
    assert sch.avg_bits(128) == 2.375


@pytest.mark.parametrize("P,st,OL,status", [
    ((4, 3, 2), (0, 9, 5), 256, -3),   # precedence (Eq. 3)
    ((4, 3), (0, 300), 256, -3),       # range (Eq. 2)
    ((4, 3), (0, -1), 256, -3),
    ((4, 3), (2, 5), 256, -3),         # decoding starts at the decode precision
    ((3, 4), (0, 5), 256, -1),         # precisions must decrease
    ((4, 4), (0, 5), 256, -1),
    ((4, 3), (0, 5), 0, -1),
    ((), (), 16, -1),
])
def test_schedule_rejects_invalid(P, st, OL, status):
    with pytest.raises(pmpd.PMPDError) as e:
        pmpd.Schedule(P, st, OL)
    assert e.value.status == status
    if len(P) == len(st) and len(P) > 0 and OL > 0:
        assert not oracle.schedule_valid(P, st, OL)


def test_schedule_bits_rejects_negative_step():
    sch = pmpd.Schedule((4, 3), (0, 4), 8)
    with pytest.raises(pmpd.PMPDError):
        sch.bits(-1)
    with pytest.raises(pmpd.PMPDError):
        sch.avg_bits(0)


def test_fp16_reference_argument_validation_needs_no_gpu():
    L = binding._load()
    w, x, y = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x30000), ctypes.c_void_p(0x40000)
    assert L.pmpd_fp16_gemv(None, 64, 128, x, y, None) == -1
    assert L.pmpd_fp16_gemv(w, 0, 128, x, y, None) == -1
    assert L.pmpd_fp16_gemv(w, 64, 100, x, y, None) == -1
    assert L.pmpd_fp16_gemv(w, 64, 32768 + 128, x, y, None) == -1
    assert L.pmpd_fp16_gemv(ctypes.c_void_p(0x10008), 64, 128, x, y, None) == -2
    assert L.pmpd_fp16_gemv(w, 64, 128, ctypes.c_void_p(0x30002), y, None) == -2
    assert L.pmpd_fp16_gemv(w, 64, 128, x, ctypes.c_void_p(0x40001), None) == -2
    arr = (binding._Fp16Layer * 2)(binding._Fp16Layer(70, 256, 0x10000), binding._Fp16Layer(32, 128, 0x20000))
    need = ctypes.c_size_t()
    assert L.pmpd_fp16_stack_workspace_size(arr, 2, ctypes.byref(need)) == 0
    assert need.value == 256 + 256  # 2 descriptors of 32 bytes, 3 + 1 items of 8 bytes, each table padded to 256
    assert L.pmpd_fp16_stack_workspace_size(arr, 0, ctypes.byref(need)) == -1
    assert L.pmpd_fp16_stack_workspace_size(None, 2, ctypes.byref(need)) == -1
    bad = (binding._Fp16Layer * 1)(binding._Fp16Layer(70, 256, 0x10004))
    assert L.pmpd_fp16_stack_workspace_size(bad, 1, ctypes.byref(need)) == -2
    xo, yo = (ctypes.c_int64 * 2)(0, 256), (ctypes.c_int64 * 2)(0, 70)
    h = ctypes.c_void_p()
    assert L.pmpd_fp16_stack_create(arr, 2, xo, yo, None, 4096, ctypes.byref(h)) == -1
    assert L.pmpd_fp16_stack_create(arr, 2, xo, yo, ctypes.c_void_p(0x50010), 4096, ctypes.byref(h)) == -2
    assert L.pmpd_fp16_stack_create(arr, 2, (ctypes.c_int64 * 2)(0, 100), yo, ctypes.c_void_p(0x50000), 4096, ctypes.byref(h)) == -2
    assert L.pmpd_fp16_stack_create(arr, 2, xo, yo, ctypes.c_void_p(0x50000), 16, ctypes.byref(h)) == -5
    assert L.pmpd_fp16_step(None, x, y, None) == -1
    assert L.pmpd_fp16_step(ctypes.c_void_p(0x1234), ctypes.c_void_p(0x30008), y, None) == -2


def test_learned_scheduler_argument_validation_needs_no_gpu():
    L = binding._load()

    def net(d_k=64, d_v=128, hidden=16, n=5, q=0x1000, w1=0x2000, b1=0x3000, w2=0x4000, b2=0x5000):
        return binding._Learned(d_k, d_v, hidden, n, q, w1, b1, w2, b2)

    need = ctypes.c_size_t()
    assert L.pmpd_learned_workspace_size(ctypes.byref(net()), 100, ctypes.byref(need)) == 0
    # scores 100 floats -> 512, partial 13 chunks x 128 floats = 6656, O 512, hidden 256
    assert need.value == 512 + 6656 + 512 + 256
    for bad in (net(d_k=60), net(d_k=0), net(d_k=16392), net(d_v=12), net(hidden=0), net(n=1), net(n=1025)):
        assert L.pmpd_learned_workspace_size(ctypes.byref(bad), 100, ctypes.byref(need)) == -1
    assert L.pmpd_learned_workspace_size(ctypes.byref(net()), 0, ctypes.byref(need)) == -1
    assert L.pmpd_learned_workspace_size(None, 10, ctypes.byref(need)) == -1
    K, V, ws = ctypes.c_void_p(0x10000), ctypes.c_void_p(0x20000), ctypes.c_void_p(0x30000)
    pr, cl = ctypes.c_void_p(0x40000), ctypes.c_void_p(0x50000)

    def fwd(n=None, k=K, v=V, w=ws, wb=1 << 20, p=pr, c=cl):
        return L.pmpd_learned_forward(ctypes.byref(n or net()), k, v, 100, w, wb, None, p, c, None)

    assert fwd(net(q=None)) == -1
    assert fwd(net(w1=0x2004)) == -2
    assert fwd(k=None) == -1
    assert fwd(v=ctypes.c_void_p(0x20008)) == -2
    assert fwd(w=ctypes.c_void_p(0x30010)) == -2
    assert fwd(wb=1000) == -5
    assert fwd(p=None) == -1
    assert fwd(c=ctypes.c_void_p(0x50002)) == -2
    h = ctypes.c_void_p()
    assert L.pmpd_schedule_from_class(3, 2, 5, 64, 5, ctypes.byref(h)) == -1   # class outside 0..4
    assert L.pmpd_schedule_from_class(3, 2, -1, 64, 5, ctypes.byref(h)) == -1
    assert L.pmpd_schedule_from_class(2, 3, 1, 64, 5, ctypes.byref(h)) == -1   # precisions must decrease
    assert L.pmpd_schedule_from_class(3, 2, 1, 64, 5, None) == -1
    for cls, point in enumerate((0, 16, 32, 48, 64)):
        assert L.pmpd_schedule_from_class(4, 2, cls, 64, 5, ctypes.byref(h)) == 0
        b = ctypes.c_int32()
        got = []
        for k in range(64):
            assert L.pmpd_schedule_bits(h, k, ctypes.byref(b)) == 0
            got.append(b.value)
        assert got == [4] * point + [2] * (64 - point)
        L.pmpd_schedule_destroy(h)


def test_bench_refuses_more_than_one_gpu():
    """bench.py runs on one GPU only: any other --gpus ends with a message and a non-zero status, before
    anything touches a GPU."""
    import subprocess
    import sys

    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""
