"""ctypes binding of libpmpd.so (names follow include/pmpd.h)."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

GROUP = 128
ROW_TILE = 64
MAX_BATCH = 8

EXPORTS = (
    "pmpd_strerror", "pmpd_last_error", "pmpd_packed_size", "pmpd_pack", "pmpd_unpack", "pmpd_gemv", "pmpd_gemm",
    "pmpd_stack_workspace_size", "pmpd_stack_create", "pmpd_stack_destroy", "pmpd_decode_step",
    "pmpd_stack_variant", "pmpd_stack_set_variant",
    "pmpd_schedule_create", "pmpd_schedule_destroy", "pmpd_schedule_bits", "pmpd_schedule_avg_bits",
    "pmpd_decode_run", "pmpd_prefill_step", "pmpd_batch_step",
    "pmpd_schedule_grid", "pmpd_schedule_count", "pmpd_schedule_search", "pmpd_read_stream",
    "pmpd_ordered_workspace_size", "pmpd_ordered_create", "pmpd_ordered_destroy", "pmpd_ordered_step",
    "pmpd_ordered_status", "pmpd_ordered_set_spin_limit",
    "pmpd_fp16_gemv", "pmpd_fp16_stack_workspace_size", "pmpd_fp16_stack_create", "pmpd_fp16_stack_destroy",
    "pmpd_fp16_step", "pmpd_learned_workspace_size", "pmpd_learned_forward", "pmpd_schedule_from_class",
    "pmpd_learned_forward_static",
)

QUALITY_FN = ctypes.CFUNCTYPE(ctypes.c_double, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32),
                              ctypes.c_int32, ctypes.c_void_p)


class PMPDError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"pmpd status {status}: {message}")
        self.status = status


class _Layer(ctypes.Structure):
    _fields_ = [
        ("out_features", ctypes.c_int32),
        ("in_features", ctypes.c_int32),
        ("group_size", ctypes.c_int32),
        ("reserved", ctypes.c_int32),
        ("planes", ctypes.c_void_p * 4),
        ("scale_min", ctypes.c_void_p),
    ]


class _Chain(ctypes.Structure):
    _fields_ = [("stage", ctypes.c_int32), ("source", ctypes.c_int32), ("gain", ctypes.c_float)]


class _Fp16Layer(ctypes.Structure):
    _fields_ = [("out_features", ctypes.c_int32), ("in_features", ctypes.c_int32), ("weight", ctypes.c_void_p)]


class _Learned(ctypes.Structure):
    _fields_ = [("d_k", ctypes.c_int32), ("d_v", ctypes.c_int32), ("hidden", ctypes.c_int32),
                ("n_classes", ctypes.c_int32), ("query", ctypes.c_void_p), ("w1", ctypes.c_void_p),
                ("b1", ctypes.c_void_p), ("w2", ctypes.c_void_p), ("b2", ctypes.c_void_p)]


_lib = None


def lib_path() -> str:
    return _build.LIB


def _load():
    """Load the in-tree library; build it only if it is absent.  No fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    L = ctypes.CDLL(_build.LIB)
    i32, i64, vp, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    P = ctypes.POINTER
    L.pmpd_strerror.restype = ctypes.c_char_p
    L.pmpd_strerror.argtypes = [i32]
    L.pmpd_last_error.restype = ctypes.c_char_p
    L.pmpd_last_error.argtypes = []
    L.pmpd_packed_size.restype = i32
    L.pmpd_packed_size.argtypes = [i32, i32, i32, P(sz), P(sz)]
    L.pmpd_pack.restype = i32
    L.pmpd_pack.argtypes = [vp, vp, vp, i32, i32, i32, P(vp), vp]
    L.pmpd_unpack.restype = i32
    L.pmpd_unpack.argtypes = [P(_Layer), i32, vp]
    L.pmpd_gemv.restype = i32
    L.pmpd_gemv.argtypes = [P(_Layer), i32, vp, vp, vp]
    L.pmpd_gemm.restype = i32
    L.pmpd_gemm.argtypes = [P(_Layer), i32, vp, i32, vp, vp]
    L.pmpd_stack_workspace_size.restype = i32
    L.pmpd_stack_workspace_size.argtypes = [P(_Layer), i32, P(sz)]
    L.pmpd_stack_create.restype = i32
    L.pmpd_stack_create.argtypes = [P(_Layer), i32, P(i64), P(i64), vp, sz, P(vp)]
    L.pmpd_stack_destroy.restype = None
    L.pmpd_stack_destroy.argtypes = [vp]
    L.pmpd_decode_step.restype = i32
    L.pmpd_decode_step.argtypes = [vp, i32, vp, vp, vp]
    L.pmpd_stack_variant.restype = i32
    L.pmpd_stack_variant.argtypes = [vp, i32, P(i32)]
    L.pmpd_stack_set_variant.restype = i32
    L.pmpd_stack_set_variant.argtypes = [vp, i32, i32]
    L.pmpd_schedule_create.restype = i32
    L.pmpd_schedule_create.argtypes = [P(i32), P(i32), i32, i32, P(vp)]
    L.pmpd_schedule_destroy.restype = None
    L.pmpd_schedule_destroy.argtypes = [vp]
    L.pmpd_schedule_bits.restype = i32
    L.pmpd_schedule_bits.argtypes = [vp, i32, P(i32)]
    L.pmpd_schedule_avg_bits.restype = ctypes.c_double
    L.pmpd_schedule_avg_bits.argtypes = [vp, i32]
    L.pmpd_prefill_step.restype = i32
    L.pmpd_prefill_step.argtypes = [vp, i32, vp, i32, vp, vp]
    L.pmpd_batch_step.restype = i32
    L.pmpd_batch_step.argtypes = [vp, i32, vp, i32, vp, vp]
    L.pmpd_schedule_grid.restype = i32
    L.pmpd_schedule_grid.argtypes = [i32, i32, P(i32)]
    L.pmpd_schedule_count.restype = i64
    L.pmpd_schedule_count.argtypes = [i32, i32]
    L.pmpd_schedule_search.restype = i32
    L.pmpd_schedule_search.argtypes = [P(i32), i32, i32, i32, QUALITY_FN, vp, ctypes.c_double, ctypes.c_double, P(i32),
                                       P(ctypes.c_double), P(i64)]
    L.pmpd_ordered_workspace_size.restype = i32
    L.pmpd_ordered_workspace_size.argtypes = [vp, P(_Chain), P(sz)]
    L.pmpd_ordered_create.restype = i32
    L.pmpd_ordered_create.argtypes = [vp, P(_Chain), vp, sz, P(vp)]
    L.pmpd_ordered_destroy.restype = None
    L.pmpd_ordered_destroy.argtypes = [vp]
    L.pmpd_ordered_step.restype = i32
    L.pmpd_ordered_step.argtypes = [vp, i32, vp, vp, vp]
    L.pmpd_ordered_status.restype = i32
    L.pmpd_ordered_status.argtypes = [vp, P(i32)]
    L.pmpd_ordered_set_spin_limit.restype = i32
    L.pmpd_ordered_set_spin_limit.argtypes = [vp, ctypes.c_uint32]
    L.pmpd_read_stream.restype = i32
    L.pmpd_read_stream.argtypes = [vp, sz, vp, P(sz), vp]
    L.pmpd_fp16_gemv.restype = i32
    L.pmpd_fp16_gemv.argtypes = [vp, i32, i32, vp, vp, vp]
    L.pmpd_fp16_stack_workspace_size.restype = i32
    L.pmpd_fp16_stack_workspace_size.argtypes = [P(_Fp16Layer), i32, P(sz)]
    L.pmpd_fp16_stack_create.restype = i32
    L.pmpd_fp16_stack_create.argtypes = [P(_Fp16Layer), i32, P(i64), P(i64), vp, sz, P(vp)]
    L.pmpd_fp16_stack_destroy.restype = None
    L.pmpd_fp16_stack_destroy.argtypes = [vp]
    L.pmpd_fp16_step.restype = i32
    L.pmpd_fp16_step.argtypes = [vp, vp, vp, vp]
    L.pmpd_learned_workspace_size.restype = i32
    L.pmpd_learned_workspace_size.argtypes = [P(_Learned), i32, P(sz)]
    L.pmpd_learned_forward.restype = i32
    L.pmpd_learned_forward.argtypes = [P(_Learned), vp, vp, i32, vp, sz, vp, vp, vp, vp]
    L.pmpd_learned_forward_static.restype = i32
    L.pmpd_learned_forward_static.argtypes = [P(_Learned), vp, vp, i32, vp, vp, vp, vp]
    L.pmpd_schedule_from_class.restype = i32
    L.pmpd_schedule_from_class.argtypes = [i32, i32, i32, i32, i32, P(vp)]
    L.pmpd_decode_run.restype = i32
    L.pmpd_decode_run.argtypes = [vp, vp, i32, i32, vp, i64, vp, i64, vp]
    _lib = L
    return L


def exported_symbols() -> List[str]:
    """Names from include/pmpd.h that the loaded library really exports."""
    L = _load()
    return [n for n in EXPORTS if hasattr(L, n)]


def _check(status: int):
    if status != 0:
        raise PMPDError(status, _load().pmpd_last_error().decode())


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _stream_handle(stream) -> Optional[int]:
    if stream is None:
        import torch

        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# ------------------------------------------------------------------- packing ----
def packed_size(out_features: int, in_features: int, group_size: int = GROUP) -> Tuple[int, int]:
    pb, sb = ctypes.c_size_t(), ctypes.c_size_t()
    _check(_load().pmpd_packed_size(out_features, in_features, group_size, ctypes.byref(pb), ctypes.byref(sb)))
    return pb.value, sb.value


def pack(q4: np.ndarray, scale: np.ndarray, minv: np.ndarray, group_size: int = GROUP):
    """Host pack: (q4 uint8 [out,in], scale fp16 [out,in/128], minv fp16) -> (4 plane arrays, scale_min array)."""
    q4 = np.ascontiguousarray(q4, dtype=np.uint8)
    out_f, in_f = q4.shape
    s = np.ascontiguousarray(np.asarray(scale, dtype=np.float16)).view(np.uint16)
    a = np.ascontiguousarray(np.asarray(minv, dtype=np.float16)).view(np.uint16)
    pb, sb = packed_size(out_f, in_f, group_size)
    if s.shape != (out_f, in_f // group_size) or a.shape != s.shape:
        raise PMPDError(-1, "scale/minv must have shape [out, in/group]")
    planes = [np.empty(pb // 4, dtype=np.uint32) for _ in range(4)]
    sm = np.empty(sb // 4, dtype=np.uint32)
    arr = (ctypes.c_void_p * 4)(*[p.ctypes.data for p in planes])
    _check(_load().pmpd_pack(_np_ptr(q4), _np_ptr(s), _np_ptr(a), out_f, in_f, group_size, arr, _np_ptr(sm)))
    return planes, sm


def unpack(planes: Sequence[Optional[np.ndarray]], b: int, out_features: int, in_features: int) -> np.ndarray:
    """Host unpack of the top b planes; planes[b:] may be None."""
    lay = _Layer(out_features, in_features, GROUP, 0)
    keep = []
    for k in range(4):
        p = planes[k] if k < len(planes) else None
        if p is not None:
            p = np.ascontiguousarray(p, dtype=np.uint32)
            keep.append(p)
            lay.planes[k] = p.ctypes.data
        else:
            lay.planes[k] = None
    dummy = np.zeros(1, dtype=np.uint32)
    lay.scale_min = dummy.ctypes.data
    qb = np.empty((out_features, in_features), dtype=np.uint8)
    _check(_load().pmpd_unpack(ctypes.byref(lay), b, _np_ptr(qb)))
    return qb


# ------------------------------------------------------------- device layers ----
@dataclass
class PackedLayer:
    """A packed layer resident in device memory (tensors are owned here)."""

    out_features: int
    in_features: int
    planes: list  # 4 torch int32 tensors (entries may be None)
    scale_min: object  # torch int32 tensor
    _struct: _Layer = field(default=None, repr=False)

    def struct(self) -> _Layer:
        if self._struct is None:
            lay = _Layer(self.out_features, self.in_features, GROUP, 0)
            pb, sb = packed_size(self.out_features, self.in_features)
            for k in range(4):
                if self.planes[k] is not None:
                    lay.planes[k] = _dev_ptr(self.planes[k], "int32", pb // 4, f"planes[{k}]").value
                else:
                    lay.planes[k] = None
            lay.scale_min = _dev_ptr(self.scale_min, "int32", sb // 4, "scale_min").value
            self._struct = lay
        return self._struct

    def bytes_at(self, b: int) -> int:
        """Algorithmic bytes of a b-bit pass: b planes, the scale/min words, x once, y once."""
        pb, sb = packed_size(self.out_features, self.in_features)
        return b * pb + sb + 2 * self.in_features + 4 * self.out_features


def upload_layer(planes, scale_min, out_features: int, in_features: int, device="cuda") -> PackedLayer:
    import torch

    dp = [torch.from_numpy(p.view(np.int32)).to(device) if p is not None else None for p in planes]
    ds = torch.from_numpy(scale_min.view(np.int32)).to(device)
    return PackedLayer(out_features, in_features, dp, ds)


def _dev_ptr(t, dtype: str, min_elems: int, what: str):
    """Address of a torch tensor for the C ABI, after checking what the C side cannot see: the library
    gets a bare pointer, so a host tensor, another element type, a strided view or a buffer shorter than
    the call reads or writes would become a wild access inside a kernel.  dtype: "float16", "float32",
    "int32" or "any"; min_elems: elements the call touches."""
    import torch

    if not isinstance(t, torch.Tensor):
        raise PMPDError(-1, f"{what}: expected a torch tensor, got {type(t).__name__}")
    if not t.is_cuda:
        raise PMPDError(-1, f"{what}: tensor is on {t.device}, the kernels need device memory")
    if dtype != "any" and t.dtype != getattr(torch, dtype):
        raise PMPDError(-1, f"{what}: dtype {t.dtype}, expected torch.{dtype}")
    if not t.is_contiguous():
        raise PMPDError(-1, f"{what}: tensor is not contiguous")
    if t.numel() < min_elems:
        raise PMPDError(-5, f"{what}: {t.numel()} elements, the call needs {min_elems}")
    return ctypes.c_void_p(t.data_ptr())


def gemv(layer: PackedLayer, b: int, x, y=None, stream=None):
    """y = W_b x.  x: torch fp16 [in] on the GPU; returns torch fp32 [out]."""
    import torch

    xp = _dev_ptr(x, "float16", layer.in_features, "gemv x")
    if y is None:
        y = torch.empty(layer.out_features, dtype=torch.float32, device=x.device)
    yp = _dev_ptr(y, "float32", layer.out_features, "gemv y")
    _check(_load().pmpd_gemv(ctypes.byref(layer.struct()), b, xp, yp, _stream_handle(stream)))
    return y


def gemm(layer: PackedLayer, b: int, X, Y=None, stream=None):
    """Y = X W_b^T.  X: torch fp16 [m, in]; returns torch fp32 [m, out] (m <= 8: the memory-bound kernel; 9..16: fp16 matrix cores, codes as subnormals; above: the prefill kernel)."""
    import torch

    if X.dim() != 2 or X.shape[1] != layer.in_features:
        raise PMPDError(-1, f"gemm X: shape {tuple(X.shape)}, expected [m, {layer.in_features}]")
    m = X.shape[0]
    Xp = _dev_ptr(X, "float16", m * layer.in_features, "gemm X")
    if Y is None:
        Y = torch.empty((m, layer.out_features), dtype=torch.float32, device=X.device)
    Yp = _dev_ptr(Y, "float32", m * layer.out_features, "gemm Y")
    _check(_load().pmpd_gemm(ctypes.byref(layer.struct()), b, Xp, m, Yp, _stream_handle(stream)))
    return Y


class Stack:
    """A list of device layers prepared for one-launch decode steps."""

    def __init__(self, layers: Sequence[PackedLayer], x_offsets: Optional[Sequence[int]] = None,
                 y_offsets: Optional[Sequence[int]] = None, device="cuda"):
        import torch

        self.layers = list(layers)
        n = len(self.layers)
        if x_offsets is None:
            x_offsets, acc = [], 0
            for l in self.layers:
                x_offsets.append(acc)
                acc += l.in_features
        if y_offsets is None:
            y_offsets, acc = [], 0
            for l in self.layers:
                y_offsets.append(acc)
                acc += l.out_features
        self.x_offsets, self.y_offsets = list(x_offsets), list(y_offsets)
        self.x_elems = max(o + l.in_features for o, l in zip(self.x_offsets, self.layers)) if n else 0
        self.y_elems = max(o + l.out_features for o, l in zip(self.y_offsets, self.layers)) if n else 0
        arr = (_Layer * max(n, 1))(*[l.struct() for l in self.layers])
        need = ctypes.c_size_t()
        L = _load()
        _check(L.pmpd_stack_workspace_size(arr, n, ctypes.byref(need)))
        self.workspace = torch.empty(need.value + 256, dtype=torch.uint8, device=device)
        base = self.workspace.data_ptr()
        aligned = (base + 255) // 256 * 256
        xo = (ctypes.c_int64 * n)(*self.x_offsets)
        yo = (ctypes.c_int64 * n)(*self.y_offsets)
        h = ctypes.c_void_p()
        _check(L.pmpd_stack_create(arr, n, xo, yo, ctypes.c_void_p(aligned), need.value, ctypes.byref(h)))
        self._h = h

    def bytes_at(self, b: int) -> int:
        return sum(l.bytes_at(b) for l in self.layers)

    def variant(self, b: int) -> int:
        """Launch shape (0..4, see include/pmpd.h) that decode_step uses on this stack at bit-width b."""
        v = ctypes.c_int32()
        _check(_load().pmpd_stack_variant(self._h, b, ctypes.byref(v)))
        return v.value

    def set_variant(self, b: int, variant: int):
        _check(_load().pmpd_stack_set_variant(self._h, b, variant))

    def close(self):
        if getattr(self, "_h", None):
            _load().pmpd_stack_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def decode_step(stack: Stack, b: int, x, y, stream=None):
    """One decode step over the stack at bit-width b.  x: fp16 [x_elems], y: fp32 [y_elems]."""
    xp = _dev_ptr(x, "float16", stack.x_elems, "decode_step x")
    yp = _dev_ptr(y, "float32", stack.y_elems, "decode_step y")
    _check(_load().pmpd_decode_step(stack._h, b, xp, yp, _stream_handle(stream)))
    return y


def batch_step(stack: Stack, b: int, X, m: int, Y, stream=None):
    """m tokens through every layer: layer l reads X[m*x_off[l]:][m, in_l] and writes Y[m*y_off[l]:][m, out_l]."""
    m = int(m)
    Xp = _dev_ptr(X, "float16", max(m, 1) * stack.x_elems, "batch_step X")
    Yp = _dev_ptr(Y, "float32", max(m, 1) * stack.y_elems, "batch_step Y")
    _check(_load().pmpd_batch_step(stack._h, b, Xp, m, Yp, _stream_handle(stream)))
    return Y


def prefill_step(stack: Stack, b: int, X, m: int, Y, stream=None):
    """Prefill over the stack: layer l reads X[m*x_off[l]:][m, in_l] and writes Y[m*y_off[l]:][m, out_l]."""
    m = int(m)
    Xp = _dev_ptr(X, "float16", max(m, 1) * stack.x_elems, "prefill_step X")
    Yp = _dev_ptr(Y, "float32", max(m, 1) * stack.y_elems, "prefill_step Y")
    _check(_load().pmpd_prefill_step(stack._h, b, Xp, m, Yp, _stream_handle(stream)))
    return Y


class Schedule:
    """Precision-switching schedule <P, S>."""

    def __init__(self, precisions: Sequence[int], st: Sequence[int], max_steps: int):
        n = len(precisions)
        if len(st) != n:
            raise PMPDError(-1, "precisions and st must have the same length")
        p = (ctypes.c_int32 * max(n, 1))(*precisions)
        s = (ctypes.c_int32 * max(n, 1))(*st)
        h = ctypes.c_void_p()
        _check(_load().pmpd_schedule_create(p, s, n, max_steps, ctypes.byref(h)))
        self._h = h
        self.max_steps = max_steps

    def bits(self, step: int) -> int:
        b = ctypes.c_int32()
        _check(_load().pmpd_schedule_bits(self._h, step, ctypes.byref(b)))
        return b.value

    def avg_bits(self, n_steps: int) -> float:
        v = _load().pmpd_schedule_avg_bits(self._h, n_steps)
        if v < 0:
            raise PMPDError(-1, _load().pmpd_last_error().decode())
        return v

    def close(self):
        if getattr(self, "_h", None):
            _load().pmpd_schedule_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Ordered:
    """A stack whose layers run in dependency order inside one cooperative launch per step.

    stages[l], sources[l] (-1 = external input), gains[l] per layer of the stack."""

    def __init__(self, stack: Stack, stages: Sequence[int], sources: Sequence[int], gains: Sequence[float],
                 device="cuda"):
        import torch

        n = len(stack.layers)
        if not (len(stages) == len(sources) == len(gains) == n):
            raise PMPDError(-1, "stages, sources and gains need one entry per layer")
        self.stack = stack  # keeps the stack alive
        chain = (_Chain * max(n, 1))(*[_Chain(int(s), int(k), float(g)) for s, k, g in zip(stages, sources, gains)])
        L = _load()
        need = ctypes.c_size_t()
        _check(L.pmpd_ordered_workspace_size(stack._h, chain, ctypes.byref(need)))
        self.workspace = torch.empty(need.value + 256, dtype=torch.uint8, device=device)
        aligned = (self.workspace.data_ptr() + 255) // 256 * 256
        h = ctypes.c_void_p()
        _check(L.pmpd_ordered_create(stack._h, chain, ctypes.c_void_p(aligned), need.value, ctypes.byref(h)))
        self._h = h

    def step(self, b: int, x, y, stream=None):
        xp = _dev_ptr(x, "float16", self.stack.x_elems, "ordered step x")
        yp = _dev_ptr(y, "float32", self.stack.y_elems, "ordered step y")
        _check(_load().pmpd_ordered_step(self._h, b, xp, yp, _stream_handle(stream)))
        return y

    def timed_out(self) -> bool:
        """Synchronous: did a wait between stages run out since the last call?"""
        flag = ctypes.c_int32()
        _check(_load().pmpd_ordered_status(self._h, ctypes.byref(flag)))
        return bool(flag.value)

    def set_spin_limit(self, polls: int):
        _check(_load().pmpd_ordered_set_spin_limit(self._h, polls))

    def close(self):
        if getattr(self, "_h", None):
            _load().pmpd_ordered_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ----------------------------------------------------- learned scheduler ----
class LearnedScheduler:
    """Parameters of the learned scheduler resident on the device (fp32 tensors owned here)."""

    def __init__(self, query, w1, b1, w2, b2, device="cuda"):
        import torch

        def dev(a):
            return torch.as_tensor(np.ascontiguousarray(a, dtype=np.float32)).to(device).contiguous()

        self.query, self.w1, self.b1, self.w2, self.b2 = dev(query), dev(w1), dev(b1), dev(w2), dev(b2)
        self.hidden, self.d_v = self.w1.shape
        self.n_classes = self.w2.shape[0]
        self.d_k = self.query.shape[0]
        if self.w2.shape[1] != self.hidden or self.b1.shape[0] != self.hidden or self.b2.shape[0] != self.n_classes:
            raise PMPDError(-1, "learned scheduler: parameter shapes do not fit together")
        self._struct = _Learned(self.d_k, self.d_v, self.hidden, self.n_classes, self.query.data_ptr(),
                                self.w1.data_ptr(), self.b1.data_ptr(), self.w2.data_ptr(), self.b2.data_ptr())
        self._ws = None

    def workspace_size(self, T: int) -> int:
        need = ctypes.c_size_t()
        _check(_load().pmpd_learned_workspace_size(ctypes.byref(self._struct), T, ctypes.byref(need)))
        return need.value

    def forward_static(self, K, V, probs, cls, context, stream=None):
        """forward() through the entry point that allocates nothing: the work area is the library's own
        device array, and the outputs must be passed in (this wrapper creates no tensor either)."""
        if K.dim() != 2 or V.dim() != 2:
            raise PMPDError(-1, "learned scheduler: K and V must be [T, d] matrices")
        T = int(K.shape[0])
        if K.shape[1] != self.d_k or V.shape[0] != T or V.shape[1] != self.d_v:
            raise PMPDError(-1, "learned scheduler: K / V shapes do not fit the parameters")
        _check(_load().pmpd_learned_forward_static(
            ctypes.byref(self._struct), _dev_ptr(K, "float16", T * self.d_k, "learned scheduler K"),
            _dev_ptr(V, "float16", T * self.d_v, "learned scheduler V"), T,
            _dev_ptr(context, "float32", self.d_v, "learned scheduler context"),
            _dev_ptr(probs, "float32", self.n_classes, "learned scheduler probs"),
            _dev_ptr(cls, "int32", 1, "learned scheduler cls"), _stream_handle(stream)))
        return probs, cls, context

    def forward(self, K, V, probs=None, cls=None, context=None, stream=None):
        """K [T, d_k], V [T, d_v]: fp16 device tensors.  Returns (probs, cls, context) device tensors; asynchronous."""
        import torch

        if K.dim() != 2 or V.dim() != 2:
            raise PMPDError(-1, "learned scheduler: K and V must be [T, d] matrices")
        T = int(K.shape[0])
        if K.shape[1] != self.d_k or V.shape[0] != T or V.shape[1] != self.d_v:
            raise PMPDError(-1, "learned scheduler: K / V shapes do not fit the parameters")
        Kp = _dev_ptr(K, "float16", T * self.d_k, "learned scheduler K")
        Vp = _dev_ptr(V, "float16", T * self.d_v, "learned scheduler V")
        need = self.workspace_size(T)
        if self._ws is None or self._ws.numel() < need + 256:
            self._ws = torch.empty(need + 256, dtype=torch.uint8, device=K.device)
        base = (self._ws.data_ptr() + 255) // 256 * 256
        if probs is None:
            probs = torch.empty(self.n_classes, dtype=torch.float32, device=K.device)
        if cls is None:
            cls = torch.empty(1, dtype=torch.int32, device=K.device)
        if context is None:
            context = torch.empty(self.d_v, dtype=torch.float32, device=K.device)
        _check(_load().pmpd_learned_forward(ctypes.byref(self._struct), Kp, Vp, T, base, need,
                                            _dev_ptr(context, "float32", self.d_v, "learned scheduler context"),
                                            _dev_ptr(probs, "float32", self.n_classes, "learned scheduler probs"),
                                            _dev_ptr(cls, "int32", 1, "learned scheduler cls"), _stream_handle(stream)))
        return probs, cls, context


def schedule_from_class(high: int, low: int, cls: int, max_steps: int, n_points: int) -> "Schedule":
    """The two-precision schedule that switches at candidate point `cls` of the n_points grid."""
    h = ctypes.c_void_p()
    _check(_load().pmpd_schedule_from_class(high, low, cls, max_steps, n_points, ctypes.byref(h)))
    sch = Schedule.__new__(Schedule)
    sch._h = h
    sch.max_steps = max_steps
    return sch


# ------------------------------------------------------- fp16 reference ----
def fp16_gemv(W, x, y=None, stream=None):
    """y = W x for an unquantised fp16 device matrix W [out, in] (the paper's fp16 baseline kernel)."""
    import torch

    if W.dim() != 2:
        raise PMPDError(-1, "fp16_gemv W: expected an [out, in] matrix")
    out_f, in_f = W.shape
    Wp = _dev_ptr(W, "float16", out_f * in_f, "fp16_gemv W")
    xp = _dev_ptr(x, "float16", in_f, "fp16_gemv x")
    if y is None:
        y = torch.empty(out_f, dtype=torch.float32, device=W.device)
    yp = _dev_ptr(y, "float32", out_f, "fp16_gemv y")
    _check(_load().pmpd_fp16_gemv(Wp, out_f, in_f, xp, yp, _stream_handle(stream)))
    return y


class Fp16Stack:
    """A list of fp16 device matrices prepared for one-launch steps (tables live in a tensor owned here)."""

    def __init__(self, weights, x_offsets: Optional[Sequence[int]] = None, y_offsets: Optional[Sequence[int]] = None):
        import torch

        self.weights = list(weights)
        n = len(self.weights)
        for w in self.weights:
            if w.dim() != 2:
                raise PMPDError(-1, "Fp16Stack: every weight must be an [out, in] matrix")
        arr = (_Fp16Layer * n)(*[_Fp16Layer(int(w.shape[0]), int(w.shape[1]),
                                            _dev_ptr(w, "float16", int(w.shape[0]) * int(w.shape[1]), "Fp16Stack weight"))
                                 for w in self.weights])
        if x_offsets is None or y_offsets is None:
            x_offsets, y_offsets, xo, yo = [], [], 0, 0
            for w in self.weights:
                x_offsets.append(xo)
                y_offsets.append(yo)
                xo += int(w.shape[1])
                yo += int(w.shape[0])
        self.x_offsets, self.y_offsets = list(x_offsets), list(y_offsets)
        self.x_elems = max(o + int(w.shape[1]) for o, w in zip(self.x_offsets, self.weights))
        self.y_elems = max(o + int(w.shape[0]) for o, w in zip(self.y_offsets, self.weights))
        need = ctypes.c_size_t()
        _check(_load().pmpd_fp16_stack_workspace_size(arr, n, ctypes.byref(need)))
        self.workspace = torch.empty(need.value + 256, dtype=torch.uint8, device=self.weights[0].device)
        base = (self.workspace.data_ptr() + 255) // 256 * 256
        xo = (ctypes.c_int64 * n)(*self.x_offsets)
        yo = (ctypes.c_int64 * n)(*self.y_offsets)
        h = ctypes.c_void_p()
        _check(_load().pmpd_fp16_stack_create(arr, n, xo, yo, base, need.value, ctypes.byref(h)))
        self.handle = h

    def weight_bytes(self) -> int:
        return sum(2 * int(w.shape[0]) * int(w.shape[1]) for w in self.weights)

    def close(self):
        if getattr(self, "handle", None):
            _load().pmpd_fp16_stack_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def fp16_step(stack: Fp16Stack, x, y, stream=None):
    xp = _dev_ptr(x, "float16", stack.x_elems, "fp16_step x")
    yp = _dev_ptr(y, "float32", stack.y_elems, "fp16_step y")
    _check(_load().pmpd_fp16_step(stack.handle, xp, yp, _stream_handle(stream)))
    return y


def read_stream(buf, sink, stream=None) -> int:
    """Launch the read-only stream kernel over the torch tensor buf; returns the bytes it reads."""
    n = ctypes.c_size_t()
    bp = _dev_ptr(buf, "any", 1, "read_stream buf")
    sp = _dev_ptr(sink, "int32", 1, "read_stream sink")
    _check(_load().pmpd_read_stream(bp, buf.numel() * buf.element_size(), sp, ctypes.byref(n), _stream_handle(stream)))
    return n.value


def schedule_grid(max_steps: int, n_points: int) -> List[int]:
    """Candidate switch points 0, OL/(N-1), ..., OL."""
    pts = (ctypes.c_int32 * max(n_points, 1))()
    _check(_load().pmpd_schedule_grid(max_steps, n_points, pts))
    return list(pts)


def schedule_count(max_steps: int, n_precisions: int) -> int:
    v = _load().pmpd_schedule_count(max_steps, n_precisions)
    if v < 0:
        raise PMPDError(-1, _load().pmpd_last_error().decode())
    return v


def schedule_search(precisions: Sequence[int], max_steps: int, n_points: int, quality, q_ref: float, eps: float):
    """Static-scheduler search; quality(precisions, st) -> float is called on the host.
    Returns (st, avg_bits, number of quality evaluations)."""
    n = len(precisions)

    def _cb(p_ptr, st_ptr, nn, _user):
        return float(quality([p_ptr[i] for i in range(nn)], [st_ptr[i] for i in range(nn)]))

    cb = QUALITY_FN(_cb)
    p = (ctypes.c_int32 * max(n, 1))(*precisions)
    st = (ctypes.c_int32 * max(n, 1))()
    avg = ctypes.c_double()
    cnt = ctypes.c_int64()
    _check(_load().pmpd_schedule_search(p, n, max_steps, n_points, cb, None, q_ref, eps, st, ctypes.byref(avg),
                                        ctypes.byref(cnt)))
    return list(st), avg.value, cnt.value


def decode_run(stack: Stack, schedule: Schedule, step0: int, n_steps: int, x, x_step_stride: int, y,
               y_step_stride: int, stream=None):
    """Steps step0..step0+n_steps-1, each at the schedule's bit-width."""
    last = max(int(n_steps) - 1, 0)
    xp = _dev_ptr(x, "float16", last * int(x_step_stride) + stack.x_elems, "decode_run x")
    yp = _dev_ptr(y, "float32", last * int(y_step_stride) + stack.y_elems, "decode_run y")
    _check(_load().pmpd_decode_run(stack._h, schedule._h, step0, n_steps, xp, x_step_stride, yp, y_step_stride,
                                   _stream_handle(stream)))
    return y
