"""CPU oracle for the PMPD decode linear-layer path (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It is a thin ctypes wrapper over ``pmpd_oracle.c`` (plain C, fp64,
plain loops) plus a few closed-form accounting helpers.  It shares no code with
the HIP library and never imports it.

Definitions followed (paper: Section 2.1 and Section 5 "PMPD Implementation
Details" for the nested weight store; Algorithm 1 for the per-step linear
layers; Section 4.2 with Eq. 1-3 for the schedule; Section 5 "Baselines" for
the average bit-width; Table 3 caption and Appendix A.5 for the
schedule-weighted latency):

    q_b = q4 >> (4 - b)
    W_b = a_g + s_g * 2^(4-b) * (q_b + 0.5)          (group g = i // 128)
    y   = W_b @ x                                    (fp64)
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from math import comb
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pmpd_oracle.c")
_LIB = os.path.join(_HERE, "libpmpd_oracle.so")

GROUP = 128
TILE = 64


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU code involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i64, i32 = ctypes.c_int64, ctypes.c_int32
        vp = ctypes.c_void_p
        L.orc_plane_words.restype = i64
        L.orc_plane_words.argtypes = [i64, i64]
        L.orc_sa_words.restype = i64
        L.orc_sa_words.argtypes = [i64, i64]
        L.orc_pack.restype = ctypes.c_int
        L.orc_pack.argtypes = [vp, vp, vp, i64, i64, vp, vp, vp, vp, vp]
        L.orc_unpack.restype = ctypes.c_int
        L.orc_unpack.argtypes = [vp, vp, vp, vp, ctypes.c_int, i64, i64, vp]
        L.orc_unpack_sa.restype = None
        L.orc_unpack_sa.argtypes = [vp, i64, i64, vp, vp]
        L.orc_dequant.restype = ctypes.c_int
        L.orc_dequant.argtypes = [vp, vp, vp, ctypes.c_int, i64, i64, vp]
        L.orc_linear_logical.restype = ctypes.c_int
        L.orc_linear_logical.argtypes = [vp, vp, vp, ctypes.c_int, i64, i64, vp, i64, vp, vp]
        L.orc_linear_packed.restype = ctypes.c_int
        L.orc_linear_packed.argtypes = [vp, vp, vp, vp, vp, ctypes.c_int, i64, i64, i64, i64, vp, i64, vp, vp]
        L.orc_threads.restype = ctypes.c_int
        L.orc_fp16_value.restype = ctypes.c_double
        L.orc_fp16_value.argtypes = [ctypes.c_uint16]
        L.orc_schedule_valid.restype = ctypes.c_int
        L.orc_schedule_valid.argtypes = [vp, vp, i32, i32]
        L.orc_schedule_bits.restype = ctypes.c_int
        L.orc_schedule_bits.argtypes = [vp, vp, i32, i32]
        L.orc_schedule_avg_bits.restype = ctypes.c_double
        L.orc_schedule_avg_bits.argtypes = [vp, vp, i32, i32]
        _lib = L
    return _lib


def _p(arr: Optional[np.ndarray]):
    return None if arr is None else arr.ctypes.data_as(ctypes.c_void_p)


def _c(arr, dtype) -> np.ndarray:
    return np.ascontiguousarray(arr, dtype=dtype)


def _bits16(arr) -> np.ndarray:
    """fp16 array -> its uint16 bit patterns (contiguous)."""
    return np.ascontiguousarray(np.asarray(arr, dtype=np.float16)).view(np.uint16)


def threads() -> int:
    return int(_load().orc_threads())


def fp16_value(bits: int) -> float:
    return float(_load().orc_fp16_value(int(bits) & 0xFFFF))


def padded_rows(out_f: int) -> int:
    return (out_f + TILE - 1) // TILE * TILE


def pack(q4, s, a) -> Tuple[Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray], np.ndarray]:
    """4-bit codes + fp16 scale/min -> (4 planes of uint32 words, scale/min words)."""
    L = _load()
    q4 = _c(q4, np.uint8)
    out_f, in_f = q4.shape
    sb, ab = _bits16(s), _bits16(a)
    pw = L.orc_plane_words(out_f, in_f)
    planes = tuple(np.empty(pw, dtype=np.uint32) for _ in range(4))
    sa = np.empty(L.orc_sa_words(out_f, in_f), dtype=np.uint32)
    rc = L.orc_pack(_p(q4), _p(sb), _p(ab), out_f, in_f, *[_p(p) for p in planes], _p(sa))
    if rc:
        raise ValueError(f"orc_pack failed ({rc})")
    return planes, sa


def unpack(planes: Sequence[Optional[np.ndarray]], b: int, out_f: int, in_f: int) -> np.ndarray:
    """b-bit codes from planes[0..b-1]; planes[b..3] are never touched (may be None)."""
    L = _load()
    ps = [(_c(p, np.uint32) if (p is not None and k < b) else None) for k, p in enumerate(planes)]
    while len(ps) < 4:
        ps.append(None)
    qb = np.empty((out_f, in_f), dtype=np.uint8)
    rc = L.orc_unpack(*[_p(p) for p in ps], b, out_f, in_f, _p(qb))
    if rc:
        raise ValueError(f"orc_unpack failed ({rc})")
    return qb


def unpack_sa(sa, out_f: int, in_f: int):
    L = _load()
    sa = _c(sa, np.uint32)
    G = in_f // GROUP
    s = np.empty((out_f, G), dtype=np.uint16)
    a = np.empty((out_f, G), dtype=np.uint16)
    L.orc_unpack_sa(_p(sa), out_f, in_f, _p(s), _p(a))
    return s.view(np.float16), a.view(np.float16)


def dequant(q4, s, a, b: int) -> np.ndarray:
    """Dense fp64 W_b from the logical inputs."""
    L = _load()
    q4 = _c(q4, np.uint8)
    out_f, in_f = q4.shape
    W = np.empty((out_f, in_f), dtype=np.float64)
    rc = L.orc_dequant(_p(q4), _p(_bits16(s)), _p(_bits16(a)), b, out_f, in_f, _p(W))
    if rc:
        raise ValueError(f"orc_dequant failed ({rc})")
    return W


def linear(q4, s, a, b: int, x, want_budget: bool = True):
    """Y[j][r] = sum_i W_b[r][i] X[j][i] in fp64, plus T[j][r] = sum |W_b||X|.

    x: fp16, shape (in,) or (m, in).  Returns arrays of shape (m, out).
    """
    L = _load()
    q4 = _c(q4, np.uint8)
    out_f, in_f = q4.shape
    xb = _bits16(x).reshape(-1, in_f)
    m = xb.shape[0]
    y = np.empty((m, out_f), dtype=np.float64)
    t = np.empty((m, out_f), dtype=np.float64) if want_budget else None
    rc = L.orc_linear_logical(_p(q4), _p(_bits16(s)), _p(_bits16(a)), b, out_f, in_f, _p(xb), m, _p(y), _p(t))
    if rc:
        raise ValueError(f"orc_linear_logical failed ({rc})")
    return y, t


def linear_dense(q4, s, a, b: int, x):
    """linear() with a library matmul as the summation step, for whole layers at hundreds of tokens (the
    plain loops of linear() take minutes there): the dense fp64 matrix W_b of dequant() (every entry exact),
    then Y = X W_b^T and T = |X| |W_b|^T by numpy's fp64 matmul.  Same definition; only the order of the fp64
    additions differs (relative 1e-13).  Returns (Y [m, out], T [m, out])."""
    W = dequant(q4, s, a, b)
    X = np.asarray(x, dtype=np.float16).astype(np.float64).reshape(-1, W.shape[1])
    return X @ W.T, np.abs(X) @ np.abs(W).T


def linear_packed(planes, sa, b: int, out_f: int, in_f: int, x, row0: int = 0,
                  nrows: Optional[int] = None, want_budget: bool = True):
    """Same as linear() but from the packed store, reading planes[0..b-1] only."""
    L = _load()
    nrows = out_f - row0 if nrows is None else nrows
    ps = [(_c(p, np.uint32) if (p is not None and k < b) else None) for k, p in enumerate(planes)]
    while len(ps) < 4:
        ps.append(None)
    sa = _c(sa, np.uint32)
    xb = _bits16(x).reshape(-1, in_f)
    m = xb.shape[0]
    y = np.empty((m, nrows), dtype=np.float64)
    t = np.empty((m, nrows), dtype=np.float64) if want_budget else None
    rc = L.orc_linear_packed(*[_p(p) for p in ps], _p(sa), b, out_f, in_f, row0, nrows, _p(xb), m, _p(y), _p(t))
    if rc:
        raise ValueError(f"orc_linear_packed failed ({rc})")
    return y, t


def linear_fp16(W, x):
    """The fp16 baseline the paper measures its speedups against (Section 5.2, Table 3): y = W x for
    unquantised fp16 W [out, in] and fp16 x [in] or [m, in], every product and sum in fp64.
    Returns (Y [m, out], T [m, out] = sum |W||x|)."""
    W64 = np.asarray(W, dtype=np.float16).astype(np.float64)
    X64 = np.asarray(x, dtype=np.float16).astype(np.float64).reshape(-1, W64.shape[1])
    return X64 @ W64.T, np.abs(X64) @ np.abs(W64).T


# ---------------------------------------------------------------- schedule ----
def _i32(seq) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(seq, dtype=np.int32))


def schedule_valid(precisions, st, OL: int) -> bool:
    p, s = _i32(precisions), _i32(st)
    if len(p) != len(s):
        return False
    return bool(_load().orc_schedule_valid(_p(p), _p(s), len(p), OL))


def schedule_bits(precisions, st, step: int) -> int:
    p, s = _i32(precisions), _i32(st)
    return int(_load().orc_schedule_bits(_p(p), _p(s), len(p), step))


def schedule_avg_bits(precisions, st, n_steps: int) -> float:
    p, s = _i32(precisions), _i32(st)
    return float(_load().orc_schedule_avg_bits(_p(p), _p(s), len(p), n_steps))


def progressive_schedule_count(OL: int, n_precisions: int) -> int:
    """Number of progressive schedules (Section 4.3): sum over the number of
    switches r of C(OL, r) * C(|P| - 1, r)."""
    return sum(comb(OL, r) * comb(n_precisions - 1, r) for r in range(n_precisions))


def schedule_weighted_latency(lat_high: float, lat_low: float, frac_high: float) -> float:
    """Latency of a two-precision PMPD run as the step-weighted mean of the two
    fixed-precision kernel latencies (Table 3 caption; Appendix A.5)."""
    return frac_high * lat_high + (1.0 - frac_high) * lat_low


def high_precision_fraction(avg_bits: float, high: int, low: int) -> float:
    """Fraction of decode steps run at the high precision given the average bit-width."""
    return (avg_bits - low) / (high - low)


# ------------------------------------------------ static scheduler (Section 4.3) ----
def schedule_grid(OL: int, N: int):
    """Candidate switch points {0} u {k OL/(N-1)}: exact rationals rounded to the nearest step (halves up)."""
    from fractions import Fraction
    from math import floor

    return [int(floor(Fraction(k * OL, N - 1) + Fraction(1, 2))) for k in range(N)]


def schedule_search_brute_force(precisions, OL: int, N: int, quality, q_ref: float, eps: float):
    """Every progressive schedule on the candidate grid (st[0] = 0, st non-decreasing, Eq. 3) is measured;
    the feasible one (Eq. 2: quality >= q_ref - eps) with the fewest high-precision tokens wins (Eq. 1):
    lowest average bit-width over OL steps, ties to the lexicographically smallest st.
    Returns (st, avg_bits, number of schedules on the grid) or None when nothing is feasible."""
    from itertools import combinations_with_replacement

    grid = sorted(set(schedule_grid(OL, N)))
    n = len(precisions)
    best = None
    count = 0
    for tail in combinations_with_replacement(grid, n - 1):  # non-decreasing tuples
        st = (0,) + tuple(tail)
        count += 1
        if quality(list(precisions), list(st)) < q_ref - eps:
            continue
        avg = schedule_avg_bits(precisions, st, OL)
        key = (avg, st)
        if best is None or key < best[0]:
            best = (key, st, avg)
    if best is None:
        return None
    return list(best[1]), best[2], count


# ------------------------------------------- learned scheduler (Section 4.3, Appendix A.1.1 "Model Architecture") ----
def learned_scheduler(q, K, V, W1, b1, W2, b2):
    """Forward pass of the learned scheduler in fp64, step by step as the appendix states it:
        scores_t = (q . K_t) / sqrt(D_k)            K: [T, D_k] key cache of the chosen block
        p        = softmax over the T prompt tokens
        O        = sum_t p_t V_t                     V: [T, D_v] value cache
        hid      = relu(W1 O + b1)                   one hidden layer
        probs    = softmax(W2 hid + b2)              one class per candidate switch point
    Returns (O [D_v], probs [N], class) with class = the first index of the largest probability."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K).astype(np.float64)
    V = np.asarray(V).astype(np.float64)
    T, Dk = K.shape
    scores = np.empty(T)
    for t in range(T):
        scores[t] = np.dot(q, K[t]) / np.sqrt(float(Dk))
    e = np.exp(scores - scores.max())
    p = e / e.sum()
    O = np.zeros(V.shape[1])
    for t in range(T):
        O += p[t] * V[t]
    hid = np.maximum(np.asarray(W1, dtype=np.float64) @ O + np.asarray(b1, dtype=np.float64), 0.0)
    z = np.asarray(W2, dtype=np.float64) @ hid + np.asarray(b2, dtype=np.float64)
    ez = np.exp(z - z.max())
    probs = ez / ez.sum()
    return O, probs, int(np.argmax(probs))
