"""Pins for the CPU oracle: each check ties it to something other than itself
(exact rational brute force, numpy library routines, closed forms, invariants,
numbers printed in the paper)."""
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
import pmpd_synth as synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- helpers ---
def frac_of_half(h) -> Fraction:
    """Exact rational value of a numpy float16 (via its float64 widening, which is exact)."""
    return Fraction(float(np.float16(h)))


def brute_force_linear(q4, s, a, b, x):
    """y[r] = sum_i (a + s*2^(4-b)*((q4>>(4-b)) + 1/2)) * x[i], in exact rationals."""
    out_f, in_f = q4.shape
    ys, ts = [], []
    for r in range(out_f):
        acc = Fraction(0)
        tb = Fraction(0)
        for i in range(in_f):
            g = i // 128
            qb = int(q4[r, i]) >> (4 - b)
            w = frac_of_half(a[r, g]) + frac_of_half(s[r, g]) * (2 ** (4 - b)) * (Fraction(qb) + Fraction(1, 2))
            xv = frac_of_half(x[i])
            acc += w * xv
            tb += abs(w) * abs(xv)
        ys.append(acc)
        ts.append(tb)
    return ys, ts


# ------------------------------------------------- fp16 decoding (library) ---
def test_fp16_decode_matches_numpy_for_every_bit_pattern():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.fp16_value(int(v)) for v in bits])
    both_nan = np.isnan(ref) & np.isnan(got)
    assert np.all(both_nan | (ref == got))
    # signed zero keeps its sign
    assert np.signbit(oracle.fp16_value(0x8000))


# ------------------------------------------------------ P1: brute force ------
@pytest.mark.parametrize("b", [4, 3, 2])
@pytest.mark.parametrize("out_f,in_f,random_min", [(5, 128, False), (8, 256, True), (3, 384, True)])
def test_linear_matches_exact_rational_brute_force(b, out_f, in_f, random_min):
    q4, s, a = synth.draw_weights(11, 0, out_f, out_f, in_f, random_min=random_min)
    x = synth.draw_x(11, 0, 0, 0, in_f)[0]
    ys, ts = brute_force_linear(q4, s, a, b, x)
    y, t = oracle.linear(q4, s, a, b, x)
    planes, sa = oracle.pack(q4, s, a)
    yp, tp = oracle.linear_packed(planes, sa, b, out_f, in_f, x)
    for r in range(out_f):
        scale = float(ts[r])
        assert abs(y[0, r] - float(ys[r])) <= 1e-13 * scale
        assert abs(yp[0, r] - float(ys[r])) <= 1e-13 * scale
        assert abs(t[0, r] - scale) <= 1e-13 * scale
        assert abs(tp[0, r] - scale) <= 1e-13 * scale


@pytest.mark.parametrize("b", [4, 3, 2])
def test_dequant_is_exact_against_rationals(b):
    q4, s, a = synth.draw_weights(5, 1, 2, 4, 256, random_min=True)
    W = oracle.dequant(q4, s, a, b)
    for r in range(4):
        for i in range(256):
            g = i // 128
            w = frac_of_half(a[r, g]) + frac_of_half(s[r, g]) * (2 ** (4 - b)) * (
                Fraction(int(q4[r, i]) >> (4 - b)) + Fraction(1, 2))
            assert Fraction(float(W[r, i])) == w  # fp64 holds the value exactly


# -------------------------------------- P2: special case of a library matmul --
@pytest.mark.parametrize("b", [4, 3, 2])
def test_linear_equals_numpy_matmul_on_dense_matrix(b):
    out_f, in_f, m = 70, 512, 3
    q4, s, a = synth.draw_weights(3, 0, 1, out_f, in_f, random_min=True)
    x = synth.draw_x(3, 0, 0, 1, in_f, m=m)
    qb = (q4 >> (4 - b)).astype(np.float64)
    sd = np.repeat(s.astype(np.float64), 128, axis=1)
    ad = np.repeat(a.astype(np.float64), 128, axis=1)
    W = ad + sd * 2.0 ** (4 - b) * (qb + 0.5)
    ref = x.astype(np.float64) @ W.T
    y, t = oracle.linear(q4, s, a, b, x)
    assert y.shape == (m, out_f)
    assert np.allclose(y, ref, rtol=0, atol=1e-12 * np.abs(t).max())
    assert np.allclose(t, np.abs(x.astype(np.float64)) @ np.abs(W).T, rtol=1e-13)
    assert np.array_equal(oracle.dequant(q4, s, a, b), W)


# ------------------------------------------- P3: nested bin-midpoint invariant --
@pytest.mark.parametrize("b", [4, 3, 2])
def test_linear_dense_is_the_same_definition(b):
    """The matmul form used for whole layers agrees with the plain loops (themselves pinned by exact
    rationals above) far below any tolerance in use, and its budget T is the loops' budget."""
    q4, s, a = synth.draw_weights(41, 0, 0, 70, 384, random_min=True)
    x = synth.draw_x(41, 0, 0, 0, 384, m=5)
    y, t = oracle.linear(q4, s, a, b, x)
    yd, td = oracle.linear_dense(q4, s, a, b, x)
    assert yd.shape == y.shape == (5, 70)
    assert np.max(np.abs(yd - y)) <= 1e-12 * np.max(t)
    assert np.max(np.abs(td - t)) <= 1e-12 * np.max(t)


def test_nested_bin_midpoints():
    rng = np.random.default_rng(0)
    s = rng.uniform(1e-3, 1e-2, size=(1, 1)).astype(np.float16)
    a = rng.uniform(-0.1, 0.1, size=(1, 1)).astype(np.float16)
    q4 = np.tile(np.arange(16, dtype=np.uint8), 8)[None, :]  # every code, one group
    W = {b: oracle.dequant(q4, s, a, b)[0, :16] for b in (4, 3, 2, 1)}
    sv, av = float(s[0, 0]), float(a[0, 0])
    for b in (3, 2, 1):
        for q in range(16):
            qb = q >> (4 - b)
            # the b-bit level is the midpoint of the two (b+1)-bit levels it contains
            lo = W[b + 1][(2 * qb) << (4 - b - 1)]
            hi = W[b + 1][(2 * qb + 1) << (4 - b - 1)]
            assert W[b][q] == 0.5 * (lo + hi)
            # and it sits inside its own bin, which contains the 4-bit level of q
            width = sv * 2 ** (4 - b)
            assert av + width * qb <= W[4][q] < av + width * (qb + 1)
            assert av + width * qb < W[b][q] < av + width * (qb + 1)
            assert abs(W[b][q] - W[4][q]) <= sv * (2 ** (4 - b) - 1) / 2 + 1e-15


# ------------------------------------------------- P4: round trip and prefix --
@pytest.mark.parametrize("out_f,in_f", [(64, 128), (100, 384), (130, 256)])
def test_pack_unpack_round_trip_and_prefix(out_f, in_f):
    q4, s, a = synth.draw_weights(7, 2, 3, out_f, in_f, random_min=True)
    planes, sa = oracle.pack(q4, s, a)
    assert all(p.size == oracle.padded_rows(out_f) * in_f // 32 for p in planes)
    assert np.array_equal(oracle.unpack(planes, 4, out_f, in_f), q4)
    s2, a2 = oracle.unpack_sa(sa, out_f, in_f)
    assert np.array_equal(s2.view(np.uint16), s.view(np.uint16))
    assert np.array_equal(a2.view(np.uint16), a.view(np.uint16))
    rng = np.random.default_rng(1)
    for b in (3, 2, 1):
        # planes below the top b are absent (None) or garbage: the result must not change
        poisoned = list(planes[:b]) + [rng.integers(0, 2 ** 32, size=planes[0].size, dtype=np.uint32)
                                       for _ in range(4 - b)]
        assert np.array_equal(oracle.unpack(poisoned, b, out_f, in_f), q4 >> (4 - b))
        absent = list(planes[:b]) + [None] * (4 - b)
        assert np.array_equal(oracle.unpack(absent, b, out_f, in_f), q4 >> (4 - b))


def test_pack_is_a_bijection_onto_the_plane_bits():
    out_f, in_f = 64, 256
    # all-ones codes fill every bit of every plane
    q4 = np.full((out_f, in_f), 15, dtype=np.uint8)
    s = np.ones((out_f, in_f // 128), dtype=np.float16)
    planes, _ = oracle.pack(q4, s, s)
    for p in planes:
        assert np.all(p == 0xFFFFFFFF)
    # a single weight sets exactly one bit per plane, distinct weights distinct bits
    seen = [set() for _ in range(4)]
    for (r, i) in [(0, 0), (0, 1), (0, 2), (0, 31), (0, 32), (0, 127), (0, 128), (1, 0), (63, 255), (17, 77)]:
        q = np.zeros((out_f, in_f), dtype=np.uint8)
        q[r, i] = 15
        pl, _ = oracle.pack(q, s, s)
        for k in range(4):
            nz = np.flatnonzero(pl[k])
            assert nz.size == 1
            word = int(pl[k][nz[0]])
            assert bin(word).count("1") == 1
            key = (int(nz[0]), word)
            assert key not in seen[k]
            seen[k].add(key)
    # formula anchors, worked by hand from the storage-format definition.
    # (r, i) = (0, 0): t = j = kb = v = c = n = 0 -> word 0; even planes bit 1, odd planes bit 0
    q = np.zeros((out_f, in_f), dtype=np.uint8)
    q[0, 0] = 0b1010
    pl, _ = oracle.pack(q, s, s)
    assert [int(pl[k][0]) for k in range(4)] == [1 << 1, 0, 1 << 1, 0]
    # (r, i) = (17, 77): rr = 16*1 + 1; e = 32*2 + 8*1 + 5 -> kb 2, v 1, c 5, n = 2 + 4 = 6;
    # word (16*2 + 1)*4 + 1 = 133; even planes bit 4*6 + 3 = 27, odd planes bit 4*6 + 2 = 26
    q = np.zeros((out_f, in_f), dtype=np.uint8)
    q[17, 77] = 0b0111
    pl, _ = oracle.pack(q, s, s)
    assert [int(pl[k][133]) for k in range(4)] == [0, 1 << 26, 1 << 27, 1 << 26]
    # (r, i) = (63, 255): group 1; rr = 16*3 + 15; e = 127 -> kb 3, v 3, c 7, n = 3 + 4 = 7;
    # word 256 + (16*3 + 15)*4 + 3 = 511; even planes bit 28 + 2 = 30, odd planes bit 28 + 1 = 29
    q = np.zeros((out_f, in_f), dtype=np.uint8)
    q[63, 255] = 0b1100
    pl, _ = oracle.pack(q, s, s)
    assert [int(pl[k][511]) for k in range(4)] == [1 << 30, 1 << 29, 0, 0]
    # v = 2 of an odd plane wraps: (0, 16): kb 0, v 2, c 0, n 0 -> bit (0 + 31) mod 32 of word 0
    q = np.zeros((out_f, in_f), dtype=np.uint8)
    q[0, 16] = 0b0001
    pl, _ = oracle.pack(q, s, s)
    assert [int(pl[k][0]) for k in range(4)] == [0, 0, 0, 1 << 31]


def test_pack_pads_rows_with_zeros_and_rejects_bad_codes():
    q4, s, a = synth.draw_weights(1, 0, 0, 65, 128)
    planes, sa = oracle.pack(q4, s, a)
    assert planes[0].size == 128 * 128 // 32
    # tile 1 holds one real row (position 0: word t = 0 of the 16-byte units j = 0 of each of the
    # four 32-column slices); every other word is padding and stays zero
    t1 = planes[0].reshape(2, 1, 4, 16, 4)[1, 0]  # [kb][j][t]
    assert np.all(t1[:, 1:, :] == 0) and np.all(t1[:, 0, 1:] == 0)
    assert np.all(sa.reshape(2, 1, 64)[1, 0, 1:] == 0)
    bad = q4.copy()
    bad[3, 5] = 16
    with pytest.raises(ValueError):
        oracle.pack(bad, s, a)


# ----------------------------------------------------------- P5: closed forms --
@pytest.mark.parametrize("b,c_hi,c_lo", [(4, 7.5, -7.5), (3, 7.0, -7.0), (2, 6.0, -6.0)])
def test_constant_codes_closed_form(b, c_hi, c_lo):
    out_f, in_f = 6, 512
    _, s, a = synth.draw_weights(2, 0, 0, out_f, in_f)  # a = -8 s
    x = synth.draw_x(2, 0, 0, 0, in_f)[0]
    Xg = x.astype(np.float64).reshape(-1, 128).sum(axis=1)
    for code, c in ((15, c_hi), (0, c_lo)):
        q4 = np.full((out_f, in_f), code, dtype=np.uint8)
        W = oracle.dequant(q4, s, a, b)
        assert np.array_equal(W, np.repeat(c * s.astype(np.float64), 128, axis=1))
        y, _ = oracle.linear(q4, s, a, b, x)
        ref = c * (s.astype(np.float64) @ Xg)
        assert np.allclose(y[0], ref, rtol=0, atol=1e-12)


@pytest.mark.parametrize("b", [4, 3, 2])
def test_all_ones_and_one_hot_activations(b):
    out_f, in_f = 9, 384
    q4, s, a = synth.draw_weights(4, 0, 0, out_f, in_f, random_min=True)
    sd, ad = s.astype(np.float64), a.astype(np.float64)
    qb = (q4 >> (4 - b)).astype(np.int64).reshape(out_f, -1, 128)
    # x = 1: y_r = sum_g [128 a_g + s_g 2^(4-b) (sum q_b + 64)]
    ones = np.ones(in_f, dtype=np.float16)
    y, _ = oracle.linear(q4, s, a, b, ones)
    ref = (128 * ad + sd * 2 ** (4 - b) * (qb.sum(axis=2) + 64)).sum(axis=1)
    assert np.allclose(y[0], ref, rtol=1e-14, atol=0)
    # one-hot x picks single weights out of the whole pipeline
    W = oracle.dequant(q4, s, a, b)
    planes, sa = oracle.pack(q4, s, a)
    for j in (0, 1, 127, 128, 200, in_f - 1):
        e = np.zeros(in_f, dtype=np.float16)
        e[j] = 1
        y, _ = oracle.linear(q4, s, a, b, e)
        yp, _ = oracle.linear_packed(planes, sa, b, out_f, in_f, e)
        assert np.array_equal(y[0], W[:, j])
        assert np.array_equal(yp[0], W[:, j])


# ------------------------------------------------------------ P6: statistics ---
def test_generator_and_reconstruction_statistics():
    out_f, in_f = 256, 4096
    q4, s, a = synth.draw_weights(0, 0, 0, out_f, in_f)
    assert q4.min() == 0 and q4.max() == 15
    assert abs(q4.mean() - 7.5) < 0.02
    sd = s.astype(np.float64)
    assert 1e-3 <= sd.min() and sd.max() <= 1e-2 + 1e-5
    assert np.array_equal(a.astype(np.float64), -8 * sd)
    for b, var in ((4, 21.25), (3, 21.0), (2, 20.0)):
        W = oracle.dequant(q4, s, a, b) / np.repeat(sd, 128, axis=1)
        assert abs(W.mean()) < 0.02
        assert abs(W.var() - var) < 0.1
    x = synth.draw_x(0, 0, 0, 0, in_f)[0]
    y, _ = oracle.linear(q4, s, a, 4, x)
    expect = np.sqrt(in_f * np.mean(sd ** 2) * 21.25)
    assert 0.8 * expect < y.std() < 1.2 * expect


# ------------------------------------------------------------- P7: linearity ---
@pytest.mark.parametrize("b", [4, 2])
def test_linearity_in_x_and_in_scale(b):
    out_f, in_f = 12, 256
    q4, s, a = synth.draw_weights(9, 0, 0, out_f, in_f, random_min=True)
    x = synth.draw_x(9, 0, 0, 0, in_f)[0]
    y, _ = oracle.linear(q4, s, a, b, x)
    y4, _ = oracle.linear(q4, s, a, b, (x * np.float16(4)).astype(np.float16))
    assert np.array_equal(y4, 4 * y)
    y2, _ = oracle.linear(q4, (s * np.float16(2)).astype(np.float16), (a * np.float16(2)).astype(np.float16), b, x)
    assert np.array_equal(y2, 2 * y)
    # rows are independent and ordered: permuting rows permutes outputs
    perm = np.random.default_rng(0).permutation(out_f)
    yp, _ = oracle.linear(q4[perm], s[perm], a[perm], b, x)
    assert np.array_equal(yp[0], y[0][perm])


# ----------------------------------------------- P8: schedule closed forms ------
def test_schedule_lookup_and_average_bits():
    P, st, OL = synth.SCHEDULE_7B_256
    assert oracle.schedule_valid(P, st, OL)
    bits = [oracle.schedule_bits(P, st, k) for k in range(OL)]
    assert bits[0] == 4 and bits[63] == 4 and bits[64] == 3 and bits[159] == 3
    assert bits[160] == 2 and bits[255] == 2
    assert bits.count(4) == 64 and bits.count(3) == 96 and bits.count(2) == 96
    assert oracle.schedule_avg_bits(P, st, OL) == 2.875
    P, st, OL = synth.SCHEDULE_13B_128
    assert [oracle.schedule_bits(P, st, k) for k in (0, 47, 48, 127)] == [3, 3, 2, 2]
    assert oracle.schedule_avg_bits(P, st, OL) == 2.375


def test_schedule_edge_cases():
    # equal switch points skip the middle precision; st = OL is never reached
    assert [oracle.schedule_bits((4, 3, 2), (0, 10, 10), k) for k in (0, 9, 10, 11)] == [4, 4, 2, 2]
    assert oracle.schedule_bits((4, 3), (0, 8), 7) == 4
    assert oracle.schedule_avg_bits((4, 3), (0, 8), 8) == 4.0
    # lowest precision from the first step: the average is exactly the low bit-width
    # (Table 1 lists such entries with Bit = 2.0 and 3.0)
    assert oracle.schedule_avg_bits((3, 2), (0, 0), 100) == 2.0
    assert oracle.schedule_valid((3, 2), (0, 0), 100)
    assert oracle.schedule_valid((4, 3, 2), (0, 5, 256), 256)
    # precedence (Eq. 3), range (Eq. 2), ordering, and the start of the high precision
    assert not oracle.schedule_valid((4, 3, 2), (0, 9, 5), 256)
    assert not oracle.schedule_valid((4, 3), (0, 300), 256)
    assert not oracle.schedule_valid((4, 3), (0, -1), 256)
    assert not oracle.schedule_valid((3, 4), (0, 5), 256)
    assert not oracle.schedule_valid((4, 3), (2, 5), 256)
    assert not oracle.schedule_valid((4, 3), (0,), 256)


def test_progressive_schedule_count():
    # Section 4.3: sum_r C(OL, r) C(|P|-1, r); OL = 256, |P| = 3 -> 1 + 512 + 32640
    assert oracle.progressive_schedule_count(256, 3) == 33153
    assert oracle.progressive_schedule_count(256, 1) == 1
    # brute force on a tiny case: non-increasing precision sequences of length OL over P
    import itertools
    OL, P = 5, (4, 3, 2)
    n = 0
    for seq in itertools.product(P, repeat=OL):
        if seq[0] == P[0] and all(seq[i] >= seq[i + 1] for i in range(OL - 1)):
            n += 1
    # the formula counts switch positions among OL slots (a switch may also sit before
    # the first step), i.e. sequences that may start below the top precision
    n_any_start = sum(1 for seq in itertools.product(P, repeat=OL)
                      if all(seq[i] >= seq[i + 1] for i in range(OL - 1)))
    assert n <= oracle.progressive_schedule_count(OL, len(P))
    assert n_any_start == oracle.progressive_schedule_count(OL, len(P))


# --------------------------- P9: the paper's own worked example (Tables 1,3,7,8) --
def _golden():
    rows = {}
    with open(os.path.join(GOLDEN, "vicuna7b_linear_latency.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            tok = line.split()
            if tok[0] == "avg_bits":
                rows["avg_bits"] = [float(v) for v in tok[1:]]
            elif tok[0] == "speedup":
                rows[("speedup", tok[1], tok[2])] = (float(tok[3]), float(tok[4]))
            else:
                rows[(tok[0], tok[1])] = dict(zip(("fp16", "w2", "w3", "w4"), map(float, tok[2:])))
    return rows


def test_schedule_weighted_latency_reproduces_table3():
    g = _golden()
    avg = sum(g["avg_bits"]) / len(g["avg_bits"])
    f_hi = oracle.high_precision_fraction(avg, 3, 2)
    assert abs(f_hi - 0.3567) < 1e-3

    def speedup(gpu, proj):
        row = g[(gpu, proj)]
        return row["fp16"] / oracle.schedule_weighted_latency(row["w3"], row["w2"], f_hi)

    # the table prints two decimals (some truncated, some rounded): allow one unit in the last place
    assert abs(speedup("rtx4090", "down_proj") - g[("speedup", "rtx4090", "pmpd")][1]) < 0.011
    assert abs(speedup("rtx4090", "q_proj") - g[("speedup", "rtx4090", "pmpd")][0]) < 0.011
    assert abs(speedup("a40", "k_proj") - g[("speedup", "a40", "pmpd")][0]) < 0.011
    assert abs(speedup("a40", "down_proj") - g[("speedup", "a40", "pmpd")][1]) < 0.011
    # uniform high precision (Baseline-h) is the f_hi = 1 special case
    for gpu, col, proj in (("rtx4090", 0, "q_proj"), ("rtx4090", 1, "down_proj"),
                           ("a40", 0, "k_proj"), ("a40", 1, "down_proj")):
        row = g[(gpu, proj)]
        base = row["fp16"] / oracle.schedule_weighted_latency(row["w3"], row["w2"], 1.0)
        assert abs(base - g[("speedup", gpu, "baseline_h")][col]) < 0.015


def test_fp16_baseline_definition_against_exact_rationals():
    """linear_fp16 against exact rational arithmetic on a tiny case, and a closed form: rows of constants."""
    from fractions import Fraction

    W = synth.draw_fp16_weights(1, 0, 0, 5, 128)
    x = synth.draw_x(1, 0, 0, 0, 128)[0]
    y, t = oracle.linear_fp16(W, x)
    for r in range(5):
        exact = sum(Fraction(float(W[r, i])) * Fraction(float(x[i])) for i in range(128))
        budget = sum(abs(Fraction(float(W[r, i])) * Fraction(float(x[i]))) for i in range(128))
        assert abs(Fraction(float(y[0, r])) - exact) <= Fraction(1, 2 ** 45) * budget
        assert abs(Fraction(float(t[0, r])) - budget) <= Fraction(1, 2 ** 45) * budget
    Wc = np.repeat(np.arange(1, 4, dtype=np.float16)[:, None], 256, axis=1)  # row r holds r + 1
    y, t = oracle.linear_fp16(Wc, np.ones(256, dtype=np.float16))
    assert np.array_equal(y[0], [256.0, 512.0, 768.0]) and np.array_equal(t, y)
    # transposition mistake would show here: a non-square W with distinct rows and columns
    Wn = np.arange(6, dtype=np.float16).reshape(2, 3).repeat(128, axis=1)[:, :384]
    xn = np.concatenate([np.full(128, v, dtype=np.float16) for v in (1, 0, -1)])
    y, _ = oracle.linear_fp16(Wn, xn)
    assert np.array_equal(y[0], [128.0 * (0 - 2), 128.0 * (3 - 5)])
