"""Static-scheduler search (Section 4.3): candidate grid, schedule count, and the offline optimisation of
Eq. 1-3 against a brute-force enumeration.  The quality function is synthetic (the paper's needs its
validation sets): any function of the schedule works, the search only compares it with q_ref - eps."""
import random

import pytest

import oracle
import paper_2410_13461_amd as pmpd


def test_grid_values_worked_by_hand():
    # OL/(N-1) = 64: 0, 64, 128, 192, 256
    assert pmpd.schedule_grid(256, 5) == [0, 64, 128, 192, 256]
    # 100/3 = 33.33 -> 33, 66.67 -> 67
    assert pmpd.schedule_grid(100, 4) == [0, 33, 67, 100]
    # halves round up: 10/4 = 2.5 -> 3, 5, 7.5 -> 8
    assert pmpd.schedule_grid(10, 5) == [0, 3, 5, 8, 10]
    # N = OL + 1: every step is a candidate
    assert pmpd.schedule_grid(7, 8) == list(range(8))
    for OL, N in ((256, 5), (100, 4), (10, 5), (1000, 17), (3, 2), (129, 130)):
        assert pmpd.schedule_grid(OL, N) == oracle.schedule_grid(OL, N)
    for OL, N in ((10, 1), (10, 12), (0, 2)):
        with pytest.raises(pmpd.PMPDError):
            pmpd.schedule_grid(OL, N)


def test_schedule_count_closed_form():
    # the figure for OL = 256 and three precisions: 1 + 256*2 + C(256,2) = 33153
    assert pmpd.schedule_count(256, 3) == 33153 == oracle.progressive_schedule_count(256, 3)
    for OL, n in ((1, 1), (12, 3), (128, 2), (256, 4), (2048, 3), (4096, 5)):
        assert pmpd.schedule_count(OL, n) == oracle.progressive_schedule_count(OL, n)
    # with every step a candidate the enumeration visits exactly that many schedules
    _, _, visited = oracle.schedule_search_brute_force((4, 3, 2), 12, 13, lambda P, st: 1.0, 0.0, 0.0)
    assert visited == pmpd.schedule_count(12, 3) == 91


def test_brute_force_oracle_on_hand_worked_cases():
    """Pins of the oracle's own choice (no product code involved), worked by hand.

    (a) P = (4, 3, 2), OL = 4, every step a candidate (N = 5); the quality bar forbids 2 bits before step 2.
        Bits of st = (0, a, b): 4 a + 3 (b - a) + 2 (4 - b) = 8 + a + b, smallest for a = 0 and the smallest
        allowed b = 2: steps 0, 1 at 3 bits, steps 2, 3 at 2 bits = 10 bits = 2.5 per step.  Non-decreasing
        pairs (a, b) out of 5 points: C(6, 2) = 15 schedules.
    (b) The same P and OL on the grid {0, 2, 4} (N = 3), feasible iff a + b >= 4.  The fewest bits among the
        feasible ones is 12 (3.0 per step), reached twice: (0, 0, 4) = four steps at 3 bits, and (0, 2, 2) = two
        steps at 4 bits then two at 2 bits.  The tie goes to the lexicographically smallest st: (0, 0, 4).
        C(4, 2) = 6 schedules on the grid."""
    got = oracle.schedule_search_brute_force((4, 3, 2), 4, 5, lambda P, st: 1.0 if st[2] >= 2 else 0.0, 1.0, 0.0)
    assert got == ([0, 0, 2], 2.5, 15)
    got = oracle.schedule_search_brute_force((4, 3, 2), 4, 3, lambda P, st: 1.0 if st[1] + st[2] >= 4 else 0.0, 1.0, 0.0)
    assert got == ([0, 0, 4], 3.0, 6)
    # the product agrees on both (its own visit count is at most the oracle's)
    st, avg, n = pmpd.schedule_search((4, 3, 2), 4, 5, lambda P, st: 1.0 if st[2] >= 2 else 0.0, 1.0, 0.0)
    assert (st, avg) == ([0, 0, 2], 2.5) and n <= 15
    st, avg, n = pmpd.schedule_search((4, 3, 2), 4, 3, lambda P, st: 1.0 if st[1] + st[2] >= 4 else 0.0, 1.0, 0.0)
    assert (st, avg) == ([0, 0, 4], 3.0) and n <= 6
    # limits: a bar everything passes -> the lowest precision from step 0; a bar only all-high passes
    OL = 256
    assert oracle.schedule_search_brute_force((4, 3, 2), OL, 5, lambda P, st: 0.0, 1.0, 1.0)[:2] == ([0, 0, 0], 2.0)
    assert oracle.schedule_search_brute_force((4, 3, 2), OL, 5, lambda P, st: 1.0 if st[1] == OL else 0.0, 1.0, 0.0)[:2] == ([0, OL, OL], 4.0)


def _synthetic_quality(P, OL, rng):
    """Quality falls with the tokens spent at low precision, faster early in the sequence."""
    w = {p: rng.uniform(0.0, 0.3) * (max(P) - p) for p in P}
    early = rng.uniform(0.0, 2.0)

    def q(prec, st):
        loss = 0.0
        for j, p in enumerate(prec):
            lo = st[j]
            hi = st[j + 1] if j + 1 < len(prec) else OL
            for k in range(lo, hi):
                loss += w[p] * (1.0 + early * (1.0 - k / OL))
        return 1.0 - loss / OL

    return q


@pytest.mark.parametrize("P,OL,N", [((4, 3, 2), 256, 5), ((4, 3, 2), 100, 4), ((3, 2), 128, 9), ((4, 2), 64, 65),
                                    ((8, 4, 3, 2), 60, 7), ((4,), 32, 3)])
def test_search_matches_brute_force(P, OL, N):
    rng = random.Random(hash((P, OL, N)) & 0xFFFF)
    for trial in range(6):
        q = _synthetic_quality(P, OL, rng)
        q_ref = q(list(P), [0] + [OL] * (len(P) - 1))  # everything at the highest precision
        eps = rng.choice([0.0, 0.01, 0.05, 0.2, 1.0])
        want = oracle.schedule_search_brute_force(P, OL, N, q, q_ref, eps)
        assert want is not None  # the all-high schedule is always feasible
        st, avg, evaluated = pmpd.schedule_search(P, OL, N, q, q_ref, eps)
        assert st == want[0]
        assert avg == pytest.approx(want[1], abs=1e-12)
        assert 1 <= evaluated <= want[2]
        # the result is a valid schedule for the run-time scheduler and gives that average
        sch = pmpd.Schedule(P, st, OL)
        assert sch.avg_bits(OL) == pytest.approx(avg, abs=1e-12)
        assert oracle.schedule_valid(P, st, OL)


def test_search_limits():
    P, OL, N = (4, 3, 2), 256, 5
    # eps large enough: everything at the lowest precision from step 0
    st, avg, _ = pmpd.schedule_search(P, OL, N, lambda p, s: 0.0, 1.0, 1.0)
    assert st == [0, 0, 0] and avg == 2.0
    # only the all-high schedule passes: the lower precisions are never reached
    st, avg, _ = pmpd.schedule_search(P, OL, N, lambda p, s: 1.0 if s[1] == OL else 0.0, 1.0, 0.0)
    assert st == [0, OL, OL] and avg == 4.0
    # nothing passes
    with pytest.raises(pmpd.PMPDError) as e:
        pmpd.schedule_search(P, OL, N, lambda p, s: 0.0, 1.0, 0.0)
    assert e.value.status == -3
    assert oracle.schedule_search_brute_force(P, OL, N, lambda p, s: 0.0, 1.0, 0.0) is None
    with pytest.raises(pmpd.PMPDError):
        pmpd.schedule_search((2, 3), OL, N, lambda p, s: 1.0, 1.0, 0.0)  # not decreasing
