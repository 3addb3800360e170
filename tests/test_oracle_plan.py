"""Pins of the oracle's concurrency rule (Sec. 4.1 Eq. 1-3): a hand-worked table and the rule's properties."""
import math
import os

import pytest
from hypothesis import given, settings, strategies as st

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "plan_table.txt")


def rows():
    out = []
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            f = line.split()
            out.append((int(f[0]), float(f[1]), float(f[2]), int(f[3]), int(f[4]), int(f[5]),
                        (int(f[6]), int(f[7]), int(f[8]))))
    return out


@pytest.mark.parametrize("B,C,alpha,Kmax,Lmax,Ncap,want", rows())
def test_plan_table(orc32, B, C, alpha, Kmax, Lmax, Ncap, want):
    assert orc32.plan(B, C, alpha, Kmax, Lmax, Ncap) == want


@settings(max_examples=300, deadline=None)
@given(B=st.integers(1, 4096), C=st.floats(1.0, 8192.0), alpha=st.floats(0.05, 8.0), Kmax=st.integers(0, 8),
       Lmax=st.integers(0, 8))
def test_plan_properties(orc32, B, C, alpha, Kmax, Lmax):
    N, K, L = orc32.plan(B, C, alpha, Kmax, Lmax, 64)
    assert 1 <= N <= 64
    assert N * B <= max(C, B)                 # Eq. 1: the verify batch does not exceed C_peak (floor)
    if N == 1:
        assert K == 0 and L == 0              # nothing to draft
    else:
        assert 1 <= K <= min(N - 1, Kmax)     # Eq. 2
        assert 1 <= L <= min(Lmax, N - 1)
        assert N <= 1 + K + (L - 1) * K * K   # cannot verify more nodes than candidates
        n_eq1 = min(64, int(math.floor(C / B)))
        assert 2.0 ** L <= n_eq1 / alpha * (1 + 1e-12)   # Eq. 3 with Eq. 1's N: L <= log2(N / alpha)


@settings(max_examples=100, deadline=None)
@given(C=st.floats(8.0, 4096.0), B1=st.integers(1, 512), B2=st.integers(1, 512))
def test_plan_monotone_in_concurrency(orc32, C, B1, B2):
    """More live sequences never get a larger tree (the strategy's point: shrink speculation as B grows)."""
    lo, hi = min(B1, B2), max(B1, B2)
    n_lo, n_hi = orc32.plan(lo, C), orc32.plan(hi, C)
    assert n_lo[0] >= n_hi[0] and n_lo[2] >= n_hi[2]


def test_plan_rejects_bad_arguments(orc32):
    from oracle.oracle import OracleError
    for args in [(0, 256.0), (4, 0.0), (4, -1.0)]:
        with pytest.raises(OracleError):
            orc32.plan(*args)
    with pytest.raises(OracleError):
        orc32.plan(4, 256.0, alpha=0.0)


# ---- knee of a latency curve (appendix, empirical measurement of C_peak) --------------------------------------
def two_segment(xs, brk, flat, slope):
    return [flat if x <= brk else flat + slope * (x - brk) for x in xs]


@pytest.mark.parametrize("brk", [2, 5, 17, 40, 63])
def test_knee_of_a_two_segment_curve_is_its_break(orc32, brk):
    """Flat, then linear: the chord's height above the curve grows up to the break and shrinks after it, so the
    farthest sample is the break itself."""
    xs = list(range(1, 65))
    ys = two_segment(xs, brk, 3.0, 0.25)
    assert xs[orc32.knee(xs, ys)] == brk


def test_knee_is_invariant_under_affine_maps_of_either_axis(orc32):
    xs = [1, 2, 4, 8, 16, 32, 64, 128, 256, 512]
    ys = [4.0, 4.0, 4.01, 4.03, 4.05, 4.2, 4.9, 8.8, 17.0, 33.5]
    k = orc32.knee(xs, ys)
    assert orc32.knee([3 * x + 7 for x in xs], ys) == k
    assert orc32.knee(xs, [1000 * y - 50 for y in ys]) == k
    assert xs[k] in (32, 64)                   # the sample where the flat part ends, judged by eye


def test_knee_edge_cases(orc32):
    assert orc32.knee([1, 2, 3], [1.0, 2.0, 3.0]) == 0          # a straight line has no knee: first sample
    assert orc32.knee([1, 2, 3, 4], [5.0, 5.0, 5.0, 5.0]) == 0  # constant
    with pytest.raises(Exception):
        orc32.knee([1, 2], [1.0, 2.0])
    with pytest.raises(Exception):
        orc32.knee([1, 1, 2], [1.0, 2.0, 3.0])                  # x must increase


@settings(max_examples=100, deadline=None)
@given(brk=st.integers(2, 30), flat=st.floats(0.5, 50.0), slope=st.floats(0.01, 10.0), n=st.integers(34, 80))
def test_knee_break_property(orc32, brk, flat, slope, n):
    xs = list(range(1, n + 1))
    assert xs[orc32.knee(xs, two_segment(xs, brk, flat, slope))] == brk
