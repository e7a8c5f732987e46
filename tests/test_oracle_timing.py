"""Pins of the timing-model oracle (Sec. 3.1, App. C): the paper's printed table and claims."""
import math
import os

import pytest

from oracle import timing as Tm

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "optimal_microbatches.txt")


def test_optimal_microbatch_table_of_the_appendix():
    rows = 0
    for line in open(GOLDEN):
        if not line.strip() or line.startswith("#"):
            continue
        method, A, M = line.split()
        A, M = int(A), int(M)
        N = A if method == "e2e" else int(method)
        assert Tm.optimal_microbatches(A, N) == M, line
        rows += 1
    assert rows == 35


def test_end_to_end_degenerates_to_the_gpipe_formula():
    """Sec. 3.1: for N = A the time per batch is 2 (M + A - 1) c(M)."""
    for A in range(1, 12):
        for M in (3, 4, 8, 16, 64):
            assert math.isclose(Tm.time_per_batch(A, M, A), 2 * (M + A - 1) * Tm.microbatch_cost(M), rel_tol=1e-14)


def test_fifty_percent_speed_up_of_two_wise_from_fifteen_accelerators():
    """Sec. 3.1: with the optimal M on both sides 2-wise is 50 % faster than end-to-end with GPipe at
    15 or more accelerators (and not yet at 14)."""
    def speedup(A):
        e2e = Tm.time_per_batch(A, Tm.optimal_microbatches(A, A), A)
        two = Tm.time_per_batch(A, Tm.optimal_microbatches(A, 2), 2)
        return e2e / two
    assert speedup(14) < 1.495 <= round(speedup(15), 2) and speedup(15) > 1.49
    assert all(speedup(A + 1) > speedup(A) for A in range(4, 40))


def test_independent_of_depth_below_half_the_stack():
    """Sec. 3.1: for N < 1 + A/2 the time per batch does not depend on the number of modules."""
    for N in (1, 2, 3, 4):
        for M in (1, 2, 4, 16):
            ts = {round(Tm.time_per_batch(A, M, N), 12) for A in range(2 * N - 1, 40)}
            assert len(ts) == 1


def test_without_microbatching():
    """M = 1: N forward and N backward slots of cost c(1) = c0 + c1; N = 1 local, N = A end-to-end."""
    assert math.isclose(Tm.time_per_batch(8, 1, 1), 2 * (Tm.C0 + Tm.C1))
    assert math.isclose(Tm.time_per_batch(8, 1, 8), 16 * (Tm.C0 + Tm.C1))
    assert Tm.time_per_batch(4, 1, 9) == Tm.time_per_batch(4, 1, 4)        # the window is clamped to A
    with pytest.raises(ValueError):
        Tm.time_per_batch(0, 1, 1)


def test_partial_window_branch_follows_the_appendix_derivation():
    """App. C, Case 4 (M > 2, A < 2N - 1): every accelerator removed from the stack takes M - 2 slots
    off the period, starting from the end-to-end period of an N-deep stack,
        T(A, M, N) = (A - N)(M - 2) c(M) + 2 (M + N - 1) c(M),
    and at A = 2N - 1 the branch meets the (N + 1) M c(M) of the deep-stack case.  The right-hand
    sides are written from the derivation, not from the case formula the oracle evaluates."""
    checked = 0
    for N in range(3, 12):
        for A in range(N + 1, 2 * N - 1):
            for M in (3, 4, 5, 8, 16, 64):
                c = Tm.C0 + Tm.C1 / M
                want = (A - N) * (M - 2) * c + 2 * (M + N - 1) * c
                assert math.isclose(Tm.time_per_batch(A, M, N), want, rel_tol=1e-13), (A, M, N)
                # one accelerator fewer: exactly M - 2 slots less
                step = Tm.time_per_batch(A, M, N) - Tm.time_per_batch(A - 1, M, N)
                assert math.isclose(step, (M - 2) * c, rel_tol=1e-10), (A, M, N)
                checked += 1
        for M in (3, 4, 8, 16):
            c = Tm.C0 + Tm.C1 / M
            A = 2 * N - 1
            below = (A - 1 - N) * (M - 2) * c + 2 * (M + N - 1) * c      # the derivation at A - 1
            assert math.isclose(Tm.time_per_batch(A, M, N), (N + 1) * M * c, rel_tol=1e-13)
            assert math.isclose(Tm.time_per_batch(A, M, N) - below, (M - 2) * c, rel_tol=1e-10)
    assert checked > 100
