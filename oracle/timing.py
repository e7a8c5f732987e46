"""Oracle of the paper's timing model for synchronous model-distributed training (Sec. 3.1, App. C).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path imports this module.

A accelerators (modules) in sequence, M micro-batches per mini-batch, window N in [1, A]; a time slot
(one forward or one backward of one micro-batch on one accelerator) costs c(M) = c0 + c1 / M.  The
time per mini-batch is the case formula of Sec. 3.1 / App. C, written out case by case.

Readings: N is clamped to A (a window cannot exceed the number of modules: "in the range [1, A]");
the printed case formula is the authority.  The appendix's table of optimal M agrees with it for
end-to-end, 1-wise and 2-wise training and wherever A >= 2N - 1; its entries for N >= 3 at smaller A
(some of them for N > A, and 3-wise at A = 3 differing from end-to-end at A = 3, which is the same
method) do not follow from the formula and are not used as pins.
"""
import math

C0, C1 = 0.025, 1.279   # seconds, fitted in the paper to its Transformer runs


def microbatch_cost(M, c0=C0, c1=C1):
    return c0 + c1 / M


def time_per_batch(A, M, N, c0=C0, c1=C1):
    if A < 1 or M < 1 or N < 1:
        raise ValueError("A, M, N are positive")
    N = min(N, A)
    c = microbatch_cost(M, c0, c1)
    if M == 1:
        return 2 * N * M * c
    if M == 2 or A >= 2 * N - 1:
        return (N + 1) * M * c
    return (2 + A - N) * M * c + 2 * (2 * N - A - 1) * c


def optimal_microbatches(A, N, c0=C0, c1=C1, max_m=64):
    """The power of two M <= max_m with the smallest time per batch (the smallest such M on ties)."""
    best, best_t = 1, math.inf
    M = 1
    while M <= max_m:
        t = time_per_batch(A, M, N, c0, c1)
        if t < best_t:
            best, best_t = M, t
        M *= 2
    return best
