"""Oracle for the offline tiling helpers (TEST INFRASTRUCTURE ONLY; plain Python, no shared code with the library).

grid(E): Appendix B (Evaluation Details, "Tiling-size"): M is the integer closest to sqrt(E), N = ceil(E / M).

place(ideal, M, N): Section 3.1, Step 4 (Eq. 9-10).  Experts in index order; the anchor is the ideal tile clamped
into the grid; among the unoccupied cells the one with the smallest Chebyshev distance to the anchor is taken.  The
paper does not order the cells of one ring; the reading taken (and stated in the library's header) is row by row:
smaller m first, then smaller n.  Written here as the plain definition: sort all free cells by
(distance, m, n) and take the first.
"""
from fractions import Fraction


def grid(E: int):
    # the integer closest to sqrt(E), by exact comparison of squares: |m - sqrt(E)| minimal
    best = None
    for m in range(1, E + 2):
        # distance to sqrt(E) compared through (2m - 1)^2 < 4E <= (2m + 1)^2  <=>  m - 1/2 < sqrt(E) <= m + 1/2
        if (2 * m - 1) ** 2 < 4 * E <= (2 * m + 1) ** 2:
            best = m
            break
    assert best is not None
    return best, -(-E // best)


def place(ideal, M: int, N: int):
    E = len(ideal)
    assert M * N >= E
    free = {(m, n) for m in range(M) for n in range(N)}
    phi = []
    for k in range(E):
        am = min(max(int(ideal[k][0]), 0), M - 1)
        an = min(max(int(ideal[k][1]), 0), N - 1)
        cell = min(free, key=lambda c: (max(abs(c[0] - am), abs(c[1] - an)), c[0], c[1]))
        free.remove(cell)
        phi.append(cell)
    return phi
