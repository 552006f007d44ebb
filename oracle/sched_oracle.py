"""Reference for the work-item list of the persistent kernels (test infrastructure only; shares
nothing with the HIP path).

The cost of a sequence is quadratic in its length (paper Sec. 2.1, packing paragraph: the sum of
S_i^2; App. C.2: the quadratic term of T(l, P)).  Split into tiles of `tile` rows, sequence s of
length L_s has n_s = ceil(L_s / tile) tiles, and its tile number c (1 <= c <= n_s, counted so that
tile c has c tiles of causal work) costs c units: a ramp 1..n_s.  Longest-processing-time-first
list scheduling hands the items out in order of decreasing cost, so the list is: every (s, c)
exactly once, by decreasing c; the order among equal c is free.
"""


def items(lengths, tile):
    """All (sequence, level) items by decreasing level; equal levels by sequence index."""
    out = []
    for s, L in enumerate(lengths):
        n = -(-int(L) // tile)
        for c in range(1, n + 1):
            out.append((s, c))
    out.sort(key=lambda it: (-it[1], it[0]))
    return out


def records(lengths, tile):
    """The items with the sequence's first packed row and length: (s, c, row0, L)."""
    row0, acc = [], 0
    for L in lengths:
        row0.append(acc)
        acc += int(L)
    return [(s, c, row0[s], int(lengths[s])) for s, c in items(lengths, tile)]


def total_cost(lengths, tile):
    """Sum of the item costs = sum_s n_s (n_s + 1) / 2: the number of (query tile, key tile) pairs
    on or below the diagonal."""
    return sum(c for _, c in items(lengths, tile))
