"""Identities the kernels rest on, checked on the CPU by brute force.

Nothing here calls the library or the oracle.  The rank formula and the exchange + bitonic
rounds of the kernels for more than 169 rows are statements about sorted sequences, tried on
every 0/1 input of small sizes (comparator networks and min/max formulas that are right on all
0/1 inputs are right on all inputs) and on random integers with many ties at the sizes the
kernels use.  The single pass's rule for the copy that feeds the median, and the condition
under which its output stands, are modelled on small vectors.
"""
import itertools

import numpy as np
import pytest


def rank_from_halves(A, B):
    """Rank H-1 (0-based) of the union of two ascending sequences of H values each."""
    H = len(A)
    best = min(A[H - 1], B[H - 1])
    for m in range(H - 1):
        best = min(best, max(A[m], B[H - 2 - m]))
    return best


@pytest.mark.parametrize("H", [1, 2, 3, 4, 5, 6, 7])
def test_rank_of_two_sorted_halves_all_zero_one_inputs(H):
    for bits in itertools.product((0, 1), repeat=2 * H):
        A, B = sorted(bits[:H]), sorted(bits[H:])
        assert rank_from_halves(A, B) == sorted(bits)[H - 1], bits


@pytest.mark.parametrize("H", [96, 112, 128])
def test_rank_of_two_sorted_halves_with_spare_wires(H):
    # f values on 2H wires: the spare wires at the end, H-1-(f-1)/2 of them smallest, the rest
    # largest, put the median of the f values at rank H-1
    rng = np.random.default_rng(H)
    for f in (H + 1, H + 2, 2 * H - 3, 2 * H - 1):
        if f % 2 == 0:
            f += 1
        for _ in range(200):
            v = rng.integers(1, 9, size=f).tolist()
            low = H - 1 - (f - 1) // 2
            wires = v + [0] * low + [10 ** 6] * (2 * H - f - low)
            A, B = sorted(wires[:H]), sorted(wires[H:])
            assert rank_from_halves(A, B) == sorted(v)[(f - 1) // 2], (H, f)


def bitonic_rounds(k):
    P = len(k)
    apart = P // 2
    while apart >= 1:
        for i in range(P):
            if (i & apart) == 0 and k[i] > k[i + apart]:
                k[i], k[i + apart] = k[i + apart], k[i]
        apart //= 2
    return k


def split_and_sort(A, B, P):
    """What the two waves do after sorting their halves A and B of H values: minima and maxima of
    A[m] against B[H-1-m], each padded to P wires and run through the bitonic rounds."""
    H = len(A)
    lo = [min(A[m], B[H - 1 - m]) for m in range(H)]          # rises, then falls
    hi = [0] * H
    for m in range(H):
        hi[H - 1 - m] = max(A[m], B[H - 1 - m])               # falls, then rises
    lo_sorted = bitonic_rounds([-1] * (P - H) + lo)[P - H:]    # smallest key in front
    hi_sorted = bitonic_rounds(hi + [10 ** 9] * (P - H))[:H]   # largest key behind
    return lo_sorted + hi_sorted


@pytest.mark.parametrize("H,P", [(1, 1), (2, 2), (3, 4), (4, 4), (5, 8), (6, 8), (7, 8), (8, 8)])
def test_exchange_and_bitonic_rounds_sort_all_zero_one_inputs(H, P):
    for bits in itertools.product((0, 1), repeat=2 * H):
        A, B = sorted(bits[:H]), sorted(bits[H:])
        assert split_and_sort(A, B, P) == sorted(bits), bits


@pytest.mark.parametrize("H", [96, 112, 128])
def test_exchange_and_bitonic_rounds_sort_at_the_kernels_sizes(H):
    rng = np.random.default_rng(1000 + H)
    for _ in range(60):
        v = rng.integers(0, 12, size=2 * H).tolist()
        assert split_and_sort(sorted(v[:H]), sorted(v[H:]), 128) == sorted(v)


def _single_pass_model(copies, wave):
    """The single pass's choice of the copy that feeds the median, modelled on small vectors:
    per stretch of `wave` coordinates the first copy of the largest class of copies identical on
    that stretch feeds; `differs[b]` says whether some stretch fed a copy that differed from copy
    b there.  -> (fed vector, differs, winner by plurality with the lowest index on ties)."""
    r, n = copies.shape
    fed = np.zeros(n, dtype=copies.dtype)
    differs = [False] * r
    for c0 in range(0, n, wave):
        seg = copies[:, c0:c0 + wave]
        same = [[bool((seg[a] == seg[b]).all()) for b in range(r)] for a in range(r)]
        sizes = [sum(row) for row in same]
        pick = sizes.index(max(sizes))
        fed[c0:c0 + wave] = seg[pick]
        for b in range(r):
            differs[b] = differs[b] or not same[pick][b]
    same_all = [[bool((copies[a] == copies[b]).all()) for b in range(r)] for a in range(r)]
    counts = [sum(row) for row in same_all]
    winner = counts.index(max(counts))
    return fed, differs, winner, counts[winner]


@pytest.mark.parametrize("r", [3, 5, 7])
def test_wave_local_choice_feeds_the_winner_or_says_so(r):
    # (1) if no stretch fed a copy that differed from the winner there, the fed vector is the
    # winner's; (2) a winner with a strict majority of the copies is never differed from
    rng = np.random.default_rng(r)
    stood = redone = 0
    for _ in range(6000):
        n, wave = 12, 4
        n_kinds = int(rng.integers(1, r + 1))
        kinds = rng.integers(0, 2, size=(n_kinds, n))
        # kinds that agree on most stretches: start from one vector, change a few words
        kinds[1:] = kinds[0]
        for k in range(1, n_kinds):
            for c in rng.integers(0, n, size=int(rng.integers(1, 3))):
                kinds[k, c] = rng.integers(2, 5)
        copies = kinds[rng.integers(0, n_kinds, size=r)]
        fed, differs, winner, count = _single_pass_model(copies, wave)
        if not differs[winner]:
            assert (fed == copies[winner]).all()
            stood += 1
        else:
            redone += 1
        if 2 * count > r:
            assert not differs[winner]
    assert stood > 0 and redone > 0
