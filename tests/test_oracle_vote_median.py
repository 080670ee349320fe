"""Pins for the oracle's majority vote (Eq. 3) and coordinate-wise median (Sec. 2, Sec. 6.1)."""
import itertools
import struct

import numpy as np
import pytest

from oracle import byz_oracle as O
from oracle import c_oracle as C

IMPLS = [("numpy", O.vote, O.median), ("c", C.vote, lambda X, ri, d: C.median(X, ri, d, threads=2))]


def _set_partitions(n):
    """All partitions of {0..n-1} as label lists in restricted-growth form."""
    def rec(prefix, mx):
        if len(prefix) == n:
            yield list(prefix)
            return
        for lab in range(mx + 2):
            yield from rec(prefix + [lab], max(mx, lab))
    yield from rec([0], 0)


def _definition_winner(labels):
    """Most frequent label; among equally frequent ones the one containing the lowest index."""
    best_a, best_c = None, -1
    for a in range(len(labels)):
        c = labels.count(labels[a])
        if c > best_c:
            best_a, best_c = a, c
    return best_a


@pytest.mark.parametrize("name,vote,median", IMPLS)
@pytest.mark.parametrize("r", [3, 5])
def test_vote_every_equality_pattern(name, vote, median, r):
    # 5 patterns for r = 3 (Bell number), 52 for r = 5
    parts = list(_set_partitions(r))
    assert len(parts) == {3: 5, 5: 52}[r]
    rng = np.random.default_rng(11)
    d = 37
    for where in ["everywhere", "last", "first"]:
        base = rng.standard_normal((r + 1, d)).astype(np.float32)
        X = np.zeros((len(parts) * r, d), dtype=np.float32)
        rows = np.arange(len(parts) * r, dtype=np.int32).reshape(len(parts), r)
        for j, labels in enumerate(parts):
            for k, lab in enumerate(labels):
                v = base[0].copy()
                if where == "everywhere":
                    v = base[lab].copy()
                elif where == "last":
                    v[d - 1] = np.float32(lab)  # copies differ only in the last coordinate
                else:
                    v[0] = np.float32(lab)
                X[rows[j, k]] = v
        wrep, wrow, neq = vote(X, rows, d)
        pairs = O.pair_index(r)
        for j, labels in enumerate(parts):
            a = _definition_winner(labels)
            assert wrep[j] == a and wrow[j] == rows[j, a]
            want = sum(1 << p for p, (x, y) in enumerate(pairs) if labels[x] != labels[y])
            assert neq[j] == want


@pytest.mark.parametrize("name,vote,median", IMPLS)
def test_vote_is_bitwise(name, vote, median):
    # +0 and -0 are different copies; NaNs with the same payload are the same copy
    d = 8
    X = np.zeros((6, d), dtype=np.float32)
    X[1, 3] = -0.0
    X[2, 3] = -0.0
    nan_a = np.array([0x7FC00001], dtype=np.uint32).view(np.float32)[0]
    nan_b = np.array([0x7FC00002], dtype=np.uint32).view(np.float32)[0]
    X[3, 5] = nan_a
    X[4, 5] = nan_a
    X[5, 5] = nan_b
    rows = np.array([[0, 1, 2], [3, 4, 5]], dtype=np.int32)
    wrep, wrow, neq = vote(X, rows, d)
    assert wrep.tolist() == [1, 0] and neq.tolist() == [0b011, 0b110]
    # only the first d words are compared: padding beyond d is ignored
    X2 = np.zeros((3, d + 4), dtype=np.float32)
    X2[:, d:] = np.arange(12, dtype=np.float32).reshape(3, 4)
    wrep, _, neq = vote(X2, np.array([[0, 1, 2]], dtype=np.int32), d)
    assert wrep.tolist() == [0] and neq.tolist() == [0]


def _honest_and_attacked(H, S, d, seed, attack):
    K, f, l, r = O.dims(H)
    rng = np.random.default_rng(seed)
    g = (0.01 * rng.standard_normal((f, d))).astype(np.float32)
    rows = O.file_rows(H)
    fw = O.file_workers(H)
    X = np.zeros((K * l, d), dtype=np.float32)
    for j in range(f):
        for k in range(r):
            X[rows[j, k]] = attack(g[j]) if int(fw[j, k]) in S else g[j]
    return g, X, rows


@pytest.mark.parametrize("name,vote,median", IMPLS)
def test_vote_all_honest_and_below_threshold(name, vote, median):
    # Sec. 2 / Sec. 5.3.1: with fewer than r' Byzantine copies per file nothing is distorted
    H = O.mols_biadjacency(5, 3)
    d = 50
    for S in [(), (4,), (7,)]:
        g, X, rows = _honest_and_attacked(H, set(S), d, 3, lambda v: -100.0 * v)
        wrep, wrow, _ = vote(X, rows, d)
        for j in range(25):
            assert np.array_equal(X[wrow[j]], g[j])
        out = median(X, wrow, d)
        assert np.array_equal(out, np.median(g, axis=0))


@pytest.mark.parametrize("name,vote,median", IMPLS)
@pytest.mark.parametrize("scheme,a,b,q,cmax", [("mols", 5, 3, 3, 3), ("mols", 5, 3, 4, 5),
                                               ("ram", 5, 5, 6, 4)])
def test_vote_distorts_exactly_cmax_files(name, vote, median, scheme, a, b, q, cmax):
    # Sec. 2: a file is distorted iff at least r' of its copies are Byzantine; for the
    # worst-case set the number of such files is the c_max the paper's tables print.
    H = O.mols_biadjacency(a, b) if scheme == "mols" else O.ramanujan_biadjacency(a, b)
    c, S = C.worst_case(H, q)
    assert c == cmax
    d = 40
    g, X, rows = _honest_and_attacked(H, set(S), d, 5, lambda v: -100.0 * v)
    wrep, wrow, _ = vote(X, rows, d)
    wrong = [j for j in range(H.shape[1]) if not np.array_equal(X[wrow[j]], g[j])]
    assert wrong == O.distorted_files(H, S).tolist() and len(wrong) == cmax


def _total_order_rank(u):
    """IEEE totalOrder written independently: sign-magnitude value of the bit pattern."""
    sign = u >> 31
    mag = u & 0x7FFFFFFF
    return -(mag + 1) if sign else mag


def test_order_key_special_values():
    words = [0xFFC00000, 0xFF800000, 0xC0000000, 0xBF800000, 0x80000001, 0x80000000,
             0x00000000, 0x00000001, 0x3F800000, 0x40000000, 0x7F800000, 0x7FC00000]
    keys = O.order_key(np.array(words, dtype=np.uint32)).tolist()
    assert keys == sorted(keys) and len(set(keys)) == len(keys)  # listed in ascending order
    rng = np.random.default_rng(0)
    u = rng.integers(0, 2**32, size=5000, dtype=np.uint64).astype(np.uint32)
    k = O.order_key(u)
    ranks = np.array([_total_order_rank(int(x)) for x in u])
    assert np.array_equal(np.argsort(k, kind="stable"), np.argsort(ranks, kind="stable"))


@pytest.mark.parametrize("name,vote,median", IMPLS)
@pytest.mark.parametrize("f", [1, 3, 9, 25, 49])
def test_median_matches_numpy_on_ordinary_data(name, vote, median, f):
    rng = np.random.default_rng(f)
    d = 301
    X = rng.standard_normal((f + 3, d)).astype(np.float32)
    X[:, :7] = np.round(X[:, :7])  # repeated values
    X[X == 0] = 0.0  # no negative zeros in this test
    idx = rng.permutation(f + 3)[:f].astype(np.int32)
    out = median(X, idx, d)
    assert np.array_equal(out, np.median(X[idx], axis=0))
    assert np.array_equal(out, np.sort(X[idx], axis=0)[(f - 1) // 2])
    # invariant under permuting the files, and the median of identical vectors is that vector
    assert np.array_equal(median(X, idx[::-1].copy(), d), out)
    same = np.full(f, idx[0], dtype=np.int32)
    assert np.array_equal(median(X, same, d), X[idx[0]])


@pytest.mark.parametrize("name,vote,median", IMPLS)
def test_median_bruteforce_small_alphabet(name, vote, median):
    # every vector over a 3-letter alphabet (incl. -0/+0 and a NaN) for f = 5: rank-2 element
    letters = np.array([0x80000000, 0x00000000, 0x7FC00000], dtype=np.uint32)  # -0 < +0 < NaN
    combos = list(itertools.product(range(3), repeat=5))
    X = np.zeros((5, len(combos)), dtype=np.uint32)
    for c, combo in enumerate(combos):
        X[:, c] = letters[list(combo)]
    out = median(X.view(np.float32), np.arange(5, dtype=np.int32), len(combos)).view(np.uint32)
    for c, combo in enumerate(combos):
        assert out[c] == letters[sorted(combo)[2]]


@pytest.mark.parametrize("name,vote,median", IMPLS)
def test_median_counting_definition_random_bits(name, vote, median):
    # rank definition checked by counting, on raw random bit patterns (NaNs, infs, denormals)
    rng = np.random.default_rng(5)
    f, d = 25, 400
    U = rng.integers(0, 2**32, size=(f, d), dtype=np.uint64).astype(np.uint32)
    out = median(U.view(np.float32), np.arange(f, dtype=np.int32), d).view(np.uint32)
    for c in range(d):
        col = [_total_order_rank(int(x)) for x in U[:, c]]
        m = _total_order_rank(int(out[c]))
        assert int(out[c]) in [int(x) for x in U[:, c]]
        assert sum(1 for x in col if x < m) <= (f - 1) // 2
        assert sum(1 for x in col if x > m) <= (f - 1) // 2


@pytest.mark.parametrize("name,vote,median", IMPLS)
def test_median_stays_within_honest_range(name, vote, median):
    # with fewer than (f+1)/2 distorted winners the median lies between honest values
    rng = np.random.default_rng(9)
    f, d, bad = 25, 200, 12
    X = rng.standard_normal((f, d)).astype(np.float32)
    X[:bad // 2] = 1e6
    X[bad // 2:bad] = -1e6
    out = median(X, np.arange(f, dtype=np.int32), d)
    assert (out >= X[bad:].min(axis=0)).all() and (out <= X[bad:].max(axis=0)).all()


def test_aggregate_numpy_vs_c():
    H = O.ramanujan_biadjacency(5, 5)
    _, S = C.worst_case(H, 6)
    g, X, rows = _honest_and_attacked(H, set(S), 333, 2, lambda v: np.full_like(v, 1e3))
    out_py, w_py = O.aggregate(X, rows, 333)
    out_c, w_c, threads = C.aggregate(X, rows, 333, threads=3)
    assert threads == 3
    assert np.array_equal(out_py.view(np.uint32), out_c.view(np.uint32))
    assert np.array_equal(w_py, w_c)


def test_struct_roundtrip_sanity():
    # the fixtures above build floats from bit patterns; make sure the view does what we think
    assert struct.unpack("<I", struct.pack("<f", -0.0))[0] == 0x80000000


TM_IMPLS = [("numpy", O.trimmed_mean), ("c", lambda X, ri, d, b: C.trimmed_mean(X, ri, d, b, threads=2))]


@pytest.mark.parametrize("name,tmean", TM_IMPLS)
def test_trimmed_mean_against_scipy_mean_and_median(name, tmean):
    from scipy import stats
    rng = np.random.default_rng(21)
    for f in (5, 9, 25, 49):
        d = 173
        X = rng.standard_normal((f + 2, d)).astype(np.float32)
        X[:, :5] = np.round(X[:, :5])
        idx = rng.permutation(f + 2)[:f].astype(np.int32)
        V = X[idx].astype(np.float64)
        # b = 0: the mean; b = (f-1)/2: the median
        assert np.allclose(tmean(X, idx, d, 0), V.mean(axis=0), rtol=0, atol=1e-14)
        assert np.array_equal(tmean(X, idx, d, (f - 1) // 2), np.median(V, axis=0))
        for b in range(1, (f - 1) // 2):
            want = stats.trim_mean(V, b / f + 1e-9, axis=0)  # cuts int(f * proportion) = b per side
            assert np.allclose(tmean(X, idx, d, b), want, rtol=0, atol=1e-14), (f, b)
        # permuting the files changes nothing
        assert np.array_equal(tmean(X, idx[::-1].copy(), d, 2), tmean(X, idx, d, 2))


@pytest.mark.parametrize("name,tmean", TM_IMPLS)
def test_trimmed_mean_hand_worked_and_outliers(name, tmean):
    # one coordinate, values 1..7 shuffled, b = 2: mean of {3,4,5} = 4; with -inf/NaN/+inf
    # among them the extremes are what gets cut (total order puts NaN beyond the infinities)
    X = np.array([[5], [1], [7], [3], [2], [6], [4]], dtype=np.float32)
    idx = np.arange(7, dtype=np.int32)
    assert tmean(X, idx, 1, 2)[0] == 4.0
    assert tmean(X, idx, 1, 1)[0] == 4.0 and tmean(X, idx, 1, 0)[0] == 4.0
    Y = np.array([[5], [np.nan], [np.inf], [3], [-np.inf], [6], [4]], dtype=np.float32)
    assert tmean(Y, idx, 1, 2)[0] == (4.0 + 5.0 + 6.0) / 3  # cut: -inf, 3 | inf, nan
    # up to b huge outliers per side leave the result inside the honest range
    rng = np.random.default_rng(3)
    f, d, b = 25, 64, 4
    Z = rng.standard_normal((f, d)).astype(np.float32)
    Z[:b] = 1e9
    Z[b:2 * b] = -1e9
    out = tmean(Z, np.arange(f, dtype=np.int32), d, b)
    assert (out >= Z[2 * b:].min(axis=0)).all() and (out <= Z[2 * b:].max(axis=0)).all()


def test_multi_krum_hand_worked_and_invariants():
    from scipy.spatial.distance import cdist
    # five points on a line: 0, 1, 2, 3, 100; c = 1 -> each score sums the f-c-2 = 2 nearest
    X = np.array([[0.0], [1.0], [2.0], [3.0], [100.0]], dtype=np.float32)
    idx = np.arange(5, dtype=np.int32)
    mean, sel, scores, dist = O.multi_krum(X, idx, 1, c=1, m=4)
    assert scores.tolist() == [1 + 4, 1 + 1, 1 + 1, 1 + 4, 97 ** 2 + 98 ** 2]
    assert sel.tolist() == [1, 1, 1, 1, 0] and mean[0] == 1.5
    # Krum (m = 1): lowest score, lower index on the tie between points 1 and 2
    mean, sel, _, _ = O.multi_krum(X, idx, 1, c=1, m=1)
    assert sel.tolist() == [0, 1, 0, 0, 0] and mean[0] == 1.0
    # distances equal an independent library routine; selection excludes far outliers
    rng = np.random.default_rng(8)
    f, d, c = 25, 300, 5
    V = (0.01 * rng.standard_normal((f, d))).astype(np.float32)
    bad = [2, 7, 11, 19, 24]
    V[bad] = 1e3
    mean, sel, scores, dist = O.multi_krum(V, np.arange(f, dtype=np.int32), d, c=c, m=f - c)
    assert np.allclose(dist, cdist(V.astype(np.float64), V.astype(np.float64), "sqeuclidean"),
                       rtol=1e-12, atol=0)
    assert [i for i in range(f) if sel[i] == 0] == bad
    good = [i for i in range(f) if i not in bad]
    assert np.allclose(mean, V[good].astype(np.float64).mean(axis=0), rtol=1e-12, atol=1e-18)
    # all vectors identical: every score is zero, the first m are selected, the mean is the vector
    W_ = np.tile(V[:1], (7, 1))
    mean, sel, scores, _ = O.multi_krum(W_, np.arange(7, dtype=np.int32), d, c=2, m=5)
    assert (scores == 0).all() and sel.tolist() == [1, 1, 1, 1, 1, 0, 0]
    assert np.array_equal(mean, V[0].astype(np.float64))
    with pytest.raises(AssertionError):
        O.multi_krum(V, np.arange(6, dtype=np.int32), d, c=2, m=1)  # needs f >= 2c + 3


def test_mean_around_median_against_brute_force_and_by_hand():
    # by hand: values 1 2 3 10 20 (median 3): the 3 closest are {1,2,3} (distances 2,1,0 < 7)
    m, lo, hi = O.mean_around_median([10, 1, 3, 20, 2], 3)
    assert (m, lo, hi) == (2.0, 0, 2)
    # beta = 1: the median itself; beta = n: the plain mean
    assert O.mean_around_median([10, 1, 3, 20, 2], 1)[0] == 3.0
    assert O.mean_around_median([10, 1, 3, 20, 2], 5)[0] == 36.0 / 5
    # tie between a lower and an upper neighbour at the same distance: the lower one is taken
    assert O.mean_around_median([1, 2, 3, 4, 5], 2)[0] == 2.5
    assert O.mean_around_median([1, 2, 3, 4, 5], 4)[0] == 2.5   # {3,2,4,1}
    # brute force: among all subsets of size beta that contain the median element, the chosen
    # window has the smallest sum of distances to the median (unique when the distances differ)
    rng = np.random.default_rng(4)
    for n in (3, 5, 7, 9, 11):
        for _ in range(20):
            v = rng.standard_normal(n).astype(np.float32)
            med = np.median(v)
            dist = np.abs(v.astype(np.float64) - float(med))
            for beta in range(1, n + 1):
                got, lo, hi = O.mean_around_median(v, beta)
                best = min(itertools.combinations(range(n), beta),
                           key=lambda S: sum(dist[i] for i in S))
                assert got == pytest.approx(float(np.mean(v[list(best)].astype(np.float64))), abs=1e-12)
                assert hi - lo + 1 == beta
    # special values: the infinities are the farthest, NaNs sort beyond them
    m, lo, hi = O.mean_around_median([np.inf, 1, 2, 3, -np.inf, 4, np.nan], 3)
    # sorted: -inf 1 2 3 4 inf nan, median 3 -> window {2,3,4}
    assert (m, lo, hi) == (3.0, 2, 4)


def test_bulyan_selection_and_whole_rule():
    from scipy.spatial.distance import cdist
    # points on a line 0 1 2 3 4 5 100, c = 1: theta = 5 picks, beta = 3
    X = np.array([[0.0], [1.0], [2.0], [3.0], [4.0], [5.0], [100.0]], dtype=np.float32)
    idx = np.arange(7, dtype=np.int32)
    out, chosen, dist = O.bulyan(X, idx, 1, 1)
    # Krum pass 1 (n'=7, 4 nearest): scores 0:1+4+9+16=30, 1:1+1+4+9=15, 2:1+1+4+4=10, 3:10, 4:15,
    #   5:30 -> point 2 (tie with 3: lower index); pass 2 on {0,1,3,4,5,100} (3 nearest):
    #   0:1+9+16=26, 1:1+4+9=14, 3:1+4+4=9, 4:1+1+9=11, 5:1+4+16=21 -> 3; pass 3 on
    #   {0,1,4,5,100} (2 nearest): 0:1+16=17, 1:1+9=10, 4:1+9=10, 5:1+16=17 -> 1; pass 4 on
    #   {0,4,5,100} (1 nearest): 0:16, 4:1, 5:1 -> 4; pass 5 on {0,5,100} (0 terms) -> 0
    assert chosen == [2, 3, 1, 4, 0]
    # chosen values 0 1 2 3 4, median 2, the 3 closest: {1,2,3}
    assert out[0] == 2.0
    # the first pick is Krum's pick (same score rule on the full set), distances as cdist
    rng = np.random.default_rng(12)
    f, d, c = 23, 40, 5
    V = rng.standard_normal((f, d)).astype(np.float32) * rng.uniform(0.5, 2.0, size=(f, 1)).astype(np.float32)
    bad = [0, 5, 9, 17, 22]
    V[bad] = 50.0 * rng.standard_normal((len(bad), d)).astype(np.float32)  # far from all, also from each other
    out, chosen, dist = O.bulyan(V, np.arange(f, dtype=np.int32), d, c)
    assert np.allclose(dist, cdist(V.astype(np.float64), V.astype(np.float64), "sqeuclidean"),
                       rtol=1e-12, atol=0)
    _, sel1, _, _ = O.multi_krum(V, np.arange(f, dtype=np.int32), d, c=c, m=1)
    assert chosen[0] == int(np.argmax(sel1))
    assert len(chosen) == f - 2 * c and len(set(chosen)) == len(chosen)
    assert not set(chosen) & set(bad)                      # far outliers are never chosen
    good = [i for i in range(f) if i not in bad]
    assert (out >= V[good].min(axis=0)).all() and (out <= V[good].max(axis=0)).all()
    # colluding outliers (c identical far vectors) do get chosen in the last rounds, where a
    # score has at most c - 1 terms and theirs is zero; the per-coordinate phase removes them
    U = V.copy()
    U[bad] = 50.0
    outu, chosenu, _ = O.bulyan(U, np.arange(f, dtype=np.int32), d, c)
    assert 1 <= len(set(chosenu) & set(bad)) <= c and set(chosenu[:f - 3 * c]).isdisjoint(bad)
    assert (outu >= U[good].min(axis=0)).all() and (outu <= U[good].max(axis=0)).all()
    # c = 0: every vector is chosen and every coordinate is the plain mean
    out0, chosen0, _ = O.bulyan(V, np.arange(f, dtype=np.int32), d, 0)
    assert sorted(chosen0) == list(range(f))
    assert np.allclose(out0, V.astype(np.float64).mean(axis=0), rtol=0, atol=1e-12)
    # identical vectors: lowest indices first, the output is the vector
    W_ = np.tile(V[1:2], (11, 1))
    outi, choseni, _ = O.bulyan(W_, np.arange(11, dtype=np.int32), d, 2)
    assert choseni == list(range(7)) and np.array_equal(outi, V[1].astype(np.float64))
    # even with c Byzantine vectors chosen, the 2c trimmed per coordinate keep the output inside
    # the honest range: place the Byzantine vectors close enough to be chosen
    Z = rng.standard_normal((f, d)).astype(np.float32)
    Z[bad] = Z[good].mean(axis=0) + 3.0 * np.sign(rng.standard_normal(d)).astype(np.float32)
    outz, chosenz, _ = O.bulyan(Z, np.arange(f, dtype=np.int32), d, c)
    assert (outz >= Z[good].min(axis=0)).all() and (outz <= Z[good].max(axis=0)).all()
    with pytest.raises(AssertionError):
        O.bulyan(V, np.arange(22, dtype=np.int32), d, 5)    # needs f >= 4c + 3


def test_c_oracle_bulyan_equals_the_definition():
    # the plain-C oracle (used at full sizes) against the NumPy one on the hand-worked line,
    # on random data with colluding and with scattered outliers, signed zeros and ties
    X = np.array([[0.0], [1.0], [2.0], [3.0], [4.0], [5.0], [100.0]], dtype=np.float32)
    out, chosen, _ = C.bulyan(X, np.arange(7, dtype=np.int32), 1, 1)
    assert chosen == [2, 3, 1, 4, 0] and out[0] == 2.0
    rng = np.random.default_rng(21)
    for f, c, d in [(7, 1, 33), (11, 2, 50), (23, 5, 64), (25, 5, 40), (25, 3, 40), (9, 0, 20)]:
        V = np.zeros((f + 3, d + 5), dtype=np.float32)
        V[:, :d] = rng.standard_normal((f + 3, d)) * rng.uniform(0.5, 2.0, size=(f + 3, 1))
        idx = rng.permutation(f + 3)[:f].astype(np.int32)
        for kind in ("collude", "scatter", "none"):
            W_ = V.copy()
            if kind == "collude":
                W_[idx[:c], :d] = 30.0
            elif kind == "scatter":
                W_[idx[:c], :d] = 30.0 * rng.standard_normal((c, d))
            # signed zeros and exact ties (non-finite values make the distances of the first
            # phase NaN, for which the rule says nothing: not exercised)
            W_[idx[-1], 0] = -0.0
            W_[idx[-2], 0] = 0.0
            W_[idx[-3], 2] = W_[idx[-1], 2]
            out_p, chosen_p, dist_p = O.bulyan(W_, idx, d, c)
            out_c, chosen_c, dist_c = C.bulyan(W_, idx, d, c)
            finite = np.isfinite(dist_p)
            assert np.array_equal(finite, np.isfinite(dist_c))
            assert np.allclose(dist_c[finite], dist_p[finite], rtol=1e-12, atol=0)
            assert chosen_c == chosen_p, (f, c, kind)
            assert np.array_equal(np.isnan(out_c), np.isnan(out_p))
            ok = ~np.isnan(out_p)
            assert np.allclose(out_c[ok], out_p[ok], rtol=0, atol=1e-12), (f, c, kind)


def test_c_oracle_mean_around_median_equals_the_definition_on_special_values():
    # phase 2 alone, including infinities, NaNs, signed zeros and many ties
    rng = np.random.default_rng(33)
    d, n = 400, 17
    U = rng.standard_normal((n + 2, d)).astype(np.float32)
    special = np.array([np.inf, -np.inf, np.nan, 0.0, -0.0, 1.0, 1.0, -1.0], dtype=np.float32)
    mask = rng.random((n + 2, d)) < 0.3
    U[mask] = special[rng.integers(0, len(special), size=int(mask.sum()))]
    row_index = rng.permutation(n + 2).astype(np.int32)
    for theta, beta in [(17, 1), (17, 5), (17, 17), (9, 4), (3, 2), (1, 1)]:
        chosen = rng.permutation(n)[:theta].astype(np.int32)
        got = C.mean_around_median(U, row_index, chosen, d, beta)
        for t in range(d):
            want = O.mean_around_median(U[row_index[chosen], t], beta)[0]
            assert (np.isnan(got[t]) and np.isnan(want)) or got[t] == pytest.approx(want, abs=1e-12), (theta, beta, t)


TOL_VOTES = [("numpy", O.vote_tolerant), ("c", C.vote_tolerant)]


@pytest.mark.parametrize("name,tvote", TOL_VOTES)
def test_tolerant_vote_closeness_is_isclose_both_ways(name, tvote):
    # |a-b| <= atol + rtol*max(|a|,|b|)  <=>  isclose(a, b) or isclose(b, a) (numpy's test uses
    # |b| alone); identical bit patterns (same-sign infinities, equal NaNs) are close as well
    rng = np.random.default_rng(5)
    d = 64
    for atol, rtol in [(1e-6, 0.0), (0.0, 1e-5), (1e-7, 1e-6), (0.0, 0.0)]:
        for trial in range(40):
            a = rng.standard_normal(d).astype(np.float32)
            b = a + (rng.standard_normal(d) * rng.choice([0.0, 1e-7, 1e-6, 1e-3])).astype(np.float32)
            if trial % 5 == 0:
                a[3] = b[3] = np.inf
                a[4] = b[4] = np.nan
            if trial % 7 == 0:
                a[5], b[5] = 0.0, -0.0
            X = np.stack([a, b, a]).astype(np.float32)
            rows = np.array([[0, 1, 2]], dtype=np.int32)
            _, _, far = tvote(X, rows, d, atol, rtol)
            with np.errstate(invalid="ignore"):
                close = (np.isclose(a, b, rtol=rtol, atol=atol) | np.isclose(b, a, rtol=rtol, atol=atol)
                         | (a.view(np.uint32) == b.view(np.uint32)))
            want_far_01 = not close.all()
            assert bool(far[0] & 1) == want_far_01          # pair (0,1)
            assert not (far[0] & 2)                          # pair (0,2): identical copies
            assert bool(far[0] & 4) == want_far_01          # pair (1,2)


@pytest.mark.parametrize("name,tvote", TOL_VOTES)
def test_tolerant_vote_hand_worked_and_limits(name, tvote):
    one = np.ones((1, 8), dtype=np.float32)
    # a chain: 0, 0.9, 1.8 with atol = 1: a~b, b~c, a!~c -> counts 2, 3, 2 -> replica 1 wins
    X = np.concatenate([0.0 * one, 0.9 * one, 1.8 * one])
    rows = np.array([[0, 1, 2]], dtype=np.int32)
    wrep, wrow, far = tvote(X, rows, 8, 1.0, 0.0)
    assert (wrep[0], wrow[0], far[0]) == (1, 1, 0b010)      # only pair (0,2) is far
    # two close copies against one far copy: lower replica of the close pair
    X = np.concatenate([5.0 * one, 1.0 * one, (1.0 + 1e-6) * one]).astype(np.float32)
    wrep, _, far = tvote(X, rows, 8, 1e-5, 0.0)
    assert (wrep[0], far[0]) == (1, 0b011)
    # nothing close: replica 0
    wrep, _, far = tvote(X, rows, 8, 1e-9, 0.0)
    assert (wrep[0], far[0]) == (0, 0b111)
    # one coordinate out of tolerance is enough to be far
    Y = np.concatenate([one, one, one]).astype(np.float32)
    Y[2, 7] = 1.5
    wrep, _, far = tvote(Y, rows, 8, 1e-3, 1e-3)
    assert (wrep[0], far[0]) == (0, 0b110)
    # zero tolerance: the exact vote, except that +0 and -0 (equal as numbers) count as close
    rng = np.random.default_rng(6)
    H = O.mols_biadjacency(5, 3)
    rows5 = O.file_rows(H)
    G = rng.standard_normal((25, 50)).astype(np.float32)
    Xc = np.zeros((75, 50), dtype=np.float32)
    for j in range(25):
        for k in range(3):
            Xc[rows5[j, k]] = G[j]
    for j in (2, 9, 17):
        Xc[rows5[j, 1]] *= 2.0
    Xc[rows5[4, 0]], Xc[rows5[4, 2]] = 1.0, 7.0
    want = O.vote(Xc, rows5, 50)
    got = tvote(Xc, rows5, 50, 0.0, 0.0)
    for a, b in zip(want, got):
        assert np.array_equal(a, b)
    Xz = Xc.copy()
    Xz[rows5[0, 0], 0], Xz[rows5[0, 1], 0], Xz[rows5[0, 2], 0] = 0.0, -0.0, 0.0
    assert O.vote(Xz, rows5, 50)[2][0] == 0b101 and tvote(Xz, rows5, 50, 0.0, 0.0)[2][0] == 0


@pytest.mark.parametrize("name,tvote", TOL_VOTES)
def test_tolerant_vote_majority_property_under_rounding_noise(name, tvote):
    # Sec. 2: a file is distorted iff at least r' of its copies are Byzantine -- still true when
    # the honest copies differ by rounding noise below the tolerance and the Byzantine copies
    # are far (and, colluding, close to each other)
    rng = np.random.default_rng(7)
    H = O.ramanujan_biadjacency(5, 5)
    K, f, l, r = O.dims(H)
    rows = O.file_rows(H)
    fw = O.file_workers(H)
    d = 40
    G = rng.standard_normal((f, d)).astype(np.float32)
    byz = {0, 1, 5, 7, 14, 20}
    X = np.zeros((K * l, d), dtype=np.float32)
    for j in range(f):
        for k in range(r):
            if int(fw[j, k]) in byz:
                X[rows[j, k]] = -100.0 * G[j] * np.float32(1.0 + 1e-7 * k)
            else:
                X[rows[j, k]] = G[j] * (1.0 + 3e-7 * rng.standard_normal(d)).astype(np.float32)
    wrep, wrow, far = tvote(X, rows, d, 1e-6, 1e-5)
    exact_wrep, _, exact_neq = O.vote(X, rows, d)
    assert (exact_neq != 0).all()                      # bitwise, no two copies agree any more
    for j in range(f):
        n_byz = sum(1 for k in range(r) if int(fw[j, k]) in byz)
        honest_wins = int(fw[j, wrep[j]]) not in byz
        assert honest_wins == (n_byz < (r + 1) // 2), j
    assert np.array_equal(np.stack(O.vote_tolerant(X, rows, d, 1e-6, 1e-5)),
                          np.stack(C.vote_tolerant(X, rows, d, 1e-6, 1e-5)))


def test_c_vote_spread_over_threads_takes_the_same_decisions():
    # the loop over files may run on several host threads (used when the oracle is timed as the
    # CPU baseline); every file is still decided exactly as in the plain loop and as the NumPy
    # definition decides it, including ties, a difference in the last word only, and +-0
    rng = np.random.default_rng(77)
    for (f, r, d) in [(9, 3, 257), (25, 5, 1000), (7, 7, 33)]:
        G = rng.standard_normal((f, d)).astype(np.float32)
        X = np.zeros((f * r, d + 3), dtype=np.float32)
        rows = rng.permutation(f * r).astype(np.int32).reshape(f, r)
        for j in range(f):
            for k in range(r):
                X[rows[j, k], :d] = G[j]
        for j in range(f):
            kind = j % 5
            if kind == 1:
                X[rows[j, 0], d - 1] += 1.0
            elif kind == 2:
                for k in range(r):
                    X[rows[j, k], 0] = float(k)
            elif kind == 3:
                X[rows[j, r - 1], :d] = -100.0 * G[j]
                X[rows[j, r - 2], :d] = -100.0 * G[j]
            elif kind == 4:
                X[rows[j, 1], 5] = 0.0
                X[rows[j, 0], 5] = -0.0
        X[:, d:] = rng.standard_normal((f * r, 3)).astype(np.float32)  # padding differs everywhere
        want = O.vote(X, rows, d)
        plain = C.vote(X, rows, d)
        for t in (1, 3, 64):
            got = C.vote(X, rows, d, threads=t)
            assert got[3] == min(t, f)
            for a, b, c in zip(want, plain, got[:3]):
                assert np.array_equal(a, b) and np.array_equal(a, c)
        out_t, wrep_t, _ = C.aggregate(X, rows, d, threads=3) if f % 2 else (None, want[0], None)
        assert np.array_equal(wrep_t, want[0])
