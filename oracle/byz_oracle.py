"""CPU oracle for the ByzShield parameter-server aggregation path (arXiv 2010.04902).

TEST INFRASTRUCTURE ONLY.  This module is the plain, slow, by-the-definition
implementation that the HIP path is checked against.  It shares no code with
the HIP path or its host library and imports neither; only tests, the smoke
check and the benchmark's CPU-baseline leg may use it.

Everything follows the paper's notation: K workers U_0..U_{K-1}, f files,
replication r (odd), r' = (r+1)/2, load l = f*r/K, d coordinates.

Parity status of each function (what pins it, see tests/test_oracle_*.py):
  latin_square, mols_biadjacency      Table 1, Example 1, Table 2 cell by cell
  finite_field (prime-power l)        field axioms by brute force, textbook products in
                                      GF(4), GF(8), GF(9); Definition 2 (orthogonality) cell by cell;
                                      numbering of the elements: paper silent, "parity unpinned"
  ramanujan_biadjacency               Eq. 6 degrees, Lemma 2 spectrum, Table 4
  frc_biadjacency                     Sec. 5.3.1: floor(q/r') lost groups, FRC column of Tables 3-6
  worst_case                          Tables 3-6, Claim 2, naive brute force
  gamma_bound                         Tables 3-6 (gamma column), closed forms Sec. 5.1
  vote                                brute force over all equality patterns, Sec. 2
                                      statements (all-honest, distorted iff >= r')
  vote_tolerant, words_close          numpy.isclose both ways, zero tolerance = exact vote, hand-worked
                                      chain a~b~c, Sec. 2 majority property under noise (the paper
                                      gives no rule: "parity unpinned")
  median                              numpy sort/median on ordinary data, brute force
  multi_krum                          scipy cdist, hand-worked line example, outlier exclusion
                                      (the paper cites but does not define the rule)
  bulyan_select, mean_around_median, bulyan
                                      first pick = Krum (cdist), c = 0 -> plain mean, brute force over
                                      subsets (closest-to-median set), hand-worked cases, honest-range
                                      property (the paper cites but does not define the rule)
  trimmed_mean                        scipy.stats.trim_mean, b=0 mean, b=(f-1)/2 median, hand-worked case
  tie-break rules (vote plurality ties -> lowest replica; total order of
  +-0 / NaN in the median; lexicographically first worst-case set):
      the paper is silent on these -> "parity unpinned" by the paper; both
      sides implement the reading written here.
"""
import itertools

import numpy as np

# --------------------------------------------------------------------------
# Task assignment (Sec. 4)
# --------------------------------------------------------------------------


def is_prime(n):
    n = int(n)
    if n < 2:
        return False
    for p in range(2, n):
        if p * p > n:
            break
        if n % p == 0:
            return False
    return True


def prime_power(l):
    """(p, k) with l = p**k and p prime, or None."""
    l = int(l)
    for p in range(2, l + 1):
        if is_prime(p) and l % p == 0:
            k, t = 0, l
            while t % p == 0:
                t //= p
                k += 1
            return (p, k) if t == 1 else None
    return None


def finite_field(l):
    """Addition and multiplication tables (l x l) of F_l for a prime power l = p**k.

    The paper (Sec. 4.1.1) takes R = C = S = F_l = {0, .., l-1} without saying which integer is
    which field element when k > 1.  Reading used here: integer n stands for the polynomial
    whose coefficients are the base-p digits of n (lowest digit = constant term); products are
    reduced modulo the monic degree-k polynomial x^k + c(x) with the smallest integer c for
    which the result is a field.  For k = 1 this is arithmetic modulo p.

    Written from the definition: schoolbook polynomial product, the substitution
    x^k -> -c(x) applied from the top degree down, and "field" tested as "no two nonzero
    elements multiply to zero".
    """
    pk = prime_power(l)
    assert pk is not None, "l must be a prime power"
    p, k = pk

    def digits(n):
        return [(n // p ** t) % p for t in range(k)]

    def number(coeffs):
        return sum(int(c) * p ** t for t, c in enumerate(coeffs))

    add = np.zeros((l, l), dtype=np.int64)
    for a in range(l):
        for b in range(l):
            add[a, b] = number([(x + y) % p for x, y in zip(digits(a), digits(b))])
    for c in range(l):
        low = digits(c)
        mul = np.zeros((l, l), dtype=np.int64)
        for a in range(l):
            for b in range(l):
                prod = [0] * (2 * k - 1)
                for i, x in enumerate(digits(a)):
                    for j, y in enumerate(digits(b)):
                        prod[i + j] = (prod[i + j] + x * y) % p
                for t in range(2 * k - 2, k - 1, -1):  # x^t = x^(t-k) * x^k = -x^(t-k) * c(x)
                    top, prod[t] = prod[t], 0
                    for j in range(k):
                        prod[t - k + j] = (prod[t - k + j] - top * low[j]) % p
                mul[a, b] = number(prod[:k])
        if (mul[1:, 1:] != 0).all():
            return add, mul
    raise AssertionError("no irreducible polynomial found")


def latin_square(l, alpha):
    """Sec. 4.1.1: the square L_alpha(i, j) = alpha*i + j over F_l (l a prime power, alpha a
    nonzero element; elements numbered as in finite_field)."""
    assert 0 < alpha < l
    add, mul = finite_field(l)
    L = np.zeros((l, l), dtype=np.int64)
    for i in range(l):
        for j in range(l):
            L[i, j] = add[mul[alpha, i], j]
    return L


def mols_biadjacency(l, r):
    """Algorithm 2 (MOLS-based assignment): K = r*l workers, f = l*l files.

    For k = 0..r-1 and every symbol s, each cell (i, j) of L_{k+1} that holds s
    connects file i*l + j to worker U_{k*l + s}.  Returns H (K x f, 0/1), Eq. 4.
    """
    assert 1 <= r <= l - 1
    H = np.zeros((r * l, l * l), dtype=np.int64)
    for k in range(r):
        L = latin_square(l, k + 1)
        for s in range(l):
            for i in range(l):
                for j in range(l):
                    if L[i, j] == s:
                        H[k * l + s, i * l + j] = 1
    return H


def cyclic_shift_matrix(s):
    """Sec. 4.2.1 Step 2: P[i][j] = 1 iff j = i - 1 (mod s)."""
    P = np.zeros((s, s), dtype=np.int64)
    for i in range(s):
        P[i, (i - 1) % s] = 1
    return P


def array_code_matrix(m, s):
    """Sec. 4.2.1 Step 3: B, an s x m grid of s x s blocks, block (a, b) = P^(a*b)."""
    assert m >= 2 and is_prime(s)
    P = cyclic_shift_matrix(s)
    B = np.zeros((s * s, m * s), dtype=np.int64)
    for a in range(s):
        for b in range(m):
            B[a * s:(a + 1) * s, b * s:(b + 1) * s] = np.linalg.matrix_power(P, a * b)
    return B


def ramanujan_biadjacency(m, s):
    """Sec. 4.2.1 / Eq. 6: H = B when m >= s (Case 2), H = B^T when m < s (Case 1).

    Rows of H are workers, columns are files.
    """
    B = array_code_matrix(m, s)
    return B if m >= s else B.T.copy()


def frc_biadjacency(K, r):
    """Sec. 5.3.1: Fractional Repetition Code of DETOX / DRACO.  K/r groups of r workers; every
    worker of group j holds file j.  Replica k of file j is worker k*(K/r) + j (the paper does
    not number the workers; this keeps one replica of every file per block of K/r workers)."""
    assert K % r == 0
    f = K // r
    H = np.zeros((K, f), dtype=np.int64)
    for j in range(f):
        for k in range(r):
            H[k * f + j, j] = 1
    return H


def dims(H):
    """(K, f, l, r) of a biregular biadjacency matrix (Sec. 2: l = f*r/K)."""
    K, f = H.shape
    l = int(H[0].sum())
    r = int(H[:, 0].sum())
    assert (H.sum(axis=1) == l).all() and (H.sum(axis=0) == r).all()
    assert l * K == f * r
    return K, f, l, r


def worker_files(H):
    """N(U_w): ascending list of the l files worker w holds."""
    return np.array([np.flatnonzero(H[w]) for w in range(H.shape[0])], dtype=np.int32)


def file_workers(H):
    """N(B_j): ascending list of the r workers holding file j (replica k = k-th of them)."""
    return np.array([np.flatnonzero(H[:, j]) for j in range(H.shape[1])], dtype=np.int32)


def file_rows(H):
    """Row of the stacked returns that holds replica k of file j.

    A worker returns the gradients of its files in ascending file order
    (Algorithm 1, the return step), worker after worker, so worker w's t-th
    file sits in row w*l + t.
    """
    K, f, l, r = dims(H)
    wf = worker_files(H)
    fw = file_workers(H)
    rows = np.zeros((f, r), dtype=np.int32)
    for j in range(f):
        for k in range(r):
            w = int(fw[j, k])
            t = list(wf[w]).index(j)
            rows[j, k] = w * l + t
    return rows


# --------------------------------------------------------------------------
# Worst-case adversary (Sec. 5.2, 5.3.2) and the expansion bound (Sec. 3)
# --------------------------------------------------------------------------


def distorted_files(H, S):
    """Files with at least r' of their r copies on workers in S (Sec. 2)."""
    K, f, l, r = dims(H)
    rp = (r + 1) // 2
    S = list(S)
    cnt = H[S].sum(axis=0) if S else np.zeros(f, dtype=np.int64)
    return np.flatnonzero(cnt >= rp)


def worst_case(H, q):
    """c_max^(q): exhaustive search over all q-subsets of the K workers (Sec. 5.3.2).

    Subsets are visited in lexicographic order of their ascending tuple and
    the first one attaining the maximum is returned (the paper only says "a
    set such that the distortion is maximised").
    Returns (c_max, S as a tuple, ascending array of distorted files).
    """
    K = H.shape[0]
    best, best_S = -1, None
    for S in itertools.combinations(range(K), q):
        c = len(distorted_files(H, S))
        if c > best:
            best, best_S = c, S
    return best, best_S, distorted_files(H, best_S)


def gamma_bound(K, f, l, r, q, mu1=None):
    """Eq. 5 then Claim 1: beta = (q l / r) / (mu1 + (1 - mu1) q / K), gamma = (q l - beta) / ((r - 1)/2).

    mu1 defaults to 1/r (Lemma 2, all three constructions).
    """
    if mu1 is None:
        mu1 = 1.0 / r
    beta = (q * l / r) / (mu1 + (1.0 - mu1) * q / K)
    return (q * l - beta) / ((r - 1) / 2.0)


# --------------------------------------------------------------------------
# Majority vote (Eq. 3) and coordinate-wise median (Sec. 2, Sec. 6.1)
# --------------------------------------------------------------------------


def pair_index(r):
    """Pairs (a, b), a < b, in lexicographic order; bit p of pair_neq is pair p."""
    return [(a, b) for a in range(r) for b in range(a + 1, r)]


def vote(X, rows, d):
    """Eq. 3 with the paper's implementation note: the copy that appears most often.

    X: [R, ld] array of 32-bit words (float32 or uint32), rows: [f, r] row ids.
    Two copies are equal iff all d 32-bit words are identical bit patterns.
    count[a] = number of copies equal to copy a (itself included); the winner
    is the smallest a with the largest count.
    Returns (winner_replica[f], winner_row[f], pair_neq[f]) where bit p of
    pair_neq[j] is 1 iff the copies of pair p (see pair_index) differ.
    """
    U = np.ascontiguousarray(X).view(np.uint32)
    f, r = rows.shape
    pairs = pair_index(r)
    winner_replica = np.zeros(f, dtype=np.int32)
    winner_row = np.zeros(f, dtype=np.int32)
    pair_neq = np.zeros(f, dtype=np.uint32)
    for j in range(f):
        copies = [U[rows[j, k], :d].tobytes() for k in range(r)]
        count = [sum(1 for b in range(r) if copies[a] == copies[b]) for a in range(r)]
        best = max(count)
        a_star = count.index(best)
        winner_replica[j] = a_star
        winner_row[j] = rows[j, a_star]
        bits = 0
        for p, (a, b) in enumerate(pairs):
            if copies[a] != copies[b]:
                bits |= 1 << p
        pair_neq[j] = bits
    return winner_replica, winner_row, pair_neq


def words_close(xa, xb, atol, rtol):
    """Element-wise "close" test of the tolerant vote, all in fp32: two words are close iff their
    bit patterns are identical, or |xa - xb| <= atol + rtol * max(|xa|, |xb|) with the
    subtraction, the product and the sum each rounded to fp32 (comparisons with NaN are false)."""
    xa = np.ascontiguousarray(xa, dtype=np.float32)
    xb = np.ascontiguousarray(xb, dtype=np.float32)
    same_bits = xa.view(np.uint32) == xb.view(np.uint32)
    with np.errstate(invalid="ignore", over="ignore"):
        diff = np.abs((xa - xb).astype(np.float32))
        big = np.maximum(np.abs(xa), np.abs(xb)).astype(np.float32)
        prod = (np.float32(rtol) * big).astype(np.float32)
        bound = (np.float32(atol) + prod).astype(np.float32)
        return same_bits | (diff <= bound)


def vote_tolerant(X, rows, d, atol, rtol):
    """Majority vote for honest copies that agree only up to rounding (Sec. 2 remarks that
    precision differences between honest workers could be dealt with by voting over clusters of
    nearby vectors, without giving a rule).  Reading used here: two copies are close iff every one of their d
    coordinates is close (words_close); count[a] = number of copies close to copy a, itself
    included; the winner is the smallest a with the largest count.  Closeness is not
    transitive, so this is a count of neighbours, not a partition.
    Returns (winner_replica[f], winner_row[f], pair_far[f]): bit p of pair_far[j] is 1 iff the
    copies of pair p (see pair_index) are not close."""
    V = np.ascontiguousarray(X).view(np.float32)
    f, r = rows.shape
    pairs = pair_index(r)
    winner_replica = np.zeros(f, dtype=np.int32)
    winner_row = np.zeros(f, dtype=np.int32)
    pair_far = np.zeros(f, dtype=np.uint32)
    for j in range(f):
        close = np.eye(r, dtype=bool)
        bits = 0
        for p, (a, b) in enumerate(pairs):
            ok = bool(words_close(V[rows[j, a], :d], V[rows[j, b], :d], atol, rtol).all())
            close[a, b] = close[b, a] = ok
            if not ok:
                bits |= 1 << p
        count = [int(close[a].sum()) for a in range(r)]
        a_star = count.index(max(count))
        winner_replica[j] = a_star
        winner_row[j] = rows[j, a_star]
        pair_far[j] = bits
    return winner_replica, winner_row, pair_far


def order_key(u):
    """Total order on float32 bit patterns used by the median.

    key = bits ^ 0xFFFFFFFF for negative-sign patterns, bits ^ 0x80000000
    otherwise, compared as unsigned integers:
      -NaN < -inf < ... < -0 < +0 < ... < +inf < +NaN.
    On NaN-free data it is the usual '<' except that -0 sorts before +0.
    """
    u = np.asarray(u, dtype=np.uint32)
    neg = (u >> np.uint32(31)).astype(bool)
    return np.where(neg, u ^ np.uint32(0xFFFFFFFF), u ^ np.uint32(0x80000000))


def median(X, row_index, d):
    """Coordinate-wise median of f rows (f odd): the element of rank (f-1)/2.

    Sorts the f order keys of every coordinate and returns, bit for bit, the
    input value whose key lands in the middle.
    """
    U = np.ascontiguousarray(X).view(np.uint32)
    row_index = np.asarray(row_index)
    f = len(row_index)
    assert f % 2 == 1
    vals = np.stack([U[int(row_index[j]), :d] for j in range(f)])  # [f, d]
    keys = order_key(vals)
    order = np.argsort(keys, axis=0, kind="stable")
    mid = order[(f - 1) // 2]  # [d] index of the file holding the median
    out = vals[mid, np.arange(d)]
    return out.view(np.float32)


def trimmed_mean(X, row_index, d, b):
    """Coordinate-wise trimmed mean (the aggregator the paper's Sec. 1 cites beside the median):
    sort the f values of a coordinate by order_key, drop the b smallest and the b largest,
    return the fp64 mean of the f - 2b that remain (summed in ascending order)."""
    U = np.ascontiguousarray(X).view(np.uint32)
    row_index = np.asarray(row_index)
    f = len(row_index)
    assert 0 <= b and 2 * b < f
    vals = np.stack([U[int(row_index[j]), :d] for j in range(f)])  # [f, d]
    order = np.argsort(order_key(vals), axis=0, kind="stable")
    srt = np.take_along_axis(vals, order, axis=0).view(np.float32).astype(np.float64)
    acc = np.zeros(d, dtype=np.float64)
    for i in range(b, f - b):
        acc = acc + srt[i]
    return acc / float(f - 2 * b)


def multi_krum(X, row_index, d, c, m):
    """Multi-Krum (the aggregator Sec. 6.1 / Sec. 7 of the paper name for use on the vote
    winners; rule as published by Blanchard et al. and Damaskinos et al.): with f vectors of
    which c may be Byzantine (f >= 2c + 3), score(i) = sum of the f - c - 2 smallest squared
    distances from vector i to the others; the m lowest scores (ties: lower index) are
    selected and averaged.  Everything in fp64, distances as sums of squared differences.
    Returns (mean[d], selected[f] 0/1, scores[f], dist[f, f])."""
    V = np.stack([np.ascontiguousarray(X)[int(j), :d] for j in row_index]).astype(np.float64)
    f = V.shape[0]
    assert f >= 2 * c + 3 and 1 <= m <= f - c
    dist = np.zeros((f, f))
    for i in range(f):
        for j in range(f):
            diff = V[i] - V[j]
            dist[i, j] = float(np.dot(diff, diff))
    scores = np.zeros(f)
    for i in range(f):
        others = sorted(dist[i, j] for j in range(f) if j != i)
        scores[i] = sum(others[:f - c - 2])
    order = sorted(range(f), key=lambda i: (scores[i], i))
    selected = np.zeros(f, dtype=np.int32)
    selected[order[:m]] = 1
    acc = np.zeros(d)
    for i in range(f):
        if selected[i]:
            acc = acc + V[i]
    return acc / m, selected, scores, dist


def bulyan_select(dist, c):
    """First phase of Bulyan (El Mhamdi, Guerraoui, Rouault 2018; the paper cites it as an
    aggregator that can take the median's place, Sec. 7, without defining it): Krum is applied
    again and again to the vectors not yet chosen until theta = n - 2c are chosen.

    One round on the remaining set R (n' = |R|): score(i) = sum of the n' - c - 2 smallest
    dist[i, j], j in R, j != i (no terms when n' - c - 2 <= 0, which happens in the last rounds:
    the published rule is silent there; all scores are then 0); the lowest score wins, ties go
    to the lowest index.  Returns the chosen indices in the order they were chosen.
    """
    n = dist.shape[0]
    assert c >= 0 and n >= 4 * c + 3
    remaining = list(range(n))
    chosen = []
    while len(chosen) < n - 2 * c:
        k = max(len(remaining) - c - 2, 0)
        best, best_score = None, None
        for i in remaining:
            others = sorted(dist[i, j] for j in remaining if j != i)
            score = 0.0
            for v in others[:k]:
                score += v
            if best is None or score < best_score:
                best, best_score = i, score
        chosen.append(best)
        remaining.remove(best)
    return chosen


def mean_around_median(values, beta):
    """Second phase of Bulyan for one coordinate: the beta values closest to the median of
    `values` (odd count), averaged.  The values are put in the total order of the median
    kernel; starting from the middle one the window grows one neighbour at a time, taking the
    lower neighbour when its distance to the median, computed in fp32 as (median - x), is <=
    the upper neighbour's (x - median) or there is no upper neighbour left (comparisons with
    NaN are false, as in IEEE arithmetic).  The mean is taken in fp64 over the window in
    ascending order.  Returns (mean, lo, hi): window = sorted positions lo..hi inclusive.
    """
    v = np.asarray(values, dtype=np.float32)
    n = len(v)
    assert n % 2 == 1 and 1 <= beta <= n
    order = np.argsort(order_key(v.view(np.uint32)), kind="stable")
    s = v[order]
    h = (n - 1) // 2
    med = s[h]
    lo = hi = h
    with np.errstate(invalid="ignore", over="ignore"):
        for _ in range(beta - 1):
            can_l, can_r = lo > 0, hi < n - 1
            take_left = False
            if can_l and not can_r:
                take_left = True
            elif can_l and can_r:
                dl = np.float32(med - s[lo - 1])
                dr = np.float32(s[hi + 1] - med)
                take_left = bool(dl <= dr)
            if take_left:
                lo -= 1
            else:
                hi += 1
        acc = 0.0
        for t in range(lo, hi + 1):
            acc += float(s[t])
    return acc / beta, lo, hi


def bulyan(X, row_index, d, c):
    """Bulyan over the f rows row_index of X with c of them possibly Byzantine (f >= 4c + 3,
    the requirement Sec. 6.1 of the paper quotes): theta = f - 2c vectors are chosen by
    repeated Krum (bulyan_select, squared distances in fp64 as sums of squared differences),
    then every coordinate is the mean of the beta = theta - 2c chosen values closest to their
    median (mean_around_median).  Returns (out[d] fp64, chosen indices in order, dist[f, f])."""
    V32 = np.stack([np.ascontiguousarray(X)[int(j), :d] for j in row_index]).astype(np.float32)
    V = V32.astype(np.float64)
    f = V.shape[0]
    assert f >= 4 * c + 3
    dist = np.zeros((f, f))
    for i in range(f):
        for j in range(f):
            diff = V[i] - V[j]
            dist[i, j] = float(np.dot(diff, diff))
    chosen = bulyan_select(dist, c)
    beta = f - 4 * c
    out = np.zeros(d)
    S = V32[chosen]
    for t in range(d):
        out[t] = mean_around_median(S[:, t], beta)[0]
    return out, chosen, dist


def aggregate(X, rows, d):
    """Vote per file, then the coordinate-wise median across the f winners."""
    winner_replica, winner_row, _ = vote(X, rows, d)
    return median(X, winner_row, d), winner_replica
