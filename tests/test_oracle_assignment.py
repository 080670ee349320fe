"""Pins for the oracle's task assignment against what the paper prints and proves."""
import itertools

import numpy as np
import pytest

from oracle import byz_oracle as O
from tests import golden_io


def test_table1_squares_cell_by_cell():
    # Table 1: L_1, L_2, L_3 of degree 5
    for alpha, cells in golden_io.table1_squares().items():
        assert O.latin_square(5, alpha).tolist() == cells


@pytest.mark.parametrize("l", [3, 4, 5, 7, 8, 9, 11, 16])
def test_squares_are_latin_and_mutually_orthogonal(l):
    # Definitions 1 and 2 (Sec. 4.1.1)
    squares = [O.latin_square(l, a) for a in range(1, l)]
    sym = list(range(l))
    for L in squares:
        for i in range(l):
            assert sorted(L[i, :].tolist()) == sym and sorted(L[:, i].tolist()) == sym
    for L1, L2 in itertools.combinations(squares, 2):
        pairs = {(int(L1[i, j]), int(L2[i, j])) for i in range(l) for j in range(l)}
        assert len(pairs) == l * l


@pytest.mark.parametrize("l", [2, 3, 4, 5, 7, 8, 9, 16, 25, 27])
def test_finite_field_axioms(l):
    # F_l of Sec. 4.1.1 for prime powers: commutative ring with 0 and 1 in which every nonzero
    # element has an inverse, of characteristic p
    add, mul = O.finite_field(l)
    p, k = O.prime_power(l)
    E = range(l)
    assert (add == add.T).all() and (mul == mul.T).all()
    assert (add[0] == np.arange(l)).all() and (mul[1] == np.arange(l)).all() and (mul[0] == 0).all()
    for a in E:
        assert sorted(add[a].tolist()) == list(E)          # a + . is a bijection
        if a:
            assert sorted(mul[a].tolist()) == list(E)      # a * . is a bijection (inverse exists)
        x = 0
        for _ in range(p):
            x = add[x, a]
        assert x == 0                                      # characteristic p
    rng = np.random.default_rng(l)
    for a, b, c in rng.integers(0, l, size=(300, 3)):
        assert add[add[a, b], c] == add[a, add[b, c]]
        assert mul[mul[a, b], c] == mul[a, mul[b, c]]
        assert mul[a, add[b, c]] == add[mul[a, b], mul[a, c]]
    if k == 1:
        assert all(add[a, b] == (a + b) % l and mul[a, b] == (a * b) % l for a in E for b in E)


def test_finite_field_textbook_products():
    # GF(4) = F_2[x]/(x^2+x+1), elements 0, 1, x=2, x+1=3: x*x = x+1, x*(x+1) = 1, (x+1)^2 = x
    _, m4 = O.finite_field(4)
    assert (m4[2, 2], m4[2, 3], m4[3, 3]) == (3, 1, 2)
    # GF(8) = F_2[x]/(x^3+x+1) (x^3+x+1 = 1011b is below x^3+x^2+1 = 1101b): x^3 = x+1,
    # x^4 = x^2+x, x^7 = 1
    a8, m8 = O.finite_field(8)
    assert m8[2, 4] == 3 and m8[4, 4] == 6
    x = 1
    for _ in range(7):
        x = m8[x, 2]
    assert x == 1
    # GF(9) = F_3[i]/(i^2+1): i = 3, i*i = -1 = 2, (1+i)^2 = 2i = 6
    _, m9 = O.finite_field(9)
    assert m9[3, 3] == 2 and m9[4, 4] == 6
    # not prime powers
    for l in (6, 10, 12, 15):
        assert O.prime_power(l) is None


def test_example1_worker0():
    # Example 1: symbol 0 of L_1 sits at (0,0),(1,4),(2,3),(3,2),(4,1) -> U_0 = {0,9,13,17,21}
    L1 = O.latin_square(5, 1)
    cells = [(i, j) for i in range(5) for j in range(5) if L1[i, j] == 0]
    assert cells == [(0, 0), (1, 4), (2, 3), (3, 2), (4, 1)]
    H = O.mols_biadjacency(5, 3)
    assert O.worker_files(H)[0].tolist() == [0, 9, 13, 17, 21]


def test_table2_full_allocation():
    H = O.mols_biadjacency(5, 3)
    wf = O.worker_files(H)
    alloc = golden_io.table2_allocation()
    assert len(alloc) == 15
    for w, files in alloc.items():
        assert wf[w].tolist() == files


@pytest.mark.parametrize("l,r", [(5, 3), (7, 3), (7, 5), (5, 4), (11, 3), (4, 3), (8, 5), (9, 3),
                                 (9, 7)])
def test_mols_structure(l, r):
    H = O.mols_biadjacency(l, r)
    K, f, ll, rr = O.dims(H)
    assert (K, f, ll, rr) == (r * l, l * l, l, r)
    # Sec. 4.1.2: same-square workers share no file, different-square workers exactly one
    G = H @ H.T
    for u in range(K):
        for v in range(K):
            if u == v:
                assert G[u, v] == l
            elif u // l == v // l:
                assert G[u, v] == 0
            else:
                assert G[u, v] == 1
    # a parallel class holds exactly one replica of every file (Appendix, proof of Lemma 2)
    for k in range(r):
        assert (H[k * l:(k + 1) * l].sum(axis=0) == 1).all()


def _spectrum(H):
    K, f, l, r = O.dims(H)
    A = H / np.sqrt(l * r)
    return np.sort(np.linalg.eigvalsh(A @ A.T))[::-1], (K, f, l, r)


@pytest.mark.parametrize("l,r", [(5, 3), (7, 3), (7, 5), (4, 3), (8, 3), (9, 5)])
def test_lemma2_spectrum_mols(l, r):
    # Lemma 2: {(1,1), (1/r, r(l-1)), (0, r-1)}
    ev, _ = _spectrum(O.mols_biadjacency(l, r))
    expect = [1.0] + [1.0 / r] * (r * (l - 1)) + [0.0] * (r - 1)
    assert np.allclose(ev, expect, atol=1e-9)


def test_lemma2_block_form_mols():
    # Appendix: A A^T = (1/(l r)) C (x) J_l + (1/r) I with C = J_r - I_r
    l, r = 5, 3
    H = O.mols_biadjacency(l, r)
    A = H / np.sqrt(l * r)
    C = np.ones((r, r)) - np.eye(r)
    assert np.allclose(A @ A.T, np.kron(C, np.ones((l, l))) / (l * r) + np.eye(l * r) / r)


def test_cyclic_shift_and_array_code_blocks():
    # Step 2/3 of Sec. 4.2.1: P is a permutation, P^s = I, block (a,b) of B is P^(ab)
    s, m = 5, 5
    P = O.cyclic_shift_matrix(s)
    assert (P.sum(axis=0) == 1).all() and (P.sum(axis=1) == 1).all()
    assert P[0, s - 1] == 1 and P[1, 0] == 1  # j = i - 1 (mod s)
    assert (np.linalg.matrix_power(P, s) == np.eye(s, dtype=int)).all()
    B = O.array_code_matrix(m, s)
    assert B.shape == (s * s, m * s)
    # first block row and first block column are identities
    for b in range(m):
        assert (B[0:s, b * s:(b + 1) * s] == np.eye(s, dtype=int)).all()
    for a in range(s):
        assert (B[a * s:(a + 1) * s, 0:s] == np.eye(s, dtype=int)).all()
    assert (B[2 * s:3 * s, 3 * s:4 * s] == np.linalg.matrix_power(P, 6)).all()


@pytest.mark.parametrize("m,s,expect", [(5, 5, (25, 25, 5, 5)), (3, 5, (15, 25, 5, 3)),
                                        (3, 7, (21, 49, 7, 3)), (10, 5, (25, 50, 10, 5))])
def test_ramanujan_dims_eq6(m, s, expect):
    # Eq. 6: (K,f,l,r) = (ms, s^2, s, m) if m < s else (s^2, ms, m, s)
    H = O.ramanujan_biadjacency(m, s)
    assert O.dims(H) == expect


def test_lemma2_spectrum_ramanujan():
    # Case 2 (m=s=5): {(1,1), (1/r, r(r-1)), (0, r-1)}, r = 5
    ev, (K, f, l, r) = _spectrum(O.ramanujan_biadjacency(5, 5))
    assert np.allclose(ev, [1.0] + [1.0 / r] * (r * (r - 1)) + [0.0] * (r - 1), atol=1e-9)
    # Case 1 (m=3, s=5): same spectrum as MOLS(5,3)
    ev, (K, f, l, r) = _spectrum(O.ramanujan_biadjacency(3, 5))
    assert np.allclose(ev, [1.0] + [1.0 / r] * (r * (l - 1)) + [0.0] * (r - 1), atol=1e-9)


def test_ramanujan_case2_pairwise_sharing():
    H = O.ramanujan_biadjacency(5, 5)
    G = H @ H.T
    off = G - np.diag(np.diag(G))
    assert off.max() == 1  # any two workers share at most one file
    s = 5
    for a in range(s):  # block row a is a parallel class: every file exactly once
        assert (H[a * s:(a + 1) * s].sum(axis=0) == 1).all()


def test_fig1_toy_shape_counts():
    # Fig. 1 of the paper: K=6 workers, f=4 files, r=3, two files per worker: l = f r / K
    K, f, r = 6, 4, 3
    assert f * r // K == 2


@pytest.mark.parametrize("H", [O.mols_biadjacency(5, 3), O.ramanujan_biadjacency(5, 5)])
def test_file_rows_layout(H):
    K, f, l, r = O.dims(H)
    wf, fw, rows = O.worker_files(H), O.file_workers(H), O.file_rows(H)
    assert sorted(rows.reshape(-1).tolist()) == list(range(K * l))  # a bijection onto the rows
    for j in range(f):
        for k in range(r):
            w, t = divmod(int(rows[j, k]), l)
            assert w == fw[j, k] and wf[w][t] == j
            assert w // l == k  # replica k comes from parallel class k
