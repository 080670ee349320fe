"""Host-side logic through the C-ABI (no GPU): the library loads, exports every declared
symbol, builds the paper's assignments and reproduces its distortion tables."""
import ctypes
import math
import os
import re
import sys

import numpy as np
import pytest

import paper_2010_04902_amd as B
from oracle import byz_oracle as O
from oracle import c_oracle as C
from tests import golden_io

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TABLES = golden_io.distortion_tables()


def _H(asg):
    H = np.zeros((asg.K, asg.f), dtype=np.int64)
    wf = asg.worker_files()
    for w in range(asg.K):
        H[w, wf[w]] = 1
    return H


def _build(scheme, a, b):
    return B.byz_build_assignment(B.BYZ_SCHEME_MOLS if scheme == "mols" else B.BYZ_SCHEME_RAMANUJAN,
                                  a, b)


def test_library_exports_every_declared_symbol():
    names = set()
    for h in ("byzshield.h", "byzshield_bench.h"):
        header = open(os.path.join(ROOT, "include", h)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        found = set(re.findall(r"\b(byz_[a-z_0-9]+)\s*\(", header))
        assert len(found) >= 5, h
        names |= found
    names = sorted(names)
    assert len(names) >= 30
    lib = ctypes.CDLL(B.library_path())
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c_and_agrees_with_the_binding(tmp_path):
    # the boundary is a C header: it compiles as C, and its limits, status codes and flag
    # macros have the values the Python binding uses
    src = tmp_path / "consts.c"
    src.write_text('''#include <stdio.h>
#include "byzshield.h"
#include "byzshield_bench.h"
int main(void) {
    printf("%d %d %d %d\\n", BYZ_MAX_F, BYZ_MAX_F_KRUM, BYZ_MAX_F_WIDE, BYZ_MAX_R);
    printf("%u %u %u %u\\n", BYZ_AGG_EARLY_MAJORITY, BYZ_AGG_TRIM(7), BYZ_AGG_PROBE_SHIFT(0x1234),
           BYZ_AGG_PROBE_SHIFT(0x12345));
    printf("%d %d %d\\n", (int)BYZ_SCHEME_MOLS, (int)BYZ_SCHEME_RAMANUJAN, (int)BYZ_SCHEME_FRC);
    printf("%u %u\\n", (unsigned)BYZ_SEARCH_EXHAUSTIVE, (unsigned)BYZ_SEARCH_SYMMETRY);
    printf("%d %d %d %d\\n", (int)BYZ_PATH_SINGLE_PASS, (int)BYZ_PATH_MEDIAN_REDONE,
           (int)BYZ_PATH_REVOTED, (int)BYZ_PATH_TWO_STEP);
    return 0;
}
''')
    exe = tmp_path / "consts"
    import subprocess
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src),
                    "-o", str(exe)], check=True)
    lines = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    assert [int(x) for x in lines[0].split()] == [B.BYZ_MAX_F, B.BYZ_MAX_F_KRUM, B.BYZ_MAX_F_WIDE, B.BYZ_MAX_R]
    assert [int(x) for x in lines[1].split()] == [B.BYZ_AGG_EARLY_MAJORITY, B.BYZ_AGG_TRIM(7),
                                                  B.BYZ_AGG_PROBE_SHIFT(0x1234), B.BYZ_AGG_PROBE_SHIFT(0x12345)]
    assert [int(x) for x in lines[2].split()] == [B.BYZ_SCHEME_MOLS, B.BYZ_SCHEME_RAMANUJAN, B.BYZ_SCHEME_FRC]
    assert [int(x) for x in lines[3].split()] == [B.BYZ_SEARCH_EXHAUSTIVE, B.BYZ_SEARCH_SYMMETRY]
    assert [int(x) for x in lines[4].split()] == [B.BYZ_PATH_SINGLE_PASS, B.BYZ_PATH_MEDIAN_REDONE,
                                                  B.BYZ_PATH_REVOTED, B.BYZ_PATH_TWO_STEP]


def test_table2_through_the_library():
    asg = _build("mols", 5, 3)
    assert (asg.K, asg.f, asg.l, asg.r) == (15, 25, 5, 3)
    wf = asg.worker_files()
    for w, files in golden_io.table2_allocation().items():
        assert wf[w].tolist() == files


@pytest.mark.parametrize("scheme,a,b", [("mols", 5, 3), ("mols", 7, 3), ("mols", 7, 5),
                                        ("mols", 11, 3), ("mols", 3, 1), ("mols", 5, 4),
                                        ("ram", 5, 5), ("ram", 5, 3), ("ram", 7, 3), ("ram", 5, 10),
                                        ("ram", 3, 3), ("ram", 3, 2), ("ram", 5, 7), ("ram", 2, 2),
                                        # prime-power l: F_4, F_8, F_9, F_16, F_25, F_27
                                        ("mols", 4, 3), ("mols", 8, 7), ("mols", 9, 3),
                                        ("mols", 9, 8), ("mols", 16, 3), ("mols", 25, 3),
                                        ("mols", 27, 2)])
def test_assignment_equals_oracle_construction(scheme, a, b):
    asg = _build(scheme, a, b)
    Ho = O.mols_biadjacency(a, b) if scheme == "mols" else O.ramanujan_biadjacency(b, a)
    assert O.dims(Ho) == (asg.K, asg.f, asg.l, asg.r)
    assert np.array_equal(_H(asg), Ho)
    assert np.array_equal(asg.worker_files(), O.worker_files(Ho))
    assert np.array_equal(asg.file_workers(), O.file_workers(Ho))
    assert np.array_equal(asg.file_rows(), O.file_rows(Ho))


def test_build_errors():
    def code(*args):
        with pytest.raises(B.ByzError) as e:
            B.byz_build_assignment(*args)
        return e.value.code
    assert code(B.BYZ_SCHEME_MOLS, 5, 5) == -1        # Algorithm 2 needs r <= l-1
    assert code(B.BYZ_SCHEME_MOLS, 5, 0) == -1
    assert code(B.BYZ_SCHEME_MOLS, 6, 3) == -2        # l must be a prime power
    assert code(B.BYZ_SCHEME_MOLS, 12, 3) == -2
    assert code(B.BYZ_SCHEME_MOLS, 256, 3) == -1
    assert code(B.BYZ_SCHEME_RAMANUJAN, 4, 3) == -2   # s must be prime
    assert code(B.BYZ_SCHEME_RAMANUJAN, 5, 1) == -1   # m >= 2
    assert code(7, 5, 3) == -1
    assert code(B.BYZ_SCHEME_MOLS, 1, 1) == -1
    assert B.byz_strerror(-2).startswith("valid but")


@pytest.mark.parametrize("name", sorted(TABLES))
def test_cmax_tables_every_row(name):
    scheme, a, b, rows = TABLES[name]
    asg = _build("mols" if scheme == "mols" else "ram", a, b)
    H = _H(asg)
    for q, cmax, _, _, _, gamma in rows:
        S, c, mask = B.byz_worst_case(asg, q)
        assert c == cmax, (name, q)
        files = O.distorted_files(H, S)
        assert len(files) == cmax and mask == sum(1 << int(j) for j in files)
        assert list(S) == sorted(set(S)) and len(S) == q
        assert abs(B.byz_gamma_bound(asg, q) - gamma) < 0.011
        assert B.byz_gamma_bound(asg, q) == pytest.approx(O.gamma_bound(asg.K, asg.f, asg.l, asg.r, q),
                                                          rel=1e-12)
        assert c <= B.byz_gamma_bound(asg, q)  # Claim 1


@pytest.mark.parametrize("scheme,a,b,qs", [("mols", 5, 3, range(0, 8)), ("mols", 7, 3, range(0, 6)),
                                           ("ram", 5, 5, range(0, 7)), ("ram", 3, 3, range(0, 10)),
                                           ("ram", 5, 3, range(0, 7))])
def test_worst_case_first_argmax_equals_oracle(scheme, a, b, qs):
    asg = _build(scheme, a, b)
    H = _H(asg)
    for q in qs:
        S, c, _ = B.byz_worst_case(asg, q)
        c_o, S_o = C.worst_case(H, q)
        assert (c, tuple(S)) == (c_o, tuple(S_o)), q


def test_worst_case_workload_sets():
    # the Byzantine sets the five workloads use (lexicographically first maximisers)
    want = {("mols", 5, 3, 3): (0, 5, 11), ("mols", 5, 3, 4): (0, 1, 5, 11),
            ("mols", 7, 3, 5): (0, 1, 7, 8, 17), ("ram", 5, 5, 6): (0, 1, 5, 7, 14, 20),
            ("mols", 7, 3, 6): (0, 1, 7, 8, 17, 18)}
    for (scheme, a, b, q), S_want in want.items():
        asg = _build(scheme, a, b)
        S, c, _ = B.byz_worst_case(asg, q)
        assert tuple(S) == S_want
        assert C.worst_case(_H(asg), q)[1] == S_want  # the oracle finds the same set


def test_worst_case_errors():
    asg = _build("mols", 5, 3)
    for q in (-1, 16):
        with pytest.raises(B.ByzError) as e:
            B.byz_worst_case(asg, q)
        assert e.value.code == -1
    big = _build("mols", 17, 3)  # f = 289 > 256
    with pytest.raises(B.ByzError) as e:
        B.byz_worst_case(big, 2)
    assert e.value.code == -2
    assert math.isnan(B.byz_gamma_bound(asg, 99))
    assert B.byz_aggregate_workspace_bytes(25, 3) > 0 and B.byz_aggregate_workspace_bytes(255, 3) > 0
    assert B.byz_aggregate_workspace_bytes(25, 4) == 0 and B.byz_aggregate_workspace_bytes(257, 3) == 0


@pytest.mark.parametrize("scheme,a,b,qs", [("ram", 5, 13, (0, 1, 2, 3, 5)),     # f = 65, K = 25
                                           ("mols", 9, 3, (2, 3, 4)),            # F_9: f = 81
                                           ("mols", 11, 3, (2, 4)),              # f = 121
                                           ("mols", 13, 3, (3,)),                # f = 169
                                           ("mols", 16, 3, (2, 3))])             # F_16: f = 256
def test_worst_case_more_than_64_files(scheme, a, b, qs):
    asg = _build(scheme, a, b)
    H = _H(asg)
    for q in qs:
        S, c, mask = B.byz_worst_case(asg, q)
        c_o, S_o = C.worst_case(H, q)
        assert (c, tuple(S)) == (c_o, tuple(S_o)), q
        files = O.distorted_files(H, S)
        assert mask == sum(1 << int(j) for j in files) and len(files) == c
        assert c <= B.byz_gamma_bound(asg, q)  # Claim 1


# ------------------------------------------------------------- selection network generator

sys.path.insert(0, os.path.join(ROOT, "paper_2010_04902_amd", "csrc"))
import gen_selnet  # noqa: E402


@pytest.mark.parametrize("f", [3, 5, 7, 9, 15, 21, 25])
def test_selection_network_zero_one_exhaustive(f):
    # 0/1 principle: the network selects the median of every input iff it outputs the
    # majority bit for every 0/1 input; all 2^f inputs, one per array element.
    ops, wire = gen_selnet.best_network(f)
    idx = np.arange(1 << f, dtype=np.uint32)
    v = [((idx >> i) & 1).astype(np.uint8) for i in range(f)]
    for (i, j, lo, hi) in ops:
        a, b = v[i], v[j]
        if lo:
            v[i] = a & b
        if hi:
            v[j] = a | b
    pop = sum(((idx >> i) & 1) for i in range(f))
    assert np.array_equal(v[wire], (pop > f // 2).astype(np.uint8))


@pytest.mark.parametrize("f", [35, 49, 63, 65, 81, 121, 169])
def test_selection_network_near_balanced_inputs(f):
    ops, wire = gen_selnet.best_network(f)
    rng = np.random.default_rng(f)
    n = 200_000
    # 0/1 inputs whose number of ones is within 2 of f/2 (the critical weights), random positions
    w = rng.integers(f // 2 - 1, f // 2 + 3, size=n)
    M = (np.argsort(rng.random((n, f)), axis=1) < w[:, None]).astype(np.uint8)
    v = [M[:, i].copy() for i in range(f)]
    for (i, j, lo, hi) in ops:
        a, b = v[i], v[j]
        if lo:
            v[i] = a & b
        if hi:
            v[j] = a | b
    assert np.array_equal(v[wire], (w > f // 2).astype(np.uint8))
    # and on random integers against a sort
    vals = rng.integers(0, 1000, size=(2000, f))
    for row in vals:
        assert gen_selnet.apply_network(ops, row.tolist())[wire] == sorted(row.tolist())[f // 2]


def _run_network_columns(ops, cols):
    """cols: list of numpy arrays, one per wire; applies (i, j, lo, hi) comparators in place."""
    for (i, j, lo, hi) in ops:
        a, b = cols[i], cols[j]
        if lo:
            cols[i] = np.minimum(a, b)
        if hi:
            cols[j] = np.maximum(a, b)
    return cols


@pytest.mark.parametrize("f", [49, 63, 65, 81, 121])
def test_pruned_median_network_equals_the_unpruned_sort_on_tie_heavy_data(f):
    # a second check that shares nothing with the pruning: Batcher's sort on the next power of
    # two, every comparator kept, spare wires holding the largest value, must leave on wire
    # (f-1)/2 what the pruned network selects -- on two million columns drawn from a four-letter
    # alphabet (ties everywhere) and, for one in eight of them, with a single outlier
    n_pow = 1
    while n_pow < f:
        n_pow *= 2
    full = [(i, j, True, True) for (i, j) in gen_selnet.batcher_sort(n_pow)]
    ops, wire = gen_selnet.best_network(f)
    rng = np.random.default_rng(1000 + f)
    n = 2_000_000
    data = rng.integers(0, 4, size=(f, n), dtype=np.uint8)
    data[rng.integers(0, f, size=n // 8), np.arange(n // 8)] = 9
    pruned = _run_network_columns(ops, [data[i].copy() for i in range(f)])
    cols = [data[i].copy() for i in range(f)] + [np.full(n, 255, dtype=np.uint8)] * (n_pow - f)
    sorted_cols = _run_network_columns(full, cols)
    assert np.array_equal(pruned[wire], sorted_cols[(f - 1) // 2])
    # and the unpruned sort really sorts: equal to numpy's sort on a slice
    ref = np.sort(data[:, :20000], axis=0)
    for i in range(f):
        assert np.array_equal(sorted_cols[i][:20000], ref[i])


@pytest.mark.parametrize("f", gen_selnet.SORT_SIZES)
def test_sorting_network_sorts(f):
    # the full-sort networks behind the trimmed mean and Bulyan's second phase: every 0/1 input
    # for small f (0/1 principle), random 0/1 inputs of every weight and tie-heavy integers
    # against numpy's sort otherwise; and the streamed order is a valid order of the same network
    ops, _ = gen_selnet.best_network(f, True)
    assert all(lo and hi for (_, _, lo, hi) in ops)
    rng = np.random.default_rng(2000 + f)
    if f <= 21:
        idx = np.arange(1 << f, dtype=np.uint32)
        cols = [((idx >> i) & 1).astype(np.uint8) for i in range(f)]
    else:
        n = 300_000
        w = rng.integers(0, f + 1, size=n)
        M = (np.argsort(rng.random((n, f)), axis=1) < w[:, None]).astype(np.uint8)
        cols = [M[:, i].copy() for i in range(f)]
    ones = sum(c.astype(np.int32) for c in cols)
    out = _run_network_columns(ops, cols)
    for i in range(f):
        assert np.array_equal(out[i], (ones > f - 1 - i).astype(np.uint8)), i
    vals = rng.integers(0, 7, size=(f, 50_000)).astype(np.int32)
    out = _run_network_columns(ops, [vals[i].copy() for i in range(f)])
    assert np.array_equal(np.stack(out), np.sort(vals, axis=0))
    prog = gen_selnet.streamed_program(f, True)
    assert len([s_ for s_ in prog if s_[0] == "ce"]) == len(ops)
    for depth in gen_selnet.DEPTHS:
        for _ in range(20):
            v = rng.integers(0, 60, size=f).tolist()
            assert gen_selnet.run_streamed(prog, v, depth) == sorted(v)


@pytest.mark.parametrize("f", gen_selnet.STREAMED_SIZES)
def test_streamed_program_is_the_same_network_in_a_valid_order(f):
    # the single-pass kernel runs the network interleaved with its file loop: every depth's
    # program must use a file only after loading it, and select the median
    prog = gen_selnet.streamed_program(f)
    ops, wire = gen_selnet.best_network(f)
    assert [s[1:] for s in prog if s[0] == "ce"].__len__() == len(ops)
    rng = np.random.default_rng(f)
    for depth in gen_selnet.DEPTHS:
        loads = [s[2] for s in prog if s[0] == "load" and s[1] == depth]
        assert loads == list(range(f))
        for _ in range(200):
            vals = rng.integers(0, 60, size=f).tolist()
            assert gen_selnet.run_streamed(prog, vals, depth) == sorted(vals)[(f - 1) // 2]


def test_worst_case_edges_and_threaded_search():
    asg = _build("mols", 5, 3)
    assert B.byz_worst_case(asg, 0) == ((), 0, 0)
    S, c, mask = B.byz_worst_case(asg, asg.K)
    assert S == tuple(range(asg.K)) and c == asg.f and mask == (1 << asg.f) - 1
    # a search large enough for the multi-threaded path must return what the one-thread
    # oracle enumeration returns, including the first maximiser: C(25,9) = 2.0e6 (1 thread)
    # and C(25,12) = 5.2e6 are below the threshold, C(35,8) = 2.35e7 is above
    big = _build("mols", 7, 5)
    S, c, mask = B.byz_worst_case(big, 8)
    c_o, S_o = C.worst_case(_H(big), 8)
    assert (c, S) == (c_o, S_o) and c == 8
    # beyond the last row the paper could compute (q = 13): still below Claim 1's bound
    S14, c14, _ = B.byz_worst_case(big, 14)
    assert 20 <= c14 <= B.byz_gamma_bound(big, 14) and len(O.distorted_files(_H(big), S14)) == c14


@pytest.mark.parametrize("name", sorted(TABLES))
def test_frc_comparison_column(name):
    # Sec. 5.3.1: under the worst-case attack FRC loses floor(q / r') groups, i.e.
    # eps_FRC = floor(q / r') * r / K -- the FRC column of Tables 3-6, here by exhaustive search
    # on the FRC graph itself (library) and on the oracle's construction
    scheme, a, b, rows = TABLES[name]
    ref = _build("mols" if scheme == "mols" else "ram", a, b)
    K, r = ref.K, ref.r
    frc = B.byz_build_assignment(B.BYZ_SCHEME_FRC, K, r)
    assert (frc.K, frc.f, frc.l, frc.r) == (K, K // r, 1, r)
    Ho = O.frc_biadjacency(K, r)
    assert np.array_equal(_H(frc), Ho)
    assert np.array_equal(frc.file_rows(), O.file_rows(Ho))
    rp = (r + 1) // 2
    for q, _, _, _, eps_frc, _ in rows:
        if math.comb(K, q) > 3_000_000_000:
            continue
        S, c, mask = B.byz_worst_case(frc, q)
        assert c == min(q // rp, K // r)
        assert abs(c / frc.f - eps_frc) < 0.0051
        if math.comb(K, q) < 300_000:
            assert C.worst_case(Ho, q) == (c, S)
    with pytest.raises(B.ByzError):
        B.byz_build_assignment(B.BYZ_SCHEME_FRC, 15, 4)


@pytest.mark.parametrize("scheme,a,b,qs", [
    ("mols", 5, 3, range(0, 9)), ("mols", 7, 3, range(2, 8)), ("mols", 7, 5, (6, 8)),
    ("ram", 5, 5, range(2, 9)), ("ram", 5, 3, range(2, 7)), ("ram", 3, 5, range(2, 6)),
    ("ram", 5, 7, range(2, 8)), ("ram", 5, 13, (2, 4)), ("frc", 15, 3, range(1, 7)),
    ("frc", 25, 5, (5, 7)), ("mols", 4, 3, range(2, 6)), ("mols", 8, 3, (3, 5)),
    ("mols", 9, 3, range(2, 6)), ("mols", 11, 3, (3, 4))])
def test_symmetry_reduced_search_equals_the_exhaustive_one(scheme, a, b, qs):
    # Sec. 5.3.2's search over one representative per orbit of the design's translations, then
    # the first maximiser by an early-exit walk: same value, same first set, same file mask
    code = {"mols": B.BYZ_SCHEME_MOLS, "ram": B.BYZ_SCHEME_RAMANUJAN, "frc": B.BYZ_SCHEME_FRC}[scheme]
    asg = B.byz_build_assignment(code, a, b)
    fewer = 0
    for q in qs:
        plain = B.byz_worst_case(asg, q, B.BYZ_SEARCH_EXHAUSTIVE)
        v_plain = B.byz_worst_case_last_visited()
        assert v_plain == (math.comb(asg.K, q) if q > 0 else 0)
        reduced = B.byz_worst_case(asg, q, B.BYZ_SEARCH_SYMMETRY)
        v_reduced = B.byz_worst_case_last_visited()
        assert reduced == plain, q
        assert B.byz_worst_case(asg, q) == plain
        fewer += v_reduced < v_plain
    assert fewer >= len(list(qs)) - 2  # q <= 1 has nothing to reduce


def test_symmetry_reduced_search_on_the_largest_table_row():
    # Table 5's last row, C(35,13) = 1.48e9 subsets: a fifth of them visited, same answer as
    # the table; the default strategy picks the reduced search at this size
    big = _build("mols", 7, 5)
    S, c, mask = B.byz_worst_case(big, 13)
    assert c == 20 and B.byz_worst_case_last_visited() < 0.3 * math.comb(35, 13)
    S12, c12, _ = B.byz_worst_case(big, 12, B.BYZ_SEARCH_EXHAUSTIVE)
    assert (S12, c12) == B.byz_worst_case(big, 12, B.BYZ_SEARCH_SYMMETRY)[:2] and c12 == 16
    for flags in (3, 4, 8):
        with pytest.raises(B.ByzError) as e:
            B.byz_worst_case(big, 3, flags)
        assert e.value.code == -1


def test_binding_refuses_row_tables_that_point_outside_the_matrix():
    # the kernels do not range-check row numbers; the binding does, before anything is launched
    # (the check comes first, so it can be exercised here with host tensors and no GPU)
    import torch
    X = torch.zeros((75, 64), dtype=torch.float32)
    good = torch.arange(75, dtype=torch.int32)
    for bad in (good.clone().index_fill_(0, torch.tensor([7]), 75),
                good.clone().index_fill_(0, torch.tensor([74]), -1),
                good + 1):
        with pytest.raises(ValueError, match="names rows"):
            B.byz_vote(X, 64, bad, 25, 3)
        with pytest.raises(ValueError, match="names rows"):
            B.byz_aggregate(X, 64, bad, 25, 3)
        with pytest.raises(ValueError, match="names rows"):
            B.byz_aggregate_static(X, 64, bad, 25, 3, torch.zeros(64), torch.zeros(25, dtype=torch.int32))
        for fn in (lambda t: B.byz_median(X, 64, t[:25]), lambda t: B.byz_trimmed_mean(X, 64, t[:25], 2),
                   lambda t: B.byz_multi_krum(X, 64, t[:25], 3, 20), lambda t: B.byz_bulyan(X, 64, t[:25], 3)):
            if int(bad[:25].min()) < 0 or int(bad[:25].max()) >= 75:
                with pytest.raises(ValueError, match="names rows"):
                    fn(bad)
    # a table that is too short is still refused by length, and a good one gets past the row
    # check (to the next complaint: these are host tensors)
    with pytest.raises(ValueError, match="elements"):
        B.byz_vote(X, 64, good[:74], 25, 3)
    with pytest.raises(ValueError, match="CUDA"):
        B.byz_vote(X, 64, good, 25, 3)
    # an edit in place is seen (torch's modification counter is part of the cache key)
    t = good.clone()
    with pytest.raises(ValueError, match="CUDA"):
        B.byz_median(X, 64, t[:25])
    t[3] = 1000
    with pytest.raises(ValueError, match="names rows"):
        B.byz_median(X, 64, t[:25])
