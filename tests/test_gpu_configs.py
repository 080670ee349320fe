"""GPU parity at the five workloads' full sizes, in the launch configuration bench.py times.

Configs 1-4 and two steps of config 5: every output word against the C oracle run on the
same bytes (copied back from the device).  The other steps of config 5: the oracle on a
sample of coordinates (columns gathered from the device buffer).
"""
import numpy as np
import pytest
import torch

import paper_2010_04902_amd as B
import synth
from oracle import c_oracle as C
from tests import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _full_check(w, tag):
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    out, wrep, ws = B.byz_aggregate(w.X, w.d, rows_dev, w.f, w.r)
    out_e, wrep_e, ws_e = B.byz_aggregate_opts(w.X, w.d, rows_dev, w.f, w.r,
                                               B.BYZ_AGG_EARLY_MAJORITY)
    wrep_v, wrow_v, neq_v = B.byz_vote(w.X, w.d, rows_dev, w.f, w.r)
    out_m = B.byz_median(w.X, w.d, wrow_v)
    torch.cuda.synchronize()
    path = B.byz_aggregate_path(ws)
    Xh = w.X.cpu().numpy()
    wrep_o, wrow_o, neq_o = C.vote(Xh, w.file_rows, w.d)
    out_o = C.median(Xh, wrow_o, w.d)
    del Xh
    assert np.array_equal(wrep.cpu().numpy(), wrep_o), tag
    assert np.array_equal(wrep_v.cpu().numpy(), wrep_o), tag
    assert np.array_equal(wrow_v.cpu().numpy(), wrow_o), tag
    assert np.array_equal(W.bits(neq_v), neq_o), tag
    assert np.array_equal(W.bits(out), W.bits(out_o)), tag
    assert np.array_equal(W.bits(out_e), W.bits(out_o)), tag
    assert np.array_equal(wrep_e.cpu().numpy(), wrep_o), tag
    assert B.byz_aggregate_path(ws_e) == B.BYZ_PATH_SINGLE_PASS, tag
    assert np.array_equal(W.bits(out_m), W.bits(out_o)), tag
    # every file has a majority among its copies
    assert path == B.BYZ_PATH_SINGLE_PASS, tag
    # the trimmed mean in the single pass at this size (b = c_max per side): the same words as
    # vote + byz_trimmed_mean, and within the rounding contract's bound of the fp64 oracle on
    # the head, the tail and 100,000 random coordinates
    from tests.test_gpu_parity import _assert_trimmed_mean_close
    b = min(w.cmax, (w.f - 1) // 2)
    out_t, wrep_t, ws_t = B.byz_aggregate_opts(w.X, w.d, rows_dev, w.f, w.r, B.BYZ_AGG_TRIM(b))
    out_t2 = B.byz_trimmed_mean(w.X, w.d, wrow_v, b)
    torch.cuda.synchronize()
    assert B.byz_aggregate_path(ws_t) == B.BYZ_PATH_SINGLE_PASS, tag
    assert np.array_equal(wrep_t.cpu().numpy(), wrep_o), tag
    assert torch.equal(out_t.view(torch.int32), out_t2.view(torch.int32)), tag
    rng = np.random.default_rng(w.f * 1000 + w.r)
    cols = np.unique(np.concatenate([np.arange(0, 1024), np.arange(w.d - 1024, w.d),
                                     rng.integers(0, w.d, size=100_000)]))
    cols_dev = torch.tensor(cols, dtype=torch.int64, device=DEV)
    Xs = np.ascontiguousarray(w.X[:, cols_dev].cpu().numpy())
    _assert_trimmed_mean_close(out_t[cols_dev], Xs, wrow_o, len(cols), b, tag)
    # Sec. 2: exactly the files with >= r' Byzantine copies lose the vote; the paper's c_max
    wrong = 0
    for j in range(w.f):
        byz_copies = sum(1 for k in range(w.r) if int(w.file_workers[j, k]) in w.byz)
        honest_wins = int(w.file_workers[j, wrep_o[j]]) not in w.byz
        assert honest_wins == (byz_copies < (w.r + 1) // 2), (tag, j)
        wrong += 0 if honest_wins else 1
    return wrong


@pytest.mark.parametrize("idx,padded", [(0, False), (1, False), (1, True), (2, True), (3, True),
                                        (3, False)])
def test_config_full_size(idx, padded):
    cfg = synth.CONFIGS[idx]
    ld = synth.padded_ld(cfg.d, 64) if padded else cfg.d
    w = W.from_config(cfg, DEV, ld=ld)
    assert (w.K, w.f, w.l, w.r) == (cfg.K, cfg.f, cfg.l, cfg.r) and w.cmax == cfg.cmax
    wrong = _full_check(w, cfg.name)
    assert wrong == cfg.cmax  # number of distorted files = the paper's c_max for this (graph, q)


def test_config5_twenty_steps():
    cfg = synth.CONFIGS[4]
    ld = synth.padded_ld(cfg.d, 64)
    rng = np.random.default_rng(55)
    cols = np.unique(np.concatenate([np.arange(0, 2048), np.arange(cfg.d - 2048, cfg.d),
                                     rng.integers(0, cfg.d, size=8192)])).astype(np.int64)
    cols_dev = torch.tensor(cols, device=DEV)
    prev = None
    for step in range(cfg.steps):
        w = W.from_config(cfg, DEV, step=step, ld=ld)
        if step in (0, cfg.steps - 1):
            assert _full_check(w, (cfg.name, step)) == cfg.cmax
        else:
            rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
            out, wrep, ws = B.byz_aggregate(w.X, w.d, rows_dev, w.f, w.r)
            torch.cuda.synchronize()
            Xs = w.X[:, cols_dev].contiguous().cpu().numpy()  # [R, n] sampled columns
            out_o, wrep_o, _ = C.aggregate(Xs, w.file_rows, len(cols))
            assert np.array_equal(W.bits(out[cols_dev]), W.bits(out_o)), step
            assert np.array_equal(wrep.cpu().numpy(), wrep_o), step
            assert B.byz_aggregate_path(ws) == B.BYZ_PATH_SINGLE_PASS
        # fresh gradients every step
        head = w.X[0, :64].clone()
        assert prev is None or not torch.equal(head, prev)
        prev = head
        del w


def test_table5_cluster_shape_full_size():
    # MOLS (K,f,l,r) = (35,49,7,5) of the paper's Table 5 (245 rows), q = 6 worst-case set
    # (c_max = 4), mixed ALIE / constant attack, at the ResNet-18 size
    attack = {"kind": "mixed", "z": 1.0, "value": 1e3, "file_scales": True}
    d = 11173962
    w = W.make(B.BYZ_SCHEME_MOLS, 7, 5, 6, d, attack, seed=20101004 + 35, ld=synth.padded_ld(d, 64),
               device=DEV)
    assert (w.K, w.f, w.l, w.r) == (35, 49, 7, 5) and w.cmax == 4
    assert _full_check(w, "mols7x5") == 4


def test_ramanujan_case2_cluster_full_size():
    # Ramanujan m=7 > s=5 (Sec. 4.2.1, Case 2): (K,f,l,r) = (25,35,7,5), 175 rows, q = 6
    # worst-case set, reversed gradient, at the ResNet-18 size.  No table of the paper has this
    # cluster: c_max comes from the oracle's exhaustive search.
    from oracle import byz_oracle as O
    cfg = synth.CONFIGS[6]
    w = W.from_config(cfg, DEV, ld=synth.padded_ld(cfg.d, 64))
    assert (w.K, w.f, w.l, w.r) == (25, 35, 7, 5)
    cmax_o, _ = C.worst_case(O.ramanujan_biadjacency(7, 5), cfg.q)
    assert w.cmax == cmax_o == cfg.cmax
    assert _full_check(w, cfg.name) == cmax_o


@pytest.mark.parametrize("s_,m_,q,shape", [(7, 7, 5, (49, 49, 7, 7)), (7, 9, 5, (49, 63, 9, 7)),
                                           (5, 13, 5, (25, 65, 13, 5))])
def test_ramanujan_case2_wide_clusters_full_size(s_, m_, q, shape):
    # Sec. 4.2.1, Eq. 6, Case 2 (m >= s): (K,f,l,r) = (s^2, m*s, m, s) with r = 7 and with r = 5 at
    # f > 64, at the ResNet-18 size (343, 441 and 325 rows); single-pass kernels with seven copies
    # of a file in flight resp. 65 keys.  c_max from the library's search (no table has these).
    free_bytes, _ = torch.cuda.mem_get_info()
    d = 11173962
    if free_bytes < (shape[1] * shape[3] + 2 * shape[1] + 8) * 4 * d:
        pytest.skip("needs more device memory")
    attack = {"kind": "mixed", "z": 1.0, "value": 1e3, "file_scales": True}
    w = W.make(B.BYZ_SCHEME_RAMANUJAN, s_, m_, q, d, attack, seed=20101004 + 10 * s_ + m_,
               ld=synth.padded_ld(d, 64), device=DEV)
    assert (w.K, w.f, w.l, w.r) == shape and B.byz_aggregate_has_single_pass(w.f, w.r)
    assert _full_check(w, "ram%dx%d" % (s_, m_)) == w.cmax
    del w
    torch.cuda.empty_cache()


@pytest.mark.parametrize("idx,shape", [(11, (33, 121, 11, 3)), (12, (39, 169, 13, 3))])
def test_mols_over_f11_and_f13_full_size(idx, shape):
    # MOLS over F_11 and F_13 at the ResNet-18 size (363 and 507 rows, 16 and 23 GB): the
    # single pass with one word per thread on the 121- and 169-wire networks, median and
    # trimmed mean, in the launch configuration the measurements use
    cfg = synth.CONFIGS[idx]
    free_bytes, _ = torch.cuda.mem_get_info()
    if free_bytes < (cfg.f * cfg.r + 2 * cfg.f + 8) * 4 * cfg.d:
        pytest.skip("needs more device memory")
    w = W.from_config(cfg, DEV, ld=synth.padded_ld(cfg.d, 64))
    assert (w.K, w.f, w.l, w.r) == shape and w.cmax == cfg.cmax
    assert B.byz_aggregate_has_single_pass(w.f, w.r)
    assert _full_check(w, cfg.name) == cfg.cmax
    del w
    torch.cuda.empty_cache()


def test_widest_cluster_full_size():
    # 255 files (Ramanujan Case 2, s = 3, m = 85: (K,f,l,r) = (9,255,85,3)), 765 rows of the
    # ResNet-18 size: no single pass at this width, so byz_aggregate runs the vote kernel and the
    # two-wave median over the 255 winners.  The vote is checked in full, the median and the
    # trimmed mean on the head, the tail and 60,000 random coordinates
    from tests.test_gpu_parity import _assert_trimmed_mean_close
    cfg = synth.CONFIGS[13]
    free_bytes, _ = torch.cuda.mem_get_info()
    if free_bytes < (cfg.f * cfg.r + 2 * cfg.f + 8) * 4 * cfg.d:
        pytest.skip("needs more device memory")
    w = W.from_config(cfg, DEV, ld=synth.padded_ld(cfg.d, 64))
    assert (w.K, w.f, w.l, w.r) == (9, 255, 85, 3) and w.cmax == cfg.cmax
    assert not B.byz_aggregate_has_single_pass(w.f, w.r)
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    out, wrep, ws = B.byz_aggregate(w.X, w.d, rows_dev, w.f, w.r)
    out_t, wrep_t, _ = B.byz_aggregate_opts(w.X, w.d, rows_dev, w.f, w.r, B.BYZ_AGG_TRIM(w.cmax))
    torch.cuda.synchronize()
    assert B.byz_aggregate_path(ws) == B.BYZ_PATH_TWO_STEP
    Xh = w.X.cpu().numpy()
    wrep_o, wrow_o, _ = C.vote(Xh, w.file_rows, w.d)
    del Xh
    assert np.array_equal(wrep.cpu().numpy(), wrep_o) and np.array_equal(wrep_t.cpu().numpy(), wrep_o)
    lost = sum(1 for j in range(w.f) if int(w.file_workers[j, wrep_o[j]]) in w.byz)
    assert lost == cfg.cmax
    rng = np.random.default_rng(255)
    cols = np.unique(np.concatenate([np.arange(0, 1024), np.arange(w.d - 1024, w.d),
                                     rng.integers(0, w.d, size=60_000)]))
    cols_dev = torch.tensor(cols, dtype=torch.int64, device=DEV)
    Xs = np.ascontiguousarray(w.X[:, cols_dev].cpu().numpy())
    assert np.array_equal(W.bits(out[cols_dev]), W.bits(C.median(Xs, wrow_o, len(cols))))
    _assert_trimmed_mean_close(out_t[cols_dev], Xs, wrow_o, len(cols), w.cmax, cfg.name)
    del w
    torch.cuda.empty_cache()


def test_prime_power_cluster_full_size():
    # MOLS over F_9: (K,f,l,r) = (27,81,9,3), 243 rows of the ResNet-18 size, q = 5 worst-case
    # set, ALIE.  f > 64: pair bits in two 64-file groups, 81-wire network with two words a thread.
    from oracle import byz_oracle as O
    cfg = synth.CONFIGS[7]
    w = W.from_config(cfg, DEV, ld=synth.padded_ld(cfg.d, 64))
    assert (w.K, w.f, w.l, w.r) == (27, 81, 9, 3)
    cmax_o, S_o = C.worst_case(O.mols_biadjacency(9, 3), cfg.q)
    assert w.cmax == cmax_o == cfg.cmax and tuple(w.byz) == S_o
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    out, wrep, ws = B.byz_aggregate(w.X, w.d, rows_dev, w.f, w.r)
    wrep_v, wrow_v, neq_v = B.byz_vote(w.X, w.d, rows_dev, w.f, w.r)
    out_m = B.byz_median(w.X, w.d, wrow_v)
    torch.cuda.synchronize()
    Xh = w.X.cpu().numpy()
    wrep_o, wrow_o, neq_o = C.vote(Xh, w.file_rows, w.d)
    out_o = C.median(Xh, wrow_o, w.d)
    del Xh
    assert np.array_equal(wrep.cpu().numpy(), wrep_o) and np.array_equal(wrep_v.cpu().numpy(), wrep_o)
    assert np.array_equal(wrow_v.cpu().numpy(), wrow_o) and np.array_equal(W.bits(neq_v), neq_o)
    assert np.array_equal(W.bits(out), W.bits(out_o))
    assert np.array_equal(W.bits(out_m), W.bits(out_o))
    lost = sum(1 for j in range(w.f) if int(w.file_workers[j, wrep_o[j]]) in w.byz)
    assert lost == cmax_o


@pytest.mark.parametrize("idx", [1, 2])
def test_trimmed_mean_full_size(idx):
    # trimmed mean (b = c_max per side) over the vote winners at full size, fp64 oracle,
    # tolerance n * 2^-24 * max|kept| (see tests/test_gpu_parity.py)
    from tests.test_gpu_parity import _trimmed_mean_check
    cfg = synth.CONFIGS[idx]
    w = W.from_config(cfg, DEV, ld=synth.padded_ld(cfg.d, 64))
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    _, wrow, _ = B.byz_vote(w.X, w.d, rows_dev, w.f, w.r)
    torch.cuda.synchronize()
    _trimmed_mean_check(w.X, wrow.cpu().numpy(), w.d, cfg.cmax, cfg.name)


def test_multi_krum_full_size():
    # Multi-Krum over the vote winners of workload 2 (c = c_max = 5, m = f - c = 20) at full
    # size: 11,173,962 coordinates = 43,649 chunks, 86 per block
    from tests.test_gpu_parity import _multi_krum_check
    cfg = synth.CONFIGS[1]
    w = W.from_config(cfg, DEV, ld=synth.padded_ld(cfg.d, 64))
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    _, wrow, _ = B.byz_vote(w.X, w.d, rows_dev, w.f, w.r)
    torch.cuda.synchronize()
    _multi_krum_check(w.X, wrow.cpu().numpy(), w.d, cfg.cmax, w.f - cfg.cmax, cfg.name)


def test_multi_krum_81_files():
    # Multi-Krum over the 81 vote winners of the F_9 cluster (six row tiles in the Gram kernel,
    # two distances per lane in the row sort), c = c_max = 8, m = f - c = 73; 3,000,001
    # coordinates (24 chunks per block and a ragged last one) keep the fp64 oracle to seconds
    from tests.test_gpu_parity import _multi_krum_check
    cfg = synth.CONFIGS[7]
    d = 3000001
    w = W.make(cfg.scheme, cfg.a, cfg.b, cfg.q, d, cfg.attack, cfg.seed, ld=synth.padded_ld(d, 64),
               device=DEV)
    assert w.f == 81 and w.cmax == cfg.cmax
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    _, wrow, _ = B.byz_vote(w.X, w.d, rows_dev, w.f, w.r)
    torch.cuda.synchronize()
    _multi_krum_check(w.X, wrow.cpu().numpy(), w.d, cfg.cmax, w.f - cfg.cmax, cfg.name)


def test_bulyan_full_size():
    # Bulyan over the vote winners of workload 2 (f = 25, c = c_max = 5: theta = 15, beta = 5)
    # at full size, against the plain-C oracle
    from tests.test_gpu_parity import _bulyan_check
    # per-file gradient scales (as in workload 4) keep the honest vectors' scores apart, so the
    # chosen order is decided and the whole output is compared
    cfg = synth.CONFIGS[1]
    attack = dict(cfg.attack, file_scales=True)
    w = W.make(cfg.scheme, cfg.a, cfg.b, cfg.q, cfg.d, attack, cfg.seed,
               ld=synth.padded_ld(cfg.d, 64), device=DEV)
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    _, wrow, _ = B.byz_vote(w.X, w.d, rows_dev, w.f, w.r)
    torch.cuda.synchronize()
    assert _bulyan_check(w.X, wrow.cpu().numpy(), w.d, cfg.cmax, cfg.name, big=True)


def test_tolerant_vote_full_size():
    # workload 2 with relative rounding noise on every copy: bitwise no two copies agree, the
    # tolerant vote still loses exactly the c_max files with r' Byzantine copies
    from tests.test_gpu_parity import _tolerant_check
    cfg = synth.CONFIGS[1]
    w = W.from_config(cfg, DEV, ld=synth.padded_ld(cfg.d, 64))
    gen = torch.Generator(device=DEV)
    gen.manual_seed(20101004)
    X = w.X
    for row in range(X.shape[0]):  # row by row: no second full-size buffer
        X[row, :w.d] *= 1.0 + 2e-7 * torch.randn(w.d, device=DEV, generator=gen)
    wrep_o, far_o = _tolerant_check(X, w.file_rows, w.d, w.f, w.r, 1e-6, 1e-5, cfg.name)
    lost = [j for j in range(w.f) if int(w.file_workers[j, wrep_o[j]]) in w.byz]
    assert len(lost) == cfg.cmax
    wrep_v, _, neq_v = B.byz_vote(X, w.d, torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32,
                                                       device=DEV), w.f, w.r)
    torch.cuda.synchronize()
    assert (W.bits(neq_v) == 7).all()  # the exact vote finds no two equal copies


def test_largest_d():
    # d = 2^30, the largest the entry points take (byte offsets inside a row use all 32 bits):
    # Ramanujan (s=3, m=3): (K,f,l,r) = (9,9,3,3), 27 rows of 4 GiB.  The oracle runs on sampled
    # coordinates (head, tail, random), gathered column-wise from the device buffer; the
    # winners follow from how the rows are built.
    d = 1 << 30
    asg = B.byz_build_assignment(B.BYZ_SCHEME_RAMANUJAN, 3, 3)
    rows_np = asg.file_rows()
    f, r = asg.f, asg.r
    free_bytes, _ = torch.cuda.mem_get_info()
    if free_bytes < (f * r + 3) * 4 * d:
        pytest.skip("needs %d GiB of device memory" % ((f * r + 3) * 4 * d >> 30))
    X = torch.empty((f * r, d), dtype=torch.float32, device=DEV)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(2010)
    for j in range(f):
        X[int(rows_np[j, 0])].normal_(generator=gen)
        for k in range(1, r):
            X[int(rows_np[j, k])].copy_(X[int(rows_np[j, 0])])
    # file 2: copies 0 and 1 carry the same wrong vector (they win); file 5: copy 2 differs in
    # the last word only; file 7: copy 0 differs in one word no probe sample touches; file 4:
    # copies 1 and 2 carry the same wrong vector but for one such word (three distinct copies)
    X[int(rows_np[2, 0])].mul_(-100.0)
    X[int(rows_np[2, 1])].copy_(X[int(rows_np[2, 0])])
    X[int(rows_np[5, 2]), d - 1] += 1.0
    hidden = (d // 2) + 12345
    X[int(rows_np[7, 0]), hidden] += 1.0
    X[int(rows_np[4, 1])].mul_(-100.0)
    X[int(rows_np[4, 2])].copy_(X[int(rows_np[4, 1])])
    X[int(rows_np[4, 2]), hidden + 777] += 1.0
    rows_dev = torch.tensor(rows_np.reshape(-1), dtype=torch.int32, device=DEV)
    out, wrep, ws = B.byz_aggregate(X, d, rows_dev, f, r)
    wrep_v, wrow_v, neq_v = B.byz_vote(X, d, rows_dev, f, r)
    out_m = B.byz_median(X, d, wrow_v)
    torch.cuda.synchronize()
    want_rep = np.zeros(f, dtype=np.int32)
    want_rep[7] = 1                                   # copies 1 and 2 of file 7 agree
    want_neq = np.zeros(f, dtype=np.uint32)
    want_neq[2] = 0b110                               # pairs (0,2), (1,2)
    want_neq[5] = 0b110
    want_neq[7] = 0b011                               # pairs (0,1), (0,2)
    want_neq[4] = 0b111                               # no two alike: copy 0 wins the tie
    assert np.array_equal(wrep.cpu().numpy(), want_rep)
    assert np.array_equal(wrep_v.cpu().numpy(), want_rep)
    assert np.array_equal(W.bits(neq_v), want_neq)
    # file 7 keeps a majority, so its changed word costs nothing; file 4 has none, nearly every
    # wave fed the median from copy 1 where copy 0 is the winner: one more median
    assert B.byz_aggregate_path(ws) == B.BYZ_PATH_MEDIAN_REDONE
    assert torch.equal(out.view(torch.int32), out_m.view(torch.int32))
    rng = np.random.default_rng(30)
    cols = np.unique(np.concatenate([np.arange(0, 2048), np.arange(d - 2048, d),
                                     np.array([hidden - 1, hidden, hidden + 1, hidden + 777]),
                                     rng.integers(0, d, size=200_000)]))
    cols_dev = torch.tensor(cols, dtype=torch.int64, device=DEV)
    Xs = X[:, cols_dev].cpu().numpy()
    # a vote on the sample alone cannot see the single differing words of files 5 and 7 unless
    # they were drawn, so the oracle's median runs on the winners' rows derived above
    win_rows = np.array([rows_np[j, want_rep[j]] for j in range(f)], dtype=np.int32)
    out_w = C.median(np.ascontiguousarray(Xs), win_rows, len(cols))
    assert np.array_equal(W.bits(out[cols_dev]), W.bits(out_w))
    del X, out, out_m
    torch.cuda.empty_cache()
