"""byz_aggregate_static (the entry point for callers that cannot allocate: its scratch is a fixed
array in the library's device image) against byz_aggregate_opts, through the C-ABI, bit for bit.
"""
import numpy as np
import pytest
import torch

import paper_2010_04902_amd as B
import synth
from tests import workloads as W

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
MOLS, RAM = B.BYZ_SCHEME_MOLS, B.BYZ_SCHEME_RAMANUJAN
ALIE = {"kind": "alie", "z": 1.0}
MIXED = {"kind": "mixed", "z": 1.0, "value": 1e3, "file_scales": True}


def _both(w, d, flags, X=None):
    X = w.X if X is None else X
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    ref, wrep_ref, _ = B.byz_aggregate_opts(X, d, rows_dev, w.f, w.r, flags)
    out = torch.full((d,), float("nan"), dtype=torch.float32, device=DEV)
    wrep = torch.full((w.f,), -1, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()
    B.byz_aggregate_static(X, d, rows_dev, w.f, w.r, out, wrep, flags)
    torch.cuda.synchronize()
    assert np.array_equal(W.bits(out), W.bits(ref)), (d, w.f, w.r, flags)
    assert np.array_equal(wrep.cpu().numpy(), wrep_ref.cpu().numpy()), (d, w.f, w.r, flags)


def test_static_scratch_equals_caller_workspace_two_calls_in_a_row():
    # first call: 49 files, several tiles and a ragged tail; second call: a smaller input
    # (fewer files, fewer copies, fewer coordinates) on whatever the first call left behind
    big = W.make(MOLS, 7, 3, 5, 70_001, ALIE, seed=31, ld=synth.padded_ld(70_001, 4), device=DEV)
    small = W.make(MOLS, 5, 3, 4, 4_099, ALIE, seed=32, device=DEV)
    _both(big, big.d, 0)
    _both(small, small.d, 0)
    # again the other way round, with the options the single pass knows, r = 5, a two-step
    # shape (f = 27), and an input whose off-sample difference needs more than the single pass
    _both(small, small.d, B.BYZ_AGG_EARLY_MAJORITY)
    _both(big, big.d, B.BYZ_AGG_TRIM(3) | B.BYZ_AGG_EARLY_MAJORITY)
    r5 = W.make(RAM, 5, 5, 6, 30_011, MIXED, seed=33, device=DEV)
    _both(r5, r5.d, 0)
    two_step = W.make(RAM, 3, 9, 2, 2_222, ALIE, seed=34, device=DEV)
    _both(two_step, two_step.d, 0)
    P = big.X.clone()
    P[int(big.file_rows[4, 0]), big.d - 3] += 1.0  # first copy of file 4, outside the probe's sample
    _both(big, big.d, 0, X=P)
    _both(small, small.d, 0)
    _both(small, 3, 0)
    _both(small, 0, 0)


def test_static_scratch_refuses_what_it_cannot_hold():
    w = W.make(MOLS, 5, 3, 3, 100, ALIE, seed=35, device=DEV)
    rows_long = torch.zeros(300 * 9, dtype=torch.int32, device=DEV)
    out = torch.empty(100, dtype=torch.float32, device=DEV)
    wrep = torch.empty(300, dtype=torch.int32, device=DEV)
    for (f, r, code) in [(257, 3, -3), (25, 9, -3), (25, 4, -1), (24, 3, -2)]:
        with pytest.raises(B.ByzError) as e:
            B.byz_aggregate_static(w.X, 100, rows_long, f, r, out, wrep)
        assert e.value.code == code, (f, r)


def test_static_scratch_under_graph_capture():
    # the use the entry point is for: captured into a HIP graph (after a first eager call on
    # the device) and replayed, with eager calls in between; every replay gives the result of
    # byz_aggregate_opts on the same input, also when the input sends the call past the single pass
    w = W.make(MOLS, 5, 3, 4, 50_003, ALIE, seed=36, ld=synth.padded_ld(50_003, 64), device=DEV)
    rows_dev = torch.tensor(w.file_rows.reshape(-1), dtype=torch.int32, device=DEV)
    # second input: replicas 1 and 2 of file 3 hold a false vector, equal but for one word off
    # the probe's sample; without a majority replica 0 wins the tie and the median is redone
    X2 = w.X.clone()
    X2[int(w.file_rows[3, 1]), :w.d] = -50.0 * w.G[3]
    X2[int(w.file_rows[3, 2])] = X2[int(w.file_rows[3, 1])]
    X2[int(w.file_rows[3, 2]), 33_333] += 1.0
    want = []
    for X in (w.X, X2):
        o, r_, ws_ = B.byz_aggregate_opts(X, w.d, rows_dev, w.f, w.r, 0)
        want.append((o.clone(), r_.clone(), B.byz_aggregate_path(ws_)))
    torch.cuda.synchronize()
    assert [p for _, _, p in want] == [B.BYZ_PATH_SINGLE_PASS, B.BYZ_PATH_MEDIAN_REDONE]
    Xs = w.X.clone()
    out = torch.empty(w.d, dtype=torch.float32, device=DEV)
    wrep = torch.empty(w.f, dtype=torch.int32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.byz_aggregate_static(Xs, w.d, rows_dev, w.f, w.r, out, wrep, 0)   # first call: eager
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.byz_aggregate_static(Xs, w.d, rows_dev, w.f, w.r, out, wrep, 0)
    for rep, which in enumerate([0, 1, 1, 0]):
        Xs.copy_((w.X, X2)[which])
        out.zero_()
        wrep.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.view(torch.int32), want[which][0].view(torch.int32)), (rep, which)
        assert torch.equal(wrep, want[which][1]), (rep, which)
        o2 = torch.empty_like(out)
        r2 = torch.empty_like(wrep)
        B.byz_aggregate_static((w.X, X2)[1 - which], w.d, rows_dev, w.f, w.r, o2, r2, 0)  # eager, other input
        torch.cuda.synchronize()
        assert torch.equal(o2.view(torch.int32), want[1 - which][0].view(torch.int32)), (rep, which)
    assert want[1][1][3].item() == 0
