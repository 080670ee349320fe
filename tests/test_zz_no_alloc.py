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
