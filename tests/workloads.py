"""Builds one aggregation workload (graph, Byzantine set, stacked returns) for the tests."""
import numpy as np
import torch

import paper_2010_04902_amd as B
import synth


class Workload:
    pass


def make(scheme, a, b, q, d, attack, seed, step=0, ld=None, device="cpu", byz=None):
    """scheme: 0 MOLS (l, r) / 1 Ramanujan (s, m).  The graph and the worst-case set come from
    the library (both are checked against the oracle in the host tests)."""
    w = Workload()
    asg = B.byz_build_assignment(scheme, a, b)
    w.asg, w.K, w.f, w.l, w.r, w.d = asg, asg.K, asg.f, asg.l, asg.r, d
    w.file_rows = asg.file_rows()
    w.file_workers = asg.file_workers()
    w.worker_files = asg.worker_files()
    if byz is None:
        byz, w.cmax, _ = B.byz_worst_case(asg, q)
    w.byz = tuple(byz)
    w.G = synth.honest_gradients(w.f, d, seed, step=step, device=device,
                                 file_scales=bool(attack.get("file_scales")))
    w.X = synth.build_copies(w.G, w.file_workers, w.worker_files, w.byz, attack, ld=ld)
    w.ld = w.X.shape[1]
    return w


def from_config(cfg, device, step=0, d=None, ld=None):
    return make(cfg.scheme, cfg.a, cfg.b, cfg.q, cfg.d if d is None else d, cfg.attack, cfg.seed,
                step=step, ld=ld, device=device)


def bits(t):
    """float32/int32 torch tensor or numpy array -> numpy uint32 view on the host."""
    if isinstance(t, torch.Tensor):
        t = t.detach().cpu().numpy()
    return np.ascontiguousarray(t).view(np.uint32)
