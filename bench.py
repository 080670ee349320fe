"""Benchmark of the ByzShield aggregation path (majority vote + coordinate-wise median) on one MI355X.

A step is one pass of the whole path (byz_aggregate: probe, single-pass vote+median kernel,
decision, gated median) over one batch of stacked worker returns that is already resident in
HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--unpadded] [--no-cpu]
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak


def kernel_code_digest():
    """sha256 of kernels.hip without // comments, blank lines and indentation: changes when the
    code does, not when a comment is reworded."""
    src = os.path.join(ROOT, "paper_2010_04902_amd", "csrc", "kernels.hip")
    lines = []
    with open(src) as fh:
        for line in fh:
            code = line.split("//", 1)[0].strip()
            if code:
                lines.append(" ".join(code.split()))
    return hashlib.sha256("\n".join(lines).encode()).hexdigest()


def _traffic_from_profiles(workload, kernel="fused_kernel"):
    """(HBM bytes per launch, where the figure comes from) from the committed rocprofv3 counter
    summary of this kernel and workload; (None, why) if there is none or the kernels' code has
    changed since the counters were taken.  Nothing is counted during the benchmark run."""
    name = "%s_%s_hbm_traffic.txt" % (kernel, workload)
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, "no counter summary profiles/%s" % name
    kv = {}
    with open(path) as fh:
        for line in fh:
            if "=" in line and not line.startswith("#"):
                k, v = line.strip().split("=", 1)
                kv[k.strip()] = v.strip()
    if kv.get("kernels_hip_code_sha256") != kernel_code_digest():
        return None, "profiles/%s is older than the kernels' code" % name
    try:
        return float(kv["hbm_bytes_per_launch"]), (
            "profiles/%s: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of this "
            "command, scaled by the calibration copy; code digest matches" % name)
    except (KeyError, ValueError):
        return None, "profiles/%s has no hbm_bytes_per_launch" % name


def _cpu_model():
    """'model name' of /proc/cpuinfo plus family/model/stepping (virtual machines often shorten
    the name) and the number of logical CPUs this process may use."""
    info = {}
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if ":" in line:
                    k, v = line.split(":", 1)
                    k = k.strip()
                    if k in ("model name", "vendor_id", "cpu family", "model", "stepping") and k not in info:
                        info[k] = v.strip()
                if len(info) == 5:
                    break
    except OSError:
        pass
    usable = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    return "%s (%s family %s model %s stepping %s), %d logical CPUs usable" % (
        info.get("model name", "unknown"), info.get("vendor_id", "?"), info.get("cpu family", "?"),
        info.get("model", "?"), info.get("stepping", "?"), usable)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload 1..14 (default 2, the headline)")
    ap.add_argument("--unpadded", action="store_true", help="row pitch ld = d instead of d rounded up to 64")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-early", action="store_true", help="skip the early-majority leg")
    ap.add_argument("--no-extra", action="store_true",
                    help="skip the adversarial, repeat and graph-replay legs (profiling runs)")
    ap.add_argument("--components", action="store_true",
                    help="also time the two-step path's kernels (byz_vote, byz_median) on their own")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU only (the path would shard by coordinate "
                 "range); --gpus %d is not supported" % args.gpus)

    import numpy as np
    import torch

    import paper_2010_04902_amd as B
    import synth

    dev = "cuda:0"
    cfg = synth.CONFIGS[args.config - 1]
    d = cfg.d
    ld = d if args.unpadded else synth.padded_ld(d, 64)
    asg = B.byz_build_assignment(cfg.scheme, cfg.a, cfg.b)
    byz, cmax, _ = B.byz_worst_case(asg, cfg.q)
    assert cmax == cfg.cmax
    rows = asg.file_rows()
    rows_dev = torch.tensor(rows.reshape(-1), dtype=torch.int32, device=dev)
    fw, wf = asg.file_workers(), asg.worker_files()

    # distinct input buffers: one per step for the multi-step workload (rotating), one otherwise
    n_buf = min(cfg.steps, 3)
    # an input that fits the 256 MB last-level cache must not be served from it step after step
    input_bytes = 4 * asg.f * asg.r * ld
    if input_bytes < (1 << 30):
        n_buf = max(n_buf, 4)
    bufs = []
    for t in range(n_buf):
        G = synth.honest_gradients(asg.f, d, cfg.seed, step=t, device=dev,
                                   file_scales=bool(cfg.attack.get("file_scales")))
        bufs.append(synth.build_copies(G, fw, wf, byz, cfg.attack, ld=ld))
        del G
    out = torch.empty(d, dtype=torch.float32, device=dev)
    wrep = torch.empty(asg.f, dtype=torch.int32, device=dev)
    ws = torch.empty(B.byz_aggregate_workspace_bytes(asg.f, asg.r), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def step(i, flags=0, on=stream):
        B.byz_aggregate_opts(bufs[i % n_buf], d, rows_dev, asg.f, asg.r, flags, out=out,
                             winner_replica=wrep, workspace=ws, stream=on)

    def timed(flags, profile=True):
        """W warm-up steps, then K timed steps; returns (ms per step, kernel ms list, byz_path)."""
        for i in range(args.warmup):
            step(i, flags)
        torch.cuda.synchronize()
        path = B.byz_aggregate_path(ws)
        if profile:
            B.byz_profile_enable(args.steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i, flags)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        kernel_ms = []
        if profile:
            kernel_ms = B.byz_profile_collect(args.steps)
            B.byz_profile_enable(0)
        return (t1 - t0) * 1e3 / args.steps, kernel_ms, path

    if args.calibration_copy:
        # a plain copy of known size: reads 2^30 bytes and writes 2^30 bytes
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        B.byz_calibration_copy(src, dst, stream=stream)
        torch.cuda.synchronize()
        assert torch.equal(src[-1024:], dst[-1024:])
        del src, dst

    single_pass = B.byz_aggregate_has_single_pass(asg.f, asg.r)
    # The timed region: K steps back to back, nothing else on the stream.  The dominant kernel's
    # duration comes from a second region of the same K steps with a HIP event before and after
    # that kernel in every step (byz_profile_enable); those events sit between the launches and
    # cost a few microseconds per step, so they stay out of the headline region.
    ms_per_step, _, path = timed(0, profile=False)
    ms_per_step_events, kernel_ms, _ = timed(0)
    coords_per_s = d / (ms_per_step * 1e-3)
    if single_pass:
        alg_bytes = 4.0 * (asg.r * asg.f + 1) * d  # every copy read once, one value written
        kernel_bytes, kernel_name = alg_bytes, "fused_kernel<%d,%d>" % (asg.f, asg.r)
    else:
        # vote kernel, then median kernel over the winners: the winners are read twice
        alg_bytes = 4.0 * ((asg.r + 1) * asg.f + 1) * d
        kernel_bytes, kernel_name = 4.0 * asg.r * asg.f * d, "vote_pairs_kernel<%d,4>" % asg.r
    result = {
        "metric": "aggregated coords/sec (vote+median)",
        "value": coords_per_s,
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "data": "synthetic",
        "config": {"workload": cfg.name, "d": d, "ld": ld, "K": asg.K, "f": asg.f, "r": asg.r,
                   "l": asg.l, "q": cfg.q, "c_max": cmax, "attack": cfg.attack["kind"],
                   "rows": asg.f * asg.r, "input_bytes": 4 * asg.f * asg.r * d, "rotating_buffers": n_buf,
                   "byz_path": int(path)},
        "step_hbm_gbps_algorithmic": alg_bytes / (ms_per_step * 1e-3) / 1e9,
        "step_hbm_frac_algorithmic": alg_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "ms_per_step_with_kernel_events": ms_per_step_events,
    }
    if kernel_ms:
        avg_ms = sum(kernel_ms) / len(kernel_ms)
        achieved = kernel_bytes / (avg_ms * 1e-3) / 1e9
        traffic, traffic_source = _traffic_from_profiles(
            cfg.name, "fused_kernel" if single_pass else "vote_pairs_kernel")
        result["roofline"] = {
            "bound": "hbm", "kernel": kernel_name,
            "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": traffic, "traffic_source": traffic_source,
            "algorithmic_bytes_per_launch": kernel_bytes,
            "avg_kernel_ms": avg_ms, "median_kernel_ms": sorted(kernel_ms)[len(kernel_ms) // 2],
            "min_kernel_ms": min(kernel_ms), "launches_timed": len(kernel_ms),
            "timed_by": "HIP events around this kernel in each of K steps on the launch stream "
                        "(second region; see ms_per_step_with_kernel_events)",
        }

    if not args.no_extra:
        # the same K-step region four more times: how much one region scatters
        result["ms_per_step_repeats"] = [timed(0, profile=False)[0] for _ in range(4)]

    # What Byzantine workers can do to the time (Sec. 2: the adversary knows everything).
    # (a) Send a vector with one word changed where the probe does not look: the file keeps its
    # majority, every wave feeds the median from a copy that equals the majority on the wave's
    # own coordinates, nothing is redone, whichever copy it is.
    # (b) In the files where they hold a majority of the copies, make their copies pairwise
    # different by one such word each: those files have no majority left, the waves still saw
    # the false copies as the largest class, and wherever Eq. 3's tie rule now picks another
    # copy the median is redone from the true winners (byz_path 1).  The price is theirs: the
    # false vector no longer wins those files.
    # `adversarial_ms_per_step` is the slowest of these; the output stays the oracle's throughout.
    byz_set = set(int(b) for b in byz)
    clean = [j for j in range(asg.f) if not any(int(w) in byz_set for w in fw[j])]
    held = [j for j in range(asg.f) if sum(int(w) in byz_set for w in fw[j]) >= (asg.r + 1) // 2]
    if single_pass and not args.no_extra and d > 1000:
        c_hidden = d // 2 + 7
        legs = []
        if clean:
            for k, key in ((1, "changed_word_in_second_copy"), (0, "changed_word_in_first_copy")):
                legs.append((key, [(int(rows[clean[0], k]), c_hidden)], {}))
        if held:
            words = []
            for j in held:
                ks = [k for k in range(asg.r) if int(fw[j][k]) in byz_set]
                words += [(int(rows[j, k]), c_hidden + 64 * i) for i, k in enumerate(ks)]
            legs.append(("false_copies_made_pairwise_different", words, {"files": len(held)}))
        for key, words, more in legs:
            saved = [[b[row, c].clone() for row, c in words] for b in bufs]
            for b in bufs:
                for row, c in words:
                    b[row, c] += 1.0
            a_ms, _, a_path = timed(0, profile=False)
            for b, vals in zip(bufs, saved):
                for (row, c), v in zip(words, vals):
                    b[row, c] = v
            result[key] = {"ms_per_step": a_ms, "byz_path": int(a_path),
                           "value": d / (a_ms * 1e-3), "unit": "coords/s", **more}
        if legs:
            result["adversarial_ms_per_step"] = max(result[key]["ms_per_step"] for key, _, _ in legs)
            result["adversarial_note"] = (
                "slowest of: one word of one copy changed off the probe's sample (costs nothing: "
                "byz_path 0); the Byzantine copies of every file they hold a majority of made "
                "pairwise different by one word each (byz_path 1 where the tie rule then picks "
                "another copy: single pass + median over the winners, and the false vector "
                "loses those files)")

    # The same steps replayed from a HIP graph (n_buf consecutive steps captured once): what is
    # left of the launch gaps between the four kernels of a step.
    if not args.no_extra:
        side = torch.cuda.Stream()
        side.wait_stream(stream)
        with torch.cuda.stream(side):
            for i in range(n_buf):
                step(i, 0, on=side)
        stream.wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(n_buf):
                step(i, 0, on=torch.cuda.current_stream())
        reps = max(args.steps // n_buf, 1)
        for _ in range(2):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / (reps * n_buf)
        result["hip_graph_replay"] = {"ms_per_step": g_ms, "value": d / (g_ms * 1e-3), "unit": "coords/s",
                                      "steps_per_graph": n_buf, "replays": reps,
                                      "step_hbm_frac_algorithmic": alg_bytes / (g_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        del graph

    # Same result with fewer bytes: r' identical copies already are the majority, so the
    # other r - r' copies of a file need not be read (BYZ_AGG_EARLY_MAJORITY).  Reported
    # beside the headline, never as `value`.
    if not args.no_early and single_pass:
        rp = (asg.r + 1) // 2
        e_ms, _, e_path = timed(B.BYZ_AGG_EARLY_MAJORITY, profile=False)
        _, e_kernel_ms, _ = timed(B.BYZ_AGG_EARLY_MAJORITY)
        e_bytes = 4.0 * (rp * asg.f + 1) * d
        e_avg = sum(e_kernel_ms) / len(e_kernel_ms) if e_kernel_ms else None
        result["early_majority"] = {
            "value": d / (e_ms * 1e-3), "unit": "coords/s", "ms_per_step": e_ms,
            "byz_path": int(e_path),
            "note": "reads r'=%d of r=%d copies of a file when the probe finds a majority class; "
                    "falls back to all r (as the headline run) if any file has none" % (rp, asg.r),
            "roofline": None if e_avg is None else {
                "bound": "hbm", "achieved": e_bytes / (e_avg * 1e-3) / 1e9, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": e_bytes / (e_avg * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                "algorithmic_bytes_per_launch_if_all_files_have_a_majority": e_bytes,
                "avg_kernel_ms": e_avg},
        }

    if args.components:
        # the separate kernels of the two-step path, each timed with events on the launch stream
        def timed_call(fn):
            for _ in range(args.warmup):
                fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(stream)
            for _ in range(args.steps):
                fn()
            b.record(stream)
            torch.cuda.synchronize()
            return a.elapsed_time(b) / args.steps
        wrep_v, wrow_v, neq_v = B.byz_vote(bufs[0], d, rows_dev, asg.f, asg.r, stream=stream)
        ms_vote = timed_call(lambda: B.byz_vote(bufs[0], d, rows_dev, asg.f, asg.r, stream=stream))
        ms_vote_tol = timed_call(lambda: B.byz_vote_tolerant(bufs[0], d, rows_dev, asg.f, asg.r, 1e-6,
                                                             1e-5, stream=stream))
        ms_med = timed_call(lambda: B.byz_median(bufs[0], d, wrow_v, out=out, stream=stream))
        ms_tm = timed_call(lambda: B.byz_trimmed_mean(bufs[0], d, wrow_v, cmax, out=out, stream=stream))
        ms_mam, mam_beta = None, max(1, asg.f - 2 * cmax)
        if asg.f <= B.BYZ_MAX_F_KRUM:
            ms_mam = timed_call(lambda: B.byz_mean_around_median(bufs[0], d, wrow_v, mam_beta, out=out,
                                                                 stream=stream))
        ms_agg_tm = timed_call(lambda: step(0, B.BYZ_AGG_TRIM(cmax)))
        mk_m = asg.f - cmax
        ms_mk = None
        if asg.f <= B.BYZ_MAX_F_KRUM:
            mk_ws = torch.empty(B.byz_multi_krum_workspace_bytes(asg.f), dtype=torch.uint8, device=dev)
            ms_mk = timed_call(lambda: B.byz_multi_krum(bufs[0], d, wrow_v, cmax, mk_m, out=out,
                                                        workspace=mk_ws, stream=stream))
        ms_bu, bu_c = None, min(cmax, (asg.f - 3) // 4)
        if asg.f <= B.BYZ_MAX_F_KRUM:
            ms_bu = timed_call(lambda: B.byz_bulyan(bufs[0], d, wrow_v, bu_c, out=out,
                                                    workspace=mk_ws, stream=stream))
        # early-majority mode when its assumption breaks (one changed word in one of the r' copies
        # it reads of a clean file): single pass, then all copies of that file are compared
        ms_revote, revote_path = None, None
        if single_pass and d > 1000 and clean:
            planted = bufs[0].clone()
            planted[int(rows[clean[0], 1]), d // 2 + 7] += 1.0
            ms_revote = timed_call(lambda: B.byz_aggregate_opts(
                planted, d, rows_dev, asg.f, asg.r, B.BYZ_AGG_EARLY_MAJORITY, out=out,
                winner_replica=wrep, workspace=ws, stream=stream))
            revote_path = int(B.byz_aggregate_path(ws))
            del planted
        # what a kernel that only reads the r*f rows the way the single pass does can reach,
        # without and with the one output row
        n_rows = asg.f * asg.r
        ms_rd = timed_call(lambda: B.byz_calibration_read_rows(bufs[0], d, n_rows, out, 0, stream=stream))
        ms_rdst = timed_call(lambda: B.byz_calibration_read_rows(bufs[0], d, n_rows, out, 1, stream=stream))
        bb = 4.0 * asg.f * d + 4.0 * (asg.f - 2 * bu_c + 1) * d  # Gram pass + theta rows + output
        kb = 4.0 * asg.f * d + 4.0 * (mk_m + 1) * d  # Gram pass over f rows + mean of m rows
        vb, mb = 4.0 * asg.r * asg.f * d, 4.0 * (asg.f + 1) * d
        result["components"] = {
            "byz_vote": {"ms": ms_vote, "algorithmic_bytes": vb, "gbps": vb / ms_vote / 1e6,
                         "frac": vb / ms_vote / 1e6 / HBM_PEAK_GBPS,
                         "note": "fill + vote_pairs_kernel + vote_decide_kernel"},
            "byz_vote_tolerant": {"ms": ms_vote_tol, "algorithmic_bytes": vb,
                                  "gbps": vb / ms_vote_tol / 1e6,
                                  "frac": vb / ms_vote_tol / 1e6 / HBM_PEAK_GBPS,
                                  "note": "copies close within 1e-6 + 1e-5*max|x| instead of identical"},
            "byz_median": {"ms": ms_med, "algorithmic_bytes": mb, "gbps": mb / ms_med / 1e6,
                           "frac": mb / ms_med / 1e6 / HBM_PEAK_GBPS},
            "byz_aggregate_trimmed_mean": {"ms": ms_agg_tm, "b": cmax, "algorithmic_bytes": alg_bytes,
                                           "gbps": alg_bytes / ms_agg_tm / 1e6,
                                           "frac": alg_bytes / ms_agg_tm / 1e6 / HBM_PEAK_GBPS,
                                           "note": "whole path with the trimmed mean instead of the median"},
            "access_pattern_ceiling": {
                "read_only_ms": ms_rd, "read_only_gbps": 4.0 * n_rows * d / ms_rd / 1e6,
                "read_and_store_ms": ms_rdst,
                "read_and_store_gbps": 4.0 * (n_rows + 1) * d / ms_rdst / 1e6,
                "read_and_store_frac": 4.0 * (n_rows + 1) * d / ms_rdst / 1e6 / HBM_PEAK_GBPS,
                "note": "byz_calibration_read_rows: the single pass's loads (and its store) with "
                        "no vote and no median; the gap between the two is what writing 1/(rf+1) "
                        "of the bytes costs"},
            "early_majority_revote": None if ms_revote is None else {
                "ms": ms_revote, "byz_path": revote_path,
                "algorithmic_bytes": 4.0 * (((asg.r + 1) // 2) * asg.f + 1) * d + 4.0 * asg.r * d,
                "note": "early-majority mode with one changed word in one of the r' copies it reads "
                        "(the second): single pass over r' copies, then all r copies of that one "
                        "file are compared; the first copy wins and is what the pass fed, no median"},
            "byz_multi_krum": None if ms_mk is None else {
                "ms": ms_mk, "c": cmax, "m": mk_m, "algorithmic_bytes": kb,
                "gbps": kb / ms_mk / 1e6, "frac": kb / ms_mk / 1e6 / HBM_PEAK_GBPS,
                "gram_tflops": 2.0 * asg.f * asg.f * d / ms_mk / 1e9,
                "note": "Gram (fp32 MFMA) + reduce + select + mean of m rows"},
            "byz_bulyan": None if ms_bu is None else {
                "ms": ms_bu, "c": bu_c, "theta": asg.f - 2 * bu_c, "beta": asg.f - 4 * bu_c,
                "algorithmic_bytes": bb, "gbps": bb / ms_bu / 1e6,
                "frac": bb / ms_bu / 1e6 / HBM_PEAK_GBPS,
                "note": "Gram + reduce + repeated Krum + mean around the median of theta rows"},
            "byz_trimmed_mean": {"ms": ms_tm, "b": cmax, "algorithmic_bytes": mb,
                                 "gbps": mb / ms_tm / 1e6, "frac": mb / ms_tm / 1e6 / HBM_PEAK_GBPS},
            "byz_mean_around_median": None if ms_mam is None else {
                "ms": ms_mam, "beta": mam_beta, "algorithmic_bytes": mb,
                "gbps": mb / ms_mam / 1e6, "frac": mb / ms_mam / 1e6 / HBM_PEAK_GBPS},
        }

    if not args.no_cpu:
        # The oracle as it stands, on the host cores of this machine: vote (memcmp per pair of copies,
        # files spread over the threads) and median (sort per coordinate, coordinates spread over
        # the threads), each timed on its own, on the whole batch.
        from oracle import c_oracle as C
        Xh = bufs[0].cpu().numpy()
        threads = C.default_threads()
        reps = 2
        best_vote = best_med = None
        for _ in range(reps):
            c0 = time.perf_counter()
            wrep_o, wrow_o, _, vote_threads = C.vote(Xh, rows, d, threads=threads)
            c1 = time.perf_counter()
            out_o = C.median(Xh, wrow_o, d, threads=threads)
            c2 = time.perf_counter()
            best_vote = (c1 - c0) if best_vote is None else min(best_vote, c1 - c0)
            best_med = (c2 - c1) if best_med is None else min(best_med, c2 - c1)
        best = best_vote + best_med
        step(0)
        torch.cuda.synchronize()
        same = bool(np.array_equal(out.cpu().numpy().view(np.uint32), out_o.view(np.uint32))
                    and np.array_equal(wrep.cpu().numpy(), wrep_o))
        # one core, on the first eighth of the coordinates (same rows, same row pitch)
        d1 = max(d // 8, 1)
        c0 = time.perf_counter()
        C.aggregate(Xh, rows, d1, threads=1)
        one_core = time.perf_counter() - c0
        result["cpu_baseline"] = {
            "value": d / best, "unit": "coords/s", "cores": int(threads), "kind": "oracle",
            "cpu_model": _cpu_model(),
            "vote_seconds": best_vote, "vote_threads": int(vote_threads),
            "median_seconds": best_med, "median_threads": int(threads),
            "one_core": {"value": d1 / one_core, "unit": "coords/s",
                         "sample": "first %d coordinates of the same batch, one run" % d1},
            "sample": "whole %s batch (d=%d, %d rows), best of %d runs of the C oracle: vote = memcmp "
                      "per pair of copies with the %d files spread over %d threads, median = sort per "
                      "coordinate with the coordinates spread over %d threads (OpenMP)"
                      % (cfg.name, d, asg.f * asg.r, reps, asg.f, vote_threads, threads),
            "seconds": best, "gpu_matches_oracle": same,
        }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
