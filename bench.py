#!/usr/bin/env python3
"""Throughput of the draft-then-verify exploration path on one MI355X.

A step is one pass of the whole path over one synthetic population, inputs resident in HBM:
    pruner_prior_filter (= draft score of every candidate, then the draft set) -> pruner_verify_score -> pruner_topk (final set)
The workload is the stress population (16M candidates of an fp16 GEMM 4096^3 in fragment mode + 4M of a
depthwise conv, draft top-4096 per subgraph, verify, final top-32); --config picks another one.
The statement features of the drafted candidates are an input of the verify stage (a compiler's feature
extractor makes them); they are generated once, before timing, from the drafted ids.

Prints ONE JSON line.  `value` is draft-scored candidates per second over the whole step.  `roofline` describes
the dominant kernel (the draft-score kernel: one launch per loop-nest class of the population, after one small
table-upload launch), timed as a whole with events on the launch stream inside the timed steps.
`cpu_baseline` is the CPU oracle, as it stands, on a bounded sample of the same workload on this host.
"""
import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
# HBM bytes per launch of the draft kernel from rocprofv3 counters (profiles/draft_kernel_cfg4_traffic.txt), valid for
# the kernel source with this SHA-256 only; any other source reports null.
MEASURED_TRAFFIC = {"workload": "cfg4_stress_gemm4096_dwconv_20M", "source_sha256": "6a84ef97fd50e1561e3d8008b6c2fff259857a61dbff70a329c80d27f6af7c4d",
                    "bytes": 588933196, "dominant_bytes": 403769839}


def draft_traffic(workload, which="bytes"):
    import hashlib
    src = os.path.join(ROOT, "paper_2402_02361_amd", "csrc", "draft_score.hip")
    if MEASURED_TRAFFIC.get(which) is None or workload != MEASURED_TRAFFIC["workload"] or not os.path.exists(src):
        return None
    digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    return MEASURED_TRAFFIC[which] if digest == MEASURED_TRAFFIC["source_sha256"] else None

# One VALU instruction retires 64 lanes in 4 cycles on a 16-lane SIMD: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz.
# (The published 157.3 TFLOP/s fp32 vector figure counts packed dual-issue FMAs: 4x this lane rate.)
VALU_PEAK_GLANEOPS = 256 * 4 * 16 * 2.4


def algorithmic_bytes(wl, w):
    """Bytes the draft-score kernel must move: one uint16 per tile slot in, one float out, per candidate."""
    total = 0
    for t, sg in enumerate(wl.subgraphs):
        cnt = int(wl.seg_off[t + 1] - wl.seg_off[t])
        total += cnt * (2 * w.n_slots(sg) + 4)
    return total


def cpu_baseline(idx, w, oracle, scale):
    """The oracle on a scaled-down copy of the workload, single thread."""
    wl = w.make_config(idx, scale=scale)
    m = w.make_mlp_weights(seed=1)
    t0 = time.perf_counter()
    s32, _, _ = oracle.draft_score(wl.subgraphs, wl.seg_off, wl.tiles)
    ids, _ = oracle.topk(s32, wl.seg_off, wl.k_draft)
    t1 = time.perf_counter()
    n_ver = 0
    if wl.verify:
        n_stmt = np.repeat(np.array(wl.n_stmt, np.int32), wl.k_draft)
        feat = w.make_statement_features(ids.reshape(-1), n_stmt, seed=wl.seed)
        t1 = time.perf_counter()       # feature synthesis is input generation, not the path
        t_draft = t1 - t0
        vs, _ = oracle.verify(feat, n_stmt, m, want_f64=False)
        seg2 = np.arange(len(wl.subgraphs) + 1, dtype=np.int64) * wl.k_draft
        oracle.topk(vs, seg2, wl.k_final)
        t2 = time.perf_counter()
        n_ver = len(n_stmt)
        total = t_draft + (t2 - t1)
    else:
        total = t1 - t0
    return {
        "value": wl.n / total, "unit": "candidates/s", "cores": 1, "kind": "oracle",
        "sample": f"{wl.name} at scale {scale:g}: {wl.n} candidates scored, top-{wl.k_draft} per subgraph, "
                  f"{n_ver} drafted candidates verified; {total:.1f} s of CPU work",
    }


def cpu_baseline_all_cores(idx, w, oracle, scale, cores):
    """The same oracle on the same sample with its draft and verify loops cut into candidate ranges, one range per
    thread (the C oracle runs outside the interpreter lock); the selections stay single calls."""
    from concurrent.futures import ThreadPoolExecutor
    wl = w.make_config(idx, scale=scale)
    m = w.make_mlp_weights(seed=1)
    pieces = []
    for t, sg in enumerate(wl.subgraphs):
        a, b = int(wl.seg_off[t]), int(wl.seg_off[t + 1])
        cuts = np.linspace(a, b, max(1, min(cores, (b - a) // 4096 + 1)) + 1).astype(np.int64)
        pieces += [(sg, int(lo), int(hi)) for lo, hi in zip(cuts[:-1], cuts[1:]) if hi > lo]
    s32 = np.empty(wl.n, np.float32)

    def score_piece(p):
        sg, lo, hi = p
        s32[lo:hi] = oracle.draft_score([sg], [0, hi - lo], wl.tiles[:, lo:hi])[0]

    t0 = time.perf_counter()
    with ThreadPoolExecutor(cores) as pool:
        list(pool.map(score_piece, pieces))
        ids, _ = oracle.topk(s32, wl.seg_off, wl.k_draft)
        t1 = time.perf_counter()
        total = t1 - t0
        if wl.verify:
            n_stmt = np.repeat(np.array(wl.n_stmt, np.int32), wl.k_draft)
            feat = w.make_statement_features(ids.reshape(-1), n_stmt, seed=wl.seed)
            vs = np.empty(len(n_stmt), np.float32)
            cuts = np.linspace(0, len(n_stmt), cores + 1).astype(np.int64)

            def verify_piece(i):
                lo, hi = int(cuts[i]), int(cuts[i + 1])
                if hi > lo:
                    vs[lo:hi] = oracle.verify(feat[lo:hi], n_stmt[lo:hi], m, want_f64=False)[0]

            t2 = time.perf_counter()
            list(pool.map(verify_piece, range(cores)))
            oracle.topk(vs, np.arange(len(wl.subgraphs) + 1, dtype=np.int64) * wl.k_draft, wl.k_final)
            total += time.perf_counter() - t2
    return {"value": wl.n / total, "unit": "candidates/s", "cores": cores, "kind": "oracle",
            "sample": f"{wl.name} at scale {scale:g}, draft and verify loops split into candidate ranges over {cores} threads; "
                      f"{total:.1f} s of wall time"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, help="workload 0..4 (default: the stress population)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-scale", type=float, default=None, help="fraction of the workload the CPU oracle is timed on")
    ap.add_argument("--lse-steps", type=int, default=4,
                    help="steps of the on-device explorer loop (pruner_lse) timed after the main measurement; 0 skips it")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 1 GiB device copy, so that a counter profile of this command holds a kernel of known traffic")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU; --gpus above 1 is not supported "
              "(candidates are independent: a population would be split across GPUs by segment ranges and the k best merged)", file=sys.stderr)
        sys.exit(2)

    import torch

    import oracle
    import paper_2402_02361_amd as P
    import workloads as w

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    P.load_library()
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()

    wl = w.make_config(args.config)
    m = w.make_mlp_weights(seed=1)
    n, n_sg = wl.n, len(wl.subgraphs)
    csg = P.to_c_subgraphs(wl.subgraphs)
    tiles = dev(wl.tiles)
    # two copies of the population, read in turn: whatever of one step's columns is left in the 256 MB cache in front of
    # HBM belongs to the copy that the next step does not read
    pops = [tiles, tiles.clone()]
    score = torch.empty(n, dtype=torch.float32, device="cuda")
    idx = torch.empty((n_sg, wl.k_draft), dtype=torch.int32, device="cuda")
    ws_filter = torch.empty(P.workspace_bytes(P.WS_PRIOR_FILTER, n, n_sg, wl.k_draft), dtype=torch.uint8, device="cuda")

    # untimed pre-pass: the drafted ids decide which feature rows the verify stage is given
    P.prior_filter(csg, wl.seg_off, tiles, wl.k_draft, score=score, idx_out=idx, want_values=False, workspace=ws_filter)
    torch.cuda.synchronize()
    n_d = 0
    if wl.verify:
        ids = idx.cpu().numpy().reshape(-1)
        n_stmt_h = np.repeat(np.array(wl.n_stmt, np.int32), wl.k_draft)
        feat0 = dev(w.make_statement_features(ids, n_stmt_h, seed=wl.seed))
        # the verify stage reads a different copy each step, so that the 256 MB cache in front of HBM cannot hold them
        n_copies = max(1, min(16, -(-(320 << 20) // max(feat0.numel() * 4, 1))))
        feats = [feat0] + [feat0.clone() for _ in range(n_copies - 1)]
        n_stmt = dev(n_stmt_h)
        gm = {k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in m.items()}
        n_d = len(ids)
        vscore = torch.empty(n_d, dtype=torch.float32, device="cuda")
        seg2 = np.arange(n_sg + 1, dtype=np.int64) * wl.k_draft
        fin = torch.empty((n_sg, wl.k_final), dtype=torch.int32, device="cuda")
        ws_ver = torch.empty(P.workspace_bytes(P.WS_VERIFY, n_d, 0, 0), dtype=torch.uint8, device="cuda")
        ws_topk2 = torch.empty(P.workspace_bytes(P.WS_TOPK, n_d, n_sg, wl.k_final), dtype=torch.uint8, device="cuda")

    # events of all timed steps are made beforehand; a first record creates the handle that the library is handed
    pool = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(args.steps)]
    for es in pool:
        for e in es:
            e.record()
    torch.cuda.synchronize()
    marks = []

    def step(timed, flags=0, rotate=True):
        e = pool[len(marks)] if timed else None
        if timed:
            e[0].record()
        # e[1] is recorded by the library between the draft-score launches and the selection launches
        step.calls += 1
        P.prior_filter(csg, wl.seg_off, pops[step.calls % 2 if rotate else 0], wl.k_draft, flags=flags, score=score, idx_out=idx,
                       want_values=False, workspace=ws_filter, scored_event=e[1] if timed else None)
        if timed:
            e[2].record()
        if wl.verify:
            P.verify_score(feats[step.count % len(feats)], n_stmt, gm, vscore=vscore, workspace=ws_ver)
            step.count += 1
            if timed:
                e[3].record()
            P.topk(vscore, seg2, wl.k_final, idx_out=fin, want_values=False, workspace=ws_topk2)
        if timed:
            e[4].record()
            marks.append(e)

    step.count = 0
    step.calls = 0
    dominant_bytes = ctypes.c_int64(0)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step(False)
    # The timed region: exactly --steps steps between two synchronisations.  It is run three times over and the median
    # region is reported (all three are in the line): the regions are a few milliseconds long, and a host thread that the
    # operating system parks for a few tens of milliseconds in one of them (seen once in some dozen runs on the shared
    # hosts this runs on) would otherwise decide the figure.
    regions = []
    for _ in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step(False)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        regions.append((t1 - t0) * 1e3 / args.steps)
    ms_per_step = float(np.median(regions))

    def timed_loop(**kw):
        for _ in range(args.warmup):
            step(False, **kw)
        took = []
        for _ in range(3):   # as for the headline: the median of three regions of --steps steps
            torch.cuda.synchronize()
            a = time.perf_counter()
            for _ in range(args.steps):
                step(False, **kw)
            torch.cuda.synchronize()
            took.append((time.perf_counter() - a) * 1e3 / args.steps)
        return float(np.median(took))

    # the same steps with one rounded operation per step of Eq. 1 for every population size (the draft selection is then
    # the oracle's row by row on any input), with the fused form forced, and with a single copy of the population
    ms_reference = timed_loop(flags=P.REFERENCE_ROUNDING)
    ms_fused = timed_loop(flags=P.FUSED_ARITHMETIC)
    ms_one_copy = timed_loop(rotate=False)

    # The split into stages comes from a pass of its own over the same steps, outside the timed region: the five event
    # records per step that it needs sit between dependent launches and cost about 20 us per step on this machine.
    t2 = time.perf_counter()
    for _ in range(args.steps):
        step(True)
    torch.cuda.synchronize()
    ms_per_step_with_events = (time.perf_counter() - t2) * 1e3 / args.steps

    # The dominant kernel by itself, outside the timed region (the two extra event records would widen the gaps between
    # the step's launches): the same call as in the step, the library recording e[5] and e[6] right before and after the
    # draft kernel launch that covers the most candidates.
    for e in marks:
        P.time_dominant_draft_launch(e[5], e[6], dominant_bytes)
        step.calls += 1
        P.prior_filter(csg, wl.seg_off, pops[step.calls % 2], wl.k_draft, score=score, idx_out=idx, want_values=False, workspace=ws_filter)
    P.time_dominant_draft_launch(None, None)
    torch.cuda.synchronize()

    def avg(a, b):
        return float(np.mean([e[a].elapsed_time(e[b]) for e in marks]))

    ms_draft, ms_topk = avg(0, 1), avg(1, 2)
    ms_verify = avg(2, 3) if wl.verify else 0.0
    ms_final = avg(3, 4) if wl.verify else 0.0

    abytes = algorithmic_bytes(wl, w)
    gbs = abytes / (ms_draft * 1e-3) / 1e9
    ms_dominant = avg(5, 6)
    dom_gbs = dominant_bytes.value / (ms_dominant * 1e-3) / 1e9
    out = {
        "metric": "draft-scored candidates/sec over the whole draft-then-verify step",
        "value": n / (ms_per_step * 1e-3),
        "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "ms_per_step_of_each_timed_region": regions,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "candidates": n, "subgraphs": n_sg, "k_draft": wl.k_draft,
                   "verified": n_d, "k_final": wl.k_final},
        "arithmetic": {"timed": "default: reference rounding in single-launch calls (below 2^20 candidates), fused form above",
                       "ms_per_step_reference_rounding": ms_reference, "value_reference_rounding": n / (ms_reference * 1e-3),
                       "ms_per_step_fused": ms_fused,
                       "draft_selection_vs_oracle": "row by row equal on this workload in either form (tests/test_gpu_parity.py)"},
        "ms_per_step_single_population_copy": ms_one_copy,
        "stages_ms": {"draft_score": ms_draft, "draft_topk": ms_topk, "verify_mlp": ms_verify, "final_topk": ms_final},
        "stages_from": "a second pass over the same steps with five event records per step (ms_per_step there: %.4f)" % ms_per_step_with_events,
        "draft_candidates_per_s": n / (ms_draft * 1e-3),
        "draft_and_select_candidates_per_s": n / ((ms_draft + ms_topk) * 1e-3),
        "verify_candidates_per_s": (n_d / (ms_verify * 1e-3)) if wl.verify else None,
        "verify_and_select_candidates_per_s": (n_d / ((ms_verify + ms_final) * 1e-3)) if wl.verify else None,
        "roofline": {"kernel": "draft_kernel, the launch that covers the most candidates (one launch per loop-nest class; events recorded "
                               "by the library right before and after that launch)",
                     "bound": "hbm", "achieved": dom_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dom_gbs / HBM_PEAK_GBS,
                     "traffic": draft_traffic(wl.name, "dominant_bytes"), "algorithmic_bytes": dominant_bytes.value,
                     "avg_launch_ms": ms_dominant},
        "roofline_draft_stage": {"what": "all of pruner_draft_score's launches: table upload + one draft_kernel launch per loop-nest class, "
                                         "with the gaps between them", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS,
                                 "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": draft_traffic(wl.name),
                                 "algorithmic_bytes": abytes, "avg_ms": ms_draft},
    }
    # draft + draft selection as one HBM-bound stage: the draft stage's bytes, the scores read once more, the k best written
    sel_bytes = abytes + 4 * n + 8 * wl.k_draft * n_sg
    sel_gbs = sel_bytes / ((ms_draft + ms_topk) * 1e-3) / 1e9
    out["roofline_draft_and_select"] = {"what": "pruner_prior_filter as a whole: the draft stage plus the selection's launches; algorithmic bytes = "
                                                "the draft stage's, 4 per candidate for one more pass over the scores, 8 k per subgraph out",
                                        "bound": "hbm", "achieved": sel_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": sel_gbs / HBM_PEAK_GBS,
                                        "algorithmic_bytes": sel_bytes, "avg_ms": ms_draft + ms_topk}
    if wl.verify:
        rows = int(n_stmt_h.sum())
        flops = rows * 2 * (164 * 256 + 256 * 256 + 256)
        tf = flops / (ms_verify * 1e-3) / 1e12
        out["roofline_verify"] = {"kernel": "mlp_kernel (one launch: row numbering, three layers on the matrix cores, statement sums)", "bound": "mfma", "achieved": tf,
                                  "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0, "valid_rows": rows,
                                  "avg_call_ms": ms_verify}
        # the same kernel on sets large enough to keep every CU busy for many tiles (a caller verifying several rounds'
        # drafted sets at once): what it sustains when the launch, the weights' way into registers and the first rows'
        # way from memory (about 10 us per call at any size) are spread over 36 tiles per compute unit (16 x) or 144 (64 x)
        def steady(times):
            big_d = times * n_d
            rng = np.random.default_rng(7)
            big_stmt_h = rng.choice(np.array(wl.n_stmt, np.int32), size=big_d).astype(np.int32)
            big_feat = torch.rand((big_d, 8, 164), device="cuda") * 24.0
            big_stmt = dev(big_stmt_h)
            big_vs = torch.empty(big_d, dtype=torch.float32, device="cuda")
            big_ws = torch.empty(P.workspace_bytes(P.WS_VERIFY, big_d, 0, 0), dtype=torch.uint8, device="cuda")
            P.verify_score(big_feat, big_stmt, gm, vscore=big_vs, workspace=big_ws)
            torch.cuda.synchronize()
            b0, b1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            b0.record()
            for _ in range(5):
                P.verify_score(big_feat, big_stmt, gm, vscore=big_vs, workspace=big_ws)
            b1.record()
            torch.cuda.synchronize()
            big_ms = b0.elapsed_time(b1) / 5
            big_rows = int(big_stmt_h.sum())
            big_tf = big_rows * 2 * (164 * 256 + 256 * 256 + 256) / (big_ms * 1e-3) / 1e12
            del big_feat
            return {"candidates": big_d, "valid_rows": big_rows, "avg_call_ms": big_ms, "bound": "mfma", "achieved": big_tf, "peak": 2500.0,
                    "unit": "TFLOP/s", "frac": big_tf / 2500.0, "feature_GBps": big_rows * 656 / (big_ms * 1e-3) / 1e9,
                    "note": "one launch; features of this set (%.0f MB) exceed the 256 MB cache; fp32 feature rows put the stage at "
                            "the HBM ridge" % (big_d * 8 * 164 * 4 / 1e6)}
        if n_d:
            out["roofline_verify_steady"] = steady(16)
            out["roofline_verify_steady_64x"] = steady(64)
    if args.lse_steps > 0:
        # the explorer loop of Alg. 2 on the same population (a copy: the loop rewrites it); not part of `value`
        q16 = 52000
        ws_lse = torch.empty(P.workspace_bytes(P.WS_LSE, n, n_sg, wl.k_draft), dtype=torch.uint8, device="cuda")
        pop = tiles.clone()
        P.lse(csg, wl.seg_off, pop, wl.k_draft, args.lse_steps, 1, q16, score=score, workspace=ws_lse)
        pop.copy_(tiles)
        torch.cuda.synchronize()
        l0, l1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        l0.record()
        _, _, _, spec_n = P.lse(csg, wl.seg_off, pop, wl.k_draft, args.lse_steps, 1, q16, score=score, workspace=ws_lse)
        l1.record()
        torch.cuda.synchronize()
        lse_ms = l0.elapsed_time(l1)
        out["lse"] = {"steps": args.lse_steps, "k": wl.k_draft, "mutate_q16": q16, "ms_per_step": lse_ms / args.lse_steps,
                      "candidates_per_s": n * args.lse_steps / (lse_ms * 1e-3), "spec_count": [int(v) for v in spec_n.cpu().numpy()]}
        # RandomInitSch (the loop's initial S_x, Alg. 2; the random part of S_draft, Alg. 1) into the same buffer
        P.random_init(csg, wl.seg_off, pop.shape[0], 1, tiles=pop)
        torch.cuda.synchronize()
        r0, r1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        r0.record()
        for rep in range(5):
            P.random_init(csg, wl.seg_off, pop.shape[0], 2 + rep, tiles=pop)
        r1.record()
        torch.cuda.synchronize()
        ri_ms = r0.elapsed_time(r1) / 5
        slot_bytes = sum(2 * w.n_slots(sg) * int(wl.seg_off[t + 1] - wl.seg_off[t]) for t, sg in enumerate(wl.subgraphs))
        out["random_init"] = {"ms": ri_ms, "candidates_per_s": n / (ri_ms * 1e-3), "written_GBps": slot_bytes / (ri_ms * 1e-3) / 1e9}
        del pop, ws_lse
    if args.lse_steps > 0:
        # Update_MoA (Sec. 4.3) on a model of this size (back-to-back calls from Python: the rate at which this binding
        # can launch, the kernel itself takes 2 us), and on a vector large enough to show the rate the kernel is bound by
        out["moa_update"] = {}
        for label, count, reps in (("model", 164 * 256 + 256 + 256 * 256 + 256 + 256, 50), ("large", 1 << 26, 5)):
            ps = torch.rand(count, device="cuda") - 0.5
            pt = ps + 1e-3
            pb = torch.empty(count, dtype=torch.uint16, device="cuda")
            P.moa_update(ps, pt, 0.99, bf16=pb)
            torch.cuda.synchronize()
            m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            m0.record()
            for _ in range(reps):
                P.moa_update(ps, pt, 0.99, bf16=pb)
            m1.record()
            torch.cuda.synchronize()
            us = m0.elapsed_time(m1) * 1e3 / reps
            out["moa_update"][label] = {"weights": count, "us_per_call": us, "GBps": count * 14 / (us * 1e-6) / 1e9}
            del ps, pt, pb
    if args.lse_steps > 0 and wl.verify:
        # the whole Pattern-aware Transformer (Sec. 4.2) on the drafted set: the statement rows of the step plus synthetic
        # dataflow rows (five to eight blocks per candidate)
        pm = w.make_pacm_weights(seed=1)
        gpm = {k: (dev(v) if isinstance(v, np.ndarray) else v) for k, v in pm.items()}
        blk_h = (5 + np.arange(n_d) % 4).astype(np.int32)
        flow = dev(w.make_flow_features(np.arange(n_d), blk_h))
        blk = dev(blk_h)
        yv = torch.empty(n_d, dtype=torch.float32, device="cuda")
        ws_pacm = torch.empty(P.workspace_bytes(P.WS_PACM, n_d, 0, 0), dtype=torch.uint8, device="cuda")
        P.pacm_score(feats[0], n_stmt, flow, blk, gpm, y=yv, workspace=ws_pacm)
        torch.cuda.synchronize()
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        for rep in range(10):
            P.pacm_score(feats[rep % len(feats)], n_stmt, flow, blk, gpm, y=yv, workspace=ws_pacm)
        p1.record()
        torch.cuda.synchronize()
        pacm_ms = p0.elapsed_time(p1) / 10
        # useful flops: valid statement rows through two layers, valid blocks through embedding, four 64x64 products and the
        # attention, every candidate through the head
        rows_s, rows_b = int(n_stmt_h.sum()), int(blk_h.sum())
        att = int((blk_h.astype(np.int64) ** 2).sum())
        pacm_flops = 2 * (rows_s * (164 * 256 + 256 * 256) + rows_b * (23 * 64 + 4 * 64 * 64) + att * 2 * 64 + n_d * (320 * 256 + 256))
        out["pacm"] = {"candidates": n_d, "ms": pacm_ms, "candidates_per_s": n_d / (pacm_ms * 1e-3),
                       "TFLOPs": pacm_flops / (pacm_ms * 1e-3) / 1e12, "useful_GFLOP": pacm_flops / 1e9}
        del flow, ws_pacm
        # the same call on 16 drafted sets at once: the rate of the three kernels when launches and weight loads no longer
        # count (random feature values of the same range; statement and block counts with the same mix)
        big_d = 16 * n_d
        rng = np.random.default_rng(11)
        bs_h = rng.choice(np.array(wl.n_stmt, np.int32), size=big_d).astype(np.int32)
        bb_h = (5 + np.arange(big_d) % 4).astype(np.int32)
        bfeat = torch.rand((big_d, 8, 164), device="cuda") * 24.0
        bflow = torch.rand((big_d, 8, 23), device="cuda") * 24.0
        bs, bb = dev(bs_h), dev(bb_h)
        by = torch.empty(big_d, dtype=torch.float32, device="cuda")
        bws = torch.empty(P.workspace_bytes(P.WS_PACM, big_d, 0, 0), dtype=torch.uint8, device="cuda")
        P.pacm_score(bfeat, bs, bflow, bb, gpm, y=by, workspace=bws)
        torch.cuda.synchronize()
        p0.record()
        for rep in range(5):
            P.pacm_score(bfeat, bs, bflow, bb, gpm, y=by, workspace=bws)
        p1.record()
        torch.cuda.synchronize()
        big_ms = p0.elapsed_time(p1) / 5
        rows_s, rows_b = int(bs_h.sum()), int(bb_h.sum())
        att = int((bb_h.astype(np.int64) ** 2).sum())
        big_flops = 2 * (rows_s * (164 * 256 + 256 * 256) + rows_b * (23 * 64 + 4 * 64 * 64) + att * 2 * 64 + big_d * (320 * 256 + 256))
        out["pacm_steady"] = {"candidates": big_d, "ms": big_ms, "candidates_per_s": big_d / (big_ms * 1e-3),
                              "TFLOPs": big_flops / (big_ms * 1e-3) / 1e12, "frac_of_bf16_peak": big_flops / (big_ms * 1e-3) / 2.5e15,
                              "useful_GFLOP": big_flops / 1e9}
        del bfeat, bflow, bws
    # what this chip sustains in the same run on the two resources the rooflines are quoted against: a 1 GiB device copy
    # (torch's copy kernel; bytes read plus bytes written) and a dense bfloat16 product from the vendor's GEMM library
    # (8192^3: matrix-core work only, no bandwidth pressure).  Context for `roofline.frac`, not its denominator.
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)
    dst = torch.empty_like(src)
    dst.copy_(src)
    a0, a1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a0.record()
    for _ in range(5):
        dst.copy_(src)
    a1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * src.numel() * 4 / (a0.elapsed_time(a1) * 1e-3) / 1e9
    del src, dst
    ga = torch.randn(8192, 8192, device="cuda").to(torch.bfloat16)
    gb = torch.randn(8192, 8192, device="cuda").to(torch.bfloat16)
    gc = torch.mm(ga, gb)
    a0.record()
    for _ in range(5):
        torch.mm(ga, gb, out=gc)
    a1.record()
    torch.cuda.synchronize()
    gemm_tf = 5 * 2 * 8192 ** 3 / (a0.elapsed_time(a1) * 1e-3) / 1e12
    del ga, gb, gc
    out["achievable"] = {"hbm_copy_GBps": copy_gbs, "hbm_copy_frac_of_peak": copy_gbs / HBM_PEAK_GBS,
                         "bf16_gemm_TFLOPs": gemm_tf, "bf16_gemm_frac_of_peak": gemm_tf / 2500.0,
                         "what": "1 GiB torch device copy (read + written bytes); torch.mm 8192^3 bfloat16 (vendor GEMM library)"}
    if not args.no_cpu_baseline:
        scale = args.cpu_scale if args.cpu_scale is not None else 1.0
        out["cpu_baseline"] = cpu_baseline(args.config, w, oracle, scale)
        cores = min(16, len(os.sched_getaffinity(0)))     # a one-GPU machine gives a job 16 cores, whatever the host has
        out["cpu_baseline_all_cores"] = cpu_baseline_all_cores(args.config, w, oracle, scale, cores)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
