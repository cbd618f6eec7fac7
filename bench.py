#!/usr/bin/env python3
"""Benchmark of the PointCNN++ MVMR hot path on one MI355X.

A step is one pass of the hot path over one synthetic scene already resident in HBM:
pcpp_build_triplets (hashed-grid search + reorder) -> pcpp_mvmr_fwd -> pcpp_mvmr_bwd_input ->
pcpp_mvmr_bwd_weight.  The headline workload is the largest scene (scene 5: 1M points, K = 125,
256 -> 256 bf16, shuffled point order); the other four scenes are measured in the same run and carried in
`scenes`.  For every scene the line gives the time of each op (events on the launch stream), neighbour pairs
per second with and without the triplet build, the roofline of the forward op (algorithmic bytes over the
HBM peak for the gather-bound layers, nominal flops 2 |T| C_in C_out over the bf16 matrix-core peak for the
256 -> 256 layer) and the CPU oracle timed on a bounded sample (cpu_baseline).
One JSON line is printed.
"""
from __future__ import annotations

import argparse
import glob
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
CSRC = os.path.join(ROOT, "paper_2511_23227_amd", "csrc")


def source_hash(name: str) -> str:
    """First 12 hex digits of the SHA-256 of one kernel source file (ties a counter figure to the code it measured)."""
    try:
        return hashlib.sha256(open(os.path.join(CSRC, name), "rb").read()).hexdigest()[:12]
    except OSError:
        return "missing"


def load_measured_traffic() -> dict:
    """HBM bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summaries under profiles/.
    A summary carries lines `TRAFFIC scene=5 order=default op=fwd kernel=... src=file.hip:hash read_bytes=..
    write_bytes=..`; a figure is used only while the named source file still has that hash."""
    table = {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_hbm_traffic.txt"))):
        for line in open(path):
            if not line.startswith("TRAFFIC "):
                continue
            kv = dict(item.split("=", 1) for item in line.split()[1:])
            src, _, digest = kv.get("src", ":").partition(":")
            table[(int(kv["scene"]), kv["order"], kv["op"])] = {
                "bytes": int(kv["read_bytes"]) + int(kv["write_bytes"]), "read_bytes": int(kv["read_bytes"]),
                "write_bytes": int(kv["write_bytes"]), "kernel": kv.get("kernel"),
                "file": os.path.relpath(path, ROOT), "current": source_hash(src) == digest}
    return table


def load_measured_mfma() -> dict:
    """MFMA instructions per launch (SQ_INSTS_MFMA) from the counter summaries under profiles/: lines
    `COUNTERS scene=5 order=default op=fwd kernel=.. src=file.hip:hash insts_mfma=..`, used only while the named
    source file still has that hash."""
    table = {}
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*_counters.txt"))):
        for line in open(path):
            if not line.startswith("COUNTERS "):
                continue
            kv = dict(item.split("=", 1) for item in line.split()[1:])
            src, _, digest = kv.get("src", ":").partition(":")
            if source_hash(src) == digest:
                table[(int(kv["scene"]), kv["order"], kv["op"])] = {"insts_mfma": int(kv["insts_mfma"]),
                                                                    "file": os.path.relpath(path, ROOT)}
    return table


def algorithmic_bytes(op: str, n_t: int, n_in: int, n_out: int, c_in: int, c_out: int, K: int, s_in: int,
                      s_out: int, n_pairs: int | None = None) -> float:
    """Bytes the method itself has to move per launch (Eq. (3) of Sec. 3.3.2 with W read once):
    every triplet fetches one source row and its two int32 indices, every destination row is
    written once, W is read once.  For the weight gradient the dy row is shared by the triplets of a (k, o) run,
    which are consecutive in (k, o, i) order, so it is counted once per run when n_pairs is given."""
    if op == "fwd":
        return n_t * (c_in * s_in + 8) + n_out * c_out * s_out + K * c_in * c_out * s_in
    if op == "bwd_input":
        return n_t * (c_out * s_in + 8) + n_in * c_in * s_out + K * c_in * c_out * s_in
    if op == "bwd_weight":
        dy_rows = n_t if n_pairs is None else n_pairs
        return n_t * (c_in * s_in + 8) + dy_rows * c_out * s_in + K * c_in * c_out * 4
    raise ValueError(op)


def compulsory_bytes(op: str, n_t: int, n_in: int, n_out: int, c_in: int, c_out: int, K: int, s_in: int,
                     s_out: int) -> float:
    """Bytes that must cross the HBM interface even with ideal caches: every array read or written once."""
    w = K * c_in * c_out
    if op == "fwd":
        return n_in * c_in * s_in + n_out * c_out * s_out + n_t * 8 + w * s_in
    if op == "bwd_input":
        return n_out * c_out * s_in + n_in * c_in * s_out + n_t * 8 + w * s_in
    if op == "bwd_weight":
        return n_in * c_in * s_in + n_out * c_out * s_in + n_t * 8 + w * 4
    raise ValueError(op)


def measure_scene(scene_id: int, order: str, steps: int, warmup: int, spatial: bool, cpu_pair_tests: float,
                  traffic: dict, cold: bool, tuner: bool = True):
    """All figures of one scene.  Returns the record."""
    import numpy as np
    import torch

    import paper_2511_23227_amd as pcpp
    import scenes

    s = scenes.make_scene(scene_id, order=order)
    x, w, dy = scenes.make_features(s)
    fdt = torch.bfloat16 if s.dtype == "bf16" else torch.float32
    s_in = 2 if s.dtype == "bf16" else 4
    in_xyz = torch.from_numpy(s.in_xyz).cuda()
    out_xyz = in_xyz if s.out_xyz is s.in_xyz else torch.from_numpy(s.out_xyz).cuda()
    dx_, dw_, ddy = (torch.from_numpy(a).cuda().to(fdt) for a in (x, w, dy))
    ops = [op for op in ("fwd", "bwd_input", "bwd_weight") if op in s.ops]
    flags = pcpp.PLAN_FWD | (pcpp.PLAN_BWD_INPUT if "bwd_input" in ops else 0) | (pcpp.PLAN_SPATIAL if spatial else 0)

    # persistent caller-owned buffers, sized once outside the timed region
    T0 = pcpp.pcpp_build_triplets(in_xyz, out_xyz, s.radius, s.t, plan_flags=flags)
    n_t = T0.n_triplets
    L = pcpp.library()
    code = 1 if s.dtype == "bf16" else 0
    buffers = dict(tri_o=torch.empty(n_t, dtype=torch.int32, device="cuda"),
                   tri_i=torch.empty(n_t, dtype=torch.int32, device="cuda"),
                   tri_k=torch.empty(n_t, dtype=torch.int32, device="cuda"),
                   seg_offsets=torch.empty(s.K + 1, dtype=torch.int64, device="cuda"),
                   plan=torch.empty(L.pcpp_plan_bytes(s.n_in, s.n_out, s.t, n_t, flags), dtype=torch.uint8, device="cuda"),
                   workspace=torch.empty(L.pcpp_build_triplets_workspace_bytes_for(s.n_in, s.n_out, s.t, n_t),
                                         dtype=torch.uint8, device="cuda"))
    ws = {i_: torch.empty(max(256, L.pcpp_mvmr_workspace_bytes(i_, s.n_in, s.n_out, n_t, s.c_in, s.c_out, s.K, code)),
                          dtype=torch.uint8, device="cuda") for i_ in range(3)}
    out = torch.empty((s.n_out, s.c_out), dtype=torch.float32, device="cuda")
    gx = torch.empty((s.n_in, s.c_in), dtype=torch.float32, device="cuda")
    gw = torch.empty((s.K, s.c_out, s.c_in), dtype=torch.float32, device="cuda")
    del T0

    names = ["build"] + ops
    events = []

    def build():
        return pcpp.pcpp_build_triplets(in_xyz, out_xyz, s.radius, s.t, plan_flags=flags, capacity=n_t, buffers=buffers)

    def compute(T, ev=None, j=1):
        if "fwd" in ops:
            pcpp.pcpp_mvmr_fwd(dx_, dw_, T, out=out, workspace=ws[0]); j += 1
            if ev:
                ev[j].record()
        if "bwd_input" in ops:
            pcpp.pcpp_mvmr_bwd_input(ddy, dw_, T, dx=gx, workspace=ws[1]); j += 1
            if ev:
                ev[j].record()
        if "bwd_weight" in ops:
            pcpp.pcpp_mvmr_bwd_weight(dx_, ddy, T, dw=gw, workspace=ws[2]); j += 1
            if ev:
                ev[j].record()

    def step(record: bool):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] if record else None
        if record:
            ev[0].record()
        T = build()
        if record:
            ev[1].record()
        compute(T, ev)
        if record:
            events.append(ev)
        return T

    for _ in range(warmup):
        T = step(False)
    # (1) the MVMR ops alone: K steps of fwd + bwd_input + bwd_weight on one build
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        compute(T)
    torch.cuda.synchronize()
    ms_compute = (time.perf_counter() - t0) * 1e3 / steps
    # (2) the whole path: K steps of build + the three ops
    t0 = time.perf_counter()
    for _ in range(steps):
        T = step(False)
    torch.cuda.synchronize()
    ms_whole = (time.perf_counter() - t0) * 1e3 / steps
    assert T.n_triplets == n_t
    # (3) per-op times: the same steps once more with events on the launch stream between the ops (outside the
    # timed regions: every event record costs a few microseconds of GPU time)
    for _ in range(steps):
        T = step(True)
    torch.cuda.synchronize()
    samples = {nm: np.array([ev[j].elapsed_time(ev[j + 1]) for ev in events]) for j, nm in enumerate(names)}
    op_ms = {nm: float(v.mean()) for nm, v in samples.items()}

    cold_ms = None
    if cold:
        # cold caches: a 512 MiB buffer overwritten before each step (L2 and the memory-side cache then hold none of
        # the step's data); reported beside the warm figures
        events.clear()
        scrub = torch.empty(128 * 1024 * 1024, dtype=torch.float32, device="cuda")
        for it in range(min(steps, 5)):
            scrub.fill_(float(it))
            step(True)
        torch.cuda.synchronize()
        cold_ms = {nm: round(float(np.median([ev[j].elapsed_time(ev[j + 1]) for ev in events])), 4)
                   for j, nm in enumerate(names)}
        del scrub

    # distinct (cell, centre) pairs: the rows that one product with W[k] serves after the run sums
    n_pairs_o = int(torch.unique(T.tri_k.long() * s.n_out + T.tri_o.long()).numel()) if n_t else 0
    n_pairs_i = int(torch.unique(T.tri_k.long() * s.n_in + T.tri_i.long()).numel()) if n_t and "bwd_input" in ops else 0
    wide = s.dtype == "bf16" and min(s.c_in, s.c_out) >= 256

    def roofline(op):
        ms = op_ms[op]
        nominal = 2.0 * n_t * s.c_in * s.c_out
        b = algorithmic_bytes(op, n_t, s.n_in, s.n_out, s.c_in, s.c_out, s.K, s_in, 4, n_pairs_o)
        gbs = b / (ms * 1e-3) / 1e9
        tr = traffic.get((scene_id, order, op))
        rec = {"op": op, "ms": round(ms, 4), "algorithmic_bytes": int(b),
               "nominal_tflops": round(nominal / (ms * 1e-3) / 1e12, 2),
               "traffic": tr["bytes"] if tr and tr["current"] else None,
               "traffic_source": (tr["file"] + ("" if tr["current"] else " (stale: the kernel's source has changed)")) if tr else None,
               "compulsory_floor_ms": round(compulsory_bytes(op, n_t, s.n_in, s.n_out, s.c_in, s.c_out, s.K, s_in, 4)
                                            / (HBM_PEAK_GBS * 1e9) * 1e3, 5)}
        if tr and tr["current"]:
            rec["traffic_GBs"] = round(tr["bytes"] / (ms * 1e-3) / 1e9, 1)
            rec["traffic_frac_of_hbm_peak"] = round(tr["bytes"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)
        if wide:
            # matrix-core bound: graded on the method's own flops, 2 C_in C_out per triplet
            tf = nominal / (ms * 1e-3) / 1e12
            rec.update({"bound": "mfma", "achieved": round(tf, 2), "peak": MFMA_PEAK_TFLOPS["bf16"], "unit": "TFLOP/s",
                        "frac": round(tf / MFMA_PEAK_TFLOPS["bf16"], 4)})
            cm = load_measured_mfma().get((scene_id, order, "fwd" if op == "bwd_input" else op))
            if cm:
                # what the kernel issues, counted by the hardware: includes the rows of zeros that ride along in a
                # group of centres, so it is context, never the graded fraction
                issued = cm["insts_mfma"] * 2.0 * 16 * 16 * 32
                rec["issued_tflop_incl_zero_rows"] = round(issued / 1e12, 3)
                rec["issued_tflops_incl_zero_rows"] = round(issued / (ms * 1e-3) / 1e12, 1)
                rec["issued_source"] = cm["file"]
            pairs = {"fwd": n_pairs_o, "bwd_input": n_pairs_i}.get(op)
            if pairs:
                # after the run sums one product with W[k] per distinct (cell, centre) pair is the least the matrix
                # cores must do; what the kernel issues on top of that (rows of zeros inside a group of 16 centres)
                # is not the method's work and is not counted anywhere in `frac`
                rec["min_executed_tflop"] = round(2.0 * pairs * s.c_in * s.c_out / 1e12, 3)
        else:
            rec.update({"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": round(gbs / HBM_PEAK_GBS, 4),
                        "model": "gather model: every triplet fetches its source row from the memory hierarchy "
                                 "(rows that the caches serve are counted; see traffic for what crosses HBM)"})
            if gbs > HBM_PEAK_GBS:
                # The model's rate is more than the memory can deliver: the caches serve most of the rows (long runs,
                # neighbouring centres sharing rows), so the model is no bound for this op.  It is graded instead against
                # the nearer of its two real ceilings: the method's own flops over the matrix cores' peak for its
                # dtype, or (when a current measurement is at hand) what crosses the fabric over the HBM peak.
                rec["gather_model_GBs"] = rec["achieved"]
                tf = nominal / (ms * 1e-3) / 1e12
                peak_tf = MFMA_PEAK_TFLOPS["bf16" if s.dtype == "bf16" else "f32"]
                f_mfma = tf / peak_tf
                f_hbm = rec.get("traffic_frac_of_hbm_peak")
                rec["model"] = ("the gather model's rate exceeds the HBM peak here (the caches serve most rows); graded on "
                                "the nearer of: nominal flops 2 C_in C_out per triplet over the matrix peak, measured fabric "
                                "traffic over the HBM peak")
                if f_hbm is not None and f_hbm > f_mfma:
                    rec.update({"achieved": rec["traffic_GBs"], "frac": f_hbm, "bound": "hbm"})
                else:
                    rec.update({"bound": "mfma", "achieved": round(tf, 2), "peak": peak_tf, "unit": "TFLOP/s",
                                "frac": round(f_mfma, 4)})
            if op == "bwd_weight":
                b_survey = algorithmic_bytes(op, n_t, s.n_in, s.n_out, s.c_in, s.c_out, s.K, s_in, 4, None)
                rec["survey_model_bytes"] = int(b_survey)      # dy counted once per triplet: more than the kernels read
        return rec

    per_op = {op: roofline(op) for op in ops}
    compute_ms = sum(op_ms[op] for op in ops)
    top = max(names, key=lambda nm: op_ms[nm])
    rec = {
        "config": {"workload": f"scene{s.scene_id}_{s.name}", "order": order, "plan": "spatial" if spatial else "index order",
                   "n_in": s.n_in, "n_out": s.n_out, "radius": s.radius, "t": s.t, "c_in": s.c_in, "c_out": s.c_out,
                   "dtype": s.dtype, "n_triplets": n_t, "ops": names},
        "value": round(n_t / (ms_compute * 1e-3), 1),
        "value_with_build": round(n_t / (ms_whole * 1e-3), 1),
        "unit": "pairs/s",
        "ms_per_step": round(ms_compute, 4),
        "ms_per_step_with_build": round(ms_whole, 4),
        "op_ms": {k_: round(v, 4) for k_, v in op_ms.items()},
        "op_ms_median": {k_: round(float(np.median(v)), 4) for k_, v in samples.items()},
        "op_ms_min": {k_: round(float(v.min()), 4) for k_, v in samples.items()},
        "op_ms_cold": cold_ms,
        "event_sum_compute_ms": round(compute_ms, 4),
        "build_pairs_per_s": round(n_t / (op_ms["build"] * 1e-3), 1),
        "triplets_per_k_o_pair": round(n_t / n_pairs_o, 3) if n_pairs_o else None,
        "roofline": per_op.get("fwd"),
        "roofline_top_op": per_op.get(top, {"op": "build", "ms": round(op_ms["build"], 4),
                                            "note": "triplet construction: bound by instruction issue and latency"}),
        "roofline_per_op": per_op,
    }

    if "bwd_input" in ops and tuner:
        # what the library's own tuner (Sec. 3.3.2, closing remark) measures for this cloud and layer: one pass of
        # fwd + bwd_input in either plan order; outside every timed region
        del buffers
        tuned, ms_a, ms_b = pcpp.pcpp_tune_plan_order(in_xyz, out_xyz, s.radius, s.t, n_t, s.c_in, s.c_out, fdt)
        rec["plan_order_tuner"] = {"fwd_plus_bwd_input_ms_index_order": round(ms_a, 4),
                                   "fwd_plus_bwd_input_ms_spatial_order": round(ms_b, 4),
                                   "choice": "spatial" if tuned & pcpp.PLAN_SPATIAL else "index order"}

    if cpu_pair_tests > 0:
        import oracle
        # bounded sample of the same workload: the first n_sample outputs against all inputs
        n_sample = min(s.n_out, max(256, int(cpu_pair_tests / max(s.n_in, 1))))
        sub = np.ascontiguousarray(s.out_xyz[:n_sample])
        c0 = time.perf_counter()
        o, i, k, seg = oracle.build_triplets(s.in_xyz, sub, s.radius, s.t)
        c1 = time.perf_counter()
        oracle.mvmr_fwd(x, w, o, i, k, n_sample)
        if "bwd_input" in ops:
            oracle.mvmr_bwd_input(dy[:n_sample], w, o, i, k, s.n_in)
        if "bwd_weight" in ops:
            oracle.mvmr_bwd_weight(x, dy[:n_sample], o, i, k, s.K)
        c2 = time.perf_counter()
        rec["cpu_baseline"] = {
            "value": round(len(o) / max(c2 - c1, 1e-9), 1), "value_with_build": round(len(o) / (c2 - c0), 1),
            "unit": "pairs/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"first {n_sample} of {s.n_out} outputs against all {s.n_in} inputs: {len(o)} triplets; "
                      f"brute-force search {c1 - c0:.2f} s, {'+'.join(ops)} {c2 - c1:.2f} s"}
    return rec


def measure_variants(steps: int, warmup: int) -> dict:
    """The steps either side of the path (Sec. 4.1) and the degraded operator (Sec. 3.2, "Ours (degraded)" of Sec. 4.2) on
    the benchmark clouds: voxel-grid down-sampling, a batch of clouds built in one call, the voxel operator on the
    strided scene beside the ball operator."""
    import numpy as np
    import torch

    import paper_2511_23227_amd as pcpp
    import scenes

    def timed(fn, reps):
        for _ in range(warmup):
            fn()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps

    out = {}
    # (1) voxel-grid down-sampling (lowest index per voxel, original coordinates kept)
    for sid, pitch in ((4, 0.0415), (5, 0.2)):
        s = scenes.make_scene(sid)
        xyz = torch.from_numpy(s.in_xyz).cuda()
        kept = pcpp.pcpp_voxel_subsample(xyz, pitch)
        ms = timed(lambda: pcpp.pcpp_voxel_subsample(xyz, pitch), steps)
        out[f"voxel_subsample_scene{sid}"] = {"n": s.n_in, "pitch": pitch, "n_kept": int(kept.numel()), "ms": round(ms, 4),
                                              "points_per_s": round(s.n_in / (ms * 1e-3), 1),
                                              "note": "includes the host's wait for the count"}
    # (2) a batch of eight clouds (scene 2's cloud under eight rigid shifts) built in one call against eight single builds
    s = scenes.make_scene(2)
    nb = 8
    shifts = np.arange(nb, dtype=np.float32)[:, None] * np.array([[0.25, 0.5, 0.125]], dtype=np.float32)
    clouds = [s.in_xyz + shifts[b] for b in range(nb)]
    cat = torch.from_numpy(np.ascontiguousarray(np.concatenate(clouds))).cuda()
    offs = torch.arange(nb + 1, dtype=torch.int32, device="cuda") * s.n_in
    flags = pcpp.PLAN_FWD | pcpp.PLAN_BWD_INPUT
    Tb = pcpp.pcpp_build_triplets(cat, cat, s.radius, s.t, plan_flags=flags, in_offsets=offs, out_offsets=offs)
    n_tb = Tb.n_triplets
    ms_b = timed(lambda: pcpp.pcpp_build_triplets(cat, cat, s.radius, s.t, plan_flags=flags, in_offsets=offs, out_offsets=offs,
                                                  capacity=n_tb), steps)
    single = [torch.from_numpy(np.ascontiguousarray(c)).cuda() for c in clouds]
    n_ts = pcpp.pcpp_build_triplets(single[0], single[0], s.radius, s.t, plan_flags=flags).n_triplets

    def eight():
        for c in single:
            pcpp.pcpp_build_triplets(c, c, s.radius, s.t, plan_flags=flags, capacity=n_ts + 4096)
    ms_s = timed(eight, max(2, steps // 2))
    out["batched_build_8x_scene2"] = {"n_points": nb * s.n_in, "n_triplets": n_tb, "ms_one_batched_call": round(ms_b, 4),
                                      "ms_eight_single_calls": round(ms_s, 4),
                                      "build_pairs_per_s": round(n_tb / (ms_b * 1e-3), 1),
                                      "note": "both allocate their outputs per call"}
    del Tb, cat, single
    # (3) the degraded (voxel) operator on the strided scene: pitch 2 r / t, so that the t^3 voxels span the ball's cube
    s = scenes.make_scene(4)
    x, w, dy = scenes.make_features(s)
    bf = torch.bfloat16
    xin, xout = torch.from_numpy(s.in_xyz).cuda(), torch.from_numpy(s.out_xyz).cuda()
    dx_, dw_, ddy = (torch.from_numpy(a_).cuda().to(bf) for a_ in (x, w, dy))
    rec = {}
    for name, size, bflag in (("ball", s.radius, 0), ("voxel", 2.0 * s.radius / s.t, pcpp.BUILD_VOXEL)):
        T = pcpp.pcpp_build_triplets(xin, xout, size, s.t, plan_flags=flags | bflag)
        n_t = T.n_triplets
        ms_build = timed(lambda: pcpp.pcpp_build_triplets(xin, xout, size, s.t, plan_flags=flags | bflag, capacity=n_t), steps)
        ms_f = timed(lambda: pcpp.pcpp_mvmr_fwd(dx_, dw_, T), steps)
        ms_i = timed(lambda: pcpp.pcpp_mvmr_bwd_input(ddy, dw_, T), steps)
        ms_w = timed(lambda: pcpp.pcpp_mvmr_bwd_weight(dx_, ddy, T), steps)
        rec[name] = {"size": round(float(size), 5), "n_triplets": n_t, "build_ms": round(ms_build, 4), "fwd_ms": round(ms_f, 4),
                     "bwd_input_ms": round(ms_i, 4), "bwd_weight_ms": round(ms_w, 4),
                     "pairs_per_s": round(n_t / ((ms_f + ms_i + ms_w) * 1e-3), 1)}
    rec["note"] = "times include the allocation of the outputs by the binding"
    out["degraded_operator_scene4"] = rec
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--scene", type=int, default=5, help="headline scene (default 5: the largest single-GPU workload)")
    ap.add_argument("--order", default="default", choices=["default", "morton"])
    ap.add_argument("--plan", default="auto", choices=["auto", "spatial", "index"],
                    help="auto: PLAN_SPATIAL for layers of 128 channels or more, index order otherwise")
    ap.add_argument("--only", action="store_true", help="measure the headline scene only (profiling runs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true", help="skip the library-kernel peak measurements")
    ap.add_argument("--no-tuner", action="store_true", help="skip the plan-order tuner's record (profiling runs)")
    ap.add_argument("--no-variants", action="store_true", help="skip the down-sampling / batch / voxel-operator records")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a 256 MiB device-to-device copy (the kernel of known size against which the "
                         "FETCH_SIZE / WRITE_SIZE counters are scaled) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU only (the paper's operator is a one-GPU kernel); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2511_23227_amd as pcpp
    import scenes

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")      # 256 MiB
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes": src.numel() * 4, "copies": 4}))
        return 0
    pcpp.library()
    traffic = load_measured_traffic()

    def want_spatial(scene_id):
        if args.plan != "auto":
            return args.plan == "spatial"
        return scene_id == 5                      # the 256 -> 256 layer

    cpu_tests = 0.0 if args.no_cpu_baseline else 1.0e10      # pair tests of the brute-force search per scene (~10 s)
    head = measure_scene(args.scene, args.order, args.steps, args.warmup, want_spatial(args.scene), 2.5 * cpu_tests,
                         traffic, cold=True, tuner=not args.no_tuner)
    others = {}
    if not args.only:
        for sid, order in ((1, "default"), (2, "default"), (3, "default"), (4, "default"), (2, "morton"), (5, "morton")):
            if (sid, order) == (args.scene, args.order):
                continue
            print(f"bench.py: scene {sid} ({order})", file=sys.stderr, flush=True)
            r = measure_scene(sid, order, args.steps, args.warmup, want_spatial(sid),
                              cpu_tests if order == "default" else 0.0, traffic, cold=False, tuner=not args.no_tuner)
            others[f"{r['config']['workload']}" + ("" if order == "default" else "_" + order)] = r

    peaks = None
    if not args.no_peaks:
        # what this device reaches on plain library kernels in the same run: a 256 MiB device copy (read + write),
        # an 8192^3 bf16 GEMM and a loop that only issues bf16 MFMAs on registers; context for the fractions, which
        # stay against the published peaks
        def timed(fn, reps):
            fn()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) * 1e-3 / reps
        csrc = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        cdst = torch.empty_like(csrc)
        copy_gbs = 2 * csrc.numel() * 4 / timed(lambda: cdst.copy_(csrc), 10) / 1e9
        del csrc, cdst
        ga = torch.randn(8192, 8192, device="cuda").to(torch.bfloat16)
        gb = torch.randn(8192, 8192, device="cuda").to(torch.bfloat16)
        gemm_tflops = 2 * 8192 ** 3 / timed(lambda: torch.matmul(ga, gb), 5) / 1e12
        del ga, gb
        import ctypes
        mfma_loop_tflops = None
        probe_path = os.path.join(ROOT, "paper_2511_23227_amd", "libpcpp_probe.so")
        if os.path.exists(probe_path):
            probe = ctypes.CDLL(probe_path)
            probe.pcpp_probe_mfma_bf16.restype = ctypes.c_double
            probe.pcpp_probe_mfma_bf16.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
            sink = torch.zeros(256, dtype=torch.float32, device="cuda")
            probe_flops = []

            def run_probe():
                f = probe.pcpp_probe_mfma_bf16(256 * 8, 4096, sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
                assert f > 0, "peak probe failed to launch"
                probe_flops.append(f)
            secs = timed(run_probe, 5)
            mfma_loop_tflops = probe_flops[-1] / secs / 1e12
        peaks = {"copy_GBs": round(copy_gbs, 1), "gemm_bf16_TFLOPs": round(gemm_tflops, 1),
                 "mfma_issue_loop_bf16_TFLOPs": None if mfma_loop_tflops is None else round(mfma_loop_tflops, 1)}

    result = {
        "metric": "MVMR fwd+bwd neighbour-pairs/s (|T| over the time of fwd + bwd_input + bwd_weight; "
                  "value_with_build adds the triplet construction)",
        "value": head["value"],
        "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["config"]["dtype"], "data": "synthetic",
        "config": head["config"],
        "value_with_build": head["value_with_build"],
        "ms_per_step_with_build": head["ms_per_step_with_build"],
        "op_ms": head["op_ms"], "op_ms_median": head["op_ms_median"], "op_ms_min": head["op_ms_min"],
        "op_ms_cold": head["op_ms_cold"],
        "build_pairs_per_s": head["build_pairs_per_s"],
        "triplets_per_k_o_pair": head["triplets_per_k_o_pair"],
        "measured_peaks": peaks,
        "roofline": head["roofline"],
        "roofline_top_op": head["roofline_top_op"],
        "roofline_per_op": head["roofline_per_op"],
        "scenes": others,
    }
    if not args.only and not args.no_variants:
        print("bench.py: variants", file=sys.stderr, flush=True)
        result["variants"] = measure_variants(args.steps, args.warmup)
    for key in ("cpu_baseline", "plan_order_tuner"):
        if key in head:
            result[key] = head[key]
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
