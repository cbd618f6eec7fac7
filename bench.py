#!/usr/bin/env python3
"""Benchmark of the PointCNN++ MVMR hot path on one MI355X.

A step is one pass of the whole hot path over one synthetic scene already resident in HBM:
pcpp_build_triplets (hashed-grid search + reorder) -> pcpp_mvmr_fwd -> pcpp_mvmr_bwd_input ->
pcpp_mvmr_bwd_weight.  The headline value is neighbour pairs per second = |T| / step time.
One JSON line is printed; it also carries the per-op times, the roofline of the dominant MVMR
kernel (algorithmic bytes over the kernel time measured with events on the launch stream) and the
CPU oracle timed on the host cores (cpu_baseline).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0           # MI355X HBM3E, published
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}

# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (see profiles/), keyed by
# (scene, order, op); absent entries are reported as null.
MEASURED_TRAFFIC: dict = {
    (2, "default", "fwd"): int(289.4e6 + 16.0e6),         # rows_kernel: scaled FETCH_SIZE + WRITE_SIZE
    (2, "default", "bwd_input"): int(289.4e6 + 16.0e6),
    (2, "default", "bwd_weight"): int(388.4e6 + 8.4e6),   # weight_f32_kernel (weight_reduce adds 8.5e6 read)
    (5, "default", "fwd"): int(27668e6 + 1024e6),         # rows_wide_kernel
    (5, "default", "bwd_input"): int(27668e6 + 1024e6),
    (5, "default", "bwd_weight"): int(25407e6 + 567e6),   # weight_lds_kernel (weight_reduce adds 567e6 read)
}


def algorithmic_bytes(op: str, n_t: int, n_in: int, n_out: int, c_in: int, c_out: int, K: int, s_in: int,
                      s_out: int) -> float:
    """Bytes the method itself has to move per launch (Eq. (3) of Sec. 3.3.2 with W read once):
    every triplet fetches one source row and its two int32 indices, every destination row is
    written once, W is read once."""
    if op == "fwd":
        return n_t * (c_in * s_in + 8) + n_out * c_out * s_out + K * c_in * c_out * s_in
    if op == "bwd_input":
        return n_t * (c_out * s_in + 8) + n_in * c_in * s_out + K * c_in * c_out * s_in
    if op == "bwd_weight":
        return n_t * ((c_in + c_out) * s_in + 8) + K * c_in * c_out * 4
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


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--scene", type=int, default=2, help="synthetic scene id (default 2: the headline workload)")
    ap.add_argument("--order", default="default", choices=["default", "morton"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run only a 256 MiB device-to-device copy (the kernel of known size against which the "
                         "FETCH_SIZE / WRITE_SIZE counters are scaled) and exit")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build is single-GPU only (the paper's operator is a one-GPU kernel); "
              "run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
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

    s = scenes.make_scene(args.scene, order=args.order)
    x, w, dy = scenes.make_features(s)
    fdt = torch.bfloat16 if s.dtype == "bf16" else torch.float32
    s_in = 2 if s.dtype == "bf16" else 4
    in_xyz = torch.from_numpy(s.in_xyz).cuda()
    out_xyz = in_xyz if s.out_xyz is s.in_xyz else torch.from_numpy(s.out_xyz).cuda()
    dx_, dw_, ddy = (torch.from_numpy(a).cuda().to(fdt) for a in (x, w, dy))
    ops = [op for op in ("fwd", "bwd_input", "bwd_weight") if op in s.ops]
    flags = pcpp.PLAN_FWD | (pcpp.PLAN_BWD_INPUT if "bwd_input" in ops else 0)

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

    def step(record: bool):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(names) + 1)] if record else None
        if record:
            ev[0].record()
        T = pcpp.pcpp_build_triplets(in_xyz, out_xyz, s.radius, s.t, plan_flags=flags, capacity=n_t, buffers=buffers)
        j = 1
        if record:
            ev[j].record()
        if "fwd" in ops:
            pcpp.pcpp_mvmr_fwd(dx_, dw_, T, out=out, workspace=ws[0]); j += 1
            if record:
                ev[j].record()
        if "bwd_input" in ops:
            pcpp.pcpp_mvmr_bwd_input(ddy, dw_, T, dx=gx, workspace=ws[1]); j += 1
            if record:
                ev[j].record()
        if "bwd_weight" in ops:
            pcpp.pcpp_mvmr_bwd_weight(dx_, ddy, T, dw=gw, workspace=ws[2]); j += 1
            if record:
                ev[j].record()
        if record:
            events.append(ev)
        return T

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        T = step(False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    assert T.n_triplets == n_t
    # per-op times: the same steps once more with events on the launch stream between the ops (outside the timed
    # region: every event record costs a few microseconds of GPU time)
    for _ in range(args.steps):
        T = step(True)
    torch.cuda.synchronize()

    samples = {nm: np.array([ev[j].elapsed_time(ev[j + 1]) for ev in events]) for j, nm in enumerate(names)}
    op_ms = {nm: float(v.mean()) for nm, v in samples.items()}

    # cold caches: the same steps with a 512 MiB buffer overwritten before each one (L2 and the memory-side cache
    # then hold none of the step's data); reported beside the warm figures, never part of `value`
    events.clear()
    scrub = torch.empty(128 * 1024 * 1024, dtype=torch.float32, device="cuda")
    for it in range(min(args.steps, 10)):
        scrub.fill_(float(it))
        step(True)
    torch.cuda.synchronize()
    cold_ms = {nm: float(np.median([ev[j].elapsed_time(ev[j + 1]) for ev in events])) for j, nm in enumerate(names)}
    del scrub

    # what this device reaches on plain library kernels in the same run: a 256 MiB device copy (read + write) and
    # an 8192^3 bf16 GEMM; the graded fractions stay against the published peaks
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
    # and on a loop that only issues bf16 MFMAs on registers (eight waves per SIMD, sixteen independent chains each)
    # (a measurement aid in a shared object of its own; reported as null if it has not been built)
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

    def roofline(op):
        b = algorithmic_bytes(op, n_t, s.n_in, s.n_out, s.c_in, s.c_out, s.K, s_in, 4)
        gbs = b / (op_ms[op] * 1e-3) / 1e9
        return {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": MEASURED_TRAFFIC.get((args.scene, args.order, op)),
                "kernel": op, "algorithmic_bytes": int(b), "ms": round(op_ms[op], 4),
                "nominal_tflops": round(2.0 * n_t * s.c_in * s.c_out / (op_ms[op] * 1e-3) / 1e12, 2),
                "frac_of_measured_copy": round(gbs / copy_gbs, 4),
                "compulsory_bytes": int(compulsory_bytes(op, n_t, s.n_in, s.n_out, s.c_in, s.c_out, s.K, s_in, 4)),
                "compulsory_floor_ms": round(compulsory_bytes(op, n_t, s.n_in, s.n_out, s.c_in, s.c_out, s.K, s_in, 4)
                                             / (HBM_PEAK_GBS * 1e9) * 1e3, 5)}

    per_op = {op: roofline(op) for op in ops}
    dominant = max(ops, key=lambda o_: op_ms[o_])

    # Matrix-core work actually issued by the rows kernels (fwd / bwd_input): one 32 x C_src x C_dst product per
    # (cell, 32-centre block) that holds a triplet, plus the run sums (one selection product per 16 triplets --
    # 32 in the wide kernel -- and 32 source channels; three for fp32 inputs, whose 32 -> 32 product itself runs as
    # six bf16 products).  Blocks without a triplet are skipped.
    def executed_flops(centre, c_src, c_dst):
        key = T.tri_k.long() * ((int(centre.max()) >> 5) + 1) + (centre.long() >> 5)
        _, cnt = torch.unique(key, return_counts=True)
        wide = s.dtype == "bf16" and c_src == 256 and c_dst == 256
        per = 32 if wide else 16                      # triplets per selection product
        steps = ((cnt + per - 1) // per).sum().item()
        terms = 1 if s.dtype == "bf16" else 3
        stage2 = 2.0 * 32 * c_src * c_dst
        if s.dtype == "f32" and c_src == 32 and c_dst == 32:
            stage2 *= 6                               # six bf16 products of the three-term splits
        return cnt.numel() * stage2 + steps * terms * 2.0 * per * 32 * c_src
    pair_ratio = None
    if n_t > 0:
        # triplets per distinct (cell, output point): how many rows one product with W[k] serves after the run sums
        pair_ratio = round(n_t / torch.unique(T.tri_k.long() * s.n_out + T.tri_o.long()).numel(), 3)
        ex = {"fwd": executed_flops(T.tri_o, s.c_in, s.c_out)}
        if "bwd_input" in ops:
            ex["bwd_input"] = executed_flops(T.tri_i, s.c_out, s.c_in)
        if "bwd_weight" in ops:
            ex["bwd_weight"] = 2.0 * n_t * s.c_in * s.c_out      # one outer product per triplet, nothing skipped
        split = s.dtype == "f32" and s.c_in == 32 and s.c_out == 32   # rows kernels issue bf16 products for this layer
        for op in ops:
            peak = MFMA_PEAK_TFLOPS["bf16" if (split and op != "bwd_weight") else s.dtype]
            tf = ex[op] / (op_ms[op] * 1e-3) / 1e12
            per_op[op]["executed_mfma_tflops"] = round(tf, 2)
            per_op[op]["mfma_frac"] = round(tf / peak, 4)
            if peak == MFMA_PEAK_TFLOPS["bf16"]:
                per_op[op]["mfma_frac_of_measured_gemm"] = round(tf / gemm_tflops, 4)
                if mfma_loop_tflops:
                    per_op[op]["mfma_frac_of_issue_loop"] = round(tf / mfma_loop_tflops, 4)
            if s.dtype == "bf16" and min(s.c_in, s.c_out) >= 256:   # wide layers are matrix-core bound
                per_op[op].update({"bound": "mfma", "achieved": round(tf, 2), "peak": peak, "unit": "TFLOP/s",
                                   "frac": round(tf / peak, 4)})

    result = {
        "metric": "MVMR fwd+bwd neighbour-pairs/s (whole hot path: triplet build + fwd + bwd_input + bwd_weight)",
        "value": round(n_t / (ms_per_step * 1e-3), 1),
        "unit": "pairs/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": s.dtype, "data": "synthetic",
        "config": {"workload": f"scene{s.scene_id}_{s.name}", "order": args.order, "n_in": s.n_in, "n_out": s.n_out,
                   "radius": s.radius, "t": s.t, "c_in": s.c_in, "c_out": s.c_out, "n_triplets": n_t,
                   "ops": names},
        "op_ms": {k_: round(v, 4) for k_, v in op_ms.items()},
        "op_ms_median": {k_: round(float(np.median(v)), 4) for k_, v in samples.items()},
        "op_ms_min": {k_: round(float(v.min()), 4) for k_, v in samples.items()},
        "op_ms_cold": {k_: round(v, 4) for k_, v in cold_ms.items()},
        "measured_peaks": {"copy_GBs": round(copy_gbs, 1), "gemm_bf16_TFLOPs": round(gemm_tflops, 1),
                           "mfma_issue_loop_bf16_TFLOPs": None if mfma_loop_tflops is None else round(mfma_loop_tflops, 1)},
        "triplets_per_k_o_pair": pair_ratio,
        "pairs_per_s": {k_: round(n_t / (v * 1e-3), 1) for k_, v in op_ms.items()},
        "roofline": per_op[dominant],
        "roofline_per_op": per_op,
    }

    if not args.no_cpu_baseline:
        import oracle
        # bounded sample of the same workload: the first n_sample outputs against all inputs
        n_sample = min(s.n_out, max(1024, int(2.0e10 / max(s.n_in, 1))))   # about 10-30 s of host work
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
        result["cpu_baseline"] = {
            "value": round(len(o) / (c2 - c0), 1), "unit": "pairs/s", "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"first {n_sample} of {s.n_out} outputs against all {s.n_in} inputs: {len(o)} triplets; "
                      f"brute-force search {c1 - c0:.2f} s, {'+'.join(ops)} {c2 - c1:.2f} s"}
    print(json.dumps(result))
    return 0


if __name__ == "__main__":
    sys.exit(main())
