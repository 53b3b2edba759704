#!/usr/bin/env python3
"""Benchmark of the tile-centric mixed-precision GEMM hot path on one MI355X.

One step = one pass of the whole path over one synthetic problem whose dense FP64 inputs are
already resident in HBM: tile scan + norm rule (where the workload's maps come from the rule),
pack of A and B (and of C when beta != 0), schedule, and gemm_mp_run.  Unpacking is
verification only and is not timed.

The default workload is the largest single-GPU configuration, cov64k (65536^3, tile 2048).  With
no --workload given the two other large configurations (cov16k, rect32k) are run after it, a few
steps each, and reported under "also" in the same line.

Prints ONE JSON line.  `value` is the effective rate 2*M*N*K / t_step in TFLOP/s; `roofline`
prices gemm_mp_run (the owner-workgroup GEMM kernels) against the precision-weighted MFMA peak of
this workload's product mix; `cpu_baseline` is the CPU oracle timed on a bounded sample of the
same workload on this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published dense peaks, TFLOP/s, by product precision code (FP64, FP32, FP16, FP8).
PEAK_TFLOPS = [78.6, 157.3, 2516.6, 5033.2]
PEAK_FP4_TFLOPS = 10066.4
DTYPE_NAMES = ["f64", "f32", "f16", "f8e4m3"]
HEADLINE = "cov64k"
ALSO = ("cov16k", "rect32k")
# the second argument of the 256 x 256 kernels: block-scaled tiles of up to 1024 take the instance that moves the scale
# bytes through LDS
KERNEL_NAMES = ["gemm_mp_owner_kernel<double%s>", "gemm_mp_owner_kernel<float%s>", "gemm_mp_fp8_region_kernel<0, false>",
                "gemm_mp_fp8_region_kernel<1, %s>", "gemm_mp_fp8_region_kernel<2, %s>", "gemm_mp_fp8_region_kernel<3, false>",
                "gemm_mp_fp8_region_kernel<4, false>", "gemm_mp_fp8_region_kernel<5, %s>"]
INSTANCE = [", false, false", ", true, false", ", true, true", None]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default=None,
                    choices=["tiny", "random8k", "cov16k", "rect32k", "cov64k",
                             "paper100", "paper80", "paper50", "paper20", "paper0",
                             "format-fp64", "format-fp32", "format-fp16", "format-fp8", "format-bf16", "format-mxfp8",
                             "format-mxfp4", "format-mxfp6"],
                    help="default: cov64k, followed by short runs of cov16k and rect32k.  paperNN: the paper's own runs, "
                         "NN %% of the tiles FP64 and the rest FP32 (Section 5.2); format-X: 16384^3, tile 1024, every tile "
                         "of A and B stored as X (per-format rates; no CPU baseline)")
    ap.add_argument("--policy", type=int, default=None, choices=[0, 1],
                    help="0 = operand policy, 1 = C-tile policy (default: the workload's own)")
    ap.add_argument("--conversion", default="receiver", choices=["receiver", "sender"],
                    help="receiver: every task converts its operands on the fly (the paper's strategy); sender: tiles are "
                         "converted once per needed precision into a workspace before the run (timed as its own stage)")
    ap.add_argument("--cpu-seconds", type=float, default=24.0, help="target CPU time of the oracle sample")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="only the headline workload")
    ap.add_argument("--operand-values", default="workload", choices=["workload", "zeros"],
                    help="zeros: format-X workloads only, A and B all zero (same kernels, same accesses; shows how much of a "
                         "format's rate the chip's power management takes on real data)")
    ap.add_argument("--sample-clocks", type=float, default=0.0, metavar="SECONDS",
                    help="after the timed steps, loop gemm_mp_run alone for SECONDS while a thread reads the shader clock "
                         "from rocm-smi about once a second; reported under clock_probe")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain 1 GiB device copy, three times (reference for the HBM byte counters)")
    return ap.parse_args()


def cpu_baseline(w, A, B, C0, seconds):
    """Time the oracle, as it stands, on a bounded sample of this workload's C tiles."""
    import numpy as np
    from oracle import gemm_mp_oracle as orc
    from oracle.checker import OracleSide

    side = OracleSide(w, A, B, C0)
    tiles = w.sample_tiles(64)
    nb = w.nb
    rows = min(nb, 64)
    flops_per_row = 2.0 * nb * w.K

    def run(jobs):
        t0 = time.perf_counter()
        side.gemm(np.array(jobs, dtype=np.int32))
        return time.perf_counter() - t0

    def sample(want_rows):
        jobs, left = [], want_rows
        for (I, J) in tiles:
            if left <= 0:
                break
            r = min(nb, left)
            jobs.append([I, J, 0, r, 0, nb])
            left -= r
        return jobs

    # the first call pays thread start-up and page faults: probe twice, then size the sample
    run(sample(rows))
    jobs = sample(4 * rows)
    t = run(jobs)
    for _ in range(3):
        done = sum(j[3] for j in jobs)
        if t >= seconds / 3 or done >= len(tiles) * nb:
            break
        want = int(min(len(tiles) * nb, max(2 * done, done * seconds / max(t, 1e-3))))
        jobs = sample(want)
        t = run(jobs)
    done_rows = sum(j[3] for j in jobs)
    return {"value": done_rows * flops_per_row / t / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(),
            "kind": "oracle", "seconds": round(t, 2),
            "sample": "%d rows x %d cols of %d seeded C tiles of %s (all reduction tiles), %.3g flop"
                      % (done_rows, nb, len(jobs), w.name, done_rows * flops_per_row)}


def clock_probe(d, w, seconds):
    """Loop gemm_mp_run alone for `seconds`; a thread samples the shader clock meanwhile (rocm-smi, a child process)."""
    import re
    import subprocess
    import threading

    import numpy as np
    import torch

    samples, stop = [], threading.Event()

    def sampler():
        while not stop.is_set():
            try:
                txt = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=20).stdout
                m = re.search(r"sclk[^\n]*\((\d+)Mhz\)", txt)
                if m:
                    samples.append(int(m.group(1)))
            except Exception:
                pass
            stop.wait(0.5)

    d.run(w.alpha, w.beta)
    torch.cuda.synchronize()
    th = threading.Thread(target=sampler)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    th.start()
    time.sleep(1.0)                       # the first sample may still see the idle clock
    t0, runs = time.perf_counter(), 0
    e0.record()
    while time.perf_counter() - t0 < seconds:
        for _ in range(4):
            d.run(w.alpha, w.beta)
        runs += 4
        torch.cuda.synchronize()
    e1.record()
    torch.cuda.synchronize()
    stop.set()
    th.join()
    under_load = samples[1:] if len(samples) > 1 else samples
    return {"seconds": seconds, "runs": runs, "run_ms": e0.elapsed_time(e1) / runs,
            "sclk_mhz": {"median": float(np.median(under_load)) if under_load else None,
                         "min": min(under_load) if under_load else None, "max": max(under_load) if under_load else None,
                         "samples": len(under_load)},
            "source": "rocm-smi --showclocks, about one reading a second while gemm_mp_run loops (beta as in the workload)"}


def hbm_rates(w, st, ms, packs_c):
    """The HBM-bound passes in GB/s of their algorithmic bytes (peak 8000): the tile scan reads 8 bytes per
    element of A and of B (its time includes the rule on the host and the waits for it); pack reads 8 bytes per
    element and writes the packed tiles."""
    elems = [w.M * w.K, w.K * w.N, w.M * w.N]
    out = {}
    if w.rule is not None and ms["scan_rule"] > 0:
        out["scan_rule_GBps"] = 8.0 * (elems[0] + elems[1]) / (ms["scan_rule"] * 1e-3) / 1e9
    which = (0, 1, 2) if packs_c else (0, 1)
    if ms["pack"] > 0:
        out["pack_GBps"] = sum(8.0 * elems[i] + st["packed_bytes"][i] for i in which) / (ms["pack"] * 1e-3) / 1e9
    out["note"] = "algorithmic bytes over the stage's HIP-event time; where the maps were set by hand, pack first scans the matrices that have FP16 / FP8 tiles (8 more bytes per element, not counted)"
    return out


def measure(name, steps, warmup, policy, conversion, cpu_seconds, operand_values="workload", clock_seconds=0.0):
    """Run one workload; returns the fields of its JSON record.  cpu_seconds = 0: no CPU baseline."""
    import numpy as np
    import torch

    import workloads as W
    from paper_2508_14848_amd.device import DeviceGemmMP

    dev = "cuda:0"
    w = W.CONFIGS[name]()
    if policy is None:
        policy = w.policy
    t0 = time.perf_counter()
    A = w.dense("A")
    B = A if w.a_equals_b else w.dense("B")
    C0 = w.dense("C") if w.beta != 0.0 else None
    t_gen = time.perf_counter() - t0
    if operand_values == "zeros":
        assert name.startswith("format-"), "--operand-values zeros: format-X workloads only (their maps do not depend on the data)"
        A = np.zeros_like(A)
        B = A if w.a_equals_b else np.zeros_like(B)
    dA = torch.from_numpy(A).to(dev)
    dB = dA if w.a_equals_b else torch.from_numpy(B).to(dev)
    dC = torch.from_numpy(C0).to(dev) if C0 is not None else None
    torch.cuda.synchronize()

    d = DeviceGemmMP(w.M, w.N, w.K, w.nb, device=dev, policy=policy)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    stage_names = ("scan_rule", "pack", "convert", "schedule", "run")
    stage_ms = {k: [] for k in stage_names}

    def step(record):
        e = [ev() for _ in range(6)]
        e[0].record()
        if w.rule is not None:
            d.compute_precision_map("A", dA, w.rule["eps"], w.rule["allowed"])
            d.compute_precision_map("B", dB, w.rule["eps"], w.rule["allowed"])
        else:
            d.set_precision_map("A", w.mapA)
            d.set_precision_map("B", w.mapB)
        d.set_precision_map("C", w.mapC)
        e[1].record()
        d.pack_tiles("A", dA)
        d.pack_tiles("B", dB)
        if dC is not None:
            d.pack_tiles("C", dC)
        e[2].record()
        if conversion == "sender":
            d.convert_tiles()
        e[3].record()
        d.prepare()                   # the schedule: host work plus small copies queued on the stream
        e[4].record()
        d.run(w.alpha, w.beta)        # the product table kernel and the GEMM launches, nothing else
        e[5].record()
        if record:
            torch.cuda.synchronize()
            for k, a in zip(stage_names, range(5)):
                stage_ms[k].append(e[a].elapsed_time(e[a + 1]))

    for _ in range(warmup):
        step(False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step(True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / steps * 1e3

    st = d.ctx.get_stats()
    flops_total = 2.0 * w.M * w.N * w.K
    assert abs(sum(st["flops"]) + st["flops_bf16"] + st["flops_mxfp8"] + st["flops_mxfp4"] + st["flops_mxfp6"] - flops_total) < 1e-6 * flops_total
    t_roof = sum(f / (p * 1e12) for f, p in zip(st["flops"], PEAK_TFLOPS))          # seconds
    t_roof += st["flops_bf16"] / (PEAK_TFLOPS[2] * 1e12)                             # BF16 peak = FP16 peak
    t_roof += st["flops_mxfp8"] / (PEAK_TFLOPS[3] * 1e12)                            # block-scaled FP8: the FP8 peak
    t_roof += (st["flops_mxfp4"] + st["flops_mxfp6"]) / (PEAK_FP4_TFLOPS * 1e12)     # block-scaled FP4 and FP6: 10.1 PFLOP/s
    run_ms = float(np.mean(stage_ms["run"]))
    achieved = flops_total / (run_ms * 1e-3) / 1e12
    peak_mix = flops_total / t_roof / 1e12
    traffic, traffic_from = None, None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        key = w.name + ("" if policy == w.policy else "-policy%d" % policy) + ("" if conversion == "receiver" else "-sender")
        entry = json.load(open(tpath)).get(key)
        if entry:
            traffic, traffic_from = entry.get("bytes_per_launch"), "profiles/traffic.json: " + entry.get("source", "")
    used = [DTYPE_NAMES[q] for q in range(4) if st["products"][q]]
    used += [n for n in ("bf16", "mxfp8", "mxfp4", "mxfp6") if st["products_" + n]]
    launched = []
    for k, n in enumerate(st["launch_items"][:8]):
        if n:
            kn = KERNEL_NAMES[k]
            if k < 2:
                inst = INSTANCE[st["owner_instance"][k]]
                kn = kn % inst if inst else "gemm_mp_owner_low_kernel<false>"
            elif "%s" in kn:
                kn = kn % ("true" if w.nb <= 1024 else "false")
            launched.append({"kernel": kn, "workgroups": n})
    out = {
        "metric": "effective TFLOP/s (2MNK/t) and % of precision-weighted MFMA peak, 1 GPU",
        "value": flops_total / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "+".join(used), "data": "synthetic",
        "config": {"workload": w.name, "M": w.M, "N": w.N, "K": w.K, "tile_nb": w.nb,
                   "alpha": w.alpha, "beta": w.beta, "policy": ["operand", "c_tile"][policy],
                   "conversion": conversion, "converted_tiles": st["converted_tiles"],
                   "converted_bytes": st["converted_bytes"],
                   "products_by_precision": dict(list(zip(DTYPE_NAMES, st["products"])) +
                                                 [(n, st["products_" + n]) for n in ("bf16", "mxfp8", "mxfp4", "mxfp6") if st["products_" + n]]),
                   "work_items": st["work_items"], "host_generation_s": round(t_gen, 1),
                   "operand_values": operand_values},
        "stages_ms": {k: float(np.mean(v)) for k, v in stage_ms.items()},
        "stages_hbm": hbm_rates(w, st, {k: float(np.mean(v)) for k, v in stage_ms.items()}, dC is not None),
        "run_only": {"ms": run_ms, "min_ms": float(np.min(stage_ms["run"])), "effective_tflops": achieved,
                     "roofline_ms": t_roof * 1e3, "frac_of_precision_weighted_peak": t_roof * 1e3 / run_ms},
        "roofline": {"bound": "mfma", "kernel": "gemm_mp_run: product_table_kernel + " + " + ".join(k["kernel"] for k in launched),
                     "launches": launched, "achieved": achieved, "peak": peak_mix,
                     "unit": "TFLOP/s", "frac": achieved / peak_mix, "traffic": traffic, "traffic_source": traffic_from,
                     "note": "peak = 2MNK / sum_q(F_q/P_q), P = 78.6/157.3/2516.6/5033.2 TFLOP/s for f64/f32/f16/f8; "
                             "achieved = 2MNK / mean HIP-event time of gemm_mp_run on its stream (the launches listed); "
                             "traffic = HBM bytes per gemm_mp_run from rocprofv3 counter passes of this command, kept in "
                             "profiles/ (null: no pass recorded for this workload)"},
    }
    if clock_seconds > 0:
        out["clock_probe"] = clock_probe(d, w, clock_seconds)
    if cpu_seconds > 0 and not w.name.startswith("format-"):
        out["cpu_baseline"] = cpu_baseline(w, A, B, C0, cpu_seconds)
    del d, dA, dB, dC, A, B, C0
    torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU path (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import torch

    from paper_2508_14848_amd import gemm_mp as G

    G.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.calibrate_copy:
        src = torch.ones(1 << 27, dtype=torch.float64, device="cuda:0")          # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "plain copy", "bytes_read": src.numel() * 8, "bytes_written": src.numel() * 8}))
        return
    name = args.workload or HEADLINE
    out = measure(name, args.steps, args.warmup, args.policy, args.conversion, 0.0 if args.no_cpu_baseline else args.cpu_seconds,
                  args.operand_values, args.sample_clocks)
    if args.workload is None and not args.no_also:
        # the other configurations of 16384^3 and more, a few steps each: run-only figures
        out["also"] = {}
        for other in ALSO:
            r = measure(other, min(args.steps, 5), min(args.warmup, 2), None, args.conversion, 0.0)
            out["also"][other] = {"ms_per_step": r["ms_per_step"], "value": r["value"], "run_only": r["run_only"],
                                  "roofline_frac": r["roofline"]["frac"], "launches": r["roofline"]["launches"],
                                  "products_by_precision": r["config"]["products_by_precision"], "steps": r["steps"]}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
