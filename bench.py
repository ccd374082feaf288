#!/usr/bin/env python3
"""Benchmark of the fitness-and-validity evaluation step on one MI355X.

One step = one pass of the whole hot path over one synthetic population: the
batched (or segmented) tolerance check of every candidate against its reference,
then the median-timing / speedup / fitness reduction.  Inputs are resident in HBM
before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--spinup-ms MS] [--workload c2|c1|c3|c3h|c4|c5|cases|f64|i32|i64]
                    [--no-cpu-baseline] [--no-read-ceiling] [--copy-calibration] [--no-extra-workloads]
                    [--sweep populations|small|cases|broken]

The JSON line is about --workload (default c2, the configuration the metric is quoted on).  With
the default workload it also carries "workloads": the same measurement of the other large
single-GPU workloads (c3, c4, c5; 20 steps each, after a spin-up of their own, the previous
workload's tensors released first) with their roofline fractions and an agreement check of a
stated pick of their rows against the CPU oracle on the whole tensors.

--copy-calibration runs only a plain device-to-device copy of known size (used to
scale the rocprofv3 FETCH_SIZE / WRITE_SIZE counters) and prints its own JSON line.

Before the workload is built, the stand-alone probe paper_2510_03760_amd/read_ceiling
(a trivial read-only kernel over 8 GiB, run as a child process) measures what this
machine streams at best; the JSON line carries it beside the vendor peak.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "candidate-elements validated/sec and achieved HBM GB/s vs MI355X peak"
HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, vendor figure


def measured_traffic(workload_name: str):
    """HBM bytes per launch of the check kernel from the committed rocprofv3 counter
    summary, or None when there is none for this workload or the kernel sources have
    changed since the counters were taken."""
    import glob
    import hashlib
    try:
        with open(os.path.join(ROOT, "profiles", "hbm_traffic.json")) as fh:
            table = json.load(fh)
        entry = table[workload_name]
        h = hashlib.sha256()
        for f in sorted(glob.glob(os.path.join(ROOT, "paper_2510_03760_amd", "csrc", "*"))):
            with open(f, "rb") as src:
                h.update(src.read())
        if h.hexdigest()[:16] != entry["src_hash"]:
            return None
        return entry["traffic_bytes"]
    except (OSError, KeyError, ValueError):
        return None


def read_ceiling():
    """Best read-only streaming rate of this GPU in GB/s from the stand-alone probe, or
    None when the probe is not built or fails."""
    import subprocess
    exe = os.path.join(ROOT, "paper_2510_03760_amd", "read_ceiling")
    if not os.path.exists(exe):
        return None
    try:
        res = subprocess.run([exe, "8"], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True,
                             timeout=120)
        if res.returncode != 0:
            return None
        return json.loads(res.stdout.strip().splitlines()[-1])
    except (OSError, ValueError, subprocess.TimeoutExpired, IndexError):
        return None


def build_workload(name: str):
    import synth
    if name == "c1":
        return synth.tiny("cuda")
    if name == "c2":
        return synth.dense_f32("cuda", side=8192, P=16, T=100)
    if name == "c3":
        return synth.softmax_bf16("cuda", B=32, R=128, C=4096, P=64, T=100)
    if name == "c4":
        return synth.ragged_f32("cuda", P_s=32, T=100)
    if name == "c5":
        return synth.heavy_tail_f32("cuda", log2n=30, P=8, T=1000)
    if name == "c3h":
        import torch
        return synth.softmax_bf16("cuda", B=32, R=128, C=4096, P=64, T=100, dtype=torch.float16)
    if name in ("f64", "i32", "i64"):
        import torch
        dt = {"f64": torch.float64, "i32": torch.int32, "i64": torch.int64}[name]
        # the bytes of the default workload: 2^26 four-byte or 2^25 eight-byte elements
        return synth.dense_typed("cuda", dt, n=(1 << 26) if name == "i32" else (1 << 25), P=16, T=100)
    if name == "cases":
        return synth.multi_case_f32("cuda", K=5, side=4096, P=16, T=100)
    raise SystemExit("unknown workload %r" % name)


def cpu_baseline(w, budget_elems: int):
    """Times the CPU oracle, as it stands, on one thread over a bounded sample of the
    same population (a prefix of each tensor, all candidates)."""
    import numpy as np
    import oracle
    import synth
    total = w.cand_elems
    frac = min(1.0, budget_elems / float(total))
    t_all = 0.0
    done = 0
    rows = []
    for seg in w.segments:
        m = seg.n if frac >= 1.0 else max(1, int(seg.n * frac))
        dt = {"bf16": oracle.BF16, "f16": oracle.F16, "f64": oracle.F64, "i32": oracle.I32,
              "i64": oracle.I64}.get(seg.dtype_name, oracle.F32)
        ref = synth.to_oracle_array(seg.ref[:m])
        for c in seg.cands:
            ch = synth.to_oracle_array(c[:m])
            t0 = time.perf_counter()
            rows.append(oracle.check_one(ref, ch, dt, w.atol, w.rtol))
            t_all += time.perf_counter() - t0
            done += m
    tim = w.timings.cpu().numpy()
    base = w.baseline.cpu().numpy()
    if w.notes.get("cases"):   # a candidate is valid iff it passes every case
        P = w.P
        valid = np.array([int(all(rows[k * P + p]["valid"] for k in range(len(w.segments))))
                          for p in range(P)], np.uint32)
    else:
        valid = np.array([r["valid"] for r in rows], np.uint32)
    t0 = time.perf_counter()
    oracle.fitness(tim, base, valid)
    t_all += time.perf_counter() - t0
    sample = ("first %.1f%% of every tensor, all %d candidates, plus the full timing table"
              % (100.0 * done / total, w.P))
    one = {"value": done / t_all, "unit": "cand-elem/s", "cores": 1, "kind": "oracle",
           "sample": sample, "seconds": round(t_all, 3)}

    # The same oracle on the same sample with whole candidates side by side (every candidate
    # is still reduced sequentially by one thread, so the rows are the same bytes).
    threads = max(1, min(16, os.cpu_count() or 1, max(len(s.cands) for s in w.segments)))
    t_par = 0.0
    for seg in w.segments:
        m = seg.n if frac >= 1.0 else max(1, int(seg.n * frac))
        dt = {"bf16": oracle.BF16, "f16": oracle.F16, "f64": oracle.F64, "i32": oracle.I32,
              "i64": oracle.I64}.get(seg.dtype_name, oracle.F32)
        ref = synth.to_oracle_array(seg.ref[:m])
        cands = [synth.to_oracle_array(c[:m]) for c in seg.cands]
        t0 = time.perf_counter()
        oracle.check_batch(ref, cands, dt, w.atol, w.rtol, threads=threads)
        t_par += time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.fitness(tim, base, valid)
    t_par += time.perf_counter() - t0
    one["all_cores"] = {"value": done / t_par, "unit": "cand-elem/s", "cores": threads,
                        "seconds": round(t_par, 3)}
    return one, rows, frac


def oracle_agreement(w, got, cand_pick, threads: int, chunk: int = 1 << 24):
    """The GPU rows of the picked candidates of every group against the oracle on the WHOLE
    tensors (copied to the host chunk by chunk; whole candidates side by side on `threads`
    threads, each still reduced sequentially): integers, flags and maxima byte for byte,
    the two error sums to 1e-6.  Part of the cpu_baseline leg."""
    import numpy as np
    import oracle
    import synth
    from concurrent.futures import ThreadPoolExecutor
    t0 = time.perf_counter()
    same, n_rows, row0 = True, 0, 0
    for seg in w.segments:
        dt = {"bf16": oracle.BF16, "f16": oracle.F16, "f64": oracle.F64, "i32": oracle.I32,
              "i64": oracle.I64}.get(seg.dtype_name, oracle.F32)
        picked = [p for p in range(len(seg.cands)) if cand_pick(p)]
        accs = [oracle.CheckAccumulator(dt, w.atol, w.rtol) for _ in picked]
        with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
            for lo in range(0, seg.n, chunk):
                hi = min(seg.n, lo + chunk)
                r = synth.to_oracle_array(seg.ref[lo:hi])
                list(ex.map(lambda ap: ap[0].feed(r, synth.to_oracle_array(seg.cands[ap[1]][lo:hi])),
                            zip(accs, picked)))
        for acc, p in zip(accs, picked):
            o, g = acc.result(), got[row0 + p]
            ok = (int(g["n_mismatch"]) == o["n_mismatch"] and int(g["n_finite"]) == o["n_finite"] and
                  int(g["flags"]) == o["flags"] and int(g["valid"]) == o["valid"] and
                  g["max_abs_err"].tobytes() == o["max_abs_err"].tobytes() and
                  g["max_rel_err"].tobytes() == o["max_rel_err"].tobytes())
            for f in ("sum_abs_err", "sum_rel_err"):
                a, b = float(g[f]), float(o[f])
                ok = ok and (a == b or abs(a - b) <= 1e-6 * abs(b))
            same = same and ok
            n_rows += 1
        row0 += len(seg.cands)
    return same, n_rows, time.perf_counter() - t0


def sweep(mode: str, steps: int) -> int:
    """Other shapes than the five workloads, evo_check_batch / evo_check_cases alone (no timing
    reduction), one JSON line per shape: median time between HIP events around each call and the
    algorithmic bytes over it as a fraction of the HBM peak.
      populations  P = 1..33 candidates at 2.4-4.6 GB per launch, fp32 and bf16
      small        fp32 launches of 8 MB to 1.1 GB
      cases        K = 5 test cases of P = 1..8 candidates (the shape of one evaluation in the
                   paper's loop), fp32, 2^20 / 2^24 / 2^26 elements per tensor
      broken       16 candidates of which 0, 1, 4 or all hold a NaN in every 64th place or are
                   NaN throughout (what kernels with a bug produce), and a reference that holds
                   -Inf in every 65536th, 4096th or 64th place with candidates that copy it;
                   fp32, bf16 and fp64 at 2.3 GB per launch"""
    import torch
    import paper_2510_03760_amd as evo

    def run(dt, n, P, K=1, spoil=None, note=None):
        tdt = {"f32": torch.float32, "bf16": torch.bfloat16, "f64": torch.float64}[dt]
        code = {"f32": evo.EVO_F32, "bf16": evo.EVO_BF16, "f64": evo.EVO_F64}[dt]
        g = torch.Generator(device="cuda")
        g.manual_seed(1)
        refs = [torch.rand(n, device="cuda", generator=g).to(tdt) for _ in range(K)]
        if spoil is not None and spoil[0] == "ref":
            refs[0][::spoil[1]] = float("-inf")
        cands = [[(r.double() * 1.0001).to(tdt) for _ in range(P)] for r in refs]
        if spoil is not None and spoil[0] == "cand":
            for k in range(spoil[2]):
                cands[0][(5 * k + 3) % P][::spoil[1]] = float("nan")
        chk = evo.Checker(code, n, 1e-2, 1e-2)
        stats = chk.new_stats(P)
        cases = [{"ref": r, "cand_ptrs": c, "n_elems": n, "dtype": code} for r, c in zip(refs, cands)]
        call = ((lambda: chk.check_batch(refs[0], cands[0], stats)) if K == 1 else
                (lambda: chk.check_cases(cases, stats)))
        for _ in range(25):
            call()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        ev[0].record()
        for i in range(steps):
            call()
            ev[i + 1].record()
        torch.cuda.synchronize()
        ms = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
        med = ms[len(ms) // 2]
        byt = K * (P + 1) * n * refs[0].element_size()
        line = {"sweep": mode, "dtype": dt, "n_elems": n, "P": P, "K": K, "algorithmic_bytes": byt,
                "median_us": round(med * 1e3, 1), "GBps": round(byt / med / 1e6, 0),
                "frac_of_peak": round(byt / med / 1e6 / HBM_PEAK_GBS, 3),
                "entry": "evo_check_batch" if K == 1 else "evo_check_cases"}
        if note is not None:
            line["input"] = note
        print(json.dumps(line), flush=True)
        chk.close()

    if mode == "populations":
        for dt, es in (("f32", 4), ("bf16", 2)):
            for P in (1, 2, 3, 4, 5, 7, 8, 9, 11, 12, 13, 15, 16, 17, 24, 33):
                n = (1 << 29) if dt == "f32" else (1 << 30)
                while (P + 1) * n * es > 4.7e9:
                    n >>= 1
                run(dt, n, P)
    elif mode == "small":
        for P, lg in ((1, 20), (1, 22), (1, 24), (4, 22), (16, 20), (16, 21), (16, 22), (16, 23), (16, 24), (64, 20)):
            run("f32", 1 << lg, P)
    elif mode == "cases":
        for P in (1, 2, 4, 8):
            for lg in (20, 24, 26):
                run("f32", 1 << lg, P, K=5)
    elif mode == "broken":
        for dt, lg in (("f32", 25), ("bf16", 26), ("f64", 24)):
            run(dt, 1 << lg, 16, note="clean")
            for k in (1, 4, 16):
                run(dt, 1 << lg, 16, spoil=("cand", 64, k), note="%d of 16 candidates with NaN in every 64th place" % k)
            for k in (4, 16):
                run(dt, 1 << lg, 16, spoil=("cand", 1, k), note="%d of 16 candidates NaN throughout" % k)
            for stride in (65536, 4096, 64):
                run(dt, 1 << lg, 16, spoil=("ref", stride), note="reference -Inf in every %dth place, candidates copy it" % stride)
    else:
        print("bench.py: unknown sweep %r (populations, small, cases, broken)" % mode, file=sys.stderr)
        return 2
    return 0


def measure(name: str, steps: int, warmup: int, spinup_ms: float, split: bool):
    """Builds workload `name`, spins the device up, runs `warmup` untimed and `steps` timed steps
    and returns (result fields, workload, checker, stats, summary).  Two events on the launch
    stream, one before and one behind the K launches, give the dominant kernel's average launch
    duration (see the timed region below)."""
    import torch
    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy, summary_to_numpy

    w = build_workload(name)
    torch.cuda.synchronize()
    segs = w.segments
    dcode = lambda s: {"bf16": evo.EVO_BF16, "f16": evo.EVO_F16, "f64": evo.EVO_F64,  # noqa: E731
                       "i32": evo.EVO_I32, "i64": evo.EVO_I64}.get(s.dtype_name, evo.EVO_F32)
    chk = evo.Checker(dcode(segs[0]), segs[0].n, w.atol, w.rtol)
    P = w.P
    stats = chk.new_stats(P)
    summary = chk.new_summary()
    stream = torch.cuda.current_stream()
    seg_descs = None
    is_cases = bool(w.notes.get("cases"))
    if is_cases:
        seg_descs = [{"ref": s.ref, "cand_ptrs": s.cands, "n_elems": s.n, "dtype": dcode(s)}
                     for s in segs]
    elif len(segs) > 1:
        row0, seg_descs = 0, []
        for s in segs:
            seg_descs.append({"ref": s.ref, "cand_ptrs": s.cands, "n_elems": s.n,
                              "dtype": dcode(s), "stats_row0": row0})
            row0 += len(s.cands)

    def check():
        if seg_descs is None:
            chk.check_batch(segs[0].ref, segs[0].cands, stats, stream=stream)
        elif is_cases:
            chk.check_cases(seg_descs, stats, stream=stream)
        else:
            chk.check_segmented(seg_descs, stats, P, stream=stream)

    # One call (one launch) for the whole step: evo_evaluate where the population has one
    # reference per test case, evo_evaluate_segmented for the ragged workload.
    fused = not split
    ragged = seg_descs is not None and not is_cases
    eval_cases = seg_descs if is_cases else [{"ref": segs[0].ref, "cand_ptrs": segs[0].cands,
                                              "n_elems": segs[0].n, "dtype": dcode(segs[0])}]

    def step(mid=None):
        if fused and ragged:
            chk.evaluate_segmented(seg_descs, w.timings, w.baseline, stats, P, summary, stream=stream)
        elif fused:
            chk.evaluate(eval_cases, w.timings, w.baseline, stats, summary, stream=stream)
        else:
            check()
            if mid is not None:
                mid.record(stream)
            chk.fitness(w.timings, w.baseline, stats, summary, stream=stream)

    # Spin-up: the first tens of milliseconds of load in a process run at a varying clock (the
    # same launch took 345-460 us over its first 60 repetitions and 345-355 us afterwards), and
    # on a device that has been idle the first process can run at 0.6 of its later rate for
    # longer than that.  The device is kept busy with the step for a stated time before the W
    # warm-up steps, and beyond it (up to 2 s) until two consecutive batches of steps take the
    # same time within 3 %.
    # no cyclic garbage collection between here and the end of the timed region: with torch
    # imported a full collection takes 5-20 ms, during which nothing is launched (as timeit does)
    gc.collect()
    gc.disable()
    spun, per_batch = 0, 4
    t_spin = time.perf_counter()
    last = None
    while spinup_ms > 0:
        t_b = time.perf_counter()
        for _ in range(per_batch):
            step()
        torch.cuda.synchronize()
        now = time.perf_counter()
        spun += per_batch
        took = now - t_b
        if took < 1e-3:                       # batches of at least a millisecond
            per_batch *= 4
            last = None
            continue
        elapsed_ms = (now - t_spin) * 1e3
        settled = last is not None and abs(took - last) <= 0.03 * last
        last = took
        if elapsed_ms >= 2000.0 or (elapsed_ms >= spinup_ms and settled):
            break
    spin_ms = (time.perf_counter() - t_spin) * 1e3
    # the warm-up steps record events the way the timed steps do, so that whatever the runtime
    # sets up for the first events of a process is set up before the timed region
    for _ in range(warmup):
        torch.cuda.Event(enable_timing=True).record(stream)
        step(None if fused else torch.cuda.Event(enable_timing=True))
    torch.cuda.Event(enable_timing=True).record(stream)
    torch.cuda.synchronize()

    # The timed region.  One launch per step (the fused entry points): one event before the K
    # steps and one after them, on the launch stream -- the kernel's average launch duration is
    # the time between the two over K, launch gaps included.  An event between every two
    # launches would cost 2.8-3.0 us per launch by itself (measured: 2^26 x 16 fp32 677.4 against
    # 674.4 us per launch, 2^24 x 64 bf16 345.8 / 343.0), which is the measurement's, not the
    # path's.  Two launches per step (--split): one event per launch boundary, since the two
    # kernels have to be told apart.
    bounds = [torch.cuda.Event(enable_timing=True) for _ in range(2 if fused else steps + 1)]
    mids = [None if fused else torch.cuda.Event(enable_timing=True) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    bounds[0].record(stream)
    for k in range(steps):
        step(mids[k])
        if not fused:
            bounds[k + 1].record(stream)
    if fused:
        bounds[1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_per_step = wall * 1e3 / steps
    if fused:
        check_avg = bounds[0].elapsed_time(bounds[1]) / steps
        # the spread of single launches, from a pass of its own behind the timed region (one
        # event per launch boundary, so each figure carries that event's 3 us)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        marks[0].record(stream)
        for k in range(steps):
            step()
            marks[k + 1].record(stream)
        torch.cuda.synchronize()
        check_ms = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(steps))
        fit_ms = [0.0]
    else:
        check_ms = sorted(bounds[k].elapsed_time(mids[k]) for k in range(steps))
        fit_ms = sorted(mids[k].elapsed_time(bounds[k + 1]) for k in range(steps))
        check_avg = sum(check_ms) / len(check_ms)
    gc.enable()
    alg_bytes = w.algorithmic_bytes
    achieved = alg_bytes / (check_avg * 1e-3) / 1e9

    fields = {
        "ms_per_step": ms_per_step,
        "cand_elems_per_s": w.cand_elems / (wall / steps),
        "spinup": {"min_ms": spinup_ms, "ms": spin_ms, "steps": spun},
        "dtype": {"bf16": "bf16->f32", "f16": "f16->f32", "f64": "f64", "i32": "i32",
                  "i64": "i64"}.get(segs[0].dtype_name, "f32"),
        "config": {"workload": w.name, "P": P, "cand_elems": w.cand_elems,
                   "algorithmic_bytes": alg_bytes, "T": int(w.timings.shape[1]),
                   "atol": w.atol, "rtol": w.rtol,
                   "entry": ("evo_evaluate_segmented" if ragged else "evo_evaluate") if fused else
                            ("evo_check_batch" if seg_descs is None else
                             "evo_check_cases" if is_cases else "evo_check_segmented") + "+evo_fitness"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic(w.name),
                     "kernel": "evo_evaluate_kernel" if fused else "evo_check_kernel", "avg_ms": check_avg,
                     "how": ("events around the K timed launches" if fused else "one event per launch boundary"),
                     "median_ms": check_ms[len(check_ms) // 2], "min_ms": check_ms[0],
                     "single_launches": ("separate pass, one event per launch" if fused else "timed region")},
        "fitness_kernel_us": None if fused else {"avg": 1e3 * sum(fit_ms) / len(fit_ms),
                                                 "median": 1e3 * fit_ms[len(fit_ms) // 2]},
        "hbm_gbps_whole_step": alg_bytes / (wall / steps) / 1e9,
    }
    return fields, w, chk, stats, summary, stream, is_cases


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2")
    ap.add_argument("--spinup-ms", type=float, default=60.0,
                    help="untimed load before the warm-up steps, in milliseconds")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget-elems", type=float, default=2.0e9,
                    help="candidate-elements the CPU oracle is timed on (about 160 M/s/core)")
    ap.add_argument("--copy-calibration", action="store_true")
    ap.add_argument("--no-read-ceiling", action="store_true")
    ap.add_argument("--split", action="store_true",
                    help="two calls per step (check, then fitness) also where evo_evaluate applies")
    ap.add_argument("--sweep", default=None, help="populations | small | cases | broken: other shapes and inputs, one JSON line each")
    ap.add_argument("--no-extra-workloads", action="store_true",
                    help="with the default workload: do not measure the other large workloads afterwards")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path is built and measured on ONE GPU; --gpus %d is not "
              "supported (a population shards by candidate: every GPU checks the candidates it "
              "ran, and only the 72-byte result rows are gathered)" % args.gpus,
              file=sys.stderr)
        return 2

    # child process, finished before this process touches the GPU
    ceiling = None if (args.no_read_ceiling or args.copy_calibration or args.sweep) else read_ceiling()

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    torch.cuda.set_device(0)

    if args.sweep:
        return sweep(args.sweep, min(args.steps, 40))

    if args.copy_calibration:
        n = 1 << 30   # bytes
        src = torch.empty(n, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "launches": args.steps + 3,
                          "ms_per_copy": ms, "GBps_read_plus_write": 2 * n / ms / 1e6}))
        return 0

    import paper_2510_03760_amd as evo
    from paper_2510_03760_amd.binding import stats_to_numpy, summary_to_numpy

    fields, w, chk, stats, summary, stream, is_cases = measure(args.workload, args.steps, args.warmup,
                                                               args.spinup_ms, args.split)
    P = w.P
    out = {
        "metric": METRIC,
        "value": fields["cand_elems_per_s"],
        "unit": "cand-elem/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "spinup": fields["spinup"],
        "ms_per_step": fields["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": fields["dtype"],
        "data": "synthetic",
        "config": fields["config"],
        "roofline": fields["roofline"],
        "fitness_kernel_us": fields["fitness_kernel_us"],
        "hbm_gbps_whole_step": fields["hbm_gbps_whole_step"],
    }
    achieved = fields["roofline"]["achieved"]
    if ceiling is not None:
        best = max(ceiling["nontemporal_GBps"], ceiling["plain_GBps"])
        out["read_ceiling"] = {"GBps": best, "plain_loads_GBps": ceiling["plain_GBps"],
                               "frac_of_ceiling": achieved / best,
                               "how": "read-only sweep of 8 GiB, paper_2510_03760_amd/read_ceiling"}

    # Outside the timed step: elite selection (population management) on the same rows.
    k_elite = min(4, P)
    elite = torch.zeros(k_elite, dtype=torch.int32, device="cuda")
    n_elite = torch.zeros(1, dtype=torch.int32, device="cuda")
    sel = []
    for _ in range(10):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(stream)
        chk.select_elite(stats, P, k_elite, elite, n_elite, stream=stream)
        b.record(stream)
        sel.append((a, b))
    torch.cuda.synchronize()
    sel_us = sorted(1e3 * a.elapsed_time(b) for a, b in sel)
    out["elite_select_us"] = {"median": sel_us[len(sel_us) // 2], "k": k_elite,
                              "elite": elite.cpu().tolist()}

    got = stats_to_numpy(stats)
    pop = summary_to_numpy(summary)[0]
    out["result"] = {"n_valid": int(pop["n_valid"]), "best_idx": int(pop["best_idx"]),
                     "best_speedup": float(pop["best_speedup"]),
                     "n_mismatch_total": int(got["n_mismatch"].sum())}

    host_cores = os.cpu_count() or 1
    oracle_threads = max(1, min(16, host_cores))
    if not args.no_cpu_baseline:
        base, rows, frac = cpu_baseline(w, int(args.cpu_budget_elems))
        out["cpu_baseline"] = base
        out["cpu_baseline"]["host_cores"] = host_cores
        if frac >= 1.0 and not is_cases:   # the sample was the whole population: report agreement too
            same = all(int(g["n_mismatch"]) == r["n_mismatch"] and
                       g["max_abs_err"].tobytes() == r["max_abs_err"].tobytes() and
                       g["max_rel_err"].tobytes() == r["max_rel_err"].tobytes()
                       for g, r in zip(got, rows))
            out["cpu_baseline"]["agrees_with_gpu"] = bool(same)
    chk.close()

    # The other large single-GPU workloads, each after its own spin-up, with the tensors of the
    # previous one released first: the same measurement, a compact record each.  Agreement with
    # the oracle is checked on the whole tensors of a stated pick of candidates.
    if args.workload == "c2" and not args.no_extra_workloads:
        del w, chk, stats, summary, got
        gc.collect()
        torch.cuda.empty_cache()
        picks = {"c3": ("every 4th candidate and the 8 with permuted rows", lambda p: p % 4 == 0 or p % 8 == 7),
                 "c4": ("every 4th candidate of every group and every corrupted one",
                        lambda p: p % 4 == 0 or p % 4 == 3),
                 "c5": ("candidates 0, 2 (extra NaN sites) and 6 (Inf signs flipped)", lambda p: p in (0, 2, 6))}
        out["workloads"] = {}
        for name in ("c3", "c4", "c5"):
            f2, w2, chk2, stats2, summary2, _, _ = measure(name, min(args.steps, 20), min(args.warmup, 10),
                                                         args.spinup_ms, args.split)
            r2 = f2["roofline"]
            rec = {"ms_per_step": f2["ms_per_step"], "kernel_avg_ms": r2["avg_ms"], "kernel_min_ms": r2["min_ms"],
                   "achieved": r2["achieved"], "frac": r2["frac"], "traffic": r2["traffic"],
                   "cand_elems_per_s": f2["cand_elems_per_s"], "dtype": f2["dtype"],
                   "entry": f2["config"]["entry"], "algorithmic_bytes": f2["config"]["algorithmic_bytes"],
                   "steps": min(args.steps, 20)}
            if not args.no_cpu_baseline:
                torch.cuda.synchronize()
                got2 = stats_to_numpy(stats2)
                same, n_rows, secs = oracle_agreement(w2, got2, picks[name][1], oracle_threads)
                rec["agrees_with_gpu"] = {"value": bool(same), "rows": n_rows, "sample": picks[name][0] +
                                          ", whole tensors", "oracle_threads": oracle_threads,
                                          "seconds": round(secs, 2)}
            out["workloads"][f2["config"]["workload"]] = rec
            chk2.close()
            del w2, chk2, stats2, summary2
            gc.collect()
            torch.cuda.empty_cache()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
