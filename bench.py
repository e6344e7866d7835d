#!/usr/bin/env python3
"""Benchmark of the jagged HSTU attention hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic jagged batch: schedule build,
forward, dk/dv pass, dq pass (forward only for the forward-only workload; for the
context-parallel workload every rank's reorder into its local layout, its partial and the
reorder back, ranks one after the other on the one GPU).
Inputs are resident in HBM before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg5|cfg3|cfg2|cfg4|cfg4_ring|cfg5_bias|short|mid]
                    [--flags N] [--probes] [--no-other-workloads]

A run of the default workload also measures cfg3 and cfg4 (same steps, no CPU leg) and reports them
under `other_workloads`, so that one line carries the fractions of all three long-sequence
configurations; `value` is the default workload's alone.

Beside the nominal peaks the line carries what the machine sustains on matrix instructions alone
(`roofline.measured_peak`, measured in the same run by the library's matrix-instruction loop), and
the CPU leg checks sampled rows of the timed run's own outputs against the oracle.
--probes prints a second JSON line with the measurement kernels alone (matrix loop with constant and
random operands, fp32 atomic adds in the pattern of a dq produced by the dk/dv pass).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E peak


def _traffic_from_profiles(kernel: str, workload: str):
    """HBM bytes per launch measured with rocprofv3 --pmc, if a summary for it is committed."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic_%s_%s.txt" % (kernel, workload))
    try:
        for line in open(path):
            if line.startswith("hbm_bytes_per_launch:"):
                return float(line.split(":")[1].split()[0])
    except OSError:
        pass
    return None


def _measured_mfma_peak(lib, dev, launches: int = 5, iterations: int = 40000):
    """TFLOP/s of the library's matrix-instruction loop (constant operands, random operands):
    HIP events recorded by the library around each launch on the stream it launches on."""
    sink = torch.zeros(64, dtype=torch.float32, device=dev)
    out = {}
    for name, rnd in (("constant", False), ("random", True)):
        lib.hstu_debug_mfma_loop(rnd, iterations, sink)  # warm-up
        torch.cuda.synchronize()
        lib.hstu_debug_timing_begin(launches)
        flops = 0.0
        for _ in range(launches):
            flops = lib.hstu_debug_mfma_loop(rnd, iterations, sink)
        recs = lib.hstu_debug_timing_end(launches)
        ms = float(np.mean([m for k, m in recs if k == "mfma_loop"]))
        out[name] = flops / (ms * 1e-3) / 1e12
    return out


def _dq_atomic_rate(lib, dev, rows: int = 96016, heads: int = 8, blocks: int = 512, launches: int = 3):
    """GB/s of fp32 atomic adds in the pattern of a dq produced by the dk/dv pass."""
    buf = torch.zeros((rows, heads, 128), dtype=torch.float32, device=dev)
    out = {}
    for name, local in (("head_per_xcd", True), ("heads_mixed", False)):
        lib.hstu_debug_dq_atomic_rate(buf, blocks, local)
        torch.cuda.synchronize()
        lib.hstu_debug_timing_begin(launches)
        nbytes = 0.0
        for _ in range(launches):
            nbytes = lib.hstu_debug_dq_atomic_rate(buf, blocks, local)
        recs = lib.hstu_debug_timing_end(launches)
        ms = float(np.mean([m for k, m in recs if k == "dq_atomic"]))
        out[name] = nbytes / (ms * 1e-3) / 1e9
    return out


def _check_timed_outputs(w, vals_cpu, off, outs, rows_per_seq: int = 4):
    """Sampled rows of the outputs the timed steps left behind, against the oracle (exact rows:
    rows do not interact).  Part of the CPU leg, which is the one place bench.py uses the oracle."""
    import oracle
    rng = np.random.default_rng(5)
    sel = []
    for b, L in enumerate(w.lengths):
        if L > 0:
            sel += [int(off[b]), int(off[b]) + L - 1] + [int(off[b]) + int(x) for x in rng.integers(0, L, size=rows_per_seq)]
    sel = sorted(set(sel))
    f64 = {k: workloads.to_f64(v) for k, v in vals_cpu.items()}
    d_o = f64.get("d_o")
    if d_o is None:
        d_o = np.zeros_like(f64["v"])
    want = oracle.rows(f64["q"], f64["k"], f64["v"], d_o, off, w.max_len, w.alpha, True, sel)
    res, ok = {}, True
    for name, ref in zip(("o", "dq", "dk", "dv"), want):
        if name not in outs:
            continue
        g = outs[name][sel].double().cpu().numpy()
        rms = float(np.sqrt((ref ** 2).mean()))
        # bf16-stored outputs: the stated bar plus half a bf16 unit of the value itself
        bad = np.abs(g - ref) > 2e-2 * rms + np.abs(ref) * 2.0 ** -8
        res[name] = float(np.abs(g - ref).max() / rms)
        ok = ok and not bool(bad.any())
    return {"rows": len(sel), "max_abs_err_over_rms": res, "within_tolerance": ok}


def _cpu_baseline(w: workloads.Workload, prefix_rows: int):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample."""
    import oracle  # CPU-baseline leg only
    lengths = [min(l, prefix_rows) for l in w.lengths]
    sub = workloads.custom("sample", lengths, w.num_heads, w.d_qk, w.d_v, w.max_len, w.dtype,
                           w.scale, w.seed, w.backward)
    vals = workloads.values(sub)
    f64 = {k: workloads.to_f64(v) for k, v in vals.items()}
    off = sub.seq_offsets()
    t0 = time.perf_counter()
    oracle.fwd(f64["q"], f64["k"], f64["v"], off, sub.max_len, sub.alpha, True)
    fl = sub.flops()["fwd"]
    if w.backward:
        oracle.bwd(f64["q"], f64["k"], f64["v"], f64["d_o"], off, sub.max_len, sub.alpha, True)
        fl += sub.flops()["bwd"]
    dt = time.perf_counter() - t0
    return {
        "value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
        "sample": "first %d rows of each of the %d sequences, all %d heads, %s, %.1f s of oracle time"
                  % (prefix_rows, sub.batch, sub.num_heads, "fwd+bwd" if w.backward else "fwd", dt),
    }


def _parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg5", choices=["cfg2", "cfg3", "cfg4", "cfg4_ring", "cfg5", "cfg5_bias", "short", "mid"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--flags", type=int, default=0, help="hstu_flags passed with every call (A/B runs)")
    ap.add_argument("--probes", action="store_true", help="also print the measurement kernels' line")
    ap.add_argument("--cpu-prefix-rows", type=int, default=0, help="rows per sequence in the CPU sample")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="default workload only: leave out the short runs of cfg3 and cfg4 reported beside it")
    return ap.parse_args()


def measure(args):
    """One workload: the JSON line's dictionary, and what the probes line needs."""
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (run with --gpus 1)",
              file=sys.stderr)
        return None
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return None

    import paper_2508_04711_amd as lib
    lib.load_library()  # fail loudly if the HIP library is not built
    lib.binding.default_flags = args.flags

    ring = args.workload.endswith("_ring")
    with_bias = args.workload.endswith("_bias")  # the same batch with the timestamp bias
    if args.workload in ("short", "mid"):  # large batches of short sequences
        cfg = 0
        w = workloads.large_batch(args.workload)
    else:
        cfg = int(args.workload[3:4])
        w = workloads.config(cfg)
    dev = torch.device("cuda:0")
    vals_cpu = workloads.values(w)
    vals = {k: v.to(dev) for k, v in vals_cpu.items()}
    off_np = w.seq_offsets()
    off = torch.from_numpy(off_np).to(dev)
    T, H = w.total_rows, w.num_heads
    dt = workloads.torch_dtype(w)
    fl = w.flops()
    step_flops = fl["fwd"] + (fl["bwd"] if w.backward else 0.0)

    if w.cp_size:
        # Emulate every rank on the one GPU: rank r's query rows (mini-chunks r and 2CP-1-r of
        # every sequence, gathered beforehand) against all causally visible keys.
        cp = w.cp_size
        ranks = []
        for r in range(cp):
            n = 0
            for L in w.lengths:
                c = -(-L // (2 * cp))
                n += sum(min((m + 1) * c, L) - min(m * c, L) for m in (r, 2 * cp - 1 - r))
            ranks.append({
                "n": n,
                "q": torch.empty((n, H, w.d_qk), dtype=dt, device=dev),
                "d_o": torch.empty((n, H, w.d_v), dtype=dt, device=dev),
                "o": torch.empty((n, H, w.d_v), dtype=dt, device=dev),
                "dq": torch.empty((n, H, w.d_qk), dtype=dt, device=dev),
                "dk": torch.empty((T, H, w.d_qk), dtype=dt, device=dev),
                "dv": torch.empty((T, H, w.d_v), dtype=dt, device=dev),
            })
        o_glob = torch.empty((T, H, w.d_v), dtype=dt, device=dev)
        dq_glob = torch.empty((T, H, w.d_qk), dtype=dt, device=dev)
        ws = torch.empty(lib.hstu_jagged_attn_workspace_bytes(
            (w.batch, H, w.d_qk, w.d_v, w.max_len, w.alpha, True, 0, T), 2), dtype=torch.uint8, device=dev)

        if ring:
            # the ring variant: every rank's K/V part resident in its local layout (as on its own
            # GPU), fetched part by part on a second stream while the previous step computes;
            # o and dq accumulate in fp32 across the steps
            kparts, vparts = [], []
            for r, rk in enumerate(ranks):
                kl, vl = lib.hstu_cp_reorder([vals["k"], vals["v"]], off, T, cp, r, rk["n"])
                kparts.append(kl); vparts.append(vl)
            recv_rows = max(rk["n"] for rk in ranks)
            recv = [torch.empty((recv_rows, H, d), dtype=dt, device=dev) for d in (w.d_qk, w.d_qk, w.d_v, w.d_v)]
            for rk in ranks:
                rk["o32"] = torch.empty((rk["n"], H, w.d_v), dtype=torch.float32, device=dev)
                rk["dq32"] = torch.empty((rk["n"], H, w.d_qk), dtype=torch.float32, device=dev)
            dks = [torch.empty((rk["n"], H, w.d_qk), dtype=torch.float32, device=dev) for rk in ranks]
            dvs = [torch.empty((rk["n"], H, w.d_v), dtype=torch.float32, device=dev) for rk in ranks]
            o_glob = torch.empty((T, H, w.d_v), dtype=torch.float32, device=dev)
            dq_glob = torch.empty((T, H, w.d_qk), dtype=torch.float32, device=dev)
            copy_stream = torch.cuda.Stream(device=dev)

        def step_ring():
            for r, rk in enumerate(ranks):
                lib.hstu_cp_reorder([vals["q"], vals["d_o"]], off, T, cp, r, rk["n"],
                                    out=[rk["q"], rk["d_o"]])
                lib.hstu_cp_ring_pass(rk["q"], rk["d_o"], kparts, vparts, off, T, w.max_len, w.alpha, True,
                                      cp, r, out=(rk["o32"], rk["dq32"], dks, dvs), recv=recv,
                                      workspace=ws, copy_stream=copy_stream)
                lib.hstu_cp_reorder([rk["o32"], rk["dq32"]], off, T, cp, r, rk["n"], scatter=True,
                                    out=[o_glob, dq_glob])

        def step():
            if ring:
                return step_ring()
            # per rank: reorder kernel global -> local (q, d_o), the partial, local -> global (o, dq)
            for r, rk in enumerate(ranks):
                lib.hstu_cp_reorder([vals["q"], vals["d_o"]], off, T, cp, r, rk["n"],
                                    out=[rk["q"], rk["d_o"]])
                lib.hstu_jagged_attn_cp_partial(rk["q"], vals["k"], vals["v"], rk["d_o"], off, T,
                                                w.max_len, w.alpha, True, cp, r, -1,
                                                out=(rk["o"], rk["dq"], rk["dk"], rk["dv"]), workspace=ws)
                lib.hstu_cp_reorder([rk["o"], rk["dq"]], off, T, cp, r, rk["n"], scatter=True,
                                    out=[o_glob, dq_glob])
    else:
        o = torch.empty((T, H, w.d_v), dtype=dt, device=dev)
        dq = torch.empty((T, H, w.d_qk), dtype=dt, device=dev)
        dk = torch.empty_like(dq)
        dv = torch.empty_like(o)
        p = (w.batch, H, w.d_qk, w.d_v, w.max_len, w.alpha, True, 0, T)
        ws = torch.empty(max(lib.hstu_jagged_attn_workspace_bytes(p, 0),
                             lib.hstu_jagged_attn_workspace_bytes(p, 1)), dtype=torch.uint8, device=dev)

        if with_bias:
            # sorted event timestamps (see workloads.timestamps), 64 buckets, 4 groups per octave
            ts = torch.from_numpy(workloads.timestamps(w, "events", 0)).to(dev)
            tab = torch.from_numpy(workloads.bias_table(64, 0, 1.0)).to(dev)
            dtab = torch.empty_like(tab)
            ws = torch.empty(max(lib.hstu_jagged_attn_bias_workspace_bytes(p, 0),
                                 lib.hstu_jagged_attn_bias_workspace_bytes(p, 1)),
                             dtype=torch.uint8, device=dev)

        def step():
            if with_bias:
                lib.hstu_jagged_attn_bias_fwd(vals["q"], vals["k"], vals["v"], off, ts, tab, 2, w.max_len,
                                              w.alpha, True, out=o, workspace=ws)
                lib.hstu_jagged_attn_bias_bwd(vals["q"], vals["k"], vals["v"], vals["d_o"], off, ts, tab, 2,
                                              w.max_len, w.alpha, True, out=(dq, dk, dv, dtab), workspace=ws)
                return
            lib.hstu_jagged_attn_fwd(vals["q"], vals["k"], vals["v"], off, w.max_len, w.alpha, True,
                                     out=o, workspace=ws)
            if w.backward:
                lib.hstu_jagged_attn_bwd(vals["q"], vals["k"], vals["v"], vals["d_o"], off, w.max_len,
                                         w.alpha, True, out=(dq, dk, dv), workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    tflops = step_flops / (ms_per_step * 1e-3) / 1e12

    # Per-kernel durations over the same steps: HIP events recorded by the library on the
    # stream it launches on, one pair per kernel launch.
    prof_steps = max(1, min(args.steps, 10))
    nrec = 64 * prof_steps * max(1, w.cp_size) * (max(1, w.cp_size) if ring else 1)
    lib.hstu_debug_timing_begin(nrec)
    for _ in range(prof_steps):
        step()
    recs = lib.hstu_debug_timing_end(nrec)
    per_kind = {}
    for kind, ms in recs:
        per_kind.setdefault(kind, []).append(ms)
    launches_per_step = {k: len(v) // prof_steps for k, v in per_kind.items()}
    avg_ms = {k: float(np.mean(v)) for k, v in per_kind.items()}
    ms_by_kind_per_step = {k: avg_ms[k] * launches_per_step[k] for k in avg_ms}

    # Dominant kernel and its roofline.  Algorithmic flops per visible pair and head:
    # forward 2*d_qk + 2*d_v; dk/dv pass 4*d_qk + 4*d_v (S recompute, dP, dV, dK);
    # dq pass 2*d_qk (dS K; its own recomputation of S and dP is not counted).
    pairs = w.pairs_per_head * H
    alg = {"fwd": (2 * w.d_qk + 2 * w.d_v) * pairs, "dkdv": (4 * w.d_qk + 4 * w.d_v) * pairs,
           "dq": 2 * w.d_qk * pairs}
    hw = {"fwd": alg["fwd"], "dkdv": alg["dkdv"], "dq": (4 * w.d_qk + 2 * w.d_v) * pairs}
    dom = max((k for k in ms_by_kind_per_step if k in alg), key=lambda k: ms_by_kind_per_step[k])
    n_launch = launches_per_step[dom]
    dom_ms = avg_ms[dom]
    achieved = alg[dom] / n_launch / (dom_ms * 1e-3) / 1e12
    # (the dk/dv pass of the long-sequence workloads at d = 128 is the kernel with two waves per 32 keys)
    pair = (w.d_qk == 128 and w.d_v == 128 and not (args.flags & lib.HSTU_FLAG_DKDV_ONE_WAVE)
            and args.workload not in ("short", "mid", "cfg2"))
    kernel_name = {"fwd": "hstu_fwd_bf16", "dkdv": "hstu_dkdv_pair_bf16" if pair else "hstu_dkdv_bf16",
                   "dq": "hstu_dq_bf16"}[dom]
    # What this machine sustains on matrix instructions alone, measured now: the published peak
    # assumes a 2.4 GHz clock that the chip does not hold under matrix load (and holds less of on
    # random operands than on constant ones).
    measured = _measured_mfma_peak(lib, dev)
    roofline = {
        "bound": "mfma", "kernel": kernel_name, "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
        "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
        "measured_peak": measured["random"], "measured_peak_constant_operands": measured["constant"],
        "frac_of_measured_peak": achieved / measured["random"],
        "traffic": None if with_bias else _traffic_from_profiles(kernel_name, w.name),
        "avg_launch_ms": dom_ms, "launches_per_step": n_launch,
        "kernels": {k: {"avg_ms": avg_ms[k], "launches_per_step": launches_per_step[k],
                        "algorithmic_tflops": (alg[k] / launches_per_step[k] / (avg_ms[k] * 1e-3) / 1e12)
                        if k in alg else None,
                        "executed_tflops": (hw[k] / launches_per_step[k] / (avg_ms[k] * 1e-3) / 1e12)
                        if k in hw else None}
                    for k in avg_ms},
    }
    if "reorder" in avg_ms:
        # two tensors of H*d bf16 rows per launch, read once and written once
        moved = 2.0 * (T / w.cp_size) * H * (w.d_qk + w.d_v) * 2
        roofline["kernels"]["reorder"]["algorithmic_gbs"] = moved / (avg_ms["reorder"] * 1e-3) / 1e9
    # Algorithmic bytes per launch: every input row read once, every output row written once.
    row = 2.0 * T * H
    bytes_alg = {"fwd": row * (2 * w.d_qk + 2 * w.d_v), "dkdv": row * (3 * w.d_qk + 3 * w.d_v),
                 "dq": row * (3 * w.d_qk + 2 * w.d_v)}
    if not w.cp_size and alg[dom] / bytes_alg[dom] < PEAK_BF16_TFLOPS * 1e3 / PEAK_HBM_GBS:
        # below the ridge (flops per byte under peak flops / peak bandwidth): the dominant kernel
        # is reported against HBM bandwidth over its algorithmic bytes
        gbs = bytes_alg[dom] / (dom_ms * 1e-3) / 1e9
        roofline.update({"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                         "frac": gbs / PEAK_HBM_GBS, "frac_of_mfma_peak": achieved / PEAK_BF16_TFLOPS})
        roofline.pop("frac_of_measured_peak")
        if gbs / PEAK_HBM_GBS < 0.5 and achieved / PEAK_BF16_TFLOPS < 0.25:
            roofline["note"] = ("below the ridge, so reported against HBM, but bound by neither roofline: "
                                "%.0f %% of the HBM peak and %.0f %% of the matrix peak"
                                % (100 * gbs / PEAK_HBM_GBS, 100 * achieved / PEAK_BF16_TFLOPS))
        for k in roofline["kernels"]:
            if k in bytes_alg:
                roofline["kernels"][k]["algorithmic_gbs"] = bytes_alg[k] / (avg_ms[k] * 1e-3) / 1e9

    out = {
        "metric": "jagged HSTU attn fwd+bwd TFLOP/s (causal-visible, bf16)" if w.backward
                  else "jagged HSTU attn fwd TFLOP/s (causal-visible, bf16)",
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name + ("_ring" if ring else "") + ("_ts_bias" if with_bias else ""), "batch": w.batch, "total_rows": T, "num_heads": H,
                   "d_qk": w.d_qk, "d_v": w.d_v, "max_len": w.max_len, "causal": True,
                   "cp_size": w.cp_size, "pairs_per_head": w.pairs_per_head,
                   "flops_per_step": step_flops},
        "frac_of_bf16_mfma_peak": tflops / PEAK_BF16_TFLOPS,
        "frac_of_measured_mfma_peak": tflops / measured["random"],
        "roofline": roofline,
    }
    if not args.no_cpu_baseline:
        prefix = args.cpu_prefix_rows or {0: 300, 2: 1024, 3: 4096, 4: 4096, 5: 4096}[cfg]
        out["cpu_baseline"] = _cpu_baseline(w, prefix)
        if not w.cp_size and not with_bias:
            outs = {"o": o}
            if w.backward:
                outs.update({"dq": dq, "dk": dk, "dv": dv})
            out["cpu_baseline"]["timed_outputs_check"] = _check_timed_outputs(w, vals_cpu, off_np, outs)
    return out, measured, lib, dev


def main() -> int:
    args = _parse_args()
    res = measure(args)
    if res is None:
        return 2
    out, measured, lib, dev = res
    if args.workload == "cfg5" and not args.no_other_workloads:
        # The other long-sequence configurations in the same run, so that one line carries all three
        # fractions: the same steps and warm-up, no CPU leg.  (`value` above is cfg5's alone.)
        others = {}
        for name in ("cfg3", "cfg4"):
            a2 = argparse.Namespace(**vars(args))
            a2.workload, a2.no_cpu_baseline = name, True
            o2 = measure(a2)[0]
            r2 = o2["roofline"]
            others[o2["config"]["workload"]] = {
                "value": o2["value"], "unit": o2["unit"], "ms_per_step": o2["ms_per_step"],
                "frac_of_bf16_mfma_peak": o2["frac_of_bf16_mfma_peak"],
                "frac_of_measured_mfma_peak": o2["frac_of_measured_mfma_peak"],
                "roofline": {k: r2[k] for k in ("kernel", "achieved", "frac", "frac_of_measured_peak",
                                                "avg_launch_ms", "launches_per_step") if k in r2}}
        out["other_workloads"] = others
    print(json.dumps(out))
    if args.probes:
        print(json.dumps({"probes": {"mfma_loop_tflops": measured, "dq_atomic_gbs": _dq_atomic_rate(lib, dev)}}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
