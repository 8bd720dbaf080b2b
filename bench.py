#!/usr/bin/env python3
"""Benchmark of the locally bi-directional selective scan on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]

A step is one lbscan_fwd call over one batch of synthetic input (the
Vim-tiny-shaped workload by default).  Inputs are resident in HBM before the
timed region; launches rotate over several independent input sets so that the
256 MB Infinity Cache cannot serve them.  One JSON line is printed:
tokens/s of the locally bi-directional scan, the HBM roofline of its kernel,
the speed-up over the two-pass global bi-directional scan on the same inputs,
and the fp64 CPU oracle timed on the host cores as a reported baseline.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published
FWD_KEYS = ("x", "delta", "A", "Bm", "Cm", "Dskip", "z", "delta_bias")

# HBM bytes per lbscan_fwd launch from rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE,
# scaled by the copy-kernel calibration); see profiles/.  None until measured.
MEASURED_TRAFFIC_BYTES = {}


def algorithmic_bytes(w, which="fwd"):
    """Bytes one call must move: x, delta, z read + y written over (B,D,L), Bm and
    Cm read over (B,N,L), plus the small per-channel parameters."""
    e = 4 if w["dtype"] == "fp32" else 2
    bdl = w["batch"] * w["dim"] * w["seqlen"]
    bnl = w["batch"] * w["dstate"] * w["seqlen"]
    par = w["dim"] * (w["dstate"] + 2) * 4
    if which == "fwd":
        return 4 * bdl * e + 2 * bnl * e + par
    if which == "bwd":     # x, delta, z, dout read; dx, ddelta, dz written; Bm, Cm read; dBm, dCm written
        return 7 * bdl * e + 4 * bnl * e + 2 * par
    if which == "bidir":   # pass 1: x, delta read, partial written; pass 2: x, delta, z, partial read, y written
        return (3 + 5) * bdl * e + 4 * bnl * e + 2 * par
    raise ValueError(which)


def upload(s, dtype):
    import numpy as np
    import torch
    from paper_2506_15976_amd.inputs import fp32_to_bf16_bits
    out = {}
    for k in FWD_KEYS:
        v = s.get(k)
        if v is None:
            out[k] = None
        elif dtype == "bf16" and v.ndim == 3:
            out[k] = torch.from_numpy(fp32_to_bf16_bits(v).view(np.int16)).view(torch.bfloat16).to("cuda:0")
        else:
            out[k] = torch.from_numpy(v).to("cuda:0")
    return out


def time_calls(calls, steps, warmup):
    """Run `calls[i % len]()` warmup + steps times on the current stream; return
    average milliseconds per step from HIP events around the timed region."""
    import torch
    for i in range(warmup):
        calls[i % len(calls)]()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(steps):
        calls[i % len(calls)]()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="vim_tiny")
    ap.add_argument("--shape", default="", help="B,D,N,L,M[,dtype]: time a custom shape instead of a named workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bwd", action="store_true", help="skip the backward-pass timing")
    ap.add_argument("--waves-log2", type=int, default=-1, help="force the state-split launch shape (tuning)")
    ap.add_argument("--segments", type=int, default=0, help="force the number of row segments (tuning)")
    ap.add_argument("--sets", type=int, default=0, help="independent input sets to rotate over (0: enough for 640 MB)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the scan needs no cross-GPU exchange in "
              "forward; see DESIGN.md for how it would shard); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2506_15976_amd as lb
    from paper_2506_15976_amd import binding
    from paper_2506_15976_amd.inputs import BASE_SEED, WORKLOADS, make_inputs, make_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    lib = lb.load()
    lb.lbscan_set_option("waves_log2", a.waves_log2)
    lb.lbscan_set_option("segments", a.segments)
    if a.shape:
        f = a.shape.split(",")
        w = dict(batch=int(f[0]), dim=int(f[1]), dstate=int(f[2]), seqlen=int(f[3]), window=int(f[4]),
                 dtype=f[5] if len(f) > 5 else "fp32", grad=False, idx=99)
        a.workload = "custom"
    else:
        w = WORKLOADS[a.workload]
    fwd_bytes = algorithmic_bytes(w, "fwd")
    nsets = a.sets or max(2, int(np.ceil(640e6 / fwd_bytes)))
    nsets = min(nsets, 16)

    # independent input sets (same distribution, different seeds); set 0 is the named workload
    sets, sets_b = [], []
    host0 = (make_workload(a.workload) if not a.shape else
             make_inputs(w["batch"], w["dim"], w["dstate"], w["seqlen"], seed=BASE_SEED + 99, dtype=w["dtype"]))
    for i in range(nsets):
        s = host0 if i == 0 else make_inputs(w["batch"], w["dim"], w["dstate"], w["seqlen"],
                                             seed=BASE_SEED + 100 * (i + 1) + w["idx"], dtype=w["dtype"])
        sets.append(upload(s, w["dtype"]))
    # second parameter set for the reverse direction of the two-pass comparison: the
    # (B,D,L)/(B,N,L) tensors of another rotation slot, so both passes read distinct memory
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    ys = [torch.empty_like(s["x"]) for s in sets]
    fwd_args = [lb.make_args(**s, window=w["window"], y=y) for s, y in zip(sets, ys)]
    need = lb.lbscan_workspace_bytes(fwd_args[0], binding.WS_FWD)
    ws_fwd = torch.empty(max(need // 4, 1), dtype=torch.float32, device="cuda:0")
    for ar in fwd_args:
        ar.workspace, ar.workspace_bytes = ws_fwd.data_ptr(), need
    fwd_calls = [(lambda ar=ar: lib.lbscan_fwd(ctypes.byref(ar), stream)) for ar in fwd_args]
    rc = fwd_calls[0]()
    assert rc == 0, f"lbscan_fwd failed: {rc}"

    ms_fwd = time_calls(fwd_calls, a.steps, a.warmup)
    ms_hot = time_calls(fwd_calls[:1], a.steps, a.warmup)

    # two-pass global bi-directional scan on the same inputs (direction b = next slot)
    bi_f = [lb.make_args(**s, window=1, y=y) for s, y in zip(sets, ys)]
    bi_b = [lb.make_args(**sets[(i + 1) % nsets], window=1) for i in range(nsets)]
    need = lb.lbscan_workspace_bytes(bi_f[0], binding.WS_BIDIR)
    ws = torch.empty(max(need // 4, 1), dtype=torch.float32, device="cuda:0")
    for ar in bi_f:
        ar.workspace, ar.workspace_bytes = ws.data_ptr(), need
    bi_calls = [(lambda f=f, b=b: lib.lbscan_bidir_fwd(ctypes.byref(f), ctypes.byref(b), stream))
                for f, b in zip(bi_f, bi_b)]
    rc = bi_calls[0]()
    assert rc == 0, f"lbscan_bidir_fwd failed: {rc}"
    ms_bidir = time_calls(bi_calls, max(a.steps // 2, 1), max(a.warmup // 2, 1))

    # backward pass (training shapes; timed for every workload as extra information)
    ms_bwd = None
    if not a.no_bwd:
        import torch
        g_args, keep = [], []
        for s_, ar in zip(sets, fwd_args):
            dout = torch.randn_like(s_["x"])
            outs = [torch.empty_like(s_["x"]) for _ in range(3)] + [torch.empty_like(s_["Bm"]) for _ in range(2)] + \
                   [torch.empty_like(s_["A"]), torch.empty_like(s_["Dskip"]), torch.empty_like(s_["delta_bias"])]
            keep.append((dout, outs))
            g_args.append((ar, dout, outs))
            if len(g_args) == 2:
                break                    # two sets are enough to defeat the cache for these sizes
        need = lb.lbscan_workspace_bytes(fwd_args[0], binding.WS_BWD)
        ws_bwd = torch.empty(max(need // 4, 1), dtype=torch.float32, device="cuda:0")

        def bwd_call(ar, dout, outs):
            ar.workspace, ar.workspace_bytes = ws_bwd.data_ptr(), need
            rc_ = lib.lbscan_bwd(ctypes.byref(ar), dout.data_ptr(), *[o.data_ptr() for o in outs], stream)
            ar.workspace, ar.workspace_bytes = ws_fwd.data_ptr(), ws_fwd.numel() * 4
            return rc_
        assert bwd_call(*g_args[0]) == 0, "lbscan_bwd failed"
        ms_bwd = time_calls([(lambda g=g: bwd_call(*g)) for g in g_args], max(a.steps // 4, 1), max(a.warmup // 4, 1))

    tokens = w["batch"] * w["seqlen"]
    gbps = fwd_bytes / (ms_fwd * 1e-3) / 1e9
    traffic = MEASURED_TRAFFIC_BYTES.get(a.workload)

    cpu = None
    if not a.no_cpu_baseline:
        import oracle
        host = {k: host0.get(k) for k in FWD_KEYS}
        # bounded sample: whole batch entries of the same workload, sized for ~2e8 state updates
        su_per_b = w["dim"] * w["dstate"] * w["seqlen"]
        nb = max(1, min(w["batch"], int(2e8 // su_per_b)))
        sub = {k: (v[:nb] if isinstance(v, np.ndarray) and v.ndim == 3 else v) for k, v in host.items()}
        oracle.fwd(**{k: (v[:1] if isinstance(v, np.ndarray) and v.ndim == 3 else v) for k, v in host.items()},
                   window=w["window"])
        best = 1e30
        for _ in range(3):
            t0 = time.perf_counter()
            oracle.fwd(**sub, window=w["window"])
            best = min(best, time.perf_counter() - t0)
        cpu = {"value": nb * w["seqlen"] / best, "unit": "tokens/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"fp64 oracle forward on {nb} of {w['batch']} batch entries of {a.workload}, best of 3, "
                         f"{best:.3f} s"}

    line = {
        "metric": "lbscan_fwd_tokens_per_s", "value": tokens / (ms_fwd * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_fwd,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{a.workload}: B={w['batch']} D={w['dim']} N={w['dstate']} L={w['seqlen']} "
                               f"M={w['window']} {w['dtype']} storage, forward", "input_sets_rotated": nsets},
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "rowlane_fwd_kernel", "algorithmic_bytes_per_launch": fwd_bytes},
        "cpu_baseline": cpu,
        "speedup_vs_two_pass_bidir": ms_bidir / ms_fwd,
        "two_pass_bidir_ms": ms_bidir,
        "cache_hot_ms_per_step": ms_hot,
        "bwd_ms": ms_bwd,
        "bwd_algorithmic_gbps": None if ms_bwd is None else algorithmic_bytes(w, "bwd") / (ms_bwd * 1e-3) / 1e9,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
