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
# Plain (unpacked) fp32 VALU issue: 256 CUs x 64 lanes x 2.4 GHz; packed FP32 is off by
# build rule, so the 157.3 TFLOP/s figure (packed FMA) does not apply.  v_exp_f32 issues
# at half rate on this chip (measured), i.e. it takes two issue slots.
VALU_PEAK_LANE_OPS = 256 * 64 * 2.4e9
# Issue slots per state update of rowlane_fwd_kernel, from SQ_INSTS_VALU and
# SQ_INSTS_VALU_TRANS_F32 in profiles/lbscan_counters_vim_small.md (10.4 VALU instructions
# incl. 1.3 transcendental, which take two slots each).
FWD_SLOTS_PER_STATE_UPDATE = 11.7
FWD_VALU_PER_SU, FWD_TRANS_PER_SU = 9.1, 1.3
FWD_KEYS = ("x", "delta", "A", "Bm", "Cm", "Dskip", "z", "delta_bias")

# L2-to-fabric bytes per lbscan_fwd call from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE
# (KiB per dispatch, summed over the launches of one call), each scaled by what the
# same counter reads for a plain elementwise kernel that reads and writes 1 GiB
# (bench.py --copy-calibration: FETCH_SIZE x2.0, WRITE_SIZE x1.0); profiles/ has the runs.
MEASURED_TRAFFIC_BYTES = {
    "vim_tiny": int((42414.4 * 2.0 + 25978.7) * 1024),
    "vim_small": int((234641.4 * 2.0 + 97432.1) * 1024),
    # summary launch + carry chain + full pass
    "hires_4096": int(((128629.7 + 73254.8 + 2357.1) * 2.0 + 58316.8 + 3265.7 + 3072.0) * 1024),
    "wsi_bag": int(((116334.2 + 82034.2 + 12812.9) * 2.0 + 65552.7 + 3179.2 + 6014.8) * 1024),
}


def alu_bound(su_per_s, rates):
    """fp32 VALU issue bound of the forward kernel at its present instruction count:
    FWD_VALU_PER_SU plain instructions and FWD_TRANS_PER_SU transcendental ones per
    state update, priced at the nominal issue peak (transcendentals at half rate) or,
    with measured rates, at what the probe kernels reached on this machine."""
    if rates:
        t = FWD_VALU_PER_SU / rates["fma"] + FWD_TRANS_PER_SU / rates["exp2"]
        peak, how = 1.0 / t, "measured issue rates"
    else:
        peak, how = VALU_PEAK_LANE_OPS / FWD_SLOTS_PER_STATE_UPDATE, "nominal issue peak"
    return {"unit": "state updates/s", "achieved": su_per_s, "peak": peak, "frac": su_per_s / peak,
            "rates_lane_ops_per_s": rates,
            "note": f"fp32 VALU issue bound of the forward kernel at its present instruction count, {how}"}


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


def time_calls(calls, steps, warmup, per_launch=False):
    """Run `calls[i % len]()` warmup + steps times on the current stream.  Returns the
    average milliseconds per step from HIP events around the whole timed region and,
    with per_launch, also mean / median / min of per-launch durations from an event
    pair around every launch (without the gaps between dependent launches)."""
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
    region = e0.elapsed_time(e1) / steps
    if not per_launch:
        return region
    n = min(steps, 200)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
    for i in range(n):
        ev[i][0].record()
        calls[i % len(calls)]()
        ev[i][1].record()
    torch.cuda.synchronize()
    per = sorted(a.elapsed_time(b) for a, b in ev)
    return region, {"mean": sum(per) / n, "median": per[n // 2], "min": per[0]}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default="vim_tiny")
    ap.add_argument("--shape", default="", help="B,D,N,L,M[,dtype]: time a custom shape instead of a named workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-bwd", action="store_true", help="skip the backward-pass timing")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB elementwise copy kernel, for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE")
    ap.add_argument("--waves-log2", type=int, default=-1, help="force the state-split launch shape (tuning)")
    ap.add_argument("--segments", type=int, default=0, help="force the number of row segments (tuning)")
    ap.add_argument("--sets", type=int, default=0, help="independent input sets to rotate over (0: enough for 640 MB)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the scan needs no cross-GPU exchange in "
              "forward: rows shard over batch or channels); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2506_15976_amd as lb
    from paper_2506_15976_amd import binding
    from paper_2506_15976_amd.inputs import BASE_SEED, WORKLOADS, make_inputs, make_workload

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if a.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")      # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 1.0, out=dst)     # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
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

    ms_fwd, ms_kernel = time_calls(fwd_calls, a.steps, a.warmup, per_launch=True)
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
    ms_train = None
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
        # training step with the forward call saving checkpoints for the backward call
        sneed = lb.lbscan_workspace_bytes(fwd_args[0], binding.WS_SAVED)
        if sneed:
            saved = torch.empty(sneed // 4, dtype=torch.float32, device="cuda:0")

            def train_call(ar, dout, outs):
                ar.saved_state, ar.saved_state_bytes = saved.data_ptr(), sneed
                r1 = lib.lbscan_fwd(ctypes.byref(ar), stream)
                r2 = bwd_call(ar, dout, outs)
                ar.saved_state, ar.saved_state_bytes = None, 0
                return r1 or r2
        else:
            def train_call(ar, dout, outs):
                return lib.lbscan_fwd(ctypes.byref(ar), stream) or bwd_call(ar, dout, outs)
        assert train_call(*g_args[0]) == 0, "training step failed"
        ms_train = time_calls([(lambda g=g: train_call(*g)) for g in g_args], max(a.steps // 4, 1), max(a.warmup // 4, 1))

    # the block's pre-scan step (depthwise causal conv + SiLU, width 4) on the same x
    # tensors: an HBM-bound kernel of the same library, timed as extra information
    wconv = torch.randn(w["dim"], 4, device="cuda:0") * 0.5
    bconv = torch.randn(w["dim"], device="cuda:0")
    conv_sets = list(zip(sets, ys))[:max(2, min(nsets, 4))]
    conv_calls = [(lambda s_=s_, y_=y_: lb.lbscan_conv1d_fwd(s_["x"], wconv, bconv, out=y_)) for s_, y_ in conv_sets]
    ms_conv = time_calls(conv_calls, max(a.steps // 4, 1), max(a.warmup // 4, 1))
    conv_bytes = 2 * w["batch"] * w["dim"] * w["seqlen"] * (2 if w["dtype"] == "bf16" else 4)

    rates = None
    tokens = w["batch"] * w["seqlen"]
    # average launch duration over the timed region (includes the ~5 us gap between
    # dependent launches; an event pair per launch reads slightly more, a kernel trace less)
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
        t0 = time.perf_counter()
        oracle.fwd(**sub, window=w["window"])
        once = time.perf_counter() - t0
        reps = max(3, int(np.ceil(1.5 / max(once, 1e-4))))       # about 1.5 s of wall time on all cores
        t0 = time.perf_counter()
        for _ in range(reps):
            oracle.fwd(**sub, window=w["window"])
        per_call = (time.perf_counter() - t0) / reps
        # the same loop on one core, on a smaller slice
        threads = oracle.num_threads()
        nb1 = max(1, nb // 8)
        sub1 = {k: (v[:nb1] if isinstance(v, np.ndarray) and v.ndim == 3 else v) for k, v in host.items()}
        oracle.set_num_threads(1)
        t0 = time.perf_counter()
        oracle.fwd(**sub1, window=w["window"])
        one_core = time.perf_counter() - t0
        oracle.set_num_threads(threads)
        cpu = {"value": nb * w["seqlen"] / per_call, "unit": "tokens/s", "cores": threads,
               "kind": "oracle",
               "sample": f"fp64 oracle forward on {nb} of {w['batch']} batch entries of {a.workload}, "
                         f"mean of {reps} calls, {per_call:.4f} s per call",
               "one_core_value": nb1 * w["seqlen"] / one_core,
               "one_core_sample": f"{nb1} batch entries, one call, {one_core:.3f} s"}

    line = {
        "metric": "lbscan_fwd_tokens_per_s", "value": tokens / (ms_fwd * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_fwd,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{a.workload}: B={w['batch']} D={w['dim']} N={w['dstate']} L={w['seqlen']} "
                               f"M={w['window']} {w['dtype']} storage, forward", "input_sets_rotated": nsets},
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS, "traffic": traffic,
                     "kernel": "rowlane_fwd_kernel", "algorithmic_bytes_per_launch": fwd_bytes,
                     "launch_ms": ms_fwd, "launch_ms_event_pairs": ms_kernel["mean"],
                     "launch_ms_median": ms_kernel["median"], "launch_ms_min": ms_kernel["min"]},
        "alu_bound": alu_bound(tokens * w["dim"] * w["dstate"] / (ms_fwd * 1e-3), rates),
        "cpu_baseline": cpu,
        "speedup_vs_two_pass_bidir": ms_bidir / ms_fwd,
        "two_pass_bidir_ms": ms_bidir,
        "cache_hot_ms_per_step": ms_hot,
        "bwd_ms": ms_bwd,
        "fwd_plus_bwd_ms": ms_train,
        "bwd_algorithmic_gbps": None if ms_bwd is None else algorithmic_bytes(w, "bwd") / (ms_bwd * 1e-3) / 1e9,
        "prescan_conv_fwd_ms": ms_conv,
        "prescan_conv_fwd_gbps": conv_bytes / (ms_conv * 1e-3) / 1e9,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
