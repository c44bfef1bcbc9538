#!/usr/bin/env python3
"""Benchmark of the pipelined online learner on one MI355X.

A "step" is one stream tick: forward + delayed-error backward + SGD update of
ALL stages (one grouped kernel launch).  Default workload: the 8 x (4096x4096)
fp32 ReLU MLP, depth 8, MSE, lr 1e-4, smooth synthetic stream (workload 1 of
partime_streams).  Inputs are resident in HBM before the timed region.

Prints ONE JSON line with the metric (stream ticks/sec), the roofline of the
dominant kernel and the CPU oracle timed on a bounded sample of the same
workload.
"""
import argparse
import json
import numpy as np
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes_per_tick(w, learn=True):
    """Every weight read once per tick and, when learning, written once; vectors are negligible
    (a few hundred KB against hundreds of MB) and not counted."""
    esz = 4 if w.w_dtype == 0 else 2
    if learn and w.adam:
        # weights read + written, and both fp32 moments read + written
        return w.n_weights * (2 * esz + 4 * 4)
    if learn and w.balance:
        # a layer that is not the last of its stage is read by its forward pass and read + written by its backward
        # pass (its delta exists only after the layers behind it have run): 3 passes instead of 2
        n, i = 0, 0
        for cnt in w.balance:
            for j in range(cnt):
                n += int(np.prod(w.layers[i].w_shape)) * (2 if j == cnt - 1 else 3)
                i += 1
        return n * esz
    return w.n_weights * esz * (2 if learn else 1)


def batched_flops_per_tick(w, learn=True):
    """Multiply-adds x 2 of the three products of every stage under S streams (no backward product in the first stage)."""
    fl = 0
    for i, l in enumerate(w.layers):
        one = 2 * int(np.prod(l.w_shape)) * w.n_streams
        fl += one * ((3 if i > 0 else 2) if learn else 1)
    return fl


def conv_flops_per_tick(w, learn=True):
    """Multiply-adds x 2 of the conv stages: forward, backward-data (not for the first stage) and weight gradient."""
    fl = 0
    for i, l in enumerate(w.layers):
        if l.kind != 1:
            continue
        one = 2 * l.c_out * l.c_in * 9 * l.h * l.w
        fl += one * ((3 if i > 0 else 2) if learn else 1)
    return fl


def read_traffic(name, mode):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    import glob
    found = glob.glob(os.path.join(ROOT, "profiles", f"*_{name}_{mode}_pmc.txt"))
    if not found:
        return None
    path = found[0]
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


def read_mfma_util(name, mode):
    """Matrix-pipe busy fraction of the kernels of one tick (SQ_VALU_MFMA_BUSY_CYCLES over SIMD-cycles of the launch)
    from the committed rocprofv3 --pmc summary, if there is one."""
    import glob
    found = glob.glob(os.path.join(ROOT, "profiles", f"*_{name}_{mode}_mfma.txt"))
    if not found:
        return None
    m = re.search(r"^mfma_util:\s*([0-9.eE+-]+)", open(found[0]).read(), flags=re.M)
    return float(m.group(1)) if m else None


def cpu_baseline(w, Ws, bs, budget_s=15.0):
    """The oracle as it stands, on the host cores, on the first ticks of the same stream (the generators are seeded, so
    these are the ticks the GPU run started with); the sample is drawn here, whatever --steps and --warmup are."""
    import oracle
    import partime_streams as ps
    ref = oracle.Oracle(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, w_bf16=w.w_dtype == 1,
                        n_streams=w.n_streams, balance=w.balance, operands_bf16=w.n_streams > 1, adam=w.adam)
    threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    n0 = 2 if w.n_streams < 64 else 1      # a tick of a replay batch is tens of seconds of plain loops
    x, tg = ps.make_inputs(w, n0)
    t0 = time.perf_counter()
    ref.step(x[:1], tg[:1])                # the first tick also touches every page of the oracle's arrays
    per = time.perf_counter() - t0
    if n0 > 1 and per <= budget_s:
        t0 = time.perf_counter()
        ref.step(x[1:], tg[1:])
        per = (time.perf_counter() - t0) / (n0 - 1)
    if per > budget_s:
        # one tick is already the whole sample (fill ticks cost what every tick costs: nothing is skipped on zeros)
        return {"value": 1.0 / per, "unit": "ticks/s", "cores": threads, "kind": "oracle",
                "sample": f"tick 0 of the same stream (1 tick, {per:.1f} s)"}
    n = int(max(4 if per < budget_s / 4 else 1, min(2000, budget_s / max(per, 1e-6))))
    m = int(max(0, min(200, 3.0 / max(per * threads, 1e-6))))      # ticks of the one-thread leg (about 3 s, or none)
    if per * threads > 20.0:
        m = 0                                                       # the one-thread figure would take minutes
    x, tg = ps.make_inputs(w, n0 + n + m)
    t0 = time.perf_counter()
    ref.step(x[n0:n0 + n], tg[n0:n0 + n])
    dt = time.perf_counter() - t0
    rec = {"value": n / dt, "unit": "ticks/s", "cores": threads, "kind": "oracle",
           "sample": f"ticks {n0}..{n0 + n - 1} of the same stream ({n} ticks, {dt:.1f} s)"}
    if m >= 2:
        # the same oracle on one thread, on the next ticks of the stream (context for the figure above)
        try:
            import ctypes
            gomp = ctypes.CDLL("libgomp.so.1")
        except OSError:
            return rec
        gomp.omp_set_num_threads(1)
        try:
            t0 = time.perf_counter()
            ref.step(x[n0 + n:], tg[n0 + n:])
            rec["value_1_thread"] = m / (time.perf_counter() - t0)
            rec["sample_1_thread"] = f"ticks {n0 + n}..{n0 + n + m - 1} ({m} ticks)"
        finally:
            gomp.omp_set_num_threads(threads)
    return rec


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", type=int, default=1, help="index into partime_streams.workload (default 1)")
    ap.add_argument("--mode", choices=["learn", "infer"], default="learn")
    ap.add_argument("--exec", dest="exec_mode", choices=["auto", "per-tick", "persistent"], default="auto")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="first run a plain device copy of this many MiB five times (a known-size "
                         "reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (all pipeline stages share it); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import partime_streams as ps
    from paper_2210_09147_amd import Pipeline, binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    w = ps.workload(args.workload)
    K, Wm = args.steps, args.warmup
    T = K + Wm
    Ws, bs = ps.init_weights(w.layers, w.seed)
    x, tg = ps.make_inputs(w, T)
    learn = args.mode == "learn"

    p = Pipeline(w.layers, Ws, bs, loss=w.loss, lr=w.lr, target_delay=w.k, n_streams=w.n_streams, balance=w.balance, adam=w.adam,
                 w_dtype=w.w_dtype, exec_mode={"auto": 0, "per-tick": 1, "persistent": 2}[args.exec_mode])
    xd, td = torch.from_numpy(x).cuda(), torch.from_numpy(tg).cuda()
    out = torch.empty((T, w.n_streams, w.out_size), dtype=torch.float32, device="cuda")
    loss = torch.zeros((T,), dtype=torch.float32, device="cuda")

    def run(i, j):
        if learn:
            p.step(xd[i:j], td[i:j], out=out[i:j], loss=loss[i:j])
        else:
            p.infer(xd[i:j], out=out[i:j])

    if args.calib_copy_mib:
        src = torch.ones(args.calib_copy_mib * (1 << 20) // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if Wm:
        run(0, Wm)
    torch.cuda.synchronize()
    # HIP events on the stream the library launches on (torch's current stream was handed to it)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(p.stream)
    run(Wm, T)
    ev1.record(p.stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    dev_ms = ev0.elapsed_time(ev1)
    launches = B.partime_last_launch_count(p.ctx)
    # the paper's streaming call: one partime_step per tick, host launch included (same state, ticks re-used)
    ns = min(200, K)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for i in range(ns):
        run(Wm + i, Wm + i + 1)
    torch.cuda.synchronize()
    streaming = ns / (time.perf_counter() - t1)
    ms_per_tick = wall * 1e3 / K
    kern_ms = dev_ms / K          # device time per tick-kernel launch (back-to-back launches)
    abytes = algorithmic_bytes_per_tick(w, learn)
    achieved = abytes / (kern_ms * 1e-3) / 1e9
    final_loss = float(loss[T - 50:T].mean().item()) if learn else None
    assert bool(torch.isfinite(out[T - 1]).all())

    is_conv = w.layers[0].kind == 1
    if w.n_streams >= 64:
        kernel_name = "rb_gemm_kernel (forward, backward, update) + rb_input / rb_head / rb_bias kernels (one tick)"
    elif w.n_streams > 1:
        kernel_name = "ms_vec_kernel + ms_mat_kernel (one tick)" if learn else "ms_infer_kernel"
    elif is_conv:
        kernel_name = "cv_conv_kernel (forward, backward-data) + cv_wgrad_kernel + cv_update_kernel (one tick)"
    else:
        kernel_name = "tick_kernel"
    rec = {
        "metric": "stream ticks/sec (fwd+bwd+SGD, all stages)" if learn else "stream ticks/sec (inference only, all stages)",
        "value": K / wall, "unit": "ticks/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_tick, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if w.w_dtype == 0 else "bf16 weights, f32 arithmetic", "data": "synthetic",
        "config": {"workload": w.name, "depth": w.depth, "n_streams": w.n_streams, "mode": args.mode, "exec": args.exec_mode,
                   "lr": w.lr, "target_delay": w.k, "launches": launches,
                   "streaming_ticks_per_s_one_call_per_tick": streaming,
                   "mean_loss_last_50_ticks": final_loss},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": read_traffic(w.name, args.mode),
                     "kernel": kernel_name, "algorithmic_bytes_per_launch": abytes,
                     "avg_launch_ms": kern_ms},
    }
    if is_conv:
        fl = conv_flops_per_tick(w, learn)
        tf = fl / (kern_ms * 1e-3) / 1e12
        rec["roofline"] = {"bound": "mfma", "achieved": tf, "peak": 157.3, "unit": "TFLOP/s", "frac": tf / 157.3,
                           "traffic": None, "kernel": kernel_name, "flops_per_tick": fl, "avg_launch_ms": kern_ms}
    is_batched = w.n_streams >= 64
    if is_batched:
        # the three products per stage are real matrix products: report against whichever limit binds, the bf16
        # matrix cores (2.5 PFLOP/s) or HBM (weights, and with Adam the moments, move once per tick)
        fl = batched_flops_per_tick(w, learn)
        rec["roofline"]["flops_per_tick"] = fl
        rec["roofline"]["tflops"] = fl / (kern_ms * 1e-3) / 1e12
        if fl / 2.5e15 > abytes / (HBM_PEAK_GBS * 1e9):
            tf = rec["roofline"]["tflops"]
            rec["roofline"].update({"bound": "mfma", "achieved": tf, "peak": 2500.0, "unit": "TFLOP/s", "frac": tf / 2500.0})
    if is_conv or w.n_streams > 1:
        rec["roofline"]["mfma_util"] = read_mfma_util(w.name, args.mode)     # counted, not derived from flops / time
    p.close()
    del xd, td, out
    if not is_conv and not is_batched:
        # a reference rate, not a ceiling: what a kernel with no arithmetic reaches streaming a buffer of the same size
        # as the weights (in place read + write when learning, read only for inference) in a plain grid-stride loop
        nbytes = max(1 << 20, abytes // (2 if learn else 1))
        ref_gbs = B.partime_bandwidth_probe(nbytes, 2 if learn else 0, 20)
        rec["roofline"]["plain_stream_gbs"] = ref_gbs
        rec["roofline"]["vs_plain_stream"] = achieved / ref_gbs
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(w, Ws, bs)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
