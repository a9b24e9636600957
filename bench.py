#!/usr/bin/env python3
"""Benchmark of the 1-bit LAMB compression-stage optimizer step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input already resident in
HBM: compress_local -> (gather copy) -> server_reduce -> ratios_apply (= layer_ratios + decompress_apply).
Prints ONE JSON line: the metric, the dominant kernel's roofline from HIP-event timings of its
launches, per-call and per-kernel times, and the CPU oracle timed beside it.  `--gpus N` with N > 1 is refused: this
build measures one GPU's share of the data-parallel step and uses no collectives.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

# Algorithmic HBM bytes per element of one launch of each kernel (every input read once, every
# output written once), by momentum representation.  Units per launch: n_pad for the N-sized
# kernels, n_c for the server ones.
KERNEL_BYTES = {
    "dense": {   # momentum read and written as an fp32 array
        "compress_resident": (16.125, "n_pad"),  # R g, m, err (12) + W err (4) + W bits (1/8)
        "momentum_z_sumsq": (16.0, "n_pad"),     # R g, m, err (12) + W z (4)
        "ratios_pass": (16.125, "n_pad"),        # R bits, m, v_fresh, v_frozen (12.125) + W v_fresh (4)
        "decompress_apply": (16.125, "n_pad"),   # R bits, v_frozen, x (8.125) + W x, m (8)
        "ratios_apply_resident": (28.125, "fused"),  # R bits, m, v_fresh, v_frozen, x (16.125) + W v_fresh, x, m (12)
    },
    "packed": {  # momentum read from last step's sign words, never written as fp32
        "compress_resident": (12.25, "n_pad"),   # R g, err (8) + m bits (1/8) + W err (4) + bits (1/8)
        "momentum_z_sumsq": (12.125, "n_pad"),
        "ratios_pass": (12.25, "n_pad"),         # R bits, m bits (1/4), v_fresh, v_frozen (8) + W v_fresh (4)
        "decompress_apply": (12.125, "n_pad"),   # R bits, v_frozen, x (8.125) + W x (4)
        "ratios_apply_resident": (20.25, "fused"),   # R bits x2, v_fresh, v_frozen, x (12.25) + W v_fresh, x (8)
    },
    "both": {
        "sign_pack_error": (8.125, "n_pad"),     # R z (4) + W err (4) + W bits (1/8)
        "server_unpack_avg": (None, "n_c"),      # W/8 + 8, filled in below
        "server_resident": (None, "n_c"),        # W/8 + 8.125, filled in below
        "server_sign_pack": (8.125, "n_c"),
        "warmup_moments": (24.0, "n_pad"),       # R g, m, v, x (16) + W m, v (8)
        "warmup_apply": (16.0, "n_pad"),         # R m, v, x (12) + W x (4)
        "warmup_resident": (28.0, "wfused"),     # R g, m, v, x (16) + W m, v, x (12)
    },
}


def compulsory_step_bytes_per_param(W):
    """The step's compulsory bytes with an fp32 momentum array (the accounting this build was
    specified against): compress_local 16.125 + server_reduce (0.125 + 8.125/W) + layer_ratios
    16.125 + decompress_apply 12.0."""
    return 16.125 + 0.125 + 8.125 / W + 16.125 + 12.0


def algorithmic_step_bytes_per_param(W, mode, fused_frac=0.0):
    """What the N-sized calls as implemented must move (each call's inputs once, outputs once),
    plus the server call.  fused_frac: share of the parameters whose ratio pass and update run as
    one kernel (ob_lamb_ratios_apply), reading v_frozen and the sign words once."""
    k = KERNEL_BYTES[mode]
    separate = k["ratios_pass"][0] + k["decompress_apply"][0]
    return (k["compress_resident"][0] + fused_frac * k["ratios_apply_resident"][0]
            + (1.0 - fused_frac) * separate + 0.125 + 8.125 / W)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="bert_large")
    ap.add_argument("--profile-steps", type=int, default=5)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy 10 times (for scaling rocprofv3 "
                         "FETCH_SIZE/WRITE_SIZE readings) and exit")
    ap.add_argument("--mom-scale", action="store_true", help="with Appendix A.5.2 momentum scaling")
    ap.add_argument("--separate-calls", action="store_true",
                    help="ob_lamb_layer_ratios + ob_lamb_decompress_apply instead of the fused "
                         "ob_lamb_ratios_apply")
    ap.add_argument("--grad-dtype", choices=["f32", "f16", "bf16"], default="f32",
                    help="mixed-precision variant: the gradient arrives in 16 bits (2 bytes/param less)")
    ap.add_argument("--x-lp", choices=["none", "f16", "bf16"], default="none",
                    help="mixed-precision variant: also write a 16-bit copy of the parameters "
                         "(2 bytes/param more)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a HIP graph that holds two consecutive steps (for launch-bound "
                         "sizes; --steps must be even)")
    ap.add_argument("--dense-momentum", action="store_true",
                    help="keep the momentum as an fp32 array (default: the 1-bit form it has after "
                         "Algorithm 1 line 13; same results, 12 bytes/param less traffic)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures ONE GPU's share of the data-parallel step (no "
              "collectives, no second GPU); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.calibrate_copy:
        n = 1 << 28  # 2^28 fp32 = 1 GiB read + 1 GiB written per copy
        a = torch.ones(n, device=dev); b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(10):
            b.copy_(a)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read": 4 * n, "bytes_written": 4 * n,
                          "launches": 10}))
        return

    import paper_2104_06069_amd as ob
    from paper_2104_06069_amd.step import DeviceStep
    from workloads import (Streams, foreign_server_chunks, foreign_worker_chunks, gradient,
                           init_state, make_config)

    cfg = make_config(args.workload)
    pl, W = cfg["plist"], cfg["W"]
    hyper = dict(beta1=0.9, beta2=0.999, beta3=0.9, eta=1e-6, c_min=0.01, c_max=0.3, r_min=0.5,
                 r_max=4.0, r_threshold=0.1, weight_decay=0.0)
    server_chunk = W // 2
    st = Streams(0, device="cuda:0")
    mom_scale = st.uniform_host("mom_scale", 0, pl.L, 0.25, 4.0) if args.mom_scale else None
    mode = "dense" if args.dense_momentum else "packed"
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "none": None}
    ds = DeviceStep(pl.offsets, W, server_chunk, device="cuda:0", mom_scale=mom_scale,
                    packed_momentum=(mode == "packed"), fused_apply=not args.separate_calls,
                    x_lp_dtype=tdt[args.x_lp], **hyper)
    ds.load_state(init_state(st, cfg))
    n_grads = 3
    grads = [gradient(st, cfg, t).to(tdt[args.grad_dtype]) for t in range(n_grads)]
    lp_variant = args.grad_dtype != "f32" or args.x_lp != "none"
    if lp_variant and not args.no_cpu_baseline:
        print("bench.py: the CPU-baseline leg covers the fp32 entry points; add --no-cpu-baseline "
              "to time the mixed-precision variant", file=sys.stderr)
        sys.exit(2)
    fw, fs = foreign_worker_chunks(st, cfg, 0)
    ds.packed_in.copy_(fw); ds.scales_in.copy_(torch.from_numpy(fs))
    for i in range(len(ds._pa)):   # what the other ranks' servers send, for both buffer pairs
        fa, fss = foreign_server_chunks(st, cfg, i)
        ds._pa[i].copy_(fa); ds._ss[i].copy_(torch.from_numpy(fss))
    lr = 1e-3
    torch.cuda.synchronize()

    def one_step(t):
        ds.begin_step()
        ds.step(grads[t % n_grads], lr)

    host0 = None
    if not args.no_cpu_baseline:
        # host copy of the initial state and inputs for the CPU-baseline leg, taken before any step
        host0 = dict(state={k: ds.get(k).copy() for k in
                            ("x", "m", "v_fresh", "v_frozen", "err_worker", "err_server", "c_avg", "r_prev")},
                     grads=[g.cpu().numpy() for g in grads[:2]],
                     fw=ds.packed_in.cpu().numpy(), fs=fs.copy(), fa=ds._pa[0].cpu().numpy(),
                     fss=ds._ss[0].cpu().numpy())

    for t in range(args.warmup + (args.warmup % 2 if args.graph else 0)):
        one_step(t)
    torch.cuda.synchronize()
    if args.graph:
        # two steps return the alternating buffer pairs to where they started: one graph, replayed
        assert args.steps % 2 == 0, "--graph replays pairs of steps"
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                one_step(0); one_step(1)
        torch.cuda.current_stream().wait_stream(side)
        graph.replay(); torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps // 2):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        t0 = time.perf_counter()
        for t in range(args.steps):
            one_step(t)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    # per-call times (events on the launch stream) and per-kernel durations (library's own events)
    calls = {}
    tail = ([("ratios_apply", lambda: ds.ratios_apply(lr))] if ds.fused_apply else
            [("layer_ratios", ds.layer_ratios), ("decompress_apply", lambda: ds.decompress_apply(lr))])
    evs = []
    for t in range(args.profile_steps):
        ds.begin_step()
        seq = [("compress_local", lambda: ds.compress_local(grads[t % n_grads])), ("gather", ds.gather),
               ("server_reduce", ds.server_reduce)] + tail
        e = [torch.cuda.Event(enable_timing=True) for _ in range(len(seq) + 1)]
        for i, (_, fn) in enumerate(seq):
            e[i].record(); fn()
        e[len(seq)].record()
        evs.append(e)
    torch.cuda.synchronize()
    for i, (nm, _) in enumerate(seq):
        calls[nm] = round(float(np.mean([e[i].elapsed_time(e[i + 1]) for e in evs])), 4)

    ob.ob_lamb_profile_enable(ds.ctx, True)
    for t in range(args.profile_steps):
        one_step(t)
    prof = ob.ob_lamb_profile_read(ds.ctx)
    ob.ob_lamb_profile_enable(ds.ctx, False)
    kern = {k: {"avg_ms": round(v[0] / v[1], 4), "launches": v[1]} for k, v in prof.items()}
    KB = dict(KERNEL_BYTES["both"])
    KB.update(KERNEL_BYTES[mode])
    KB["server_unpack_avg"] = (W / 8.0 + 8.0, "n_c")
    KB["server_resident"] = (W / 8.0 + 8.125, "n_c")   # R W*bits, err (4) + W err (4), bits (1/8)
    g_less = 2.0 if args.grad_dtype != "f32" else 0.0     # 16-bit gradient read
    x_more = 2.0 if args.x_lp != "none" else 0.0          # 16-bit parameter copy written
    for k in ("compress_resident", "momentum_z_sumsq", "warmup_moments", "warmup_resident"):
        KB[k] = (KB[k][0] - g_less, KB[k][1])
    for k in ("decompress_apply", "ratios_apply_resident", "warmup_apply", "warmup_resident"):
        KB[k] = (KB[k][0] + x_more, KB[k][1])
    fused_params = ob.ob_lamb_fused_params(ds.ctx) if ds.fused_apply else 0
    wfused = ob.ob_lamb_warmup_fused_params(ds.ctx)
    units = {"n_pad": ds.n_pad, "n_c": ds.n_c, "fused": fused_params, "wfused": wfused}
    if wfused:   # the two-pass warmup kernels then cover only the remaining layers (two launches each)
        for k in ("warmup_moments", "warmup_apply"):
            KB[k] = (KB[k][0], "rest_w")
        units["rest_w"] = ds.n_pad - wfused
    if ds.fused_apply:   # the plain ratio/update kernels then cover only the remaining layers
        for k in ("ratios_pass", "decompress_apply"):
            KB[k] = (KB[k][0], "rest")
        units["rest"] = ds.n_pad - fused_params
    for k, v in kern.items():
        if k in KB:
            bpe, unit = KB[k]
            # "rest" is covered by two launches per call (tiles on the boundaries of the fused
            # layers, then the remaining layers): per-launch mean
            per_call = max(1, round(v["launches"] / args.profile_steps)) if unit in ("rest", "rest_w") else 1
            v["algo_bytes"] = bpe * units[unit] / per_call
            v["GBps"] = round(v["algo_bytes"] / (v["avg_ms"] * 1e-3) / 1e9, 1)
    dom = max((k for k in kern if "GBps" in kern[k]), key=lambda k: kern[k]["avg_ms"] * kern[k]["launches"])
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            key = f"{args.workload}:{mode}:{'fused' if ds.fused_apply else 'separate'}"
            if lp_variant:
                key += f":g{args.grad_dtype}:x{args.x_lp}"
            traffic = json.load(open(tpath)).get(key, {}).get(dom)
        except Exception:
            traffic = None
    roofline = {"bound": "hbm", "kernel": dom, "achieved": kern[dom]["GBps"], "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(kern[dom]["GBps"] / HBM_PEAK_GBS, 4),
                "avg_launch_ms": kern[dom]["avg_ms"], "algo_bytes_per_launch": kern[dom]["algo_bytes"],
                "traffic": traffic}

    step_bytes = compulsory_step_bytes_per_param(W) * ds.n_pad
    algo_bytes = (algorithmic_step_bytes_per_param(W, mode, fused_params / float(ds.n_pad))
                  - g_less + x_more) * ds.n_pad
    out = {
        "metric": "1-bit LAMB compressed step: params/sec and % of HBM peak GB/s, 1 GPU",
        "value": round(pl.N / (ms_per_step * 1e-3), 1), "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}_shaped_W{W}", "N": pl.N, "N_pad": ds.n_pad, "L": pl.L,
                   "W": W, "n_c": ds.n_c, "server_chunk": server_chunk,
                   "mom_scale": bool(args.mom_scale), "momentum": mode,
                   "grad_dtype": args.grad_dtype, "x_lp": args.x_lp, "graph_replay": bool(args.graph),
                   "fused_ratios_apply": ds.fused_apply, "fused_layers": ob.ob_lamb_fused_layers(ds.ctx),
                   "fused_params": fused_params,
                   "single_pass_compress": ob.ob_lamb_uses_single_pass(ds.ctx)},
        "step_algorithmic_bytes": algo_bytes,
        "step_algorithmic_GBps": round(algo_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_algorithmic_pct_of_hbm_peak": round(100 * algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "step_compulsory_bytes": step_bytes,
        "step_compulsory_GBps": round(step_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_pct_of_hbm_peak": round(100 * step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "roofline": roofline,
        "calls_ms": calls,
        "kernels": kern,
    }

    ob.ob_lamb_check_device_status(ds.ctx, ds.stream)  # raises if a bounded device wait expired

    # reference timings outside the headline metric: one uncompressed LAMB warmup step (eq. (1)) and
    # the end-of-warmup momentum-scale generation (Appendix A.5.2), on the same buffers
    def timed(fn, reps=5):
        fn(); torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    ds.m_is_packed = False
    wu_ms = timed(lambda: ds.warmup_step(grads[0], lr))
    ms_ms = timed(lambda: ds.momentum_scale())
    out["reference_calls"] = {
        "warmup_step_ms": round(wu_ms, 4),
        # 28 B/elem where g, m, v, x are read once, 24 + 16 in the two-pass form
        "warmup_step_GBps": round(((28.0 - g_less + x_more) * wfused + (40.0 - g_less + x_more) * (ds.n_pad - wfused))
                                  / (wu_ms * 1e-3) / 1e9, 1),
        "warmup_single_pass_params": wfused,
        "warmup_step_params_per_s": round(pl.N / (wu_ms * 1e-3), 1),
        "momentum_scale_ms": round(ms_ms, 4),
        "momentum_scale_GBps": round(4.0 * ds.n_pad / (ms_ms * 1e-3) / 1e9, 1)}
    if host0 is not None:
        out["cpu_baseline"] = cpu_baseline(cfg, server_chunk, hyper, mom_scale, host0, lr,
                                           args.cpu_seconds)
    ds.close()
    print(json.dumps(out))


def cpu_baseline(cfg, server_chunk, hyper, mom_scale, h, lr, budget_s):
    """The oracle as it stands, single thread, on the same workload: whole steps until `budget_s`
    seconds of CPU work have been spent (at least one step, at most three)."""
    import numpy as np
    from tests.refstep import RefStep
    ref = RefStep(cfg["plist"].offsets, cfg["W"], server_chunk, mom_scale=mom_scale, **hyper)
    ref.load_state(h["state"])
    ref.set_foreign_in(h["fw"], h["fs"])
    ref.set_foreign_all(h["fa"], h["fss"])
    times = []
    while len(times) < 3 and (not times or sum(times) < budget_s):
        g = h["grads"][len(times) % len(h["grads"])]
        t0 = time.perf_counter()
        ref.step(g, lr)
        times.append(time.perf_counter() - t0)
    sec = float(np.median(times))
    return {"value": round(cfg["plist"].N / sec, 1), "unit": "params/s", "cores": 1, "kind": "oracle",
            "sample": f"{len(times)} whole step(s) of the same workload, median {sec:.2f} s/step",
            "host_cpus": os.cpu_count(), "cpu_model": _cpu_model()}


def _cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


if __name__ == "__main__":
    main()
