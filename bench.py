#!/usr/bin/env python3
"""Benchmark of the 1-bit LAMB compression-stage optimizer step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input already resident in
HBM: compress_local -> (gather copy) -> server_reduce -> ratios_apply (= layer_ratios + decompress_apply).
Prints ONE JSON line: the metric on the BERT-Large-shaped list at W = 64, the dominant kernel's
roofline from HIP-event timings of its launches, per-call and per-kernel times (each kernel also
against a plain copy kernel's rate measured in the same run), the other benchmark configurations in
brief (`workloads`), and the CPU oracle timed beside it (serial, and through its multi-threaded
drivers).  `--gpus N` with N > 1 is refused: this build measures one GPU's share of the
data-parallel step and uses no collectives.
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
PREWARM = 16           # untimed steps that bring the device back to its full rate before the warm-up steps
HYPER = dict(beta1=0.9, beta2=0.999, beta3=0.9, eta=1e-6, c_min=0.01, c_max=0.3, r_min=0.5,
             r_max=4.0, r_threshold=0.1, weight_decay=0.0)

# Algorithmic HBM bytes per element of one launch of each kernel (every input read once, every
# output written once), by momentum representation.  Units per launch: n_pad for the N-sized
# kernels, n_c for the server ones.
KERNEL_BYTES = {
    "dense": {   # momentum read and written as an fp32 array
        "compress_resident": (16.125, "n_pad"),  # R g, m, err (12) + W err (4) + W bits (1/8)
        "compress_deferred": (16.25, "n_pad"),   # R g, m, z (12), own previous bits (1/8) + W z (4), bits (1/8)
        "momentum_z_sumsq": (16.0, "n_pad"),     # R g, m, err (12) + W z (4)
        "ratios_pass": (16.125, "n_pad"),        # R bits, m, v_fresh, v_frozen (12.125) + W v_fresh (4)
        "decompress_apply": (16.125, "n_pad"),   # R bits, v_frozen, x (8.125) + W x, m (8)
        "ratios_apply_resident": (28.125, "fused"),  # R bits, m, v_fresh, v_frozen, x (16.125) + W v_fresh, x, m (12)
    },
    "packed": {  # momentum read from last step's sign words, never written as fp32
        "compress_resident": (12.25, "n_pad"),   # R g, err (8) + m bits (1/8) + W err (4) + bits (1/8)
        "compress_deferred": (12.375, "n_pad"),  # R g, z (8), m bits, own previous bits (1/4) + W z (4), bits (1/8)
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


def fp32_momentum_equivalent_bytes_per_param(W):
    """The accounting this build was specified against: an fp32 momentum array and two N-sized
    update calls -- compress_local 16.125 + server_reduce (0.125 + 8.125/W) + layer_ratios 16.125 +
    decompress_apply 12.0 bytes per parameter.  The implemented step moves fewer bytes (see
    algorithmic_step_bytes_per_param), so a rate formed from these bytes is an equivalent, not an
    achieved bandwidth."""
    return 16.125 + 0.125 + 8.125 / W + 16.125 + 12.0


def hist_kernel_bytes_per_param(ages, period):
    """ob_lamb_ratios_apply_hist's kernel with the per-layer barrier, per element, averaged over
    steps that applied `ages` = {momentum steps applied: count}: R v_fresh as last written, v_frozen,
    x (12) + the sign words of a + 1 momenta ((a + 1)/8) + W x (4), and W v_fresh (4) on the steps
    that bring the array up to date (a == period)."""
    n = sum(ages.values())
    return sum(c * (16.0 + 0.125 * (a + 1) + (4.0 if a >= period else 0.0)) for a, c in ages.items()) / n


def hist_big_ratio_bytes_per_param(ages, period):
    """The ratio pass from the history on the 8192-element tiles of the layers that are too large for
    the kernel with the per-layer barrier: R v_fresh as last written, v_frozen (8) + the sign words of
    a + 1 momenta, and W v_fresh (4) on the steps that bring the array up to date."""
    n = sum(ages.values())
    return sum(c * (8.0 + 0.125 * (a + 1) + (4.0 if a >= period else 0.0)) for a, c in ages.items()) / n


def algorithmic_step_bytes_per_param(W, mode, fused_frac, compress_form, server_single_pass, fused_bytes=None,
                                     big_frac=0.0, big_ratio_bytes=None):
    """What the calls as implemented must move (each kernel's inputs once, outputs once).
    fused_frac: share of the parameters whose ratio pass and update run as one kernel
    (ob_lamb_ratios_apply), reading v_frozen and the sign words once.
    fused_bytes: that kernel's bytes per element if not KERNEL_BYTES' (hist_kernel_bytes_per_param).
    big_frac, big_ratio_bytes: share of the parameters whose ratio pass runs from the history on
    8192-element tiles (hist_big_ratio_bytes_per_param); their update is the plain kernel's."""
    k = KERNEL_BYTES[mode]
    separate = k["ratios_pass"][0] + k["decompress_apply"][0]
    compress = {"deferred": k["compress_deferred"][0], "barrier": k["compress_resident"][0],
                "two_pass": k["momentum_z_sumsq"][0] + 8.125}[compress_form]
    if compress_form == "deferred":    # the server error is deferred too: one pass over the chunk
        server = 0.125 + 8.375 / W     # R W packed chunks, zb, own previous bits; W zb, bits twice
    else:
        server = (0.125 + 8.125 / W) if server_single_pass else (0.125 + 16.125 / W)
    fb = k["ratios_apply_resident"][0] if fused_bytes is None else fused_bytes
    big = big_frac * ((big_ratio_bytes if big_ratio_bytes is not None else k["ratios_pass"][0]) + k["decompress_apply"][0])
    return (compress + fused_frac * fb + big + (1.0 - fused_frac - big_frac) * separate + server)


class Workload:
    """One benchmark configuration resident in HBM: state, a few gradients, what the other ranks send."""

    def __init__(self, name, args, torch):
        import paper_2104_06069_amd as ob
        from paper_2104_06069_amd.step import DeviceStep
        from workloads import (Streams, foreign_server_chunks, foreign_worker_chunks, gradient,
                               init_state, make_config)
        self.ob, self.torch, self.name = ob, torch, name
        self.cfg = cfg = make_config(name)
        self.pl, self.W = cfg["plist"], cfg["W"]
        self.server_chunk = self.W // 2
        st = Streams(0, device="cuda:0")
        self.mode = "dense" if args.dense_momentum else "packed"
        tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16, "none": None}
        # momentum scaling (Appendix A.5.2) off, or with the coefficients GENERATED by the library from
        # a momentum that a LAMB step has formed (below)
        self.ds = DeviceStep(self.pl.offsets, self.W, self.server_chunk, device="cuda:0", mom_scale=None,
                             packed_momentum=(self.mode == "packed"), fused_apply=not args.separate_calls,
                             x_lp_dtype=tdt[args.x_lp], status_interval=0,
                             deferred_error=not args.barrier_compress,
                             deferred_variance=self.variance_period(args),
                             flags=(ob.OB_CFG_NO_BARRIERS if getattr(args, "no_barriers", False) else 0), **HYPER)
        ds = self.ds
        ds.load_state(init_state(st, cfg))
        self.grads = [gradient(st, cfg, t).to(tdt[args.grad_dtype]) for t in range(3)]
        if args.mom_scale:
            # one LAMB step on a scratch copy of the state gives every layer a momentum of its own
            # scale; the coefficients are formed from it, then the state is put back
            keep = {k: ds.t[k].clone() for k in ("x", "m", "v_fresh", "c_avg")}
            ds.warmup_step(self.grads[0], 1e-3)
            ds.momentum_scale()
            for k, v in keep.items():
                ds.t[k].copy_(v)
            del keep
        self.fw, self.fs = foreign_worker_chunks(st, cfg, 0)
        ds.packed_in.copy_(self.fw); ds.scales_in.copy_(torch.from_numpy(self.fs))
        for i in range(len(ds._pa)):   # what the other ranks' servers send, for both buffer pairs
            fa, fss = foreign_server_chunks(st, cfg, i)
            ds._pa[i].copy_(fa); ds._ss[i].copy_(torch.from_numpy(fss))
        self.lr = 1e-3
        torch.cuda.synchronize()
        # (with a dense momentum ob_lamb_ratios_apply runs the two plain kernels for every layer)
        self.fused_params = ob.ob_lamb_fused_params(ds.ctx) if (ds.fused_apply and self.mode == "packed") else 0
        self.wfused = ob.ob_lamb_warmup_fused_params(ds.ctx)
        # (only ob_lamb_ratios_apply_hist treats the large layers' whole tiles differently from the rest)
        self.big_params = ob.ob_lamb_big_tile_params(ds.ctx) if ds.vf_period else 0

    @staticmethod
    def variance_period(args):
        """The fresh variance in deferred form needs the 1-bit momentum and the one-call ratio+update."""
        k = int(getattr(args, "variance_period", 0))
        if args.dense_momentum or args.separate_calls:
            return 0
        return k

    def ages_since(self, before):
        """{momentum steps applied: steps} of the ratio+update calls since the snapshot `before`."""
        now = self.ds.vf_ages
        d = {a: now[a] - before.get(a, 0) for a in now if now[a] - before.get(a, 0) > 0}
        return d

    def one_step(self, t):
        self.ds.begin_step()
        self.ds.step(self.grads[t % len(self.grads)], self.lr)

    def timed(self, steps, warmup, graph=False):
        """-> (mean ms per step over exactly `steps` steps bracketed by synchronisations,
               median ms per step from events recorded between the steps of a second pass).
        PREWARM untimed steps always precede the `warmup` ones: after any pause (set-up, host copies)
        the device needs about ten 2 ms steps to return to its full rate, whatever --warmup says."""
        torch = self.torch
        for t in range(PREWARM - PREWARM % 2):
            self.one_step(t)
        P = self.ds.graph_period if graph else 1
        for t in range(warmup + (-warmup % P)):
            self.one_step(t)
        torch.cuda.synchronize()
        if graph:
            # P steps return the buffer pairs (and the variance's history) to where they started: one
            # graph of P steps, replayed
            assert steps % P == 0, f"--graph replays groups of {P} steps"
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            g = torch.cuda.CUDAGraph()
            ages0 = dict(self.ds.vf_ages)
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    for t in range(P):
                        self.one_step(t)
            torch.cuda.current_stream().wait_stream(side)
            self.ages_timed = self.ages_since(ages0)     # (one group's; every replay repeats it)
            g.replay(); torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps // P):
                g.replay()
            torch.cuda.synchronize()
            mean = 1e3 * (time.perf_counter() - t0) / steps
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps // P + 1)]
            for i in range(steps // P):
                ev[i].record(); g.replay()
            ev[-1].record(); torch.cuda.synchronize()
            per = [ev[i].elapsed_time(ev[i + 1]) / P for i in range(steps // P)]
        else:
            ages0 = dict(self.ds.vf_ages)
            t0 = time.perf_counter()
            for t in range(steps):
                self.one_step(t)
            torch.cuda.synchronize()
            mean = 1e3 * (time.perf_counter() - t0) / steps
            self.ages_timed = self.ages_since(ages0)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
            for t in range(steps):
                ev[t].record(); self.one_step(t)
            ev[-1].record(); torch.cuda.synchronize()
            per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
        per.sort()
        return mean, per[len(per) // 2]

    def step_bytes(self, g_less, x_more):
        """Algorithmic bytes of one step, averaged over the steps of the last timed() loop."""
        ob, ds = self.ob, self.ds
        fb = bb = None
        big = 0.0
        if ds.vf_period and getattr(self, "ages_timed", None):
            fb = hist_kernel_bytes_per_param(self.ages_timed, ds.vf_period)
            bb = hist_big_ratio_bytes_per_param(self.ages_timed, ds.vf_period)
            big = self.big_params / float(ds.n_pad)
        return (algorithmic_step_bytes_per_param(self.W, self.mode, self.fused_params / float(ds.n_pad),
                                                 self.compress_form(),
                                                 ob.ob_lamb_server_single_pass(ds.ctx) > 0, fused_bytes=fb,
                                                 big_frac=big, big_ratio_bytes=bb)
                - g_less + x_more) * ds.n_pad

    def compress_form(self):
        if self.ds.deferred_error:
            return "deferred"
        return "barrier" if self.ob.ob_lamb_uses_single_pass(self.ds.ctx) else "two_pass"

    def warmup_reference(self, reps=5):
        """One uncompressed LAMB step (eq. (1)) on the same buffers, timed alone."""
        torch, ds = self.torch, self.ds
        ds.m_is_packed = False
        fn = lambda: ds.warmup_step(self.grads[0], self.lr)
        fn(); torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record(); torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    def close(self):
        self.ob.ob_lamb_check_device_status(self.ds.ctx, self.ds.stream)  # raises if a device wait expired
        self.ds.close()
        self.grads = self.fw = None
        self.torch.cuda.empty_cache()


def copy_ceiling(torch, ob, src, dst, reps=20):
    """Rate of the library's plain nontemporal copy kernel (1024-element tiles) between two existing
    N_pad-long arrays, timed with events on the launch stream: the device's practical streaming
    ceiling.  (No allocation here: releasing a 2 GiB buffer before a measurement left every later
    step about 1 % slower.)"""
    n = src.numel()
    s = torch.cuda.current_stream().cuda_stream
    for _ in range(5):
        ob.ob_lamb_diag_copy(src, dst, n, s)
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        ob.ob_lamb_diag_copy(src, dst, n, s)
    e1.record(); torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    assert torch.equal(src[-5:], dst[-5:]) and torch.equal(src[:5], dst[:5])
    gbps = 8.0 * n / (ms * 1e-3) / 1e9
    return {"kernel": "plain nontemporal copy, 1024-element tiles (ob_lamb_diag_copy)",
            "bytes_per_launch": 8 * n, "avg_launch_ms": round(ms, 4), "GBps": round(gbps, 1),
            "frac_of_hbm_peak": round(gbps / HBM_PEAK_GBS, 4)}


def brief(name, args, torch, steps, graph_too=False):
    """A benchmark configuration other than the headline one: step time, rate, the step's own
    algorithmic bytes against the peak, share of the parameters in the single-kernel paths, and one
    uncompressed LAMB step as reference."""
    if name == "tiny":   # launch-bound: the extra small launch of the deferred variance does not pay
        import copy
        args = copy.copy(args)
        args.variance_period = 0
    w = Workload(name, args, torch)
    mean, med = w.timed(steps, args.warmup)
    b = w.step_bytes(0.0, 0.0)
    out = {"N": w.pl.N, "W": w.W, "L": w.pl.L, "steps": steps, "ms_per_step": round(mean, 4),
           "ms_per_step_median": round(med, 4), "params_per_s": round(w.pl.N / (mean * 1e-3), 1),
           "step_algorithmic_bytes": b,
           "step_algorithmic_pct_of_hbm_peak": round(100 * b / (mean * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
           "fused_share": round(w.fused_params / float(w.ds.n_pad), 4),
           "big_tile_share": round(w.big_params / float(w.ds.n_pad), 4),
           "compress_form": w.compress_form(),
           "server_single_pass": int(w.ob.ob_lamb_server_single_pass(w.ds.ctx))}
    out["variance_period"] = w.ds.vf_period
    if graph_too:
        import copy
        ag = copy.copy(args)
        ag.graph = True
        wg = Workload(name, ag, torch)
        gm, gmed = wg.timed(steps + (-steps % wg.ds.graph_period), args.warmup, graph=True)
        bg = wg.step_bytes(0.0, 0.0)
        wg.close()
        out["graph_replay_ms_per_step"] = round(gm, 4)
        out["graph_replay_pct_of_hbm_peak"] = round(100 * bg / (gm * 1e-3) / 1e9 / HBM_PEAK_GBS, 2)
    wu = w.warmup_reference()
    out["warmup_step_ms"] = round(wu, 4)
    out["warmup_step_params_per_s"] = round(w.pl.N / (wu * 1e-3), 1)
    out["warmup_single_pass_share"] = round(w.wfused / float(w.ds.n_pad), 4)
    w.close()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="bert_large")
    ap.add_argument("--profile-steps", type=int, default=8)
    ap.add_argument("--variance-period", type=int, default=4,
                    help="bring the v_fresh array up to date every that many steps and let the steps in between form "
                         "the variance from it and the momenta's sign words (ob_lamb_ratios_apply_hist); 0: rewrite "
                         "the array at every step (ob_lamb_ratios_apply)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-workloads", action="store_true",
                    help="skip the brief runs of the other benchmark configurations")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run the library's plain copy kernel on 2 x 1 GiB 10 times (for scaling "
                         "rocprofv3 FETCH_SIZE/WRITE_SIZE readings) and exit")
    ap.add_argument("--mom-scale", action="store_true",
                    help="with Appendix A.5.2 momentum scaling, coefficients generated by the library")
    ap.add_argument("--separate-calls", action="store_true",
                    help="ob_lamb_layer_ratios + ob_lamb_decompress_apply instead of the fused "
                         "ob_lamb_ratios_apply")
    ap.add_argument("--grad-dtype", choices=["f32", "f16", "bf16"], default="f32",
                    help="mixed-precision variant: the gradient arrives in 16 bits (2 bytes/param less)")
    ap.add_argument("--x-lp", choices=["none", "f16", "bf16"], default="none",
                    help="mixed-precision variant: also write a 16-bit copy of the parameters "
                         "(2 bytes/param more)")
    ap.add_argument("--graph", action="store_true",
                    help="time replays of a HIP graph that holds as many consecutive steps as it takes for the "
                         "buffers to be arranged as at the start (2, or twice --variance-period; for launch-bound "
                         "sizes; --steps is rounded up to a multiple)")
    ap.add_argument("--no-barriers", action="store_true",
                    help="OB_CFG_NO_BARRIERS: none of the kernels with an in-kernel barrier")
    ap.add_argument("--barrier-compress", action="store_true",
                    help="ob_lamb_compress_local as one kernel with a chunk barrier that writes the error itself "
                         "(default: the deferred error form, one barrier-free pass)")
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
    import paper_2104_06069_amd as ob

    if args.calibrate_copy:
        n = 1 << 28  # 2^28 fp32 = 1 GiB read + 1 GiB written per launch
        a = torch.ones(n, device=dev); b = torch.empty_like(a)
        torch.cuda.synchronize()
        for _ in range(10):
            ob.ob_lamb_diag_copy(a, b, n, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read": 4 * n, "bytes_written": 4 * n,
                          "launches": 10}))
        return

    lp_variant = args.grad_dtype != "f32" or args.x_lp != "none"
    if lp_variant and not args.no_cpu_baseline:
        print("bench.py: the CPU-baseline leg covers the fp32 entry points; add --no-cpu-baseline "
              "to time the mixed-precision variant", file=sys.stderr)
        sys.exit(2)

    wl = Workload(args.workload, args, torch)
    ds, cfg, pl, W, mode, lr = wl.ds, wl.cfg, wl.pl, wl.W, wl.mode, wl.lr
    grads, n_grads = wl.grads, len(wl.grads)
    host0 = None
    if not args.no_cpu_baseline:
        # host copy of the initial state and inputs for the CPU-baseline leg, taken before any step
        host0 = dict(state={k: ds.get(k).copy() for k in
                            ("x", "m", "v_fresh", "v_frozen", "err_worker", "err_server", "c_avg", "r_prev")},
                     grads=[g.cpu().numpy() for g in grads[:2]],
                     fw=ds.packed_in.cpu().numpy(), fs=wl.fs.copy(), fa=ds._pa[0].cpu().numpy(),
                     fss=ds._ss[0].cpu().numpy(),
                     mom_scale=None if ds.t["mom_scale"] is None else ds.t["mom_scale"].cpu().numpy())

    if args.graph:
        args.steps += -args.steps % wl.ds.graph_period
    ms_per_step, ms_median = wl.timed(args.steps, args.warmup, graph=args.graph)

    # per-kernel durations (the library's own events: each kernel's start and end on the device) and
    # per-call times (events on the launch stream), both straight after the timed steps so that the
    # device never pauses in between
    ob.ob_lamb_profile_enable(ds.ctx, True)
    ages0 = dict(ds.vf_ages)
    for t in range(args.profile_steps):
        wl.one_step(t)
    ages_prof = wl.ages_since(ages0)
    prof = ob.ob_lamb_profile_read(ds.ctx)
    ob.ob_lamb_profile_enable(ds.ctx, False)
    for t in range(5):
        wl.one_step(t)
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
        calls[nm] = round(float(np.median([e[i].elapsed_time(e[i + 1]) for e in evs])), 4)

    # the streaming ceiling, on two of the workload's own arrays (the dense momentum array is not
    # part of the state while the momentum is kept in its 1-bit form; v_frozen is only read)
    for t in range(5):
        wl.one_step(t)
    scratch_dst = ds.t["m"] if mode == "packed" else torch.empty_like(ds.t["v_frozen"])
    ceiling = copy_ceiling(torch, ob, ds.t["v_frozen"], scratch_dst)
    if mode == "packed":
        scratch_dst.zero_()
    kern = {k: {"avg_ms": round(v[0] / v[1], 4), "launches": v[1]} for k, v in prof.items()}
    KB = dict(KERNEL_BYTES["both"])
    KB.update(KERNEL_BYTES[mode])
    KB["server_unpack_avg"] = (W / 8.0 + (8.375 if ds.deferred_error else 8.0), "n_c")
    KB["server_resident"] = (W / 8.0 + 8.125, "n_c")   # R W*bits, err (4) + W err (4), bits (1/8)
    if ages_prof:   # mean over the profiled launches, which differ in how many momentum steps they applied
        KB["ratios_apply_hist"] = (hist_kernel_bytes_per_param(ages_prof, ds.vf_period), "fused")
        KB["ratios_big_hist"] = (hist_big_ratio_bytes_per_param(ages_prof, ds.vf_period), "big")
    g_less = 2.0 if args.grad_dtype != "f32" else 0.0     # 16-bit gradient read
    x_more = 2.0 if args.x_lp != "none" else 0.0          # 16-bit parameter copy written
    for k in ("compress_resident", "compress_deferred", "momentum_z_sumsq", "warmup_moments", "warmup_resident"):
        KB[k] = (KB[k][0] - g_less, KB[k][1])
    for k in ("decompress_apply", "ratios_apply_resident", "ratios_apply_hist", "warmup_apply", "warmup_resident"):
        if k in KB:
            KB[k] = (KB[k][0] + x_more, KB[k][1])
    fused_params, wfused = wl.fused_params, wl.wfused
    units = {"n_pad": ds.n_pad, "n_c": ds.n_c, "fused": fused_params, "wfused": wfused, "big": wl.big_params}
    if wfused:   # the two-pass warmup kernels then cover only the remaining layers (two launches each)
        for k in ("warmup_moments", "warmup_apply"):
            KB[k] = (KB[k][0], "rest_w")
        units["rest_w"] = ds.n_pad - wfused
    if ds.fused_apply and fused_params:   # the plain ratio/update kernels then cover only the remaining layers
        KB["ratios_pass"] = (KB["ratios_pass"][0], "rest_ratio")
        KB["decompress_apply"] = (KB["decompress_apply"][0], "rest")
        units["rest"] = ds.n_pad - fused_params
        units["rest_ratio"] = ds.n_pad - fused_params - wl.big_params
    for k, v in kern.items():
        if k in KB:
            bpe, unit = KB[k]
            # (should a call cover its elements with several launches of one kernel: per-launch mean)
            per_call = max(1, round(v["launches"] / args.profile_steps)) if unit in ("rest", "rest_w", "rest_ratio") else 1
            v["algo_bytes"] = bpe * units[unit] / per_call
            v["GBps"] = round(v["algo_bytes"] / (v["avg_ms"] * 1e-3) / 1e9, 1)
            v["frac_of_hbm_peak"] = round(v["GBps"] / HBM_PEAK_GBS, 4)
            v["frac_of_copy_ceiling"] = round(v["GBps"] / ceiling["GBps"], 4)
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
                "frac_of_copy_ceiling": kern[dom]["frac_of_copy_ceiling"],
                "avg_launch_ms": kern[dom]["avg_ms"], "algo_bytes_per_launch": kern[dom]["algo_bytes"],
                "traffic": traffic}

    equiv_bytes = fp32_momentum_equivalent_bytes_per_param(W) * ds.n_pad
    algo_bytes = wl.step_bytes(g_less, x_more)
    out = {
        "metric": "1-bit LAMB compressed step: params/sec and % of HBM peak GB/s, 1 GPU",
        "value": round(pl.N / (ms_per_step * 1e-3), 1), "unit": "params/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "prewarm_steps": PREWARM,
        "ms_per_step": round(ms_per_step, 4), "ms_per_step_median": round(ms_median, 4),
        "value_at_median": round(pl.N / (ms_median * 1e-3), 1),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}_shaped_W{W}", "N": pl.N, "N_pad": ds.n_pad, "L": pl.L,
                   "W": W, "n_c": ds.n_c, "server_chunk": wl.server_chunk,
                   "mom_scale": bool(args.mom_scale), "momentum": mode,
                   "grad_dtype": args.grad_dtype, "x_lp": args.x_lp, "graph_replay": bool(args.graph),
                   "fused_ratios_apply": ds.fused_apply, "fused_layers": ob.ob_lamb_fused_layers(ds.ctx),
                   "fused_params": fused_params, "big_tile_params": wl.big_params,
                   "compress_form": wl.compress_form(),
                   "server_single_pass": ob.ob_lamb_server_single_pass(ds.ctx),
                   "variance_period": ds.vf_period,
                   "timed_steps_by_momentum_steps_applied": {str(a): c for a, c in sorted(getattr(wl, "ages_timed", {}).items())}},
        "step_algorithmic_bytes": algo_bytes,
        "step_algorithmic_GBps": round(algo_bytes / (ms_per_step * 1e-3) / 1e9, 1),
        "step_algorithmic_pct_of_hbm_peak": round(100 * algo_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 2),
        "step_algorithmic_pct_of_copy_ceiling": round(100 * algo_bytes / (ms_per_step * 1e-3) / 1e9 / ceiling["GBps"], 2),
        # NOT an achieved bandwidth: the bytes of the fp32-momentum, two-update-call accounting divided
        # by the measured step time (the implemented step moves step_algorithmic_bytes)
        "fp32_momentum_equivalent": {
            "bytes": equiv_bytes,
            "equivalent_GBps": round(equiv_bytes / (ms_per_step * 1e-3) / 1e9, 1),
            "equivalent_pct_of_hbm_peak": round(100 * equiv_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 2)},
        "ceiling": ceiling,
        "roofline": roofline,
        "calls_ms": calls,
        "kernels": kern,
    }

    # reference timings outside the headline metric: one uncompressed LAMB warmup step (eq. (1)) and
    # the end-of-warmup momentum-scale generation (Appendix A.5.2), on the same buffers
    wu_ms = wl.warmup_reference()
    ds.m_is_packed = False
    ds.momentum_scale(); torch.cuda.synchronize()
    e0 = torch.cuda.Event(enable_timing=True); e1 = torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(5):
        ds.momentum_scale()
    e1.record(); torch.cuda.synchronize()
    ms_ms = e0.elapsed_time(e1) / 5
    out["reference_calls"] = {
        "warmup_step_ms": round(wu_ms, 4),
        # 28 B/elem where g, m, v, x are read once, 24 + 16 in the two-pass form
        "warmup_step_GBps": round(((28.0 - g_less + x_more) * wfused + (40.0 - g_less + x_more) * (ds.n_pad - wfused))
                                  / (wu_ms * 1e-3) / 1e9, 1),
        "warmup_single_pass_params": wfused,
        "warmup_step_params_per_s": round(pl.N / (wu_ms * 1e-3), 1),
        "momentum_scale_ms": round(ms_ms, 4),
        "momentum_scale_GBps": round(4.0 * ds.n_pad / (ms_ms * 1e-3) / 1e9, 1)}
    wl.close()
    del wl, ds, grads

    if not args.no_workloads and not lp_variant:
        # the other benchmark configurations (parity-test cases), same defaults
        others = {}
        for name, steps, graph_too in (("tiny", 200, True), ("bert_base", 50, True),
                                       ("bert_large", 50, False), ("bert_large_w256", 50, False),
                                       ("gpt_1p3b", 20, False)):
            if name == args.workload:
                continue
            others[name] = brief(name, args, torch, steps, graph_too)
        out["workloads"] = others
        # the same workload with no in-kernel wait anywhere (OB_CFG_NO_BARRIERS; what a caller who cannot
        # accept the per-layer barrier's assumptions runs): deferred errors, the ratio pass of every layer
        # with enough whole tiles from the variance's history, the update as the plain kernel
        import copy
        a2 = copy.copy(args)
        a2.no_barriers = True
        if not args.separate_calls and not args.barrier_compress and not args.no_barriers:
            out["wait_free_configuration"] = brief(args.workload, a2, torch, args.steps)
    if host0 is not None:
        out["cpu_baseline"] = cpu_baseline(cfg, cfg["W"] // 2, host0, lr, args.cpu_seconds, False)
        mt = cpu_baseline(cfg, cfg["W"] // 2, host0, lr, args.cpu_seconds, True)
        if mt["cores"] > 1:
            out["cpu_baseline_mt"] = mt
    print(json.dumps(out))


def cpu_baseline(cfg, server_chunk, h, lr, budget_s, multi_threaded):
    """The oracle as it stands on the same workload: whole steps until `budget_s` seconds of CPU work
    have been spent (at least one step, at most three).  Serial routines, or its multi-threaded
    drivers, which run the same scalar routines on chunks and layers in parallel on the host's share
    of cores."""
    import numpy as np
    from tests.refstep import RefStep, default_threads
    threads = default_threads() if multi_threaded else 1
    ref = RefStep(cfg["plist"].offsets, cfg["W"], server_chunk, mom_scale=h["mom_scale"], threads=threads,
                  **HYPER)
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
    return {"value": round(cfg["plist"].N / sec, 1), "unit": "params/s", "cores": threads, "kind": "oracle",
            "sample": f"{len(times)} whole step(s) of the same workload, median {sec:.2f} s/step",
            "host_cpus": os.cpu_count(), "cpu_model": _cpu_model()}


def _cpu_model():
    """Model name as the host reports it, with family/model numbers (virtual machines often shorten
    the name)."""
    f = {}
    try:
        with open("/proc/cpuinfo") as fh:
            for line in fh:
                if ":" in line:
                    k, v = line.split(":", 1)
                    k = k.strip()
                    if k in ("model name", "cpu family", "model") and k not in f:
                        f[k] = v.strip()
                if len(f) == 3:
                    break
    except OSError:
        pass
    if not f:
        return "unknown"
    return f"{f.get('model name', 'unknown')} (family {f.get('cpu family', '?')}, model {f.get('model', '?')})"


if __name__ == "__main__":
    main()
