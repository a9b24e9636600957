"""GPU parity at the benchmark configurations' full sizes, in the launch configuration bench.py
times.  BERT-Large-shaped (W = 64 and W = 256): one whole step against the whole oracle.
GPT-1.3B-shaped: the oracle recomputes windows of chunks (the compressor is chunk-local, the
ratio/update are layer-local, so a window of whole chunks is an independent sub-problem for every
layer that lies inside it) plus the served chunk.
"""
import time

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from tests.refstep import HYPER, RefStep  # noqa: E402
from tests.test_gpu_parity import (assert_close, assert_mostly_close, sign_bit_mismatch, words_of, _need_gpu,  # noqa: E402
                                   DeviceStep, finish)
from workloads import Streams, make_config, gradient, init_state, foreign_worker_chunks, foreign_server_chunks  # noqa: E402
from workloads.gen import init_state_items  # noqa: E402
from workloads.gen import layer_kappa  # noqa: E402

pytestmark = pytest.mark.gpu


def device_setup(cfg, server_chunk, seed=0, two_pass=False, packed=False, fused=False, x_lp_dtype=None,
                 deferred=False):
    st = Streams(seed, device="cuda:0")
    pl = cfg["plist"]
    import paper_2104_06069_amd as ob
    if two_pass:
        dev = DeviceStep(pl.offsets, cfg["W"], server_chunk, two_pass=True, packed_momentum=packed,
                         fused_apply=fused, x_lp_dtype=x_lp_dtype, deferred_error=deferred, **HYPER)
    else:  # whatever the library selects for this size on this device
        from paper_2104_06069_amd.step import DeviceStep as D
        # (with the deferred errors also the variance in deferred form: the benchmarked configuration)
        dev = D(pl.offsets, cfg["W"], server_chunk, packed_momentum=packed, fused_apply=fused,
                x_lp_dtype=x_lp_dtype, deferred_error=deferred,
                deferred_variance=(4 if deferred and packed and fused and x_lp_dtype is None else 0), **HYPER)
    print(f"{cfg['name']}: single-pass worker compression = {ob.ob_lamb_uses_single_pass(dev.ctx)}", flush=True)
    s = init_state(st, cfg)
    # non-trivial momentum and errors, as after many steps
    s["m"] = st.normal("m0", 0, cfg["n_pad"], 1e-4); s["m"][pl.N:] = 0
    s["err_worker"] = st.normal("ew0", 0, cfg["n_pad"], 5e-5)
    s["err_server"] = st.normal("es0", 0, cfg["n_c"], 5e-5)
    dev.load_state(s)
    g = gradient(st, cfg, 0, kappa=layer_kappa(st, cfg))
    fw, fs = foreign_worker_chunks(st, cfg, 0)
    fa, fss = foreign_server_chunks(st, cfg, 0)
    dev.packed_in.copy_(fw); dev.scales_in.copy_(torch.from_numpy(fs))
    dev.packed_all.copy_(fa); dev.server_scales.copy_(torch.from_numpy(fss))
    torch.cuda.synchronize()
    return st, dev, g


@pytest.mark.parametrize("name,two_pass,packed,fused,lp,serial", [
    # (this one with the oracle's serial routines, the others with its multi-threaded drivers, which
    # tests/test_oracle_mt.py pins bit-equal to them)
    ("bert_large", False, False, False, None, True), ("bert_large_w256", False, False, False, None, False),
    ("bert_large", True, False, False, None, False), ("bert_large", False, True, False, None, False),
    # the configuration the benchmark times (1-bit momentum, ratio pass and update in one call) at W = 256;
    # at W = 64 it runs among simulated ranks in the test below
    ("bert_large_w256", False, True, True, None, False),
    # ... and its mixed-precision variant: binary16 gradient (inverse loss scale 1/512), bfloat16 copy of x
    ("bert_large", False, True, True, ("f16", "bf16", 1.0 / 512), False)])
def test_bert_large_whole_step(name, two_pass, packed, fused, lp, serial):
    """Whole steps against the whole oracle; with the 1-bit momentum two steps, so that the second
    one reads the momentum from the first one's packed output."""
    _need_gpu()
    from tests.refstep import default_threads
    cfg = make_config(name)
    c = cfg["W"] // 2
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}
    st, dev, g = device_setup(cfg, c, two_pass=two_pass, packed=packed, fused=fused,
                              x_lp_dtype=tdt[lp[1]] if lp else None, deferred=packed)
    if fused:
        import paper_2104_06069_amd as ob
        print(f"{name}: layers in the single-kernel ratio+update path: {ob.ob_lamb_fused_layers(dev.ctx)}", flush=True)
        assert ob.ob_lamb_fused_layers(dev.ctx) > 100
    ref = RefStep(cfg["plist"].offsets, cfg["W"], c, threads=1 if serial else default_threads())
    ref.load_state({k: dev.get(k) for k in ref.t})
    if lp:
        dev.grad_scale = ref.grad_scale = lp[2]
    lr = 2e-3
    N = ref.N
    for t in range(2 if packed else 1):
        if t > 0:
            dev.begin_step()
            g = gradient(st, cfg, t)
            fa, fss = foreign_server_chunks(st, cfg, t)
            dev.packed_all.copy_(fa); dev.server_scales.copy_(torch.from_numpy(fss))
            torch.cuda.synchronize()
        ref.set_foreign_in(dev.packed_in.cpu().numpy(), dev.scales_in.cpu().numpy())
        ref.set_foreign_all(dev.packed_all.cpu().numpy(), dev.server_scales.cpu().numpy())
        if lp:   # the gradient as the backward pass of a loss-scaled fp16 run would hand it over
            g = (g / lp[2]).to(tdt[lp[0]])
            gh = (1 if lp[0] == "f16" else 2, g.view(torch.int16).cpu().numpy().view(np.uint16))
        else:
            gh = g.cpu().numpy()
        t0 = time.time()
        ref.step(gh, lr)
        print(f"{name}: oracle step {time.time() - t0:.1f} s", flush=True)
        dev.step(g, lr)
        torch.cuda.synchronize()
        assert np.array_equal(words_of(dev.packed_local), ref.bits_local), "worker sign words"
        assert_close(dev.scales_local.cpu().numpy(), ref.scales_local, "worker scales")
        assert np.array_equal(words_of(dev.packed_all), ref.bits_all), "server sign words"
        assert_close(dev.server_scales.cpu().numpy(), ref.server_scales, "server scales")
        nd = {}
        for k in ("err_worker", "err_server", "v_fresh", "r_prev", "coeff_c", "x", "m"):
            nd[k] = assert_close(dev.get(k), ref.t[k], k)
        print(f"{name}: step {t}: elements not bit-equal (within 1e-6): {nd}", flush=True)
        if lp:
            got = dev.x_lp.view(torch.int16).cpu().numpy().view(np.uint16)
            want = ref.x_lp(1 if lp[1] == "f16" else 2)
            same = dev.get("x")[:N].view(np.uint32) == ref.t["x"][:N].view(np.uint32)
            assert same.mean() > 0.99
            assert np.array_equal(got[:N][same], want[:N][same]), "16-bit parameter copy"
            assert np.all(got[N:] == 0)
    finish(dev)


def test_bert_large_whole_steps_among_simulated_ranks():
    """Two whole steps at the full BERT-Large size (W = 64) in the benchmarked configuration, with
    what the other 63 ranks send taken from simulated ranks instead of random words:
    the packed chunks that arrive for the served chunk come from 63 workers that each compress, with
    the oracle's compressor and an error buffer of their own, the same global momentum advanced by
    their own gradient draw; the recompressed chunks of the other 63 servers come from servers that
    each hold an error buffer of their own and receive what this worker sent.  Both carry their
    error buffers from the first step into the second."""
    _need_gpu()
    import paper_2104_06069_amd as ob
    from paper_2104_06069_amd.step import DeviceStep as D
    from tests.refstep import default_threads, simulated_server_chunks, simulated_worker_chunks
    cfg = make_config("bert_large")
    pl, W, n_c = cfg["plist"], cfg["W"], cfg["n_c"]
    c = 21
    MT = default_threads()
    st = Streams(12, device="cuda:0")
    dev = D(pl.offsets, W, c, packed_momentum=True, fused_apply=True, deferred_error=True, **HYPER)
    assert ob.ob_lamb_fused_layers(dev.ctx) > 100 and ob.ob_lamb_uses_single_pass(dev.ctx)
    s = init_state(st, cfg)
    s["m"] = st.normal("m0", 0, cfg["n_pad"], 1e-4); s["m"][pl.N:] = 0
    s["err_worker"] = st.normal("ew0", 0, cfg["n_pad"], 5e-5)
    s["err_server"] = st.normal("es0", 0, n_c, 5e-5)
    dev.load_state(s)
    del s
    ref = RefStep(pl.offsets, W, c, threads=MT)
    ref.load_state({k: dev.get(k) for k in ref.t})
    errs_w = {w: st.normal(f"ew_{w}", 0, n_c, 5e-5).cpu().numpy() for w in range(W) if w != c}
    errs_s = {k: st.normal(f"es_{k}", 0, n_c, 5e-5).cpu().numpy() for k in range(W) if k != c}
    lr = 2e-3
    for t in range(2):
        g = gradient(st, cfg, t)
        t0 = time.time()
        grads_w = {w: st.student_t3(f"grad_{w}", t, n_c, 1e-3).cpu().numpy() for w in range(W) if w != c}
        m_chunk = np.ascontiguousarray(ref.t["m"][c * n_c:(c + 1) * n_c])   # the same on every rank
        fw, fs = simulated_worker_chunks(ref.F, pl.offsets, W, n_c, c, None, HYPER["beta1"], m_chunk,
                                         grads_w, errs_w, threads=MT)
        ref.compress_local(g.cpu().numpy())
        fa, fss = simulated_server_chunks(ref.F, W, n_c, c, ref.bits_local, ref.scales_local, errs_s,
                                          threads=MT)
        ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
        ref.gather(); ref.server_reduce(); ref.layer_ratios(); ref.decompress_apply(lr)
        print(f"simulated ranks: step {t}: oracle and the 126 simulated ranks {time.time() - t0:.1f} s; "
              f"scales received {fs[fs > 0].min():.3g} .. {fs.max():.3g}", flush=True)
        dev.begin_step()
        dev.packed_in.copy_(torch.from_numpy(fw.view(np.int32))); dev.scales_in.copy_(torch.from_numpy(fs))
        dev.packed_all.copy_(torch.from_numpy(fa.view(np.int32))); dev.server_scales.copy_(torch.from_numpy(fss))
        dev.step(g, lr)
        torch.cuda.synchronize()
        assert np.array_equal(words_of(dev.packed_local), ref.bits_local), "worker sign words"
        assert_close(dev.scales_local.cpu().numpy(), ref.scales_local, "worker scales")
        assert np.array_equal(words_of(dev.packed_all), ref.bits_all), "server sign words"
        assert_close(dev.server_scales.cpu().numpy(), ref.server_scales, "server scales")
        nd = {k: assert_close(dev.get(k), ref.t[k], k)
              for k in ("err_worker", "err_server", "v_fresh", "r_prev", "coeff_c", "x", "m")}
        print(f"simulated ranks: step {t}: elements not bit-equal (within 1e-6): {nd}", flush=True)
    finish(dev)


def window_cfg(cfg, c0, c1):
    """Sub-problem made of chunks [c0, c1): offsets clipped to the window."""
    n_c = cfg["n_c"]
    A, B = c0 * n_c, c1 * n_c
    off = np.clip(cfg["plist"].offsets, A, B) - A
    inside = (cfg["plist"].offsets[:-1] >= A) & (cfg["plist"].offsets[1:] <= B) & \
             (cfg["plist"].offsets[1:] > cfg["plist"].offsets[:-1])
    return A, B, off.astype(np.int64), inside


def test_gpt_1p3b_windows():
    _need_gpu()
    cfg = make_config("gpt_1p3b")
    W, n_c, pl = cfg["W"], cfg["n_c"], cfg["plist"]
    c_srv = 77
    st, dev, g = device_setup(cfg, c_srv)
    lr = 2e-3
    before = {k: dev.t[k].clone() for k in ("x", "m", "v_fresh", "v_frozen", "err_worker", "err_server",
                                            "c_avg", "r_prev")}
    fin_words, fin_scales = dev.packed_in.clone(), dev.scales_in.clone()
    dev.step(g, lr)
    torch.cuda.synchronize()
    # windows: the first chunks (embedding start), chunks around the served one, the last chunks
    # (small tensors, final LayerNorm, padding), and a stretch of a transformer block
    whole = 0
    for (c0, c1) in ((0, 2), (10, 13), (c_srv - 1, c_srv + 2), (W - 3, W)):
        A, B, off, inside = window_cfg(cfg, c0, c1)
        Wn = c1 - c0
        srv_in = c0 <= c_srv < c1
        ref = RefStep(off, Wn, (c_srv - c0) if srv_in else 0, n_pad=B - A)
        assert ref.n_pad == B - A and ref.n_c == n_c
        for k in ("x", "m", "v_fresh", "v_frozen", "err_worker"):
            ref.t[k][...] = before[k][A:B].cpu().numpy()
        ref.t["c_avg"][...] = before["c_avg"].cpu().numpy()
        ref.t["r_prev"][...] = before["r_prev"].cpu().numpy()
        gw = g[A:B].cpu().numpy()
        ref.compress_local(gw)
        assert np.array_equal(words_of(dev.packed_local[A // 32:B // 32]), ref.bits_local), (c0, "worker words")
        assert_close(dev.scales_local[c0:c1].cpu().numpy(), ref.scales_local, "worker scales")
        assert_close(dev.err_dense()[A:B].cpu().numpy(), ref.t["err_worker"], "worker error")
        if srv_in:
            ref.t["err_server"][...] = before["err_server"].cpu().numpy()
            refs = RefStep(np.array([0, n_c]), W, c_srv, n_pad=W * n_c)   # served chunk, full fan-in
            refs.t["err_server"][...] = before["err_server"].cpu().numpy()
            refs.set_foreign_in(fin_words.cpu().numpy(), fin_scales.cpu().numpy())
            b = n_c // 8
            refs.bits_in[c_srv * b:(c_srv + 1) * b] = ref.bits_local[(c_srv - c0) * b:(c_srv - c0 + 1) * b]
            refs.scales_in[c_srv] = ref.scales_local[c_srv - c0]
            from oracle.obref import Ref
            bo, so = Ref(np.float32).server_reduce(W, refs.bits_in, refs.scales_in, refs.t["err_server"])
            wpc = n_c // 32
            assert np.array_equal(words_of(dev.packed_all[c_srv * wpc:(c_srv + 1) * wpc]), bo), "server words"
            assert_close(dev.server_scales[c_srv:c_srv + 1].cpu().numpy(), np.array([so]), "server scale")
            assert_close(dev.get("err_server"), refs.t["err_server"], "server error")
        # ratio and update from the device's packed_all / scales (inputs), window only
        ref.set_foreign_all(dev.packed_all[A // 32:B // 32].cpu().numpy(),
                            dev.server_scales[c0:c1].cpu().numpy())
        ref.layer_ratios()
        ref.decompress_apply(lr)
        assert_close(dev.v_fresh_dense()[A:B].cpu().numpy(), ref.t["v_fresh"], "v_fresh")
        idx = np.nonzero(inside)[0]
        whole += idx.size
        assert_close(dev.get("r_prev")[idx], ref.t["r_prev"][idx], "r")
        assert_close(dev.get("coeff_c")[idx], ref.t["coeff_c"][idx], "c")
        offs = pl.offsets
        for l in idx:
            a, b_ = int(offs[l]) - A, int(offs[l + 1]) - A
            assert_close(dev.t["x"][A + a:A + b_].cpu().numpy(), ref.t["x"][a:b_], f"x layer {l}")
            assert np.array_equal(dev.t["m"][A + a:A + b_].cpu().numpy(), ref.t["m"][a:b_]), f"m layer {l}"
        print(f"gpt window chunks [{c0},{c1}): {idx.size} whole layers checked", flush=True)
    assert whole >= 12
    finish(dev)


def test_bert_base_two_stage_with_generated_momentum_scale():
    """BERT-Base-shaped list (L = 158, W = 16) with per-tensor gradient scales spread over a factor
    of 100 -- the case momentum scaling (Appendix A.5.2) is for: two LAMB steps, the end-of-warmup
    snapshot with the coefficients GENERATED on the device, then compression-stage steps in the
    benchmarked configuration (1-bit momentum, ratio pass and update in one call)."""
    _need_gpu()
    from paper_2104_06069_amd.step import DeviceStep as D
    cfg = make_config("bert_base")
    pl, W, c = cfg["plist"], cfg["W"], 5
    hyper = dict(HYPER, c_min=1e-3)
    st = Streams(4, device="cuda:0")
    dev = D(pl.offsets, W, c, packed_momentum=True, fused_apply=True, **hyper)
    s = init_state(st, cfg)
    for k in ("v_fresh", "v_frozen", "c_avg"):
        s[k].zero_() if hasattr(s[k], "zero_") else s[k].fill(0)
    dev.load_state(s)
    from tests.refstep import default_threads
    ref = RefStep(pl.offsets, W, c, threads=default_threads(), **hyper)
    ref.load_state({k: dev.get(k) for k in ref.t})
    kappa = layer_kappa(st, cfg)
    assert kappa.max() / kappa.min() > 20
    T_w, T = 2, 5
    for t in range(T):
        g = gradient(st, cfg, t, kappa=kappa)
        gh = g.cpu().numpy()
        fw, fs = foreign_worker_chunks(st, cfg, t)
        fa, fss = foreign_server_chunks(st, cfg, t)
        fwh, fah = fw.cpu().numpy(), fa.cpu().numpy()

        def fill_ref(r):
            r.set_foreign_in(fwh, fs); r.set_foreign_all(fah, fss)

        def fill_dev(d):
            d.packed_in.copy_(fw); d.scales_in.copy_(torch.from_numpy(fs))
            d.packed_all.copy_(fa); d.server_scales.copy_(torch.from_numpy(fss))

        t0 = time.time()
        ref.train_step(t, T_w, gh, 1e-3, fill_ref)
        print(f"bert_base: oracle step {t}: {time.time() - t0:.1f} s", flush=True)
        dev.train_step(t, T_w, g, 1e-3, fill_dev)
        torch.cuda.synchronize()
        if t == T_w - 1:
            k_dev = dev.t["mom_scale"].cpu().numpy()
            assert_close(k_dev, ref.mom_scale, "generated momentum-scale coefficients")
            print(f"bert_base: k_l spans {k_dev.min():.3g} .. {k_dev.max():.3g}", flush=True)
            assert k_dev.max() / k_dev.min() > 20
            assert np.array_equal(dev.get("v_frozen"), dev.get("v_fresh"))
            dev.load_state(ref.t)                      # identical bits at the hand-off ...
            dev.t["mom_scale"].copy_(torch.from_numpy(ref.mom_scale))   # ... coefficients included
        if t >= T_w:
            assert np.array_equal(words_of(dev.packed_local), ref.bits_local), f"step {t}: worker sign words"
            assert np.array_equal(words_of(dev.packed_all), ref.bits_all), f"step {t}: server sign words"
        nd = {k: assert_close(dev.get(k), ref.t[k], f"step {t} {k}")
              for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c", "c_avg")}
        print(f"bert_base: step {t}: elements not bit-equal (within 1e-6): {nd}", flush=True)
    import paper_2104_06069_amd as ob
    assert ob.ob_lamb_fused_layers(dev.ctx) > 50
    finish(dev)


@pytest.mark.parametrize("two_pass_warmup", [False, True], ids=["single_pass", "two_pass"])
def test_bert_large_warmup_step(two_pass_warmup):
    """One uncompressed LAMB step (eq. (1)) at the full BERT-Large size against the whole oracle, in
    the form the library selects by default (g, m, v, x read once for the 148 layers that fit on the
    device) and in the two-pass form."""
    _need_gpu()
    import paper_2104_06069_amd as ob
    cfg = make_config("bert_large")
    pl, W = cfg["plist"], cfg["W"]
    st = Streams(7, device="cuda:0")
    dev = DeviceStep(pl.offsets, W, 0, two_pass_warmup=two_pass_warmup, **HYPER)
    nf = ob.ob_lamb_warmup_fused_layers(dev.ctx)
    print(f"bert_large: layers in the single-pass warmup kernel: {nf}", flush=True)
    assert (nf == 0) if two_pass_warmup else (nf > 100)
    s = init_state(st, cfg)
    s["m"] = st.normal("m0", 0, cfg["n_pad"], 1e-4); s["m"][pl.N:] = 0
    dev.load_state(s)
    from tests.refstep import default_threads
    ref = RefStep(pl.offsets, W, 0, threads=default_threads())
    ref.load_state({k: dev.get(k) for k in ref.t})
    for t in range(2):
        g = gradient(st, cfg, t)
        t0 = time.time()
        ref.warmup_step(g.cpu().numpy(), 2e-3)
        print(f"bert_large: oracle warmup step {time.time() - t0:.1f} s", flush=True)
        dev.warmup_step(g, 2e-3)
        torch.cuda.synchronize()
        nd = {k: assert_close(dev.get(k), ref.t[k], k) for k in ("m", "v_fresh", "x", "coeff_c", "c_avg")}
        print(f"bert_large: warmup step {t}: elements not bit-equal (within 1e-6): {nd}", flush=True)
    finish(dev)


def trajectory_on_windows(capsys, name, c_srv, windows, steps, must_cover, warmup_steps=0, seed=9,
                          check_every=10):
    """`steps` compression-stage steps at full size in the benchmarked configuration (single-pass
    compression, 1-bit momentum, ratio pass and update in one call, errors and fresh variance in
    deferred form), followed by the oracle on
    windows of whole chunks (tests/refstep.py::WindowRef): the compressor, the error feedback, the
    decompressed momentum and the fresh variance are compared for every element of every window,
    the ratio, the coefficient and the parameters for every layer that lies wholly inside one, and
    the server step with its full fan-in on the served chunk, which lies in one of the windows.
    must_cover: tensor names that have to be among those layers.
    warmup_steps > 0: the run starts with that many LAMB steps (eq. (1)), the end-of-warmup snapshot
    and the momentum-scale coefficients GENERATED on the device (Appendix A.5.2), which are compared
    with the oracle's from the whole momentum and then drive the compression stage."""
    import paper_2104_06069_amd as ob
    from paper_2104_06069_amd.step import DeviceStep as D
    from tests.refstep import WindowRef, default_threads
    from oracle.obref import Ref
    cfg = make_config(name)
    pl, W, n_c = cfg["plist"], cfg["W"], cfg["n_c"]
    names = [n for n, _ in pl.tensors]
    MT = default_threads()
    hyper = dict(HYPER, c_min=1e-3) if warmup_steps else dict(HYPER)
    st = Streams(seed, device="cuda:0")
    dev = D(pl.offsets, W, c_srv, packed_momentum=True, fused_apply=True, deferred_error=True,
            deferred_variance=4, **hyper)
    # one array at a time: at the largest sizes two sets of N-sized arrays would not fit beside the
    # gradient and the dense views taken at the end
    for k, a in init_state_items(st, cfg):
        if warmup_steps:
            if k in ("v_fresh", "v_frozen"):
                a.zero_()
            elif k == "c_avg":
                a[...] = 0
        elif k == "m":          # as after many steps: non-trivial momentum and errors
            a = st.normal("m0", 0, cfg["n_pad"], 1e-4); a[pl.N:] = 0
        elif k == "err_worker":
            a = st.normal("ew0", 0, cfg["n_pad"], 5e-5)
        elif k == "err_server":
            a = st.normal("es0", 0, cfg["n_c"], 5e-5)
        dev.load_state({k: a})
        del a
    wins = [WindowRef(pl.offsets, W, n_c, c0, c1, c_srv, threads=MT, **hyper) for (c0, c1) in windows]
    assert sum(w.served for w in wins) == 1, "the served chunk must lie in exactly one window"
    covered = set()
    for w in wins:
        covered |= {names[l] for l in w.layers}
    assert set(must_cover) <= covered, sorted(set(must_cover) - covered)

    def get(k, A, B):
        return (dev.t[k] if A is None else dev.t[k][A:B]).cpu().numpy()
    for w in wins:
        w.load(get)
    x0 = [w.t["x"].copy() for w in wins]
    kappa = layer_kappa(st, cfg)
    exact = True       # until a scale differs in its last bit between the two sides
    t_or = 0.0
    for t in range(warmup_steps + steps):
        lr = 1e-3 * (1 + t % 5)
        g = gradient(st, cfg, t, kappa=kappa)
        if t < warmup_steps:
            dev.warmup_step(g, lr)
            t0 = time.time()
            for w in wins:
                w.ref.warmup_step(g[w.A:w.B].cpu().numpy(), lr)
            if t == warmup_steps - 1:
                dev.freeze(); dev.momentum_scale()
                # the coefficients need every layer's RMS: the oracle forms them from the whole momentum
                m_all = dev.t["m"].cpu().numpy()
                k_ref = Ref(np.float32, MT).momentum_scale(pl.offsets, m_all)
                k_dev = dev.t["mom_scale"].cpu().numpy()
                assert_close(k_dev, k_ref, "generated momentum-scale coefficients")
                print(f"{name}: k_l spans {k_dev.min():.3g} .. {k_dev.max():.3g}", flush=True)
                for w in wins:
                    assert np.array_equal(m_all[w.A:w.B], w.t["m"]), "momentum at the hand-off"
                    assert_close(dev.t["x"][w.A:w.B].cpu().numpy()[w.lo[w.layers[0]]:w.hi[w.layers[-1]]],
                                 w.t["x"][w.lo[w.layers[0]]:w.hi[w.layers[-1]]], "x at the hand-off")
                    w.ref.freeze()
                    w.ref.mom_scale = k_ref
                    # identical bits at the hand-off: the oracle's windows continue from the device's
                    # state (compared above), coefficients included
                    w.load(get)
                del m_all
                dev.t["mom_scale"].copy_(torch.from_numpy(k_ref))
            t_or += time.time() - t0
            continue
        fw, fs = foreign_worker_chunks(st, cfg, t)
        fa, fss = foreign_server_chunks(st, cfg, t)
        dev.begin_step()
        dev.packed_in.copy_(fw); dev.scales_in.copy_(torch.from_numpy(fs))
        dev.packed_all.copy_(fa); dev.server_scales.copy_(torch.from_numpy(fss))
        dev.step(g, lr)
        t0 = time.time()
        fw_h = None
        for w in wins:
            if w.served:
                fw_h = fw.cpu().numpy().view(np.uint32)
            w.step(g[w.A:w.B].cpu().numpy(), lr, fa[w.A // 32:w.B // 32].cpu().numpy().view(np.uint32),
                   fss[w.c0:w.c1], fw_h if w.served else None, fs if w.served else None)
        t_or += time.time() - t0
        k = t - warmup_steps
        if k % check_every == 0 or k == steps - 1:
            for w in wins:
                sl = dev.scales_local[w.c0:w.c1].cpu().numpy()
                assert_close(sl, w.ref.scales_local, f"step {k}: worker scales")
                exact = exact and np.array_equal(sl, w.ref.scales_local)
                if w.served:
                    ssv = dev.server_scales[c_srv:c_srv + 1].cpu().numpy()
                    assert_close(ssv, np.array([w.server_scale]), f"step {k}: server scale")
                    exact = exact and ssv[0] == w.server_scale
            for w in wins:
                wl = words_of(dev.packed_local[w.A // 32:w.B // 32])
                wpc = n_c // 32
                if exact:
                    assert np.array_equal(wl, w.ref.bits_local), f"step {k}: worker words"
                    if w.served:
                        assert np.array_equal(words_of(dev.packed_all[c_srv * wpc:(c_srv + 1) * wpc]),
                                              w.server_bits), f"step {k}: server words"
                else:
                    assert sign_bit_mismatch(wl, w.ref.bits_local) <= 1e-4, f"step {k}: worker words"
            with capsys.disabled():   # a sign of life for whoever watches the run
                print(f" [{name}: step {k} ok{'' if exact else ' (a scale differed in its last bit)'}, "
                      f"oracle {t_or:.0f} s so far]", end="", flush=True)
    torch.cuda.synchronize()
    m_dev = dev.get("m")
    err_dev = dev.err_dense()
    vf_dev = dev.v_fresh_dense()
    r_dev, c_dev = dev.get("r_prev"), dev.get("coeff_c")
    num = den = 0.0
    n_layers = 0
    for i, w in enumerate(wins):
        close = assert_close if exact else assert_mostly_close
        close(err_dev[w.A:w.B].cpu().numpy(), w.t["err_worker"], "worker error")
        close(vf_dev[w.A:w.B].cpu().numpy(), w.t["v_fresh"], "v_fresh")
        if w.served:
            close(dev.get("err_server"), w.t["err_server"], "server error")
        assert_close(r_dev[w.layers], w.t["r_prev"][w.layers], "r")
        assert_close(c_dev[w.layers], w.t["coeff_c"][w.layers], "c")
        xw = dev.t["x"][w.A:w.B].cpu().numpy()
        for l in w.layers:
            a, b_ = int(w.lo[l]), int(w.hi[l])
            close(xw[a:b_], w.t["x"][a:b_], f"x of {names[l]}")
            if exact:
                assert np.array_equal(m_dev[w.A + a:w.A + b_], w.t["m"][a:b_]), f"m of {names[l]}"
            num += float(np.sum((xw[a:b_].astype(np.float64) - w.t["x"][a:b_]) ** 2))
            den += float(np.sum(w.t["x"][a:b_].astype(np.float64) ** 2))
            assert not np.array_equal(xw[a:b_], x0[i][a:b_]), f"{names[l]} never moved"
            n_layers += 1
    rel = (num / den) ** 0.5
    print(f"{name}: {steps} compression steps after {warmup_steps} LAMB steps, {n_layers} whole layers in "
          f"{len(wins)} windows ({sum(w.B - w.A for w in wins) / 1e6:.0f} M elements), oracle on {MT} threads "
          f"{t_or:.0f} s, relative L2 error of x = {rel:.3e}, exact = {exact}", flush=True)
    assert rel <= 1e-4
    r = dev.get("r_prev")
    assert np.all(r >= hyper["r_min"]) and np.all(r <= hyper["r_max"])
    print(f"{name}: layers in the single-kernel ratio+update path: {ob.ob_lamb_fused_layers(dev.ctx)}", flush=True)
    finish(dev)


def chunks_of(cfg, first, last):
    """The chunks [c0, c1) that hold tensors first..last (names) entirely."""
    pl = cfg["plist"]
    names = [n for n, _ in pl.tensors]
    a = int(pl.offsets[names.index(first)]); b = int(pl.offsets[names.index(last) + 1])
    return a // cfg["n_c"], -(-b // cfg["n_c"])


def test_bert_large_100_steps_on_windows_with_the_served_chunk(capsys):
    """configs[2] at its stated length: 100 steps, W = 64; the window holds the served chunk."""
    trajectory_on_windows(capsys, "bert_large", c_srv=33, windows=[(32, 35)], steps=100,
                          must_cover=[])


def test_bert_base_100_steps_two_stage_on_windows(capsys):
    """configs[1] at its stated length: 100 compression steps, W = 16, per-tensor gradient scales
    spread over a factor of 100, momentum scaling generated on the device after two LAMB steps.
    The window holds the 23.4 M-element word embedding (too large for the kernels with a per-layer
    barrier: plain kernels on tile lists) and the served chunk."""
    cfg = make_config("bert_base")
    c0, c1 = chunks_of(cfg, "emb.word", "emb.ln.b")
    trajectory_on_windows(capsys, "bert_base", c_srv=1, windows=[(c0, c1)], steps=100, warmup_steps=2,
                          must_cover=["emb.word", "emb.pos", "emb.type"])


def test_gpt_1p3b_50_steps_two_stage_on_windows(capsys):
    """configs[4] at its stated length: 50 compression steps, W = 128, 1 % of the tensors with
    gradients of 1e-9 (their momentum-scale coefficients, generated on the device after two LAMB
    steps, are about 10^6 times the others').  One window holds the 103 M-element word embedding and
    the position table, the other a whole transformer block (QKV 12.6 M, FFN 16.8 M: the tensors
    that are too large for the kernels with a per-layer barrier), among them one of the tensors with
    near-zero gradients, and the served chunk."""
    cfg = make_config("gpt_1p3b")
    seed = 9
    names = [n for n, _ in cfg["plist"].tensors]
    kappa = layer_kappa(Streams(seed), cfg)
    assert kappa[names.index("l11.out.w")] < 1e-3    # this seed's choice of near-zero tensors
    e0, e1 = chunks_of(cfg, "emb.word", "emb.pos")
    b0, b1 = chunks_of(cfg, "l11.qkv.w", "l11.ffn2.w")
    assert e1 <= b0
    trajectory_on_windows(capsys, "gpt_1p3b", c_srv=b0 + 1, windows=[(e0, e1), (b0, b1)], steps=50,
                          warmup_steps=2, check_every=10, seed=seed,
                          must_cover=["emb.word", "emb.pos", "l11.qkv.w", "l11.out.w", "l11.ffn1.w",
                                      "l11.ffn2.w"])


def test_flat_buffer_longer_than_2_to_32_on_windows(capsys):
    """Maximum sizes: a flat buffer of 4.54e9 elements (the GPT-1.3B block repeated 88 times; 18 GB per
    fp32 array, W = 256), so that element indices pass 2^31 and 2^32 and byte offsets 2^34.  Four
    compression steps in the benchmarked configuration, compared with the oracle on three windows:
    the transformer block in which index 2^31 falls plus the first tensors of the next one, the
    same around index 2^32 (with the served chunk), and the last block with the end of the
    parameters and the padding.  Each window holds tensors of both paths: 12.6 M / 16.8 M-element
    ones (plain kernels) and 4.2 M-element and small ones (kernel with the per-layer barrier)."""
    _need_gpu()
    if torch.cuda.get_device_properties(0).total_memory < 200 * 2 ** 30:
        pytest.skip("needs about 170 GB of device memory")
    import gc
    gc.collect(); torch.cuda.empty_cache()    # what earlier tests left in torch's cache
    cfg = make_config("gpt_beyond_2p32")
    pl, n_c = cfg["plist"], cfg["n_c"]
    assert pl.N > 2 ** 32
    names = [n for n, _ in pl.tensors]
    off = pl.offsets

    def block_of(i):
        l = int(np.searchsorted(off, i, side="right")) - 1
        return int(names[l].split(".")[0][1:])
    b31, b32 = block_of(2 ** 31), block_of(2 ** 32)
    w31 = chunks_of(cfg, f"l{b31}.qkv.w", f"l{b31 + 1}.out.w")
    w32 = chunks_of(cfg, f"l{b32}.qkv.w", f"l{b32 + 1}.out.w")
    wend = (chunks_of(cfg, "l87.qkv.w", "lnf.b")[0], cfg["W"])
    assert w31[0] * n_c < 2 ** 31 < w31[1] * n_c and w32[0] * n_c < 2 ** 32 < w32[1] * n_c
    assert w31[1] <= w32[0] and w32[1] <= wend[0]
    c_srv = -(-2 ** 32 // n_c)          # the first chunk that lies wholly beyond 2^32
    assert w32[0] <= c_srv < w32[1]
    trajectory_on_windows(capsys, "gpt_beyond_2p32", c_srv=c_srv, windows=[w31, w32, wend], steps=4,
                          check_every=1, seed=4,
                          must_cover=[f"l{b31}.ffn2.w", f"l{b31 + 1}.qkv.w", f"l{b31 + 1}.out.w",
                                      f"l{b32}.out.w", f"l{b32}.ffn1.w", f"l{b32 + 1}.out.w",
                                      "l87.ffn2.w", "lnf.w", "lnf.b"])
    gc.collect(); torch.cuda.empty_cache()


def test_bert_large_bitwise_reproducible():
    """Two runs of three steps at the full BERT-Large size in the benchmarked configuration give
    identical bits everywhere: with thousands of workgroups arriving at the barriers in whatever
    order the hardware runs them, the order must not enter any result."""
    _need_gpu()
    cfg = make_config("bert_large")
    outs = []
    for run in range(2):
        st, dev, g = device_setup(cfg, cfg["W"] // 2, seed=5, packed=True, fused=True, deferred=True)
        for t in range(3):
            if t > 0:
                dev.begin_step()
                g = gradient(st, cfg, t)
                fa, fss = foreign_server_chunks(st, cfg, t)
                dev.packed_all.copy_(fa); dev.server_scales.copy_(torch.from_numpy(fss))
            dev.step(g, 1e-3)
        torch.cuda.synchronize()
        out = {k: dev.t[k].clone() for k in ("x", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c")}
        out["err_dense"] = dev.err_dense().clone()
        out["v_fresh_dense"] = dev.v_fresh_dense().clone()
        out["packed_local"] = dev.packed_local.clone(); out["packed_all"] = dev.packed_all.clone()
        out["scales_local"] = dev.scales_local.clone(); out["server_scales"] = dev.server_scales.clone()
        outs.append(out)
        finish(dev)
    for k in outs[0]:
        a, b = outs[0][k], outs[1][k]
        same = torch.equal(a.view(torch.int32), b.view(torch.int32)) if a.dtype == torch.float32 else torch.equal(a, b)
        assert same, k
