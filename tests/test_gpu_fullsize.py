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
from tests.test_gpu_parity import assert_close, words_of, _need_gpu, DeviceStep, finish  # noqa: E402
from workloads import Streams, make_config, gradient, init_state, foreign_worker_chunks, foreign_server_chunks  # noqa: E402
from workloads.gen import layer_kappa  # noqa: E402

pytestmark = pytest.mark.gpu


def device_setup(cfg, server_chunk, seed=0, two_pass=False, packed=False, fused=False, x_lp_dtype=None):
    st = Streams(seed, device="cuda:0")
    pl = cfg["plist"]
    import paper_2104_06069_amd as ob
    if two_pass:
        dev = DeviceStep(pl.offsets, cfg["W"], server_chunk, two_pass=True, packed_momentum=packed,
                         fused_apply=fused, x_lp_dtype=x_lp_dtype, **HYPER)
    else:  # whatever the library selects for this size on this device
        from paper_2104_06069_amd.step import DeviceStep as D
        dev = D(pl.offsets, cfg["W"], server_chunk, packed_momentum=packed, fused_apply=fused,
                x_lp_dtype=x_lp_dtype, **HYPER)
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


@pytest.mark.parametrize("name,two_pass,packed,fused,lp", [
    ("bert_large", False, False, False, None), ("bert_large_w256", False, False, False, None),
    ("bert_large", True, False, False, None), ("bert_large", False, True, False, None),
    # the configuration the benchmark times: 1-bit momentum, ratio pass and update in one call
    ("bert_large", False, True, True, None), ("bert_large_w256", False, True, True, None),
    # ... and its mixed-precision variant: binary16 gradient (inverse loss scale 1/512), bfloat16 copy of x
    ("bert_large", False, True, True, ("f16", "bf16", 1.0 / 512))])
def test_bert_large_whole_step(name, two_pass, packed, fused, lp):
    """Whole steps against the whole oracle; with the 1-bit momentum two steps, so that the second
    one reads the momentum from the first one's packed output."""
    _need_gpu()
    cfg = make_config(name)
    c = cfg["W"] // 2
    tdt = {"f16": torch.float16, "bf16": torch.bfloat16}
    st, dev, g = device_setup(cfg, c, two_pass=two_pass, packed=packed, fused=fused,
                              x_lp_dtype=tdt[lp[1]] if lp else None)
    if fused:
        import paper_2104_06069_amd as ob
        print(f"{name}: layers in the single-kernel ratio+update path: {ob.ob_lamb_fused_layers(dev.ctx)}", flush=True)
        assert ob.ob_lamb_fused_layers(dev.ctx) > 100
    ref = RefStep(cfg["plist"].offsets, cfg["W"], c)
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
        assert_close(dev.t["err_worker"][A:B].cpu().numpy(), ref.t["err_worker"], "worker error")
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
        assert_close(dev.t["v_fresh"][A:B].cpu().numpy(), ref.t["v_fresh"], "v_fresh")
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
    ref = RefStep(pl.offsets, W, c, **hyper)
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
    ref = RefStep(pl.offsets, W, 0)
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


def trajectory_on_a_window(capsys, name, c_srv, c0, c1, steps, min_layers, seed=9):
    """`steps` compression-stage steps at full size in the benchmarked configuration (single-pass
    compression, 1-bit momentum, ratio pass and update in one call), checked against the oracle on
    the window of chunks [c0, c1).  The compressor, the error feedback, the decompressed momentum
    and the fresh variance are chunk-local, so the oracle can follow them exactly on the window
    alone; the ratio and the parameters are compared for the layers that lie wholly inside it.
    (The served chunk is outside the window: its W-way fan-in alone would cost the oracle a second
    per step; whole steps with it are compared in test_bert_large_whole_step and, for the
    GPT-shaped list, in test_gpt_1p3b_windows.)"""
    import paper_2104_06069_amd as ob
    cfg = make_config(name)
    pl, W, n_c = cfg["plist"], cfg["W"], cfg["n_c"]
    assert not (c0 <= c_srv < c1)
    A, B, off, inside = window_cfg(cfg, c0, c1)
    idx = np.nonzero(inside)[0]
    assert idx.size >= min_layers
    st, dev, _ = device_setup(cfg, c_srv, seed=seed, packed=True, fused=True)
    assert ob.ob_lamb_fused_layers(dev.ctx) > 0
    ref = RefStep(off, c1 - c0, 0, n_pad=B - A)
    for k in ("x", "m", "v_fresh", "v_frozen", "err_worker"):
        ref.t[k][...] = dev.t[k][A:B].cpu().numpy()
    ref.t["c_avg"][...] = dev.get("c_avg"); ref.t["r_prev"][...] = dev.get("r_prev")
    x0 = ref.t["x"].copy()
    t_or = 0.0
    for t in range(steps):
        lr = 1e-3 * (1 + t % 5)
        g = gradient(st, cfg, t)
        fw, fs = foreign_worker_chunks(st, cfg, t)
        fa, fss = foreign_server_chunks(st, cfg, t)
        dev.begin_step()
        dev.packed_in.copy_(fw); dev.scales_in.copy_(torch.from_numpy(fs))
        dev.packed_all.copy_(fa); dev.server_scales.copy_(torch.from_numpy(fss))
        dev.step(g, lr)
        # --- oracle on the window
        t0 = time.time()
        ref.compress_local(g[A:B].cpu().numpy())
        ref.set_foreign_all(fa[A // 32:B // 32].cpu().numpy(), fss[c0:c1])
        ref.layer_ratios(); ref.decompress_apply(lr)
        t_or += time.time() - t0
        if t % 10 == 0 or t == steps - 1:
            assert np.array_equal(words_of(dev.packed_local[A // 32:B // 32]), ref.bits_local), f"step {t}: worker words"
            assert_close(dev.scales_local[c0:c1].cpu().numpy(), ref.scales_local, f"step {t}: worker scales")
            with capsys.disabled():   # a sign of life for whoever watches the run
                print(f" [{name} trajectory: step {t} ok, oracle {t_or:.0f} s so far]", end="", flush=True)
    torch.cuda.synchronize()
    assert_close(dev.t["err_worker"][A:B].cpu().numpy(), ref.t["err_worker"], "worker error")
    assert_close(dev.t["v_fresh"][A:B].cpu().numpy(), ref.t["v_fresh"], "v_fresh")
    assert_close(dev.get("r_prev")[idx], ref.t["r_prev"][idx], "r")
    m_dev = dev.get("m")[A:B]
    offs = pl.offsets
    num = den = 0.0
    for l in idx:
        a, b_ = int(offs[l]) - A, int(offs[l + 1]) - A
        xd = dev.t["x"][A + a:A + b_].cpu().numpy()
        assert_close(xd, ref.t["x"][a:b_], f"x layer {l}")
        assert np.array_equal(m_dev[a:b_], ref.t["m"][a:b_]), f"m layer {l}"
        num += float(np.sum((xd.astype(np.float64) - ref.t["x"][a:b_]) ** 2))
        den += float(np.sum(ref.t["x"][a:b_].astype(np.float64) ** 2))
        assert not np.array_equal(xd, x0[a:b_])
    rel = (num / den) ** 0.5
    print(f"{name} trajectory: {steps} steps, {idx.size} whole layers in the window, "
          f"relative L2 error of x = {rel:.3e}", flush=True)
    assert rel <= 1e-4
    r = dev.get("r_prev")
    assert np.all(r >= HYPER["r_min"]) and np.all(r <= HYPER["r_max"])
    finish(dev)


def test_bert_large_100_step_trajectory_on_a_window(capsys):
    trajectory_on_a_window(capsys, "bert_large", c_srv=32, c0=33, c1=35, steps=100, min_layers=4)


def test_gpt_1p3b_trajectory_on_a_window(capsys):
    """The GPT-1.3B-shaped list in the benchmarked configuration: most of its tensors are too large for
    the single-kernel paths, so the plain kernels on tile lists and the barrier kernels run side by
    side; 1 % of the tensors have gradients of 1e-9."""
    trajectory_on_a_window(capsys, "gpt_1p3b", c_srv=77, c0=10, c1=13, steps=6, min_layers=5)


def test_bert_large_bitwise_reproducible():
    """Two runs of three steps at the full BERT-Large size in the benchmarked configuration give
    identical bits everywhere: with thousands of workgroups arriving at the barriers in whatever
    order the hardware runs them, the order must not enter any result."""
    _need_gpu()
    cfg = make_config("bert_large")
    outs = []
    for run in range(2):
        st, dev, g = device_setup(cfg, cfg["W"] // 2, seed=5, packed=True, fused=True)
        for t in range(3):
            if t > 0:
                dev.begin_step()
                g = gradient(st, cfg, t)
                fa, fss = foreign_server_chunks(st, cfg, t)
                dev.packed_all.copy_(fa); dev.server_scales.copy_(torch.from_numpy(fss))
            dev.step(g, 1e-3)
        torch.cuda.synchronize()
        out = {k: dev.t[k].clone() for k in ("x", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c")}
        out["packed_local"] = dev.packed_local.clone(); out["packed_all"] = dev.packed_all.clone()
        out["scales_local"] = dev.scales_local.clone(); out["server_scales"] = dev.server_scales.clone()
        outs.append(out)
        finish(dev)
    for k in outs[0]:
        a, b = outs[0][k], outs[1][k]
        same = torch.equal(a.view(torch.int32), b.view(torch.int32)) if a.dtype == torch.float32 else torch.equal(a, b)
        assert same, k
