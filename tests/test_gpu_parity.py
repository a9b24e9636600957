"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element, on the
same seeded inputs.  Bar: packed sign words bit-exact; fp32 state within 1e-6 relative per element
(|gpu - ref| <= 1e-6 * max(|ref|, rms(ref))); trajectories within 1e-4 relative in parameter L2.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from tests.refstep import HYPER, RefStep  # noqa: E402
from workloads import Streams, make_config, gradient, init_state, foreign_worker_chunks, foreign_server_chunks  # noqa: E402
from workloads.shapes import ParamList, padded_len  # noqa: E402

pytestmark = pytest.mark.gpu

REL = 1e-6


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")


def DeviceStep(*a, two_pass=False, fused_max_tiles=None, spin_limit=None, two_pass_warmup=False, **k):
    """two_pass=True forces the two-kernel worker compression (the default picks the single-pass
    kernel whenever the chunk's workgroups fit on the device, which is the case for every size here).
    The selection travels in the context's configuration (flags, fused_max_tiles, spin_limit)."""
    from paper_2104_06069_amd.step import DeviceStep as D
    import paper_2104_06069_amd as ob
    flags = (ob.OB_CFG_TWO_PASS_COMPRESS if two_pass else 0) | (ob.OB_CFG_TWO_PASS_WARMUP if two_pass_warmup else 0)
    if fused_max_tiles == 0:    # no layer at all in the kernels with a per-layer barrier
        flags |= ob.OB_CFG_NO_FUSED_APPLY | ob.OB_CFG_TWO_PASS_WARMUP
        fused_max_tiles = None
    if spin_limit == 0:
        spin_limit = ob.OB_SPIN_NONE
    d = D(*a, flags=flags, fused_max_tiles=fused_max_tiles or 0, spin_limit=spin_limit or 0, **k)
    assert ob.ob_lamb_uses_single_pass(d.ctx) == (not two_pass)
    return d


def finish(dev):
    """No bounded device-side wait expired; then release the context."""
    import paper_2104_06069_amd as ob
    ob.ob_lamb_check_device_status(dev.ctx, dev.stream)
    dev.close()


def assert_close(gpu, ref, what, rel=REL):
    gpu = np.asarray(gpu); ref = np.asarray(ref)
    assert gpu.shape == ref.shape, what
    fin = np.isfinite(ref)
    # non-finite values must agree exactly (NaN with NaN, +-Inf with the same Inf)
    assert np.array_equal(np.isnan(gpu), np.isnan(ref)), f"{what}: NaN pattern differs"
    inf = np.isinf(ref)
    assert np.array_equal(gpu[inf], ref[inf]), f"{what}: Inf pattern differs"
    if not fin.any():
        return 0
    r = ref[fin].astype(np.float64); g = gpu[fin].astype(np.float64)
    rms = np.sqrt(np.mean(r * r))
    tol = rel * np.maximum(np.abs(r), rms)
    bad = np.abs(g - r) > tol
    assert not bad.any(), (f"{what}: {bad.sum()} of {r.size} beyond {rel} relative; worst "
                           f"{np.max(np.abs(g - r) / np.maximum(np.abs(r), rms)):.3e}")
    return int(np.count_nonzero(g != r))


def sign_bit_mismatch(a, b):
    """Fraction of differing bits between two packed streams (uint8 views)."""
    x = np.bitwise_xor(np.asarray(a).view(np.uint8), np.asarray(b).view(np.uint8))
    return float(np.unpackbits(x).sum()) / (8.0 * x.size)


def assert_mostly_close(gpu, ref, what, rel=1e-4, max_frac=1e-4):
    """After a scale has differed in its last bit, elements within one unit in the last place of zero
    may take the other sign, and their error and momentum then differ by 2*scale on BOTH sides
    legitimately: all but a fraction max_frac of the elements must agree within rel."""
    g = np.asarray(gpu, np.float64); r = np.asarray(ref, np.float64)
    rms = np.sqrt(np.mean(r * r))
    bad = np.abs(g - r) > rel * np.maximum(np.abs(r), rms)
    assert bad.mean() <= max_frac, f"{what}: {bad.sum()} of {r.size} elements beyond {rel}"


def words_of(t):
    return t.detach().cpu().numpy().view(np.uint8)


def make_case(name):
    """-> cfg dict (plist, W, n_pad, n_c, grad, server_chunk, mom_scale flag)"""
    if name in ("tiny", "bert_mini"):
        cfg = make_config(name)
        cfg["server_chunk"] = 0 if name == "tiny" else 5
        cfg["use_k"] = (name == "bert_mini")
        return cfg
    if name == "odd":      # 1-, 2-, 3-element and empty tensors, boundaries unaligned to 4, W = 3
        sizes = [1, 2, 3, 0, 4099, 5, 0, 0, 1024, 2, 4866, 1]
    elif name == "w1":     # a single chunk; several tiles and a ragged tail
        sizes = [3000, 1, 9000, 777]
    elif name == "small":  # N below one 256-element span
        sizes = [7, 90, 3]
    elif name == "one_layer":  # the whole model as one tensor (1-bit Adam's view of it)
        sizes = [50000]
    elif name == "big_and_small":
        # one tensor of 70+ tiles of 8192 elements, unaligned at both ends, between tensors of a few
        # tiles: with a low limit on the tiles per layer the large one is "too large" for the kernel
        # with the per-layer barrier while the others are not
        sizes = [3 * 8192 + 5, 75 * 8192 + 1234, 100, 4 * 8192, 2 * 8192 + 77]
    else:
        raise KeyError(name)
    W = {"odd": 3, "w1": 1, "small": 2, "one_layer": 4, "big_and_small": 2}[name]
    pl = ParamList(name, [(f"t{i}", s) for i, s in enumerate(sizes)])
    n_pad = padded_len(pl.N, W)
    return dict(name=name, plist=pl, W=W, n_pad=n_pad, n_c=n_pad // W, grad="student_t3",
                steps=3, server_chunk=W - 1, use_k=(name != "w1"))


def start_pair(cfg, seed=0, warm_state=True, two_pass=False, packed=False, fused=False,
               fused_max_tiles=None, hyper=None, deferred=False, deferred_variance=0):
    """Oracle-side and device-side steps with identical, non-trivial state."""
    st = Streams(seed)
    pl = cfg["plist"]
    k = None
    if cfg.get("use_k"):
        k = st.uniform_host("mom_scale", 0, pl.L, 0.25, 4.0)
    h = dict(HYPER)
    h.update(hyper or {})
    ref = RefStep(pl.offsets, cfg["W"], cfg["server_chunk"], mom_scale=k, **h)
    dev = DeviceStep(pl.offsets, cfg["W"], cfg["server_chunk"], mom_scale=k, two_pass=two_pass, packed_momentum=packed, fused_apply=fused,
                     fused_max_tiles=fused_max_tiles, deferred_error=deferred, deferred_variance=deferred_variance, **h)
    assert (dev.N, dev.n_pad, dev.n_c) == (ref.N, ref.n_pad, ref.n_c)
    s = init_state(st, cfg)
    if warm_state:  # non-zero momentum and errors so that every term is exercised
        s["m"] = st.normal("m0", 0, cfg["n_pad"], 1e-4); s["m"][pl.N:] = 0
        s["err_worker"] = st.normal("ew0", 0, cfg["n_pad"], 5e-5)
        s["err_server"] = st.normal("es0", 0, cfg["n_c"], 5e-5)
    ref.load_state(s)
    dev.load_state(ref.t)
    return st, ref, dev


def sync_dev_from_ref(ref, dev):
    dev.load_state(ref.t)
    dev.t["coeff_c"].copy_(torch.from_numpy(ref.t["coeff_c"]))


def push_wire(ref, dev):
    dev.packed_in.copy_(torch.from_numpy(ref.bits_in.view(np.int32)))
    dev.scales_in.copy_(torch.from_numpy(ref.scales_in))
    dev.packed_all.copy_(torch.from_numpy(ref.bits_all.view(np.int32)))
    dev.server_scales.copy_(torch.from_numpy(ref.server_scales))


CASES = ["small", "odd", "w1", "tiny", "bert_mini"]


@pytest.mark.parametrize("two_pass", [False, True, "deferred"], ids=["single_pass", "two_pass", "deferred"])
@pytest.mark.parametrize("case", CASES)
def test_phasewise_single_step(case, two_pass):
    """Each call is fed the oracle's outputs of the previous phase; signs must be bit-exact.
    The worker side in its three forms: one kernel with a chunk barrier, two passes, and the deferred
    error (one pass, the subtraction of C[z] postponed to the next call)."""
    _need_gpu()
    cfg = make_case(case)
    st, ref, dev = start_pair(cfg, two_pass=(two_pass is True), deferred=(two_pass == "deferred"))
    g = gradient(st, cfg, 0)
    gd = torch.from_numpy(g).to(dev.device)
    lr = 2e-3

    # phase 1: worker side (Algorithm 1 lines 6-7)
    ref.compress_local(g)
    dev.compress_local(gd)
    assert np.array_equal(words_of(dev.packed_local), ref.bits_local), "worker sign words"
    assert_close(dev.scales_local.cpu().numpy(), ref.scales_local, "worker scales")
    assert_close(dev.get("err_worker"), ref.t["err_worker"], "worker error")
    assert np.array_equal(dev.get("m"), ref.t["m"])  # untouched

    # phase 2: server side (line 10) on identical inputs
    fw, fs = foreign_worker_chunks(st, cfg, 0)
    ref.set_foreign_in(fw, fs)
    ref.gather()
    sync_dev_from_ref(ref, dev)
    push_wire(ref, dev)
    fa, fss = foreign_server_chunks(st, cfg, 0)
    ref.set_foreign_all(fa, fss)
    dev.packed_all.copy_(torch.from_numpy(ref.bits_all.view(np.int32)))
    dev.server_scales.copy_(torch.from_numpy(ref.server_scales))
    ref.server_reduce()
    dev.server_reduce()
    assert np.array_equal(words_of(dev.packed_all), ref.bits_all), "server sign words"
    assert_close(dev.server_scales.cpu().numpy(), ref.server_scales, "server scales")
    assert_close(dev.get("err_server"), ref.t["err_server"], "server error")

    # phase 3: ratios (lines 13-20)
    sync_dev_from_ref(ref, dev)
    push_wire(ref, dev)
    ref.layer_ratios()
    dev.layer_ratios()
    assert_close(dev.get("v_fresh"), ref.t["v_fresh"], "v_fresh")
    assert_close(dev.get("r_prev"), ref.t["r_prev"], "r")
    assert_close(dev.get("coeff_c"), ref.t["coeff_c"], "c")
    assert np.array_equal(dev.get("m"), ref.t["m"]) and np.array_equal(dev.get("x"), ref.t["x"])

    # phase 4: update (lines 13, 21)
    sync_dev_from_ref(ref, dev)
    ref.decompress_apply(lr)
    dev.decompress_apply(lr)
    assert_close(dev.get("x"), ref.t["x"], "x")
    assert_close(dev.get("m"), ref.t["m"], "m")
    # padding never touched by the layer-wise phases
    N = ref.N
    assert np.array_equal(dev.get("x")[N:], ref.t["x"][N:]) and np.all(dev.get("m")[N:] == 0)
    finish(dev)


def run_trajectory(cfg, steps, seed=0, two_pass=False, packed=False, warm_state=False, fused=False,
                   fused_max_tiles=None, hyper=None, c_avg=None, nudge_step=None, deferred=False,
                   deferred_variance=0, check_every=10):
    """The device feeds itself for `steps` steps; the oracle does the same on the host.
    While every scale has been bit-equal on both sides, everything must be bit-equal.  Once a scale
    has differed in its last bit (the two sides add the same fp64 terms in different groupings; about
    once in 10^8 reductions), elements within an ulp of zero may take the other sign: from then on
    every step still asserts the scales within 1e-6, bounds the fraction of differing sign bits and,
    every 10 steps, the errors, momentum, variance and parameters (all but 1e-4 of the elements
    within 1e-4).
    nudge_step: after that step the ORACLE's state is given what a last-bit-different scale of one
    chunk it does not serve would have left there (scale one ulp up, the chunk's errors moved by that
    ulp), so that the second regime is exercised."""
    st, ref, dev = start_pair(cfg, seed=seed, warm_state=warm_state, two_pass=two_pass, packed=packed,
                              fused=fused, fused_max_tiles=fused_max_tiles, hyper=hyper, deferred=deferred,
                              deferred_variance=deferred_variance)
    if c_avg is not None:
        ref.t["c_avg"][...] = c_avg
        dev.load_state(ref.t)
    stats = dict(word_mismatch_steps=0, scale_ulp_steps=0)
    nudged = False
    for t in range(steps):
        g = gradient(st, cfg, t)
        lr = 1e-3 * (1 + t % 5)
        fw, fs = foreign_worker_chunks(st, cfg, t)
        fa, fss = foreign_server_chunks(st, cfg, t)
        ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
        dev.begin_step()
        dev.packed_in.copy_(torch.from_numpy(np.ascontiguousarray(fw).view(np.int32)))
        dev.scales_in.copy_(torch.from_numpy(fs))
        dev.packed_all.copy_(torch.from_numpy(np.ascontiguousarray(fa).view(np.int32)))
        dev.server_scales.copy_(torch.from_numpy(fss))
        ref.step(g, lr)
        dev.step(torch.from_numpy(g).to(dev.device), lr)
        same_words = (np.array_equal(words_of(dev.packed_local), ref.bits_local)
                      and np.array_equal(words_of(dev.packed_all), ref.bits_all))
        same_scales = (np.array_equal(dev.scales_local.cpu().numpy(), ref.scales_local)
                       and np.array_equal(dev.server_scales.cpu().numpy(), ref.server_scales))
        stats["word_mismatch_steps"] += (not same_words)
        stats["scale_ulp_steps"] += (not same_scales)
        if stats["scale_ulp_steps"] == 0 and not nudged:
            # a sign may differ only after a scale differed in its last bit at an earlier step
            assert same_words, f"step {t}: sign words differ although all scales were bit-equal"
            if t % check_every == 0 or t == steps - 1:
                for k in ("x", "v_fresh", "err_worker", "r_prev"):
                    assert np.array_equal(dev.get(k), ref.t[k]), (t, k)
        else:
            assert_close(dev.scales_local.cpu().numpy(), ref.scales_local, f"step {t}: worker scales")
            assert_close(dev.server_scales.cpu().numpy(), ref.server_scales, f"step {t}: server scales")
            assert sign_bit_mismatch(words_of(dev.packed_local), ref.bits_local) <= 1e-4, f"step {t}: worker words"
            assert sign_bit_mismatch(words_of(dev.packed_all), ref.bits_all) <= 1e-4, f"step {t}: server words"
            if t % 10 == 0 or t == steps - 1:
                for k in ("err_worker", "err_server", "m", "v_fresh", "x"):
                    assert_mostly_close(dev.get(k), ref.t[k], f"step {t}: {k}")
        if t == nudge_step:
            c = (ref.c + 1) % ref.W
            assert c != ref.c, "needs a chunk that this rank does not serve"
            s0 = ref.scales_local[c]
            ulp = np.nextafter(s0, np.float32(np.inf)) - s0
            sl = slice(c * ref.n_c, (c + 1) * ref.n_c)
            sign = np.where(np.unpackbits(ref.bits_local[c * ref.n_c // 8:(c + 1) * ref.n_c // 8],
                                          bitorder="little") == 1, 1.0, -1.0)
            ref.t["err_worker"][sl] = (ref.t["err_worker"][sl].astype(np.float64) - sign * float(ulp)).astype(np.float32)
            nudged = True
    assert dev.m_is_packed == packed
    return ref, dev, stats


@pytest.mark.parametrize("case,steps,period,fused_max_tiles", [
    ("tiny", 12, 4, None), ("tiny", 20, 8, None), ("bert_mini", 30, 4, None), ("bert_mini", 21, 8, None),
    ("bert_mini", 13, 2, 1), ("odd", 14, 3, None), ("odd", 12, 5, 0), ("w1", 10, 4, None), ("small", 10, 4, None),
    ("big_and_small", 11, 4, 8), ("big_and_small", 7, 3, 5),
    ("big_and_small", 9, 4, 0)])     # no barrier kernel at all: the large tensor still works from the history
def test_trajectory_with_the_variance_in_deferred_form(case, steps, period, fused_max_tiles):
    """ob_lamb_ratios_apply_hist: the v_fresh array is brought up to date only every `period`-th
    step; in between every step forms the up-to-date variance from the array and the sign words and
    scales of the momenta since then.  After EVERY step the dense view of the variance
    (ob_lamb_variance_dense), the parameters, the errors and the ratios equal the oracle's bit for
    bit, in the kernel with the per-layer barrier and in the plain kernels (tiles at layer
    boundaries, empty and tiny tensors, momentum scaling on bert_mini)."""
    _need_gpu()
    cfg = make_case(case)
    ref, dev, stats = run_trajectory(cfg, steps, packed=True, fused=True, warm_state=True, deferred=True,
                                     deferred_variance=period, fused_max_tiles=fused_max_tiles, check_every=1)
    assert stats["scale_ulp_steps"] == 0, "bit-equality was not tested all the way"
    ages = dev.vf_ages
    assert set(ages) == set(range(1, period + 1)), ages     # every history length was exercised
    if case == "big_and_small":   # the large tensor's whole tiles take the ratio pass from the history too
        import paper_2104_06069_amd as ob
        assert ob.ob_lamb_big_tile_params(dev.ctx) >= 70 * 8192
        assert ob.ob_lamb_fused_layers(dev.ctx) == (0 if fused_max_tiles == 0 else 3)
    # what the array itself holds is the variance of the last step that wrote it
    for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c"):
        assert np.array_equal(dev.get(k), ref.t[k]), k
    finish(dev)


def test_resume_from_a_checkpoint_continues_bit_for_bit():
    """DeviceStep.checkpoint() materialises every compact form (1-bit momentum, deferred errors, the
    variance's history -- taken here in the middle of a history, two steps after the array was last
    written); a new context that loads it continues exactly where the first one would have gone:
    after four more steps every array equals the uninterrupted run's bit for bit."""
    _need_gpu()
    cfg = make_case("bert_mini")
    opts = dict(packed=True, fused=True, warm_state=True, deferred=True, deferred_variance=4)

    def steps(dev, st, t0, t1):
        for t in range(t0, t1):
            g = gradient(st, cfg, t)
            fw, fs = foreign_worker_chunks(st, cfg, t)
            fa, fss = foreign_server_chunks(st, cfg, t)
            dev.begin_step()
            dev.packed_in.copy_(torch.from_numpy(np.ascontiguousarray(fw).view(np.int32)))
            dev.scales_in.copy_(torch.from_numpy(fs))
            dev.packed_all.copy_(torch.from_numpy(np.ascontiguousarray(fa).view(np.int32)))
            dev.server_scales.copy_(torch.from_numpy(fss))
            dev.step(torch.from_numpy(g).to(dev.device), 1e-3 * (1 + t % 3))

    st, _, straight = start_pair(cfg, **opts)
    steps(straight, st, 0, 11)
    want = straight.checkpoint()
    finish(straight)

    st, _, first = start_pair(cfg, **opts)
    steps(first, st, 0, 7)
    assert first._vf_pending is not None and first._vf_n_old == 2   # in the middle of a history
    ck = first.checkpoint()
    finish(first)
    st2, _, second = start_pair(cfg, **opts)
    second.load_state(ck)
    second.t["mom_scale"].copy_(torch.from_numpy(ck["mom_scale"]))
    steps(second, st2, 7, 11)
    got = second.checkpoint()
    for k in want:
        assert np.array_equal(got[k].view(np.uint32), want[k].view(np.uint32)), k
    finish(second)


def test_trajectory_after_a_last_bit_difference_of_a_scale():
    """The regime that a last-bit difference of a scale opens (planted in the oracle's state, on the
    CPU): the two sides stay within the stated bounds for the rest of a 60-step run."""
    _need_gpu()
    cfg = make_case("bert_mini")
    ref, dev, stats = run_trajectory(cfg, 60, packed=True, fused=True, nudge_step=4, deferred=True)
    x_ref = ref.t["x"][:ref.N].astype(np.float64)
    x_gpu = dev.get("x")[:ref.N].astype(np.float64)
    rel = np.linalg.norm(x_gpu - x_ref) / np.linalg.norm(x_ref)
    print(f"nudged trajectory: relative L2 error of x = {rel:.3e}, {stats}")
    assert rel <= 1e-4
    assert not np.array_equal(dev.get("err_worker"), ref.t["err_worker"])   # the nudge did reach the state
    finish(dev)


@pytest.mark.parametrize("case,steps,two_pass,packed", [
    ("tiny", 10, False, False), ("bert_mini", 100, False, False), ("odd", 30, False, False),
    ("bert_mini", 30, True, False),
    # momentum kept in its 1-bit form from the first step on
    ("tiny", 10, False, True), ("bert_mini", 100, False, True), ("odd", 30, False, True),
    ("bert_mini", 30, True, True), ("w1", 10, True, True), ("small", 10, False, True),
    # the worker error in deferred form (z kept, C[z] subtracted by the next step)
    ("tiny", 10, "deferred", False), ("bert_mini", 100, "deferred", True), ("odd", 30, "deferred", True),
    ("w1", 10, "deferred", False), ("small", 10, "deferred", True)])
def test_trajectory(case, steps, two_pass, packed):
    """The device feeds itself for `steps` steps; the oracle does the same on the host."""
    _need_gpu()
    cfg = make_case(case)
    ref, dev, stats = run_trajectory(cfg, steps, two_pass=(two_pass is True), packed=packed,
                                     warm_state=(case in ("odd", "w1")), deferred=(two_pass == "deferred"))
    x_ref = ref.t["x"][:ref.N].astype(np.float64)
    x_gpu = dev.get("x")[:ref.N].astype(np.float64)
    rel = np.linalg.norm(x_gpu - x_ref) / np.linalg.norm(x_ref)
    print(f"{case}: {steps} steps, relative L2 error of x = {rel:.3e}, {stats}")
    assert rel <= 1e-4
    if stats["scale_ulp_steps"] == 0:
        for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev"):
            assert np.array_equal(dev.get(k), ref.t[k]), k
    else:
        for k in ("x", "m", "v_fresh", "r_prev"):
            assert_close(dev.get(k), ref.t[k], k, rel=1e-4)
    finish(dev)


@pytest.mark.parametrize("case,path", [
    ("odd", "single"), ("bert_mini", "single"), ("small", "single"), ("tiny", "single"), ("w1", "single"),
    ("bert_mini", "two_pass"), ("tiny", "two_pass"),
    ("bert_mini", 1), ("tiny", 7)])      # layers over that many tiles of 8192 take two passes
@pytest.mark.parametrize("wd", [0.0, 0.01])
def test_warmup_and_freeze(case, path, wd):
    """eq. (1) with the moving average of c, then the end-of-warmup snapshot.  path: the single-pass
    kernel with a per-layer barrier for every layer that qualifies (the default), two passes for
    every layer, or a lowered size limit so that both run side by side."""
    _need_gpu()
    import paper_2104_06069_amd as ob
    cfg = make_case(case)
    st = Streams(3)
    pl = cfg["plist"]
    hyper = dict(HYPER); hyper["weight_decay"] = wd
    if wd == 0.0:
        # with these inputs ||x||/||u|| is about 0.006, below the paper's c_min: lower the bound so that
        # the coefficient is the ratio of the two norms itself and not the clip's bound (checked below);
        # the wd = 0.01 cases keep the paper's bounds and run clipped
        hyper["c_min"] = 1e-4
    ref = RefStep(pl.offsets, cfg["W"], cfg["server_chunk"], **hyper)
    dev = DeviceStep(pl.offsets, cfg["W"], cfg["server_chunk"], two_pass_warmup=(path == "two_pass"),
                     fused_max_tiles=(path if isinstance(path, int) else None), **hyper)
    nf = ob.ob_lamb_warmup_fused_layers(dev.ctx)
    assert nf == {("tiny", "single"): 4, ("tiny", 7): 0, ("bert_mini", "two_pass"): 0,
                  ("tiny", "two_pass"): 0, ("small", "single"): 0}.get((case, path), nf)
    if (case, path) == ("bert_mini", "single"):
        assert nf >= 2
    if (case, path) == ("tiny", "single"):
        assert ob.ob_lamb_warmup_fused_params(dev.ctx) == 4 * 262144
    if (case, path) == ("bert_mini", 1):
        assert 1 <= nf
    s = init_state(st, cfg)
    s["v_fresh"][...] = 0
    s["c_avg"][...] = 0
    ref.load_state(s); dev.load_state(ref.t)
    for t in range(5):
        g = gradient(st, cfg, t)
        ref.warmup_step(g, 1e-3 * (t + 1))
        dev.warmup_step(torch.from_numpy(g).to(dev.device), 1e-3 * (t + 1))
        for k in ("m", "v_fresh", "x", "coeff_c", "c_avg"):
            assert_close(dev.get(k), ref.t[k], f"step {t}: {k}")
        if wd == 0.0:
            c = ref.t["coeff_c"][np.diff(pl.offsets) > 0]
            assert ((c > hyper["c_min"]) & (c < hyper["c_max"])).mean() > 0.5, "most coefficients should be unclipped"
    ref.freeze(); dev.freeze()
    assert np.array_equal(dev.get("v_frozen"), dev.get("v_fresh"))
    assert np.all(dev.get("r_prev") == 1.0)
    assert_close(dev.get("v_frozen"), ref.t["v_frozen"], "v_frozen")
    # first compression step after the hand-off
    g = gradient(st, cfg, 99)
    fw, fs = foreign_worker_chunks(st, cfg, 0); fa, fss = foreign_server_chunks(st, cfg, 0)
    ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
    push_wire(ref, dev)
    ref.step(g, 1e-3); dev.step(torch.from_numpy(g).to(dev.device), 1e-3)
    assert np.array_equal(words_of(dev.packed_local), ref.bits_local)
    for k in ("x", "m", "v_fresh", "r_prev", "coeff_c"):
        assert_close(dev.get(k), ref.t[k], k)
    finish(dev)


@pytest.mark.parametrize("packed,fused", [(False, False), (True, True)])
def test_previous_ratio_outside_its_bounds(packed, fused):
    """Algorithm 1 applies line 18 (the window around the previous ratio) before line 19 (r_min,
    r_max); the order shows when a loaded r_prev lies outside [r_min, r_max], and when it is not 1
    the window is a factor, not a distance.  Two steps from previous ratios between 0.05 and 20."""
    _need_gpu()
    cfg = make_case("bert_mini")
    st, ref, dev = start_pair(cfg, warm_state=True, packed=packed, fused=fused)
    r0 = np.exp(np.random.default_rng(3).uniform(np.log(0.05), np.log(20.0), ref.L)).astype(np.float32)
    assert (r0 < HYPER["r_min"]).sum() >= 3 and (r0 > HYPER["r_max"]).sum() >= 3
    ref.t["r_prev"][...] = r0
    sync_dev_from_ref(ref, dev)
    for t in range(2):
        g = gradient(st, cfg, t)
        fw, fs = foreign_worker_chunks(st, cfg, t); fa, fss = foreign_server_chunks(st, cfg, t)
        ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
        if t:
            dev.begin_step()
        push_wire(ref, dev)
        ref.step(g, 1e-3); dev.step(torch.from_numpy(g).to(dev.device), 1e-3)
        for k in ("r_prev", "coeff_c", "x", "v_fresh"):
            assert_close(dev.get(k), ref.t[k], f"step {t}: {k}")
        r = dev.get("r_prev")
        assert np.all(r >= HYPER["r_min"]) and np.all(r <= HYPER["r_max"])
    finish(dev)


@pytest.mark.parametrize("case,packed,fused", [("odd", False, False), ("tiny", True, True),
                                               ("bert_mini", True, True), ("bert_mini", False, True)])
def test_degenerate_values(case, packed, fused):
    """Zero chunks, NaN/Inf gradients, zero fresh variance, near-zero layers: IEEE behaviour of the
    device matches the oracle's -- in the plain kernels and in the ones with in-kernel barriers."""
    _need_gpu()
    cfg = make_case(case)
    st, ref, dev = start_pair(cfg, warm_state=False, packed=packed, fused=fused)
    N = ref.N
    # step 0: all-zero gradient and momentum -> every scale is 0, every bit is 1
    g = np.zeros(cfg["n_pad"], np.float32)
    fw, fs = foreign_worker_chunks(st, cfg, 0); fa, fss = foreign_server_chunks(st, cfg, 0)
    fs[...] = 0
    ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss); push_wire(ref, dev)
    ref.step(g, 1e-3); dev.step(torch.from_numpy(g).to(dev.device), 1e-3)
    assert np.all(ref.scales_local == 0) and np.all(ref.bits_local == 0xFF)
    assert np.array_equal(words_of(dev.packed_local), ref.bits_local)
    assert np.array_equal(words_of(dev.packed_all), ref.bits_all)
    for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev"):
        assert_close(dev.get(k), ref.t[k], k)
    # step 1: NaN and +-Inf in the gradient, zero fresh variance on some elements, a layer whose
    # frozen variance is 0 as well (0/0), gradients of 1e-9 on one layer
    g = gradient(st, cfg, 1)
    g[5] = np.nan; g[4200] = np.inf; g[4300] = -np.inf
    g[9000:9100] *= 1e-6
    ref.t["v_fresh"][10:20] = 0; ref.t["m"][10:20] = 0
    ref.t["v_fresh"][0] = 0; ref.t["v_frozen"][0] = 0
    ref.t["v_frozen"][30] = np.nan; ref.t["v_frozen"][31] = np.inf   # NaN skipped by the max; Inf clipped
    sync_dev_from_ref(ref, dev)
    fw, fs = foreign_worker_chunks(st, cfg, 1); fa, fss = foreign_server_chunks(st, cfg, 1)
    ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss); push_wire(ref, dev)
    ref.step(g, 1e-3); dev.step(torch.from_numpy(g).to(dev.device), 1e-3)
    assert np.array_equal(words_of(dev.packed_local), ref.bits_local)
    assert np.array_equal(words_of(dev.packed_all), ref.bits_all)
    assert_close(dev.scales_local.cpu().numpy(), ref.scales_local, "scales with NaN/Inf")
    for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c"):
        assert_close(dev.get(k), ref.t[k], k)
    assert np.all(np.isfinite(dev.get("r_prev")))
    # step 2 (with the 1-bit momentum this is the step that runs the kernel with the per-layer
    # barrier): the variances now hold NaN, Inf and 0 from step 1; one more Inf in the gradient
    g = gradient(st, cfg, 2)
    g[77] = np.inf
    fw, fs = foreign_worker_chunks(st, cfg, 2); fa, fss = foreign_server_chunks(st, cfg, 2)
    ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
    dev.begin_step()
    push_wire(ref, dev)
    ref.step(g, 1e-3); dev.step(torch.from_numpy(g).to(dev.device), 1e-3)
    assert np.array_equal(words_of(dev.packed_local), ref.bits_local)
    assert np.array_equal(words_of(dev.packed_all), ref.bits_all)
    for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c"):
        assert_close(dev.get(k), ref.t[k], k)
    assert np.all(np.isfinite(dev.get("r_prev")))
    finish(dev)


@pytest.mark.parametrize("case,packed,fused", [("bert_mini", False, False), ("bert_mini", True, True),
                                               ("tiny", True, True)])
def test_bitwise_reproducible(case, packed, fused):
    """Same inputs twice -> identical bits everywhere (fixed-order reductions, no float atomics; in
    the kernels with barriers the order of arrival does not enter the result).  Two steps, so that
    the second one runs the single-pass ratio+update kernel when the momentum is in 1-bit form."""
    _need_gpu()
    cfg = make_case(case)
    outs = []
    for _ in range(2):
        st, ref, dev = start_pair(cfg, packed=packed, fused=fused)
        for t in range(2):
            g = torch.from_numpy(gradient(st, cfg, t)).to(dev.device)
            fw, fs = foreign_worker_chunks(st, cfg, t); fa, fss = foreign_server_chunks(st, cfg, t)
            ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
            dev.begin_step()
            push_wire(ref, dev)
            dev.step(g, 1e-3)
        outs.append({k: dev.get(k).copy() for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev")}
                    | {"scales": dev.scales_local.cpu().numpy(), "w": words_of(dev.packed_local).copy()})
        finish(dev)
    for k in outs[0]:
        assert np.array_equal(outs[0][k], outs[1][k], equal_nan=True) if outs[0][k].dtype.kind == "f" \
            else np.array_equal(outs[0][k], outs[1][k]), k


def test_argument_errors():
    """Host-side validation: nothing is enqueued and a negative status comes back."""
    _need_gpu()
    import paper_2104_06069_amd as ob
    cfg = make_case("small")
    st, ref, dev = start_pair(cfg)
    g = torch.zeros(cfg["n_pad"], device=dev.device)
    state = dev._state("read")
    x0 = dev.get("x").copy()
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_compress_local(dev.ctx, state, None, dev.packed_local, dev.scales_local)
    assert e.value.status == -1
    with pytest.raises(ob.ObLambError) as e:   # misaligned gradient pointer
        ob.ob_lamb_compress_local(dev.ctx, state, g[1:], dev.packed_local, dev.scales_local)
    assert e.value.status == -3
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_decompress_apply(dev.ctx, state, dev.packed_all, dev.server_scales, float("nan"))
    assert e.value.status == -2
    # no momentum source at all / 1-bit momentum aliased with the output buffer
    nom = ob.make_state(**dict(dev.t, m=None))
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_compress_local(dev.ctx, nom, g, dev.packed_local, dev.scales_local)
    assert e.value.status == -1
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_decompress_apply(dev.ctx, nom, dev.packed_all, dev.server_scales, 1e-3)
    assert e.value.status == -1
    alias = ob.make_state(**dict(dev.t, m=None, m_packed=dev.packed_local, m_scales=dev.scales_local))
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_compress_local(dev.ctx, alias, g, dev.packed_local, dev.scales_local)
    assert e.value.status == -2
    # the second destination of the rank's own chunk: both pointers or neither
    half = ob.make_state(**dict(dev.t, own_packed_in=dev.packed_in))
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_compress_local(dev.ctx, half, g, dev.packed_local, dev.scales_local)
    assert e.value.status == -1
    # the variance in deferred form: needs the 1-bit momentum; history within its limit, complete, aligned
    with pytest.raises(ob.ObLambError) as e:   # dense momentum
        ob.ob_lamb_ratios_apply_hist(dev.ctx, state, dev.packed_all, dev.server_scales, 1e-3, None)
    assert e.value.status == -2
    other = torch.zeros_like(dev.packed_all); other_s = torch.ones_like(dev.server_scales)
    bits1 = ob.make_state(**dict(dev.t, m=None, m_packed=other, m_scales=other_s))
    too_long = ob.make_vf_history([], [], False); too_long.n_old = ob.OB_VF_MAX_OLD + 1
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_ratios_apply_hist(dev.ctx, bits1, dev.packed_all, dev.server_scales, 1e-3, too_long)
    assert e.value.status == -2
    missing = ob.make_vf_history([other], [other_s], False); missing.scales[0] = None
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_ratios_apply_hist(dev.ctx, bits1, dev.packed_all, dev.server_scales, 1e-3, missing)
    assert e.value.status == -1
    odd = ob.make_vf_history([other[1:]], [other_s], False)
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_variance_dense(dev.ctx, bits1, dev.packed_all, dev.server_scales, odd, torch.empty_like(dev.t["x"]))
    assert e.value.status == -3
    with pytest.raises(ob.ObLambError) as e:   # the previous momentum aliased with the new one
        ob.ob_lamb_ratios_apply_hist(dev.ctx, ob.make_state(**dict(dev.t, m=None, m_packed=dev.packed_all,
                                                                   m_scales=dev.server_scales)),
                                     dev.packed_all, dev.server_scales, 1e-3, None)
    assert e.value.status == -2
    torch.cuda.synchronize()
    assert np.array_equal(dev.get("x"), x0)
    finish(dev)


@pytest.mark.parametrize("two_pass", [False, True], ids=["single_pass", "two_pass"])
@pytest.mark.parametrize("case", ["odd", "bert_mini"])
def test_own_chunk_written_into_the_server_input(case, two_pass):
    """ob_lamb_compress_local with ob_lamb_state.own_packed_in / own_scale_in: the served chunk of the
    worker output lands in its slot of the server's input as well (what the exchange's copy of the
    rank's own data would do), and nothing else of that buffer is touched."""
    _need_gpu()
    cfg = make_case(case)
    st, ref, dev = start_pair(cfg, two_pass=two_pass)
    assert dev.fold_gather
    g = gradient(st, cfg, 0)
    fw, fs = foreign_worker_chunks(st, cfg, 0)
    dev.packed_in.copy_(torch.from_numpy(np.ascontiguousarray(fw).view(np.int32)))
    dev.scales_in.copy_(torch.from_numpy(fs))
    ref.set_foreign_in(fw, fs)
    ref.compress_local(g); ref.gather()
    dev.compress_local(torch.from_numpy(g).to(dev.device)); dev.gather()
    assert np.array_equal(words_of(dev.packed_in), ref.bits_in)
    assert np.array_equal(dev.scales_in.cpu().numpy(), ref.scales_in)
    assert np.array_equal(words_of(dev.packed_local), ref.bits_local)
    finish(dev)


@pytest.mark.parametrize("case", ["odd", "bert_mini"])
def test_momentum_scale_generation(case):
    """Appendix A.5.2 coefficients from the momentum at the end of warmup."""
    _need_gpu()
    cfg = make_case(case)
    cfg["use_k"] = False
    st, ref, dev = start_pair(cfg)
    # momentum with very different scales per layer (the case A.5.2 describes), one all-zero layer
    m = st.normal("m_ms", 0, cfg["n_pad"], 1.0)
    off = cfg["plist"].offsets
    kap = st.uniform_host("kap_ms", 0, cfg["plist"].L, -6, 0)
    for l in range(cfg["plist"].L):
        m[off[l]:off[l + 1]] *= np.float32(10.0 ** kap[l])
    m[off[1]:off[2]] = 0
    m[cfg["plist"].N:] = 0
    ref.t["m"][...] = m
    dev.load_state(ref.t)
    ref.momentum_scale(); dev.momentum_scale()
    k_gpu = dev.t["mom_scale"].cpu().numpy()
    assert_close(k_gpu, ref.mom_scale, "mom_scale")
    assert k_gpu[1] == 1.0
    finish(dev)


@pytest.mark.parametrize("case,packed", [("bert_mini", True), ("odd", False)])
def test_two_stage_schedule(case, packed):
    """Algorithm 1 end to end: LAMB warmup with the moving average of c, the end-of-warmup snapshot
    and momentum-scale generation, then compression-stage steps -- with the paper's warmup share
    (16.7 %) and the shape of its learning-rate schedule, scaled down to 48 steps."""
    _need_gpu()
    from workloads import lr_seqlen128
    cfg = make_case(case)
    T, T_w = 48, 8
    st = Streams(11)
    pl = cfg["plist"]
    hyper = dict(HYPER, c_min=1e-3)   # so that LAMB's coefficient is not clipped on every layer
    ref = RefStep(pl.offsets, cfg["W"], cfg["server_chunk"], **hyper)
    dev = DeviceStep(pl.offsets, cfg["W"], cfg["server_chunk"], packed_momentum=packed, **hyper)
    s = init_state(st, cfg)
    for k in ("v_fresh", "v_frozen", "c_avg"):
        s[k][...] = 0          # Algorithm 1 line 1: m = v = 0, c_avg = 0
    ref.load_state(s); dev.load_state(ref.t)
    for t in range(T):
        g = gradient(st, cfg, t)
        lr = lr_seqlen128(t, rampup=4, decay_every=10)
        fw, fs = foreign_worker_chunks(st, cfg, t); fa, fss = foreign_server_chunks(st, cfg, t)

        def fill_ref(r):
            r.set_foreign_in(fw, fs); r.set_foreign_all(fa, fss)

        def fill_dev(d):
            d.packed_in.copy_(torch.from_numpy(np.ascontiguousarray(fw).view(np.int32)))
            d.scales_in.copy_(torch.from_numpy(fs))
            d.packed_all.copy_(torch.from_numpy(np.ascontiguousarray(fa).view(np.int32)))
            d.server_scales.copy_(torch.from_numpy(fss))

        ref.train_step(t, T_w, g, lr, fill_ref)
        dev.train_step(t, T_w, torch.from_numpy(g).to(dev.device), lr, fill_dev)
        if t == T_w - 1:
            assert_close(dev.t["mom_scale"].cpu().numpy(), ref.mom_scale, "mom_scale at hand-off")
            assert np.array_equal(dev.get("v_frozen"), dev.get("v_fresh"))
            for k in ("c_avg", "m", "x", "v_fresh"):
                assert_close(dev.get(k), ref.t[k], f"hand-off {k}")
        if t >= T_w:
            assert np.array_equal(words_of(dev.packed_local), ref.bits_local), t
    for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c", "c_avg"):
        assert_close(dev.get(k), ref.t[k], k, rel=1e-5)
    r = dev.get("r_prev")
    assert np.all(r >= 0.5) and np.all(r <= 4.0)
    finish(dev)


@pytest.mark.parametrize("case,steps,packed,max_tiles", [
    ("bert_mini", 60, True, None),    # every layer in the fused kernel
    ("bert_mini", 60, False, None),   # ... with the fp32 momentum read and written in place
    ("bert_mini", 40, True, 2),       # layers over 2 tiles of 8192 go to the two-kernel path
    ("bert_mini", 40, False, 1),
    ("odd", 30, True, None),          # tiny tensors: every tile meets several layer boundaries
    ("odd", 30, False, 0),            # nothing eligible: plain kernels behind the fused entry point
    ("tiny", 10, True, None), ("w1", 10, True, 1), ("small", 10, False, None)])
def test_trajectory_fused_ratios_apply(case, steps, packed, max_tiles):
    """ob_lamb_ratios_apply (ratio pass, clips and update in one call, one kernel where the layer
    fits on the device) against the oracle's separate phases."""
    _need_gpu()
    import paper_2104_06069_amd as ob
    cfg = make_case(case)
    ref, dev, stats = run_trajectory(cfg, steps, packed=packed, warm_state=(case in ("odd", "w1")),
                                     fused=True, fused_max_tiles=max_tiles)
    nf = ob.ob_lamb_fused_layers(dev.ctx)
    print(f"{case}: {nf} of {cfg['plist'].L} layers in the fused kernel, {stats}")
    if max_tiles == 0 or case in ("odd", "small", "w1"):   # no eligible layer holds a whole tile
        assert nf == 0
    else:
        assert 0 < nf <= cfg["plist"].L
    assert stats["scale_ulp_steps"] == 0 and stats["word_mismatch_steps"] == 0
    for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c"):
        assert np.array_equal(dev.get(k), ref.t[k]), k
    finish(dev)


@pytest.mark.parametrize("case,fused,packed,one_adam", [
    ("bert_mini", False, False, False), ("bert_mini", True, True, False), ("odd", True, True, False),
    ("one_layer", False, False, True), ("one_layer", True, True, True)])
def test_degenerate_variants(case, fused, packed, one_adam):
    """The method's relatives as settings of the same step (Section 3.4 / Appendix A.4): r pinned
    to 1 freezes c at its warmup average ("LAMB + basic 1-bit"); one layer with c_avg = 1 is the
    compression stage of 1-bit Adam."""
    _need_gpu()
    cfg = make_case(case)
    ref, dev, stats = run_trajectory(cfg, 20, packed=packed, fused=fused, warm_state=True,
                                     hyper=dict(r_min=1.0, r_max=1.0),
                                     c_avg=(1.0 if one_adam else None))
    assert stats["scale_ulp_steps"] == 0
    assert np.all(dev.get("r_prev") == 1.0)
    assert np.array_equal(dev.get("coeff_c"), ref.t["c_avg"])
    for k in ("x", "m", "v_fresh", "err_worker", "err_server"):
        assert np.array_equal(dev.get(k), ref.t[k]), k
    finish(dev)


def _to_lp(g32, fmt):
    """Input generation for the mixed-precision variant: a 16-bit gradient tensor (torch's
    conversion) and its raw patterns for the oracle."""
    t = torch.from_numpy(g32).to({"f16": torch.float16, "bf16": torch.bfloat16}[fmt])
    return t, (1 if fmt == "f16" else 2, t.view(torch.int16).numpy().view(np.uint16).copy())


@pytest.mark.parametrize("case,gfmt,xfmt,fused,packed,scale,vperiod", [
    ("bert_mini", "f16", "f16", True, True, 1.0 / 1024, 0),
    ("bert_mini", "bf16", "bf16", True, True, 1.0, 0),
    ("bert_mini", "f16", "bf16", False, False, 1.0 / 1000, 0),   # scale not a power of two; separate calls
    ("odd", "bf16", "f16", True, True, 1.0 / 64, 0),
    ("odd", "f16", "f16", True, False, 1.0, 0),                 # fp32 momentum behind the fused entry point
    ("tiny", "f32", "f16", True, True, 1.0, 0),                 # only the 16-bit parameter copy
    ("small", "f16", None, False, True, 0.5, 0),                # only the 16-bit gradient
    ("w1", "bf16", "bf16", True, True, 1.0 / 8, 0),
    # with the variance in deferred form (ob_lamb_ratios_apply_hist_lp)
    ("bert_mini", "f16", "f16", True, True, 1.0 / 1024, 4),
    ("tiny", "bf16", "bf16", True, True, 1.0, 3),
    ("odd", "f32", "f16", True, True, 1.0, 2),
    ("big_and_small", "bf16", "bf16", True, True, 1.0 / 16, 4)])
def test_mixed_precision_variant(case, gfmt, xfmt, fused, packed, scale, vperiod):
    """16-bit gradient in (times the inverse loss scale), 16-bit copy of the parameters out, through
    3 LAMB steps, the snapshot and 12 compression steps; state and arithmetic stay fp32, so every
    comparison is as strict as for the fp32 entry points and the 16-bit copy is bit-exact."""
    _need_gpu()
    cfg = make_case(case)
    st = Streams(11)
    pl = cfg["plist"]
    ref = RefStep(pl.offsets, cfg["W"], cfg["server_chunk"], **HYPER)
    ref.grad_scale = scale
    tdt = {None: None, "f16": torch.float16, "bf16": torch.bfloat16}[xfmt]
    dev = DeviceStep(pl.offsets, cfg["W"], cfg["server_chunk"], packed_momentum=packed, fused_apply=fused,
                     x_lp_dtype=tdt, grad_scale=scale, deferred_variance=vperiod, **HYPER)
    s = init_state(st, cfg)
    s["v_fresh"][...] = 0
    s["c_avg"][...] = 0
    # parameters whose 16-bit copy overflows, lands on the largest finite value or is subnormal
    # (binary16: max 65504, ties at 65520, subnormals below 6.1e-5; bfloat16: max 3.39e38)
    special = [7e4, 65519.0, 65520.0, -65536.0, -1e-7, 3e-8, 3.39e38, -3.4e38, 1e-40]
    i0 = int(np.argmax(np.diff(pl.offsets) >= len(special)))      # the first tensor that can hold them
    s["x"][pl.offsets[i0]:pl.offsets[i0] + len(special)] = np.array(special, np.float32)
    ref.load_state(s)
    dev.load_state(ref.t)
    N = ref.N
    T_w, T = 3, 15

    def check_x_lp(t):
        """Where the fp32 parameters agree bit for bit (everywhere, but for a last-bit difference of
        a layer's coefficient after an fp64 reduction), the 16-bit copy must agree bit for bit."""
        if xfmt is None:
            return
        got = dev.x_lp.view(torch.int16).cpu().numpy().view(np.uint16)
        want = ref.x_lp(1 if xfmt == "f16" else 2)
        same = dev.get("x")[:N].view(np.uint32) == ref.t["x"][:N].view(np.uint32)
        assert same.mean() >= 0.9, f"step {t}: fp32 parameters differ in {(~same).sum()} places"
        assert np.array_equal(got[:N][same], want[:N][same]), f"step {t}: 16-bit parameter copy"
        assert np.all(got[N:] == 0), "padding of the 16-bit copy was written"

    for t in range(T):
        g32 = (gradient(st, cfg, t) / np.float32(scale)).astype(np.float32)
        if gfmt == "f32":
            assert scale == 1.0
            gd, gr = torch.from_numpy(g32), g32
        else:
            gd, gr = _to_lp(g32, gfmt)
        gd = gd.to(dev.device)
        lr = 1e-3 * (1 + t % 3)
        if t < T_w:
            ref.warmup_step(gr, lr)
            dev.warmup_step(gd, lr)
            for k in ("x", "m", "v_fresh", "c_avg"):
                assert_close(dev.get(k), ref.t[k], f"warmup step {t} {k}")
            check_x_lp(t)
            if t == T_w - 1:
                ref.freeze(); dev.freeze()
                assert np.array_equal(dev.get("v_frozen"), dev.get("v_fresh"))
                dev.load_state(ref.t)   # the compression stage starts from identical bits
            continue
        fw, fs = foreign_worker_chunks(st, cfg, t)
        fa, fss = foreign_server_chunks(st, cfg, t)
        ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
        dev.begin_step()
        dev.packed_in.copy_(torch.from_numpy(np.ascontiguousarray(fw).view(np.int32)))
        dev.scales_in.copy_(torch.from_numpy(fs))
        dev.packed_all.copy_(torch.from_numpy(np.ascontiguousarray(fa).view(np.int32)))
        dev.server_scales.copy_(torch.from_numpy(fss))
        ref.step(gr, lr)
        dev.step(gd, lr)
        assert np.array_equal(words_of(dev.packed_local), ref.bits_local), f"step {t}: worker sign words"
        assert np.array_equal(words_of(dev.packed_all), ref.bits_all), f"step {t}: server sign words"
        for k in ("x", "v_fresh", "err_worker", "err_server", "r_prev"):
            assert_close(dev.get(k), ref.t[k], f"step {t} {k}")
        check_x_lp(t)
    if vperiod:
        assert set(dev.vf_ages) == set(range(1, vperiod + 1)), dev.vf_ages
    finish(dev)


def test_mixed_precision_argument_errors():
    _need_gpu()
    import paper_2104_06069_amd as ob
    cfg = make_case("small")
    pl = cfg["plist"]
    dev = DeviceStep(pl.offsets, cfg["W"], cfg["server_chunk"], **HYPER)
    g = torch.zeros(dev.n_pad, device=dev.device)
    g16 = g.to(torch.float16)
    stt = dev._state("read")
    def status(fn, *a):
        with pytest.raises(ob.ObLambError) as e:
            fn(dev.ctx, stt, *a)
        return e.value.status
    # fp32 gradient with a scale, unknown dtype, non-finite scale, misaligned pointer
    assert status(ob.ob_lamb_compress_local_lp, g, ob.OB_F32, 0.5, dev.packed_local, dev.scales_local) == -2
    assert status(ob.ob_lamb_compress_local_lp, g16, 7, 1.0, dev.packed_local, dev.scales_local) == -2
    assert status(ob.ob_lamb_compress_local_lp, g16, ob.OB_F16, float("inf"), dev.packed_local, dev.scales_local) == -2
    assert status(ob.ob_lamb_compress_local_lp, g16.data_ptr() + 2, ob.OB_F16, 1.0, dev.packed_local, dev.scales_local) == -3
    # 16-bit parameter copy declared as fp32, misaligned
    assert status(ob.ob_lamb_ratios_apply_lp, dev.packed_all, dev.server_scales, 1e-3, g16, ob.OB_F32) == -2
    assert status(ob.ob_lamb_decompress_apply_lp, dev.packed_all, dev.server_scales, 1e-3, g16.data_ptr() + 2, ob.OB_BF16) == -3
    assert status(ob.ob_lamb_warmup_step_lp, g16, ob.OB_F16, 1.0, 1e-3, g16, 5) == -2
    assert status(ob.ob_lamb_ratios_apply_hist_lp, dev.packed_all, dev.server_scales, 1e-3, None, g16, ob.OB_F32) == -2
    assert status(ob.ob_lamb_ratios_apply_hist_lp, dev.packed_all, dev.server_scales, 1e-3, None,
                  g16.data_ptr() + 2, ob.OB_F16) == -3
    finish(dev)


@pytest.mark.parametrize("which", ["compress", "ratios_apply", "ratios_apply_hist", "warmup"])
def test_expired_wait_is_reported_and_recovered(which):
    """The in-kernel barriers wait a bounded number of polls.  With the bound forced to 0 from the
    host every waiting workgroup gives up without polling, raises the device flag and runs to
    its end (nothing hangs, all accesses stay in bounds).  ob_lamb_check_device_status must report
    that once, switch the context to the barrier-free kernels, and the next steps -- from a restored
    state -- must again agree with the oracle."""
    _need_gpu()
    import paper_2104_06069_amd as ob
    cfg = make_case("tiny")       # 16 tiles of 16384 per chunk, 32 tiles of 8192 per layer
    st = Streams(5)
    pl = cfg["plist"]
    ref = RefStep(pl.offsets, cfg["W"], cfg["server_chunk"], **HYPER)
    # "ratios_apply": the worker compression runs as two passes, so only the per-layer barrier trips
    # "ratios_apply_hist": the same with the variance in deferred form (its own kernel)
    dev = DeviceStep(pl.offsets, cfg["W"], cfg["server_chunk"], two_pass=which.startswith("ratios_apply"),
                     packed_momentum=True, fused_apply=True, spin_limit=0,
                     deferred_variance=(3 if which == "ratios_apply_hist" else 0), **HYPER)
    assert ob.ob_lamb_fused_layers(dev.ctx) == pl.L
    ref.load_state(init_state(st, cfg))
    dev.load_state(ref.t)

    def one_step(t, check):
        g = gradient(st, cfg, t)
        fw, fs = foreign_worker_chunks(st, cfg, t)
        fa, fss = foreign_server_chunks(st, cfg, t)
        ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
        dev.begin_step()
        dev.packed_in.copy_(torch.from_numpy(np.ascontiguousarray(fw).view(np.int32)))
        dev.scales_in.copy_(torch.from_numpy(fs))
        dev.packed_all.copy_(torch.from_numpy(np.ascontiguousarray(fa).view(np.int32)))
        dev.server_scales.copy_(torch.from_numpy(fss))
        ref.step(g, 1e-3)
        dev.step(torch.from_numpy(g).to(dev.device), 1e-3)
        if check:
            assert np.array_equal(words_of(dev.packed_local), ref.bits_local)
            for k in ("x", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c"):
                assert_close(dev.get(k), ref.t[k], f"step {t} {k}")

    if which == "warmup":
        assert ob.ob_lamb_warmup_fused_layers(dev.ctx) == pl.L
        dev.warmup_step(torch.from_numpy(gradient(st, cfg, 0)).to(dev.device), 1e-3)
    # the first step reads the fp32 momentum (two plain kernels behind ratios_apply), the second one
    # runs the kernel with the per-layer barrier
    for t in range({"compress": 1, "ratios_apply": 2, "ratios_apply_hist": 2, "warmup": 0}[which]):
        one_step(t, check=False)
    with pytest.raises(ob.ObLambError) as e:
        ob.ob_lamb_check_device_status(dev.ctx, dev.stream)
    assert e.value.status == -4
    assert ob.ob_lamb_uses_single_pass(dev.ctx) == 0 and ob.ob_lamb_fused_layers(dev.ctx) == 0
    assert ob.ob_lamb_server_single_pass(dev.ctx) == 0
    assert ob.ob_lamb_warmup_fused_layers(dev.ctx) == 0
    ob.ob_lamb_check_device_status(dev.ctx, dev.stream)      # reported once; the context is usable again
    if which == "warmup":   # the two-pass form now: two LAMB steps against the oracle, then the snapshot
        dev.load_state(ref.t)
        for t in range(2):
            g = gradient(st, cfg, 50 + t)
            ref.warmup_step(g, 1e-3)
            dev.warmup_step(torch.from_numpy(g).to(dev.device), 1e-3)
            for k in ("m", "v_fresh", "x", "coeff_c", "c_avg"):
                assert_close(dev.get(k), ref.t[k], f"warmup after recovery, step {t}: {k}")
        ref.freeze(); dev.freeze()
    # restore the state the failed step(s) clobbered, then go on
    dev.load_state(ref.t)
    dev.m_is_packed = False
    for t in range(2, 6):
        one_step(t, check=True)
    finish(dev)


@pytest.mark.parametrize("packed,fused,use_k", [(False, False, False), (True, True, True)])
def test_gpu_rank_inside_a_simulated_job(packed, fused, use_k):
    """The device plays ONE rank (worker r and server of chunk r) of a W-rank data-parallel job whose
    other ranks are oracle instances with their own gradients and error buffers (Section 5: every
    rank compresses its own momentum, chunk c of all ranks meets at server c, every rank applies the
    same recompressed momentum).  What the device sends must equal what the oracle rank r would send,
    and its parameters must stay identical to those of the other ranks."""
    _need_gpu()
    W, r = 4, 2
    pl = ParamList("job", [(f"t{i}", s) for i, s in enumerate([5000, 3, 20000, 777, 9000])])
    n_pad = padded_len(pl.N, W)
    n_c = n_pad // W
    cfg = dict(name="job", plist=pl, W=W, n_pad=n_pad, n_c=n_c, grad="student_t3")
    st = Streams(21)
    k = st.uniform_host("mom_scale", 0, pl.L, 0.25, 4.0) if use_k else None
    s0 = init_state(st, cfg)
    # one oracle rank per worker; rank w also holds the server error of chunk w
    ranks = [RefStep(pl.offsets, W, w, mom_scale=k, **HYPER) for w in range(W)]
    for w, rk in enumerate(ranks):
        rk.load_state(s0)
    dev = DeviceStep(pl.offsets, W, r, mom_scale=k, packed_momentum=packed, fused_apply=fused, **HYPER)
    dev.load_state(ranks[r].t)
    wb = n_c // 8
    for t in range(12):
        lr = 1e-3 * (1 + t % 3)
        grads = [gradient(st, cfg, t, stream=f"grad_rank{w}") for w in range(W)]
        # --- oracle job: every worker compresses, every server reduces its chunk
        for w, rk in enumerate(ranks):
            rk.compress_local(grads[w])
        for c, rk in enumerate(ranks):
            for w in range(W):
                rk.bits_in[w * wb:(w + 1) * wb] = ranks[w].bits_local[c * wb:(c + 1) * wb]
                rk.scales_in[w] = ranks[w].scales_local[c]
            rk.server_reduce()
        bits_all = np.concatenate([ranks[c].bits_all[c * wb:(c + 1) * wb] for c in range(W)])
        sscales = np.array([ranks[c].server_scales[c] for c in range(W)], np.float32)
        for rk in ranks:
            rk.bits_all[...] = bits_all
            rk.server_scales[...] = sscales
            rk.layer_ratios()
            rk.decompress_apply(lr)
        # --- the device as rank r: its own gradient, the peers' chunks r, the peers' server outputs
        dev.begin_step()
        dev.packed_in.copy_(torch.from_numpy(ranks[r].bits_in.view(np.int32)))   # the all-to-all's result ...
        dev.scales_in.copy_(torch.from_numpy(ranks[r].scales_in))
        dev.packed_in[r * (n_c // 32):(r + 1) * (n_c // 32)].zero_()             # ... own slot comes from the device
        dev.scales_in[r] = 0.0                                                   #     (compress_local / gather())
        dev.compress_local(torch.from_numpy(grads[r]).to(dev.device))
        assert np.array_equal(words_of(dev.packed_local), ranks[r].bits_local), f"step {t}: what rank r sends"
        assert_close(dev.scales_local.cpu().numpy(), ranks[r].scales_local, "worker scales")
        dev.gather()
        dev.packed_all.copy_(torch.from_numpy(bits_all.view(np.int32)))          # the all-gather's result ...
        dev.server_scales.copy_(torch.from_numpy(sscales))
        dev.packed_all[r * (n_c // 32):(r + 1) * (n_c // 32)].zero_()            # ... own slot from server_reduce()
        dev.server_scales[r] = 0.0
        dev.server_reduce()
        assert np.array_equal(words_of(dev.packed_all), bits_all), f"step {t}: recompressed momentum"
        assert_close(dev.server_scales.cpu().numpy(), sscales, "server scales")
        if fused:
            dev.ratios_apply(lr)
        else:
            dev.layer_ratios()
            dev.decompress_apply(lr)
        for key in ("x", "m", "v_fresh", "r_prev", "coeff_c", "err_worker", "err_server"):
            assert_close(dev.get(key), ranks[r].t[key], f"step {t} {key}")
        # every rank of the job holds the same parameters and momentum
        for rk in ranks:
            assert np.array_equal(rk.t["x"], ranks[0].t["x"]) and np.array_equal(rk.t["m"], ranks[0].t["m"])
    finish(dev)


@pytest.mark.parametrize("case,period", [("tiny", 0), ("bert_mini", 0), ("bert_mini", 2), ("tiny", 3), ("big_and_small", 2)])
def test_step_replayed_from_a_captured_graph(case, period):
    """The barriers of the single-pass kernels number their launches themselves, so a step needs
    nothing from the host that changes from call to call: as many consecutive steps as it takes for
    the buffers to be arranged as at the start (DeviceStep.graph_period: 2 with the 1-bit momentum,
    whose buffer pairs alternate; twice the variance's period with the variance in deferred form,
    whose history lives in a ring of that many buffers) are captured into one graph and replayed,
    with eager work and synchronisation between the replays; every replay is checked against the
    oracle."""
    _need_gpu()
    cfg = make_case(case)
    st, ref, dev = start_pair(cfg, warm_state=False, packed=True, fused=True, deferred=True,
                              deferred_variance=period, fused_max_tiles=(8 if case == "big_and_small" else None))
    P = dev.graph_period
    assert P == (2 * period if period else 2)
    n_pad = cfg["n_pad"]
    gbuf = [torch.zeros(n_pad, device=dev.device) for _ in range(P)]
    lr = 1e-3

    def wire(t):   # what the other ranks send at step t, into the pair that step t uses
        fw, fs = foreign_worker_chunks(st, cfg, t)
        fa, fss = foreign_server_chunks(st, cfg, t)
        ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
        return fw, fs, fa, fss

    # eager steps first: the momentum is then in 1-bit form and the pairs rotate regularly (an odd
    # number with the deferred variance, so that the capture starts in the middle of a history)
    n_eager = 3 if period else 2
    for t in range(n_eager):
        g = gradient(st, cfg, t)
        fw, fs, fa, fss = wire(t)
        dev.begin_step()
        push_wire(ref, dev)
        ref.step(g, lr); dev.step(torch.from_numpy(g).to(dev.device), lr)
    assert dev.m_is_packed
    torch.cuda.synchronize()
    # foreign input of the captured steps lives in fixed device buffers, refilled before each replay
    fin = [dict(pi=torch.zeros_like(dev.packed_in), si=torch.zeros_like(dev.scales_in),
                pa=torch.zeros_like(dev.packed_all), sa=torch.zeros_like(dev.server_scales)) for _ in range(P)]

    def group_of_steps():
        for j in range(P):
            dev.begin_step()
            dev.packed_in.copy_(fin[j]["pi"]); dev.scales_in.copy_(fin[j]["si"])
            dev.packed_all.copy_(fin[j]["pa"]); dev.server_scales.copy_(fin[j]["sa"])
            dev.step(gbuf[j], lr)

    cur0, n_old0 = dev._cur, dev._vf_n_old
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        # capture only records the launches; the steps themselves first run at the first replay
        with torch.cuda.graph(graph, stream=side):
            group_of_steps()
    torch.cuda.current_stream().wait_stream(side)
    assert (dev._cur, dev._vf_n_old) == (cur0, n_old0)     # back to the starting arrangement
    for rep in range(3 if period else 4):
        for j in range(P):
            t = n_eager + P * rep + j
            g = gradient(st, cfg, t)
            fw, fs, fa, fss = wire(t)
            gbuf[j].copy_(torch.from_numpy(g))
            fin[j]["pi"].copy_(torch.from_numpy(np.ascontiguousarray(fw).view(np.int32)))
            fin[j]["si"].copy_(torch.from_numpy(fs))
            fin[j]["pa"].copy_(torch.from_numpy(np.ascontiguousarray(fa).view(np.int32)))
            fin[j]["sa"].copy_(torch.from_numpy(fss))
            ref.step(g, lr)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        # eager work of the same library between the replays (its own context: nothing shared)
        assert np.array_equal(words_of(dev.packed_local), ref.bits_local), f"replay {rep}: worker words"
        assert np.array_equal(words_of(dev.packed_all), ref.bits_all), f"replay {rep}: server words"
        for k in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c"):
            assert_close(dev.get(k), ref.t[k], f"replay {rep}: {k}")
    finish(dev)



@pytest.mark.parametrize("seed", list(range(16)))
def test_random_layer_lists(seed):
    """Random tensor lists -- empty, tiny, exactly tile-sized, tile-aligned and ragged tensors, random
    W and served chunk, with or without momentum scaling, random size limit of the barrier kernels
    -- through LAMB steps, the snapshot and compression steps in the benchmarked configuration.
    Exercises the host's tiling: which tiles the barrier kernels take, what is left to the plain
    kernels, chunk ends inside and between layers."""
    _need_gpu()
    import paper_2104_06069_amd as ob
    r = np.random.default_rng(1000 + seed)
    kinds = [0, 1, 2, 3, 7, 255, 256, 1023, 1024, 1025, 4096, 8191, 8192, 8193, 16384, 24576, 40000, 65536, 100000]
    sizes = [int(r.choice(kinds)) for _ in range(int(r.integers(3, 14)))]
    if sum(sizes) == 0:
        sizes.append(5000)
    W = int(r.choice([1, 2, 3, 4, 5, 8]))
    pl = ParamList(f"rand{seed}", [(f"t{i}", s) for i, s in enumerate(sizes)])
    n_pad = padded_len(pl.N, W)
    cfg = dict(name=f"rand{seed}", plist=pl, W=W, n_pad=n_pad, n_c=n_pad // W, grad="student_t3")
    c_srv = int(r.integers(0, W))
    use_k = bool(r.integers(0, 2))
    max_tiles = [None, None, 1, 2, 3][int(r.integers(0, 5))]
    st = Streams(seed)
    k = st.uniform_host("mom_scale", 0, pl.L, 0.25, 4.0) if use_k else None
    hyper = dict(HYPER, c_min=1e-3)
    ref = RefStep(pl.offsets, W, c_srv, mom_scale=k, **hyper)
    dev = DeviceStep(pl.offsets, W, c_srv, mom_scale=k, packed_momentum=True, fused_apply=True,
                     fused_max_tiles=max_tiles, deferred_error=bool(seed % 2), **hyper)
    assert (dev.N, dev.n_pad, dev.n_c) == (ref.N, ref.n_pad, ref.n_c)
    print(f"sizes {sizes} W {W} served {c_srv} k {use_k} max_tiles {max_tiles}: "
          f"{ob.ob_lamb_fused_layers(dev.ctx)} / {ob.ob_lamb_warmup_fused_layers(dev.ctx)} layers in the barrier kernels")
    s = init_state(st, cfg)
    s["v_fresh"][...] = 0
    s["c_avg"][...] = 0
    ref.load_state(s); dev.load_state(ref.t)
    for t in range(3):
        g = gradient(st, cfg, t)
        ref.warmup_step(g, 1e-3); dev.warmup_step(torch.from_numpy(g).to(dev.device), 1e-3)
        for key in ("m", "v_fresh", "x", "coeff_c", "c_avg"):
            assert_close(dev.get(key), ref.t[key], f"warmup {t} {key}")
    ref.freeze(); dev.freeze()
    dev.load_state(ref.t)     # identical bits at the hand-off
    for t in range(3, 8):
        g = gradient(st, cfg, t)
        fw, fs = foreign_worker_chunks(st, cfg, t); fa, fss = foreign_server_chunks(st, cfg, t)
        ref.set_foreign_in(fw, fs); ref.set_foreign_all(fa, fss)
        dev.begin_step()
        push_wire(ref, dev)
        ref.step(g, 1e-3); dev.step(torch.from_numpy(g).to(dev.device), 1e-3)
        assert np.array_equal(words_of(dev.packed_local), ref.bits_local), f"step {t}: worker words"
        assert np.array_equal(words_of(dev.packed_all), ref.bits_all), f"step {t}: server words"
        for key in ("x", "m", "v_fresh", "err_worker", "err_server", "r_prev", "coeff_c"):
            assert_close(dev.get(key), ref.t[key], f"step {t} {key}")
    finish(dev)


@pytest.mark.parametrize("form", ["single_pass", "two_pass", "deferred"])
def test_server_sum_order_and_single_division(form):
    """Inputs on which the binary32 server average depends on HOW it is formed: scales (2^24, 1, 1, 1)
    give 2^24 when the workers are added in the order 0..W-1 and 2^24 + 1 otherwise; scales
    (1, 2^-24, 2^-24) at W = 3 give fl(1/3) when the sum is divided once and two ulps more when every
    term is divided.  All sign bits are set and the carried error is 0, so every element of the
    average has that value and the recompressed scale equals it: compared bit for bit."""
    _need_gpu()
    from tests.refstep import F32
    for scales in ([2.0 ** 24, 1, 1, 1], [1, 1, 1, 2.0 ** 24], [1, 2.0 ** -24, 2.0 ** -24], [2.0 ** -24, 2.0 ** -24, 1]):
        W = len(scales)
        n_c = 2048
        pl = ParamList("srv", [("a", n_c * W)])
        dev = DeviceStep(pl.offsets, W, 0, two_pass=(form == "two_pass"), deferred_error=(form == "deferred"), **HYPER)
        assert dev.n_c == n_c
        sc = np.array(scales, np.float32)
        words = np.full(W * n_c // 8, 0xFF, np.uint8)
        err = np.zeros(n_c, np.float32)
        _, s_ref = F32.server_reduce(W, words, sc, err)
        dev.packed_in.copy_(torch.from_numpy(words.view(np.int32)))
        dev.scales_in.copy_(torch.from_numpy(sc))
        dev.server_reduce()
        torch.cuda.synchronize()
        s_dev = dev.server_scales.cpu().numpy()[0]
        assert np.float32(s_dev).view(np.uint32) == np.float32(s_ref).view(np.uint32), (scales, s_dev, s_ref)
        assert np.array_equal(dev.get("err_server").view(np.uint32), err.view(np.uint32)), scales
        finish(dev)


@pytest.mark.parametrize("n_c_target,W,expect", [
    (300_000, 3, 1), (2_500_000, 2, 2), (5_000_000, 2, 4), (8_000_000, 1, 0), (300_000, 3, "two_pass"),
    # fan-ins that are not multiples of the number of workers whose words are in flight together,
    # and one above the number of scales staged at a time
    (40_000, 203, 1), (2_500_000, 13, 2), (2_000, 1100, 1), (2_000, 1100, "two_pass")])
def test_server_reduce_forms(n_c_target, W, expect):
    """ob_lamb_server_reduce in each of its forms -- one kernel with a chunk barrier on tiles of
    1024, 2048 or 4096 elements (the smallest whose workgroups all fit on the device), three
    kernels when the chunk is too large for that or when asked for -- against the oracle, two
    calls in a row (the second starts from the first one's error buffer), ragged chunk end."""
    _need_gpu()
    import paper_2104_06069_amd as ob
    from tests.refstep import F32
    N = n_c_target * W - 777
    pl = ParamList("srv", [("a", N // 3), ("b", N - N // 3)])
    two_pass = expect == "two_pass"
    dev = DeviceStep(pl.offsets, W, W - 1, two_pass=two_pass, **HYPER)
    form = ob.ob_lamb_server_single_pass(dev.ctx)
    print(f"n_c {dev.n_c} W {W}: single-pass server kernel tile = {form} x 1024", flush=True)
    assert form == (0 if two_pass else expect)
    r = np.random.default_rng(n_c_target + W)
    err = (1e-4 * r.standard_normal(dev.n_c)).astype(np.float32)
    dev.t["err_server"].copy_(torch.from_numpy(err))
    for call in range(2):
        words = r.integers(0, 2 ** 32, size=W * dev.n_c // 32, dtype=np.uint64).astype(np.uint32)
        scales = (1e-4 * r.uniform(0.5, 1.5, W)).astype(np.float32)
        dev.packed_in.copy_(torch.from_numpy(words.view(np.int32)))
        dev.scales_in.copy_(torch.from_numpy(scales))
        bits_ref, s_ref = F32.server_reduce(W, words.view(np.uint8), scales, err)   # err updated in place
        dev.server_reduce()
        torch.cuda.synchronize()
        wpc = dev.n_c // 32
        got = words_of(dev.packed_all)[(W - 1) * wpc * 4:W * wpc * 4]
        assert np.array_equal(got, bits_ref), f"call {call}: recompressed sign words"
        assert_close(dev.server_scales.cpu().numpy()[W - 1:W], np.array([s_ref], np.float32), f"call {call}: scale")
        assert_close(dev.get("err_server"), err, f"call {call}: server error")
    finish(dev)
