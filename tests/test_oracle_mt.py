"""The oracle's multi-threaded drivers against its serial routines: bit-identical, whatever the
number of threads, on tensor lists with empty, tiny, ragged and chunk-straddling tensors.

The drivers only cut the problem into pieces (chunks, layers, element ranges) and run the serial
routines on them; these tests are what allows the GPU parity tests to use them for whole
trajectories at the benchmark sizes.  CPU only.
"""
import numpy as np
import pytest

from oracle.obref import Ref, default_threads, padded_len
from tests.refstep import HYPER, RefStep


def random_offsets(rng, L, N):
    """L layers over N elements: some empty, some of 1-2 elements, the rest ragged."""
    if L == 1:
        return np.array([0, N], np.int64)
    cuts = np.sort(rng.integers(0, N + 1, L - 1))
    for j in rng.choice(L - 1, size=max(1, L // 5), replace=False):   # empty and tiny layers
        if j + 1 < L - 1:
            cuts[j + 1] = min(N, cuts[j] + rng.integers(0, 3))
    cuts = np.sort(cuts)
    return np.concatenate([[0], cuts, [N]]).astype(np.int64)


def random_state(rng, ref):
    n, L = ref.n_pad, ref.L
    N = ref.N
    f = lambda s: (rng.standard_normal(n) * s).astype(np.float32)
    st = dict(x=f(0.02), m=f(1e-4), v_fresh=np.abs(f(1e-4)) + np.float32(1e-8), err_worker=f(5e-5),
              err_server=(rng.standard_normal(ref.n_c) * 5e-5).astype(np.float32),
              c_avg=rng.uniform(0.5, 2, L).astype(np.float32), r_prev=rng.uniform(0.6, 3, L).astype(np.float32))
    st["v_frozen"] = (st["v_fresh"] * rng.uniform(0.5, 2, n)).astype(np.float32)
    for k in ("x", "m", "v_fresh", "v_frozen"):
        st[k][N:] = 0
    return st


@pytest.mark.parametrize("seed,W,L,N,threads,with_k", [
    (0, 1, 1, 300, 2, False), (1, 4, 7, 5000, 3, True), (2, 8, 40, 70001, 8, True),
    (3, 16, 25, 16 * 256 * 3, 5, False), (4, 3, 12, 2000, 16, True), (5, 64, 9, 64 * 256 + 17, 4, False)])
def test_mt_equals_serial_over_a_trajectory(seed, W, L, N, threads, with_k):
    rng = np.random.default_rng(seed)
    off = random_offsets(rng, L, N)
    k = rng.uniform(0.25, 4, L).astype(np.float32) if with_k else None
    c = int(rng.integers(0, W))
    a = RefStep(off, W, c, mom_scale=k)
    b = RefStep(off, W, c, mom_scale=k, threads=threads)
    assert b.F.threads == threads and a.F.threads == 1
    st = random_state(rng, a)
    a.load_state(st); b.load_state(st)
    n = a.n_pad
    for t in range(4):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32); g[N:] = 0
        if t < 2:   # LAMB steps, the snapshot, coefficients formed from the momentum
            for r in (a, b):
                r.warmup_step(g, 1e-3)
            if t == 1:
                for r in (a, b):
                    r.freeze()
                    if with_k:
                        r.momentum_scale()
                if with_k:
                    assert np.array_equal(a.mom_scale, b.mom_scale)
        else:
            fw = rng.integers(0, 2 ** 32, W * (a.n_c // 32), dtype=np.uint32)
            fs = rng.uniform(5e-5, 1.5e-4, W).astype(np.float32)
            fa = rng.integers(0, 2 ** 32, n // 32, dtype=np.uint32)
            fss = rng.uniform(5e-5, 1.5e-4, W).astype(np.float32)
            for r in (a, b):
                r.set_foreign_in(fw, fs); r.set_foreign_all(fa, fss)
                r.step(g, 2e-3)
            assert np.array_equal(a.bits_local, b.bits_local)
            assert np.array_equal(a.scales_local.view(np.uint32), b.scales_local.view(np.uint32))
            assert np.array_equal(a.bits_all, b.bits_all)
            assert np.array_equal(a.server_scales.view(np.uint32), b.server_scales.view(np.uint32))
        for key in a.t:
            assert np.array_equal(a.t[key].view(np.uint32), b.t[key].view(np.uint32)), (t, key)


def test_mt_special_values_and_more_threads_than_pieces():
    """NaN, Inf and zero variances take the same route through both; 16 threads on 2 pieces."""
    rng = np.random.default_rng(11)
    off = np.array([0, 100, 100, 612], np.int64)
    a = RefStep(off, 2, 1)
    b = RefStep(off, 2, 1, threads=16)
    st = random_state(rng, a)
    st["v_fresh"][5] = 0; st["v_frozen"][5] = 0; st["v_frozen"][300] = np.inf; st["v_fresh"][301] = 0
    st["err_worker"][7] = np.nan
    a.load_state(st); b.load_state(st)
    g = (rng.standard_normal(a.n_pad) * 1e-3).astype(np.float32); g[a.N:] = 0
    g[9] = np.inf
    fw = rng.integers(0, 2 ** 32, 2 * (a.n_c // 32), dtype=np.uint32)
    fa = rng.integers(0, 2 ** 32, a.n_pad // 32, dtype=np.uint32)
    s2 = np.array([1e-4, 2e-4], np.float32)
    with np.errstate(all="ignore"):
        for r in (a, b):
            r.set_foreign_in(fw, s2); r.set_foreign_all(fa, s2)
            r.step(g, 1e-3)
    assert np.array_equal(a.bits_local, b.bits_local) and np.array_equal(a.bits_all, b.bits_all)
    for key in a.t:
        assert np.array_equal(a.t[key].view(np.uint32), b.t[key].view(np.uint32)), key


def test_default_threads_is_bounded():
    assert 1 <= default_threads() <= 16
    with pytest.raises(TypeError):
        Ref(np.float64, threads=2)
    assert padded_len(5, 2) == 512


@pytest.mark.parametrize("c0,c1,c_srv,with_k", [(2, 5, 3, True), (0, 4, 6, False), (5, 8, 7, True)])
def test_window_oracle_equals_the_whole_oracle(c0, c1, c_srv, with_k):
    """The oracle restricted to a window of whole chunks (what the full-size GPU tests follow)
    against the oracle on the whole buffer: every chunk-local quantity on every element of the
    window, every per-layer quantity on the layers that lie wholly inside it, the server step when
    the served chunk lies inside -- bit for bit, over several steps."""
    from tests.refstep import WindowRef
    from workloads import make_config
    cfg = make_config("bert_mini")
    pl, W, n_c = cfg["plist"], cfg["W"], cfg["n_c"]
    rng = np.random.default_rng(c0 * 10 + c1)
    k = rng.uniform(0.25, 4, pl.L).astype(np.float32) if with_k else None
    whole = RefStep(pl.offsets, W, c_srv, mom_scale=k)
    whole.load_state(random_state(rng, whole))
    win = WindowRef(pl.offsets, W, n_c, c0, c1, c_srv, mom_scale=k, threads=3, **HYPER)
    assert win.layers.size >= 2 and win.served == (c0 <= c_srv < c1)
    win.load(lambda key, A, B: whole.t[key] if A is None else whole.t[key][A:B])
    A, B = win.A, win.B
    for t in range(5):
        g = (rng.standard_normal(whole.n_pad) * 1e-3).astype(np.float32); g[whole.N:] = 0
        fw = rng.integers(0, 2 ** 32, W * (n_c // 32), dtype=np.uint32)
        fs = rng.uniform(5e-5, 1.5e-4, W).astype(np.float32)
        fa = rng.integers(0, 2 ** 32, whole.n_pad // 32, dtype=np.uint32)
        fss = rng.uniform(5e-5, 1.5e-4, W).astype(np.float32)
        whole.set_foreign_in(fw, fs); whole.set_foreign_all(fa, fss)
        whole.step(g, 2e-3)
        win.step(g[A:B], 2e-3, fa[A // 32:B // 32], fss[c0:c1], fw if win.served else None,
                 fs if win.served else None)
        assert np.array_equal(whole.bits_local[A // 8:B // 8], win.ref.bits_local)
        assert np.array_equal(whole.scales_local[c0:c1], win.ref.scales_local)
        for key in ("err_worker", "v_fresh", "m"):
            assert np.array_equal(whole.t[key][A:B], win.t[key]), (t, key)
        if win.served:
            b = n_c // 8
            assert np.array_equal(whole.bits_all[c_srv * b:(c_srv + 1) * b], win.server_bits)
            assert whole.server_scales[c_srv] == win.server_scale
            assert np.array_equal(whole.t["err_server"], win.t["err_server"])
        ls = win.layers
        assert np.array_equal(whole.t["r_prev"][ls], win.t["r_prev"][ls])
        assert np.array_equal(whole.t["coeff_c"][ls], win.t["coeff_c"][ls])
        for l in ls:
            a, b_ = int(win.lo[l]), int(win.hi[l])
            assert np.array_equal(whole.t["x"][A + a:A + b_], win.t["x"][a:b_]), (t, l)


def test_simulated_ranks_are_what_the_oracle_itself_would_send():
    """The generators of the other ranks' traffic (tests/refstep.py) against a full simulation: W
    oracle workers compress the same momentum with their own gradients and error buffers; what
    worker w sends for chunk c is slot w of simulated_worker_chunks."""
    from tests.refstep import simulated_server_chunks, simulated_worker_chunks
    rng = np.random.default_rng(5)
    W, c_srv = 4, 2
    off = np.array([0, 700, 700, 1900, 4000], np.int64)
    n_pad = padded_len(4000, W); n_c = n_pad // W
    F = Ref(np.float32)
    k = rng.uniform(0.5, 2, 4).astype(np.float32)
    m = (rng.standard_normal(n_pad) * 1e-4).astype(np.float32); m[4000:] = 0
    grads = [(rng.standard_normal(n_pad) * 1e-3).astype(np.float32) for _ in range(W)]
    errs = [(rng.standard_normal(n_pad) * 5e-5).astype(np.float32) for _ in range(W)]
    sl = slice(c_srv * n_c, (c_srv + 1) * n_c)
    g_c = {w: np.ascontiguousarray(grads[w][sl]) for w in range(W)}
    e_c = {w: errs[w][sl].copy() for w in range(W)}
    words, scales = simulated_worker_chunks(F, off, W, n_c, c_srv, k, 0.9, np.ascontiguousarray(m[sl]),
                                            g_c, e_c, threads=2)
    for w in range(W):
        bits, sc = F.compress_local(off, W, k, 0.9, grads[w], m, errs[w])   # the full worker
        if w == c_srv:
            assert not words[w * (n_c // 32):(w + 1) * (n_c // 32)].any() and scales[w] == 0
            continue
        assert np.array_equal(words[w * (n_c // 32):(w + 1) * (n_c // 32)].view(np.uint8),
                              bits[c_srv * (n_c // 8):(c_srv + 1) * (n_c // 8)])
        assert scales[w] == sc[c_srv]
        assert np.array_equal(e_c[w], errs[w][sl])
    # servers: chunk c's output decodes, with its error, to what it received plus its old error
    bits0, sc0 = F.compress_local(off, W, k, 0.9, grads[0], m, errs[0].copy())
    se = {c: (rng.standard_normal(n_c) * 5e-5).astype(np.float32) for c in range(W)}
    se0 = {c: v.copy() for c, v in se.items()}
    sw, ssc = simulated_server_chunks(F, W, n_c, c_srv, bits0, sc0, se, threads=2)
    for c in range(W):
        if c == c_srv:
            assert ssc[c] == 0
            continue
        recv = F.decompress_chunk(np.ascontiguousarray(bits0[c * (n_c // 8):(c + 1) * (n_c // 8)]), sc0[c], n_c)
        sent = F.decompress_chunk(sw[c * (n_c // 32):(c + 1) * (n_c // 32)].view(np.uint8).copy(), ssc[c], n_c)
        assert np.allclose(sent.astype(np.float64) + se[c], recv.astype(np.float64) + se0[c], rtol=0, atol=1e-10)
