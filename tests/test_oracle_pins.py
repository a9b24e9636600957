"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle.

Each test states the expected value from a hand-worked case, a closed form, a library routine
(numpy's norm / packbits) or an algebraic identity from the paper, so that a dropped term, a
wrong sign or index, or a transposed operand in oracle/obref.cpp fails at least one of them.
CPU only.
"""
import numpy as np
import pytest

from oracle.obref import Ref, padded_len

F32, F64 = Ref(np.float32), Ref(np.float64)


def rng(seed):
    return np.random.default_rng(seed)


# --------------------------------------------------------------------------------------------
# packing format and sign convention (hand-written expected bytes; numpy packbits as library)
# --------------------------------------------------------------------------------------------
def test_pack_hand_bytes():
    # element i -> byte i/8, bit i%8, LSB first; bit = (z >= 0); +0 and -0 -> 1; NaN -> 0
    z = np.array([1, -1, 1, -1, 0.0, -0.0, np.nan, -2,     # 1,0,1,0,1,1,0,0 -> 0b00110101
                  -1, -1, -1, -1, -1, -1, -1, 3,            # only bit 7        -> 0b10000000
                  5, 5, 5, 5, 5, 5, 5, 5,                   # all               -> 0xFF
                  -5, -5, -5, -5, -5, -5, -5, -5],          # none              -> 0x00
                 dtype=np.float32)
    bits, _, _ = F32.compress_chunk(z)
    assert bits.tolist() == [0b00110101, 0b10000000, 0xFF, 0x00]
    # as little-endian 32-bit word: element i is bit i of the word
    assert int(bits.view("<u4")[0]) == 0x00FF8035


@pytest.mark.parametrize("ref", [F32, F64])
def test_pack_matches_numpy_packbits(ref):
    z = rng(1).standard_normal(4096).astype(ref.dt)
    z[::97] = 0.0
    bits, s, err = ref.compress_chunk(z)
    assert np.array_equal(bits, np.packbits(z >= 0, bitorder="little"))
    # decompress: bit -> +-scale, in the same element order
    d = ref.decompress_chunk(bits, s, z.size)
    assert np.array_equal(d, np.where(z >= 0, s, -s).astype(ref.dt))


def test_single_negative_element_position():
    for pos in (0, 1, 7, 8, 31, 32, 63, 64, 255):
        z = np.ones(256, dtype=np.float32)
        z[pos] = -1
        bits, _, _ = F32.compress_chunk(z)
        words = bits.view("<u4")
        expect = np.full(8, 0xFFFFFFFF, dtype=np.uint32)
        expect[pos // 32] ^= np.uint32(1 << (pos % 32))
        assert np.array_equal(words, expect), pos


# --------------------------------------------------------------------------------------------
# P1: the scale keeps the L2 norm; P2: error feedback is exact
# --------------------------------------------------------------------------------------------
def test_scale_hand_value():
    # z = (3, -4, 0, 0, 0, 0, 0, 0): ||z|| = 5, n = 8 -> s = 5/sqrt(8)
    z = np.array([3, -4, 0, 0, 0, 0, 0, 0], dtype=np.float64)
    bits, s, err = F64.compress_chunk(z)
    assert s == pytest.approx(5.0 / np.sqrt(8.0), rel=1e-15)
    assert bits.tolist() == [0b11111101]
    assert np.allclose(err, z - np.array([s, -s, s, s, s, s, s, s]), rtol=0, atol=1e-16)


@pytest.mark.parametrize("ref,tol", [(F32, 2e-7), (F64, 1e-14)])
def test_norm_preserved_and_matches_numpy(ref, tol):
    for seed, n in ((2, 256), (3, 8192), (4, 100000 // 8 * 8)):
        z = (rng(seed).standard_t(3, n) * 1e-3).astype(ref.dt)
        bits, s, _ = ref.compress_chunk(z)
        nz = np.linalg.norm(z.astype(np.float64))
        assert float(s) == pytest.approx(nz / np.sqrt(n), rel=tol)
        d = ref.decompress_chunk(bits, s, n)
        assert np.linalg.norm(d.astype(np.float64)) == pytest.approx(nz, rel=tol)


def test_error_feedback_exact():
    n = 4096
    z = rng(5).standard_normal(n)
    bits, s, err = F64.compress_chunk(z)
    d = F64.decompress_chunk(bits, s, n)
    assert np.array_equal(err, z - d)                      # bitwise
    # sum err*sign(z) = sum|z| - n*s
    sg = np.where(z >= 0, 1.0, -1.0)
    assert np.dot(err, sg) == pytest.approx(np.abs(z).sum() - n * s, rel=1e-12)
    z32 = z.astype(np.float32)
    bits, s, err = F32.compress_chunk(z32)
    d = F32.decompress_chunk(bits, s, n)
    assert np.array_equal(err, z32 - d)                    # one binary32 subtraction, bitwise
    # in place (err aliases z)
    zz = z32.copy()
    bits2, s2, _ = F32.compress_chunk(zz, err=zz)
    assert np.array_equal(zz, err) and s2 == s and np.array_equal(bits2, bits)


def test_zero_chunk():
    z = np.zeros(64, dtype=np.float32)
    bits, s, err = F32.compress_chunk(z)
    assert s == 0 and np.all(bits == 0xFF) and np.all(err == 0)


# --------------------------------------------------------------------------------------------
# worker side, Algorithm 1 lines 6-7 with momentum scaling (hand-worked)
# --------------------------------------------------------------------------------------------
def test_compress_local_hand():
    # one worker, W = 1, n_pad = 256, two layers [0,3) and [3,5), rest padding.
    # beta1 = 0.5: mloc = 0.5*m + 0.5*g.  k = (2, 4).
    off = [0, 3, 5]
    n_pad = 256
    m = np.zeros(n_pad); g = np.zeros(n_pad); err = np.zeros(n_pad)
    m[:5] = [2, 2, -2, 4, 0]
    g[:5] = [4, -8, 2, 0, -2]
    err[:5] = [1, 1, 1, -9, 0]
    err[5] = -0.5   # padding element: k = 1, m = g = 0 -> z = -0.5
    # mloc = (3, -3, 0, 2, -1); z = k*mloc + err = (7, -5, 1, -1, -4), pad: -0.5, then zeros
    z = np.zeros(n_pad); z[:6] = [7, -5, 1, -1, -4, -0.5]
    k = np.array([2.0, 4.0])
    bits, scales = F64.compress_local(off, 1, k, 0.5, g, m, err)
    s = np.sqrt((49 + 25 + 1 + 1 + 16 + 0.25) / 256)
    assert scales[0] == pytest.approx(s, rel=1e-15)
    expect_bits = np.packbits(z >= 0, bitorder="little")
    assert expect_bits[0] == 0b11000101
    assert np.array_equal(bits, expect_bits)
    assert np.allclose(err, z - np.where(z >= 0, s, -s), rtol=0, atol=1e-15)
    # mom_scale = None is k = 1
    err1 = np.zeros(n_pad); err1[:5] = [1, 1, 1, -9, 0]
    _, sc1 = F64.compress_local(off, 1, None, 0.5, g, m, err1)
    z1 = np.zeros(n_pad); z1[:5] = [4, -2, 1, -7, -1]
    assert sc1[0] == pytest.approx(np.sqrt((z1 ** 2).sum() / 256), rel=1e-15)


def test_chunk_independence():
    # the chunked compressor equals W independent single-chunk compressors, one per chunk
    # (Appendix A.7.1: chunk-wise parameter server); each chunk gets its own scale
    W, n_c = 4, 512
    n_pad = W * n_c
    r = rng(7)
    off = [0, 700, 701, 1500, 2000]
    g = r.standard_normal(n_pad).astype(np.float32); g[2000:] = 0
    m = r.standard_normal(n_pad).astype(np.float32); m[2000:] = 0
    e = (0.1 * r.standard_normal(n_pad)).astype(np.float32)
    # chunk 2 much larger than the others, so that a single global scale would be detected
    g[2 * n_c:3 * n_c] *= 100
    err = e.copy()
    bits, scales = F32.compress_local(off, W, None, 0.9, g, m, err)
    b1 = np.float32(0.9)
    z = (b1 * m + (np.float32(1) - b1) * g) + e
    for c in range(W):
        zc = np.ascontiguousarray(z[c * n_c:(c + 1) * n_c])
        bc, sc, ec = F32.compress_chunk(zc)
        assert sc == scales[c]
        assert np.array_equal(bc, bits[c * n_c // 8:(c + 1) * n_c // 8])
        assert np.array_equal(ec, err[c * n_c:(c + 1) * n_c])
    assert scales[2] > 5 * scales[0]


# --------------------------------------------------------------------------------------------
# server side, Algorithm 1 line 10
# --------------------------------------------------------------------------------------------
def test_server_layout_is_worker_major():
    # worker 0: all bits set, scale 1; worker 1: no bits set, scale 3 -> (1 - 3)/2 = -1 everywhere
    n_c = 64
    bits_in = np.concatenate([np.full(n_c // 8, 0xFF, np.uint8), np.zeros(n_c // 8, np.uint8)])
    sc = np.array([1.0, 3.0])
    es = np.zeros(n_c)
    bo, so = F64.server_reduce(2, bits_in, sc, es)
    assert so == 1.0 and np.all(bo == 0) and np.all(es == 0)  # zb = -1 = -so -> error 0
    # with a carried server error of +1.5 on element 5: zb[5] = 0.5 -> bit set
    es = np.zeros(n_c); es[5] = 1.5
    bo, so = F64.server_reduce(2, bits_in, sc, es)
    s = np.sqrt((63 * 1.0 + 0.25) / 64)
    assert so == pytest.approx(s, rel=1e-15)
    assert bo[0] == 0b00100000 and np.all(bo[1:] == 0)
    assert es[5] == pytest.approx(0.5 - s) and es[0] == pytest.approx(-1 + s)


def test_server_sum_is_sequential_binary32():
    # scales (2^24, 1, 1, 1), all bits set.  Sequentially in binary32: 2^24 + 1 -> 2^24 (tie to
    # even) three times; times 1/4 -> 4194304.  Any other order gives 4194305.
    n_c, W = 8, 4
    bits_in = np.full(W * n_c // 8, 0xFF, np.uint8)
    sc = np.array([2.0 ** 24, 1, 1, 1], dtype=np.float32)
    es = np.zeros(n_c, dtype=np.float32)
    es[1] = 0.5
    # undo the recompression: zb = err_after + decompressed
    bo, so = F32.server_reduce(W, bits_in, sc, es)
    zb = es + F32.decompress_chunk(bo, so, n_c)
    assert zb[0] == pytest.approx(4194304.0, abs=0.6)
    # sharper, without going through recompression: scale of the result
    # all elements equal 4194304 except element 1 (4194304.5 -> rounds to 4194304 in binary32)
    assert so == np.float32(4194304.0)
    # reversed order of workers gives the other value: the sum really is order dependent
    es2 = np.zeros(n_c, dtype=np.float32)
    _, so2 = F32.server_reduce(W, bits_in, np.ascontiguousarray(sc[::-1]), es2)
    assert so2 == np.float32(4194305.0)


def test_server_divides_once_after_the_sum():
    # W = 3 (1/W not exact), scales (1, 2^-24, 2^-24), all bits set.  Sum first: 1 + 2^-24 is a tie
    # and rounds to 1 (even), twice; one multiply by fl(1/3) = 0x3EAAAAAB gives 0x3EAAAAAB.
    # Dividing every term instead gives fl(1/3) + 1.99e-8 twice; each addend is more than half an
    # ulp (1.49e-8) of the sum and rounds it up: 0x3EAAAAAD.
    n_c, W = 8, 3
    bits_in = np.full(W * n_c // 8, 0xFF, np.uint8)
    sc = np.array([1.0, 2.0 ** -24, 2.0 ** -24], dtype=np.float32)
    es = np.zeros(n_c, dtype=np.float32)
    _, so = F32.server_reduce(W, bits_in, sc, es)     # all elements equal: the scale is that value
    assert np.float32(so).view(np.uint32) == 0x3EAAAAAB


@pytest.mark.parametrize("ref,tol", [(F32, 1e-6), (F64, 1e-13)])
def test_server_average_vs_dense_mean(ref, tol):
    # decompress every worker with the (pinned) chunk decompressor, average with numpy
    W, n_c = 16, 1024
    r = rng(11)
    bits_in = r.integers(0, 256, W * n_c // 8, dtype=np.uint8)
    sc = r.uniform(0.5, 1.5, W).astype(ref.dt)
    es0 = (0.1 * r.standard_normal(n_c)).astype(ref.dt)
    dense = np.stack([ref.decompress_chunk(np.ascontiguousarray(bits_in[w * n_c // 8:(w + 1) * n_c // 8]),
                                           sc[w], n_c) for w in range(W)]).astype(np.float64)
    zb = dense.mean(axis=0) + es0
    es = es0.copy()
    bo, so = ref.server_reduce(W, bits_in, sc, es)
    assert float(so) == pytest.approx(np.linalg.norm(zb) / np.sqrt(n_c), rel=tol)
    # signs can differ only where zb is within rounding of zero
    sure = np.abs(zb) > 1e-5
    assert np.array_equal((np.unpackbits(bo, bitorder="little") == 1)[sure], (zb >= 0)[sure])
    d = ref.decompress_chunk(bo, so, n_c).astype(np.float64)
    assert np.allclose(es, zb - d, rtol=0, atol=tol * 4)


def test_w1_server_is_idempotent():
    # P4: one worker, zero server error: the server recompresses a +-s vector -> same bits, same s
    n = 2048
    z = rng(13).standard_normal(n).astype(np.float32)
    bits, s, _ = F32.compress_chunk(z)
    es = np.zeros(n, dtype=np.float32)
    bo, so = F32.server_reduce(1, bits, np.array([s], np.float32), es)
    assert np.array_equal(bo, bits)
    assert abs(float(so) - float(s)) <= np.spacing(np.float32(s))
    assert np.max(np.abs(es)) <= 2 * np.spacing(np.float32(s))


# --------------------------------------------------------------------------------------------
# P5: telescoping identity of the proof (Appendix A.7.1, with the error factor = 1 as in
# Algorithm 1), over a full simulated W-worker x W-chunk step, in the binary64 shadow
# --------------------------------------------------------------------------------------------
def simulate_full_step(ref, off, W, k, beta1, m_prev, grads, err_w, err_s):
    """All W workers and all W server chunks.  err_w: [W, n_pad]; err_s: [n_pad] (chunk c of
    it belongs to server c).  Returns (mt, bits_all, server_scales); errors updated in place."""
    n_pad = m_prev.size
    n_c = n_pad // W
    wb, ws = [], []
    for w in range(W):
        b, s = ref.compress_local(off, W, k, beta1, grads[w], m_prev, err_w[w])
        wb.append(b); ws.append(s)
    bits_all = np.empty(n_pad // 8, np.uint8)
    sscales = np.empty(W, ref.dt)
    for c in range(W):
        bits_in = np.concatenate([wb[w][c * n_c // 8:(c + 1) * n_c // 8] for w in range(W)])
        sc_in = np.array([ws[w][c] for w in range(W)], dtype=ref.dt)
        es = np.ascontiguousarray(err_s[c * n_c:(c + 1) * n_c])
        bo, so = ref.server_reduce(W, bits_in, sc_in, es)
        err_s[c * n_c:(c + 1) * n_c] = es
        bits_all[c * n_c // 8:(c + 1) * n_c // 8] = bo
        sscales[c] = so
    mt = ref.global_momentum(off, W, k, bits_all, sscales, n_pad)
    return mt, bits_all, sscales


def test_telescoping_identity():
    W, n_c = 4, 256
    n_pad = W * n_c
    N = 1000
    off = [0, 300, 302, 1000]
    r = rng(17)
    m_prev = r.standard_normal(n_pad); m_prev[N:] = 0
    grads = r.standard_normal((W, n_pad)); grads[:, N:] = 0
    err_w = 0.3 * r.standard_normal((W, n_pad))
    err_s = 0.3 * r.standard_normal(n_pad)
    ew0, es0 = err_w.copy(), err_s.copy()
    beta1 = 0.9
    mt, _, _ = simulate_full_step(F64, off, W, None, beta1, m_prev, grads, err_w, err_s)
    # m_t = beta m_{t-1} + (1-beta) gbar + Delta_{t-1} - Delta_t, Delta = mean_w delta_w + delta_server
    gbar = grads.mean(axis=0)
    rhs = beta1 * m_prev + (1 - beta1) * gbar + (ew0.mean(axis=0) + es0) - (err_w.mean(axis=0) + err_s)
    assert np.allclose(mt[:N], rhs[:N], rtol=0, atol=1e-13)
    # and with momentum scaling k_l (A.5.2): the identity holds for k_l * m_t
    k = np.array([2.0, 0.25, 8.0])
    err_w, err_s = ew0.copy(), es0.copy()
    mt, _, _ = simulate_full_step(F64, off, W, k, beta1, m_prev, grads, err_w, err_s)
    kk = np.repeat(k, np.diff(off))
    rhs = kk * (beta1 * m_prev[:N] + (1 - beta1) * gbar[:N]) + (ew0.mean(axis=0) + es0)[:N] \
        - (err_w.mean(axis=0) + err_s)[:N]
    assert np.allclose(kk * mt[:N], rhs, rtol=0, atol=1e-12)
    assert np.all(mt[N:] == 0)


def test_global_momentum_hand():
    # two chunks of 256 with server scales (2, 4); layers [0,300) k=2, [300,400) k=0.5; rest pad
    W, n_pad = 2, 512
    off = [0, 300, 400]
    bits = np.zeros(n_pad // 8, np.uint8)
    bits[0] = 0b00000001            # element 0 positive
    bits[299 // 8] |= 1 << (299 % 8)
    bits[300 // 8] |= 1 << (300 % 8)
    mt = F32.global_momentum(off, W, np.array([2, 0.5], np.float32), bits,
                             np.array([2, 4], np.float32), n_pad)
    assert mt[0] == 1.0 and mt[1] == -1.0          # +-2 / 2
    assert mt[255] == -1.0 and mt[256] == -2.0     # chunk boundary: +-4 / 2
    assert mt[299] == 2.0                          # +4 / 2
    assert mt[300] == 8.0 and mt[301] == -8.0      # +-4 / 0.5
    assert np.all(mt[400:] == 0)
    mt1 = F32.global_momentum(off, W, None, bits, np.array([2, 4], np.float32), n_pad)
    assert mt1[0] == 2.0 and mt1[256] == -4.0 and mt1[300] == 4.0


# --------------------------------------------------------------------------------------------
# Algorithm 1 lines 15-21 (hand-worked) and P7 (bounds, closed form)
# --------------------------------------------------------------------------------------------
def test_ratios_hand():
    # beta1 = 0.5, beta2 = 0.75; layer 0 = {0,1}, layer 1 = {2}
    # element 0: m=2, mt=3 -> g=(3-1)/0.5=4; v_fresh=4 -> 0.75*4+0.25*16=7; v_frozen=14 -> q=2
    # element 1: m=0, mt=0 -> g=0; v_fresh=8 -> 6; v_frozen=3 -> q=0.5
    # element 2: m=4, mt=1 -> g=(1-2)/0.5=-2; v_fresh=4 -> 3+1=4; v_frozen=1 -> q=0.25
    off = [0, 2, 3]
    mt = np.array([3.0, 0, 1]); m = np.array([2.0, 0, 4])
    vf = np.array([4.0, 8, 4]); vz = np.array([14.0, 3, 1])
    c_avg = np.array([0.5, 3.0]); r_prev = np.array([1.0, 1.0])
    # wide bounds: r = raw max
    coeff = F64.ratios_dense(off, 0.5, 0.75, 0.01, 100.0, 0.9, mt, m, vf, vz, c_avg, r_prev)
    assert vf.tolist() == [7.0, 6.0, 4.0]
    assert r_prev.tolist() == [pytest.approx(1.9), 0.25]   # layer 0 capped by (1+0.9)*1
    assert coeff.tolist() == [pytest.approx(0.95), 0.75]
    # the paper's bounds: thr 0.1 -> [0.9, 1.1]; then [0.5, 4]
    vf = np.array([4.0, 8, 4]); r_prev = np.array([1.0, 1.0])
    coeff = F64.ratios_dense(off, 0.5, 0.75, 0.5, 4.0, 0.1, mt, m, vf, vz, c_avg, r_prev)
    assert r_prev.tolist() == [pytest.approx(1.1), pytest.approx(0.9)]
    assert coeff.tolist() == [pytest.approx(0.55), pytest.approx(2.7)]
    # second clip wins over the first: r_prev = 0.5 -> window [0.45, 0.55]; raw 0.25 -> 0.45 -> 0.5
    vf = np.array([4.0, 8, 4]); r_prev = np.array([4.0, 0.5])
    F64.ratios_dense(off, 0.5, 0.75, 0.5, 4.0, 0.1, mt, m, vf, vz, c_avg, r_prev)
    assert r_prev.tolist() == [pytest.approx(3.6), 0.5]   # raw 2 -> window [3.6, 4.4] -> 3.6
    # the window is a FACTOR around the previous ratio, above as well as below: r_prev = 1.5 -> window
    # [1.35, 1.65]; raw 2 -> 1.65 (a window of +-0.1 would give 1.6)
    vf = np.array([4.0, 8, 4]); r_prev = np.array([1.5, 1.5])
    F64.ratios_dense(off, 0.5, 0.75, 0.5, 4.0, 0.1, mt, m, vf, vz, c_avg, r_prev)
    assert r_prev.tolist() == [pytest.approx(1.65), pytest.approx(1.35)]
    # line 18 before line 19, visible when the previous ratio lies outside [r_min, r_max] (a state
    # loaded from elsewhere, or bounds changed between runs): r_prev = 0.2 -> window [0.18, 0.22];
    # raw 2 -> 0.22 -> r_min = 0.5 (the other order ends at 0.22);  r_prev = 8 -> window [7.2, 8.8];
    # raw 0.25 -> 7.2 -> r_max = 4 (the other order ends at 7.2)
    vf = np.array([4.0, 8, 4]); r_prev = np.array([0.2, 8.0])
    F64.ratios_dense(off, 0.5, 0.75, 0.5, 4.0, 0.1, mt, m, vf, vz, c_avg, r_prev)
    assert r_prev.tolist() == [0.5, 4.0]


def test_ratio_special_values():
    # v_fresh = 0 with v_frozen > 0 -> +Inf survives the max and is clipped; 0/0 -> NaN skipped;
    # an empty layer and an all-NaN layer give raw 0 -> lower window bound
    off = [0, 1, 2, 2, 3]
    mt = np.zeros(3, np.float32); m = np.zeros(3, np.float32)
    vf = np.zeros(3, np.float32); vz = np.array([1, 0, 5], np.float32)
    vf[2] = 5
    c_avg = np.ones(4, np.float32); r_prev = np.ones(4, np.float32)
    F32.ratios_dense(off, 0.9, 0.999, 0.5, 4.0, 0.1, mt, m, vf, vz, c_avg, r_prev)
    assert r_prev[0] == np.float32(1.1)                  # +Inf -> upper window
    assert r_prev[1] == np.float32(0.9)                  # NaN skipped -> 0 -> lower window
    assert r_prev[2] == np.float32(0.9)                  # empty layer
    assert r_prev[3] == pytest.approx(1 / 0.999, rel=1e-6)  # 5/(0.999*5): inside the window


def test_ratio_closed_form_zero_gradient(hp):
    # identity compressor, g = 0: m_t = beta1*m -> reconstructed g = 0 -> v_fresh *= beta2 each
    # step -> raw ratio after k steps = beta2^-k; the +-10 % window does not bind
    b1, b2 = hp["beta1"], hp["beta2"]
    n = 64
    off = [0, n]
    r = rng(19)
    m = r.standard_normal(n)
    vz = np.abs(r.standard_normal(n)) + 1e-3
    vf = vz.copy()
    c_avg = np.array([0.7]); r_prev = np.array([1.0])
    for k in range(1, 30):
        mt = b1 * m
        coeff = F64.ratios_dense(off, b1, b2, hp["r_min"], hp["r_max"], hp["r_threshold"],
                                 mt, m, vf, vz, c_avg, r_prev)
        m = mt
        # reconstructed gradient is 0 only up to rounding of (mt - b1*m)/(1-b1): exactly 0 here
        assert r_prev[0] == pytest.approx(b2 ** (-k), rel=1e-12)
        assert coeff[0] == pytest.approx(0.7 * b2 ** (-k), rel=1e-12)


def test_ratio_bounds_random(hp):
    # whatever the data, r stays in [r_min, r_max] and moves at most r_thr per step
    # (whenever the window meets [r_min, r_max])
    L, n = 6, 50
    off = np.arange(L + 1) * n
    r = rng(23)
    vz = (np.abs(r.standard_normal(L * n)) + 1e-3).astype(np.float32)
    vf = vz.copy()
    m = np.zeros(L * n, np.float32)
    c_avg = r.uniform(0.5, 2, L).astype(np.float32)
    r_prev = np.ones(L, np.float32)
    for t in range(60):
        mt = (r.standard_normal(L * n) * (10.0 if t % 7 == 0 else 0.01)).astype(np.float32)
        before = r_prev.copy()
        coeff = F32.ratios_dense(off, hp["beta1"], hp["beta2"], hp["r_min"], hp["r_max"],
                                 hp["r_threshold"], mt, m, vf, vz, c_avg, r_prev)
        m = mt
        assert np.all(r_prev >= np.float32(hp["r_min"])) and np.all(r_prev <= np.float32(hp["r_max"]))
        assert np.all(r_prev <= before * np.float32(1.1) * (1 + 1e-6))
        assert np.all(r_prev >= before * np.float32(0.9) * (1 - 1e-6))
        assert np.array_equal(coeff, r_prev * c_avg)


def test_apply_hand():
    # lr = 0.1, c = (2, 10); eta = 1
    # element 0: mt=3, v_frozen=4 -> u = 3/(2+1) = 1 -> x = 5 - 0.2*1 = 4.8 ; m <- 3
    # element 1: mt=-6, v_frozen=1 -> u = -6/2 = -3 -> x = 1 - 1.0*(-3) = 4 ; m <- -6
    off = [0, 1, 2]
    x = np.array([5.0, 1.0]); m = np.array([9.0, 9.0])
    F64.apply_dense(off, 1.0, 0.1, np.array([3.0, -6.0]), np.array([2.0, 10.0]),
                    np.array([4.0, 1.0]), x, m)
    assert x.tolist() == [pytest.approx(4.8), pytest.approx(4.0)]
    assert m.tolist() == [3.0, -6.0]
    # eta = 0 is line 21 as printed: x -= lr*c*mt/sqrt(v)
    x = np.array([5.0]); m = np.array([0.0])
    F64.apply_dense([0, 1], 0.0, 0.5, np.array([3.0]), np.array([2.0]), np.array([9.0]), x, m)
    assert x[0] == pytest.approx(4.0)


def test_packed_calls_equal_dense_calls():
    # layer_ratios / decompress_apply = global_momentum followed by the dense routines
    W, n_c = 4, 256
    n_pad, N = W * n_c, 900
    off = [0, 100, 102, 900]
    r = rng(29)
    bits = r.integers(0, 256, n_pad // 8, dtype=np.uint8)
    ss = r.uniform(0.5, 1.5, W).astype(np.float32)
    k = np.array([2, 0.5, 3], np.float32)
    m = r.standard_normal(n_pad).astype(np.float32); m[N:] = 0
    vz = (np.abs(r.standard_normal(n_pad)) + 0.1).astype(np.float32)
    vf = vz.copy()
    x = r.standard_normal(n_pad).astype(np.float32)
    c_avg = np.array([1, 2, 3], np.float32)
    rp = np.ones(3, np.float32)
    mt = F32.global_momentum(off, W, k, bits, ss, n_pad)
    vf2, rp2, x2, m2 = vf.copy(), rp.copy(), x.copy(), m.copy()
    co2 = F32.ratios_dense(off, 0.9, 0.999, 0.5, 4, 0.1, mt, m2, vf2, vz, c_avg, rp2)
    F32.apply_dense(off, 1e-6, 0.01, mt, co2, vz, x2, m2)
    co = F32.layer_ratios(off, W, k, 0.9, 0.999, 0.5, 4, 0.1, bits, ss, m, vf, vz, c_avg, rp)
    F32.decompress_apply(off, W, k, 1e-6, 0.01, bits, ss, co, vz, x, m)
    for a, b in ((vf, vf2), (rp, rp2), (co, co2), (x, x2), (m, m2)):
        assert np.array_equal(a, b)
    assert np.array_equal(x[N:], x2[N:])


# --------------------------------------------------------------------------------------------
# P8: LAMB step of eq. (1), hand-worked, and the moving average of c
# --------------------------------------------------------------------------------------------
def test_warmup_hand():
    # beta1 = 0.5, beta2 = 0.75, eta = 0, m0 = v0 = 0
    # layer 0: g = (3, 4): m = (1.5, 2); v = 0.25*(9, 16) = (2.25, 4); sqrt v = (1.5, 2); u = (1, 1)
    #          x = (3, 4): ||x|| = 5, ||u|| = sqrt 2 -> c = 5/sqrt(2) = 3.5355 (inside [0.01, 10])
    #          x <- x - 0.1*c*u = (3 - 0.35355, 4 - 0.35355)
    # layer 1: g = (-2): m = -1; v = 1; u = -1; x = (0.001): ratio 0.001 -> clipped to c_min = 0.01
    #          x <- 0.001 + 0.1*0.01 = 0.002
    off = [0, 2, 3]
    g = np.array([3.0, 4.0, -2.0]); m = np.zeros(3); v = np.zeros(3)
    x = np.array([3.0, 4.0, 0.001]); c_avg = np.array([0.0, 1.0])
    c = F64.warmup_step(off, 0.5, 0.75, 0.9, 0.0, 0.01, 10.0, 0.0, 0.1, g, m, v, x, c_avg)
    assert m.tolist() == [1.5, 2.0, -1.0] and v.tolist() == [2.25, 4.0, 1.0]
    c0 = 5 / np.sqrt(2)
    assert c.tolist() == [pytest.approx(c0, rel=1e-15), 0.01]
    assert x.tolist() == [pytest.approx(3 - 0.1 * c0), pytest.approx(4 - 0.1 * c0), pytest.approx(0.002)]
    assert c_avg.tolist() == [pytest.approx(0.1 * c0), pytest.approx(0.9 + 0.001)]
    # upper clip and the weight-decay term: wd = 0.5 -> u = m/sqrt(v) + 0.5*x
    g = np.array([3.0, 4.0]); m = np.zeros(2); v = np.zeros(2); x = np.array([3.0, 4.0])
    c_avg = np.zeros(1)
    c = F64.warmup_step([0, 2], 0.5, 0.75, 0.9, 0.0, 0.01, 0.3, 0.5, 0.1, g, m, v, x, c_avg)
    # u = (1 + 1.5, 1 + 2) = (2.5, 3); ratio = 5/sqrt(15.25) = 1.28 -> c_max = 0.3
    assert c[0] == 0.3
    assert x.tolist() == [pytest.approx(3 - 0.03 * 2.5), pytest.approx(4 - 0.03 * 3)]
    # eta enters the denominator: eta = 0.5 on layer (g=3): u = 1.5/(1.5+0.5) = 0.75
    g = np.array([3.0]); m = np.zeros(1); v = np.zeros(1); x = np.array([3.0]); c_avg = np.zeros(1)
    c = F64.warmup_step([0, 1], 0.5, 0.75, 0.9, 0.5, 0.01, 10.0, 0.0, 1.0, g, m, v, x, c_avg)
    assert c[0] == pytest.approx(4.0) and x[0] == pytest.approx(0.0)


def test_warmup_degenerate_norms():
    # ||x|| = ||u|| = 0 -> 0/0 = NaN -> c_min;  ||u|| = 0 < ||x|| -> +Inf -> c_max
    off = [0, 1, 2]
    g = np.zeros(2, np.float32); m = np.zeros(2, np.float32); v = np.ones(2, np.float32)
    x = np.array([0.0, 2.0], np.float32); c_avg = np.zeros(2, np.float32)
    c = F32.warmup_step(off, 0.9, 0.999, 0.9, 1e-6, 0.01, 0.3, 0.0, 0.1, g, m, v, x, c_avg)
    assert c.tolist() == [np.float32(0.01), np.float32(0.3)]
    assert x.tolist() == [0.0, 2.0]


def test_c_avg_closed_form(hp):
    # a constant c gives c_avg = c*(1 - beta3^k) after k steps (c_avg starts at 0, no bias correction)
    # constant c: every step clipped at c_max
    n = 32
    off = [0, n]
    r = rng(31)
    x = (r.standard_normal(n) * 10).astype(np.float64)
    m = np.zeros(n); v = np.zeros(n); c_avg = np.zeros(1)
    for k in range(1, 25):
        g = r.standard_normal(n)
        c = F64.warmup_step(off, hp["beta1"], hp["beta2"], hp["beta3"], 1e-6, hp["c_min"],
                            hp["c_max"], 0.0, 1e-3, g, m, v, x, c_avg)
        assert c[0] == hp["c_max"]
        assert c_avg[0] == pytest.approx(hp["c_max"] * (1 - hp["beta3"] ** k), rel=1e-12)


def test_warmup_vs_numpy_textbook():
    # the same step written with numpy vector operations in binary64 (library norm)
    r = rng(37)
    off = np.array([0, 5, 6, 40, 100])
    n = 100
    g = r.standard_normal(n); m = r.standard_normal(n); v = np.abs(r.standard_normal(n))
    x = r.standard_normal(n); c_avg = r.uniform(0, 1, 4)
    b1, b2, b3, eta, lr = 0.9, 0.999, 0.9, 1e-6, 0.02
    m2 = b1 * m + (1 - b1) * g
    v2 = b2 * v + (1 - b2) * g * g
    u = m2 / (np.sqrt(v2) + eta)
    x2 = x.copy(); cs = []
    for l in range(4):
        s = slice(off[l], off[l + 1])
        c = min(max(np.linalg.norm(x[s]) / np.linalg.norm(u[s]), 0.01), 0.3)
        cs.append(c)
        x2[s] = x[s] - lr * c * u[s]
    ca2 = b3 * c_avg + (1 - b3) * np.array(cs)
    c = F64.warmup_step(off, b1, b2, b3, eta, 0.01, 0.3, 0.0, lr, g, m, v, x, c_avg)
    assert np.allclose(m, m2, rtol=1e-15, atol=0) and np.allclose(v, v2, rtol=1e-15, atol=0)
    assert np.allclose(c, cs, rtol=1e-14) and np.allclose(x, x2, rtol=1e-13, atol=1e-15)
    assert np.allclose(c_avg, ca2, rtol=1e-14)


# --------------------------------------------------------------------------------------------
# P3: with the identity in place of C[.] the compression-stage step is plain LAMB
# --------------------------------------------------------------------------------------------
def test_identity_compressor_reduces_to_lamb(hp):
    # identity compressor: m_t = beta1 m + (1-beta1) mean_w g_w and errors stay 0.  Then
    #  (a) the fresh variance follows v = beta2 v + (1-beta2) gbar^2 (reconstructed gradient = gbar)
    #  (b) with v_frozen := that v and c := LAMB's c, line 21 gives LAMB's x of eq. (1)
    r = rng(41)
    off = np.array([0, 17, 19, 200])
    n, W = 200, 4
    grads = r.standard_normal((W, n)) * 1e-2
    gbar = grads.mean(axis=0)
    m0 = r.standard_normal(n) * 1e-2
    v0 = np.abs(r.standard_normal(n)) * 1e-4 + 1e-8
    x0 = r.standard_normal(n)
    b1, b2, b3 = hp["beta1"], hp["beta2"], hp["beta3"]
    # LAMB on the averaged gradient
    m, v, x, c_avg = m0.copy(), v0.copy(), x0.copy(), np.zeros(3)
    c = F64.warmup_step(off, b1, b2, b3, 1e-6, hp["c_min"], hp["c_max"], 0.0, 0.01, gbar, m, v, x, c_avg)
    # compression stage with identity compressor
    mt = b1 * m0 + (1 - b1) * gbar
    vf = v0.copy(); rp = np.ones(3)
    F64.ratios_dense(off, b1, b2, hp["r_min"], hp["r_max"], hp["r_threshold"], mt, m0, vf,
                     v0.copy(), np.ones(3), rp)
    assert np.allclose(vf, v, rtol=1e-9, atol=0)            # (a): g reconstructed to rounding
    xx, mm = x0.copy(), m0.copy()
    F64.apply_dense(off, 1e-6, 0.01, mt, c, v, xx, mm)      # (b)
    assert np.allclose(mm, m, rtol=1e-15, atol=0)
    assert np.allclose(xx, x, rtol=1e-14, atol=1e-16)


# --------------------------------------------------------------------------------------------
# binary32 oracle against its binary64 shadow on a whole simulated step
# --------------------------------------------------------------------------------------------
def test_f32_tracks_f64_shadow(hp):
    W, n_c = 4, 512
    n_pad, N = W * n_c, 2000
    off = np.array([0, 700, 702, 1500, 2000])
    r = rng(43)
    m0 = (r.standard_normal(n_pad) * 1e-3); m0[N:] = 0
    grads = r.standard_normal((W, n_pad)) * 1e-3; grads[:, N:] = 0
    out = {}
    for ref in (F32, F64):
        dt = ref.dt
        err_w = np.zeros((W, n_pad), dt); err_s = np.zeros(n_pad, dt)
        mt, bits, ss = simulate_full_step(ref, off, W, None, hp["beta1"], m0.astype(dt),
                                          grads.astype(dt), err_w, err_s)
        out[dt.name] = (mt, bits, ss, err_w, err_s)
    a, b = out["float32"], out["float64"]
    assert np.allclose(a[2], b[2], rtol=1e-6)
    # server bits may differ only where the averaged value is within rounding of 0
    nd = np.unpackbits(a[1] ^ b[1]).sum()
    assert nd <= 2
    assert np.allclose(a[3], b[3], rtol=0, atol=1e-9)


def test_padded_len():
    assert padded_len(1, 1) == 256 and padded_len(256, 1) == 256 and padded_len(257, 1) == 512
    assert padded_len(336232258, 64) == 336232448
    assert padded_len(336232258, 256) == 336265216
    assert padded_len(1048576, 4) == 1048576


def test_momentum_scale_reading():
    # sigma_l = rms of the layer; k_l = mean(sigma)/sigma_l; zero and empty layers -> 1
    off = [0, 4, 4, 6, 8]
    m = np.array([2, -2, 2, -2, 0, 0, 6, -6], np.float32)
    k = F32.momentum_scale(off, m)
    # non-empty layers: sigma = (2, 0, 6) -> mean = 8/3
    assert k.tolist() == [pytest.approx(4 / 3, rel=1e-6), 1.0, 1.0, pytest.approx(4 / 9, rel=1e-6)]


# --------------------------------------------------------------------------------------------
# Degenerate settings: the method's two relatives fall out of the same step.
#  * r_min = r_max = 1 freezes the scaling coefficient at its warmup average -- the
#    "LAMB + basic 1-bit" ablation of Section 3.4 / Appendix A.4;
#  * one layer with c_avg = 1 on top of that is the compression stage of 1-bit Adam
#    (Section 2: x -= lr * m / sqrt(v_frozen), no layerwise coefficient).
# The expected update is written out in numpy from the wire contents (numpy.unpackbits).
# --------------------------------------------------------------------------------------------
def _degenerate_steps(off, W, c_avg, steps=4, seed=41):
    from tests.refstep import RefStep
    r = rng(seed)
    ref = RefStep(off, W, server_chunk=W - 1, r_min=1.0, r_max=1.0)
    N, n_pad, n_c = ref.N, ref.n_pad, ref.n_c
    x0 = r.standard_normal(n_pad).astype(np.float32)
    v = (np.abs(r.standard_normal(n_pad)) * 1e-4 + 1e-8).astype(np.float32)
    ref.load_state(dict(x=x0, v_fresh=v, v_frozen=v, c_avg=np.asarray(c_avg, np.float32)))
    lens = np.diff(np.asarray(off))
    c_elem = np.zeros(n_pad); c_elem[:N] = np.repeat(np.asarray(c_avg, np.float64), lens)
    for t in range(steps):
        g = (r.standard_normal(n_pad) * 1e-3).astype(np.float32); g[N:] = 0
        ref.set_foreign_in(r.integers(0, 2**32, W * n_c // 32, dtype=np.uint32), r.uniform(5e-5, 2e-4, W).astype(np.float32))
        ref.set_foreign_all(r.integers(0, 2**32, n_pad // 32, dtype=np.uint32), r.uniform(5e-5, 2e-4, W).astype(np.float32))
        x_before = ref.t["x"].astype(np.float64)
        lr = 1e-3 * (t + 1)
        ref.step(g, lr)
        sign = np.unpackbits(ref.bits_all, bitorder="little").astype(np.float64) * 2 - 1
        m_bar = sign * np.repeat(ref.server_scales.astype(np.float64), n_c)
        want = x_before - lr * c_elem * m_bar / (np.sqrt(v.astype(np.float64)) + ref.h["eta"])
        assert np.all(ref.t["r_prev"] == 1.0)
        assert np.array_equal(ref.t["coeff_c"], np.asarray(c_avg, np.float32))
        assert np.allclose(ref.t["x"][:N], want[:N], rtol=2e-6, atol=0)
        assert np.array_equal(ref.t["x"][N:], x0[N:])            # padding is no layer's
        assert np.array_equal(ref.t["m"][:N], m_bar[:N].astype(np.float32))
    return ref


def test_degenerate_frozen_coefficient():
    # r pinned to 1: c_t = c_avg for ever, whatever v_fresh does (it still tracks the gradient)
    ref = _degenerate_steps([0, 700, 701, 2000, 3000], 4, [0.3, 1.7, 0.9, 1.2])
    assert not np.array_equal(ref.t["v_fresh"], ref.t["v_frozen"])


def test_degenerate_single_layer_is_1bit_adam():
    _degenerate_steps([0, 3000], 4, [1.0])
    _degenerate_steps([0, 256], 1, [1.0])


# --------------------------------------------------------------------------------------------
# 16-bit storage formats (mixed-precision variant): pinned to numpy's binary16 and torch's
# bfloat16 conversions (library routines), to hand-worked ties and to exhaustive round trips
# --------------------------------------------------------------------------------------------
def _same_bits_or_nan(a, b, fmt):
    exp_all = 0x7c00 if fmt == 1 else 0x7f80
    nan_a = ((a & exp_all) == exp_all) & ((a & ~np.uint16(exp_all | 0x8000)) != 0)
    nan_b = ((b & exp_all) == exp_all) & ((b & ~np.uint16(exp_all | 0x8000)) != 0)
    return np.all((a == b) | (nan_a & nan_b))


def test_lp_decode_all_patterns():
    from oracle.obref import lp_decode
    bits = np.arange(65536, dtype=np.uint16)
    want16 = bits.view(np.float16).astype(np.float32)
    got16 = lp_decode(1, bits)
    assert np.array_equal(got16.view(np.uint32)[~np.isnan(want16)], want16.view(np.uint32)[~np.isnan(want16)])
    assert np.array_equal(np.isnan(got16), np.isnan(want16))
    # bfloat16 is the upper half of a binary32 pattern
    wantb = (bits.astype(np.uint32) << 16).view(np.float32)
    gotb = lp_decode(2, bits)
    ok = ~np.isnan(wantb)
    assert np.array_equal(gotb.view(np.uint32)[ok], wantb.view(np.uint32)[ok])
    assert np.array_equal(np.isnan(gotb), np.isnan(wantb))
    # the scale is one binary32 multiply
    assert lp_decode(1, np.array([0x3c00, 0xc000, 0x0001], np.uint16), 0.25).tolist() == [0.25, -0.5, 2.0 ** -26]


def test_lp_round_trip_is_identity():
    from oracle.obref import lp_decode, lp_round
    bits = np.arange(65536, dtype=np.uint16)
    for fmt in (1, 2):
        back = lp_round(fmt, lp_decode(fmt, bits))
        assert _same_bits_or_nan(back, bits, fmt)


def test_lp_round_hand_cases():
    from oracle.obref import lp_round
    f = lambda *v: np.array(v, np.float32)
    # binary16: 1 + 2^-11 is a tie between 1 (even) and 1 + 2^-10 -> 1; 1 + 3*2^-11 ties up to even
    assert lp_round(1, f(1 + 2.0 ** -11, 1 + 3 * 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -20)).tolist() == [0x3c00, 0x3c02, 0x3c01]
    # largest finite 65504; 65519.99 rounds down to it, 65520 (the tie) goes to infinity
    assert lp_round(1, f(65504, 65519.996, 65520, -1e30)).tolist() == [0x7bff, 0x7bff, 0x7c00, 0xfc00]
    # subnormals: 2^-24 is the smallest; 2^-25 ties to zero (even), 3*2^-25 ties to 2*2^-24
    assert lp_round(1, f(2.0 ** -24, 2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -25 * 1.0001, -0.0)).tolist() == [1, 0, 2, 1, 0x8000]
    # rounding up across a binade and from the largest subnormal into the smallest normal
    assert lp_round(1, f(2047.5, 2.0 ** -14 - 2.0 ** -26)).tolist() == [0x6800, 0x0400]
    # bfloat16: 1 + 2^-8 ties to 1; 1 + 2^-8 + 2^-23 goes up; 3.3895314e38 -> Inf
    assert lp_round(2, f(1 + 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -23, 1 + 3 * 2.0 ** -8)).tolist() == [0x3f80, 0x3f81, 0x3f82]
    assert lp_round(2, np.array([0x7f7fffff, 0x7f7f7fff, 0x00000001, 0x00008000, 0x00018000], np.uint32).view(np.float32)).tolist() == \
        [0x7f80, 0x7f7f, 0, 0, 2]
    assert lp_round(1, f(np.nan)).tolist() == [0x7e00] and lp_round(2, f(np.nan, np.inf, -np.inf)).tolist() == [0x7fc0, 0x7f80, 0xff80]


def test_lp_round_matches_library_conversions():
    import torch
    from oracle.obref import lp_round
    r = rng(77)
    x = np.concatenate([
        (r.standard_normal(200000) * np.exp(r.uniform(-30, 12, 200000))).astype(np.float32),
        r.integers(0, 2 ** 32, 200000, dtype=np.uint32).view(np.float32),      # every exponent, NaNs, Infs
        (np.arange(65536, dtype=np.uint32) << 13 | 0x1000).view(np.float32),   # exact binary16 ties
        ((np.arange(65536, dtype=np.uint32) << 16) | 0x8000).view(np.float32)])  # exact bfloat16 ties
    with np.errstate(over="ignore", invalid="ignore"):
        want16 = x.astype(np.float16).view(np.uint16)
    assert _same_bits_or_nan(lp_round(1, x), want16, 1)
    wantb = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert _same_bits_or_nan(lp_round(2, x), wantb, 2)
