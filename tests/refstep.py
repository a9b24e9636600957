"""Host-side mirror of the device step, driving the CPU oracle on numpy arrays (tests only)."""
import numpy as np

from oracle.obref import Ref, default_threads, lp_decode, lp_round  # noqa: F401

F32 = Ref(np.float32)

HYPER = dict(beta1=0.9, beta2=0.999, beta3=0.9, eta=1e-6, c_min=0.01, c_max=0.3, r_min=0.5,
             r_max=4.0, r_threshold=0.1, weight_decay=0.0)


class RefStep:
    def __init__(self, layer_offsets, num_workers, server_chunk=0, mom_scale=None, n_pad=None, threads=1,
                 **hyper):
        # threads > 1: the oracle's multi-threaded drivers (bit-identical to the serial routines)
        self.F = F32 if threads <= 1 else Ref(np.float32, threads)
        self.off = np.asarray(layer_offsets, dtype=np.int64)
        self.L = self.off.size - 1
        self.N = int(self.off[-1])
        self.W, self.c = int(num_workers), int(server_chunk)
        q = 256 * self.W
        self.n_pad = max(q, (self.N + q - 1) // q * q) if n_pad is None else int(n_pad)
        assert self.n_pad % q == 0 and self.n_pad >= self.N
        self.n_c = self.n_pad // self.W
        self.h = dict(HYPER)
        self.h.update(hyper)
        z = lambda n: np.zeros(n, np.float32)
        self.t = dict(x=z(self.n_pad), m=z(self.n_pad), v_fresh=z(self.n_pad), v_frozen=z(self.n_pad),
                      err_worker=z(self.n_pad), err_server=z(self.n_c), c_avg=z(self.L),
                      r_prev=np.ones(self.L, np.float32), coeff_c=z(self.L))
        self.mom_scale = None if mom_scale is None else np.ascontiguousarray(mom_scale, np.float32)
        self.bits_local = self.scales_local = None
        self.bits_in = np.zeros(self.W * self.n_c // 8, np.uint8)
        self.scales_in = z(self.W)
        self.bits_all = np.zeros(self.n_pad // 8, np.uint8)
        self.server_scales = z(self.W)

    def load_state(self, st):
        for k, v in st.items():
            if k in self.t and v is not None:
                self.t[k][...] = np.asarray(v, dtype=np.float32)

    # wire buffers from generated words (uint32 / int32 arrays)
    def set_foreign_in(self, words, scales):
        self.bits_in[...] = np.ascontiguousarray(words).view(np.uint8)
        self.scales_in[...] = scales

    def set_foreign_all(self, words, scales):
        self.bits_all[...] = np.ascontiguousarray(words).view(np.uint8)
        self.server_scales[...] = scales

    # mixed-precision variant: a gradient given as (fmt, uint16 patterns) is decoded and multiplied
    # by grad_scale; x_lp(fmt) is the 16-bit copy of the parameters (padding excluded by the caller)
    grad_scale = 1.0

    def _g32(self, g):
        if isinstance(g, tuple):
            fmt, bits = g
            return lp_decode(fmt, np.ascontiguousarray(bits), self.grad_scale)
        return g

    def x_lp(self, fmt):
        return lp_round(fmt, self.t["x"])

    def warmup_step(self, g, lr):
        g = self._g32(g)
        h, t = self.h, self.t
        t["coeff_c"][...] = self.F.warmup_step(self.off, h["beta1"], h["beta2"], h["beta3"], h["eta"],
                                            h["c_min"], h["c_max"], h["weight_decay"], lr, g, t["m"],
                                            t["v_fresh"], t["x"], t["c_avg"])

    def freeze(self):
        self.t["v_frozen"][...] = self.t["v_fresh"]
        self.t["r_prev"][...] = 1.0

    def momentum_scale(self):
        self.mom_scale = self.F.momentum_scale(self.off, self.t["m"])

    def train_step(self, t, warmup_steps, g, lr, fill_wire=None, momentum_scaling=True):
        if t < warmup_steps:
            self.warmup_step(g, lr)
            if t == warmup_steps - 1:
                self.freeze()
                if momentum_scaling:
                    self.momentum_scale()
            return
        if fill_wire is not None:
            fill_wire(self)
        self.step(g, lr)

    def compress_local(self, g):
        g = self._g32(g)
        self.bits_local, self.scales_local = self.F.compress_local(
            self.off, self.W, self.mom_scale, self.h["beta1"], g, self.t["m"], self.t["err_worker"])

    def gather(self):
        b = self.n_c // 8
        self.bits_in[self.c * b:(self.c + 1) * b] = self.bits_local[self.c * b:(self.c + 1) * b]
        self.scales_in[self.c] = self.scales_local[self.c]

    def server_reduce(self):
        b = self.n_c // 8
        bo, so = self.F.server_reduce(self.W, self.bits_in, self.scales_in, self.t["err_server"])
        self.bits_all[self.c * b:(self.c + 1) * b] = bo
        self.server_scales[self.c] = so

    def layer_ratios(self):
        h, t = self.h, self.t
        t["coeff_c"][...] = self.F.layer_ratios(self.off, self.W, self.mom_scale, h["beta1"], h["beta2"],
                                             h["r_min"], h["r_max"], h["r_threshold"], self.bits_all,
                                             self.server_scales, t["m"], t["v_fresh"], t["v_frozen"],
                                             t["c_avg"], t["r_prev"])

    def decompress_apply(self, lr):
        t = self.t
        self.F.decompress_apply(self.off, self.W, self.mom_scale, self.h["eta"], lr, self.bits_all,
                             self.server_scales, t["coeff_c"], t["v_frozen"], t["x"], t["m"])

    def step(self, g, lr):
        self.compress_local(g)
        self.gather()
        self.server_reduce()
        self.layer_ratios()
        self.decompress_apply(lr)


class WindowRef:
    """The oracle on chunks [c0, c1) of a W-chunk problem with chunk length n_c.

    Worker compression, error feedback, the decompressed momentum and the fresh variance are
    chunk-local (Appendix A.7.1: each chunk is its own parameter-server instance), so the oracle
    follows them exactly on the window alone; the ratio, the coefficient and the parameters are
    per layer and are valid for the layers that lie wholly inside the window (`inside`, `layers`).
    If the served chunk c_srv lies in the window, Algorithm 1 line 10 runs on it with the full
    fan-in of W packed chunks."""

    def __init__(self, offsets, W, n_c, c0, c1, c_srv, mom_scale=None, threads=1, **hyper):
        offsets = np.asarray(offsets, dtype=np.int64)
        self.W, self.n_c, self.c0, self.c1, self.c_srv = int(W), int(n_c), int(c0), int(c1), int(c_srv)
        self.A, self.B = self.c0 * self.n_c, self.c1 * self.n_c
        off = (np.clip(offsets, self.A, self.B) - self.A).astype(np.int64)
        self.inside = (offsets[:-1] >= self.A) & (offsets[1:] <= self.B) & (offsets[1:] > offsets[:-1])
        self.layers = np.nonzero(self.inside)[0]
        self.lo = offsets[:-1] - self.A      # window-relative [lo[l], hi[l]) of layer l (valid if inside)
        self.hi = offsets[1:] - self.A
        self.served = self.c0 <= self.c_srv < self.c1
        self.ref = RefStep(off, self.c1 - self.c0, (self.c_srv - self.c0) if self.served else 0,
                           mom_scale=mom_scale, n_pad=self.B - self.A, threads=threads, **hyper)
        assert self.ref.n_c == self.n_c
        self.t = self.ref.t
        self.server_bits = self.server_scale = None

    def load(self, get):
        """get(key) -> the full-size array (numpy) of that key, or a callable slicing the device."""
        for k in ("x", "m", "v_fresh", "v_frozen", "err_worker"):
            self.t[k][...] = get(k, self.A, self.B)
        for k in ("c_avg", "r_prev"):
            self.t[k][...] = get(k, None, None)
        if self.served:
            self.t["err_server"][...] = get("err_server", None, None)

    def step(self, g_win, lr, all_words_win, all_scales_win, in_words=None, in_scales=None):
        """g_win: the gradient on the window.  all_words_win / all_scales_win: what the W servers
        broadcast, restricted to the window (uint32 words / float32; the served chunk's slot is
        overwritten here with the oracle's own server output).  in_words / in_scales: what the W
        workers sent for the served chunk (needed when it lies in the window; the own slot is
        overwritten with the oracle's own worker output)."""
        r = self.ref
        r.compress_local(g_win)
        words = np.array(all_words_win, dtype=np.uint32, copy=True)
        scales = np.array(all_scales_win, dtype=np.float32, copy=True)
        if self.served:
            b = self.n_c // 8
            bits_in = np.array(in_words, copy=True).view(np.uint8)
            sc_in = np.array(in_scales, dtype=np.float32, copy=True)
            j = self.c_srv - self.c0
            bits_in[self.c_srv * b:(self.c_srv + 1) * b] = r.bits_local[j * b:(j + 1) * b]
            sc_in[self.c_srv] = r.scales_local[j]
            bo, so = r.F.server_reduce(self.W, bits_in, sc_in, r.t["err_server"])
            self.server_bits, self.server_scale = bo, so
            words.view(np.uint8)[j * b:(j + 1) * b] = bo
            scales[j] = so
        r.set_foreign_all(words, scales)
        r.layer_ratios()
        r.decompress_apply(lr)


def _for_each(items, fn, threads):
    """fn(item) for every item, on a pool of host threads (the oracle's C routines release the GIL)."""
    if threads <= 1:
        for it in items:
            fn(it)
        return
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=threads) as ex:
        list(ex.map(fn, items))


def simulated_worker_chunks(F, offsets, W, n_c, c_srv, mom_scale, beta1, m_chunk, grads, errs, threads=1):
    """What W-1 other workers would send for chunk c_srv: each compresses, with the oracle's own
    routine and its own error buffer errs[w] (updated in place), the local momentum
    k*(beta1*m + (1-beta1)*g_w) + err_w of that chunk, g_w = grads[w] being its own gradient draw
    (Algorithm 1 lines 6-7 on the sub-problem "this chunk alone").  -> (words uint32 [W * n_c/32],
    scales [W]); slot c_srv is left zero for the caller's own output."""
    offsets = np.asarray(offsets, dtype=np.int64)
    A = c_srv * n_c
    off = (np.clip(offsets, A, A + n_c) - A).astype(np.int64)
    words = np.zeros(W * (n_c // 32), np.uint32)
    scales = np.zeros(W, np.float32)
    def one(w):
        bits, s = F.compress_local(off, 1, mom_scale, beta1, grads[w], m_chunk, errs[w])
        words[w * (n_c // 32):(w + 1) * (n_c // 32)] = bits.view(np.uint32)
        scales[w] = s[0]
    _for_each([w for w in range(W) if w != c_srv], one, threads)
    return words, scales


def simulated_server_chunks(F, W, n_c, c_srv, own_bits, own_scales, server_errs, threads=1):
    """What the W-1 other servers would broadcast if every worker had sent what this one sent
    ("all workers identical" on the chunks this rank does not serve): chunk c's server takes this
    worker's decompressed chunk c as the average (a fan-in of 1), adds its own error buffer
    server_errs[c] (updated in place) and recompresses (Algorithm 1 line 10).  -> (words uint32 [W * n_c/32], scales [W]); slot c_srv left zero."""
    b = n_c // 8
    words = np.zeros(W * (n_c // 32), np.uint32)
    scales = np.zeros(W, np.float32)
    def one(c):
        bo, so = F.server_reduce(1, np.ascontiguousarray(own_bits[c * b:(c + 1) * b]),
                                 np.ascontiguousarray(own_scales[c:c + 1]), server_errs[c])
        words[c * (n_c // 32):(c + 1) * (n_c // 32)] = bo.view(np.uint32)
        scales[c] = so
    _for_each([c for c in range(W) if c != c_srv], one, threads)
    return words, scales
