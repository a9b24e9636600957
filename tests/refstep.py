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
