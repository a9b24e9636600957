"""ctypes loader for the CPU oracle (oracle/libobref.so).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the CPU-baseline leg of
the benchmark.  It marshals numpy arrays into the C functions of obref.h and holds no arithmetic
of the method itself.  `Ref(np.float32)` binds the binary32 oracle, `Ref(np.float64)` the binary64
shadow of the same code.
"""
import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB = None


def lib():
    """Load libobref.so, compiling it with g++ first if it is missing or stale."""
    global _LIB
    if _LIB is None:
        import importlib.util
        spec = importlib.util.spec_from_file_location("_obref_build", os.path.join(_HERE, "build.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        # OBREF_LIB: a library built elsewhere from a DELIBERATELY WRONG copy of obref.cpp -- only
        # tests/test_oracle_mutants.py sets it, to show that the pins fail on such a copy
        _LIB = C.CDLL(os.environ.get("OBREF_LIB") or mod.build(force=False))
        _LIB.obref_padded_len.restype = C.c_int64
        _LIB.obref_padded_len.argtypes = [C.c_int64, C.c_int32]
    return _LIB


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _chk(a, dtype, n=None, name="array"):
    if a is None:
        return
    if not isinstance(a, np.ndarray) or a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need C-contiguous numpy array of {dtype}")
    if n is not None and a.size != n:
        raise ValueError(f"{name}: need {n} elements, got {a.size}")


def padded_len(n, W):
    return int(lib().obref_padded_len(int(n), int(W)))


LP_F16, LP_BF16 = 1, 2   # 16-bit storage formats of obref_lp_*


def lp_decode(fmt, bits, scale=1.0):
    """uint16 patterns of binary16 (fmt 1) / bfloat16 (fmt 2) -> float32 values times scale."""
    _chk(bits, np.uint16, name="bits")
    out = np.empty(bits.size, dtype=np.float32)
    lib().obref_lp_decode(C.c_int32(fmt), C.c_int64(bits.size), _p(bits), C.c_float(float(scale)), _p(out))
    return out


def lp_round(fmt, x):
    """float32 -> uint16 patterns of the nearest binary16 / bfloat16 value (ties to even)."""
    _chk(x, np.float32, name="x")
    out = np.empty(x.size, dtype=np.uint16)
    lib().obref_lp_round(C.c_int32(fmt), C.c_int64(x.size), _p(x), _p(out))
    return out


def default_threads():
    """Worker threads for the multi-threaded drivers: the host's cores, capped by OMP_NUM_THREADS
    (set to the job's CPU share on shared machines) and by 16."""
    n = os.cpu_count() or 1
    try:
        n = min(n, int(os.environ.get("OMP_NUM_THREADS", n)))
    except ValueError:
        pass
    return max(1, min(n, 16))


class Ref:
    """The oracle in one precision.  All methods update their array arguments in place.
    threads > 1 (binary32 only) routes the N-sized calls through the multi-threaded drivers, whose
    results are bit-identical to the serial routines'."""

    def __init__(self, dtype=np.float32, threads=1):
        self.dt = np.dtype(dtype)
        self.threads = int(threads)
        if self.threads > 1 and self.dt != np.float32:
            raise TypeError("the multi-threaded drivers are binary32 only")
        if self.dt == np.float32:
            self.pre, self.ct = "obref_", C.c_float
        elif self.dt == np.float64:
            self.pre, self.ct = "obref64_", C.c_double
        else:
            raise TypeError("float32 or float64")
        self.l = lib()

    def _f(self, name):
        return getattr(self.l, self.pre + name)

    def _off(self, off):
        off = np.ascontiguousarray(off, dtype=np.int64)
        return off, int(off.size - 1)

    def compress_chunk(self, z, err=None):
        """-> (bits uint8[n/8], scale, err).  err defaults to a new array."""
        n = z.size
        assert n % 8 == 0
        _chk(z, self.dt)
        if err is None:
            err = np.empty_like(z)
        _chk(err, self.dt, n)
        bits = np.empty(n // 8, dtype=np.uint8)
        s = self.ct(0)
        self._f("compress_chunk")(_p(z), C.c_int64(n), _p(bits), C.byref(s), _p(err))
        return bits, self.dt.type(s.value), err

    def decompress_chunk(self, bits, scale, n):
        _chk(bits, np.uint8, n // 8)
        out = np.empty(n, dtype=self.dt)
        self._f("decompress_chunk")(_p(bits), self.ct(float(scale)), C.c_int64(n), _p(out))
        return out

    def compress_local(self, off, W, mom_scale, beta1, g, m, err):
        """err is updated in place.  -> (bits uint8[n_pad/8], scales[W])"""
        off, L = self._off(off)
        n_pad = err.size
        assert n_pad % (256 * W) == 0 and off[-1] <= n_pad
        for a, nm in ((g, "g"), (m, "m"), (err, "err")):
            _chk(a, self.dt, n_pad, nm)
        _chk(mom_scale, self.dt, L, "mom_scale")
        bits = np.empty(n_pad // 8, dtype=np.uint8)
        scales = np.empty(W, dtype=self.dt)
        args = (C.c_int64(n_pad), C.c_int64(L), _p(off), C.c_int32(W), _p(mom_scale),
                self.ct(float(beta1)), _p(g), _p(m), _p(err), _p(bits), _p(scales))
        if self.threads > 1:
            self.l.obref_compress_local_mt(*args, C.c_int32(self.threads))
        else:
            self._f("compress_local")(*args)
        return bits, scales

    def server_reduce(self, W, bits_in, scales_in, err_server):
        """err_server updated in place. -> (bits_out uint8[n_c/8], scale_out)"""
        n_c = err_server.size
        assert n_c % 8 == 0
        _chk(bits_in, np.uint8, W * (n_c // 8), "bits_in")
        _chk(scales_in, self.dt, W, "scales_in")
        _chk(err_server, self.dt)
        bits_out = np.empty(n_c // 8, dtype=np.uint8)
        s = self.ct(0)
        args = (C.c_int64(n_c), C.c_int32(W), _p(bits_in), _p(scales_in), _p(err_server),
                _p(bits_out), C.byref(s))
        if self.threads > 1:
            self.l.obref_server_reduce_mt(*args, C.c_int32(self.threads))
        else:
            self._f("server_reduce")(*args)
        return bits_out, self.dt.type(s.value)

    def global_momentum(self, off, W, mom_scale, bits_all, server_scales, n_pad):
        off, L = self._off(off)
        _chk(bits_all, np.uint8, n_pad // 8, "bits_all")
        _chk(server_scales, self.dt, W, "server_scales")
        _chk(mom_scale, self.dt, L, "mom_scale")
        mt = np.empty(n_pad, dtype=self.dt)
        self._f("global_momentum")(C.c_int64(n_pad), C.c_int64(L), _p(off), C.c_int32(W),
                                   _p(mom_scale), _p(bits_all), _p(server_scales), _p(mt))
        return mt

    def ratios_dense(self, off, beta1, beta2, r_min, r_max, r_thr, mt, m, v_fresh, v_frozen,
                     c_avg, r_prev):
        """v_fresh, r_prev updated in place. -> coeff_c[L]"""
        off, L = self._off(off)
        n = int(off[-1])
        for a, nm in ((mt, "mt"), (m, "m"), (v_fresh, "v_fresh"), (v_frozen, "v_frozen")):
            _chk(a, self.dt, None, nm)
            assert a.size >= n
        _chk(c_avg, self.dt, L)
        _chk(r_prev, self.dt, L)
        coeff = np.empty(L, dtype=self.dt)
        t = self.ct
        self._f("ratios_dense")(C.c_int64(L), _p(off), t(float(beta1)), t(float(beta2)),
                                t(float(r_min)), t(float(r_max)), t(float(r_thr)), _p(mt), _p(m),
                                _p(v_fresh), _p(v_frozen), _p(c_avg), _p(r_prev), _p(coeff))
        return coeff

    def apply_dense(self, off, eta, lr, mt, coeff_c, v_frozen, x, m):
        off, L = self._off(off)
        n = int(off[-1])
        for a, nm in ((mt, "mt"), (v_frozen, "v_frozen"), (x, "x"), (m, "m")):
            _chk(a, self.dt, None, nm)
            assert a.size >= n
        _chk(coeff_c, self.dt, L)
        t = self.ct
        self._f("apply_dense")(C.c_int64(L), _p(off), t(float(eta)), t(float(lr)), _p(mt),
                               _p(coeff_c), _p(v_frozen), _p(x), _p(m))

    def layer_ratios(self, off, W, mom_scale, beta1, beta2, r_min, r_max, r_thr, bits_all,
                     server_scales, m, v_fresh, v_frozen, c_avg, r_prev):
        assert self.dt == np.float32
        off, L = self._off(off)
        n_pad = m.size
        for a, nm in ((m, "m"), (v_fresh, "v_fresh"), (v_frozen, "v_frozen")):
            _chk(a, self.dt, n_pad, nm)
        _chk(bits_all, np.uint8, n_pad // 8)
        _chk(server_scales, self.dt, W)
        _chk(mom_scale, self.dt, L)
        _chk(c_avg, self.dt, L)
        _chk(r_prev, self.dt, L)
        coeff = np.empty(L, dtype=self.dt)
        t = self.ct
        args = (C.c_int64(n_pad), C.c_int64(L), _p(off), C.c_int32(W), _p(mom_scale), t(float(beta1)),
                t(float(beta2)), t(float(r_min)), t(float(r_max)), t(float(r_thr)), _p(bits_all),
                _p(server_scales), _p(m), _p(v_fresh), _p(v_frozen), _p(c_avg), _p(r_prev), _p(coeff))
        if self.threads > 1:
            self.l.obref_layer_ratios_mt(*args, C.c_int32(self.threads))
        else:
            self.l.obref_layer_ratios(*args)
        return coeff

    def decompress_apply(self, off, W, mom_scale, eta, lr, bits_all, server_scales, coeff_c,
                         v_frozen, x, m):
        assert self.dt == np.float32
        off, L = self._off(off)
        n_pad = m.size
        for a, nm in ((m, "m"), (x, "x"), (v_frozen, "v_frozen")):
            _chk(a, self.dt, n_pad, nm)
        _chk(bits_all, np.uint8, n_pad // 8)
        _chk(server_scales, self.dt, W)
        _chk(mom_scale, self.dt, L)
        _chk(coeff_c, self.dt, L)
        t = self.ct
        args = (C.c_int64(n_pad), C.c_int64(L), _p(off), C.c_int32(W), _p(mom_scale), t(float(eta)),
                t(float(lr)), _p(bits_all), _p(server_scales), _p(coeff_c), _p(v_frozen), _p(x), _p(m))
        if self.threads > 1:
            self.l.obref_decompress_apply_mt(*args, C.c_int32(self.threads))
        else:
            self.l.obref_decompress_apply(*args)

    def warmup_step(self, off, beta1, beta2, beta3, eta, c_min, c_max, wd, lr, g, m, v, x, c_avg):
        """m, v, x, c_avg updated in place. -> c[L]"""
        off, L = self._off(off)
        n = int(off[-1])
        for a, nm in ((g, "g"), (m, "m"), (v, "v"), (x, "x")):
            _chk(a, self.dt, None, nm)
            assert a.size >= n
        _chk(c_avg, self.dt, L)
        c = np.empty(L, dtype=self.dt)
        t = self.ct
        args = (C.c_int64(L), _p(off), t(float(beta1)), t(float(beta2)), t(float(beta3)), t(float(eta)),
                t(float(c_min)), t(float(c_max)), t(float(wd)), t(float(lr)), _p(g), _p(m), _p(v), _p(x),
                _p(c), _p(c_avg))
        if self.threads > 1:
            self.l.obref_warmup_step_mt(*args, C.c_int32(self.threads))
        else:
            self._f("warmup_step")(*args)
        return c

    def momentum_scale(self, off, m):
        assert self.dt == np.float32
        off, L = self._off(off)
        _chk(m, self.dt)
        k = np.empty(L, dtype=np.float32)
        if self.threads > 1:
            self.l.obref_momentum_scale_mt(C.c_int64(L), _p(off), _p(m), _p(k), C.c_int32(self.threads))
        else:
            self.l.obref_momentum_scale(C.c_int64(L), _p(off), _p(m), _p(k))
        return k
