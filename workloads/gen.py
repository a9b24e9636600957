"""Seeded input generators.  Random draws and layout only -- no optimizer arithmetic.

Every array is a function of (seed, stream name, step), drawn from numpy's counter-based Philox
generator, so that any consumer can regenerate the same bytes.  For the full-size benchmark
configurations `device=` switches to torch's generator on that device (much faster; the bytes
then depend on the device type, and consumers that need them on the host copy them back).

Recipes (the benchmark configurations of this repository; "N(0,s)" is read as standard
deviation s):
  state:  x ~ N(0, 0.02); m = 0; v_frozen = v_fresh = |N(0, 1e-4)| + 1e-8; errors = 0;
          c_avg ~ U(0.5, 2) per tensor; r_prev = 1.
  normal:               g ~ N(0, 1e-3)
  normal_layer_scaled:  g ~ N(0, 1e-3) * kappa_l, kappa_l ~ U(0.1, 10) fixed per tensor
  student_t3:           g ~ 1e-3 * t_3   (t_3 = Z / sqrt(chi2_3 / 3), heavy tailed)
  normal_sparse_layers: g ~ N(0, 1e-3), except 1 % of the tensors (chosen by the seed,
                        at least one) which get N(0, 1e-9)
  foreign chunks: the packed chunks that other ranks would send are uniformly random words with
          scales base * U(0.5, 1.5), base = 1e-4 (the order of magnitude of a momentum RMS
          under the gradient recipes above).
"""
import zlib

import numpy as np

_STREAM_IDS = {}


def _sid(name: str) -> int:
    if name not in _STREAM_IDS:
        _STREAM_IDS[name] = zlib.crc32(name.encode())
    return _STREAM_IDS[name]


class Streams:
    """Independent reproducible random streams keyed by (seed, name, step)."""

    def __init__(self, seed: int = 0, device=None):
        self.seed = int(seed)
        self.device = device  # None -> numpy on the host; else a torch device string

    def rng(self, name: str, step: int = 0) -> np.random.Generator:
        key = (self.seed << 32) ^ _sid(name)
        return np.random.Generator(np.random.Philox(key=key, counter=[0, 0, int(step), 0]))

    def tgen(self, name: str, step: int = 0):
        import torch
        g = torch.Generator(device=self.device)
        g.manual_seed(((self.seed * 1000003 + _sid(name)) * 1000003 + int(step)) % (2 ** 63 - 1))
        return g

    # -- primitive draws, returning numpy (host) or torch (device) float32 arrays -------------
    def normal(self, name, step, n, sigma):
        if self.device is None:
            a = self.rng(name, step).standard_normal(n, dtype=np.float32)
            a *= np.float32(sigma)
            return a
        import torch
        a = torch.randn(n, generator=self.tgen(name, step), device=self.device, dtype=torch.float32)
        return a.mul_(float(sigma))

    def student_t3(self, name, step, n, sigma):
        if self.device is None:
            r = self.rng(name, step)
            z = r.standard_normal(n, dtype=np.float32)
            chi = np.zeros(n, dtype=np.float32)
            for _ in range(3):
                w = r.standard_normal(n, dtype=np.float32)
                chi += w * w
            z /= np.sqrt(chi / np.float32(3.0))
            z *= np.float32(sigma)
            return z
        import torch
        g = self.tgen(name, step)
        z = torch.randn(n, generator=g, device=self.device, dtype=torch.float32)
        chi = torch.zeros(n, device=self.device, dtype=torch.float32)
        for _ in range(3):
            w = torch.randn(n, generator=g, device=self.device, dtype=torch.float32)
            chi.addcmul_(w, w)
        z.div_(chi.div_(3.0).sqrt_())
        return z.mul_(float(sigma))

    def uniform_host(self, name, step, n, lo, hi):
        return self.rng(name, step).uniform(lo, hi, n).astype(np.float32)

    def words(self, name, step, n):
        if self.device is None:
            return self.rng(name, step).integers(0, 2 ** 32, n, dtype=np.uint32)
        import torch
        a = torch.randint(-2 ** 31, 2 ** 31, (n,), generator=self.tgen(name, step),
                          device=self.device, dtype=torch.int32)
        return a

    def zeros(self, n):
        if self.device is None:
            return np.zeros(n, dtype=np.float32)
        import torch
        return torch.zeros(n, device=self.device, dtype=torch.float32)


def _zero_pad(a, n):
    a[n:] = 0
    return a


def init_state_items(st: Streams, cfg):
    """The arrays of init_state, one (key, array) pair at a time, so that a consumer that copies each
    one into place never holds two sets of N-sized arrays.  v_frozen and v_fresh are yielded as the
    SAME array (the snapshot and its source are equal at the start of the compression stage)."""
    pl, n_pad, W = cfg["plist"], cfg["n_pad"], cfg["W"]
    N, L = pl.N, pl.L
    yield "x", _zero_pad(st.normal("x", 0, n_pad, 0.02), N)
    yield "m", st.zeros(n_pad)
    v = st.normal("v", 0, n_pad, 1e-4)
    v = abs(v) if st.device is None else v.abs_()
    v += 1e-8
    v = _zero_pad(v, N)
    yield "v_frozen", v
    yield "v_fresh", v
    del v
    yield "err_worker", st.zeros(n_pad)
    yield "err_server", st.zeros(n_pad // W)
    yield "c_avg", st.uniform_host("c_avg", 0, L, 0.5, 2.0)
    yield "r_prev", np.ones(L, dtype=np.float32)


def init_state(st: Streams, cfg):
    """Optimizer state at the start of the compression stage; n_pad-long arrays, pad zeroed."""
    state = {}
    for k, a in init_state_items(st, cfg):
        if k == "v_fresh":
            a = a.copy() if st.device is None else a.clone()
        state[k] = a
    return state


def layer_kappa(st: Streams, cfg):
    """Per-tensor gradient multipliers of the recipe (None if the recipe has none)."""
    pl, kind = cfg["plist"], cfg["grad"]
    if kind == "normal_layer_scaled":
        return st.uniform_host("kappa", 0, pl.L, 0.1, 10.0)
    if kind == "normal_sparse_layers":
        k = np.ones(pl.L, dtype=np.float32)
        cnt = max(1, pl.L // 100)
        idx = st.rng("sparse_layers", 0).choice(pl.L, size=cnt, replace=False)
        k[idx] = np.float32(1e-6)  # sigma 1e-3 -> 1e-9
        return k
    return None


def gradient(st: Streams, cfg, step: int, kappa=None, stream: str = "grad"):
    """One n_pad-long gradient (pad zeroed) for `step` under the configuration's recipe."""
    pl, n_pad, kind = cfg["plist"], cfg["n_pad"], cfg["grad"]
    if kind == "student_t3":
        g = st.student_t3(stream, step, n_pad, 1e-3)
    else:
        g = st.normal(stream, step, n_pad, 1e-3)
    if kind in ("normal_layer_scaled", "normal_sparse_layers"):
        if kappa is None:
            kappa = layer_kappa(st, cfg)
        off = pl.offsets
        sizes = (off[1:] - off[:-1])
        if st.device is None:
            g[:pl.N] *= np.repeat(kappa, sizes)
        else:
            import torch
            kk = torch.repeat_interleave(torch.from_numpy(kappa).to(st.device),
                                         torch.from_numpy(sizes).to(st.device))
            g[:pl.N].mul_(kk)
    return _zero_pad(g, pl.N)


def foreign_worker_chunks(st: Streams, cfg, step: int, base: float = 1e-4):
    """What the W workers would send to this rank's server chunk: (words[W * n_c/32], scales[W]).
    The caller overwrites slot `server_chunk` with its own worker output."""
    W, n_c = cfg["W"], cfg["n_c"]
    words = st.words("fw_words", step, W * (n_c // 32))
    scales = (base * st.uniform_host("fw_scales", step, W, 0.5, 1.5)).astype(np.float32)
    return words, scales


def foreign_server_chunks(st: Streams, cfg, step: int, base: float = 1e-4):
    """What the W servers would broadcast: (words[n_pad/32], scales[W]).
    The caller overwrites chunk `server_chunk` with its own server output."""
    W, n_pad = cfg["W"], cfg["n_pad"]
    words = st.words("fs_words", step, n_pad // 32)
    scales = (base * st.uniform_host("fs_scales", step, W, 0.5, 1.5)).astype(np.float32)
    return words, scales
