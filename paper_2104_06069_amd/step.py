"""Device-side plumbing around the C ABI: buffers in HBM (torch tensors) and the order of calls of
one optimizer step.  No arithmetic of the method happens here -- torch is used to allocate and
copy device memory and to own the stream.

One compression-stage step on one rank (Algorithm 1 lines 6-21):
    compress_local            this worker's full buffer -> packed signs + W scales
    [gather]                  stands in for the all-to-all: the W packed chunks "received" for the
                              served chunk are resident tensors; this rank's own chunk is copied
                              into its slot
    server_reduce             served chunk -> recompressed chunk + scale
    [scatter]                 stands in for the all-gather: the W recompressed chunks are resident
                              tensors; this rank's own output is written into its slot
    layer_ratios, decompress_apply
"""
import numpy as np
import torch

from . import binding as ob

_STATE_KEYS = ("x", "m", "v_fresh", "v_frozen", "err_worker", "err_server", "c_avg", "r_prev")


class DeviceStep:
    def __init__(self, layer_offsets, num_workers, server_chunk=0, device="cuda:0", mom_scale=None,
                 **hyper):
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.W = int(num_workers)
        self.c = int(server_chunk)
        self.L = len(layer_offsets) - 1
        self.ctx = ob.ob_lamb_create(layer_offsets, num_workers, server_chunk, **hyper)
        self.N = ob.ob_lamb_num_params(self.ctx)
        self.n_pad = ob.ob_lamb_padded_len(self.ctx)
        self.n_c = ob.ob_lamb_chunk_len(self.ctx)
        f32 = dict(device=self.device, dtype=torch.float32)
        i32 = dict(device=self.device, dtype=torch.int32)
        self.t = {k: torch.zeros(self.n_pad, **f32) for k in ("x", "m", "v_fresh", "v_frozen", "err_worker")}
        self.t["err_server"] = torch.zeros(self.n_c, **f32)
        for k in ("c_avg", "coeff_c"):
            self.t[k] = torch.zeros(self.L, **f32)
        self.t["r_prev"] = torch.ones(self.L, **f32)
        self.t["mom_scale"] = None if mom_scale is None else self._dev(mom_scale)
        # wire buffers
        self.packed_local = torch.zeros(self.n_pad // 32, **i32)      # this worker's output
        self.scales_local = torch.zeros(self.W, **f32)
        self.packed_in = torch.zeros(self.W * (self.n_c // 32), **i32)  # what the served chunk receives
        self.scales_in = torch.zeros(self.W, **f32)
        self.packed_all = torch.zeros(self.n_pad // 32, **i32)        # the W recompressed chunks
        self.server_scales = torch.zeros(self.W, **f32)
        self._refresh_state()

    def _dev(self, a):
        if isinstance(a, np.ndarray):
            a = torch.from_numpy(np.ascontiguousarray(a))
        return a.to(self.device).contiguous()

    def _refresh_state(self):
        self.state = ob.make_state(**self.t)

    def close(self):
        if self.ctx is not None:
            torch.cuda.synchronize(self.device)
            ob.ob_lamb_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # ---- state upload / download (plumbing) --------------------------------------------------
    def load_state(self, st):
        """st: dict of numpy arrays or torch tensors keyed like ob_lamb_state."""
        for k in _STATE_KEYS:
            if k in st and st[k] is not None:
                self.t[k].copy_(self._dev(st[k]))
        self._refresh_state()

    def get(self, k):
        return self.t[k].detach().cpu().numpy()

    @property
    def stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    # ---- the calls ---------------------------------------------------------------------------
    def warmup_step(self, grad, lr):
        ob.ob_lamb_warmup_step(self.ctx, self.state, grad, lr, self.stream)

    def freeze(self):
        ob.ob_lamb_freeze(self.ctx, self.state, self.stream)

    def compress_local(self, grad):
        ob.ob_lamb_compress_local(self.ctx, self.state, grad, self.packed_local, self.scales_local,
                                  self.stream)

    def gather(self):
        """Own chunk c of the worker output -> slot c of the server's input (device copies)."""
        wpc = self.n_c // 32
        self.packed_in[self.c * wpc:(self.c + 1) * wpc].copy_(
            self.packed_local[self.c * wpc:(self.c + 1) * wpc], non_blocking=True)
        self.scales_in[self.c:self.c + 1].copy_(self.scales_local[self.c:self.c + 1], non_blocking=True)

    def server_reduce(self):
        """Writes the recompressed chunk straight into slot c of packed_all / server_scales."""
        wpc = self.n_c // 32
        ob.ob_lamb_server_reduce(self.ctx, self.state, self.packed_in, self.scales_in,
                                 self.packed_all[self.c * wpc:], self.server_scales[self.c:],
                                 self.stream)

    def layer_ratios(self):
        ob.ob_lamb_layer_ratios(self.ctx, self.state, self.packed_all, self.server_scales, self.stream)

    def decompress_apply(self, lr):
        ob.ob_lamb_decompress_apply(self.ctx, self.state, self.packed_all, self.server_scales, lr,
                                    self.stream)

    def step(self, grad, lr):
        self.compress_local(grad)
        self.gather()
        self.server_reduce()
        self.layer_ratios()
        self.decompress_apply(lr)
