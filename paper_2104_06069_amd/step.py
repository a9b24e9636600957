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

With packed_momentum=True the momentum is kept in the 1-bit form it has after line 13: the step's
packed_all/server_scales buffers ARE the momentum of the next step, so two such buffer pairs
alternate (begin_step() switches to the pair that does not hold the momentum) and the dense array
is only read by the first step after warmup.
"""
import numpy as np
import torch

from . import binding as ob

_STATE_KEYS = ("x", "m", "v_fresh", "v_frozen", "err_worker", "err_server", "c_avg", "r_prev")


class DeviceStep:
    def __init__(self, layer_offsets, num_workers, server_chunk=0, device="cuda:0", mom_scale=None,
                 packed_momentum=False, fused_apply=False, x_lp_dtype=None, grad_scale=1.0,
                 status_interval=64, fold_gather=True, deferred_error=False, deferred_variance=0, **hyper):
        """hyper: the fields of ob_lamb_config (hyper-parameters, flags, fused_max_tiles, spin_limit).
        status_interval: every that many optimizer steps step()/warmup_step() ask the library whether a
        bounded device-side wait has expired (one stream synchronisation; raises ObLambError with
        OB_ERR_STATE if so, after which the state must be restored from a checkpoint); 0 = never,
        the caller calls check_status() itself."""
        # fold_gather: compress_local also writes this rank's own chunk straight into its server's
        # input slot, so gather() has nothing left to copy
        self.fold_gather = bool(fold_gather)
        # deferred_error: err_worker holds z; the error itself is z - C[z] with this worker's own
        # previous output (packed_local / scales_local, which then must survive between the steps)
        # (and err_server holds zb, with the server's own previous output kept in srv_words / srv_scale)
        self.deferred_error = bool(deferred_error)
        # deferred_variance = K >= 2: v_fresh is brought up to date only every K-th compression step;
        # in between, the steps form the up-to-date variance in registers from the array and the sign
        # words and scales of the momenta since it was written (ob_lamb_ratios_apply_hist), which are
        # the steps' own packed_all / server_scales buffers, kept in a ring.  K + 1 buffers would do;
        # the ring has 2K, so that the arrangement of buffers and history repeats every 2K steps
        # (graph_period) and a graph that holds that many consecutive steps can be replayed
        self.vf_period = int(deferred_variance)
        if self.vf_period:
            assert 2 <= self.vf_period <= ob.OB_VF_MAX_OLD + 1 and packed_momentum and fused_apply, \
                "deferred_variance needs the 1-bit momentum and ob_lamb_ratios_apply"
        self.vf_ages = {}         # steps taken so far by the number of momentum steps each had to apply
        self._vf_n_old = 0        # momenta older than the previous one since v_fresh was written
        self._vf_pending = None   # arguments of the last step that left v_fresh behind (for the dense view)
        self.status_interval = int(status_interval)
        self._steps_since_check = 0
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
        self.srv_words = torch.zeros(self.n_c // 32, **i32)             # deferred server error: own previous output
        self.srv_scale = torch.zeros(1, **f32)
        # the W recompressed chunks (two pairs when they double as the momentum)
        self.packed_momentum = bool(packed_momentum)
        self.fused_apply = bool(fused_apply)   # layer_ratios + decompress_apply as one call
        npairs = (2 * self.vf_period if self.vf_period else 2) if self.packed_momentum else 1
        self._pa = [torch.zeros(self.n_pad // 32, **i32) for _ in range(npairs)]
        self._ss = [torch.zeros(self.W, **f32) for _ in range(npairs)]
        self._cur = 0
        self.m_is_packed = False   # True once a step has committed the momentum in 1-bit form
        # mixed-precision variant: a float16/bfloat16 gradient tensor is taken as it is (times
        # grad_scale, the inverse loss scale); x_lp_dtype asks for a 16-bit copy of x after each update
        self.grad_scale = float(grad_scale)
        self.x_lp = None if x_lp_dtype is None else torch.zeros(self.n_pad, device=self.device, dtype=x_lp_dtype)

    # the buffer pair of the current step
    @property
    def packed_all(self):
        return self._pa[self._cur]

    @property
    def server_scales(self):
        return self._ss[self._cur]

    @property
    def graph_period(self):
        """Number of consecutive steps after which the buffers a step uses (wire pairs, momentum, the
        variance's history and its age) are the same again: what one captured graph must hold."""
        return len(self._pa)

    @property
    def _prev(self):
        """Ring index of the pair that holds the previous momentum."""
        return (self._cur - 1) % len(self._pa)

    def _dev(self, a):
        if isinstance(a, np.ndarray):
            a = torch.from_numpy(np.ascontiguousarray(a))
        return a.to(self.device).contiguous()

    def _state(self, momentum):
        """ob_lamb_state for one call.  momentum: 'read' (source of m_{t-1}) or 'commit'."""
        b = dict(self.t)
        if self.fold_gather:
            wpc = self.n_c // 32
            b["own_packed_in"] = self.packed_in[self.c * wpc:]
            b["own_scale_in"] = self.scales_in[self.c:]
        if self.deferred_error:
            b["err_packed"], b["err_scales"] = self.packed_local, self.scales_local
            b["srv_err_packed"], b["srv_err_scale"] = self.srv_words, self.srv_scale
        if self.packed_momentum and momentum == "commit":
            b["m"] = None                       # committed in place: packed_all is the momentum
            b["m_packed"], b["m_scales"] = self.packed_all, self.server_scales
        elif self.packed_momentum and self.m_is_packed:
            b["m"] = None
            b["m_packed"], b["m_scales"] = self._pa[self._prev], self._ss[self._prev]
        return ob.make_state(**b)

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
        """st: dict of numpy arrays or torch tensors keyed like ob_lamb_state (dense momentum)."""
        for k in _STATE_KEYS:
            if k in st and st[k] is not None:
                self.t[k].copy_(self._dev(st[k]))
        if "v_fresh" in st and st["v_fresh"] is not None:
            self._vf_n_old, self._vf_pending = 0, None    # the array is the variance again
        if "m" in st and st["m"] is not None:
            self._vf_fold()            # (a dense momentum ends the history of 1-bit momenta)
            self.m_is_packed = False
        if "err_worker" in st and st["err_worker"] is not None:
            self.scales_local.zero_()      # (deferred form: zero scales make err_worker the error itself)
        if "err_server" in st and st["err_server"] is not None:
            self.srv_scale.zero_()

    def checkpoint(self):
        """The optimizer state as host arrays in its plain form, whatever compact forms are in use:
        the momentum, both compression errors and the fresh variance are materialised (fp32, exactly
        the values the compact forms stand for), so that load_state() of the result into a new
        DeviceStep -- of any configuration -- continues the run bit for bit."""
        keys = ["x", "m", "v_fresh", "v_frozen", "err_worker", "err_server", "c_avg", "r_prev", "coeff_c"]
        ck = {k: self.get(k).copy() for k in keys}
        if self.t["mom_scale"] is not None:
            ck["mom_scale"] = self.t["mom_scale"].cpu().numpy().copy()
        return ck

    def _vf_hist(self, n_old, write_v):
        """ob_lamb_vf_history of the step whose pairs are (_cur, _prev): the n_old pairs before them."""
        R = len(self._pa)
        idx = [(self._cur - 2 - i) % R for i in range(n_old)]
        return ob.make_vf_history([self._pa[i] for i in idx], [self._ss[i] for i in idx], write_v)

    def _vf_state(self):
        """ob_lamb_state of the dense-view calls: the previous momentum in its 1-bit form, whatever
        form the next step will read it in."""
        return ob.make_state(**dict(self.t, m=None, m_packed=self._pa[self._prev], m_scales=self._ss[self._prev]))

    def v_fresh_dense(self):
        """The fresh variance as a device tensor (materialised if the array was left behind)."""
        if self._vf_pending is None:
            return self.t["v_fresh"]
        cur, n_old = self._vf_pending
        assert cur == self._cur, "the dense view belongs to the step that was taken last"
        out = torch.empty_like(self.t["v_fresh"])     # (the call copies the array, then updates what lags)
        ob.ob_lamb_variance_dense(self.ctx, self._vf_state(), self.packed_all, self.server_scales,
                                  self._vf_hist(n_old, 0), out, self.stream)
        return out

    def _vf_fold(self):
        """Bring the v_fresh array up to date (before anything that uses it as the variance itself)."""
        if self._vf_pending is None:
            return
        cur, n_old = self._vf_pending
        assert cur == self._cur
        ob.ob_lamb_variance_dense(self.ctx, self._vf_state(), self.packed_all, self.server_scales,
                                  self._vf_hist(n_old, 1), self.t["v_fresh"], self.stream)
        self._vf_n_old, self._vf_pending = 0, None

    def err_dense(self):
        """The worker error delta as a device tensor (materialised from the deferred form if that is in use)."""
        if not self.deferred_error:
            return self.t["err_worker"]
        out = torch.empty_like(self.t["err_worker"])
        ob.ob_lamb_error_dense(self.ctx, self._state("read"), out, self.stream)
        return out

    def get(self, k):
        if k == "err_worker" and self.deferred_error:
            return self.err_dense().cpu().numpy()
        if k == "err_server" and self.deferred_error:
            out = torch.empty_like(self.t["err_server"])
            ob.ob_lamb_server_error_dense(self.ctx, self._state("read"), out, self.stream)
            return out.cpu().numpy()
        if k == "v_fresh":
            return self.v_fresh_dense().cpu().numpy()
        if k == "m" and self.m_is_packed:
            # dense view of the 1-bit momentum (held by the pair of the step that committed it)
            s = ob.make_state(**dict(self.t, m_packed=self.packed_all, m_scales=self.server_scales))
            ob.ob_lamb_momentum_dense(self.ctx, s, self.t["m"], self.stream)
        return self.t[k].detach().cpu().numpy()

    @property
    def stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    # ---- the calls ---------------------------------------------------------------------------
    @staticmethod
    def _ob_dtype(t):
        return {torch.float32: ob.OB_F32, torch.float16: ob.OB_F16, torch.bfloat16: ob.OB_BF16}[t.dtype]

    def _x_lp_args(self):
        return (None, ob.OB_F32) if self.x_lp is None else (self.x_lp, self._ob_dtype(self.x_lp))

    def _is_plain(self, grad=None):
        return self.x_lp is None and (grad is None or (grad.dtype == torch.float32 and self.grad_scale == 1.0))

    def check_status(self):
        """Synchronises the stream; raises ObLambError(OB_ERR_STATE) if a device-side wait expired
        since the last check (the outputs of the steps since then are undefined)."""
        self._steps_since_check = 0
        ob.ob_lamb_check_device_status(self.ctx, self.stream)

    def _count_step(self):
        self._steps_since_check += 1
        if (self.status_interval and self._steps_since_check >= self.status_interval
                and not torch.cuda.is_current_stream_capturing()):   # (a capture cannot synchronise)
            self.check_status()

    def warmup_step(self, grad, lr):
        self._warmup_step(grad, lr)
        self._count_step()

    def _warmup_step(self, grad, lr):
        self._vf_fold()
        if self._is_plain(grad):
            ob.ob_lamb_warmup_step(self.ctx, self._state("read"), grad, lr, self.stream)
        else:
            ob.ob_lamb_warmup_step_lp(self.ctx, self._state("read"), grad, self._ob_dtype(grad),
                                      self.grad_scale, lr, *self._x_lp_args(), self.stream)

    def freeze(self):
        self._vf_fold()
        ob.ob_lamb_freeze(self.ctx, self._state("read"), self.stream)

    def momentum_scale(self):
        """End of warmup (Appendix A.5.2): form the per-layer coefficients from the dense momentum."""
        if self.t["mom_scale"] is None:
            self.t["mom_scale"] = torch.ones(self.L, device=self.device, dtype=torch.float32)
        ob.ob_lamb_momentum_scale(self.ctx, self._state("read"), self.stream)

    def train_step(self, t, warmup_steps, grad, lr, fill_wire=None, momentum_scaling=True):
        """Step t of the two-stage schedule of Algorithm 1: LAMB for t < warmup_steps (the last of
        them followed by the end-of-warmup snapshot), compression-stage steps afterwards.
        fill_wire(self) is called once the step's wire buffers are selected, to place what the
        other ranks sent (in a real job: the two collectives)."""
        if t < warmup_steps:
            self.warmup_step(grad, lr)
            if t == warmup_steps - 1:
                self.freeze()
                if momentum_scaling:
                    self.momentum_scale()
            return
        self.begin_step()
        if fill_wire is not None:
            fill_wire(self)
        self.step(grad, lr)

    def begin_step(self):
        """Select the wire buffers of the coming step: the pair that does not hold the momentum."""
        if self.packed_momentum and self.m_is_packed:
            self._cur = (self._cur + 1) % len(self._pa)

    def compress_local(self, grad):
        if self._is_plain(grad):
            ob.ob_lamb_compress_local(self.ctx, self._state("read"), grad, self.packed_local,
                                      self.scales_local, self.stream)
        else:
            ob.ob_lamb_compress_local_lp(self.ctx, self._state("read"), grad, self._ob_dtype(grad),
                                         self.grad_scale, self.packed_local, self.scales_local, self.stream)

    def gather(self):
        """Own chunk c of the worker output -> slot c of the server's input (device copies; already
        done by compress_local when fold_gather is on)."""
        if self.fold_gather:
            return
        wpc = self.n_c // 32
        self.packed_in[self.c * wpc:(self.c + 1) * wpc].copy_(
            self.packed_local[self.c * wpc:(self.c + 1) * wpc], non_blocking=True)
        self.scales_in[self.c:self.c + 1].copy_(self.scales_local[self.c:self.c + 1], non_blocking=True)

    def server_reduce(self):
        """Writes the recompressed chunk straight into slot c of packed_all / server_scales."""
        wpc = self.n_c // 32
        ob.ob_lamb_server_reduce(self.ctx, self._state("read"), self.packed_in, self.scales_in,
                                 self.packed_all[self.c * wpc:], self.server_scales[self.c:],
                                 self.stream)

    def layer_ratios(self):
        self._vf_fold()
        ob.ob_lamb_layer_ratios(self.ctx, self._state("read"), self.packed_all, self.server_scales,
                                self.stream)

    def decompress_apply(self, lr):
        if self._is_plain():
            ob.ob_lamb_decompress_apply(self.ctx, self._state("commit"), self.packed_all,
                                        self.server_scales, lr, self.stream)
        else:
            ob.ob_lamb_decompress_apply_lp(self.ctx, self._state("commit"), self.packed_all,
                                           self.server_scales, lr, *self._x_lp_args(), self.stream)
        if self.packed_momentum:
            self.m_is_packed = True

    def ratios_apply(self, lr):
        if self.vf_period and self.m_is_packed:
            # the variance in deferred form: the array is brought up to date every vf_period-th step
            # (which buffers hold the history and how old the array is changes from step to step with
            # a period of graph_period steps: a captured graph must hold a multiple of that many)
            n_old = self._vf_n_old
            write_v = (n_old + 1 >= self.vf_period)
            ob.ob_lamb_ratios_apply_hist_lp(self.ctx, self._state("read"), self.packed_all, self.server_scales, lr,
                                            self._vf_hist(n_old, write_v), *self._x_lp_args(), self.stream)
            self.vf_ages[n_old + 1] = self.vf_ages.get(n_old + 1, 0) + 1
            if write_v:
                self._vf_n_old, self._vf_pending = 0, None
            else:
                self._vf_n_old, self._vf_pending = n_old + 1, (self._cur, n_old)
        elif self._is_plain():
            ob.ob_lamb_ratios_apply(self.ctx, self._state("read"), self.packed_all, self.server_scales, lr,
                                    self.stream)
        else:
            ob.ob_lamb_ratios_apply_lp(self.ctx, self._state("read"), self.packed_all, self.server_scales,
                                       lr, *self._x_lp_args(), self.stream)
        if self.packed_momentum:
            self.m_is_packed = True

    def step(self, grad, lr):
        """One compression-stage step into the current wire buffers (call begin_step() first and
        fill packed_in / packed_all with what the other ranks sent)."""
        self.compress_local(grad)
        self.gather()
        self.server_reduce()
        if self.fused_apply:
            self.ratios_apply(lr)
        else:
            self.layer_ratios()
            self.decompress_apply(lr)
        self._count_step()
