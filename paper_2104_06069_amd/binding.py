"""ctypes binding with the same names as the C ABI (include/onebitlamb.h).

Argument marshalling only.  Device buffers are passed as raw addresses: anything with a
`data_ptr()` method (a torch tensor), an int, or None.  Streams are raw hipStream_t handles
(`torch.cuda.current_stream().cuda_stream`), 0/None = the default stream.
"""
import ctypes as C
import os

OB_OK = 0
OB_ERR_NULL, OB_ERR_ARG, OB_ERR_ALIGN, OB_ERR_STATE, OB_ERR_HIP = -1, -2, -3, -4, -5
_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB = None


class ObLambError(RuntimeError):
    def __init__(self, status, where, detail=""):
        self.status = status
        msg = f"{where}: status {status} ({ob_lamb_status_string(status)})"
        if detail:
            msg += f": {detail}"
        super().__init__(msg)


class ObLambConfig(C.Structure):
    _fields_ = [("num_layers", C.c_int64), ("layer_offsets", C.POINTER(C.c_int64)),
                ("num_workers", C.c_int32), ("server_chunk", C.c_int32),
                ("beta1", C.c_float), ("beta2", C.c_float), ("beta3", C.c_float),
                ("eta", C.c_float), ("c_min", C.c_float), ("c_max", C.c_float),
                ("r_min", C.c_float), ("r_max", C.c_float), ("r_threshold", C.c_float),
                ("weight_decay", C.c_float),
                ("flags", C.c_uint32), ("fused_max_tiles", C.c_int32), ("spin_limit", C.c_int32)]


# ob_lamb_config.flags / spin_limit
OB_CFG_TWO_PASS_COMPRESS, OB_CFG_NO_FUSED_APPLY, OB_CFG_TWO_PASS_WARMUP = 1, 2, 4
OB_CFG_NO_BARRIERS = 7
OB_SPIN_NONE = -1
OB_VF_MAX_OLD = 7


class ObLambState(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in
                ("x", "m", "v_fresh", "v_frozen", "err_worker", "err_server", "c_avg", "r_prev",
                 "coeff_c", "mom_scale", "m_packed", "m_scales", "own_packed_in", "own_scale_in",
                 "err_packed", "err_scales", "srv_err_packed", "srv_err_scale")]


class ObLambVfHistory(C.Structure):
    _fields_ = [("n_old", C.c_int32), ("write_v", C.c_int32),
                ("bits", C.c_void_p * OB_VF_MAX_OLD), ("scales", C.c_void_p * OB_VF_MAX_OLD)]


def lib_path():
    return os.path.join(_PKG, "lib", "libonebitlamb.so")


def lib():
    """The loaded shared library.  Raises if it has not been built: there is no fallback."""
    global _LIB
    if _LIB is None:
        p = lib_path()
        if not os.path.exists(p):
            raise ImportError(f"{p} is missing: build it with `python -m paper_2104_06069_amd.build`")
        L = C.CDLL(p)
        vp, i32, i64, f = C.c_void_p, C.c_int32, C.c_int64, C.c_float
        sp = C.POINTER(ObLambState)
        sig = {
            "ob_lamb_create": (C.c_int, [C.POINTER(ObLambConfig), C.POINTER(vp)]),
            "ob_lamb_destroy": (None, [vp]),
            "ob_lamb_num_params": (i64, [vp]),
            "ob_lamb_padded_len": (i64, [vp]),
            "ob_lamb_chunk_len": (i64, [vp]),
            "ob_lamb_workspace_bytes": (C.c_size_t, [vp]),
            "ob_lamb_padded_len_for": (i64, [i64, i32]),
            "ob_lamb_status_string": (C.c_char_p, [C.c_int]),
            "ob_lamb_last_hip_error": (C.c_char_p, [vp]),
            "ob_lamb_warmup_step": (C.c_int, [vp, sp, vp, f, vp]),
            "ob_lamb_freeze": (C.c_int, [vp, sp, vp]),
            "ob_lamb_compress_local": (C.c_int, [vp, sp, vp, vp, vp, vp]),
            "ob_lamb_server_reduce": (C.c_int, [vp, sp, vp, vp, vp, vp, vp]),
            "ob_lamb_layer_ratios": (C.c_int, [vp, sp, vp, vp, vp]),
            "ob_lamb_decompress_apply": (C.c_int, [vp, sp, vp, vp, f, vp]),
            "ob_lamb_ratios_apply": (C.c_int, [vp, sp, vp, vp, f, vp]),
            "ob_lamb_warmup_step_lp": (C.c_int, [vp, sp, vp, C.c_int, f, f, vp, C.c_int, vp]),
            "ob_lamb_compress_local_lp": (C.c_int, [vp, sp, vp, C.c_int, f, vp, vp, vp]),
            "ob_lamb_decompress_apply_lp": (C.c_int, [vp, sp, vp, vp, f, vp, C.c_int, vp]),
            "ob_lamb_ratios_apply_lp": (C.c_int, [vp, sp, vp, vp, f, vp, C.c_int, vp]),
            "ob_lamb_fused_layers": (i64, [vp]),
            "ob_lamb_fused_params": (i64, [vp]),
            "ob_lamb_warmup_fused_layers": (i64, [vp]),
            "ob_lamb_warmup_fused_params": (i64, [vp]),
            "ob_lamb_big_tile_params": (i64, [vp]),
            "ob_lamb_momentum_dense": (C.c_int, [vp, sp, vp, vp]),
            "ob_lamb_momentum_scale": (C.c_int, [vp, sp, vp]),
            "ob_lamb_ratios_apply_hist": (C.c_int, [vp, sp, vp, vp, f, C.POINTER(ObLambVfHistory), vp]),
            "ob_lamb_ratios_apply_hist_lp": (C.c_int, [vp, sp, vp, vp, f, C.POINTER(ObLambVfHistory), vp, C.c_int, vp]),
            "ob_lamb_variance_dense": (C.c_int, [vp, sp, vp, vp, C.POINTER(ObLambVfHistory), vp, vp]),
            "ob_lamb_error_dense": (C.c_int, [vp, sp, vp, vp]),
            "ob_lamb_server_error_dense": (C.c_int, [vp, sp, vp, vp]),
            "ob_lamb_check_device_status": (C.c_int, [vp, vp]),
            "ob_lamb_uses_single_pass": (i32, [vp]),
            "ob_lamb_server_single_pass": (i32, [vp]),
            "ob_lamb_plan_split": (C.c_int, [C.POINTER(ObLambConfig), i64, vp, vp]),
            "ob_lamb_plan_big_tiles": (C.c_int, [C.POINTER(ObLambConfig), i64, vp]),
            "ob_lamb_server_reduce_static": (C.c_int, [i32, i64, vp, vp, vp, vp, vp, vp]),
            "ob_lamb_static_max_chunk_len": (i64, []),
            "ob_lamb_diag_copy": (C.c_int, [vp, vp, i64, vp]),
            "ob_lamb_profile_enable": (C.c_int, [vp, C.c_int]),
            "ob_lamb_profile_read": (i32, [vp, i32, C.POINTER(C.c_char_p), C.POINTER(C.c_double),
                                           C.POINTER(i64)]),
        }
        for name, (res, args) in sig.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _LIB = L
    return _LIB


def _addr(t):
    if t is None:
        return None
    if hasattr(t, "data_ptr"):
        return t.data_ptr()
    return int(t)


def make_state(**buffers):
    """ObLambState from keyword buffers (tensors / addresses / None)."""
    s = ObLambState()
    for k, v in buffers.items():
        setattr(s, k, _addr(v))
    return s


def _check(status, ctx, where):
    if status != OB_OK:
        detail = lib().ob_lamb_last_hip_error(ctx).decode() if ctx else ""
        raise ObLambError(status, where, detail)


def ob_lamb_status_string(status):
    return lib().ob_lamb_status_string(int(status)).decode()


def ob_lamb_padded_len_for(n, num_workers):
    return int(lib().ob_lamb_padded_len_for(int(n), int(num_workers)))


def ob_lamb_create(layer_offsets, num_workers, server_chunk=0, beta1=0.9, beta2=0.999, beta3=0.9,
                   eta=1e-6, c_min=0.01, c_max=0.3, r_min=0.5, r_max=4.0, r_threshold=0.1,
                   weight_decay=0.0, flags=0, fused_max_tiles=0, spin_limit=0):
    """-> opaque context handle (on the current HIP device)."""
    offs = [int(o) for o in layer_offsets]
    arr = (C.c_int64 * len(offs))(*offs)
    cfg = ObLambConfig(len(offs) - 1, arr, int(num_workers), int(server_chunk), beta1, beta2, beta3,
                       eta, c_min, c_max, r_min, r_max, r_threshold, weight_decay, int(flags),
                       int(fused_max_tiles), int(spin_limit))
    out = C.c_void_p()
    st = lib().ob_lamb_create(C.byref(cfg), C.byref(out))
    if st != OB_OK:
        raise ObLambError(st, "ob_lamb_create")
    return out


def ob_lamb_plan_split(layer_offsets, num_workers, max_tiles):
    """Host-only: -> (span_owner uint8[W * ceil(n_c/1024)], layer_listed int32[L]) as numpy arrays."""
    import numpy as np
    offs = [int(o) for o in layer_offsets]
    arr = (C.c_int64 * len(offs))(*offs)
    cfg = ObLambConfig(len(offs) - 1, arr, int(num_workers), 0, 0.9, 0.999, 0.9, 1e-6, 0.01, 0.3, 0.5, 4.0,
                       0.1, 0.0, 0, 0, 0)
    n_c = ob_lamb_padded_len_for(offs[-1], num_workers) // int(num_workers)
    owner = np.zeros(int(num_workers) * ((n_c + 1023) // 1024), dtype=np.uint8)
    listed = np.zeros(len(offs) - 1, dtype=np.int32)
    st = lib().ob_lamb_plan_split(C.byref(cfg), int(max_tiles), owner.ctypes.data, listed.ctypes.data)
    if st != OB_OK:
        raise ObLambError(st, "ob_lamb_plan_split")
    return owner, listed


def ob_lamb_plan_big_tiles(layer_offsets, num_workers, max_tiles):
    """Host-only: -> span_big uint8[W * ceil(n_c/1024)] as a numpy array."""
    import numpy as np
    offs = [int(o) for o in layer_offsets]
    arr = (C.c_int64 * len(offs))(*offs)
    cfg = ObLambConfig(len(offs) - 1, arr, int(num_workers), 0, 0.9, 0.999, 0.9, 1e-6, 0.01, 0.3, 0.5, 4.0,
                       0.1, 0.0, 0, 0, 0)
    n_c = ob_lamb_padded_len_for(offs[-1], num_workers) // int(num_workers)
    big = np.zeros(int(num_workers) * ((n_c + 1023) // 1024), dtype=np.uint8)
    st = lib().ob_lamb_plan_big_tiles(C.byref(cfg), int(max_tiles), big.ctypes.data)
    if st != OB_OK:
        raise ObLambError(st, "ob_lamb_plan_big_tiles")
    return big


def ob_lamb_destroy(ctx):
    lib().ob_lamb_destroy(ctx)


def ob_lamb_num_params(ctx):
    return int(lib().ob_lamb_num_params(ctx))


def ob_lamb_padded_len(ctx):
    return int(lib().ob_lamb_padded_len(ctx))


def ob_lamb_chunk_len(ctx):
    return int(lib().ob_lamb_chunk_len(ctx))


def ob_lamb_workspace_bytes(ctx):
    return int(lib().ob_lamb_workspace_bytes(ctx))


def ob_lamb_warmup_step(ctx, state, grad, lr, stream=None):
    _check(lib().ob_lamb_warmup_step(ctx, C.byref(state), _addr(grad), lr, _addr(stream)), ctx,
           "ob_lamb_warmup_step")


def ob_lamb_freeze(ctx, state, stream=None):
    _check(lib().ob_lamb_freeze(ctx, C.byref(state), _addr(stream)), ctx, "ob_lamb_freeze")


def ob_lamb_compress_local(ctx, state, grad, packed_out, scales_out, stream=None):
    _check(lib().ob_lamb_compress_local(ctx, C.byref(state), _addr(grad), _addr(packed_out),
                                        _addr(scales_out), _addr(stream)), ctx,
           "ob_lamb_compress_local")


def ob_lamb_server_reduce(ctx, state, packed_in, scales_in, packed_out, scale_out, stream=None):
    _check(lib().ob_lamb_server_reduce(ctx, C.byref(state), _addr(packed_in), _addr(scales_in),
                                       _addr(packed_out), _addr(scale_out), _addr(stream)), ctx,
           "ob_lamb_server_reduce")


def ob_lamb_server_reduce_static(num_workers, chunk_len, packed_in, scales_in, err_server, packed_out,
                                 scale_out, stream=None):
    _check(lib().ob_lamb_server_reduce_static(int(num_workers), int(chunk_len), _addr(packed_in),
                                              _addr(scales_in), _addr(err_server), _addr(packed_out),
                                              _addr(scale_out), _addr(stream)), None,
           "ob_lamb_server_reduce_static")


def ob_lamb_diag_copy(src, dst, n, stream=None):
    _check(lib().ob_lamb_diag_copy(_addr(src), _addr(dst), int(n), _addr(stream)), None, "ob_lamb_diag_copy")


def ob_lamb_static_max_chunk_len():
    return int(lib().ob_lamb_static_max_chunk_len())


def ob_lamb_layer_ratios(ctx, state, packed_all, server_scales, stream=None):
    _check(lib().ob_lamb_layer_ratios(ctx, C.byref(state), _addr(packed_all), _addr(server_scales),
                                      _addr(stream)), ctx, "ob_lamb_layer_ratios")


def ob_lamb_decompress_apply(ctx, state, packed_all, server_scales, lr, stream=None):
    _check(lib().ob_lamb_decompress_apply(ctx, C.byref(state), _addr(packed_all),
                                          _addr(server_scales), lr, _addr(stream)), ctx,
           "ob_lamb_decompress_apply")


def ob_lamb_ratios_apply(ctx, state, packed_all, server_scales, lr, stream=None):
    _check(lib().ob_lamb_ratios_apply(ctx, C.byref(state), _addr(packed_all), _addr(server_scales),
                                      lr, _addr(stream)), ctx, "ob_lamb_ratios_apply")


# ---- mixed-precision variant: ob_dtype values and the _lp entry points ------------------------
OB_F32, OB_F16, OB_BF16 = 0, 1, 2


def ob_lamb_warmup_step_lp(ctx, state, grad, grad_dtype, grad_scale, lr, x_lp, x_dtype, stream=None):
    _check(lib().ob_lamb_warmup_step_lp(ctx, C.byref(state), _addr(grad), int(grad_dtype), grad_scale,
                                        lr, _addr(x_lp), int(x_dtype), _addr(stream)), ctx,
           "ob_lamb_warmup_step_lp")


def ob_lamb_compress_local_lp(ctx, state, grad, grad_dtype, grad_scale, packed_out, scales_out,
                              stream=None):
    _check(lib().ob_lamb_compress_local_lp(ctx, C.byref(state), _addr(grad), int(grad_dtype),
                                           grad_scale, _addr(packed_out), _addr(scales_out),
                                           _addr(stream)), ctx, "ob_lamb_compress_local_lp")


def ob_lamb_decompress_apply_lp(ctx, state, packed_all, server_scales, lr, x_lp, x_dtype, stream=None):
    _check(lib().ob_lamb_decompress_apply_lp(ctx, C.byref(state), _addr(packed_all),
                                             _addr(server_scales), lr, _addr(x_lp), int(x_dtype),
                                             _addr(stream)), ctx, "ob_lamb_decompress_apply_lp")


def ob_lamb_ratios_apply_lp(ctx, state, packed_all, server_scales, lr, x_lp, x_dtype, stream=None):
    _check(lib().ob_lamb_ratios_apply_lp(ctx, C.byref(state), _addr(packed_all), _addr(server_scales),
                                         lr, _addr(x_lp), int(x_dtype), _addr(stream)), ctx,
           "ob_lamb_ratios_apply_lp")


def ob_lamb_fused_layers(ctx):
    return int(lib().ob_lamb_fused_layers(ctx))


def ob_lamb_fused_params(ctx):
    return int(lib().ob_lamb_fused_params(ctx))


def ob_lamb_warmup_fused_layers(ctx):
    return int(lib().ob_lamb_warmup_fused_layers(ctx))


def ob_lamb_big_tile_params(ctx):
    return int(lib().ob_lamb_big_tile_params(ctx))


def ob_lamb_warmup_fused_params(ctx):
    return int(lib().ob_lamb_warmup_fused_params(ctx))


def ob_lamb_momentum_dense(ctx, state, m_out, stream=None):
    _check(lib().ob_lamb_momentum_dense(ctx, C.byref(state), _addr(m_out), _addr(stream)), ctx,
           "ob_lamb_momentum_dense")


def make_vf_history(bits, scales, write_v):
    """ob_lamb_vf_history from the older momenta's sign-word and scale tensors, NEWEST FIRST."""
    assert len(bits) == len(scales) <= OB_VF_MAX_OLD
    h = ObLambVfHistory()
    h.n_old = len(bits)
    h.write_v = 1 if write_v else 0
    for i, (b, s) in enumerate(zip(bits, scales)):
        h.bits[i] = _addr(b)
        h.scales[i] = _addr(s)
    h._keep = (list(bits), list(scales))   # the tensors must outlive the call
    return h


def ob_lamb_ratios_apply_hist(ctx, state, packed_all, server_scales, lr, hist, stream=None):
    _check(lib().ob_lamb_ratios_apply_hist(ctx, C.byref(state), _addr(packed_all), _addr(server_scales), lr,
                                           None if hist is None else C.byref(hist), _addr(stream)),
           ctx, "ob_lamb_ratios_apply_hist")


def ob_lamb_ratios_apply_hist_lp(ctx, state, packed_all, server_scales, lr, hist, x_lp, x_dtype, stream=None):
    _check(lib().ob_lamb_ratios_apply_hist_lp(ctx, C.byref(state), _addr(packed_all), _addr(server_scales), lr,
                                              None if hist is None else C.byref(hist), _addr(x_lp), int(x_dtype),
                                              _addr(stream)),
           ctx, "ob_lamb_ratios_apply_hist_lp")


def ob_lamb_variance_dense(ctx, state, packed_all, server_scales, hist, v_out, stream=None):
    _check(lib().ob_lamb_variance_dense(ctx, C.byref(state), _addr(packed_all), _addr(server_scales),
                                        None if hist is None else C.byref(hist), _addr(v_out), _addr(stream)),
           ctx, "ob_lamb_variance_dense")


def ob_lamb_error_dense(ctx, state, err_out, stream=None):
    _check(lib().ob_lamb_error_dense(ctx, C.byref(state), _addr(err_out), _addr(stream)), ctx,
           "ob_lamb_error_dense")


def ob_lamb_server_error_dense(ctx, state, err_out, stream=None):
    _check(lib().ob_lamb_server_error_dense(ctx, C.byref(state), _addr(err_out), _addr(stream)), ctx,
           "ob_lamb_server_error_dense")


def ob_lamb_momentum_scale(ctx, state, stream=None):
    _check(lib().ob_lamb_momentum_scale(ctx, C.byref(state), _addr(stream)), ctx, "ob_lamb_momentum_scale")


def ob_lamb_check_device_status(ctx, stream=None):
    _check(lib().ob_lamb_check_device_status(ctx, _addr(stream)), ctx, "ob_lamb_check_device_status")


def ob_lamb_uses_single_pass(ctx):
    return bool(lib().ob_lamb_uses_single_pass(ctx))


def ob_lamb_server_single_pass(ctx):
    return int(lib().ob_lamb_server_single_pass(ctx))


def ob_lamb_profile_enable(ctx, on):
    _check(lib().ob_lamb_profile_enable(ctx, int(bool(on))), ctx, "ob_lamb_profile_enable")


def ob_lamb_profile_read(ctx):
    """-> {kernel name: (total ms, launches)} since the last read; synchronises."""
    cap = 32
    names = (C.c_char_p * cap)()
    ms = (C.c_double * cap)()
    cnt = (C.c_int64 * cap)()
    n = lib().ob_lamb_profile_read(ctx, cap, names, ms, cnt)
    return {names[i].decode(): (ms[i], int(cnt[i])) for i in range(min(n, cap))}
