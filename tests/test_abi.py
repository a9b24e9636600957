"""The C-ABI library loads and exports every symbol that include/onebitlamb.h declares; host-side
argument validation that returns before any HIP call.  No compute, no GPU."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "onebitlamb.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ob_lamb_[a-z_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def ob():
    import paper_2104_06069_amd as ob
    if not os.path.exists(ob.lib_path()):
        from paper_2104_06069_amd.build import build
        build()
    return ob


def test_header_declares_the_five_calls():
    names = declared_functions()
    for f in ("ob_lamb_warmup_step", "ob_lamb_compress_local", "ob_lamb_server_reduce",
              "ob_lamb_decompress_apply", "ob_lamb_layer_ratios"):
        assert f in names


def test_every_declared_symbol_is_exported(ob):
    lib = ob.lib()
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_padded_len_helper(ob):
    assert ob.ob_lamb_padded_len_for(1, 1) == 256
    assert ob.ob_lamb_padded_len_for(336232258, 64) == 336232448
    assert ob.ob_lamb_padded_len_for(336232258, 256) == 336265216
    assert ob.ob_lamb_padded_len_for(5, 0) == 0


def test_status_strings(ob):
    assert ob.ob_lamb_status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -5):
        assert ob.ob_lamb_status_string(s) not in ("ok", "unknown status")


def test_create_rejects_bad_config_before_touching_the_device(ob):
    lib = ob.lib()
    out = C.c_void_p()
    assert lib.ob_lamb_create(None, C.byref(out)) == -1
    offs = (C.c_int64 * 3)(0, 10, 5)                       # decreasing offsets
    cfg = ob.ObLambConfig(2, offs, 4, 0, 0.9, 0.999, 0.9, 1e-6, 0.01, 0.3, 0.5, 4.0, 0.1, 0.0)
    assert lib.ob_lamb_create(C.byref(cfg), C.byref(out)) == -2 and not out.value
    offs = (C.c_int64 * 3)(0, 5, 10)
    for field, val in (("num_workers", 0), ("server_chunk", 4), ("num_layers", 0),
                       ("beta1", float("nan")), ("r_min", 5.0)):
        cfg = ob.ObLambConfig(2, offs, 4, 0, 0.9, 0.999, 0.9, 1e-6, 0.01, 0.3, 0.5, 4.0, 0.1, 0.0)
        setattr(cfg, field, val)
        assert lib.ob_lamb_create(C.byref(cfg), C.byref(out)) == -2, field
    offs = (C.c_int64 * 3)(1, 5, 10)                       # offsets[0] != 0
    cfg = ob.ObLambConfig(2, offs, 4, 0, 0.9, 0.999, 0.9, 1e-6, 0.01, 0.3, 0.5, 4.0, 0.1, 0.0)
    assert lib.ob_lamb_create(C.byref(cfg), C.byref(out)) == -2


def test_null_context_is_rejected(ob):
    lib = ob.lib()
    st = ob.ObLambState()
    assert lib.ob_lamb_compress_local(None, C.byref(st), None, None, None, None) == -1
    assert lib.ob_lamb_layer_ratios(None, C.byref(st), None, None, None) == -1
    assert ob.ob_lamb_num_params(None) == 0
    lib.ob_lamb_destroy(None)
    assert lib.ob_lamb_compress_local_lp(None, C.byref(st), None, 1, 1.0, None, None, None) == -1
    assert lib.ob_lamb_ratios_apply_lp(None, C.byref(st), None, None, 1e-3, None, 0, None) == -1
    assert lib.ob_lamb_warmup_step_lp(None, C.byref(st), None, 2, 1.0, 1e-3, None, 0, None) == -1


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2104_06069_amd")
    for d, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                txt = open(os.path.join(d, f)).read()
                assert "obref" not in txt and "oracle" not in txt.lower().replace("oracle-free", ""), f
