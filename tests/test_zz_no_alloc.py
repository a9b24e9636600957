"""ob_lamb_server_reduce_static -- Algorithm 1 line 10 for callers that cannot allocate -- against
ob_lamb_server_reduce, through the C ABI: two calls in a row on the same GPU, the second with a
smaller chunk (the static scratch then still holds the first call's partial sums).

Collected last on purpose (file name): a failure here must not hide the tests before it.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

import paper_2104_06069_amd as ob  # noqa: E402
from tests.refstep import HYPER  # noqa: E402

pytestmark = pytest.mark.gpu


def _inputs(seed, W, n_c, dev):
    g = torch.Generator(device=dev); g.manual_seed(seed)
    words = torch.randint(-2 ** 31, 2 ** 31, (W * (n_c // 32),), generator=g, device=dev, dtype=torch.int32)
    scales = (1e-4 * (0.5 + torch.rand(W, generator=g, device=dev))).float()
    err = (5e-5 * torch.randn(n_c, generator=g, device=dev)).float()
    return words, scales, err


def _context_call(W, n_c, words, scales, err, flags):
    """The existing entry point on a context whose only chunk layout matters: W chunks of n_c."""
    ctx = ob.ob_lamb_create([0, W * n_c], W, 0, flags=flags, **HYPER)
    assert ob.ob_lamb_chunk_len(ctx) == n_c
    e = err.clone()
    out = torch.zeros(n_c // 32, device=err.device, dtype=torch.int32)
    s = torch.zeros(1, device=err.device)
    ob.ob_lamb_server_reduce(ctx, ob.make_state(err_server=e), words, scales, out, s,
                             torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    ob.ob_lamb_check_device_status(ctx, torch.cuda.current_stream().cuda_stream)
    ob.ob_lamb_destroy(ctx)
    return out, s, e


def test_static_server_reduce_matches_the_context_call_twice_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    stream = torch.cuda.current_stream().cuda_stream
    # first a chunk of 1027 tiles with a ragged last tile, then a much smaller one (3 tiles + tail)
    for call, (W, n_c) in enumerate(((8, 1024 * 1026 + 768), (5, 1024 * 3 + 256))):
        words, scales, err = _inputs(100 + call, W, n_c, dev)
        e = err.clone()
        out = torch.zeros(n_c // 32, device=dev, dtype=torch.int32)
        s = torch.zeros(1, device=dev)
        torch.cuda.synchronize()
        print(f"static server_reduce: call {call}, W={W}, n_c={n_c}", flush=True)
        ob.ob_lamb_server_reduce_static(W, n_c, words, scales, e, out, s, stream)
        torch.cuda.synchronize()
        # same kernels (three-kernel form): bit for bit
        out3, s3, e3 = _context_call(W, n_c, words, scales, err, ob.OB_CFG_TWO_PASS_COMPRESS)
        assert torch.equal(out, out3), f"call {call}: sign words"
        assert torch.equal(s.view(torch.int32), s3.view(torch.int32)), f"call {call}: scale"
        assert torch.equal(e.view(torch.int32), e3.view(torch.int32)), f"call {call}: server error"
        # whatever form the library selects by default (one kernel with a chunk barrier here):
        # scale within 1e-6 relative; words and errors equal wherever the scale's bits are
        outd, sd, ed = _context_call(W, n_c, words, scales, err, 0)
        assert abs(float(s) - float(sd)) <= 1e-6 * abs(float(sd))
        if torch.equal(s.view(torch.int32), sd.view(torch.int32)):
            assert torch.equal(out, outd) and torch.equal(e.view(torch.int32), ed.view(torch.int32))
        assert float(s) > 0 and int(torch.count_nonzero(out)) > 0


def test_static_server_reduce_rejects_what_it_cannot_hold():
    if not torch.cuda.is_available():
        pytest.skip("no GPU visible")
    dev = torch.device("cuda:0")
    cap = ob.ob_lamb_static_max_chunk_len()
    assert cap == 1 << 25
    a = torch.zeros(64, device=dev)
    i = torch.zeros(64, device=dev, dtype=torch.int32)
    for W, n_c, status in ((4, cap + 256, -6), (4, 1000, -2), (0, 1024, -2), (4, 0, -2)):
        with pytest.raises(ob.ObLambError) as ei:
            ob.ob_lamb_server_reduce_static(W, n_c, i, a, a, i, a, None)
        assert ei.value.status == status
    with pytest.raises(ob.ObLambError) as ei:
        ob.ob_lamb_server_reduce_static(4, 1024, None, a, a, i, a, None)
    assert ei.value.status == -1
    with pytest.raises(ob.ObLambError) as ei:
        ob.ob_lamb_server_reduce_static(4, 1024, i.data_ptr() + 4, a, a, i, a, None)
    assert ei.value.status == -3
    assert "static scratch" in ob.ob_lamb_status_string(-6)
