"""zc_grad_sqnorm_static (the entry point that never allocates: its partial sums live in a
fixed array inside the library's device image) against zc_grad_sqnorm, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_2504_09983_amd import synth, zc
from tests.gpu_util import DEV, sync

pytestmark = pytest.mark.gpu


def _both(g, dtype, n):
    out = {}
    for name, fn in (("alloc", zc.grad_sqnorm), ("static", zc.grad_sqnorm_static)):
        norm = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
        flag = torch.full((1,), -1, dtype=torch.int32, device=DEV)
        fn(g, dtype, n, norm, flag)
        sync()
        out[name] = (norm.cpu().numpy().view(np.uint32)[0], int(flag.item()))
    return out


def test_static_scratch_norm_equals_allocating_norm_twice_in_a_row():
    """Two calls in a row, the second with a smaller input: the array keeps the first call's
    partial sums, which the second call must not read."""
    big, small = (1 << 24) + 4099, 70_001
    g = torch.empty(big, dtype=torch.bfloat16, device=DEV)
    synth.device_normal_(g, synth.G_STD, seed=2001)
    for n in (big, small):
        r = _both(g, zc.BF16, n)
        assert r["static"] == r["alloc"], (n, r)
        want, bad = oracle.grad_sqnorm(g[:n].view(torch.int16).cpu().numpy().view(np.uint16))
        got = np.array([r["static"][0]], np.uint32).view(np.float32)[0]
        assert bad == r["static"][1] == 0
        assert abs(float(got) - want) <= 1.3e-7 * want


def test_static_scratch_norm_fp32_flag_and_empty_input():
    n = 3_000_003
    g = torch.empty(n, dtype=torch.float32, device=DEV)
    synth.device_normal_(g, synth.G_STD, seed=2002)
    r = _both(g, zc.F32, n)
    assert r["static"] == r["alloc"] and r["static"][1] == 0
    g[n - 5] = float("inf")
    r = _both(g, zc.F32, n)
    assert r["static"][1] == r["alloc"][1] == 1
    # a smaller, finite prefix right after the flagged call: the flag must not stick
    r = _both(g, zc.F32, 1000)
    assert r["static"] == r["alloc"] and r["static"][1] == 0
    r = _both(g, zc.F32, 0)
    assert r["static"] == r["alloc"] == (0, 0)
    # unaligned start: the one-element-per-lane kernel
    r = _both(g[1:], zc.F32, 4097)
    assert r["static"] == r["alloc"]


def test_static_scratch_norm_rejects_what_the_allocating_call_rejects():
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    with pytest.raises(zc.ZcError) as e:
        zc.grad_sqnorm_static(norm, zc.F32, (1 << 40) + 1, norm, flag)
    assert e.value.status == zc.ERR_UNSUPPORTED and "2^40" in e.value.message
    with pytest.raises(zc.ZcError) as e:
        zc.grad_sqnorm_static(None, zc.F32, 8, norm, flag)
    assert e.value.status == zc.ERR_INVALID_ARG
