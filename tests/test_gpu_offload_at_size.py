"""GPU parity of the offloaded step at the size adaptive offloading exists for (paper:
Adaptive offloading, Algorithm 2): more than 2^32 streamed elements (51.5 GB of pinned host
memory), resident fractions 0, 1/4 and 1/2, 64 MiB chunks and 3 slots.

Offloaded == resident, bit for bit, over every element (device prefix and host suffix, p, m,
v and the bf16 copy), and the resident result against the oracle on windows: both ends,
around the resident/streamed boundary, around element 2^32 of the streamed part and of the
whole partition, around chunk and slot-reuse boundaries, and random ones."""
import numpy as np
import pytest
import torch

import oracle
from paper_2504_09983_amd import synth, zc
from tests.gpu_util import DEV, HP, assert_state_close, host_f32, host_u16, sync

pytestmark = pytest.mark.gpu

N_STREAMED = (1 << 32) + 4099
CHUNK = 64 << 20            # bytes per fp32 array per chunk
PIECE = 1 << 28             # elements per host <-> device comparison piece
WIDTH = 1 << 13


def _pinned_triplet(n):
    try:
        bufs = [zc.host_alloc(4 * n) for _ in range(3)]
    except zc.ZcError as e:                      # a box that pins less than 51.5 GB
        pytest.skip(f"cannot pin 3 x {4 * n} bytes on this host: {e}")
    return bufs


def _windows(n, n_res, seed):
    rng = np.random.default_rng(seed)
    ce = CHUNK // 4
    marks = [0, n - WIDTH, n_res, n_res + (1 << 32), 1 << 32, n_res + ce, n_res + 3 * ce, n_res + 4 * ce,
             n_res + 255 * ce, n - 4099]
    starts = set()
    for b in marks:
        s = min(max(0, b - WIDTH // 2), n - WIDTH)
        starts.add(s)
    starts.update(int(x) for x in rng.integers(0, n - WIDTH, size=12))
    return sorted(starts)


def _copy_host_to(dst_dev, host_np):
    """Bring a pinned host array to the device in pieces (plain torch copies)."""
    for s in range(0, host_np.size, PIECE):
        e = min(host_np.size, s + PIECE)
        dst_dev[s:e].copy_(torch.from_numpy(host_np[s:e]))


def _host_equals(dev_ref, host_np, what):
    for s in range(0, host_np.size, PIECE):
        e = min(host_np.size, s + PIECE)
        got = torch.from_numpy(host_np[s:e]).to(DEV)
        assert torch.equal(got.view(torch.int32), dev_ref[s:e].view(torch.int32)), f"{what}: piece at {s}"
        del got


@pytest.mark.parametrize("frac", [0.0, 0.25, 0.5])
def test_zero_copy_offload_with_more_than_2_to_32_streamed_elements(frac):
    n_str = N_STREAMED
    n_res = int(frac / (1.0 - frac) * n_str) // 1024 * 1024      # f = n_res / (n_res + n_str)
    n = n_res + n_str
    print(f"f={frac}: n={n} resident={n_res} streamed={n_str}", flush=True)
    bufs = _pinned_triplet(n_str)
    hp_, hm_, hv_ = (b.numpy("float32") for b in bufs)
    # reference (all resident) state: p ~ N(0, 0.02) from the seeded generator, m = v = 0
    rp = torch.empty(n, dtype=torch.float32, device=DEV)
    synth.device_normal_(rp, synth.P_STD, seed=3)
    rm = torch.zeros(n, dtype=torch.float32, device=DEV)
    rv = torch.zeros(n, dtype=torch.float32, device=DEV)
    # offloaded state: the same values, prefix on the device, suffix in pinned host memory
    dp, dm, dv = (rp[:n_res].clone(), rm[:n_res].clone(), rv[:n_res].clone()) if n_res else (None, None, None)
    for s in range(0, n_str, PIECE):
        e = min(n_str, s + PIECE)
        torch.from_numpy(hp_[s:e]).copy_(rp[n_res + s:n_res + e])
        hm_[s:e] = 0.0
        hv_[s:e] = 0.0
    print("state placed", flush=True)
    g = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    rout = torch.zeros(n, dtype=torch.int16, device=DEV)
    oout = torch.zeros(n, dtype=torch.int16, device=DEV)
    wins = _windows(n, n_res, seed=int(frac * 100) + 1)
    ohost = [(host_f32(rp[s:s + WIDTH]).copy(), np.zeros(WIDTH, np.float32), np.zeros(WIDTH, np.float32),
              np.zeros(WIDTH, np.uint16)) for s in wins]
    ctx = zc.offload_create(CHUNK, 3)
    assert zc.tune_get("offload.zero_copy") == 1
    steps = 2
    try:
        for t in range(1, steps + 1):
            synth.device_normal_(g, synth.G_STD, seed=2000 + t)
            hp = zc.hparams(step=t, **HP)
            zc.adam_step(rp, rm, rv, g, zc.BF16, n, hp, bf16_out=rout)
            ctx.adam_step(dp, dm, dv, n_res, bufs[0], bufs[1], bufs[2], n_str, g, zc.BF16, hp, bf16_out_dev=oout)
            sync()
            for s, (op, om, ov, oo) in zip(wins, ohost):
                oracle.adam_step(op, om, ov, host_u16(g[s:s + WIDTH]), step=t, bf16_out=oo, **HP)
            print(f"step {t} done", flush=True)
    finally:
        ctx.destroy()
    # offloaded == resident over every element
    assert torch.equal(rout, oout), "bf16 copy"
    if n_res:
        for name, r, d in (("p", rp, dp), ("m", rm, dm), ("v", rv, dv)):
            assert torch.equal(r[:n_res].view(torch.int32), d.view(torch.int32)), f"resident prefix of {name}"
    for name, r, h in (("p", rp, hp_), ("m", rm, hm_), ("v", rv, hv_)):
        _host_equals(r[n_res:], h, f"streamed suffix of {name}")
    print("offloaded == resident", flush=True)
    # resident == oracle on the windows
    for s, (op, om, ov, oo) in zip(wins, ohost):
        gp, gm, gv = (host_f32(x[s:s + WIDTH]) for x in (rp, rm, rv))
        assert_state_close(gp, gm, gv, op, om, ov, steps=steps, tag=f"f={frac} window@{s}")
        assert np.array_equal(host_u16(rout[s:s + WIDTH]), oracle.cast_bf16(gp)), f"window@{s}: bf16 copy"
    del hp_, hm_, hv_
    for b in bufs:
        b.free()
    del rp, rm, rv, dp, dm, dv, g, rout, oout
    torch.cuda.empty_cache()


@pytest.mark.parametrize("transport", [0, 2])
def test_staged_ring_over_more_than_2_to_30_elements(transport):
    """The 64 MiB x 3 ring (and its staged-reads variant) over 2^30 + 2^24 + 5 streamed elements:
    65 chunks through 3 slots, every slot reused 21 times, against the resident step."""
    n_str = (1 << 30) + (1 << 24) + 5
    n_res = 1 << 20
    n = n_res + n_str
    bufs = _pinned_triplet(n_str)
    hp_, hm_, hv_ = (b.numpy("float32") for b in bufs)
    rp = torch.empty(n, dtype=torch.float32, device=DEV)
    synth.device_normal_(rp, synth.P_STD, seed=5)
    rm = torch.zeros(n, dtype=torch.float32, device=DEV)
    rv = torch.zeros(n, dtype=torch.float32, device=DEV)
    dp, dm, dv = rp[:n_res].clone(), rm[:n_res].clone(), rv[:n_res].clone()
    for s in range(0, n_str, PIECE):
        e = min(n_str, s + PIECE)
        torch.from_numpy(hp_[s:e]).copy_(rp[n_res + s:n_res + e])
        hm_[s:e] = 0.0
        hv_[s:e] = 0.0
    g = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    rout = torch.zeros(n, dtype=torch.int16, device=DEV)
    oout = torch.zeros(n, dtype=torch.int16, device=DEV)
    ctx = zc.offload_create(CHUNK, 3)
    old = zc.tune_get("offload.zero_copy")
    zc.tune_set("offload.zero_copy", transport)
    try:
        for t in (1, 2):
            synth.device_normal_(g, synth.G_STD, seed=2100 + t)
            hp = zc.hparams(step=t, **HP)
            zc.adam_step(rp, rm, rv, g, zc.BF16, n, hp, bf16_out=rout)
            ctx.adam_step(dp, dm, dv, n_res, bufs[0], bufs[1], bufs[2], n_str, g, zc.BF16, hp, bf16_out_dev=oout)
            sync()
            print(f"transport {transport} step {t} done", flush=True)
    finally:
        zc.tune_set("offload.zero_copy", old)
        ctx.destroy()
    assert torch.equal(rout, oout), "bf16 copy"
    for name, r, d in (("p", rp, dp), ("m", rm, dm), ("v", rv, dv)):
        assert torch.equal(r[:n_res].view(torch.int32), d.view(torch.int32)), f"resident prefix of {name}"
    for name, r, h in (("p", rp, hp_), ("m", rm, hm_), ("v", rv, hv_)):
        _host_equals(r[n_res:], h, f"streamed suffix of {name}")
    del hp_, hm_, hv_
    for b in bufs:
        b.free()
    del rp, rm, rv, dp, dm, dv, g, rout, oout
    torch.cuda.empty_cache()
