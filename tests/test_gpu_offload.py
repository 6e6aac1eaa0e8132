"""GPU parity: the offloaded step.  Chunking and overlap must not change a bit
against the resident GPU step (elements are independent); the resident step
carries the floating-point tolerance against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2504_09983_amd import synth, zc
from tests.gpu_util import DEV, HP, assert_state_close, dev_f32, dev_u16, host_f32, host_u16, sync

pytestmark = pytest.mark.gpu


def pinned(a: np.ndarray) -> torch.Tensor:
    t = torch.empty(a.size, dtype=torch.float32, pin_memory=True)
    t.numpy()[:] = a
    return t


def offload_vs_resident(n, n_res, chunk_bytes, nbuf, steps=2, g_bf16=True, zero_copy=False):
    p0 = synth.host_params(n, 21)
    m0 = synth.host_normal(n, 1e-4, 22)
    v0 = np.abs(synth.host_normal(n, 1e-7, 23))
    # resident reference on the GPU
    rp, rm, rv = dev_f32(p0), dev_f32(m0), dev_f32(v0)
    rout = torch.zeros(n, dtype=torch.int16, device=DEV)
    # offloaded state
    dp, dm, dv = dev_f32(p0[:n_res]), dev_f32(m0[:n_res]), dev_f32(v0[:n_res])
    hp_, hm_, hv_ = pinned(p0[n_res:]), pinned(m0[n_res:]), pinned(v0[n_res:])
    oout = torch.zeros(n, dtype=torch.int16, device=DEV)
    # oracle state
    op, om, ov = p0.copy(), m0.copy(), v0.copy()
    oo = np.zeros(n, np.uint16)

    ctx = zc.offload_create(chunk_bytes, nbuf)
    old = zc.tune_get("offload.zero_copy")
    zc.tune_set("offload.zero_copy", int(zero_copy))   # 0 ring, 1 zero-copy, 2 staged reads + direct writes
    try:
        for t in range(1, steps + 1):
            g = synth.host_grads_f32(n, t)
            if g_bf16:
                g = oracle.cast_bf16(g)
                dg = dev_u16(g)
            else:
                dg = dev_f32(g)
            dt = zc.BF16 if g_bf16 else zc.F32
            hp = zc.hparams(step=t, **HP)
            zc.adam_step(rp, rm, rv, dg, dt, n, hp, bf16_out=rout)
            ctx.adam_step(dp if n_res else None, dm if n_res else None, dv if n_res else None, n_res,
                          hp_ if n > n_res else None, hm_ if n > n_res else None,
                          hv_ if n > n_res else None, n - n_res, dg, dt, hp, bf16_out_dev=oout)
            oracle.adam_step(op, om, ov, g, step=t, bf16_out=oo, **HP)
        sync()
    finally:
        zc.tune_set("offload.zero_copy", old)
        ctx.destroy()
    for res, dev_part, host_part in ((rp, dp, hp_), (rm, dm, hm_), (rv, dv, hv_)):
        r = host_f32(res)
        assert np.array_equal(r[:n_res].view(np.uint32), host_f32(dev_part).view(np.uint32))
        assert np.array_equal(r[n_res:].view(np.uint32), host_part.numpy().view(np.uint32))
    assert torch.equal(rout, oout)
    assert_state_close(host_f32(rp), host_f32(rm), host_f32(rv), op, om, ov, tag="offload")
    assert np.array_equal(host_u16(oout), oracle.cast_bf16(host_f32(rp)))


@pytest.mark.parametrize("zero_copy", [0, 1, 2])
@pytest.mark.parametrize("frac", [0.0, 0.25, 0.5, 1.0])
def test_offload_equals_resident_fractions(frac, zero_copy):
    n = 3 * (1 << 20) + 4099
    n_res = int(frac * n) // 1024 * 1024
    offload_vs_resident(n, n_res, 1 << 20, 3, zero_copy=zero_copy)


@pytest.mark.parametrize("transport", [0, 2])
@pytest.mark.parametrize("nbuf", [1, 2, 3, 5])
@pytest.mark.parametrize("chunk_bytes", [4096, 1 << 16])
def test_offload_ring_sizes(nbuf, chunk_bytes, transport):
    # many chunks through few slots: every slot is reused several times
    n = 40 * (chunk_bytes // 4) // 3 + 17
    offload_vs_resident(n, 1024, chunk_bytes, nbuf, steps=2, zero_copy=transport)


def test_offload_fp32_grads_and_single_partial_chunk():
    offload_vs_resident(1000, 0, 1 << 20, 3, g_bf16=False)       # one partial chunk
    offload_vs_resident((1 << 18), 0, 1 << 20, 2, g_bf16=False)  # exactly one full chunk


def test_offload_64mib_chunks():
    """The reference chunk size: 64 MiB per array, 3 slots, 2.5 chunks."""
    n = (16 << 20) * 2 + (8 << 20) + 5
    offload_vs_resident(n, 0, 64 << 20, 3, steps=1)
    offload_vs_resident(n, 0, 64 << 20, 3, steps=1, zero_copy=2)


def test_offload_zero_copy_mode():
    offload_vs_resident((1 << 20) + 77, 4096, 1 << 20, 3, zero_copy=True)
    offload_vs_resident((1 << 22) + 3, 0, 1 << 20, 3, zero_copy=True, g_bf16=False, steps=3)
    # misaligned host views force the scalar kernel through the link
    n = 50001
    base = [torch.zeros(n + 1, dtype=torch.float32, pin_memory=True) for _ in range(3)]
    p0 = synth.host_params(n, 41)
    base[0].numpy()[1:] = p0
    views = [b[1:] for b in base]
    g = oracle.cast_bf16(synth.host_grads_f32(n, 1))
    dg = dev_u16(g)
    out = torch.zeros(n, dtype=torch.int16, device=DEV)
    ctx = zc.offload_create(1 << 16, 2)
    old = zc.tune_get("offload.zero_copy")
    try:
        for mode in (1, 0, 2):
            zc.tune_set("offload.zero_copy", mode)
            for b in base:
                b.zero_()
            base[0].numpy()[1:] = p0
            ctx.adam_step(None, None, None, 0, *views, n, dg, zc.BF16, zc.hparams(step=1, **HP),
                          bf16_out_dev=out)
            sync()
            op, om, ov = p0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
            oracle.adam_step(op, om, ov, g, step=1, **HP)
            assert_state_close(views[0].numpy(), views[1].numpy(), views[2].numpy(), op, om, ov,
                               steps=1, tag=f"misaligned host, zero_copy={mode}")
            assert all(float(b[0]) == 0.0 for b in base)
    finally:
        zc.tune_set("offload.zero_copy", old)
        ctx.destroy()


def test_offload_rejects_unpinned_host_memory():
    n = 4096
    ctx = zc.offload_create(1 << 16, 2)
    pageable = [torch.zeros(n, dtype=torch.float32) for _ in range(3)]
    dg = torch.zeros(n, dtype=torch.int16, device=DEV)
    with pytest.raises(zc.ZcError) as ei:
        ctx.adam_step(None, None, None, 0, *pageable, n, dg, zc.BF16, zc.hparams(step=1, **HP))
    assert ei.value.status == zc.ERR_INVALID_ARG and "pinned" in ei.value.message
    # the context is still usable afterwards
    pin = [torch.zeros(n, dtype=torch.float32, pin_memory=True) for _ in range(3)]
    ctx.adam_step(None, None, None, 0, *pin, n, dg, zc.BF16, zc.hparams(step=1, **HP))
    sync()
    ctx.destroy()


def test_resume_after_round_trip_through_host():
    """5 + 5 steps with the state copied to the host and back in between == 10 steps."""
    n = 50000
    p0 = synth.host_params(n, 31)
    a = [dev_f32(p0), dev_f32(np.zeros(n)), dev_f32(np.zeros(n))]
    b = [t.clone() for t in a]
    for t in range(1, 11):
        dg = dev_f32(synth.host_grads_f32(n, t))
        hp = zc.hparams(step=t, **HP)
        zc.adam_step(*a, dg, zc.F32, n, hp)
        zc.adam_step(*b, dg, zc.F32, n, hp)
        if t == 5:
            sync()
            b = [x.cpu().to(DEV) for x in b]
    sync()
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("transport", [0, 1, 2])
def test_offload_skip_flag_leaves_host_and_device_state_untouched(transport):
    n, n_res = (1 << 19) + 13, 4096
    p0, m0, v0 = synth.host_params(n, 71), synth.host_normal(n, 1e-4, 72), np.abs(synth.host_normal(n, 1e-7, 73))
    dp, dm, dv = dev_f32(p0[:n_res]), dev_f32(m0[:n_res]), dev_f32(v0[:n_res])
    hp_, hm_, hv_ = pinned(p0[n_res:]), pinned(m0[n_res:]), pinned(v0[n_res:])
    dg = dev_u16(oracle.cast_bf16(synth.host_grads_f32(n, 1)))
    out = torch.full((n,), 0x3C3C, dtype=torch.int16, device=DEV)
    flag = torch.ones(1, dtype=torch.int32, device=DEV)
    ctx = zc.offload_create(1 << 18, 2)
    old = zc.tune_get("offload.zero_copy")
    zc.tune_set("offload.zero_copy", transport)
    try:
        ctx.adam_step(dp, dm, dv, n_res, hp_, hm_, hv_, n - n_res, dg, zc.BF16, zc.hparams(step=1, **HP),
                      bf16_out_dev=out, skip_flag=flag)
        sync()
        for host, dev, ref in ((hp_, dp, p0), (hm_, dm, m0), (hv_, dv, v0)):
            assert np.array_equal(host.numpy().view(np.uint32), ref[n_res:].view(np.uint32))
            assert np.array_equal(host_f32(dev).view(np.uint32), ref[:n_res].view(np.uint32))
        assert (out == 0x3C3C).all()
        # and with the flag cleared the same call does the step
        flag.zero_()
        ctx.adam_step(dp, dm, dv, n_res, hp_, hm_, hv_, n - n_res, dg, zc.BF16, zc.hparams(step=1, **HP),
                      bf16_out_dev=out, skip_flag=flag)
        sync()
        assert not np.array_equal(hp_.numpy(), p0[n_res:]) and (out != 0x3C3C).any()
    finally:
        zc.tune_set("offload.zero_copy", old)
        ctx.destroy()


@pytest.mark.parametrize("transport", [0, 2])
@pytest.mark.parametrize("nbuf", [1, 2, 3])
def test_ring_slots_poisoned_after_use_change_nothing(transport, nbuf):
    """Every slot is overwritten with garbage as soon as its chunk has left it; with all
    fences in place the next chunk's copy lands after that and no result bit changes."""
    old = {k: zc.tune_get(k) for k in ("offload.poison", "offload.max_ahead")}
    try:
        for ahead in (1, 0):
            zc.tune_set("offload.poison", 1)
            zc.tune_set("offload.max_ahead", ahead)
            chunk = 1 << 16
            n = 25 * (chunk // 4) + 333
            offload_vs_resident(n, 2048, chunk, nbuf, steps=2, zero_copy=transport)
    finally:
        for k, val in old.items():
            zc.tune_set(k, val)


def test_zero_copy_offloaded_step_replays_from_a_hip_graph():
    """The default transport is one kernel launch over pinned host arrays: it can be captured
    (no copy, no event wait on the host, no allocation) and every replay advances the host-resident
    state exactly as an eager call does."""
    n, n_res = (1 << 18) + 77, 8192
    p0, m0, v0 = synth.host_params(n, 81), synth.host_normal(n, 1e-4, 82), np.abs(synth.host_normal(n, 1e-7, 83))
    dg = dev_u16(oracle.cast_bf16(synth.host_grads_f32(n, 5)))
    hp = zc.hparams(step=4, **HP)

    def make():
        return ([dev_f32(p0[:n_res]), dev_f32(m0[:n_res]), dev_f32(v0[:n_res])],
                [pinned(p0[n_res:]), pinned(m0[n_res:]), pinned(v0[n_res:])],
                torch.zeros(n, dtype=torch.int16, device=DEV))

    ctx = zc.offload_create(1 << 18, 2)
    assert zc.tune_get("offload.zero_copy") == 1
    try:
        dev_a, host_a, out_a = make()          # driven by the graph
        dev_b, host_b, out_b = make()          # driven by eager calls

        def step(dev, host, out):
            ctx.adam_step(*dev, n_res, *host, n - n_res, dg, zc.BF16, hp, bf16_out_dev=out)

        warm = make()
        step(*warm)
        sync()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step(dev_a, host_a, out_a)
        sync()
        for replay in range(3):
            graph.replay()
            step(dev_b, host_b, out_b)
            sync()
            for x, y in zip(dev_a + [out_a], dev_b + [out_b]):
                assert torch.equal(x, y), f"replay {replay}"
            for x, y in zip(host_a, host_b):
                assert np.array_equal(x.numpy().view(np.uint32), y.numpy().view(np.uint32)), f"replay {replay}"
            _ = (dev_a[0] * 2).sum().item()    # unrelated eager work and a sync between replays
        assert not np.array_equal(host_a[0].numpy(), p0[n_res:])       # the state did move
    finally:
        ctx.destroy()
