"""GPU parity of the packed optimizer state: pack / unpack bit for bit against the oracle's
layout, and the packed step element by element against the CPU oracle's AdamW (the packed
array is copied to the host and taken apart by the oracle's own unpack, so the library's
unpack kernel is not trusted on its own), plus bit-identity with the three-array step."""
import numpy as np
import pytest
import torch

import oracle
from oracle import layout
from paper_2504_09983_amd import synth, zc
from tests.gpu_util import (DEV, HP, assert_state_close, bf16_ulp_diff, dev_f32, dev_u16,
                            host_f32, host_u16, sync)

pytestmark = pytest.mark.gpu

G = zc.PACKED_GRANULE


def dev_state(n, fill=None):
    """A 128-byte aligned device array for the packed state of n elements."""
    t = torch.empty(zc.packed_state_numel(n), dtype=torch.float32, device=DEV)
    assert t.data_ptr() % 128 == 0
    if fill is not None:
        t.fill_(fill)
    return t


def test_granule_and_length_agree_with_the_oracle():
    assert G == 8192
    for n in (0, 1, G - 1, G, G + 1, 5 * G, 5 * G + 17, 8_819_213_312):
        assert zc.packed_state_numel(n) == layout.packed_state_numel(n, G)
    assert zc.packed_state_numel(-3) == 0


@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, G - 1, G, G + 1, 3 * G + 4097, (1 << 20) + 3])
@pytest.mark.parametrize("offset", [0, 1])
def test_pack_and_unpack_match_the_oracle_layout(n, offset):
    rng = np.random.default_rng(n + offset)
    p, m, v = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    dp, dm, dv = (dev_f32(np.concatenate([np.zeros(offset, np.float32), a]))[offset:] for a in (p, m, v))
    state = dev_state(n, fill=float("nan"))            # the padding must come out as zeros
    zc.state_pack(dp, dm, dv, n, state)
    sync()
    want = layout.pack_state(p, m, v, G)
    assert np.array_equal(host_f32(state).view(np.uint32), want.view(np.uint32))
    # unpack: all three, and each alone with the others left untouched
    outs = [torch.full((n + offset,), 7.0, dtype=torch.float32, device=DEV)[offset:] for _ in range(3)]
    zc.state_unpack(state, n, *outs)
    sync()
    for got, ref in zip(outs, (p, m, v)):
        assert np.array_equal(host_f32(got).view(np.uint32), ref.view(np.uint32))
    for which, ref in enumerate((p, m, v)):
        outs = [torch.full((n,), 7.0, dtype=torch.float32, device=DEV) for _ in range(3)]
        args = [outs[k] if k == which else None for k in range(3)]
        zc.state_unpack(state, n, *args)
        sync()
        assert np.array_equal(host_f32(outs[which]).view(np.uint32), ref.view(np.uint32))
        assert all((host_f32(outs[k]) == 7.0).all() for k in range(3) if k != which)


def test_pack_with_missing_sources_gives_zeros():
    n = 2 * G + 5
    p = synth.host_params(n, 3)
    state = dev_state(n, fill=float("nan"))
    zc.state_pack(dev_f32(p), None, None, n, state)
    sync()
    want = layout.pack_state(p, np.zeros(n, np.float32), np.zeros(n, np.float32), G)
    assert np.array_equal(host_f32(state).view(np.uint32), want.view(np.uint32))


def run_packed(n, steps, *, g_bf16, with_out=True, seed=1, mode=zc.ADAMW, ranges=(), g_offset=0,
               m0=None, v0=None, poison_padding=True):
    """`steps` steps of the packed update next to the oracle's AdamW on separate arrays."""
    p = synth.host_params(n, seed)
    m = np.zeros(n, np.float32) if m0 is None else m0.copy()
    v = np.zeros(n, np.float32) if v0 is None else v0.copy()
    out = np.zeros(n, np.uint16)
    packed0 = layout.pack_state(p, m, v, G)
    pad = np.ones(packed0.size, dtype=bool)
    for k in range(-(-n // G)):
        cnt = min(G, n - k * G)
        for a in range(3):
            pad[3 * k * G + a * G:3 * k * G + a * G + cnt] = False
    if poison_padding:
        packed0.view(np.uint32)[pad] = 0x7FC0DEAD            # the step must leave the padding alone
    state = dev_state(n)
    state.copy_(dev_f32(packed0))
    dout = torch.zeros(n + g_offset, dtype=torch.int16, device=DEV)[g_offset:]
    for t in range(1, steps + 1):
        g = synth.host_grads_f32(n, t + 100 * seed)
        if g_bf16:
            g = oracle.cast_bf16(g)
            dg = dev_u16(np.concatenate([np.zeros(g_offset, np.uint16), g]))[g_offset:]
        else:
            dg = dev_f32(np.concatenate([np.zeros(g_offset, np.float32), g]))[g_offset:]
        hp = zc.hparams(step=t, mode=mode, **HP)
        zc.adam_step_packed(state, dg, zc.BF16 if g_bf16 else zc.F32, n, hp, ranges=ranges,
                            bf16_out=dout if with_out else None)
        oracle.adam_step_groups(p, m, v, g, ranges=ranges, step=t, mode=mode,
                                bf16_out=out if with_out else None, **HP)
    sync()
    packed = host_f32(state)
    assert np.array_equal(packed.view(np.uint32)[pad], packed0.view(np.uint32)[pad]), "padding was written"
    packed = packed.copy()
    packed[pad] = 0
    gp, gm, gv = layout.unpack_state(packed, n, G)
    return (gp, gm, gv, host_u16(dout)), (p, m, v, out)


def check(gpu, cpu, with_out=True, tag="", steps=10, **bars):
    gp, gm, gv, gout = gpu
    op, om, ov, oout = cpu
    assert_state_close(gp, gm, gv, op, om, ov, tag=tag, steps=steps, **bars)
    if with_out:
        assert np.array_equal(gout, oracle.cast_bf16(gp)), f"{tag}: fused cast is not RNE of p"
        assert bf16_ulp_diff(gout, oout).max(initial=0) <= 1, tag


@pytest.mark.parametrize("g_bf16", [False, True])
def test_tiny_config_ten_steps(g_bf16):
    gpu, cpu = run_packed(synth.TINY_N, 10, g_bf16=g_bf16)
    check(gpu, cpu, tag=f"packed cfg1 bf16={g_bf16}")


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 255, 256, 257, 4095, G - 4, G - 1, G, G + 1, G + 4, 2 * G + 252,
                               7 * G + 4097, (1 << 18) + 13])
@pytest.mark.parametrize("g_bf16", [False, True])
def test_ragged_sizes(n, g_bf16):
    gpu, cpu = run_packed(n, 3, g_bf16=g_bf16, seed=n % 97 + 1)
    check(gpu, cpu, tag=f"packed n={n}", steps=3)


@pytest.mark.parametrize("g_offset", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("g_bf16", [False, True])
def test_misaligned_gradient_and_copy(g_offset, g_bf16):
    """g and the bf16 copy shifted by a few elements: the stretch takes the one-element-per-lane
    kernel unless the shift keeps them on vector boundaries; same results either way."""
    gpu, cpu = run_packed(3 * G + 777, 2, g_bf16=g_bf16, g_offset=g_offset, seed=g_offset)
    check(gpu, cpu, tag=f"packed g_offset={g_offset}", steps=2)


def test_l2_mode_and_no_copy():
    gpu, cpu = run_packed(5 * G + 9, 4, g_bf16=True, mode=zc.ADAM_L2, with_out=False)
    check(gpu, cpu, with_out=False, tag="packed l2", steps=4)


def test_ranges_cut_stretches_anywhere():
    """Per-range hyper-parameters: stretches start inside granules, off lines and off vectors
    (peeled elements, tiles that straddle a granule boundary)."""
    n = 9 * G + 1234
    ranges = [(5, 6, 1.0, 0.0), (G - 3, G + 2, 0.5, 0.0), (2 * G + 100, 4 * G + 7, 2.0, 0.1),
              (4 * G + 7, 4 * G + 8, 1.0, 0.0), (6 * G, 7 * G, 0.25, 0.0), (9 * G + 1, n, 1.0, 0.0)]
    for g_bf16 in (False, True):
        gpu, cpu = run_packed(n, 3, g_bf16=g_bf16, ranges=ranges, seed=5)
        check(gpu, cpu, tag=f"packed ranges bf16={g_bf16}", steps=3)


def test_packed_step_is_bit_identical_to_the_three_array_step():
    n = 11 * G + 4099
    p = synth.host_params(n, 9)
    m0 = (synth.host_grads_f32(n, 4) * 0.1).astype(np.float32)
    v0 = (synth.host_grads_f32(n, 5) ** 2).astype(np.float32)
    dp, dm, dv = dev_f32(p), dev_f32(m0), dev_f32(v0)
    state = dev_state(n)
    zc.state_pack(dp, dm, dv, n, state)
    out_a = torch.zeros(n, dtype=torch.int16, device=DEV)
    out_b = torch.zeros(n, dtype=torch.int16, device=DEV)
    scale = dev_f32(np.array([0.37], np.float32))
    ranges = [(100, 5000, 0.5, 0.0), (3 * G + 1, 8 * G + 3, 1.5, 0.02)]
    for t in range(1, 6):
        g = dev_u16(oracle.cast_bf16(synth.host_grads_f32(n, 40 + t)))
        hp = zc.hparams(step=t, **HP)
        zc.adam_step_groups(dp, dm, dv, g, zc.BF16, n, hp, ranges=ranges, bf16_out=out_a, grad_scale_dev=scale)
        zc.adam_step_packed(state, g, zc.BF16, n, hp, ranges=ranges, bf16_out=out_b, grad_scale_dev=scale)
    up, um, uv = (torch.empty(n, dtype=torch.float32, device=DEV) for _ in range(3))
    zc.state_unpack(state, n, up, um, uv)
    sync()
    for a, b in ((dp, up), (dm, um), (dv, uv)):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    assert torch.equal(out_a, out_b)


def test_skip_flag_leaves_the_state_untouched():
    n = 3 * G + 5
    p = synth.host_params(n, 2)
    state = dev_state(n)
    zc.state_pack(dev_f32(p), None, None, n, state)
    before = state.clone()
    out = torch.full((n,), 0x1234, dtype=torch.int16, device=DEV)
    g = dev_u16(oracle.cast_bf16(synth.host_grads_f32(n, 1)))
    flag = torch.ones(1, dtype=torch.int32, device=DEV)
    zc.adam_step_packed(state, g, zc.BF16, n, zc.hparams(step=1, **HP), bf16_out=out, skip_flag=flag)
    sync()
    assert torch.equal(state.view(torch.int32), before.view(torch.int32)) and (out == 0x1234).all()
    flag.zero_()
    zc.adam_step_packed(state, g, zc.BF16, n, zc.hparams(step=1, **HP), bf16_out=out, skip_flag=flag)
    sync()
    assert not torch.equal(state.view(torch.int32), before.view(torch.int32))


def test_other_arithmetic_variants_take_the_element_kernel():
    """The wide packed kernel is built for the default arithmetic; with adam.arith 0 or 1 the
    packed step runs one element per lane and matches the three-array step of that variant."""
    n = 2 * G + 77
    p = synth.host_params(n, 4)
    g = dev_u16(oracle.cast_bf16(synth.host_grads_f32(n, 2)))
    for arith in (0, 1):
        zc.tune_set("adam.arith", arith)
        try:
            dp, dm, dv = dev_f32(p), torch.zeros(n, device=DEV), torch.zeros(n, device=DEV)
            state = dev_state(n)
            zc.state_pack(dp, dm, dv, n, state)
            hp = zc.hparams(step=1, **HP)
            zc.adam_step(dp, dm, dv, g, zc.BF16, n, hp)
            zc.adam_step_packed(state, g, zc.BF16, n, hp)
            up, um, uv = (torch.empty(n, dtype=torch.float32, device=DEV) for _ in range(3))
            zc.state_unpack(state, n, up, um, uv)
            sync()
            for a, b in ((dp, up), (dm, um), (dv, uv)):
                assert torch.equal(a.view(torch.int32), b.view(torch.int32)), arith
        finally:
            zc.tune_set("adam.arith", 2)


def test_argument_errors():
    n = G + 3
    state = dev_state(n)
    g = torch.zeros(n, dtype=torch.int16, device=DEV)
    hp = zc.hparams(step=1, **HP)
    with pytest.raises(zc.ZcError):                      # state off a 128-byte line
        zc.adam_step_packed(state.data_ptr() + 16, g, zc.BF16, n - 4, hp)
    with pytest.raises(zc.ZcError):                      # g inside the state array
        zc.adam_step_packed(state, state.data_ptr() + 64, zc.F32, n, hp)
    with pytest.raises(zc.ZcError):                      # range outside [0, n)
        zc.adam_step_packed(state, g, zc.BF16, n, hp, ranges=[(0, n + 1, 1.0, 0.0)])
    with pytest.raises(zc.ZcError):                      # source overlaps the packed array
        zc.state_pack(state.data_ptr() + 4, None, None, 8, state)
    zc.adam_step_packed(None, None, zc.BF16, 0, hp)      # n = 0 is a no-op
    zc.state_pack(None, None, None, 0, None)
    zc.state_unpack(None, 0)
    sync()


def test_packed_step_replays_from_a_hip_graph():
    """grad-norm (the entry point that never allocates) -> packed step with skip flag and fused
    copy, captured once and replayed: every replay equals the same calls made eagerly on a copy."""
    n = 5 * G + 1237
    p = synth.host_params(n, 8)
    state = dev_state(n)
    zc.state_pack(dev_f32(p), None, None, n, state)
    dg = dev_u16(oracle.cast_bf16(synth.host_grads_f32(n, 6)))
    send = torch.zeros(n, dtype=torch.int16, device=DEV)
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    hp = zc.hparams(step=2, **HP)

    def step(st, snd):
        zc.grad_sqnorm_static(dg, zc.BF16, n, norm, flag)
        zc.adam_step_packed(st, dg, zc.BF16, n, hp, ranges=[(G - 5, 2 * G + 3, 0.5, 0.0)], bf16_out=snd,
                            skip_flag=flag)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(state.clone(), torch.zeros_like(send))   # first use looks up the static buffer's address
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(state, send)
    sync()
    for replay in range(4):
        ref = state.clone()
        ref_send = torch.zeros_like(send)
        graph.replay()
        sync()
        step(ref, ref_send)
        sync()
        assert torch.equal(state.view(torch.int32), ref.view(torch.int32)), f"replay {replay}"
        assert torch.equal(send, ref_send)
        _ = (ref * 2).sum().item()                 # unrelated eager work and a sync between replays


PAD = 40      # guard elements around g and the bf16 copy


@pytest.mark.parametrize("seed", range(30))
def test_packed_step_random_case(seed):
    """Seeded random sizes, hyper-parameters, ranges, device-side scale, both gradient types and
    decay modes, g and the copy each at its own element offset: against the oracle, with guard
    elements around the flat arrays and the packed array's padding watched."""
    rng = np.random.default_rng(9000 + seed)
    n = int(rng.choice([1, 3, 31, 33, 4095, 4097, G - 1, G, G + 1, 2 * G + 5, 3 * G - 4, 40_011, 150_003]))
    if seed % 3 == 0:
        n = int(rng.integers(1, 6 * G))
    g_bf16 = bool(rng.integers(0, 2))
    mode = int(rng.integers(0, 2))
    with_out = bool(rng.integers(0, 2))
    steps = int(rng.integers(1, 4))
    hp = dict(lr=float(10.0 ** rng.uniform(-5, -2)), beta1=float(rng.choice([0.0, 0.8, 0.9, 0.95])),
              beta2=float(rng.choice([0.9, 0.98, 0.999])), eps=float(rng.choice([1e-8, 1e-6, 1e-10])),
              weight_decay=float(rng.choice([0.0, 0.01, 0.1])))
    grad_scale = float(rng.choice([1.0, 0.5, 1.0 / 1024, 3.0]))
    dev_scale = None if rng.integers(0, 2) else np.float32(rng.choice([1.0, 0.25, 0.7071]))
    g_off, o_off = (int(x) for x in rng.integers(0, PAD, 2))
    if rng.integers(0, 2):
        g_off = o_off = 4 * int(rng.integers(0, PAD // 4))          # keep the wide path reachable
    ranges = []
    if rng.integers(0, 2) and n >= 8:
        cuts = sorted(set(int(x) for x in rng.integers(0, n + 1, 6)))
        for b, e in zip(cuts[0::2], cuts[1::2]):
            ranges.append((b, e, float(rng.choice([1.0, 0.5, 2.0])), float(rng.choice([0.0, 0.05]))))
    case = (f"seed={seed} n={n} bf16={g_bf16} mode={mode} out={with_out} steps={steps} hp={hp} gs={grad_scale} "
            f"ds={dev_scale} g_off={g_off} o_off={o_off} ranges={ranges}")

    p = synth.host_params(n, 9100 + seed)
    m = (synth.host_grads_f32(n, 9200 + seed) * np.float32(0.1)).astype(np.float32)
    v = (synth.host_grads_f32(n, 9300 + seed) ** 2).astype(np.float32)
    out = np.zeros(n, np.uint16)
    packed0 = layout.pack_state(p, m, v, G)
    pad = np.ones(packed0.size, dtype=bool)
    for k in range(-(-n // G)):
        cnt = min(G, n - k * G)
        for a in range(3):
            pad[3 * k * G + a * G:3 * k * G + a * G + cnt] = False
    packed0.view(np.uint32)[pad] = 0x7FC0DEAD
    state = dev_state(n)
    state.copy_(dev_f32(packed0))
    out_full = torch.full((n + 2 * PAD,), 0x5EED, dtype=torch.int16, device=DEV)
    dout = out_full[o_off:o_off + n]
    scale_dev = None if dev_scale is None else torch.full((1,), float(dev_scale), dtype=torch.float32, device=DEV)
    t0 = int(rng.integers(1, 2000))
    for t in range(t0, t0 + steps):
        g = synth.host_grads_f32(n, 9400 + 10 * seed + t % 10)
        if g_bf16:
            g = oracle.cast_bf16(g)
            g_full = torch.full((n + 2 * PAD,), 0x5EED, dtype=torch.int16, device=DEV)
            dg = g_full[g_off:g_off + n]
            dg.copy_(dev_u16(g))
        else:
            g_full = torch.full((n + 2 * PAD,), 12345.0, dtype=torch.float32, device=DEV)
            dg = g_full[g_off:g_off + n]
            dg.copy_(dev_f32(g))
        zc.adam_step_packed(state, dg, zc.BF16 if g_bf16 else zc.F32, n,
                            zc.hparams(step=t, grad_scale=grad_scale, mode=mode, **hp), ranges=ranges,
                            bf16_out=dout if with_out else None, grad_scale_dev=scale_dev)
        oracle.adam_step_groups(p, m, v, g, ranges=ranges, step=t, grad_scale=grad_scale, mode=mode,
                                grad_scale_dev=dev_scale, bf16_out=out if with_out else None, **hp)
        sync()
    got = host_f32(state)
    assert np.array_equal(got.view(np.uint32)[pad], packed0.view(np.uint32)[pad]), case + ": padding written"
    got = got.copy()
    got[pad] = 0
    gp, gm, gv = layout.unpack_state(got, n, G)
    m_floor = 0.1 * 1e-3 * grad_scale * (float(dev_scale) if dev_scale is not None else 1.0)
    assert_state_close(gp, gm, gv, p, m, v, tag=case, steps=steps, lr=2.0 * hp["lr"], m_floor=max(m_floor, 1e-8))
    fill = torch.tensor(0x5EED, dtype=torch.int16, device=DEV)
    assert bool((out_full[:o_off] == fill).all()) and bool((out_full[o_off + n:] == fill).all()), case
    if with_out:
        go = host_u16(dout)
        assert np.array_equal(go, oracle.cast_bf16(gp)), case
        assert bf16_ulp_diff(go, out).max(initial=0) <= 1, case
    else:
        assert bool((dout == fill).all()), case


def test_packed_step_cut_into_several_launches():
    """A tiny launch limit forces the multi-launch path (tile offsets) of the packed kernel, with
    stretches that start inside a granule."""
    old = zc.tune_get("launch.max_grid")
    zc.tune_set("launch.max_grid", 7)
    try:
        n = 3 * G + 1031                      # 97 rows of 256 elements -> 14 launches
        gpu, cpu = run_packed(n, 2, g_bf16=True, seed=3, ranges=[(300, 2 * G + 9, 0.5, 0.0)])
        check(gpu, cpu, tag="packed cut launches", steps=2)
    finally:
        zc.tune_set("launch.max_grid", old)
