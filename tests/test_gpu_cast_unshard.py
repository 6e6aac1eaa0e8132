"""GPU parity: standalone bf16 cast, unshard copy and gradient norm against the
CPU oracle, through the C ABI.  Integer / bit work is compared bit-exactly."""
import numpy as np
import pytest
import torch

import oracle
from oracle import layout as olayout
from paper_2504_09983_amd import synth, zc
from tests.gpu_util import DEV, dev_f32, dev_u16, host_u16, sync

pytestmark = pytest.mark.gpu


def gpu_cast(x: np.ndarray, offset_src=0, offset_dst=0) -> np.ndarray:
    n = x.size
    src_full = torch.zeros(n + offset_src, dtype=torch.float32, device=DEV)
    src = src_full[offset_src:]
    src.copy_(torch.from_numpy(x.view(np.int32).copy()).to(DEV).view(torch.float32))
    dst_full = torch.full((n + offset_dst + 8,), 0x5A5A, dtype=torch.int16, device=DEV)
    dst = dst_full[offset_dst:offset_dst + n]
    zc.cast_bf16(src, dst, n)
    sync()
    assert (dst_full[:offset_dst] == 0x5A5A).all() and (dst_full[offset_dst + n:] == 0x5A5A).all()
    return host_u16(dst)


def from_bits(u):
    return np.ascontiguousarray(u, dtype=np.uint32).view(np.float32)


def test_cast_special_patterns_bit_exact():
    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    pats = np.concatenate([hi | low for low in (0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF)])
    x = from_bits(pats)
    assert np.array_equal(gpu_cast(x), oracle.cast_bf16(x))


@pytest.mark.parametrize("n", [1, 2, 3, 5, 1023, 4096, 4097, 4 * 1024 * 5 + 3, (1 << 20) + 1])
def test_cast_random_bits_ragged(n):
    rng = np.random.default_rng(n)
    x = from_bits(rng.integers(0, 1 << 32, size=n, dtype=np.uint64).astype(np.uint32))
    assert np.array_equal(gpu_cast(x), oracle.cast_bf16(x))


@pytest.mark.parametrize("osrc,odst", [(1, 0), (0, 1), (3, 2), (4, 4), (0, 2)])
def test_cast_misaligned(osrc, odst):
    x = synth.host_params(10007, 3)
    assert np.array_equal(gpu_cast(x, osrc, odst), oracle.cast_bf16(x))


def test_cast_all_2_to_32_patterns():
    """Every fp32 bit pattern, in 16 pieces of 2^28."""
    piece = 1 << 28
    src = torch.empty(piece, dtype=torch.int32, device=DEV)
    dst = torch.empty(piece, dtype=torch.int16, device=DEV)
    base = torch.arange(piece, dtype=torch.int64, device=DEV)
    for k in range(16):
        start = k * piece
        val = base + start
        val = torch.where(val >= (1 << 31), val - (1 << 32), val)    # two's-complement bit pattern
        src.copy_(val)
        del val
        zc.cast_bf16(src, dst, piece)
        sync()
        got = host_u16(dst)
        bits = np.arange(start, start + piece, dtype=np.uint64).astype(np.uint32)
        want = oracle.cast_bf16(bits.view(np.float32))
        assert np.array_equal(got, want), f"piece {k}"
        print(f"piece {k} ok", flush=True)


def test_fused_cast_equals_standalone_cast():
    n = 123457
    p = synth.host_params(n, 4)
    dp, dm, dv = dev_f32(p), dev_f32(np.zeros(n)), dev_f32(np.zeros(n))
    dg = dev_f32(synth.host_grads_f32(n, 1))
    fused = torch.zeros(n, dtype=torch.int16, device=DEV)
    alone = torch.zeros(n, dtype=torch.int16, device=DEV)
    zc.adam_step(dp, dm, dv, dg, zc.F32, n, zc.hparams(step=1, lr=1e-4, beta1=0.9, beta2=0.999,
                                                       eps=1e-8, weight_decay=0.01), bf16_out=fused)
    zc.cast_bf16(dp, alone, n)
    sync()
    assert torch.equal(fused, alone)


# ---- unshard ----------------------------------------------------------------------

GUARD = 16  # sentinel elements on both sides of every destination


def run_unshard(numels, world=8, align=8, dst_shift=None, src_shift=0, tune=None):
    offs, shard, total = olayout.flat_layout(numels, world, align)
    z_offs, z_shard, z_total = zc.flat_layout(numels, world, align)
    assert list(offs) == z_offs and shard == z_shard and total == z_total
    gathered_host = synth.host_index_hash16(0, world * shard + src_shift)
    gathered_full = dev_u16(gathered_host)
    gathered = gathered_full[src_shift:]
    g_numel = world * shard
    dsts, views = [], []
    for i, n in enumerate(numels):
        sh = 0 if dst_shift is None else dst_shift[i % len(dst_shift)]
        buf = torch.full((n + 2 * GUARD + sh,), 0x7E7E, dtype=torch.int16, device=DEV)
        dsts.append(buf)
        views.append(buf[GUARD + sh:GUARD + sh + n])
    segs = [(int(o), v if n else None, n) for o, v, n in zip(offs, views, numels)]
    old = {}
    if tune:
        for k, val in tune.items():
            old[k] = zc.tune_get(k); zc.tune_set(k, val)
    try:
        plan = zc.unshard_plan_create(segs, g_numel)
        zc.unshard(plan, gathered)
        sync()
        plan.destroy()
    finally:
        for k, val in old.items():
            zc.tune_set(k, val)
    want = oracle.unshard(gathered_host[src_shift:], offs, numels)
    for i, (buf, view, w, n) in enumerate(zip(dsts, views, want, numels)):
        assert np.array_equal(host_u16(view), w), f"tensor {i} (n={n})"
        sh = buf.numel() - n - 2 * GUARD
        assert (buf[:GUARD + sh] == 0x7E7E).all() and (buf[GUARD + sh + n:] == 0x7E7E).all(), \
            f"guard words of tensor {i} overwritten"
    return views, gathered, total


def test_tiny_config_unshard_four_matrices():
    """Tiny workload: 2^20 elements -> 4 tensors of 512 x 512 (fed by the step's bf16 copy)."""
    n = synth.TINY_N
    p = synth.host_params(n, 1)
    bits = oracle.cast_bf16(p)
    numels = [a * b for _, (a, b) in synth.TINY_TENSORS]
    offs, shard, total = zc.flat_layout(numels, 8, 1)
    assert total == n and shard * 8 == n
    src = torch.zeros(n, dtype=torch.int16, device=DEV)
    zc.cast_bf16(dev_f32(p), src, n)
    outs = [torch.zeros(512, 512, dtype=torch.bfloat16, device=DEV) for _ in numels]
    plan = zc.unshard_plan_create([(o, t, k) for o, t, k in zip(offs, outs, numels)], n)
    zc.unshard(plan, src)
    sync()
    want = oracle.unshard(bits, offs, numels)
    for t, w in zip(outs, want):
        assert np.array_equal(host_u16(t).reshape(-1), w)


@pytest.mark.parametrize("align", [1, 8, 4096])
def test_unshard_ragged_lists(align):
    run_unshard([1, 3, 7, 4097, 0, 64, 129, 8192 * 3 + 5, 0, 11], align=align)
    run_unshard([5], align=align)
    run_unshard([0, 0, 9, 0], align=align)


@pytest.mark.parametrize("src_shift", [0, 1, 2, 3])
def test_unshard_every_relative_alignment(src_shift):
    # odd tensor sizes walk the source offset through every residue mod 8 elements;
    # dst shifts walk the destination through every 16-byte residue.
    numels = [8192 + k for k in range(9)] + [40000, 7, 8, 9, 15, 16, 17]
    run_unshard(numels, align=1, dst_shift=[0, 1, 2, 3, 4, 5, 6, 7], src_shift=src_shift)


def test_unshard_occupancy_cap_and_nontemporal():
    numels = [4096 * 64 + 3, 1000, 4096 * 200, 17]
    for tune in ({"copy.waves_per_cu": 0}, {"copy.nontemporal": 0}, {"copy.nontemporal": 2},
                 {"copy.waves_per_cu": 4, "copy.nontemporal": 1}):
        run_unshard(numels, tune=tune)


def test_unshard_model_shaped_scaled_down():
    """Mixtral layer structure at 1/32 width: ragged boundaries, bit-exact, hash property."""
    shape = synth.ModelShape("mini_moe", 2, 128, 448, 4, 1, 1000, experts=8, head_dim=32)
    numels = synth.tensor_numels(shape)
    views, gathered, total = run_unshard(numels, align=4096)
    offs, shard, _ = zc.flat_layout(numels, 8, 4096)
    for o, v, n in zip(offs, views, numels):
        assert torch.equal(v, synth.device_index_hash16_values(o, n, DEV))
    # re-flattening reproduces the gathered prefix; the padding was never copied anywhere
    assert torch.equal(torch.cat([v.reshape(-1) for v in views]), gathered[:total])
    assert 8 * shard > total


def test_unshard_refuses_a_gathered_buffer_that_overlaps_a_destination():
    buf = torch.zeros(4096, dtype=torch.int16, device=DEV)
    other = torch.zeros(1024, dtype=torch.int16, device=DEV)
    plan = zc.unshard_plan_create([(0, buf[1024:2048], 1024), (1024, other, 1024)], 2048)
    for gathered in (buf[:2048], buf[1500:3548], buf[2047:]):          # share bytes with buf[1024:2048]
        with pytest.raises(zc.ZcError) as e:
            zc.unshard(plan, gathered)
        assert e.value.status == zc.ERR_INVALID_ARG and "overlaps" in e.value.message
    zc.unshard(plan, buf[2048:])                                        # touching is fine
    sync()
    plan.destroy()


def test_empty_plan_is_a_noop():
    plan = zc.unshard_plan_create([], 0)
    zc.unshard(plan, None)
    plan.destroy()
    plan = zc.unshard_plan_create([(0, None, 0), (5, None, 0)], 10)
    zc.unshard(plan, None)
    plan.destroy()


# ---- gradient norm / overflow flag ----------------------------------------------

@pytest.mark.parametrize("n", [0, 1, 7, 8, 9, 1000, 65536 + 3, (1 << 22) + 5])
@pytest.mark.parametrize("bf16", [True, False])
def test_grad_sqnorm(n, bf16):
    g = synth.host_normal(n, 1e-3, 40 + n % 7)
    if bf16:
        g = oracle.cast_bf16(g)
        dg = dev_u16(g) if n else None
    else:
        dg = dev_f32(g) if n else None
    out = torch.full((1,), -1.0, dtype=torch.float32, device=DEV)
    flag = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    zc.grad_sqnorm(dg, zc.BF16 if bf16 else zc.F32, n, out, flag)
    sync()
    want, bad = oracle.grad_sqnorm(g)
    assert flag.item() == bad == 0
    # fp32 sums of at most 8 terms folded in double: within an fp32 ulp of the rounded exact sum
    assert abs(out.item() - want) <= 1.3e-7 * want + 1e-30
    # deterministic
    out2 = torch.zeros_like(out)
    zc.grad_sqnorm(dg, zc.BF16 if bf16 else zc.F32, n, out2, flag)
    sync()
    assert out2.item() == out.item()


@pytest.mark.parametrize("bf16", [True, False])
@pytest.mark.parametrize("poison", [np.inf, -np.inf, np.nan])
def test_grad_sqnorm_flags_nonfinite(bf16, poison):
    n = 100003
    for pos in (0, 1, 50001, n - 1):
        g = synth.host_normal(n, 1e-3, 50)
        g[pos] = poison
        if bf16:
            g = oracle.cast_bf16(g)
            dg = dev_u16(g)
        else:
            dg = dev_f32(g)
        out = torch.zeros(1, dtype=torch.float32, device=DEV)
        flag = torch.zeros(1, dtype=torch.int32, device=DEV)
        zc.grad_sqnorm(dg, zc.BF16 if bf16 else zc.F32, n, out, flag)
        sync()
        want, bad = oracle.grad_sqnorm(g)
        assert bad == 1 and flag.item() == 1
        assert not np.isfinite(out.item()) and not np.isfinite(want)


def test_grad_sqnorm_misaligned_and_large_values():
    g = synth.host_normal(5001, 1e-3, 60)
    dg = dev_f32(g)
    out = torch.zeros(1, dtype=torch.float32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    zc.grad_sqnorm(dg[1:], zc.F32, 5000, out, flag)
    sync()
    want, _ = oracle.grad_sqnorm(g[1:])
    assert abs(out.item() - want) <= 1.3e-7 * want and flag.item() == 0
    # large finite bf16 values: flag stays 0 although the squares overflow fp32
    big = oracle.cast_bf16(np.full(64, 3e38, np.float32))
    zc.grad_sqnorm(dev_u16(big), zc.BF16, 64, out, flag)
    sync()
    assert flag.item() == 0 and oracle.grad_sqnorm(big)[1] == 0


# ---- per-tensor even partition (every tensor split over the ranks; fused group) -------

def run_unshard_per_tensor(numels, world=8, align=1, seed=0):
    rng = np.random.default_rng(seed)
    tensors = [rng.integers(1, 1 << 16, size=n, dtype=np.uint16) for n in numels]
    gathered_host = olayout.per_tensor_gather(tensors, world, align)
    segs, send = zc.per_tensor_layout(numels, world, align)
    assert send * world == gathered_host.size
    gathered = dev_u16(gathered_host)
    bufs = [torch.full((n + 2 * GUARD,), 0x7E7E, dtype=torch.int16, device=DEV) for n in numels]
    table = [(src, bufs[t].data_ptr() + 2 * (GUARD + dst) if k else None, k) for t, src, dst, k in segs]
    plan = zc.unshard_plan_create(table, gathered_host.size)
    zc.unshard(plan, gathered)
    sync()
    plan.destroy()
    want = oracle.unshard_per_tensor(gathered_host, numels, world, align)
    for i, (buf, w, src_t) in enumerate(zip(bufs, want, tensors)):
        got = host_u16(buf[GUARD:GUARD + numels[i]])
        assert np.array_equal(got, w) and np.array_equal(got, src_t), f"tensor {i}"
        assert (buf[:GUARD] == 0x7E7E).all() and (buf[GUARD + numels[i]:] == 0x7E7E).all()


@pytest.mark.parametrize("align", [1, 8])
def test_unshard_per_tensor_partition(align):
    run_unshard_per_tensor([1, 3, 7, 4097, 0, 64, 129, 8192 * 3 + 5, 11], align=align)
    run_unshard_per_tensor([5], align=align)
    run_unshard_per_tensor([8 * 4096, 4096, 8 * 14336], align=align)


def test_unshard_per_tensor_model_shaped():
    shape = synth.ModelShape("mini_moe", 2, 128, 448, 4, 1, 1000, experts=8, head_dim=32)
    run_unshard_per_tensor(synth.tensor_numels(shape), align=8, seed=3)


# ---- gradient accumulation ---------------------------------------------------------------

@pytest.mark.parametrize("n", [1, 3, 4, 5, 1023, 1024 * 4 + 1, (1 << 20) + 7])
@pytest.mark.parametrize("bf16", [True, False])
def test_grad_accumulate_bit_exact(n, bf16):
    acc = synth.host_normal(n, 1e-3, 70)
    dacc = dev_f32(acc)
    for k in range(4):                      # four micro-batches, scale 1/4 then an odd one
        micro = synth.host_grads_f32(n, 10 + k)
        scale = 0.25 if k < 3 else 0.37
        if bf16:
            micro = oracle.cast_bf16(micro)
            dmicro = dev_u16(micro)
        else:
            dmicro = dev_f32(micro)
        oracle.grad_accumulate(acc, micro, scale)
        zc.grad_accumulate(dacc, dmicro, zc.BF16 if bf16 else zc.F32, n, scale)
    sync()
    assert np.array_equal(dacc.cpu().numpy().view(np.uint32), acc.view(np.uint32))


def test_grad_accumulate_misaligned_then_feeds_the_step():
    n = 30001
    acc = np.zeros(n + 1, np.float32)
    dacc_full = dev_f32(acc)
    dacc = dacc_full[1:]                     # 4-byte aligned only -> scalar kernel
    micro = oracle.cast_bf16(synth.host_grads_f32(n, 3))
    dmicro = dev_u16(micro)
    zc.grad_accumulate(dacc, dmicro, zc.BF16, n, 0.5)
    zc.grad_accumulate(dacc, dmicro, zc.BF16, n, 0.5)
    a = np.zeros(n, np.float32)
    oracle.grad_accumulate(a, micro, 0.5)
    oracle.grad_accumulate(a, micro, 0.5)
    sync()
    assert float(dacc_full[0]) == 0.0
    assert np.array_equal(dacc.cpu().numpy(), a)
    # the accumulated fp32 partition is what the norm and the step consume
    out = torch.zeros(1, dtype=torch.float32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    zc.grad_sqnorm(dacc, zc.F32, n, out, flag)
    sync()
    want, bad = oracle.grad_sqnorm(a)
    assert bad == 0 and flag.item() == 0 and abs(out.item() - want) <= 1.3e-7 * want


def test_grad_sqnorm_on_two_streams_at_once():
    """Each stream has its own partial sums: interleaved launches on two streams over different
    gradients give each its own norm, every time."""
    n = (1 << 22) + 11
    ga = synth.host_grads_f32(n, 61)
    gb = (synth.host_grads_f32(n, 62) * np.float32(3.0)).astype(np.float32)
    da, db = dev_f32(ga), dev_f32(gb)
    want_a, want_b = oracle.grad_sqnorm(ga)[0], oracle.grad_sqnorm(gb)[0]
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    outs_a = torch.zeros(32, dtype=torch.float32, device=DEV)
    outs_b = torch.zeros(32, dtype=torch.float32, device=DEV)
    flags = torch.zeros(64, dtype=torch.int32, device=DEV)
    sync()
    for i in range(32):
        zc.grad_sqnorm(da, zc.F32, n, outs_a[i:i + 1], flags[i:i + 1], stream=sa)
        zc.grad_sqnorm(db, zc.F32, n, outs_b[i:i + 1], flags[32 + i:33 + i], stream=sb)
    sync()
    assert not flags.any()
    assert np.all(np.abs(outs_a.cpu().numpy() - want_a) <= 1.3e-7 * want_a)
    assert np.all(np.abs(outs_b.cpu().numpy() - want_b) <= 1.3e-7 * want_b)
    assert len(set(outs_a.cpu().numpy().tolist())) == 1 and len(set(outs_b.cpu().numpy().tolist())) == 1
