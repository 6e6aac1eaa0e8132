"""GPU parity at the full benchmark sizes, in the launch configuration the
benchmark times.  Inputs are generated on the GPU; windows of them are copied to
the host and fed to the oracle, and properties that hold at any size (index-hash
identity of the unshard copy, fused cast == RNE of the stored p) cover the rest."""
import numpy as np
import pytest
import torch

import oracle
from paper_2504_09983_amd import synth, zc
from tests.gpu_util import DEV, HP, assert_state_close, host_f32, host_u16, sync

pytestmark = pytest.mark.gpu


def windows_for(n, extra_boundaries=(), count=24, width=1 << 14, seed=0):
    """First / last window, windows around given boundaries, and random ones."""
    rng = np.random.default_rng(seed)
    starts = [0, max(0, n - width)]
    for b in extra_boundaries:
        starts.append(min(max(0, b - width // 2), max(0, n - width)))
    starts += [int(x) for x in rng.integers(0, max(1, n - width), size=count)]
    # the region just past 2^32 elements and 2^35 bytes, where 32-bit indexing would wrap
    for b in (1 << 31, 1 << 32, (1 << 33) + 12345):
        if b + width < n:
            starts.append(b - width // 2)
    return sorted(set((s, min(width, n - s)) for s in starts))


def alloc_state(n, g_dtype):
    p = torch.empty(n, dtype=torch.float32, device=DEV)
    m = torch.zeros(n, dtype=torch.float32, device=DEV)
    v = torch.zeros(n, dtype=torch.float32, device=DEV)
    g = torch.empty(n, dtype=g_dtype, device=DEV)
    synth.device_normal_(p, synth.P_STD, seed=2)
    return p, m, v, g


def run_windowed(n, steps, with_out, wins):
    """`steps` AdamW steps over n elements; the oracle follows on the windows."""
    p, m, v, g = alloc_state(n, torch.bfloat16)
    out = torch.zeros(n, dtype=torch.int16, device=DEV) if with_out else None
    host = [(host_f32(p[s:s + w]).copy(), np.zeros(w, np.float32), np.zeros(w, np.float32),
             np.zeros(w, np.uint16)) for s, w in wins]
    for t in range(1, steps + 1):
        synth.device_normal_(g, synth.G_STD, seed=2000 + t)
        zc.adam_step(p, m, v, g, zc.BF16, n, zc.hparams(step=t, **HP), bf16_out=out)
        sync()
        for (s, w), (hp_, hm_, hv_, ho_) in zip(wins, host):
            gbits = host_u16(g[s:s + w])
            oracle.adam_step(hp_, hm_, hv_, gbits, step=t, bf16_out=ho_, **HP)
        print(f"step {t} done", flush=True)
    for (s, w), (hp_, hm_, hv_, ho_) in zip(wins, host):
        gp, gm, gv = host_f32(p[s:s + w]), host_f32(m[s:s + w]), host_f32(v[s:s + w])
        assert_state_close(gp, gm, gv, hp_, hm_, hv_, steps=steps, tag=f"window@{s}")
        if with_out:
            go = host_u16(out[s:s + w])
            assert np.array_equal(go, oracle.cast_bf16(gp)), f"window@{s}: fused cast"
    return p, m, v, g, out


def test_llama8b_shard_ten_steps():
    """Llama-3-8B one-of-8 shard: n = 1,003,782,656, bf16 grads, all resident, 10 steps, no cast."""
    _, shard, _ = zc.flat_layout(synth.tensor_numels(synth.LLAMA3_8B), 8, 1)
    assert shard == 1_003_782_656
    wins = windows_for(shard, seed=2)
    p, m, v, g, _ = run_windowed(shard, 10, False, wins)
    # whole-array sanity that holds at any size: finite, v >= 0, p moved by at most 10*lr*(1+eps)
    assert torch.isfinite(p).all() and torch.isfinite(m).all() and bool((v >= 0).all())
    del p, m, v, g
    torch.cuda.empty_cache()


def test_llama70b_shard_step_and_cast():
    """Llama-3-70B one-of-8 shard: n = 8,819,213,312 (p/m/v ~105 GB resident), fused bf16 copy,
    the 10 steps the fp32 acceptance bar is defined over."""
    _, shard, _ = zc.flat_layout(synth.tensor_numels(synth.LLAMA3_70B), 8, 1)
    assert shard == 8_819_213_312
    wins = windows_for(shard, extra_boundaries=[shard // 2], seed=3)
    p, m, v, g, out = run_windowed(shard, 10, True, wins)
    # property at full size: the bf16 copy is torch's RNE narrowing of the stored p, chunked
    step = 1 << 28
    for s in range(0, shard, step * 8):          # every 8th chunk
        e = min(shard, s + step)
        assert torch.equal(p[s:e].to(torch.bfloat16).view(torch.int16), out[s:e]), f"chunk@{s}"
    del p, m, v, g, out
    torch.cuda.empty_cache()


def packed_positions(s, w, granule):
    """Positions of p[s : s + w] in the packed state array, from the layout's definition
    (granule k of p, m, v follow each other); m sits one granule and v two granules behind."""
    e = np.arange(s, s + w, dtype=np.int64)
    return (e // granule) * 3 * granule + e % granule


@pytest.mark.parametrize("shape", ["LLAMA3_8B", "LLAMA3_70B"])
def test_shard_in_packed_state_ten_steps(shape):
    """The 8B and 70B shards held as one packed state array (the layout the benchmark's headline
    times): 10 steps with the fused bf16 copy, the oracle following on windows that are read
    out of the packed array by the layout's definition."""
    G = zc.PACKED_GRANULE
    _, n, _ = zc.flat_layout(synth.tensor_numels(getattr(synth, shape)), 8, 1)
    assert n == {"LLAMA3_8B": 1_003_782_656, "LLAMA3_70B": 8_819_213_312}[shape]
    steps = 10
    state = torch.empty(zc.packed_state_numel(n), dtype=torch.float32, device=DEV)
    cube = state.view(-1, 3, G)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(11)
    for k in range(0, cube.shape[0], 1 << 12):                 # 2^25 elements of p per draw
        rows = min(1 << 12, cube.shape[0] - k)
        cube[k:k + rows, 0] = torch.randn(rows, G, generator=gen, device=DEV) * synth.P_STD
    cube[:, 1:].zero_()
    g = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    out = torch.zeros(n, dtype=torch.int16, device=DEV)
    wins = windows_for(n, extra_boundaries=[n // 2, 5 * G, (n // G) * G], seed=5)
    where = [torch.from_numpy(packed_positions(s, w, G)).to(DEV) for s, w in wins]
    host = [(host_f32(state[at]).copy(), np.zeros(w, np.float32), np.zeros(w, np.float32),
             np.zeros(w, np.uint16)) for (s, w), at in zip(wins, where)]
    for t in range(1, steps + 1):
        synth.device_normal_(g, synth.G_STD, seed=3000 + t)
        zc.adam_step_packed(state, g, zc.BF16, n, zc.hparams(step=t, **HP), bf16_out=out)
        sync()
        for (s, w), (hp_, hm_, hv_, ho_) in zip(wins, host):
            oracle.adam_step(hp_, hm_, hv_, host_u16(g[s:s + w]), step=t, bf16_out=ho_, **HP)
        print(f"step {t} done", flush=True)
    for (s, w), at, (hp_, hm_, hv_, ho_) in zip(wins, where, host):
        gp, gm, gv = host_f32(state[at]), host_f32(state[at + G]), host_f32(state[at + 2 * G])
        assert_state_close(gp, gm, gv, hp_, hm_, hv_, steps=steps, tag=f"packed window@{s}")
        assert np.array_equal(host_u16(out[s:s + w]), oracle.cast_bf16(gp)), f"window@{s}: fused cast"
    # at full size: the bf16 copy is torch's RNE narrowing of the p granules, every 8th chunk
    rows = 1 << 15                                              # 2^28 elements per chunk
    for k in range(0, cube.shape[0], rows * 8):
        k1 = min(cube.shape[0], k + rows)
        e = min(n, k1 * G)
        pk = cube[k:k1, 0].reshape(-1)[:e - k * G]
        assert torch.equal(pk.to(torch.bfloat16).view(torch.int16), out[k * G:e]), f"chunk@{k * G}"
        del pk
    whole = 3 * (n // G) * G                                    # the last granule's padding is never touched
    for s0 in range(0, whole, 1 << 30):
        assert torch.isfinite(state[s0:min(whole, s0 + (1 << 30))]).all(), f"state chunk@{s0}"
    del state, cube, g, out
    torch.cuda.empty_cache()


def test_llama70b_shard_every_element_after_step_one():
    """Step 1 from m = v = 0 has a closed form in every element: m = (1-b1) g, v = (1-b2) g^2,
    p = p0 (1 - lr wd) - lr g / (|g| + eps) up to rounding.  Checked over all 8.8 B elements with
    torch as a double-precision calculator, in chunks (a property that holds at any size; the
    windows above carry the element-by-element comparison with the oracle)."""
    _, n, _ = zc.flat_layout(synth.tensor_numels(synth.LLAMA3_70B), 8, 1)
    p, m, v, g = alloc_state(n, torch.bfloat16)
    synth.device_normal_(g, synth.G_STD, seed=2001)
    p0_head = p[:1 << 20].clone()
    chunk = 1 << 27
    # one launch over the whole shard; p0 is rebuilt from the seeded generator afterwards
    zc.adam_step(p, m, v, g, zc.BF16, n, zc.hparams(step=1, **HP))
    sync()
    b1, b2 = float(np.float32(HP["beta1"])), float(np.float32(HP["beta2"]))
    lr, eps, wd = (float(np.float32(HP[k])) for k in ("lr", "eps", "weight_decay"))
    p0 = torch.empty(n, dtype=torch.float32, device=DEV)
    synth.device_normal_(p0, synth.P_STD, seed=2)          # the same seeded stream as alloc_state
    assert torch.equal(p0[:1 << 20], p0_head)
    worst = 0.0
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        gd = g[s:e].double()
        assert torch.equal(m[s:e], (gd * (1.0 - b1)).float()), f"m chunk@{s}"
        assert torch.equal(v[s:e], ((gd * (1.0 - b2)) * gd).float()), f"v chunk@{s}"
        want = p0[s:e].double() * (1.0 - lr * wd) - lr * gd / (gd.abs() + eps)
        # one fp32 rounding of p plus ~1.2e-7 relative on the lr-sized term (m, v stored in fp32)
        err = (p[s:e].double() - want).abs()
        bound = 0.5 * torch.maximum(p[s:e].abs(), p0[s:e].abs()).double() * 2.0 ** -23 + 3e-7 * lr + 1e-12
        worst = max(worst, float((err / bound).max()))
        del gd, want, err, bound
    assert worst <= 1.0, worst
    del p, m, v, g, p0
    torch.cuda.empty_cache()


def test_mixtral_unshard_full_size():
    """Mixtral-8x7B: gathered flat bf16 buffer of 8 rank shards (rank-padded) unsharded
    into 995 separately allocated tensors; bit-exact layout check by index hash."""
    shape = synth.MIXTRAL_8X7B
    tensors = synth.tensor_list(shape)
    numels = synth.tensor_numels(shape)
    offs, shard, total = zc.flat_layout(numels, 8, 4096)
    assert total == 46_702_792_704 and shard % 4096 == 0 and 8 * shard > total
    gathered = torch.empty(8 * shard, dtype=torch.int16, device=DEV)
    synth.device_index_hash16_(gathered)
    outs = [torch.empty(dims, dtype=torch.bfloat16, device=DEV) for _, dims in tensors]
    plan = zc.unshard_plan_create([(o, t, k) for o, t, k in zip(offs, outs, numels)], 8 * shard)
    zc.unshard(plan, gathered)
    sync()
    print("unshard done", flush=True)
    # (i) every element equals the hash of its own flat index
    for i, (o, t, k) in enumerate(zip(offs, outs, numels)):
        want = synth.device_index_hash16_values(o, k, DEV)
        assert torch.equal(t.view(torch.int16).reshape(-1), want), tensors[i][0]
    print("hash identity ok", flush=True)
    # (ii) sampled tensors against the oracle's element-by-element copy
    rng = np.random.default_rng(5)
    for i in [0, 1, 5, len(outs) - 1] + [int(x) for x in rng.integers(0, len(outs), 6)]:
        o, k = offs[i], numels[i]
        w = min(k, 1 << 16)
        src = host_u16(gathered[o:o + w])
        want = oracle.unshard(src, [0], [w])[0]
        assert np.array_equal(host_u16(outs[i].reshape(-1)[:w]), want)
    # (iii) tensors straddle shard boundaries (ragged): at least one per boundary
    straddle = sum(1 for o, k in zip(offs, numels) if o // shard != (o + k - 1) // shard)
    assert straddle >= 7
    plan.destroy()
    del outs, gathered
    torch.cuda.empty_cache()


def test_mixtral_step_cast_into_rank_slot_then_unshard():
    """Config 5 as stated: AdamW + bf16 copy on rank 0's Mixtral-8x7B partition (S' = 5,837,852,672
    elements, padded to 4096), the copy written straight into rank 0's slot of the gathered buffer
    of 8 x S' elements whose other seven slots hold the index hash, then the unshard into the 995
    tensors.  Tensors (and parts of tensors) inside rank 0's slot must be RNE of the updated p,
    everything else the hash of its own index; p, m, v against the oracle on windows.
    Allocation is phased: m, v and g are released before the destinations are allocated."""
    shape = synth.MIXTRAL_8X7B
    tensors = synth.tensor_list(shape)
    numels = synth.tensor_numels(shape)
    offs, shard, total = zc.flat_layout(numels, 8, 4096)
    assert shard == 5_837_852_672 and 8 * shard - total == 8 * 3584
    n = shard
    gathered = torch.empty(8 * shard, dtype=torch.int16, device=DEV)
    synth.device_index_hash16_(gathered)
    send = gathered[:n]
    p, m, v, g = alloc_state(n, torch.bfloat16)
    wins = windows_for(n, extra_boundaries=[n // 3], count=12, seed=11)
    host = [(host_f32(p[s:s + w]).copy(), np.zeros(w, np.float32), np.zeros(w, np.float32),
             np.zeros(w, np.uint16)) for s, w in wins]
    steps = 2
    for t in range(1, steps + 1):
        synth.device_normal_(g, synth.G_STD, seed=2000 + t)
        zc.adam_step(p, m, v, g, zc.BF16, n, zc.hparams(step=t, **HP), bf16_out=send)
        sync()
        for (s, w), (hp_, hm_, hv_, ho_) in zip(wins, host):
            oracle.adam_step(hp_, hm_, hv_, host_u16(g[s:s + w]), step=t, bf16_out=ho_, **HP)
        print(f"step {t} done", flush=True)
    for (s, w), (hp_, hm_, hv_, ho_) in zip(wins, host):
        gp, gm, gv = host_f32(p[s:s + w]), host_f32(m[s:s + w]), host_f32(v[s:s + w])
        assert_state_close(gp, gm, gv, hp_, hm_, hv_, steps=steps, tag=f"window@{s}")
        assert np.array_equal(host_u16(send[s:s + w]), oracle.cast_bf16(gp)), f"window@{s}: fused cast"
    # the step must not have touched the other ranks' slots
    edge = synth.device_index_hash16_values(n, 1 << 20, DEV)
    assert torch.equal(gathered[n:n + (1 << 20)], edge)
    del m, v, g, edge
    torch.cuda.empty_cache()
    outs = [torch.empty(dims, dtype=torch.bfloat16, device=DEV) for _, dims in tensors]
    plan = zc.unshard_plan_create([(o, t, k) for o, t, k in zip(offs, outs, numels)], 8 * shard)
    zc.unshard(plan, gathered)
    sync()
    print("unshard done", flush=True)
    straddlers = 0
    for i, (o, t, k) in enumerate(zip(offs, outs, numels)):
        flat = t.view(torch.int16).reshape(-1)
        mine = max(0, min(o + k, n) - o)          # leading elements that lie in rank 0's slot
        if mine:                                   # torch's bf16 narrowing as the RNE calculator
            assert torch.equal(flat[:mine], p[o:o + mine].to(torch.bfloat16).view(torch.int16)), tensors[i][0]
        if mine < k:
            assert torch.equal(flat[mine:], synth.device_index_hash16_values(o + mine, k - mine, DEV)), tensors[i][0]
        straddlers += 0 < mine < k
    assert straddlers == 1                          # exactly one tensor crosses the end of rank 0's slot
    # sampled rank-0 tensors against the oracle's own cast and copy
    rng = np.random.default_rng(13)
    mine_idx = [i for i, (o, k) in enumerate(zip(offs, numels)) if o + k <= n]
    for i in [mine_idx[0], mine_idx[-1]] + [int(x) for x in rng.choice(mine_idx, 4)]:
        o, w = offs[i], min(numels[i], 1 << 16)
        want = oracle.unshard(oracle.cast_bf16(host_f32(p[o:o + w])), [0], [w])[0]
        assert np.array_equal(host_u16(outs[i].reshape(-1)[:w]), want), tensors[i][0]
    plan.destroy()
    del outs, gathered, send, p
    torch.cuda.empty_cache()


def test_mixtral_unshard_per_tensor_partition_full_size():
    """The paper's literal layout at Mixtral size: every one of the 995 tensors split over
    8 ranks (7960 segments), gathered buffer = 8 send buffers; bit-exact by index hash."""
    shape = synth.MIXTRAL_8X7B
    tensors = synth.tensor_list(shape)
    numels = synth.tensor_numels(shape)
    W = 8
    segs, send = zc.per_tensor_layout(numels, W, 8)
    gathered = torch.empty(W * send, dtype=torch.int16, device=DEV)
    synth.device_index_hash16_(gathered)
    outs = [torch.empty(dims, dtype=torch.bfloat16, device=DEV) for _, dims in tensors]
    table = [(src, outs[t].data_ptr() + 2 * dst if k else None, k) for t, src, dst, k in segs]
    plan = zc.unshard_plan_create(table, W * send)
    zc.unshard(plan, gathered)
    sync()
    print("unshard done", flush=True)
    # element i of tensor t came from gathered[r*send + o_t + j], r = i // s_t, j = i % s_t
    for t, src, dst, k in segs:
        if k == 0:
            continue
        want = synth.device_index_hash16_values(src, k, DEV)
        got = outs[t].view(torch.int16).reshape(-1)[dst:dst + k]
        assert torch.equal(got, want), (tensors[t][0], src)
    # sampled segments against the oracle's element-by-element copy
    rng = np.random.default_rng(7)
    live = [s for s in segs if s[3] > 0]
    for idx in rng.integers(0, len(live), 8):
        t, src, dst, k = live[int(idx)]
        w = min(k, 1 << 15)
        want = oracle.unshard(host_u16(gathered[src:src + w]), [0], [w])[0]
        assert np.array_equal(host_u16(outs[t].reshape(-1)[dst:dst + w]), want)
    plan.destroy()
    del outs, gathered
    torch.cuda.empty_cache()


def test_single_segment_longer_than_2_to_32_elements():
    """One tensor of 2^32 + 4099 elements, source and destination both off the 16-byte grid:
    tile indices inside one segment pass 2^24 and element indices 2^32."""
    k = (1 << 32) + 4099
    src_off, dst_off = 3, 1
    gathered = torch.empty(k + src_off + 5, dtype=torch.int16, device=DEV)
    synth.device_index_hash16_(gathered)
    dst_full = torch.full((k + dst_off + 8,), 0x6B6B, dtype=torch.int16, device=DEV)
    dst = dst_full[dst_off:dst_off + k]
    plan = zc.unshard_plan_create([(src_off, dst, k)], gathered.numel())
    zc.unshard(plan, gathered)
    sync()
    chunk = 1 << 28
    for s in range(0, k, chunk):
        e = min(k, s + chunk)
        assert torch.equal(dst[s:e], synth.device_index_hash16_values(src_off + s, e - s, DEV)), f"chunk@{s}"
    assert (dst_full[:dst_off] == 0x6B6B).all() and (dst_full[dst_off + k:] == 0x6B6B).all()
    # ends and the 2^32 crossing against the oracle's element-by-element copy
    for s in (0, (1 << 32) - 2048, k - 4096):
        w = 4096
        want = oracle.unshard(host_u16(gathered[src_off + s:src_off + s + w]), [0], [w])[0]
        assert np.array_equal(host_u16(dst[s:s + w]), want)
    plan.destroy()
    del gathered, dst_full
    torch.cuda.empty_cache()


def test_norm_cast_and_accumulation_at_the_70b_shard_size():
    """The other streaming kernels at n = 8,819,213,312 (element indices past 2^33): every element
    against torch used as a double-precision / RNE calculator in chunks (properties that hold at
    any size), windows around the ends and around 2^32 against the oracle."""
    _, n, _ = zc.flat_layout(synth.tensor_numels(synth.LLAMA3_70B), 8, 1)
    g = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    synth.device_normal_(g, synth.G_STD, seed=2001)
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    chunk = 1 << 28
    # squared norm: the exact sum, accumulated in double chunk by chunk
    zc.grad_sqnorm(g, zc.BF16, n, norm, flag)
    sync()
    want = 0.0
    for s in range(0, n, chunk):
        want += float(g[s:min(n, s + chunk)].double().square().sum())
    assert flag.item() == 0 and abs(norm.item() - want) <= 1.3e-7 * want, (norm.item(), want)
    # one window's share of that sum against the oracle's own
    w_sq, w_bad = oracle.grad_sqnorm(host_u16(g[(1 << 32) - 4096:(1 << 32) + 4096]))
    assert w_bad == 0 and abs(w_sq - float(g[(1 << 32) - 4096:(1 << 32) + 4096].double().square().sum())) <= 1e-12 * w_sq
    # a non-finite element beyond index 2^33 is seen, and only while it is inside n
    at = (1 << 33) + 12345
    keep = g[at].clone()
    g[at] = float("inf")
    zc.grad_sqnorm(g, zc.BF16, n, norm, flag)
    sync()
    assert flag.item() == 1
    zc.grad_sqnorm(g, zc.BF16, at, norm, flag)
    sync()
    assert flag.item() == 0
    g[at] = keep
    print("norm ok", flush=True)
    # accumulation: acc + micro * scale in double, rounded once: torch's fp64 as the calculator
    acc = torch.empty(n, dtype=torch.float32, device=DEV)
    synth.device_normal_(acc, synth.G_STD, seed=2010)
    wins = [(s, w) for s, w in windows_for(n, count=6, width=1 << 12, seed=21)]
    before = [(host_f32(acc[s:s + w]).copy(), host_u16(g[s:s + w])) for s, w in wins]
    ref_head = (acc[:chunk].double() + g[:chunk].double() * 0.25).float()
    ref_tail = (acc[n - chunk:].double() + g[n - chunk:].double() * 0.25).float()
    mid = (1 << 32) - chunk // 2
    ref_mid = (acc[mid:mid + chunk].double() + g[mid:mid + chunk].double() * 0.25).float()
    zc.grad_accumulate(acc, g, zc.BF16, n, 0.25)
    sync()
    assert torch.equal(acc[:chunk], ref_head) and torch.equal(acc[n - chunk:], ref_tail)
    assert torch.equal(acc[mid:mid + chunk], ref_mid)
    for (s, w), (a0, gb) in zip(wins, before):
        oracle.grad_accumulate(a0, gb, 0.25)
        assert np.array_equal(host_f32(acc[s:s + w]).view(np.uint32), a0.view(np.uint32)), f"accumulate window@{s}"
    del ref_head, ref_tail, ref_mid
    print("accumulate ok", flush=True)
    # cast: RNE of every element (torch's narrowing as the library routine), oracle on windows
    out = torch.zeros(n, dtype=torch.int16, device=DEV)
    zc.cast_bf16(acc, out, n)
    sync()
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        assert torch.equal(acc[s:e].to(torch.bfloat16).view(torch.int16), out[s:e]), f"cast chunk@{s}"
    for s, w in wins:
        assert np.array_equal(host_u16(out[s:s + w]), oracle.cast_bf16(host_f32(acc[s:s + w]))), f"cast window@{s}"
    del g, acc, out
    torch.cuda.empty_cache()


@pytest.mark.parametrize("state_layout", ["arrays", "packed"])
def test_update_over_more_vectors_than_one_launch_can_count(state_layout):
    """n = 2^34 + 2^20 + 5 elements: more 16-byte vectors than the 2^32 - 1 threads one launch can
    have (a larger launch does not fail, it silently runs the count modulo 2^32), so the update is
    cut into two launches.  Step 1 from m = v = 0 has a closed form in every element, checked over
    the whole partition in chunks: an element no launch reached would keep m = 0.  240 GB resident."""
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    G = zc.PACKED_GRANULE
    n = (1 << 34) + (1 << 20) + 5
    b1, b2 = float(np.float32(HP["beta1"])), float(np.float32(HP["beta2"]))
    g = torch.empty(n, dtype=torch.bfloat16, device=DEV)
    synth.device_normal_(g, synth.G_STD, seed=4001)
    if state_layout == "packed":
        state = torch.empty(zc.packed_state_numel(n), dtype=torch.float32, device=DEV)
        cube = state.view(-1, 3, G)
        cube[:, 0].fill_(0.25)
        cube[:, 1:].zero_()
        zc.adam_step_packed(state, g, zc.BF16, n, zc.hparams(step=1, **HP))
    else:
        p = torch.full((n,), 0.25, dtype=torch.float32, device=DEV)
        m = torch.zeros(n, dtype=torch.float32, device=DEV)
        v = torch.zeros(n, dtype=torch.float32, device=DEV)
        zc.adam_step(p, m, v, g, zc.BF16, n, zc.hparams(step=1, **HP))
    sync()
    print("step done", flush=True)
    rows = 1 << 14                                              # 2^27 elements per chunk
    for k in range(0, -(-n // G), rows):
        s, e = k * G, min(n, (k + rows) * G)
        gd = g[s:e].double()
        if state_layout == "packed":
            k1 = min(cube.shape[0], k + rows)
            pm, mm, vm = (cube[k:k1, a].reshape(-1)[:e - s] for a in range(3))
        else:
            pm, mm, vm = p[s:e], m[s:e], v[s:e]
        assert torch.equal(mm, (gd * (1.0 - b1)).float()), f"m chunk@{s}"
        assert torch.equal(vm, ((gd * (1.0 - b2)) * gd).float()), f"v chunk@{s}"
        # p moved by the decay and by at most lr in (nearly) every element; the few whose update
        # cancels the decay exactly are why this is not asked of all of them
        assert float((pm != 0.25).float().mean()) > 0.999, f"p chunk@{s}"
        assert float((pm - 0.25).abs().max()) <= 1.01e-4, f"p chunk@{s}"
        del gd, pm, mm, vm
    if state_layout == "packed":
        del state, cube
    else:
        del p, m, v
    del g
    torch.cuda.empty_cache()
