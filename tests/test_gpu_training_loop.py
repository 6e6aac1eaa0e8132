"""GPU parity of the calls chained the way a training loop chains them, over several
iterations: micro-batch gradients accumulated in fp32, squared norm and overflow flag,
clipping coefficient with loss-scale removal, per-range AdamW writing its bf16 copy into
this rank's slot of the gathered buffer, unshard into per-layer tensors.  One iteration
overflows and must leave every buffer as it was.  Nothing between the calls of an
iteration waits for the host; the host reads the flag once per iteration, as a dynamic
loss scaler does."""
import numpy as np
import pytest
import torch

import oracle
from oracle import layout as olayout
from paper_2504_09983_amd import synth, zc
from tests.gpu_util import (DEV, HP, assert_state_close, bf16_ulp_diff, dev_f32, dev_u16, host_f32, host_u16,
                            sync, ulp_diff)

pytestmark = pytest.mark.gpu

WORLD, RANK, ALIGN = 4, 1, 8
BF16_INF = 0x7F80


def small_model():
    """(name, numel, is_norm) in canonical order; ragged on purpose (odd vocabulary)."""
    d, out = 96, [("embed", 1003 * 96, False)]
    for l in range(5):
        out += [(f"l{l}.q", d * d, False), (f"l{l}.k", 32 * d, False), (f"l{l}.v", 32 * d, False),
                (f"l{l}.o", d * d, False), (f"l{l}.up", 257 * d, False), (f"l{l}.down", d * 257, False),
                (f"l{l}.norm1", d, True), (f"l{l}.norm2", d, True)]
    out += [("final_norm", d, True), ("head", 1003 * d, False)]
    return out


def no_decay_ranges(tensors, offs, shard):
    """Norm vectors take no weight decay: their spans, cut to this rank's shard."""
    lo, hi = RANK * shard, (RANK + 1) * shard
    ranges = []
    for (name, k, is_norm), o in zip(tensors, offs):
        b, e = max(o, lo), min(o + k, hi)
        if is_norm and e > b:
            ranges.append((b - lo, e - lo, 1.0, 0.0))
    return ranges


def test_training_loop_with_accumulation_clipping_groups_overflow_and_unshard():
    tensors = small_model()
    numels = [k for _, k, _ in tensors]
    offs, shard, total = olayout.flat_layout(numels, WORLD, ALIGN)
    assert zc.flat_layout(numels, WORLD, ALIGN) == (list(offs), shard, total)
    n = shard
    ranges = no_decay_ranges(tensors, offs, shard)
    assert len(ranges) >= 2, "the shard must hold some norm vectors for the test to mean anything"

    # host state (oracle side) and device state
    p = synth.host_params(n, 60)
    m, v = np.zeros(n, np.float32), np.zeros(n, np.float32)
    gathered_h = synth.host_index_hash16(0, WORLD * shard)          # the other ranks' bytes
    dp, dm, dv = dev_f32(p), dev_f32(m), dev_f32(v)
    gathered_d = dev_u16(gathered_h)
    acc_d = torch.zeros(n, dtype=torch.float32, device=DEV)
    norm = torch.zeros(1, dtype=torch.float32, device=DEV)
    flag = torch.zeros(1, dtype=torch.int32, device=DEV)
    scale = torch.zeros(1, dtype=torch.float32, device=DEV)
    outs = [torch.full((k,), 0x1234, dtype=torch.int16, device=DEV) for k in numels]
    plan = zc.unshard_plan_create([(o, t, k) for o, t, k in zip(offs, outs, numels)], WORLD * shard)
    slot = gathered_d[RANK * shard:(RANK + 1) * shard]

    loss_scale, max_norm, micro_batches = 4096.0, 0.02, 2
    t, applied, skipped = 1, 0, 0
    for it in range(8):
        acc_h = np.zeros(n, np.float32)
        acc_d.zero_()
        gpu_before = [x.clone() for x in (dp, dm, dv, gathered_d)]
        for k in range(micro_batches):
            g = oracle.cast_bf16(synth.host_grads_f32(n, 100 * it + k) * np.float32(loss_scale))
            if it == 4 and k == 1:
                g[n // 3] = BF16_INF                                  # an overflowed micro-batch
            zc.grad_accumulate(acc_d, dev_u16(g), zc.BF16, n, scale=1.0 / micro_batches)
            oracle.grad_accumulate(acc_h, g, 1.0 / micro_batches)
        zc.grad_sqnorm(acc_d, zc.F32, n, norm, flag)
        zc.clip_scale(norm, max_norm, 1.0 / loss_scale, scale)
        zc.adam_step_groups(dp, dm, dv, acc_d, zc.F32, n, zc.hparams(step=t, **HP), ranges=ranges,
                            bf16_out=slot, skip_flag=flag, grad_scale_dev=scale)
        zc.unshard(plan, gathered_d)
        sync()

        assert np.array_equal(host_f32(acc_d).view(np.uint32), acc_h.view(np.uint32)), "accumulation is bit-exact"
        want_sq, want_bad = oracle.grad_sqnorm(acc_h)
        overflow = int(flag.item())
        assert overflow == want_bad == (1 if it == 4 else 0)
        if overflow:
            skipped += 1
            loss_scale /= 2.0                                         # and the step number stays
        else:
            # the oracle's own chain: double sum -> fp32 -> coefficient; the GPU's norm within an
            # fp32 ulp of it, its coefficient within two
            want32 = np.float32(want_sq)
            assert ulp_diff(np.float32(norm.item()), want32) <= 1
            c = oracle.clip_scale(want32, max_norm, 1.0 / loss_scale)
            assert ulp_diff(np.float32(scale.item()), c) <= 2
            slot_h = gathered_h[RANK * shard:(RANK + 1) * shard]
            oracle.adam_step_groups(p, m, v, acc_h, ranges=ranges, step=t, grad_scale_dev=c,
                                    bf16_out=slot_h, **HP)
            t += 1
            applied += 1
        if overflow:
            for name, a, b in zip(("p", "m", "v", "gathered"), (dp, dm, dv, gathered_d), gpu_before):
                assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a,
                                   b.view(torch.int32) if b.dtype == torch.float32 else b), f"{name} moved in a skipped step"
        # State against the oracle.  The two chains are independent, so the gradient scale
        # itself may differ by 2 fp32 ulp (checked above): m follows it (2 ulp + its rounding),
        # v its square (4 ulp + rounding), both weighted averages that do not accumulate: 6 ulp.
        # In p the scale cancels only up to those roundings: m and v a few ulp apart move the
        # lr-sized term m / sqrt(v) by a few ulp of lr in every applied step, which shows in
        # elements near zero: 3 * applied + 2 ulp at max(|p|, lr).
        k = max(applied, 1)
        assert_state_close(host_f32(dp), host_f32(dm), host_f32(dv), p, m, v, tag=f"iteration {it}",
                           steps=k, m_floor=1e-5, p_ulp=3 * k + 2, mv_ulp=6)
        # the rank's slot: RNE of the GPU's own p, within 1 bf16 ulp of the oracle's copy
        got_slot = host_u16(slot)
        if applied:
            assert np.array_equal(got_slot, oracle.cast_bf16(host_f32(dp)))
            assert bf16_ulp_diff(got_slot, gathered_h[RANK * shard:(RANK + 1) * shard]).max() <= 1
        # per-layer tensors: bit copies of the GPU's gathered buffer, laid out as the oracle says
        want = oracle.unshard(host_u16(gathered_d), list(offs), numels)
        for (name, _, _), o, w in zip(tensors, outs, want):
            assert np.array_equal(host_u16(o), w), name
    assert applied == 7 and skipped == 1
    plan.destroy()
