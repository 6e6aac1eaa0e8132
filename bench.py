#!/usr/bin/env python3
"""Benchmark of one rank's sharded mixed-precision optimizer step on one MI355X.

The default run measures the largest configurations one GPU holds, the two models the
paper evaluates (Evaluation, Experimental settings), one after the other:

  headline   Llama-3-70B-shaped one-of-8 shard, 8,819,213,312 fp32 elements, 141 GB resident:
                 zc_grad_sqnorm  (overflow flag + squared norm of the bf16 gradient shard)
                 zc_adam_step_packed (fused AdamW over the packed p/m/v state array, bf16 copy into
                                 the send buffer, skipped on overflow; --state-layout arrays times
                                 zc_adam_step over three separate arrays instead, and the default
                                 run reports that one beside it)
             `value` = shard elements / wall time of one such step.  The unshard copy of this
             model (141 GB gathered + 141 GB of tensors) does not fit next to the step's state,
             so row a3 of the path is timed at its own largest size:
  unshard    Mixtral-8x7B-shaped gathered buffer of 8 rank shards (46.7 B bf16 elements,
             rank-padded) -> 995 per-layer tensors, zc_unshard.
  whole_step_llama3_8b   all three calls back to back on the Llama-3-8B-shaped shard, where
             they fit together, as in the previous default of this benchmark.

Everything is resident in HBM when a timed region starts.  Kernel durations come from HIP
events recorded on the launch stream inside the timed region.  Prints ONE JSON line.

Legs outside the timed region: the update kernel's other gradient/copy variants, rows built
after the main path, the offloaded step (pinned host p/m/v) at the largest size the host pins,
and the CPU oracle on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
PCIE_PEAK_GBS = 63.0           # Gen5 x16, per direction
WORLD = 8
GIB = 1 << 30


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="headline",
                    choices=["headline", "llama3_8b", "llama3_70b", "mixtral_8x7b", "tiny"],
                    help="headline = 70B shard step + Mixtral unshard + 8B whole step (default); "
                         "a model name = that model's shard only")
    ap.add_argument("--state-layout", default="packed", choices=["packed", "arrays"],
                    help="how the timed step holds p, m, v: the library's packed state array "
                         "(zc_adam_step_packed, default) or three arrays (zc_adam_step); the other one "
                         "is timed beside it unless --no-next-rows")
    ap.add_argument("--no-unshard", action="store_true",
                    help="single-model workloads: leave the unshard copy out")
    ap.add_argument("--only-unshard", action="store_true",
                    help="single-model workloads: time the unshard copy alone")
    ap.add_argument("--offload-elems", type=int, default=8_819_213_312,
                    help="partition size of the offload leg (0 = skip the leg); shrunk to what the "
                         "host can pin")
    ap.add_argument("--offload-fracs", default="0,0.5", help="resident fractions f of the offload leg")
    ap.add_argument("--offload-max-pinned-gib", type=float, default=60.0,
                    help="largest total of pinned host memory to ask for")
    ap.add_argument("--offload-chunk-mib", type=int, default=64)
    ap.add_argument("--offload-buffers", type=int, default=3)
    ap.add_argument("--offload-side-elems", type=int, default=1 << 30,
                    help="streamed elements for the two staged transports and the link probes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip the legs for step variants, gradient accumulation, the per-tensor "
                         "layout and the planner replay")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain copy of known size (one unshard segment of 2^30 bf16 "
                         "elements, 2 GiB read + 2 GiB written, 5 launches): the reference for "
                         "scaling the WRITE_SIZE counter")
    ap.add_argument("--calibrate-read", action="store_true",
                    help="only run a read of known size (zc_grad_sqnorm over 2^30 fp32 elements, "
                         "4 GiB read, 5 launches): the reference for scaling the FETCH_SIZE counter")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="tuning knob, e.g. adam.rows=4 (repeatable)")
    return ap.parse_args()


def gb(x):
    return x / 1e9


def time_launches(torch, fn, reps=10):
    """Average HIP-event time of `reps` calls of fn on torch's current stream (the launch stream)."""
    fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in ev) / reps


def kernel_record(name, ms_list, nbytes, units, bytes_per_unit):
    ms_sorted = sorted(ms_list)
    ms = sum(ms_sorted) / len(ms_sorted)
    gbps = gb(nbytes) / (ms * 1e-3)
    return dict(name=name, ms=round(ms, 4), ms_median=round(ms_sorted[len(ms_sorted) // 2], 4),
                ms_min=round(ms_sorted[0], 4), GBps=round(gbps, 1), frac=round(gbps / HBM_PEAK_GBS, 4),
                algorithmic_bytes=nbytes, bytes_per_unit=bytes_per_unit,
                rate_G_per_s=round(units / (ms * 1e-3) / 1e9, 2))


def shard_of(zc, synth, workload):
    import numpy as np
    tensors = synth.TINY_TENSORS if workload == "tiny" else synth.tensor_list(synth.SHAPES[workload])
    numels = [int(np.prod(d)) for _, d in tensors]
    return tensors, numels


def step_phase(torch, synth, zc, dev, workload, steps, warmup, with_unshard, with_step=True, variants=False,
               layout="packed"):
    """grad-norm + fused AdamW with bf16 copy (+ unshard of the 8-shard gathered buffer) on one
    model's one-of-8 shard.  `layout`: "packed" keeps p, m, v in the library's granule-interleaved
    state array (zc_adam_step_packed), "arrays" in three separate arrays (zc_adam_step).
    Returns (record, seconds of the timed region)."""
    tensors, numels = shard_of(zc, synth, workload)
    offs, shard, total = zc.flat_layout(numels, WORLD, 1)
    n = shard
    hp_kw = dict(synth.HP)
    packed = layout == "packed"
    if with_step:
        if packed:
            state = torch.empty(zc.packed_state_numel(n), dtype=torch.float32, device=dev)
            cube = state.view(-1, 3, zc.PACKED_GRANULE)
            gen = torch.Generator(device=dev)
            gen.manual_seed(2)
            for k in range(0, cube.shape[0], 1 << 12):          # p ~ N(0, sigma); m = v = 0
                rows = min(1 << 12, cube.shape[0] - k)
                cube[k:k + rows, 0] = torch.randn(rows, zc.PACKED_GRANULE, generator=gen, device=dev) * synth.P_STD
            cube[:, 1:].zero_()
        else:
            p = torch.empty(n, dtype=torch.float32, device=dev)
            m = torch.zeros(n, dtype=torch.float32, device=dev)
            v = torch.zeros(n, dtype=torch.float32, device=dev)
            synth.device_normal_(p, synth.P_STD, seed=2)
        g = torch.empty(n, dtype=torch.bfloat16, device=dev)
        synth.device_normal_(g, synth.G_STD, seed=2001)

    def update(grad, dtype, hp, **kw):
        if packed:
            zc.adam_step_packed(state, grad, dtype, n, hp, **kw)
        else:
            zc.adam_step(p, m, v, grad, dtype, n, hp, **kw)
    norm = torch.zeros(1, dtype=torch.float32, device=dev)
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    if with_unshard:
        gathered = torch.empty(WORLD * shard, dtype=torch.int16, device=dev)
        synth.device_index_hash16_(gathered)          # the other 7 ranks' bytes
        send = gathered[:n]                            # this rank's slot (rank 0)
        outs = [torch.empty(d, dtype=torch.bfloat16, device=dev) for _, d in tensors]
        plan = zc.unshard_plan_create([(o, t, k) for o, t, k in zip(offs, outs, numels)], WORLD * shard)
    else:
        send = torch.empty(n, dtype=torch.int16, device=dev)
    torch.cuda.synchronize()
    step_no = [0]

    def one_step(ev=None):
        step_no[0] += 1
        hp = zc.hparams(step=step_no[0], **hp_kw)
        if ev: ev[0].record()
        if with_step:
            zc.grad_sqnorm(g, zc.BF16, n, norm, flag)
        if ev: ev[1].record()
        if with_step:
            update(g, zc.BF16, hp, bf16_out=send, skip_flag=flag)
        if ev: ev[2].record()
        if with_unshard:
            zc.unshard(plan, gathered)
        if ev: ev[3].record()

    for _ in range(warmup):
        one_step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        one_step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert flag.item() == 0, "synthetic gradients must be finite"

    def times(i):
        return [e[i].elapsed_time(e[i + 1]) for e in events]

    kernels = {}
    if with_step:
        kernels["sqnorm"] = kernel_record("zc::sqnorm_bf16_kernel", times(0), 2 * n, n, 2)
        kernels["adam"] = kernel_record("zc::adam_vec_kernel", times(1), 28 * n, n, 28)
    if with_unshard:
        kernels["unshard"] = kernel_record("zc::unshard_kernel", times(2), 4 * total, total, 4)
    rec = {"workload": workload, "shard_elements": n, "model_elements": total, "tensors": len(numels),
           "state_layout": ("one packed array (granules of %d elements of p, m, v)" % zc.PACKED_GRANULE) if packed
           else "three arrays",
           "ms_per_step": round(wall * 1e3 / steps, 4),
           "gparams_per_s": round(n / (wall / steps) / 1e9, 3), "kernels": kernels}

    if variants and with_step:
        def hp_next():
            step_no[0] += 1
            return zc.hparams(step=step_no[0], **hp_kw)

        g32 = torch.empty(n, dtype=torch.float32, device=dev)
        synth.device_normal_(g32, synth.G_STD, seed=2999)
        rows = {
            "bf16_grads_fused_copy": (28, lambda: update(g, zc.BF16, hp_next(), bf16_out=send)),
            "bf16_grads_no_copy": (26, lambda: update(g, zc.BF16, hp_next())),
            "fp32_grads_fused_copy": (30, lambda: update(g32, zc.F32, hp_next(), bf16_out=send)),
            "fp32_grads_no_copy": (28, lambda: update(g32, zc.F32, hp_next())),
        }
        if not packed:                 # the standalone cast reads a contiguous p
            rows["unfused_step_then_cast"] = (32, lambda: (zc.adam_step(p, m, v, g, zc.BF16, n, hp_next()),
                                                           zc.cast_bf16(p, send, n)))
            rows["standalone_cast"] = (6, lambda: zc.cast_bf16(p, send, n))
        rec["step_variants"] = {}
        for name, (bpe, fn) in rows.items():
            ms = time_launches(torch, fn, reps=10 if n < (1 << 32) else 5)
            rec["step_variants"][name] = {"bytes_per_element": bpe, "ms": round(ms, 4),
                                          "GBps": round(gb(bpe * n) / (ms * 1e-3), 1),
                                          "frac": round(gb(bpe * n) / (ms * 1e-3) / HBM_PEAK_GBS, 4),
                                          "gparams_per_s": round(n / (ms * 1e-3) / 1e9, 2)}
        del g32
    if with_unshard:
        plan.destroy()
        del outs, gathered
    if with_step:
        if packed:
            del state, cube
        else:
            del p, m, v
        del g
    del send
    torch.cuda.empty_cache()
    return rec, wall


def placement_leg(torch, synth, zc, dev):
    """Where the caller puts p, m, v matters for small partitions: the same launch over the
    Llama-3-8B shard with the five arrays back to back (what an allocator gives for 4 GB arrays)
    and with each array 16 or 36 GiB after the previous one inside one arena."""
    n = 1_003_782_656
    arena = torch.empty(4 * 36 * GIB + 3 * GIB, dtype=torch.uint8, device=dev)
    base = arena.data_ptr()

    def noise(offset, nbytes, seed):                    # N(0, sigma) values, as in the main run
        nbytes = nbytes // 4 * 4
        synth.device_normal_(arena[offset:offset + nbytes].view(torch.float32), synth.P_STD, seed=seed)

    hp = zc.hparams(step=3, **synth.HP)

    def up(x, a):
        return (x + a - 1) // a * a

    s0 = up(4 * n, 2 << 20)
    layouts = {"back_to_back": [0, s0, 2 * s0, 3 * s0, 3 * s0 + up(2 * n, 2 << 20)],
               "16_GiB_apart": [k * 16 * GIB for k in range(5)],
               "36_GiB_apart": [k * 36 * GIB for k in range(5)]}
    out = {}
    for name, offs in layouts.items():
        for k, o in enumerate(offs):
            noise(o, (4 if k < 3 else 2) * n, seed=11 + k)
        ptr = [base + o for o in offs]
        ms = time_launches(torch, lambda: zc.adam_step(ptr[0], ptr[1], ptr[2], ptr[3], zc.BF16, n, hp,
                                                       bf16_out=ptr[4]), reps=10)
        out[name] = {"ms": round(ms, 4), "GBps": round(gb(28 * n) / (ms * 1e-3), 1),
                     "frac": round(gb(28 * n) / (ms * 1e-3) / HBM_PEAK_GBS, 4)}
    del arena
    torch.cuda.empty_cache()
    return {"elements": n, "bytes_per_element": 28, **out}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a one-GPU path (one rank's share of the step, the other "
              "ranks' bytes synthesised locally); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2504_09983_amd import synth, zc

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    for kv in args.tune:
        k, val = kv.split("=")
        zc.tune_set(k, int(val))

    if args.calibrate_copy:
        k = 1 << 30
        src = torch.empty(k, dtype=torch.int16, device=dev)
        dst = torch.empty(k, dtype=torch.int16, device=dev)
        synth.device_index_hash16_(src)
        plan = zc.unshard_plan_create([(0, dst, k)], k)
        for _ in range(5):
            zc.unshard(plan, src)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
        print(json.dumps({"calibrate_copy": {"kernel": "zc::unshard_kernel", "launches": 5,
                                             "read_bytes_per_launch": 2 * k,
                                             "written_bytes_per_launch": 2 * k}}))
        return
    if args.calibrate_read:
        k = 1 << 30
        src = torch.empty(k, dtype=torch.float32, device=dev)
        synth.device_normal_(src, synth.G_STD, seed=1)
        norm = torch.zeros(1, dtype=torch.float32, device=dev)
        flag = torch.zeros(1, dtype=torch.int32, device=dev)
        for _ in range(5):
            zc.grad_sqnorm(src, zc.F32, k, norm, flag)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_read": {"kernel": "zc::sqnorm_f32_kernel", "launches": 5,
                                             "read_bytes_per_launch": 4 * k}}))
        return

    link = link_leg(torch, synth, zc, dev, args) if args.offload_elems > 0 else None
    tuning = {k: zc.tune_get(k) for k in ("adam.arith", "adam.block", "adam.rows", "adam.waves_per_cu",
                                          "adam.nontemporal", "copy.waves_per_cu", "copy.nontemporal")}
    extra = {}
    if args.workload == "headline":
        head, wall = step_phase(torch, synth, zc, dev, "llama3_70b", args.steps, args.warmup,
                                with_unshard=False, variants=not args.no_next_rows, layout=args.state_layout)
        if not args.no_next_rows:
            other = "arrays" if args.state_layout == "packed" else "packed"
            alt, _ = step_phase(torch, synth, zc, dev, "llama3_70b", args.steps, args.warmup,
                                with_unshard=False, variants=True, layout=other)
            extra["llama3_70b_with_" + ("three_state_arrays" if other == "arrays" else "packed_state")] = alt
        unsh, _ = step_phase(torch, synth, zc, dev, "mixtral_8x7b", args.steps, args.warmup,
                             with_unshard=True, with_step=False)
        kernels = dict(head["kernels"])
        kernels["unshard"] = unsh["kernels"]["unshard"]
        extra["unshard_mixtral_8x7b"] = {k: unsh[k] for k in ("model_elements", "tensors")}
        extra["unshard_mixtral_8x7b"]["gathered_elements"] = \
            WORLD * zc.flat_layout(shard_of(zc, synth, "mixtral_8x7b")[1], WORLD, 1)[1]
        small, _ = step_phase(torch, synth, zc, dev, "llama3_8b", args.steps, args.warmup,
                              with_unshard=True, variants=not args.no_next_rows, layout=args.state_layout)
        extra["whole_step_llama3_8b"] = small
        if not args.no_next_rows:
            other = "arrays" if args.state_layout == "packed" else "packed"
            alt, _ = step_phase(torch, synth, zc, dev, "llama3_8b", args.steps, args.warmup,
                                with_unshard=False, variants=True, layout=other)
            extra["llama3_8b_with_" + ("three_state_arrays" if other == "arrays" else "packed_state")] = alt
        workload_text = ("llama3_70b one-of-8 shard: grad-norm + fused AdamW with bf16 copy (141 GB resident); "
                         "unshard timed on the mixtral_8x7b gathered buffer of 8 shards (46.7 B elements -> 995 "
                         "tensors), which does not fit beside the 70B step")
    else:
        do_unshard = not args.no_unshard
        do_step = not args.only_unshard
        head, wall = step_phase(torch, synth, zc, dev, args.workload, args.steps, args.warmup,
                                with_unshard=do_unshard, with_step=do_step, variants=not args.no_next_rows,
                                layout=args.state_layout)
        kernels = dict(head["kernels"])
        workload_text = (f"{args.workload} one-of-{WORLD} shard: "
                         + ("grad-norm + fused AdamW with bf16 copy" if do_step else "")
                         + (" + " if do_step and do_unshard else "")
                         + ("unshard of the 8-shard gathered buffer" if do_unshard else ""))

    ms_per_step = wall * 1e3 / args.steps
    n = head["shard_elements"]
    dominant = max(kernels, key=lambda k: kernels[k]["ms"])
    dom = kernels[dominant]
    dom_workload = "mixtral_8x7b" if (args.workload == "headline" and dominant == "unshard") else \
        ("llama3_70b" if args.workload == "headline" else args.workload)

    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    if os.path.exists(tpath):
        try:
            key = "adam_packed" if (dominant == "adam" and args.state_layout == "packed") else dominant
            rec = json.load(open(tpath)).get(dom_workload, {}).get(key)
            if rec:
                traffic = rec["fetch_bytes"] + rec["write_bytes"]
                traffic_source = ("profiles/pmc_traffic.json: FETCH_SIZE and WRITE_SIZE of this kernel at this "
                                  "size from separate rocprofv3 --pmc runs, not counted in this run")
        except Exception:
            traffic = None

    roofline = dict(bound="hbm", kernel=dom["name"], workload=dom_workload, achieved=dom["GBps"],
                    peak=HBM_PEAK_GBS, unit="GB/s", frac=dom["frac"], traffic=traffic,
                    traffic_source=traffic_source, algorithmic_bytes_per_launch=dom["algorithmic_bytes"],
                    avg_launch_ms=dom["ms"], target_frac=0.80,
                    below_target=[f"{k} {d['frac']}" for k, d in kernels.items() if d["frac"] < 0.80])

    result = {
        "metric": "optimizer-step Gparams/s per shard",
        "value": round(n / (ms_per_step * 1e-3) / 1e9, 3),
        "unit": "Gparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {0: "f32", 1: "f32+f64", 2: "f64"}[zc.tune_get("adam.arith")], "data": "synthetic",
        "config": {"workload": workload_text, "shard_elements": n, "model_elements": head["model_elements"],
                   "tensors": head["tensors"], "grads": "bf16",
                   "state": "fp32 p/m/v resident in HBM, " + head["state_layout"],
                   "tuning": tuning},
        "roofline": roofline,
        "kernels": kernels,
    }
    if "adam" in kernels:
        result["adam_step_gparams_per_s"] = kernels["adam"]["rate_G_per_s"]
    if "step_variants" in head:
        result["step_variants"] = head["step_variants"]
    result.update(extra)

    if not args.no_next_rows:
        result["placement_llama3_8b_shard"] = placement_leg(torch, synth, zc, dev)
        result["next_rows"] = next_rows_leg(torch, synth, zc, dev)
        result["next_rows"]["adaptive_offload_plan"] = adaptive_plan_leg(torch, zc, dev)
    if args.offload_elems > 0:
        result["offload"] = offload_leg(torch, synth, zc, dev, args, link)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline_leg(synth)
    print(json.dumps(result))


def next_rows_leg(torch, synth, zc, dev):
    """Rows built after the main path: fp32 gradient accumulation (10 B/element) and the
    unshard copy in the per-tensor even-partition layout (8 segments per tensor), with slices
    padded to 8 elements (16-byte aligned sources) and unpadded (2- and 4-byte aligned sources)."""
    import numpy as np
    shape = synth.LLAMA3_8B
    tensors = synth.tensor_list(shape)
    numels = [int(np.prod(d)) for _, d in tensors]
    n = sum(numels) // WORLD
    acc = torch.zeros(n, dtype=torch.float32, device=dev)
    micro = torch.empty(n, dtype=torch.bfloat16, device=dev)
    synth.device_normal_(micro, synth.G_STD, seed=2003)
    t_acc = time_launches(torch, lambda: zc.grad_accumulate(acc, micro, zc.BF16, n, 0.25))
    del acc, micro
    total = sum(numels)
    out = {"grad_accumulate": {"elements": n, "ms": round(t_acc, 4), "bytes_per_element": 10,
                               "GBps": round(gb(10 * n) / (t_acc * 1e-3), 1),
                               "frac": round(gb(10 * n) / (t_acc * 1e-3) / HBM_PEAK_GBS, 4)}}
    outs = [torch.empty(d, dtype=torch.bfloat16, device=dev) for _, d in tensors]
    # align 8: every slice starts on a 16-byte boundary.  The second list (every tensor nine
    # elements short, align 1) has odd slice sizes, which puts sources and destinations on 2- and
    # 4-byte boundaries: the kernel's narrow-load paths.
    for name, sizes, align in (("unshard_per_tensor", numels, 8),
                               ("unshard_per_tensor_misaligned_sources", [k - 9 for k in numels], 1)):
        segs, send = zc.per_tensor_layout(sizes, WORLD, align)
        gathered = torch.empty(WORLD * send, dtype=torch.int16, device=dev)
        synth.device_index_hash16_(gathered)
        table = [(src, outs[t].data_ptr() + 2 * dst if k else None, k) for t, src, dst, k in segs]
        plan = zc.unshard_plan_create(table, WORLD * send)
        t_un = time_launches(torch, lambda: zc.unshard(plan, gathered))
        plan.destroy()
        moved = sum(sizes)
        classes = {"16B": 0, "4B": 0, "2B": 0}
        for t, src, dst, k in segs:
            if k:
                head = ((16 - (outs[t].data_ptr() + 2 * dst) % 16) % 16) // 2
                a = (gathered.data_ptr() + 2 * (src + head)) % 16
                classes["16B" if a == 0 else ("4B" if a % 4 == 0 else "2B")] += 1
        out[name] = {"elements": moved, "segments": sum(1 for s in segs if s[3]), "source_alignment_of_segments": classes,
                     "ms": round(t_un, 4), "bytes_per_element": 4,
                     "GBps": round(gb(4 * moved) / (t_un * 1e-3), 1),
                     "frac": round(gb(4 * moved) / (t_un * 1e-3) / HBM_PEAK_GBS, 4)}
        del gathered
    del outs
    torch.cuda.empty_cache()
    return out


def adaptive_plan_leg(torch, zc, dev):
    """The paper's adaptive offloading (Algorithm 2 + backward reload) planned on a synthetic
    memory profile (rising through the forward pass, falling through the backward pass) and
    replayed with stand-in compute kernels: 32 optimizer-state fragments of 64 MiB, 24 of which
    must leave, 16 + 16 operators of 8 ms.  Compared with offloading everything synchronously
    (the comparison mode of the paper's Evaluation, Adaptive Offloading) and with no offloading."""
    nfrags, elems = 32, 16 << 20
    state = torch.zeros(nfrags * elems, dtype=torch.float32, device=dev)
    host = [zc.host_alloc(4 * elems) for _ in range(nfrags)]
    frags = [(state[f * elems:(f + 1) * elems], host[f], 4 * elems) for f in range(nfrags)]
    n_f = 16
    up = [int(10 + 90 * (i + 1) / n_f) for i in range(n_f)]
    p_mem = up + up[::-1]
    ops = zc.plan_adaptive_offload(p_mem, n_f, [2] * nfrags, 116)
    ops_all = ([(zc.OP_OFFLOAD, f) for f in range(nfrags)] + [(zc.OP_SYNC_FREE, f) for f in range(nfrags)]
               + [(zc.OP_COMPUTE, i) for i in range(len(p_mem))]
               + [(zc.OP_RELOAD, f) for f in range(nfrags)] + [(zc.OP_SYNC_RELOAD, f) for f in range(nfrags)])
    ms = [8.0] * len(p_mem)
    ctx = zc.offload_create(1 << 20, 2)

    def run(sched):
        ctx.schedule_run(sched, ms, frags, poison_freed=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.schedule_run(sched, ms, frags, poison_freed=True)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    t_none = run([(zc.OP_COMPUTE, i) for i in range(len(p_mem))])
    t_adaptive = run(ops)
    t_sync = run(ops_all)
    ctx.destroy()
    del state, frags
    for h in host:
        h.free()
    moved = sum(1 for k, _ in ops if k == zc.OP_OFFLOAD)
    return {"operators": len(p_mem), "operator_ms": 8.0, "fragments": nfrags, "fragment_MiB": 64,
            "fragments_offloaded_by_plan": moved, "ms_no_offload": round(t_none, 1),
            "ms_adaptive_plan": round(t_adaptive, 1), "ms_offload_all_sync": round(t_sync, 1),
            "sync_over_adaptive": round(t_sync / t_adaptive, 3),
            "adaptive_over_no_offload": round(t_adaptive / t_none, 3),
            "overlap_holds": bool(t_adaptive < 0.95 * t_sync and t_adaptive < 1.25 * t_none)}


def link_leg(torch, synth, zc, dev, args):
    """Plain pinned-copy ceilings of the host link (one direction at a time and both at once,
    in chunk-sized pieces on the context's two copy streams) and the two staged transports of
    the offloaded step, over --offload-side-elems streamed elements.  Runs before anything
    else in the process: both depend on the runtime giving the two copy streams hardware
    queues of their own, which it does for the first streams a process creates; created late
    in a long-lived process they were seen sharing a queue, which serialises the two
    directions (28.8 instead of 48.3 GB/s each way)."""
    side = int(args.offload_side_elems)
    bufs = [zc.host_alloc(4 * side) for _ in range(3)]
    hp_, hm_, hv_ = (torch.from_numpy(b.numpy("float32")) for b in bufs)
    tmp = torch.empty(side, dtype=torch.float32, device=dev)
    synth.device_normal_(tmp, synth.P_STD, seed=3)
    hp_.copy_(tmp)
    hm_.zero_()
    hv_.zero_()
    del tmp
    ctx = zc.offload_create(args.offload_chunk_mib << 20, args.offload_buffers)
    nbytes = 4 * side
    t_h2d = min(ctx.probe_link(bufs[0], bufs[2], nbytes, 0) for _ in range(3)) * 1e-3
    t_d2h = min(ctx.probe_link(bufs[0], bufs[2], nbytes, 1) for _ in range(3)) * 1e-3
    t_both = min(ctx.probe_link(bufs[0], bufs[2], nbytes, 2) for _ in range(3)) * 1e-3
    hv_.zero_()
    out = {"memcpy_ceiling_GBps": {"h2d": round(gb(nbytes) / t_h2d, 2), "d2h": round(gb(nbytes) / t_d2h, 2),
                                   "both_each": round(gb(nbytes) / t_both, 2), "bytes": nbytes}}
    keep = zc.tune_get("offload.zero_copy")
    for mode, name in ((2, "staged_reads_direct_writes"), (0, "staged_ring"), (1, "zero_copy_same_size")):
        zc.tune_set("offload.zero_copy", mode)
        out[name] = timed_offload(torch, synth, zc, dev, ctx, bufs, side, 0, side, reps=3)
    zc.tune_set("offload.zero_copy", keep)
    ctx.destroy()
    del hp_, hm_, hv_
    for b in bufs:
        b.free()
    return out


def timed_offload(torch, synth, zc, dev, ctx, bufs, n, n_res, n_str, reps):
    dp, dm, dv = (torch.zeros(max(n_res, 1), dtype=torch.float32, device=dev) for _ in range(3))
    g = torch.empty(n, dtype=torch.bfloat16, device=dev)
    synth.device_normal_(g, synth.G_STD, seed=2002)
    send = torch.empty(n, dtype=torch.int16, device=dev)

    def run(step):
        ctx.adam_step(dp if n_res else None, dm if n_res else None, dv if n_res else None, n_res,
                      bufs[0], bufs[1], bufs[2], n_str, g, zc.BF16, zc.hparams(step=step, **synth.HP),
                      bf16_out_dev=send)

    run(1)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(reps):
        run(2 + k)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps
    del dp, dm, dv, g, send
    torch.cuda.empty_cache()
    one_way = 12 * n_str
    return {"elements": n, "streamed_elements": n_str, "pinned_GB": round(12 * n_str / 1e9, 2),
            "resident_fraction": round(n_res / n, 4), "ms_per_step": round(dt * 1e3, 3),
            "gparams_per_s": round(n / dt / 1e9, 3),
            "link_GBps_each_direction": round(gb(one_way) / dt, 2),
            "frac_of_link_peak": round(gb(one_way) / dt / PCIE_PEAK_GBS, 4)}


def offload_leg(torch, synth, zc, dev, args, link):
    """Offloaded step in its default zero-copy transport at the largest partition the host
    pins, for each resident fraction asked (p/m/v of the streamed part in pinned host DRAM)."""
    n_asked = int(args.offload_elems)
    fracs = [float(x) for x in args.offload_fracs.split(",")]
    # three pinned arrays as large as the streamed part needs, up to the cap; a host that
    # refuses gets asked for 7/8 of that, and so on
    cap_bytes = int(args.offload_max_pinned_gib * GIB)
    need = min(cap_bytes, 12 * int(max((1.0 - f) * n_asked for f in fracs)))
    cap_elems = (need // 12) // 1024 * 1024
    refused = []
    while True:
        bufs = []
        try:
            for _ in range(3):
                bufs.append(zc.host_alloc(4 * max(cap_elems, 1)))
            break
        except zc.ZcError as e:
            refused.append({"GiB": round(12 * cap_elems / GIB, 2), "error": e.message[:80]})
            for b in bufs:
                b.free()
            cap_elems = (cap_elems * 7 // 8) // 1024 * 1024
            if cap_elems < (1 << 20):
                raise
    pinned_limit = {"asked_GiB": round(need / GIB, 2), "granted_GiB": round(12 * cap_elems / GIB, 2),
                    "refused": refused}
    hp_, hm_, hv_ = (torch.from_numpy(b.numpy("float32")) for b in bufs)
    piece = 1 << 28
    tmp = torch.empty(piece, dtype=torch.float32, device=dev)
    for s0 in range(0, cap_elems, piece):              # p ~ N(0, 0.02); m = v = 0
        e0 = min(cap_elems, s0 + piece)
        synth.device_normal_(tmp[:e0 - s0], synth.P_STD, seed=3 + s0 // piece)
        hp_[s0:e0].copy_(tmp[:e0 - s0])
    hm_.zero_()
    hv_.zero_()
    del tmp
    ctx = zc.offload_create(args.offload_chunk_mib << 20, args.offload_buffers)
    out = {"pinned_limit": pinned_limit, "chunk_MiB": args.offload_chunk_mib, "buffers": args.offload_buffers,
           "link_peak_GBps": PCIE_PEAK_GBS, "host_numa": gpu_numa_node(torch), "zero_copy": {}}
    assert zc.tune_get("offload.zero_copy") == 1
    for f in fracs:
        n = n_asked
        if (1.0 - f) * n > cap_elems:                   # shrink the partition, keep the fraction
            n = int(cap_elems / (1.0 - f)) // 1024 * 1024
        n_res = int(f * n) // 1024 * 1024
        rec = timed_offload(torch, synth, zc, dev, ctx, bufs, n, n_res, n - n_res, reps=3)
        rec["elements_asked"] = n_asked
        out["zero_copy"][f"f={f:g}"] = rec
    ctx.destroy()
    del hp_, hm_, hv_
    for b in bufs:
        b.free()
    out.update(link)
    best = out["zero_copy"][f"f={fracs[0]:g}"]["link_GBps_each_direction"]
    out["roofline"] = {"bound": "host link (PCIe Gen5 x16), each direction", "kernel": "zc::adam_vec_kernel over pinned host p/m/v",
                       "achieved": best, "peak": PCIE_PEAK_GBS, "unit": "GB/s", "frac": round(best / PCIE_PEAK_GBS, 4),
                       "algorithmic_bytes_per_element_each_way": 12, "target_frac": 0.80, "below_target": True}
    out["roofline"]["below_target"] = out["roofline"]["frac"] < 0.80
    out["headline"] = {"transport": "zero_copy", "link_GBps_each_direction": best,
                       "frac_of_link_peak_63": round(best / PCIE_PEAK_GBS, 4),
                       "frac_of_duplex_memcpy_ceiling": round(best / out["memcpy_ceiling_GBps"]["both_each"], 4),
                       "target_frac_of_link_peak": 0.80,
                       "note": "0.80 of 63 GB/s (50.4 each way at once) is above what plain pinned copies "
                               "reach on this link with both directions busy"}
    return out


def gpu_numa_node(torch):
    """NUMA node the GPU hangs off, as the kernel reports it (-1: the host exposes no node
    information, as on a single-socket or virtualised box; nothing to bind to then)."""
    info = {"gpu_numa_node": None}
    try:
        props = torch.cuda.get_device_properties(0)
        bus = getattr(props, "pci_bus_id", None)
        dom = getattr(props, "pci_domain_id", 0)
        dev_id = getattr(props, "pci_device_id", 0)
        if bus is not None:
            path = f"/sys/bus/pci/devices/{dom:04x}:{bus:02x}:{dev_id:02x}.0/numa_node"
            info["gpu_numa_node"] = int(open(path).read().strip())
    except Exception as e:
        info["error"] = repr(e)
    return info


def cpu_baseline_leg(synth):
    """The CPU oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np

    import oracle

    ns = 1 << 26                                   # shard sample; gathered sample = 8x that
    passes = 16
    p = synth.host_params(ns, 2)
    m = np.zeros(ns, np.float32)
    v = np.zeros(ns, np.float32)
    g = oracle.cast_bf16(synth.host_normal(ns, synth.G_STD, 2001))
    gathered = synth.host_index_hash16(0, WORLD * ns)
    send = gathered[:ns]
    # tensor boundaries: ragged cuts of the sample, not aligned to the shard
    cuts = [0, ns // 3 + 5, ns * 2 + 17, ns * 5 - 3, WORLD * ns]
    offs = cuts[:-1]
    nums = [b - a for a, b in zip(cuts[:-1], cuts[1:])]
    # `value` is defined like the GPU's: elements per second of grad-norm + AdamW + bf16 copy;
    # the unshard copy is timed by itself, as it is on the GPU
    t0 = time.perf_counter()
    for t in range(1, passes + 1):
        _, bad = oracle.grad_sqnorm(g)
        oracle.adam_step(p, m, v, g, step=t, bf16_out=send, skip=bool(bad), **synth.HP)
    dt = (time.perf_counter() - t0) / passes
    t0 = time.perf_counter()
    for t in range(4):
        oracle.unshard(gathered, offs, nums)
    dt_unshard = (time.perf_counter() - t0) / 4

    # The same oracle calls on disjoint slices from a pool of threads (the C functions run
    # without the interpreter lock): what all the host's cores reach together.
    from concurrent.futures import ThreadPoolExecutor
    threads = max(1, min(16, os.cpu_count() or 1))
    bounds = [ns * k // threads for k in range(threads + 1)]

    def work(k, t):
        a, b = bounds[k], bounds[k + 1]
        _, bad = oracle.grad_sqnorm(g[a:b])
        oracle.adam_step(p[a:b], m[a:b], v[a:b], g[a:b], step=t, bf16_out=send[a:b], skip=bool(bad), **synth.HP)

    par_passes = 4
    with ThreadPoolExecutor(threads) as pool:
        list(pool.map(lambda k: work(k, passes + 1), range(threads)))       # warm the pool
        t1 = time.perf_counter()
        for t in range(par_passes):
            list(pool.map(lambda k: work(k, passes + 2 + t), range(threads)))
        dt_par = (time.perf_counter() - t1) / par_passes
    return {"value": round(ns / dt / 1e9, 4), "unit": "Gparams/s", "cores": 1, "kind": "oracle",
            "all_cores": {"value": round(ns / dt_par / 1e9, 4), "unit": "Gparams/s", "cores": threads,
                          "sample": f"{par_passes} passes, the same calls on {threads} disjoint slices in {threads} threads"},
            "unshard": {"value": round(WORLD * ns / dt_unshard / 1e9, 4), "unit": "G bf16 elements/s", "cores": 1,
                        "sample": "4 passes over the 8 x 2^26-element gathered buffer, 4 ragged tensors"},
            "sample": (f"{passes} passes over a 2^26-element slice of the shard (grad-norm + AdamW + bf16 "
                       f"copy, the calls `value` times on the GPU); {round(dt, 2)} s per pass; host has "
                       f"{os.cpu_count()} logical CPUs, the oracle is sequential"),
            "seconds": round(dt * passes + dt_unshard * 4, 2)}


if __name__ == "__main__":
    main()
