#!/usr/bin/env python3
"""Benchmark of one rank's sharded mixed-precision optimizer step on one MI355X.

A *step* is one pass of the whole hot path over one batch of synthetic input:

    zc_grad_sqnorm   (overflow flag + squared norm of the bf16 gradient shard)
    zc_adam_step     (fused AdamW over the fp32 shard, bf16 copy written straight
                      into this rank's slot of the gathered buffer, skipped on overflow)
    zc_unshard       (gathered flat bf16 buffer of 8 rank shards -> per-layer tensors)

on a one-of-8 shard of a Llama-3-8B-shaped model (1,003,782,656 fp32 elements,
291 tensors, boundaries not aligned to the shards).  Everything is resident in
HBM when the timed region starts.  Prints ONE JSON line.

Extra legs outside the timed region: the offloaded step (pinned host p/m/v
streamed through a 3-slot ring) and the CPU oracle on a bounded sample.
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


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b",
                    choices=["llama3_8b", "llama3_70b", "mixtral_8x7b", "tiny"])
    ap.add_argument("--no-unshard", action="store_true",
                    help="leave the unshard copy out (needed for 70B/Mixtral to fit with the step)")
    ap.add_argument("--only-unshard", action="store_true",
                    help="time the unshard copy alone (Mixtral: the step's state and the two "
                         "93 GB buffers do not fit in HBM together)")
    ap.add_argument("--offload-elems", type=int, default=1 << 28,
                    help="elements streamed in the offload leg (0 = skip the leg)")
    ap.add_argument("--offload-frac", type=float, default=0.0, help="resident fraction f")
    ap.add_argument("--offload-max-pinned-gib", type=float, default=60.0,
                    help="largest total of pinned host memory to ask for; the partition is shrunk "
                         "(same resident fraction) when its streamed part would need more")
    ap.add_argument("--offload-chunk-mib", type=int, default=64)
    ap.add_argument("--offload-buffers", type=int, default=3)
    ap.add_argument("--offload-transports", default="1,2,0",
                    help="which transports the offload leg times: 1 zero-copy, 2 staged reads + direct "
                         "writes, 0 staged ring")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true",
                    help="skip the short legs for gradient accumulation and the per-tensor layout")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain copy of known size (one unshard segment of 2^30 bf16 "
                         "elements, 2 GiB read + 2 GiB written, 5 launches): the reference for "
                         "scaling the FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--tune", action="append", default=[], metavar="KEY=VALUE",
                    help="tuning knob, e.g. adam.rows=4 (repeatable)")
    return ap.parse_args()


def gb(x):
    return x / 1e9


def bind_to_gpu_numa_node(torch):
    """Run this process on the CPUs of the NUMA node the GPU hangs off, so that pinned
    host memory allocated afterwards is local to the GPU's PCIe root (device writes to
    memory on another socket cross the inter-socket link and run several times slower).
    Returns a small dict describing what was done."""
    info = {"gpu_numa_node": None, "bound": False}
    try:
        props = torch.cuda.get_device_properties(0)
        bus = getattr(props, "pci_bus_id", None)
        dom = getattr(props, "pci_domain_id", 0)
        dev_id = getattr(props, "pci_device_id", 0)
        if bus is None:
            return info
        path = f"/sys/bus/pci/devices/{dom:04x}:{bus:02x}:{dev_id:02x}.0/numa_node"
        node = int(open(path).read().strip())
        info["gpu_numa_node"] = node
        if node < 0:
            return info
        cpus = set()
        for part in open(f"/sys/devices/system/node/node{node}/cpulist").read().strip().split(","):
            if "-" in part:
                a, b = part.split("-")
                cpus.update(range(int(a), int(b) + 1))
            elif part:
                cpus.add(int(part))
        allowed = os.sched_getaffinity(0)
        use = cpus & allowed
        info["allowed_cpus"] = len(allowed)
        info["node_cpus_allowed"] = len(use)
        if use:
            os.sched_setaffinity(0, use)
            info["bound"] = True
    except Exception as e:  # best effort: the numbers are still valid, only maybe slower
        info["error"] = repr(e)
    return info


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

    # ---- workload ------------------------------------------------------------------
    if args.workload == "tiny":
        tensors = synth.TINY_TENSORS
    else:
        tensors = synth.tensor_list(synth.SHAPES[args.workload])
    numels = [int(__import__("numpy").prod(d)) for _, d in tensors]
    offs, shard, total = zc.flat_layout(numels, WORLD, 1)
    n = shard
    do_unshard = not args.no_unshard
    hp_kw = dict(synth.HP)

    do_step = not args.only_unshard
    if do_step:
        p = torch.empty(n, dtype=torch.float32, device=dev)
        m = torch.zeros(n, dtype=torch.float32, device=dev)
        v = torch.zeros(n, dtype=torch.float32, device=dev)
        g = torch.empty(n, dtype=torch.bfloat16, device=dev)
        synth.device_normal_(p, synth.P_STD, seed=2)
        synth.device_normal_(g, synth.G_STD, seed=2001)
    norm = torch.zeros(1, dtype=torch.float32, device=dev)
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    if do_unshard:
        gathered = torch.empty(WORLD * shard, dtype=torch.int16, device=dev)
        synth.device_index_hash16_(gathered)          # the other 7 ranks' bytes
        send = gathered[:n]                            # this rank's slot (rank 0)
        outs = [torch.empty(d, dtype=torch.bfloat16, device=dev) for _, d in tensors]
        plan = zc.unshard_plan_create([(o, t, k) for o, t, k in zip(offs, outs, numels)],
                                      WORLD * shard)
    else:
        send = torch.empty(n, dtype=torch.int16, device=dev)
    torch.cuda.synchronize()

    step_no = [0]

    def one_step(ev=None):
        step_no[0] += 1
        hp = zc.hparams(step=step_no[0], **hp_kw)
        if ev: ev[0].record()
        if do_step:
            zc.grad_sqnorm(g, zc.BF16, n, norm, flag)
        if ev: ev[1].record()
        if do_step:
            zc.adam_step(p, m, v, g, zc.BF16, n, hp, bf16_out=send, skip_flag=flag)
        if ev: ev[2].record()
        if do_unshard:
            zc.unshard(plan, gathered)
        if ev: ev[3].record()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps

    def times(i):
        return sorted(e[i].elapsed_time(e[i + 1]) for e in events)

    def avg(i):
        return sum(times(i)) / len(events)

    t_norm, t_adam, t_unshard = avg(0), avg(1), avg(2)
    spread = {"sqnorm": times(0), "adam": times(1), "unshard": times(2)}
    assert flag.item() == 0, "synthetic gradients must be finite"

    kernels = {}
    if do_step:
        kernels["sqnorm"] = dict(name="zc::sqnorm_bf16_kernel", ms=t_norm, bytes=2 * n, units=n,
                                 bytes_per_unit=2)
        kernels["adam"] = dict(name="zc::adam_vec_kernel", ms=t_adam, bytes=28 * n, units=n,
                               bytes_per_unit=28)
    if do_unshard:
        kernels["unshard"] = dict(name="zc::unshard_kernel", ms=t_unshard, bytes=4 * total,
                                  units=total, bytes_per_unit=4)
    for kd in kernels.values():
        kd["GBps"] = gb(kd["bytes"]) / (kd["ms"] * 1e-3)
        kd["frac"] = kd["GBps"] / HBM_PEAK_GBS
    dominant = max(kernels, key=lambda k: kernels[k]["ms"])

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "pmc_traffic.json")
    if os.path.exists(tpath):
        try:
            tj = json.load(open(tpath))
            rec = tj.get(args.workload, {}).get(dominant)
            if rec:
                traffic = rec["fetch_bytes"] + rec["write_bytes"]
        except Exception:
            traffic = None

    roofline = dict(bound="hbm", kernel=kernels[dominant]["name"],
                    achieved=round(kernels[dominant]["GBps"], 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(kernels[dominant]["frac"], 4), traffic=traffic,
                    algorithmic_bytes_per_launch=kernels[dominant]["bytes"],
                    avg_launch_ms=round(kernels[dominant]["ms"], 4))

    result = {
        "metric": "optimizer-step Gparams/s per shard",
        "value": round(n / (ms_per_step * 1e-3) / 1e9, 3),
        "unit": "Gparams/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": {0: "f32", 1: "f32+f64", 2: "f64"}[zc.tune_get("adam.arith")], "data": "synthetic",
        "config": {
            "workload": (f"{args.workload} one-of-{WORLD} shard: "
                         + ("grad-norm + fused AdamW with bf16 copy" if do_step else "")
                         + (" + " if do_step and do_unshard else "")
                         + ("unshard of the 8-shard gathered buffer" if do_unshard else "")),
            "shard_elements": n, "model_elements": total, "tensors": len(numels),
            "grads": "bf16", "state": "fp32 p/m/v resident in HBM",
            "tuning": {k: zc.tune_get(k) for k in ("adam.arith", "adam.block", "adam.rows",
                                                  "adam.waves_per_cu", "adam.nontemporal",
                                                  "copy.waves_per_cu", "copy.nontemporal")},
        },
        "roofline": roofline,
        "kernels": {k: dict(ms=round(d["ms"], 4), ms_median=round(spread[k][len(spread[k]) // 2], 4),
                            ms_min=round(spread[k][0], 4),
                            GBps=round(d["GBps"], 1), frac=round(d["frac"], 4),
                            algorithmic_bytes=d["bytes"],
                            rate_G_per_s=round(d["units"] / (d["ms"] * 1e-3) / 1e9, 2))
                    for k, d in kernels.items()},
    }
    if do_step:
        result["adam_step_gparams_per_s"] = round(n / (t_adam * 1e-3) / 1e9, 2)

    # ---- the update kernel's other variants on the same shard (not part of `value`) -----
    if do_step and not args.no_next_rows:
        def variant(fn):
            return time_launches(torch, fn, reps=10)

        def hp_next():
            step_no[0] += 1
            return zc.hparams(step=step_no[0], **hp_kw)

        scratch = send
        g32 = torch.empty(n, dtype=torch.float32, device=dev)
        synth.device_normal_(g32, synth.G_STD, seed=2999)
        rows = {
            "bf16_grads_no_copy": (26, lambda: zc.adam_step(p, m, v, g, zc.BF16, n, hp_next())),
            "fp32_grads_fused_copy": (30, lambda: zc.adam_step(p, m, v, g32, zc.F32, n, hp_next(), bf16_out=scratch)),
            "fp32_grads_no_copy": (28, lambda: zc.adam_step(p, m, v, g32, zc.F32, n, hp_next())),
            "unfused_step_then_cast": (32, lambda: (zc.adam_step(p, m, v, g, zc.BF16, n, hp_next()),
                                                    zc.cast_bf16(p, scratch, n))),
            "standalone_cast": (6, lambda: zc.cast_bf16(p, scratch, n)),
        }
        result["step_variants"] = {}
        for name, (bpe, fn) in rows.items():
            ms = variant(fn)
            result["step_variants"][name] = {"bytes_per_element": bpe, "ms": round(ms, 4),
                                             "GBps": round(gb(bpe * n) / (ms * 1e-3), 1),
                                             "frac": round(gb(bpe * n) / (ms * 1e-3) / HBM_PEAK_GBS, 4),
                                             "gparams_per_s": round(n / (ms * 1e-3) / 1e9, 2)}
        del g32

    # ---- free the resident workload before the extra legs --------------------------
    if do_unshard:
        plan.destroy()
        del outs, gathered
    if do_step:
        del p, m, v, g
    del send
    torch.cuda.empty_cache()

    if not args.no_next_rows:
        result["next_rows"] = next_rows_leg(torch, synth, zc, dev)
        result["next_rows"]["adaptive_offload_plan"] = adaptive_plan_leg(torch, zc, dev)
    if args.offload_elems > 0:
        legs = {}
        keep = zc.tune_get("offload.zero_copy")
        names = {1: "zero_copy", 2: "staged_reads_direct_writes", 0: "staged_ring"}
        for mode in (int(x) for x in args.offload_transports.split(",")):
            name = names[mode]
            zc.tune_set("offload.zero_copy", mode)
            legs[name] = offload_leg(torch, synth, zc, dev, args, probe=(mode == 0))
        zc.tune_set("offload.zero_copy", keep)
        result["offload"] = legs
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline_leg(synth)
    print(json.dumps(result))


def time_launches(torch, fn, reps=10):
    fn()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in ev) / reps


def next_rows_leg(torch, synth, zc, dev):
    """Rows built after the main path: fp32 gradient accumulation (10 B/element) and the
    unshard copy in the per-tensor even-partition layout (8 segments per tensor)."""
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
    segs, send = zc.per_tensor_layout(numels, WORLD, 8)
    gathered = torch.empty(WORLD * send, dtype=torch.int16, device=dev)
    synth.device_index_hash16_(gathered)
    outs = [torch.empty(d, dtype=torch.bfloat16, device=dev) for _, d in tensors]
    table = [(src, outs[t].data_ptr() + 2 * dst if k else None, k) for t, src, dst, k in segs]
    plan = zc.unshard_plan_create(table, WORLD * send)
    t_un = time_launches(torch, lambda: zc.unshard(plan, gathered))
    plan.destroy()
    total = sum(numels)
    del outs, gathered
    torch.cuda.empty_cache()
    return {
        "grad_accumulate": {"elements": n, "ms": round(t_acc, 4), "bytes_per_element": 10,
                            "GBps": round(gb(10 * n) / (t_acc * 1e-3), 1),
                            "frac": round(gb(10 * n) / (t_acc * 1e-3) / HBM_PEAK_GBS, 4)},
        "unshard_per_tensor": {"elements": total, "segments": sum(1 for s in segs if s[3]),
                               "ms": round(t_un, 4), "bytes_per_element": 4,
                               "GBps": round(gb(4 * total) / (t_un * 1e-3), 1),
                               "frac": round(gb(4 * total) / (t_un * 1e-3) / HBM_PEAK_GBS, 4)},
    }


def adaptive_plan_leg(torch, zc, dev):
    """The paper's adaptive offloading (Algorithm 2 + backward reload) planned on a synthetic
    memory profile (rising through the forward pass, falling through the backward pass) and
    replayed with stand-in compute kernels: 32 optimizer-state fragments of 64 MiB, 24 of which
    must leave, 16 + 16 operators of 8 ms.  Compared with offloading everything synchronously."""
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
            "sync_over_adaptive": round(t_sync / t_adaptive, 3)}


def offload_leg(torch, synth, zc, dev, args, probe=True):
    """Offloaded step: p/m/v of the streamed part in pinned host DRAM, 3-slot ring."""
    numa = bind_to_gpu_numa_node(torch)
    n_asked = n = int(args.offload_elems)
    cap_elems = int(args.offload_max_pinned_gib * (1 << 30)) // 12
    if (1.0 - args.offload_frac) * n > cap_elems:
        n = int(cap_elems / (1.0 - args.offload_frac)) // 1024 * 1024
    n_res = int(args.offload_frac * n) // 1024 * 1024
    n_str = n - n_res
    chunk = args.offload_chunk_mib << 20
    # exact-size pinned arrays (torch's pinned allocator rounds up to a power of two)
    bufs = [zc.host_alloc(4 * max(n_str, 1)) for _ in range(3)]
    hp_, hm_, hv_ = (torch.from_numpy(b.numpy("float32")) for b in bufs)
    piece = 1 << 28
    tmp = torch.empty(min(piece, max(n_str, 1)), dtype=torch.float32, device=dev)
    for s0 in range(0, n_str, piece):                 # p ~ N(0, 0.02); m = v = 0
        e0 = min(n_str, s0 + piece)
        synth.device_normal_(tmp[:e0 - s0], synth.P_STD, seed=3 + s0 // piece)
        hp_[s0:e0].copy_(tmp[:e0 - s0])
    hm_.zero_()
    hv_.zero_()
    del tmp
    dp, dm, dv = (torch.zeros(max(n_res, 1), dtype=torch.float32, device=dev) for _ in range(3))
    g = torch.empty(n, dtype=torch.bfloat16, device=dev)
    synth.device_normal_(g, synth.G_STD, seed=2002)
    send = torch.empty(n, dtype=torch.int16, device=dev)
    ctx = zc.offload_create(chunk, args.offload_buffers)
    torch.cuda.synchronize()

    def run(step):
        ctx.adam_step(dp if n_res else None, dm if n_res else None, dv if n_res else None, n_res,
                      hp_, hm_, hv_, n_str, g, zc.BF16, zc.hparams(step=step, **synth.HP),
                      bf16_out_dev=send)

    run(1)
    torch.cuda.synchronize()
    reps = 3
    t0 = time.perf_counter()
    for k in range(reps):
        run(2 + k)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / reps

    extra = {}
    if probe and n_str > 0:
        # plain pinned-copy ceilings with the same chunking: one direction at a time and both
        nbytes = 4 * n_str
        t_h2d = min(ctx.probe_link(hp_, hv_, nbytes, 0) for _ in range(3)) * 1e-3
        t_d2h = min(ctx.probe_link(hp_, hv_, nbytes, 1) for _ in range(3)) * 1e-3
        t_both = min(ctx.probe_link(hp_, hv_, nbytes, 2) for _ in range(3)) * 1e-3
        extra["memcpy_ceiling_GBps"] = {"h2d": round(gb(nbytes) / t_h2d, 2),
                                        "d2h": round(gb(nbytes) / t_d2h, 2),
                                        "both_each": round(gb(nbytes) / t_both, 2)}
    ctx.destroy()
    del hp_, hm_, hv_
    for b in bufs:
        b.free()
    one_way = 12 * n_str
    return {
        "elements": n, "elements_asked": n_asked, "streamed_elements": n_str,
        "pinned_GB": round(12 * n_str / 1e9, 2),
        "resident_fraction": n_res / n, "chunk_MiB": args.offload_chunk_mib,
        "buffers": args.offload_buffers, "ms_per_step": round(dt * 1e3, 3),
        "gparams_per_s": round(n / dt / 1e9, 3),
        "link_GBps_each_direction": round(gb(one_way) / dt, 2),
        "link_peak_GBps": PCIE_PEAK_GBS, "frac_of_link_peak": round(gb(one_way) / dt / PCIE_PEAK_GBS, 4),
        "zero_copy": zc.tune_get("offload.zero_copy"),
        "host_numa": numa, **extra,
    }


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
    # tensor boundaries: the 8B model's first tensors scaled into the sample
    cuts = [0, ns // 3 + 5, ns * 2 + 17, ns * 5 - 3, WORLD * ns]
    offs = cuts[:-1]
    nums = [b - a for a, b in zip(cuts[:-1], cuts[1:])]
    t0 = time.perf_counter()
    for t in range(1, passes + 1):
        _, bad = oracle.grad_sqnorm(g)
        oracle.adam_step(p, m, v, g, step=t, bf16_out=send, skip=bool(bad), **synth.HP)
        oracle.unshard(gathered, offs, nums)
    dt = (time.perf_counter() - t0) / passes

    # The same oracle calls on disjoint slices from a pool of threads (the C functions run
    # without the interpreter lock): what all the host's cores reach together.
    from concurrent.futures import ThreadPoolExecutor
    threads = max(1, min(16, os.cpu_count() or 1))
    bounds = [ns * k // threads for k in range(threads + 1)]
    gb_ = [WORLD * ns * k // threads for k in range(threads + 1)]

    def work(k, t):
        a, b = bounds[k], bounds[k + 1]
        _, bad = oracle.grad_sqnorm(g[a:b])
        oracle.adam_step(p[a:b], m[a:b], v[a:b], g[a:b], step=t, bf16_out=send[a:b], skip=bool(bad), **synth.HP)
        oracle.unshard(gathered[gb_[k]:gb_[k + 1]], [0], [gb_[k + 1] - gb_[k]])

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
            "sample": (f"{passes} passes over a 2^26-element shard slice (grad-norm + AdamW + bf16 "
                       f"copy) and its 8 x 2^26-element gathered buffer (unshard); "
                       f"{round(dt, 2)} s per pass; host has {os.cpu_count()} logical CPUs, "
                       "the oracle is sequential"),
            "seconds": round(dt * passes, 2)}


if __name__ == "__main__":
    main()
