"""Launch-shape and placement sweeps for libzc on the GPU at hand.

    python -m paper_2504_09983_amd.tune adam      [--workload llama3_8b|llama3_70b|mixtral_8x7b] [--grid coarse|fine|nt]
    python -m paper_2504_09983_amd.tune packed    [--workload ...]  the same update over the packed state array, by wave cap
    python -m paper_2504_09983_amd.tune layout    [--elements N] [--grads bf16|fp32]  stand-alone probe: three state arrays
                                                  against one packed array, by granule size
    python -m paper_2504_09983_amd.tune streams   norm, cast, accumulate and unshard: resident-wave caps, grid, unroll
    python -m paper_2504_09983_amd.tune placement how far apart p, m, v, g and the bf16 copy sit in memory
    python -m paper_2504_09983_amd.tune link      host link: one direction, both, 2:1 mix, zero-copy launch shapes,
                                                  flavours of pinned memory

Every figure is an average of HIP-event times on the launch stream over N(0, sigma) data
(zero-filled buffers run about 3 % faster and overstate what a training run sees).  The
defaults compiled into the library come from these sweeps on an MI355X; the tool is here
so that they can be checked, or redone on another machine.  Measurement only: nothing in
the library reads what this prints.
"""
from __future__ import annotations

import argparse
import ctypes
import sys
import time

HBM_PEAK_GBS = 8000.0
GIB = 1 << 30
MIB = 1 << 20


def _setup():
    import torch

    from . import synth, zc
    if not torch.cuda.is_available():
        sys.exit("tune: no GPU visible")
    torch.cuda.set_device(0)
    return torch, synth, zc


def _timeit(torch, fn, reps):
    fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return sum(a.elapsed_time(b) for a, b in evs) / reps


def _frac(nbytes, ms):
    return nbytes / ms / 1e6 / HBM_PEAK_GBS


def sweep_adam(args):
    """The update kernel's four gradient/copy variants over threads per workgroup, rows per
    lane, resident-wave cap and non-temporal mode."""
    torch, synth, zc = _setup()
    dev = "cuda:0"
    _, n, _ = zc.flat_layout(synth.tensor_numels(synth.SHAPES[args.workload]), 8, 1)
    reps = args.reps or (10 if n < (1 << 31) else 4)
    p = torch.empty(n, dtype=torch.float32, device=dev)
    synth.device_normal_(p, synth.P_STD, seed=2)
    m = torch.zeros(n, dtype=torch.float32, device=dev)
    v = torch.zeros(n, dtype=torch.float32, device=dev)
    g = torch.empty(n, dtype=torch.bfloat16, device=dev)
    synth.device_normal_(g, synth.G_STD, seed=2001)
    g32 = torch.empty(n, dtype=torch.float32, device=dev)
    synth.device_normal_(g32, synth.G_STD, seed=2002)
    out = torch.empty(n, dtype=torch.int16, device=dev)
    hp = zc.hparams(step=3, **synth.HP)
    variants = {
        "bf16 g + copy (28 B)": (28, lambda: zc.adam_step(p, m, v, g, zc.BF16, n, hp, bf16_out=out)),
        "bf16 g (26 B)": (26, lambda: zc.adam_step(p, m, v, g, zc.BF16, n, hp)),
        "fp32 g + copy (30 B)": (30, lambda: zc.adam_step(p, m, v, g32, zc.F32, n, hp, bf16_out=out)),
        "fp32 g (28 B)": (28, lambda: zc.adam_step(p, m, v, g32, zc.F32, n, hp)),
    }
    for _, fn in variants.values():
        fn()
    torch.cuda.synchronize()
    nt0 = zc.tune_get("adam.nontemporal")          # coarse and fine grids keep the library's access mode
    if args.grid == "coarse":
        grid = [(b, r, w, nt0) for b in (64, 128, 256) for r in (1, 2, 4) for w in (4, 6, 8, 9, 10, 11, 12, 14, 16, 20)]
    elif args.grid == "fine":
        grid = [(64, r, w, nt0) for r in (1, 2) for w in range(10, 17)] + [(128, 2, w, nt0) for w in (12, 14, 16)]
    else:
        grid = [(b, r, w, nt) for (b, r) in ((64, 1), (64, 2), (128, 2)) for w in (10, 12, 14, 16) for nt in (0, 1, 2, 3, 4)]
    print(f"# adam {args.workload} n={n} reps={reps}; columns: fraction of 8 TB/s per variant", flush=True)
    print("# block rows waves nt | " + " | ".join(variants), flush=True)
    seen = set()
    for b, r, w, nt in grid:
        eff = max(1, w // (b // 64)) * (b // 64)         # the cap works in whole workgroups
        if (b, r, eff, nt) in seen:
            continue
        seen.add((b, r, eff, nt))
        for k, val in (("adam.block", b), ("adam.rows", r), ("adam.waves_per_cu", w), ("adam.nontemporal", nt)):
            zc.tune_set(k, val)
        cells = [f"{_frac(bpe * n, _timeit(torch, fn, reps)):.3f}" for bpe, fn in variants.values()]
        print(f"{b:5d} {r:4d} {w:5d} {nt:2d} | " + " | ".join(cells), flush=True)


def sweep_packed(args):
    """The update over the packed state array (zc_adam_step_packed) next to the three-array
    update on the same GPU in the same process, by resident-wave cap."""
    torch, synth, zc = _setup()
    dev = "cuda:0"
    _, n, _ = zc.flat_layout(synth.tensor_numels(synth.SHAPES[args.workload]), 8, 1)
    reps = args.reps or (10 if n < (1 << 31) else 4)
    g = torch.empty(n, dtype=torch.bfloat16, device=dev)
    synth.device_normal_(g, synth.G_STD, seed=2001)
    g32 = torch.empty(n, dtype=torch.float32, device=dev)
    synth.device_normal_(g32, synth.G_STD, seed=2002)
    out = torch.empty(n, dtype=torch.int16, device=dev)
    hp = zc.hparams(step=3, **synth.HP)
    print(f"# {args.workload} n={n} reps={reps}; columns: fraction of 8 TB/s per variant", flush=True)
    print("# layout waves | bf16 g + copy (28 B) | bf16 g (26 B) | fp32 g + copy (30 B) | fp32 g (28 B)", flush=True)
    for layout in ("packed", "arrays"):
        if layout == "packed":
            state = torch.empty(zc.packed_state_numel(n), dtype=torch.float32, device=dev)
            cube = state.view(-1, 3, zc.PACKED_GRANULE)
            for k in range(0, cube.shape[0], 1 << 12):
                rows = min(1 << 12, cube.shape[0] - k)
                cube[k:k + rows, 0] = torch.randn(rows, zc.PACKED_GRANULE, device=dev) * synth.P_STD
            cube[:, 1:].zero_()

            def upd(grad, dt, **kw):
                zc.adam_step_packed(state, grad, dt, n, hp, **kw)
        else:
            p = torch.empty(n, dtype=torch.float32, device=dev)
            synth.device_normal_(p, synth.P_STD, seed=2)
            m = torch.zeros(n, dtype=torch.float32, device=dev)
            v = torch.zeros(n, dtype=torch.float32, device=dev)

            def upd(grad, dt, **kw):
                zc.adam_step(p, m, v, grad, dt, n, hp, **kw)
        variants = [(28, lambda: upd(g, zc.BF16, bf16_out=out)), (26, lambda: upd(g, zc.BF16)),
                    (30, lambda: upd(g32, zc.F32, bf16_out=out)), (28, lambda: upd(g32, zc.F32))]
        for _, fn in variants:
            fn()
        torch.cuda.synchronize()
        for w in (-1, 9, 10, 11, 12, 13, 14, 15, 16):
            zc.tune_set("adam.waves_per_cu", w)
            cells = [f"{_frac(bpe * n, _timeit(torch, fn, reps)):.3f}" for bpe, fn in variants]
            print(f"{layout:7s} {'default' if w < 0 else w:>7} | " + " | ".join(cells), flush=True)
        zc.tune_set("adam.waves_per_cu", -1)
        if layout == "packed":
            del state, cube
        else:
            del p, m, v
        torch.cuda.empty_cache()


def sweep_layout(args):
    """Runs the stand-alone state_layout_probe (built next to libzc.so): the update's memory
    pattern over three arrays, over packed arrays of different granules, and with an fp32
    gradient as a fourth slot.  The probe is a child process; this one never touches the GPU."""
    import os
    import subprocess
    probe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "state_layout_probe")
    if not os.path.exists(probe):
        sys.exit(f"tune: {probe} is missing: run `python -m paper_2504_09983_amd.build`")
    sys.exit(subprocess.call([probe, str(args.elements), args.grads]))


def sweep_streams(args):
    """The other streaming kernels: grid and unroll of the norm, resident-wave caps of the
    cast, the accumulation and the unshard copy."""
    torch, synth, zc = _setup()
    dev = "cuda:0"
    norm = torch.zeros(1, dtype=torch.float32, device=dev)
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    for which in ("llama3_8b", "llama3_70b"):
        _, n, _ = zc.flat_layout(synth.tensor_numels(synth.SHAPES[which]), 8, 1)
        reps = 20 if n < (1 << 31) else 5
        p = torch.empty(n, dtype=torch.float32, device=dev)
        synth.device_normal_(p, synth.P_STD, seed=2)
        g = torch.empty(n, dtype=torch.bfloat16, device=dev)
        synth.device_normal_(g, synth.G_STD, seed=2001)
        out = torch.empty(n, dtype=torch.int16, device=dev)
        print(f"# {which} shard, n={n}", flush=True)
        keep = {k: zc.tune_get(k) for k in ("reduce.unroll", "reduce.blocks_per_cu", "cast.waves_per_cu",
                                            "accum.waves_per_cu")}
        for dt, src, bpe, name in ((zc.BF16, g, 2, "bf16"), (zc.F32, p, 4, "fp32")):
            for u in (4, 8):
                for b in (1, 2, 3, 4, 8):
                    zc.tune_set("reduce.unroll", u)
                    zc.tune_set("reduce.blocks_per_cu", b)
                    ms = _timeit(torch, lambda: zc.grad_sqnorm(src, dt, n, norm, flag), reps)
                    print(f"sqnorm {name} unroll={u} blocks/cu={b:2d}: {ms:7.3f} ms {_frac(bpe * n, ms):.3f}", flush=True)
        zc.tune_set("reduce.unroll", keep["reduce.unroll"])
        zc.tune_set("reduce.blocks_per_cu", keep["reduce.blocks_per_cu"])
        keep_nt = zc.tune_get("copy.nontemporal")
        for nt in (2, 1):
            zc.tune_set("copy.nontemporal", nt)
            for w in (0, 8, 12, 16, 20, 24, 32):
                zc.tune_set("cast.waves_per_cu", w)
                ms = _timeit(torch, lambda: zc.cast_bf16(p, out, n), reps)
                print(f"cast nt={nt} waves={w:2d}: {ms:7.3f} ms {_frac(6 * n, ms):.3f}", flush=True)
            zc.tune_set("cast.waves_per_cu", keep["cast.waves_per_cu"])
            for w in (0, 8, 12, 16, 20, 24, 32):
                zc.tune_set("accum.waves_per_cu", w)
                ms = _timeit(torch, lambda: zc.grad_accumulate(p, g, zc.BF16, n, 0.25), reps)
                print(f"accumulate nt={nt} waves={w:2d}: {ms:7.3f} ms {_frac(10 * n, ms):.3f}", flush=True)
            zc.tune_set("accum.waves_per_cu", keep["accum.waves_per_cu"])
        zc.tune_set("copy.nontemporal", keep_nt)
        del p, g, out
        torch.cuda.empty_cache()
    for which in ("llama3_8b", "mixtral_8x7b"):
        tensors = synth.tensor_list(synth.SHAPES[which])
        numels = synth.tensor_numels(synth.SHAPES[which])
        offs, shard, total = zc.flat_layout(numels, 8, 1)
        reps = 20 if total < (1 << 34) else 5
        gathered = torch.empty(8 * shard, dtype=torch.int16, device=dev)
        synth.device_index_hash16_(gathered)
        outs = [torch.empty(d, dtype=torch.bfloat16, device=dev) for _, d in tensors]
        plan = zc.unshard_plan_create([(o, t, k) for o, t, k in zip(offs, outs, numels)], 8 * shard)
        print(f"# unshard {which}, {total} elements, {len(numels)} tensors", flush=True)
        keep = (zc.tune_get("copy.waves_per_cu"), zc.tune_get("copy.nontemporal"))
        for nt in (2, 1, 0):
            for w in (0, 8, 10, 12, 14, 16, 20, 24, 32):
                zc.tune_set("copy.waves_per_cu", w)
                zc.tune_set("copy.nontemporal", nt)
                ms = _timeit(torch, lambda: zc.unshard(plan, gathered), reps)
                print(f"unshard nt={nt} waves={w:2d}: {ms:7.3f} ms {_frac(4 * total, ms):.3f}", flush=True)
        zc.tune_set("copy.waves_per_cu", keep[0])
        zc.tune_set("copy.nontemporal", keep[1])
        plan.destroy()
        del outs, gathered
        torch.cuda.empty_cache()


def sweep_placement(args):
    """The update over the Llama-3-8B shard (five arrays of 2-4 GB) with the arrays carved out
    of one arena at a given distance from each other, for a launch shape that keeps few
    (default) and one that keeps many requests in flight."""
    torch, synth, zc = _setup()
    dev = "cuda:0"
    n = 1_003_782_656
    arena = torch.empty(200 * GIB, dtype=torch.uint8, device=dev)
    base = arena.data_ptr()
    for o in range(0, arena.numel(), 4 * GIB):
        k = min(4 * GIB, arena.numel() - o)
        synth.device_normal_(arena[o:o + k].view(torch.float32), synth.P_STD, seed=7 + o // GIB)
    torch.cuda.synchronize()
    hp = zc.hparams(step=3, **synth.HP)
    shapes = [(64, 1, -1), (64, 2, 16)]

    def run(offs):
        ptr = [base + int(o) for o in offs]
        cells = []
        for b, r, w in shapes:
            zc.tune_set("adam.block", b)
            zc.tune_set("adam.rows", r)
            zc.tune_set("adam.waves_per_cu", w)
            ms = _timeit(torch, lambda: zc.adam_step(ptr[0], ptr[1], ptr[2], ptr[3], zc.BF16, n, hp, bf16_out=ptr[4]), 8)
            cells.append(f"{_frac(28 * n, ms):.3f}")
        return " ".join(cells)

    print(f"# arena at {base:#x}; columns: block 64 / 1 row / default cap, block 64 / 2 rows / 16 waves", flush=True)
    s0 = (4 * n + 2 * MIB - 1) // (2 * MIB) * (2 * MIB)
    print(f"back to back (2 MiB-rounded sizes): {run([0, s0, 2 * s0, 3 * s0, 3 * s0 + s0 // 2])}", flush=True)
    for s in (4, 6, 8, 12, 15, 16, 17, 20, 24, 28, 32, 34, 36, 40, 44, 48):
        offs = [k * s * GIB for k in range(5)]
        if offs[4] + 2 * n <= arena.numel():
            print(f"all five {s:2d} GiB apart: {run(offs)}", flush=True)
    for s in (4, 8, 16, 32, 36, 48, 64):
        print(f"p, m, v {s:2d} GiB apart, g and copy far away: {run([0, s * GIB, 2 * s * GIB, 180 * GIB, 190 * GIB])}", flush=True)
    far = [0, 40 * GIB, 80 * GIB, 120 * GIB, 160 * GIB]
    print(f"all far apart (40 GiB): {run(far)}", flush=True)
    for name, offs in (("p, m next to each other", [0, 4 * GIB, 80 * GIB, 120 * GIB, 160 * GIB]),
                       ("m, v next to each other", [0, 40 * GIB, 44 * GIB, 120 * GIB, 160 * GIB]),
                       ("p, m, v next to each other", [0, 4 * GIB, 8 * GIB, 120 * GIB, 160 * GIB]),
                       ("g and copy next to p", [0, 40 * GIB, 80 * GIB, 4 * GIB, 7 * GIB])):
        print(f"{name}: {run(offs)}", flush=True)


def _hip():
    for line in open("/proc/self/maps"):
        if "libamdhip64" in line:
            return ctypes.CDLL(line.split()[-1])
    sys.exit("tune: the HIP runtime is not mapped")


def sweep_link(args):
    """Host link: plain pinned copies, the library's kernels reading or writing pinned host
    memory one direction at a time, a 2:1 mix, and the zero-copy offloaded step over launch
    shapes, wave caps and flavours of pinned memory."""
    torch, synth, zc = _setup()
    import numpy as np
    dev = "cuda:0"
    n = int(args.elements)
    ctx = zc.offload_create(64 << 20, 3)
    bufs = [zc.host_alloc(4 * n) for _ in range(3)]
    hviews = [torch.from_numpy(b.numpy("float32")) for b in bufs]
    tmp = torch.empty(n, dtype=torch.float32, device=dev)
    synth.device_normal_(tmp, synth.P_STD, seed=3)
    hviews[0].copy_(tmp)
    hviews[1].zero_()
    hviews[2].zero_()
    nbytes = 4 * n
    for mode, name in ((0, "host to device"), (1, "device to host"), (2, "both at once, each way")):
        t = min(ctx.probe_link(bufs[0], bufs[2], nbytes, mode) for _ in range(3)) * 1e-3
        print(f"hipMemcpyAsync in 64 MiB pieces, {name}: {nbytes / t / 1e9:.2f} GB/s", flush=True)
    hviews[2].zero_()
    norm = torch.zeros(1, dtype=torch.float32, device=dev)
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    out_dev = torch.empty(n, dtype=torch.int16, device=dev)

    def wall(fn, reps=3):
        fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps

    t = wall(lambda: zc.grad_sqnorm(bufs[0].ptr, zc.F32, n, norm, flag))
    print(f"kernel reads pinned host memory (zc_grad_sqnorm over a host fp32 array): {4 * n / t / 1e9:.2f} GB/s", flush=True)
    t = wall(lambda: zc.cast_bf16(tmp, bufs[2].ptr, n))
    print(f"kernel writes pinned host memory (zc_cast_bf16 into a host array): {2 * n / t / 1e9:.2f} GB/s", flush=True)
    t = wall(lambda: zc.cast_bf16(bufs[0].ptr, bufs[2].ptr, n))
    print(f"2:1 mix (zc_cast_bf16 host fp32 -> host bf16): {4 * n / t / 1e9:.2f} GB/s read next to "
          f"{2 * n / t / 1e9:.2f} GB/s written", flush=True)
    hviews[2].zero_()
    g = torch.empty(n, dtype=torch.bfloat16, device=dev)
    synth.device_normal_(g, synth.G_STD, seed=2002)
    step = [0]

    def offloaded(ptrs):
        step[0] += 1
        ctx.adam_step(None, None, None, 0, ptrs[0], ptrs[1], ptrs[2], n, g, zc.BF16,
                      zc.hparams(step=step[0], **synth.HP), bf16_out_dev=out_dev)

    mine = [b.ptr for b in bufs]
    print("# zero-copy offloaded step, GB/s each way, by threads per workgroup, rows and wave cap", flush=True)
    for b in (64, 128, 256):
        for r in (1, 2, 4):
            cells = []
            for w in (0, 4, 8, 16, 32):
                for k, val in (("offload.zc_block", b), ("offload.zc_rows", r), ("offload.zc_waves_per_cu", w)):
                    zc.tune_set(k, val)
                t = wall(lambda: offloaded(mine))
                cells.append(f"cap {w}: {12 * n / t / 1e9:.2f}")
            print(f"zero-copy block={b:3d} rows={r}: " + ", ".join(cells), flush=True)
    zc.tune_set("offload.zc_block", 256)
    zc.tune_set("offload.zc_rows", 2)
    zc.tune_set("offload.zc_waves_per_cu", 0)
    for nt in (0, 1, 2, 3):
        zc.tune_set("adam.nontemporal", nt)
        t = wall(lambda: offloaded(mine))
        print(f"zero-copy, adam.nontemporal={nt}: {12 * n / t / 1e9:.2f}", flush=True)
    zc.tune_set("adam.nontemporal", 1)
    for mode, name in ((2, "staged reads + direct writes"), (0, "staged ring")):
        zc.tune_set("offload.zero_copy", mode)
        t = wall(lambda: offloaded(mine))
        print(f"{name}: {12 * n / t / 1e9:.2f}", flush=True)
    zc.tune_set("offload.zero_copy", 1)
    # flavours of pinned memory, straight from the runtime (zc_host_alloc takes the default)
    hip = _hip()
    hip.hipHostMalloc.argtypes = [ctypes.POINTER(ctypes.c_void_p), ctypes.c_size_t, ctypes.c_uint]
    hip.hipHostFree.argtypes = [ctypes.c_void_p]
    flavours = {"default": 0x0, "portable | mapped": 0x3, "write-combined": 0x4, "numa-user": 0x20000000,
                "coherent": 0x40000000, "non-coherent": 0x80000000}
    for name, flag_bits in flavours.items():
        ptrs = []
        for _ in range(3):
            q = ctypes.c_void_p()
            if hip.hipHostMalloc(ctypes.byref(q), 4 * n, flag_bits) != 0:
                break
            ptrs.append(q)
        if len(ptrs) < 3:
            print(f"pinned memory '{name}': refused", flush=True)
        else:
            views = [torch.from_numpy(np.frombuffer((ctypes.c_char * (4 * n)).from_address(q.value), dtype=np.float32))
                     for q in ptrs]
            views[0].copy_(tmp)
            views[1].zero_()
            views[2].zero_()
            t = wall(lambda: offloaded([q.value for q in ptrs]))
            print(f"zero-copy over pinned memory '{name}': {12 * n / t / 1e9:.2f}", flush=True)
            del views
        for q in ptrs:
            hip.hipHostFree(q)
    ctx.destroy()
    del hviews
    for b in bufs:
        b.free()


def main():
    ap = argparse.ArgumentParser(prog="python -m paper_2504_09983_amd.tune")
    sub = ap.add_subparsers(dest="what", required=True)
    a = sub.add_parser("adam")
    a.add_argument("--workload", default="llama3_8b", choices=["llama3_8b", "llama3_70b", "mixtral_8x7b"])
    a.add_argument("--grid", default="fine", choices=["coarse", "fine", "nt"])
    a.add_argument("--reps", type=int, default=0)
    a.set_defaults(fn=sweep_adam)
    k = sub.add_parser("packed")
    k.add_argument("--workload", default="llama3_8b", choices=["llama3_8b", "llama3_70b", "mixtral_8x7b"])
    k.add_argument("--reps", type=int, default=0)
    k.set_defaults(fn=sweep_packed)
    y = sub.add_parser("layout")
    y.add_argument("--elements", type=int, default=1_003_782_656)
    y.add_argument("--grads", default="bf16", choices=["bf16", "fp32"])
    y.set_defaults(fn=sweep_layout)
    sub.add_parser("streams").set_defaults(fn=sweep_streams)
    sub.add_parser("placement").set_defaults(fn=sweep_placement)
    l = sub.add_parser("link")
    l.add_argument("--elements", type=int, default=1 << 30)
    l.set_defaults(fn=sweep_link)
    args = ap.parse_args()
    args.fn(args)


if __name__ == "__main__":
    main()
