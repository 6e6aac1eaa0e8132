"""ctypes binding over libzc.so — argument marshalling only.

Every function here has the name and meaning of the C entry point declared in
``include/zc.h``; nothing is computed in Python.  Tensors are passed as raw
device (or pinned-host) addresses; PyTorch is only the allocator and the source
of the HIP stream.  If the shared library is missing or fails to load this
module raises — there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libzc.so")

OK, ERR_INVALID_ARG, ERR_ALIGNMENT, ERR_HIP, ERR_UNSUPPORTED, ERR_NOMEM = range(6)
F32, BF16 = 0, 1
ADAMW, ADAM_L2 = 0, 1

_STATUS_NAMES = {0: "ZC_OK", 1: "ZC_ERR_INVALID_ARG", 2: "ZC_ERR_ALIGNMENT", 3: "ZC_ERR_HIP",
                 4: "ZC_ERR_UNSUPPORTED", 5: "ZC_ERR_NOMEM"}


class ZcError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"{_STATUS_NAMES.get(status, status)}: {message}")
        self.status = status
        self.message = message


class AdamHparams(ctypes.Structure):
    _fields_ = [("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float),
                ("eps", ctypes.c_float), ("weight_decay", ctypes.c_float),
                ("grad_scale", ctypes.c_float), ("step", ctypes.c_int64),
                ("mode", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class SchedOp(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("index", ctypes.c_int32)]


class Fragment(ctypes.Structure):
    _fields_ = [("dev", ctypes.c_void_p), ("host", ctypes.c_void_p), ("bytes", ctypes.c_int64)]


OP_COMPUTE, OP_OFFLOAD, OP_SYNC_FREE, OP_RELOAD, OP_SYNC_RELOAD = range(5)


class ParamRange(ctypes.Structure):
    _fields_ = [("begin", ctypes.c_int64), ("end", ctypes.c_int64), ("lr_scale", ctypes.c_float),
                ("weight_decay", ctypes.c_float)]


class Segment(ctypes.Structure):
    _fields_ = [("src_offset", ctypes.c_int64), ("dst", ctypes.c_void_p),
                ("numel", ctypes.c_int64)]


_lib = None


def lib():
    """Load libzc.so once; raise if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with "
                          "`python -m paper_2504_09983_amd.build` (hipcc, gfx950)")
    # One HIP runtime per process: PyTorch (the allocator and stream source) ships its
    # own libamdhip64 and must map it first, so that libzc binds to that same instance
    # instead of bringing in a second runtime that knows nothing of torch's streams.
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    L.zc_version.restype = ctypes.c_int
    L.zc_version.argtypes = []
    L.zc_last_error.restype = ctypes.c_char_p
    L.zc_last_error.argtypes = []
    L.zc_adam_step.restype = ctypes.c_int
    L.zc_adam_step.argtypes = [vp, vp, vp, vp, ctypes.c_int, i64, ctypes.POINTER(AdamHparams),
                               vp, vp, vp]
    L.zc_adam_step_groups.restype = ctypes.c_int
    L.zc_adam_step_groups.argtypes = [vp, vp, vp, vp, ctypes.c_int, i64, ctypes.POINTER(AdamHparams),
                                      ctypes.POINTER(ParamRange), i64, vp, vp, vp, vp]
    L.zc_packed_state_numel.restype = i64
    L.zc_packed_state_numel.argtypes = [i64]
    L.zc_state_pack.restype = ctypes.c_int
    L.zc_state_pack.argtypes = [vp, vp, vp, i64, vp, vp]
    L.zc_state_unpack.restype = ctypes.c_int
    L.zc_state_unpack.argtypes = [vp, i64, vp, vp, vp, vp]
    L.zc_adam_step_packed.restype = ctypes.c_int
    L.zc_adam_step_packed.argtypes = [vp, vp, ctypes.c_int, i64, ctypes.POINTER(AdamHparams),
                                      ctypes.POINTER(ParamRange), i64, vp, vp, vp, vp]
    L.zc_clip_scale.restype = ctypes.c_int
    L.zc_clip_scale.argtypes = [vp, ctypes.c_float, ctypes.c_float, vp, vp]
    L.zc_cast_bf16.restype = ctypes.c_int
    L.zc_cast_bf16.argtypes = [vp, vp, i64, vp]
    L.zc_flat_layout.restype = ctypes.c_int
    L.zc_flat_layout.argtypes = [ctypes.POINTER(i64), i64, i32, i64, ctypes.POINTER(i64),
                                 ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.zc_per_tensor_layout.restype = ctypes.c_int
    L.zc_per_tensor_layout.argtypes = [ctypes.POINTER(i64), i64, i32, i64, ctypes.POINTER(i64),
                                       ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i64)]
    L.zc_unshard_plan_create.restype = ctypes.c_int
    L.zc_unshard_plan_create.argtypes = [ctypes.POINTER(Segment), i64, i64, ctypes.POINTER(vp)]
    L.zc_unshard.restype = ctypes.c_int
    L.zc_unshard.argtypes = [vp, vp, vp]
    L.zc_unshard_plan_destroy.restype = ctypes.c_int
    L.zc_unshard_plan_destroy.argtypes = [vp]
    L.zc_offload_create.restype = ctypes.c_int
    L.zc_offload_create.argtypes = [i64, i32, ctypes.POINTER(vp)]
    L.zc_offload_adam_step.restype = ctypes.c_int
    L.zc_offload_adam_step.argtypes = [vp, vp, vp, vp, i64, vp, vp, vp, i64, vp, ctypes.c_int,
                                       ctypes.POINTER(AdamHparams), vp, vp, vp]
    L.zc_offload_destroy.restype = ctypes.c_int
    L.zc_offload_destroy.argtypes = [vp]
    L.zc_plan_adaptive_offload.restype = ctypes.c_int
    L.zc_plan_adaptive_offload.argtypes = [ctypes.POINTER(i64), i64, i64, ctypes.POINTER(i64), i64, i64,
                                           ctypes.POINTER(SchedOp), i64, ctypes.POINTER(i64)]
    dbl = ctypes.c_double
    L.zc_plan_prefetch.restype = ctypes.c_int
    L.zc_plan_prefetch.argtypes = [ctypes.POINTER(i32), ctypes.POINTER(i64), ctypes.POINTER(i64), i64, i64,
                                   i64, ctypes.POINTER(i64), ctypes.POINTER(dbl), i64, dbl,
                                   ctypes.POINTER(i32), ctypes.POINTER(i32)]
    L.zc_select_unsharded.restype = ctypes.c_int
    L.zc_select_unsharded.argtypes = [ctypes.POINTER(i64), i64, ctypes.POINTER(i64), ctypes.POINTER(dbl),
                                      i64, i64, ctypes.POINTER(i32), ctypes.POINTER(i64)]
    L.zc_schedule_run.restype = ctypes.c_int
    L.zc_schedule_run.argtypes = [vp, ctypes.POINTER(SchedOp), i64, ctypes.POINTER(ctypes.c_float), i64,
                                  ctypes.POINTER(Fragment), i64, i32, vp]
    L.zc_host_alloc.restype = ctypes.c_int
    L.zc_host_alloc.argtypes = [i64, ctypes.POINTER(vp)]
    L.zc_host_free.restype = ctypes.c_int
    L.zc_host_free.argtypes = [vp]
    L.zc_offload_probe_link.restype = ctypes.c_int
    L.zc_offload_probe_link.argtypes = [vp, vp, vp, i64, i32, ctypes.POINTER(ctypes.c_float)]
    L.zc_grad_accumulate.restype = ctypes.c_int
    L.zc_grad_accumulate.argtypes = [vp, vp, ctypes.c_int, i64, ctypes.c_float, vp]
    L.zc_grad_sqnorm.restype = ctypes.c_int
    L.zc_grad_sqnorm.argtypes = [vp, ctypes.c_int, i64, vp, vp, vp]
    L.zc_grad_sqnorm_static.restype = ctypes.c_int
    L.zc_grad_sqnorm_static.argtypes = [vp, ctypes.c_int, i64, vp, vp, vp]
    L.zc_tune_set.restype = ctypes.c_int
    L.zc_tune_set.argtypes = [ctypes.c_char_p, i64]
    L.zc_tune_get.restype = ctypes.c_int
    L.zc_tune_get.argtypes = [ctypes.c_char_p, ctypes.POINTER(i64)]
    _lib = L
    return L


def _check(status: int) -> None:
    if status != OK:
        raise ZcError(status, lib().zc_last_error().decode("utf-8", "replace"))


def _addr(x) -> Optional[int]:
    """Address of a torch tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    raise TypeError(f"cannot take the address of {type(x)!r}")


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream  # a hipStream_t on ROCm
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def hparams(*, lr, beta1, beta2, eps, weight_decay, step, grad_scale=1.0, mode=ADAMW) -> AdamHparams:
    return AdamHparams(lr, beta1, beta2, eps, weight_decay, grad_scale, int(step), int(mode), 0)


def version() -> int:
    return lib().zc_version()


def last_error() -> str:
    return lib().zc_last_error().decode("utf-8", "replace")


def adam_step(p, m, v, g, g_dtype: int, n: int, hp: AdamHparams, bf16_out=None, skip_flag=None,
              stream=None) -> None:
    _check(lib().zc_adam_step(_addr(p), _addr(m), _addr(v), _addr(g), g_dtype, n,
                              ctypes.byref(hp), _addr(bf16_out), _addr(skip_flag),
                              _stream(stream)))


def adam_step_groups(p, m, v, g, g_dtype: int, n: int, hp: AdamHparams, ranges=(), bf16_out=None,
                     skip_flag=None, grad_scale_dev=None, stream=None) -> None:
    """ranges = [(begin, end, lr_scale, weight_decay), ...]"""
    arr = (ParamRange * max(1, len(ranges)))(*[ParamRange(int(b), int(e), float(s), float(w))
                                               for b, e, s, w in ranges])
    _check(lib().zc_adam_step_groups(_addr(p), _addr(m), _addr(v), _addr(g), g_dtype, n,
                                     ctypes.byref(hp), arr, len(ranges), _addr(bf16_out),
                                     _addr(skip_flag), _addr(grad_scale_dev), _stream(stream)))


PACKED_GRANULE = 8192


def packed_state_numel(n: int) -> int:
    return int(lib().zc_packed_state_numel(n))


def state_pack(p, m, v, n: int, state, stream=None) -> None:
    _check(lib().zc_state_pack(_addr(p), _addr(m), _addr(v), n, _addr(state), _stream(stream)))


def state_unpack(state, n: int, p=None, m=None, v=None, stream=None) -> None:
    _check(lib().zc_state_unpack(_addr(state), n, _addr(p), _addr(m), _addr(v), _stream(stream)))


def adam_step_packed(state, g, g_dtype: int, n: int, hp: AdamHparams, ranges=(), bf16_out=None,
                     skip_flag=None, grad_scale_dev=None, stream=None) -> None:
    """ranges = [(begin, end, lr_scale, weight_decay), ...]"""
    arr = (ParamRange * max(1, len(ranges)))(*[ParamRange(int(b), int(e), float(s), float(w))
                                               for b, e, s, w in ranges])
    _check(lib().zc_adam_step_packed(_addr(state), _addr(g), g_dtype, n, ctypes.byref(hp), arr,
                                     len(ranges), _addr(bf16_out), _addr(skip_flag),
                                     _addr(grad_scale_dev), _stream(stream)))


def clip_scale(sqnorm, max_norm: float, inv_loss_scale: float, scale_out, stream=None) -> None:
    _check(lib().zc_clip_scale(_addr(sqnorm), max_norm, inv_loss_scale, _addr(scale_out),
                               _stream(stream)))


def cast_bf16(src, dst, n: int, stream=None) -> None:
    _check(lib().zc_cast_bf16(_addr(src), _addr(dst), n, _stream(stream)))


def flat_layout(numels: Sequence[int], world: int, shard_align: int = 1):
    """(offsets list, shard_numel, total) computed by the C library on the host."""
    k = len(numels)
    arr = (ctypes.c_int64 * max(1, k))(*[int(x) for x in numels])
    offs = (ctypes.c_int64 * max(1, k))()
    shard = ctypes.c_int64(0)
    total = ctypes.c_int64(0)
    _check(lib().zc_flat_layout(arr, k, world, shard_align, offs, ctypes.byref(shard),
                                ctypes.byref(total)))
    return [offs[i] for i in range(k)], shard.value, total.value


def per_tensor_layout(numels: Sequence[int], world: int, align: int = 1):
    """([(tensor, src_offset, dst_offset, numel), ...] for every (tensor, rank), send_numel)."""
    k = len(numels)
    arr = (ctypes.c_int64 * max(1, k))(*[int(x) for x in numels])
    src = (ctypes.c_int64 * max(1, k * world))()
    dst = (ctypes.c_int64 * max(1, k * world))()
    cnt = (ctypes.c_int64 * max(1, k * world))()
    send = ctypes.c_int64(0)
    _check(lib().zc_per_tensor_layout(arr, k, world, align, src, dst, cnt, ctypes.byref(send)))
    segs = [(i // world, src[i], dst[i], cnt[i]) for i in range(k * world)]
    return segs, send.value


def plan_adaptive_offload(p_mem: Sequence[int], n_forward: int, frag_bytes: Sequence[int],
                          mem_limit: int):
    """Schedule as a list of (kind, index) from the C planner."""
    n, k = len(p_mem), len(frag_bytes)
    pm = (ctypes.c_int64 * max(1, n))(*[int(x) for x in p_mem])
    fb = (ctypes.c_int64 * max(1, k))(*[int(x) for x in frag_bytes])
    cap = n + 4 * k
    out = (SchedOp * max(1, cap))()
    length = ctypes.c_int64(0)
    _check(lib().zc_plan_adaptive_offload(pm, n, n_forward, fb, k, mem_limit, out, cap,
                                          ctypes.byref(length)))
    return [(out[i].kind, out[i].index) for i in range(length.value)]


def _i64s(xs):
    return (ctypes.c_int64 * max(1, len(xs)))(*[int(x) for x in xs])


def plan_prefetch(is_allgather, bag_bytes, p_mem, mem_limit: int, prefetch_limit: int, tc_sizes,
                  tc_times, alpha: float):
    """New schedule as [("op", i) | ("allgather", [i, ...]), ...] from the C planner."""
    n = len(is_allgather)
    flags = (ctypes.c_int32 * max(1, n))(*[int(bool(x)) for x in is_allgather])
    times = (ctypes.c_double * max(1, len(tc_times)))(*[float(x) for x in tc_times])
    order = (ctypes.c_int32 * max(1, n))()
    group = (ctypes.c_int32 * max(1, n))()
    _check(lib().zc_plan_prefetch(flags, _i64s(bag_bytes), _i64s(p_mem), n, int(mem_limit),
                                  int(prefetch_limit), _i64s(tc_sizes), times, len(tc_sizes),
                                  float(alpha), order, group))
    out = []
    for k in range(n):
        if group[k] < 0:
            out.append(("op", order[k]))
        elif out and out[-1][0] == "allgather" and out[-1][2] == group[k]:
            out[-1][1].append(order[k])
        else:
            out.append(("allgather", [order[k]], group[k]))
    return [(e[0], e[1]) for e in out]


def select_unsharded(bag_bytes, tc_sizes, tc_times, budget: int):
    n = len(bag_bytes)
    times = (ctypes.c_double * max(1, len(tc_times)))(*[float(x) for x in tc_times])
    chosen = (ctypes.c_int32 * max(1, n))()
    count = ctypes.c_int64(0)
    _check(lib().zc_select_unsharded(_i64s(bag_bytes), n, _i64s(tc_sizes), times, len(tc_sizes),
                                     int(budget), chosen, ctypes.byref(count)))
    return [chosen[i] for i in range(count.value)]


class UnshardPlan:
    """Owns a zc_unshard_plan; segments are (src_offset, dst address or tensor, numel)."""

    def __init__(self, segments, gathered_numel: int):
        segs = [(int(o), _addr(d) or 0, int(n)) for o, d, n in segments]
        arr = (Segment * max(1, len(segs)))(*[Segment(o, d if d else None, n) for o, d, n in segs])
        handle = ctypes.c_void_p(None)
        _check(lib().zc_unshard_plan_create(arr, len(segs), gathered_numel, ctypes.byref(handle)))
        self._h = handle

    def run(self, gathered, stream=None) -> None:
        _check(lib().zc_unshard(self._h, _addr(gathered), _stream(stream)))

    def destroy(self) -> None:
        if self._h is not None and self._h.value is not None:
            _check(lib().zc_unshard_plan_destroy(self._h))
        self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def unshard_plan_create(segments, gathered_numel: int) -> UnshardPlan:
    return UnshardPlan(segments, gathered_numel)


def unshard(plan: UnshardPlan, gathered, stream=None) -> None:
    plan.run(gathered, stream)


class OffloadCtx:
    """Owns a zc_offload_ctx (staging ring, copy streams, events)."""

    def __init__(self, chunk_bytes: int = 64 << 20, num_buffers: int = 3):
        handle = ctypes.c_void_p(None)
        _check(lib().zc_offload_create(chunk_bytes, num_buffers, ctypes.byref(handle)))
        self._h = handle
        self.chunk_bytes = chunk_bytes
        self.num_buffers = num_buffers

    def adam_step(self, p_dev, m_dev, v_dev, n_resident: int, p_host, m_host, v_host,
                  n_streamed: int, g_dev, g_dtype: int, hp: AdamHparams, bf16_out_dev=None,
                  skip_flag=None, stream=None) -> None:
        _check(lib().zc_offload_adam_step(self._h, _addr(p_dev), _addr(m_dev), _addr(v_dev),
                                          n_resident, _addr(p_host), _addr(m_host), _addr(v_host),
                                          n_streamed, _addr(g_dev), g_dtype, ctypes.byref(hp),
                                          _addr(bf16_out_dev), _addr(skip_flag), _stream(stream)))

    def schedule_run(self, ops, op_ms, fragments, poison_freed: bool = False, stream=None) -> None:
        """Replay a schedule: ops = [(kind, index)], op_ms = per-operator milliseconds or None,
        fragments = [(device tensor/address, pinned host address, bytes)]."""
        arr = (SchedOp * max(1, len(ops)))(*[SchedOp(int(k), int(i)) for k, i in ops])
        n_ops = sum(1 for k, _ in ops if k == OP_COMPUTE)
        ms = None
        if op_ms is not None:
            ms = (ctypes.c_float * max(1, len(op_ms)))(*[float(x) for x in op_ms])
            n_ops = len(op_ms)
        fr = (Fragment * max(1, len(fragments)))(*[Fragment(_addr(d), _addr(h), int(b))
                                                   for d, h, b in fragments])
        _check(lib().zc_schedule_run(self._h, arr, len(ops), ms, n_ops, fr, len(fragments),
                                     1 if poison_freed else 0, _stream(stream)))

    def probe_link(self, host_src, host_dst, nbytes: int, mode: int) -> float:
        """Wall milliseconds of plain chunked pinned copies (0 = H2D, 1 = D2H, 2 = both)."""
        ms = ctypes.c_float(0.0)
        _check(lib().zc_offload_probe_link(self._h, _addr(host_src), _addr(host_dst), nbytes, mode,
                                           ctypes.byref(ms)))
        return ms.value

    def destroy(self) -> None:
        if self._h is not None and self._h.value is not None:
            _check(lib().zc_offload_destroy(self._h))
        self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class PinnedBuffer:
    """Owns pinned host memory from zc_host_alloc; `.numpy(dtype)` views it without a copy.
    The views do not keep the memory alive: drop them before `free()`."""

    def __init__(self, nbytes: int):
        ptr = ctypes.c_void_p(None)
        _check(lib().zc_host_alloc(nbytes, ctypes.byref(ptr)))
        self.ptr = ptr.value
        self.nbytes = nbytes

    def data_ptr(self) -> int:
        return self.ptr

    def numpy(self, dtype="float32"):
        import numpy as np
        dt = np.dtype(dtype)
        buf = (ctypes.c_char * self.nbytes).from_address(self.ptr)
        return np.frombuffer(buf, dtype=dt, count=self.nbytes // dt.itemsize)

    def free(self) -> None:
        if self.ptr:
            _check(lib().zc_host_free(ctypes.c_void_p(self.ptr)))
            self.ptr = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def host_alloc(nbytes: int) -> PinnedBuffer:
    return PinnedBuffer(nbytes)


def offload_create(chunk_bytes: int = 64 << 20, num_buffers: int = 3) -> OffloadCtx:
    return OffloadCtx(chunk_bytes, num_buffers)


def grad_accumulate(acc, micro, micro_dtype: int, n: int, scale: float = 1.0, stream=None) -> None:
    _check(lib().zc_grad_accumulate(_addr(acc), _addr(micro), micro_dtype, n, scale, _stream(stream)))


def grad_sqnorm(g, g_dtype: int, n: int, sqnorm_out, found_inf_out, stream=None) -> None:
    _check(lib().zc_grad_sqnorm(_addr(g), g_dtype, n, _addr(sqnorm_out), _addr(found_inf_out),
                                _stream(stream)))


def grad_sqnorm_static(g, g_dtype: int, n: int, sqnorm_out, found_inf_out, stream=None) -> None:
    _check(lib().zc_grad_sqnorm_static(_addr(g), g_dtype, n, _addr(sqnorm_out), _addr(found_inf_out),
                                       _stream(stream)))


def tune_set(key: str, value: int) -> None:
    _check(lib().zc_tune_set(key.encode(), int(value)))


def tune_get(key: str) -> int:
    out = ctypes.c_int64(0)
    _check(lib().zc_tune_get(key.encode(), ctypes.byref(out)))
    return out.value
