"""CPU oracle (TEST INFRASTRUCTURE, not the product).

Thin numpy front-end over ``zc_oracle.c`` (plain sequential C, double
intermediates) plus the flat-partition layout written out in numpy
(``oracle.layout``).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; it never imports
the HIP package and shares no code with it.

Definitions followed: Adam with momentum and variance buffers kept in fp32
next to fp32 master parameters (paper: Experimental settings; Adaptive
offloading), bias-corrected Adam per Kingma & Ba Algorithm 1, decoupled weight
decay per Loshchilov & Hutter, IEEE round-to-nearest-even for the bf16 copy,
and the even partition of the flattened parameters across ranks (paper:
Fully-sharded approach).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

from . import layout  # noqa: F401  (re-exported)

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zc_oracle.c")
_LIB = os.path.join(_HERE, "libzc_oracle.so")

ADAMW = 0
ADAM_L2 = 1


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no fast-math, no FMA contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math",
             "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _prepare(lib):
    """Declare the argument types of a loaded oracle library."""
    i64, f32, vp, i32 = ctypes.c_int64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int
    lib.zco_adam_step.argtypes = [vp, vp, vp, vp, i32, i64, f32, f32, f32, f32, f32,
                                  f32, i64, i32, vp, i32]
    lib.zco_adam_step.restype = None
    lib.zco_adam_step_f32.argtypes = lib.zco_adam_step.argtypes
    lib.zco_adam_step_f32.restype = None
    lib.zco_cast_bf16.argtypes = [vp, vp, i64]
    lib.zco_cast_bf16.restype = None
    lib.zco_upcast_bf16.argtypes = [vp, vp, i64]
    lib.zco_upcast_bf16.restype = None
    lib.zco_grad_sqnorm.argtypes = [vp, i32, i64, ctypes.POINTER(ctypes.c_double),
                                    ctypes.POINTER(ctypes.c_int32)]
    lib.zco_grad_sqnorm.restype = None
    lib.zco_unshard.argtypes = [vp, vp, vp, vp, i64]
    lib.zco_unshard.restype = None
    lib.zco_grad_accumulate.argtypes = [vp, vp, i32, i64, f32]
    lib.zco_grad_accumulate.restype = None
    lib.zco_clip_scale.argtypes = [f32, f32, f32]
    lib.zco_clip_scale.restype = f32
    return lib


def _load():
    global _lib
    if _lib is None:
        _lib = _prepare(ctypes.CDLL(build()))
    return _lib


def _f32(a, name):
    if not (isinstance(a, np.ndarray) and a.dtype == np.float32 and a.flags.c_contiguous
            and a.flags.writeable):
        raise TypeError(f"{name}: need a writeable C-contiguous float32 ndarray")
    return a


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def adam_step(p, m, v, g, *, lr, beta1, beta2, eps, weight_decay, step,
              grad_scale=1.0, mode=ADAMW, bf16_out=None, skip=False, all_fp32=False):
    """In-place Adam(W) step over flat fp32 ``p, m, v``.

    ``g`` is float32 (values) or uint16 (bf16 bit patterns).  ``bf16_out`` is
    an optional uint16 array that receives RNE(p_new).  ``all_fp32`` selects the
    second-opinion build whose per-element intermediates are fp32 instead of double.
    """
    _f32(p, "p"), _f32(m, "m"), _f32(v, "v")
    n = p.size
    if m.size != n or v.size != n or g.size != n:
        raise ValueError("p, m, v, g must have equal length")
    if g.dtype == np.float32:
        is_bf16 = 0
    elif g.dtype == np.uint16:
        is_bf16 = 1
    else:
        raise TypeError("g must be float32 or uint16 (bf16 bits)")
    if not g.flags.c_contiguous:
        raise TypeError("g must be contiguous")
    if step < 1:
        raise ValueError("step is 1-based")
    out_ptr = None
    if bf16_out is not None:
        if bf16_out.dtype != np.uint16 or bf16_out.size != n or not bf16_out.flags.c_contiguous:
            raise TypeError("bf16_out must be a contiguous uint16 array of length n")
        out_ptr = _ptr(bf16_out)
    fn = _load().zco_adam_step_f32 if all_fp32 else _load().zco_adam_step
    fn(_ptr(p), _ptr(m), _ptr(v), _ptr(g), is_bf16, n,
       float(np.float32(lr)), float(np.float32(beta1)), float(np.float32(beta2)),
       float(np.float32(eps)), float(np.float32(weight_decay)), float(np.float32(grad_scale)),
       int(step), int(mode), out_ptr, 1 if skip else 0)


def adam_step_groups(p, m, v, g, *, ranges=(), lr, weight_decay, grad_scale=1.0,
                     grad_scale_dev=None, bf16_out=None, **hp):
    """The step with per-range hyper-parameters, written as what it means: every stretch of
    the partition gets a plain adam_step with its own lr and weight decay.
    ranges = [(begin, end, lr_scale, weight_decay)], sorted, disjoint; the rest uses lr / weight_decay.
    grad_scale_dev models a scale that lives on the device: the effective scale is the fp32
    product grad_scale * grad_scale_dev."""
    n = p.size
    scale = np.float32(grad_scale)
    if grad_scale_dev is not None:
        scale = np.float32(scale * np.float32(grad_scale_dev))
    pieces, at = [], 0
    for b, e, lr_scale, wd in ranges:
        pieces.append((at, b, np.float32(lr), weight_decay))
        pieces.append((b, e, np.float32(np.float32(lr) * np.float32(lr_scale)), wd))
        at = e
    pieces.append((at, n, np.float32(lr), weight_decay))
    for b, e, lr_here, wd_here in pieces:
        if e > b:
            adam_step(p[b:e], m[b:e], v[b:e], g[b:e], lr=lr_here, weight_decay=wd_here,
                      grad_scale=scale, bf16_out=None if bf16_out is None else bf16_out[b:e], **hp)


def clip_scale(sqnorm, max_norm: float, inv_loss_scale: float = 1.0) -> np.float32:
    return np.float32(_load().zco_clip_scale(float(np.float32(sqnorm)), float(np.float32(max_norm)),
                                             float(np.float32(inv_loss_scale))))


def cast_bf16(src: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round-to-nearest-even."""
    src = np.ascontiguousarray(src, dtype=np.float32)
    dst = np.empty(src.shape, dtype=np.uint16)
    _load().zco_cast_bf16(_ptr(src), _ptr(dst), src.size)
    return dst


def upcast_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> fp32, exact."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    dst = np.empty(bits.shape, dtype=np.float32)
    _load().zco_upcast_bf16(_ptr(bits), _ptr(dst), bits.size)
    return dst


def grad_sqnorm(g: np.ndarray):
    """(sum of squares in double, found_inf flag) of fp32 values or bf16 bits."""
    g = np.ascontiguousarray(g)
    if g.dtype == np.float32:
        is_bf16 = 0
    elif g.dtype == np.uint16:
        is_bf16 = 1
    else:
        raise TypeError("g must be float32 or uint16 (bf16 bits)")
    s = ctypes.c_double(0.0)
    f = ctypes.c_int32(0)
    _load().zco_grad_sqnorm(_ptr(g), is_bf16, g.size, ctypes.byref(s), ctypes.byref(f))
    return s.value, int(f.value)


def grad_accumulate(acc: np.ndarray, micro: np.ndarray, scale: float = 1.0) -> None:
    """acc += upcast(micro) * scale in place; micro is float32 values or uint16 bf16 bits."""
    _f32(acc, "acc")
    micro = np.ascontiguousarray(micro)
    if micro.size != acc.size:
        raise ValueError("acc and micro must have equal length")
    if micro.dtype == np.float32:
        is_bf16 = 0
    elif micro.dtype == np.uint16:
        is_bf16 = 1
    else:
        raise TypeError("micro must be float32 or uint16 (bf16 bits)")
    _load().zco_grad_accumulate(_ptr(acc), _ptr(micro), is_bf16, acc.size, float(np.float32(scale)))


def unshard(gathered: np.ndarray, src_offsets, numels):
    """Copy ``gathered[off : off + n]`` into a fresh uint16 array per segment."""
    gathered = np.ascontiguousarray(gathered, dtype=np.uint16)
    offs = np.ascontiguousarray(src_offsets, dtype=np.int64)
    nums = np.ascontiguousarray(numels, dtype=np.int64)
    if offs.size != nums.size:
        raise ValueError("one offset per segment")
    if offs.size and (offs.min() < 0 or nums.min() < 0 or (offs + nums).max() > gathered.size):
        raise ValueError("segment outside the gathered buffer")
    outs = [np.empty(int(k), dtype=np.uint16) for k in nums]
    ptrs = (ctypes.c_void_p * max(1, len(outs)))(*[o.ctypes.data for o in outs])
    _load().zco_unshard(_ptr(gathered), _ptr(offs), ctypes.cast(ptrs, ctypes.c_void_p),
                        _ptr(nums), len(outs))
    return outs


def unshard_per_tensor(gathered: np.ndarray, numels, world: int, align: int = 1):
    """Per-tensor even partition: rebuild every tensor from its W slices."""
    segs, L = layout.per_tensor_segments(numels, world, align)
    gathered = np.ascontiguousarray(gathered, dtype=np.uint16)
    if gathered.size != world * L:
        raise ValueError("gathered buffer has the wrong length for this layout")
    outs = [np.zeros(int(n), dtype=np.uint16) for n in numels]
    pieces = unshard(gathered, [s[1] for s in segs], [s[3] for s in segs])
    for (t, _src, dst, k), piece in zip(segs, pieces):
        outs[t][dst:dst + k] = piece
    return outs


def offload_adam_step(p_res, m_res, v_res, p_host, m_host, v_host, g, *, bf16_out=None, **hp):
    """Offloaded step, by definition the plain step over [resident || streamed].

    Elements are independent, so where a value lives and in what pieces it is
    moved cannot change it (paper: Adaptive offloading keeps the update itself
    on the GPU and only moves the states).  Updates all six arrays in place.
    """
    n_res = p_res.size
    p = np.concatenate([p_res, p_host])
    m = np.concatenate([m_res, m_host])
    v = np.concatenate([v_res, v_host])
    adam_step(p, m, v, g, bf16_out=bf16_out, **hp)
    p_res[:], p_host[:] = p[:n_res], p[n_res:]
    m_res[:], m_host[:] = m[:n_res], m[n_res:]
    v_res[:], v_host[:] = v[:n_res], v[n_res:]
