"""Flat even partition of a list of tensors over W ranks, written out plainly.

TEST INFRASTRUCTURE (part of the CPU oracle).

Paper, Fully-sharded approach: every parameter is split evenly over all ranks
and an all-gather rebuilds the full parameters in one large buffer.  Reading
used here: the tensors are flattened in their canonical order into one buffer
of T elements, the buffer is cut into W equal shards of S' elements, where S'
is ceil(T / W) rounded up to a multiple of ``shard_align``; the padding sits
only at the very end (last rank's tail) and is zero.  The gathered buffer is
the W shards in rank order, i.e. the padded flat buffer, so tensor t occupies
gathered[off_t : off_t + n_t] with off_0 = 0 and off_{t+1} = off_t + n_t.
"""
from __future__ import annotations

import numpy as np


def flat_layout(numels, world: int, shard_align: int = 1):
    """Return (offsets[int64, ntensors], shard_numel S', total T)."""
    if world < 1 or shard_align < 1:
        raise ValueError("world and shard_align must be positive")
    offsets = []
    off = 0
    for n in numels:
        n = int(n)
        if n < 0:
            raise ValueError("negative tensor size")
        offsets.append(off)
        off += n
    total = off
    per_rank = -(-total // world)
    shard = -(-per_rank // shard_align) * shard_align
    return np.asarray(offsets, dtype=np.int64), int(shard), int(total)


def ranks_spanned(offset: int, numel: int, shard: int):
    """Inclusive (first_rank, last_rank) whose shards hold a non-empty tensor."""
    if numel <= 0:
        raise ValueError("empty tensor spans no rank")
    return offset // shard, (offset + numel - 1) // shard


def gather_shards(shards):
    """The all-gather result: rank shards concatenated in rank order."""
    return np.concatenate([np.asarray(s) for s in shards])


def flatten_pad(tensors, world: int, shard_align: int = 1, dtype=np.uint16):
    """Padded flat buffer (length W * S') from per-tensor arrays; tail zero."""
    numels = [np.asarray(t).size for t in tensors]
    _, shard, total = flat_layout(numels, world, shard_align)
    flat = np.zeros(world * shard, dtype=dtype)
    pos = 0
    for t in tensors:
        t = np.asarray(t, dtype=dtype).reshape(-1)
        flat[pos:pos + t.size] = t
        pos += t.size
    assert pos == total
    return flat


# ---------------------------------------------------------------------------
# Per-tensor even partition (the literal layout of the paper's Fully-sharded
# approach: every parameter tensor is split evenly over the ranks) gathered by
# one fused all-gather over a group of tensors (Proactive prefetching, Fuse(U)).
#
# Reading: tensor t of n_t elements is cut into W slices of s_t = ceil(n_t / W)
# elements rounded up to a multiple of `align`; rank r owns elements
# [r*s_t, (r+1)*s_t) of it, the part beyond n_t being zero padding.  A rank's
# send buffer is its slices of all tensors of the group back to back (length
# L = sum s_t); the gathered buffer is the W send buffers in rank order.
# ---------------------------------------------------------------------------

def per_tensor_slices(numels, world: int, align: int = 1):
    """(slice sizes s_t, offsets o_t inside a rank's send buffer, send length L)."""
    if world < 1 or align < 1:
        raise ValueError("world and align must be positive")
    sizes, offs, pos = [], [], 0
    for n in numels:
        n = int(n)
        if n < 0:
            raise ValueError("negative tensor size")
        s = -(-n // world)
        s = -(-s // align) * align
        sizes.append(s)
        offs.append(pos)
        pos += s
    return sizes, offs, pos


def per_tensor_gather(tensors, world: int, align: int = 1, dtype=np.uint16):
    """Build the gathered buffer element by element from the definition."""
    numels = [np.asarray(t).size for t in tensors]
    sizes, offs, L = per_tensor_slices(numels, world, align)
    gathered = np.zeros(world * L, dtype=dtype)
    for r in range(world):
        for t, s, o, n in zip(tensors, sizes, offs, numels):
            flat = np.asarray(t, dtype=dtype).reshape(-1)
            for j in range(s):
                i = r * s + j
                if i < n:
                    gathered[r * L + o + j] = flat[i]
    return gathered


def per_tensor_segments(numels, world: int, align: int = 1):
    """Unshard segments (tensor index, src offset in gathered, dst offset in the tensor,
    numel), one per (tensor, rank) that holds at least one real element."""
    sizes, offs, L = per_tensor_slices(numels, world, align)
    segs = []
    for t, (n, s, o) in enumerate(zip(numels, sizes, offs)):
        for r in range(world):
            k = min(s, max(0, int(n) - r * s))
            if k > 0:
                segs.append((t, r * L + o, r * s, k))
    return segs, L


# ---------------------------------------------------------------------------
# Packed optimizer state (a layout of this build, not of the paper: the paper
# only fixes that a rank keeps fp32 parameters, momentum and variance;
# Experimental settings).  Definition: the partition is cut into granules of G
# elements; granule k of p, then granule k of m, then granule k of v follow
# each other, for k = 0, 1, ...; the last granule is padded with zeros.
# ---------------------------------------------------------------------------

def packed_state_numel(n: int, granule: int) -> int:
    """Floats in the packed array of an n-element partition."""
    if granule < 1:
        raise ValueError("granule must be positive")
    if n <= 0:
        return 0
    return 3 * (-(-int(n) // granule)) * granule


def pack_state(p, m, v, granule: int):
    """The packed array, built granule by granule exactly as the definition reads."""
    p = np.asarray(p, dtype=np.float32)
    m = np.asarray(m, dtype=np.float32)
    v = np.asarray(v, dtype=np.float32)
    n = p.size
    if m.size != n or v.size != n:
        raise ValueError("p, m, v differ in length")
    out = np.zeros(packed_state_numel(n, granule), dtype=np.float32)
    k = 0
    while k * granule < n:
        lo, hi = k * granule, min((k + 1) * granule, n)
        base = 3 * k * granule
        out[base:base + (hi - lo)] = p[lo:hi]
        out[base + granule:base + granule + (hi - lo)] = m[lo:hi]
        out[base + 2 * granule:base + 2 * granule + (hi - lo)] = v[lo:hi]
        k += 1
    return out


def unpack_state(state, n: int, granule: int):
    """(p, m, v) read back out of a packed array, granule by granule."""
    state = np.asarray(state, dtype=np.float32)
    if state.size != packed_state_numel(n, granule):
        raise ValueError("packed array has the wrong length")
    p = np.empty(n, dtype=np.float32)
    m = np.empty(n, dtype=np.float32)
    v = np.empty(n, dtype=np.float32)
    k = 0
    while k * granule < n:
        first, count = k * granule, min(granule, n - k * granule)
        start = 3 * k * granule
        p[first:first + count] = state[start:start + count]
        m[first:first + count] = state[start + granule:start + granule + count]
        v[first:first + count] = state[start + 2 * granule:start + 2 * granule + count]
        k += 1
    return p, m, v
