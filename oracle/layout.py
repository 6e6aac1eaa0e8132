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
