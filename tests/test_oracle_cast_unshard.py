"""Pins for the oracle's fp32->bf16 rounding and for the flat layout / unshard."""
import numpy as np
import pytest

import oracle
from oracle import layout
from paper_2504_09983_amd import synth


def bits(x):
    return np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)


def from_bits(u):
    return np.ascontiguousarray(u, dtype=np.uint32).view(np.float32)


# ---- cast --------------------------------------------------------------------

def test_all_bf16_values_round_trip():
    b = np.arange(1 << 16, dtype=np.uint16)
    f = oracle.upcast_bf16(b)
    assert np.array_equal(bits(f), b.astype(np.uint32) << 16)
    back = oracle.cast_bf16(f)
    nan = np.isnan(f)
    assert np.array_equal(back[~nan], b[~nan])
    # NaNs stay NaNs, keep sign, become quiet
    assert np.all((back[nan] & 0x7F80) == 0x7F80) and np.all(back[nan] & 0x0040)
    assert np.array_equal(back[nan] & 0x8000, b[nan] & 0x8000)
    assert np.all((back[nan] & 0x007F) != 0)


def test_every_tie_goes_to_even():
    hi = np.arange(1 << 16, dtype=np.uint32)
    finite = (hi & 0x7F80) != 0x7F80
    hi = hi[finite]
    ties = from_bits((hi << 16) | 0x8000)
    got = oracle.cast_bf16(ties).astype(np.uint32)
    want = np.where(hi & 1, hi + 1, hi)     # odd -> up (to even), even -> stay
    assert np.array_equal(got, want)
    below = oracle.cast_bf16(from_bits((hi << 16) | 0x7FFF)).astype(np.uint32)
    above = oracle.cast_bf16(from_bits((hi << 16) | 0x8001)).astype(np.uint32)
    assert np.array_equal(below, hi)
    assert np.array_equal(above, hi + 1)


def test_special_values():
    c = oracle.cast_bf16
    assert c(np.float32(0.0))[()] == 0x0000 and c(np.float32(-0.0))[()] == 0x8000
    assert c(np.float32(np.inf))[()] == 0x7F80 and c(np.float32(-np.inf))[()] == 0xFF80
    assert c(np.float32(1.0))[()] == 0x3F80
    # largest finite fp32 rounds up to infinity under RNE
    assert c(from_bits([0x7F7FFFFF]))[0] == 0x7F80
    assert c(from_bits([0x7F7F7FFF]))[0] == 0x7F7F
    # subnormals are rounded, not flushed
    assert c(from_bits([0x00008000]))[0] == 0x0000      # tie, even
    assert c(from_bits([0x00018000]))[0] == 0x0002      # tie, odd -> up
    assert c(from_bits([0x00008001]))[0] == 0x0001
    assert c(from_bits([0x007FFFFF]))[0] == 0x0080      # carries into the smallest normal
    # NaN payload in the low half only must not turn into infinity
    assert c(from_bits([0x7F800001]))[0] == 0x7FC0
    assert c(from_bits([0xFF800001]))[0] == 0xFFC0
    assert c(from_bits([0x7FFFFFFF]))[0] == 0x7FFF


def test_nearest_value_property_on_random_bits():
    rng = np.random.default_rng(0)
    u = rng.integers(0, 1 << 32, size=200000, dtype=np.uint64).astype(np.uint32)
    x = from_bits(u)
    ok = np.isfinite(x)
    x = x[ok]
    got = oracle.cast_bf16(x)
    y = oracle.upcast_bf16(got).astype(np.float64)
    fin = np.isfinite(y)
    with np.errstate(invalid="ignore"):
        lo = oracle.upcast_bf16((got - 1).astype(np.uint16)).astype(np.float64)
        hi = oracle.upcast_bf16((got + 1).astype(np.uint16)).astype(np.float64)
    xd = x.astype(np.float64)
    d = np.abs(y - xd)
    with np.errstate(invalid="ignore"):
        assert np.all((d <= np.abs(lo - xd)) | ~np.isfinite(lo) | ~fin)
        assert np.all((d <= np.abs(hi - xd)) | ~np.isfinite(hi) | ~fin)


def test_library_conversion_agrees():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(1)
    u = rng.integers(0, 1 << 32, size=1 << 20, dtype=np.uint64).astype(np.uint32)
    u = np.concatenate([u, (np.arange(1 << 16, dtype=np.uint32) << 16) | 0x8000])
    x = from_bits(u)
    x = x[~np.isnan(x)]
    want = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.cast_bf16(x), want)
    vals = synth.host_params(100000)
    want = torch.from_numpy(vals.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.cast_bf16(vals), want)


# ---- layout and unshard ---------------------------------------------------------

@pytest.mark.parametrize("align", [1, 8, 4096])
@pytest.mark.parametrize("numels", [[1, 3, 7, 4097], [5], [0, 9, 0, 2], [4096] * 3 + [17]])
def test_layout_brute_force(numels, align):
    W = 8
    offs, shard, total = layout.flat_layout(numels, W, align)
    assert total == sum(numels)
    assert shard % align == 0 and shard * W >= total
    assert shard - align < -(-total // W) <= shard        # smallest aligned cover
    # brute force: lay the elements out one by one
    owner = []
    for t, n in enumerate(numels):
        owner += [(t, j) for j in range(n)]
    for t, n in enumerate(numels):
        for j in (0, n // 2, n - 1):
            if n:
                assert owner[offs[t] + j] == (t, j)


def test_unshard_brute_force_ragged():
    W, A = 8, 8
    numels = [1, 3, 7, 4097, 0, 64, 129]
    rng = np.random.default_rng(2)
    tensors = [rng.integers(0, 1 << 16, size=n, dtype=np.uint16) for n in numels]
    flat = layout.flatten_pad(tensors, W, A)
    offs, shard, total = layout.flat_layout(numels, W, A)
    assert flat.size == W * shard and not flat[total:].any()
    shards = [flat[r * shard:(r + 1) * shard] for r in range(W)]
    gathered = layout.gather_shards(shards)
    assert np.array_equal(gathered, flat)
    outs = oracle.unshard(gathered, offs, numels)
    for t, o in zip(tensors, outs):
        assert np.array_equal(t, o)
    # re-flattening reproduces the gathered prefix
    assert np.array_equal(np.concatenate(outs), gathered[:total])
    # element-by-element definition
    for s, (off, n) in enumerate(zip(offs, numels)):
        for j in range(0, n, max(1, n // 5)):
            assert outs[s][j] == gathered[off + j]


def test_unshard_hash_property_and_ranks_spanned():
    W = 8
    numels = [4096 * 3, 4096, 1000, 4096 * 5 + 1, 24]
    offs, shard, total = layout.flat_layout(numels, W, 16)
    gathered = synth.host_index_hash16(0, W * shard)
    outs = oracle.unshard(gathered, offs, numels)
    for off, n, o in zip(offs, numels, outs):
        assert np.array_equal(o, synth.host_index_hash16(int(off), n))
    spans = [layout.ranks_spanned(int(o), n, shard) for o, n in zip(offs, numels)]
    assert spans[0][0] == 0 and spans[-1][1] <= W - 1
    # a tensor that ends exactly where a shard ends belongs to that shard alone
    assert layout.ranks_spanned(0, shard, shard) == (0, 0)
    assert layout.ranks_spanned(shard - 1, 2, shard) == (0, 1)
    assert layout.ranks_spanned(3 * shard, 1, shard) == (3, 3)
    assert any(a != b for a, b in spans)      # some tensor straddles a shard boundary
    for (a, b), off, n in zip(spans, offs, numels):
        assert a * shard <= off < (a + 1) * shard
        assert b * shard <= off + n - 1 < (b + 1) * shard


def test_unshard_rejects_out_of_range():
    g = np.zeros(16, np.uint16)
    with pytest.raises(ValueError):
        oracle.unshard(g, [10], [7])
    with pytest.raises(ValueError):
        oracle.unshard(g, [-1], [2])
    assert oracle.unshard(g, [], []) == []
    assert oracle.unshard(g, [16], [0])[0].size == 0


# ---- model shapes vs the values the paper prints -----------------------------------

def _golden():
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_shape_pins.txt")
    out = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            k, val, _unit, tol = line.split()
            out[k] = (float(val), float(tol))
    return out


def test_model_shapes_match_paper_sizes():
    gold = _golden()
    t70 = synth.total_params(synth.LLAMA3_70B)
    tmx = synth.total_params(synth.MIXTRAL_8X7B)
    t8 = synth.total_params(synth.LLAMA3_8B)
    assert (t8, t70, tmx) == (8_030_261_248, 70_553_706_496, 46_702_792_704)
    val, tol = gold["llama3_70b_bf16_gb"]
    assert abs(2 * t70 / 1e9 - val) <= tol
    val, tol = gold["mixtral_8x7b_bf16_gb"]
    assert abs(2 * tmx / 1e9 - val) <= tol
    val, tol = gold["mixtral_8x7b_params_billion"]
    assert abs(tmx / 1e9 - val) <= tol
    assert len(synth.tensor_list(synth.LLAMA3_8B)) == 291
    assert len(synth.tensor_list(synth.LLAMA3_70B)) == 723
    assert len(synth.tensor_list(synth.MIXTRAL_8X7B)) == 995
    # one-of-8 shards are not aligned to tensor rows
    for t, s in ((t8, 1_003_782_656), (t70, 8_819_213_312), (tmx, 5_837_849_088)):
        _, shard, total = layout.flat_layout([t], 8, 1)
        assert shard == s and s % 4096 != 0


def test_host_and_device_hash_agree_on_cpu():
    torch = pytest.importorskip("torch")
    for start in (0, 12345, (1 << 33) + 7, 46_702_792_704 - 100):
        a = synth.host_index_hash16(start, 1000)
        b = synth.device_index_hash16_values(start, 1000, "cpu").numpy().view(np.uint16)
        assert np.array_equal(a, b)
    assert len(np.unique(synth.host_index_hash16(0, 1 << 16))) > 40000


# ---- per-tensor even partition (the paper's literal layout) ---------------------------

@pytest.mark.parametrize("align", [1, 8])
@pytest.mark.parametrize("numels", [[1, 3, 7, 4097], [16, 64, 8], [5], [0, 9, 0, 2], [1000, 24, 333]])
def test_per_tensor_round_trip_and_ownership(numels, align):
    W = 8
    rng = np.random.default_rng(sum(numels) + align)
    tensors = [rng.integers(1, 1 << 16, size=n, dtype=np.uint16) for n in numels]   # never 0
    gathered = layout.per_tensor_gather(tensors, W, align)
    sizes, offs, L = layout.per_tensor_slices(numels, W, align)
    assert gathered.size == W * L
    assert all(s % align == 0 and s * W >= n and (s - align) * W < max(n, 1) + align * W
               for s, n in zip(sizes, numels))
    # every real element appears exactly once; everything else is zero padding
    assert np.count_nonzero(gathered) == sum(numels)
    # brute force ownership: element i of tensor t sits in rank i // s_t at o_t + i % s_t
    for t, (n, s, o) in enumerate(zip(numels, sizes, offs)):
        for i in (0, n // 3, n - 1):
            if n:
                assert gathered[(i // s) * L + o + i % s] == tensors[t][i]
    outs = oracle.unshard_per_tensor(gathered, numels, W, align)
    for a, b in zip(tensors, outs):
        assert np.array_equal(a, b)
    # segments never read padding and cover each tensor exactly once, in order
    segs, _ = layout.per_tensor_segments(numels, W, align)
    for t, n in enumerate(numels):
        mine = sorted((d, k) for tt, _s, d, k in segs if tt == t)
        pos = 0
        for d, k in mine:
            assert d == pos and k > 0
            pos += k
        assert pos == n


def test_per_tensor_divisible_case_is_a_reshape():
    # when W divides every tensor the layout is numpy's reshape: a library routine
    W = 8
    numels = [64, 8 * 13, 8 * 512]
    rng = np.random.default_rng(9)
    tensors = [rng.integers(0, 1 << 16, size=n, dtype=np.uint16) for n in numels]
    gathered = layout.per_tensor_gather(tensors, W, 1)
    want = np.concatenate([t.reshape(W, -1) for t in tensors], axis=1).reshape(-1)
    assert np.array_equal(gathered, want)
    assert [s for s in layout.per_tensor_slices(numels, W)[0]] == [n // W for n in numels]
