"""CPU-side checks of the C-ABI library: it loads, exports what the header
declares, rejects bad arguments before touching a GPU, and its host-only layout
helper agrees with the oracle's layout."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle.layout as olayout
from paper_2504_09983_amd import synth, zc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "zc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(zc_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_loads_and_exports_every_declared_symbol():
    L = zc.lib()
    names = declared_functions()
    assert {"zc_adam_step", "zc_cast_bf16", "zc_unshard", "zc_offload_adam_step",
            "zc_unshard_plan_create", "zc_unshard_plan_destroy", "zc_offload_create",
            "zc_offload_destroy", "zc_grad_sqnorm", "zc_flat_layout", "zc_last_error",
            "zc_version", "zc_tune_set", "zc_tune_get", "zc_per_tensor_layout", "zc_host_alloc",
            "zc_host_free", "zc_offload_probe_link", "zc_grad_accumulate", "zc_adam_step_groups",
            "zc_clip_scale", "zc_plan_adaptive_offload", "zc_plan_prefetch", "zc_select_unsharded",
            "zc_schedule_run"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert zc.version() == 20100


def test_hparams_struct_layout_matches_header():
    # float x6, int64, int32 x2 -> 40 bytes with the int64 at offset 24
    assert ctypes.sizeof(zc.AdamHparams) == 40
    assert zc.AdamHparams.step.offset == 24 and zc.AdamHparams.mode.offset == 32
    assert ctypes.sizeof(zc.Segment) == 24


HP = dict(lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def _status(fn, *a, **k):
    with pytest.raises(zc.ZcError) as ei:
        fn(*a, **k)
    return ei.value.status


def test_adam_step_rejects_bad_arguments_without_a_gpu():
    hp = zc.hparams(step=1, **HP)
    A = 0x10000  # fake, never dereferenced: validation fails first
    assert _status(zc.adam_step, A, A + 64, A + 128, A + 192, zc.F32, -1, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step, 0, A + 64, A + 128, A + 192, zc.F32, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step, A, A + 64, A + 128, 0, zc.F32, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step, A + 2, A + 64, A + 128, A + 192, zc.F32, 8, hp, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.adam_step, A, A + 64, A + 128, A + 193, zc.BF16, 8, hp, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.adam_step, A, A + 64, A + 128, A + 192, zc.F32, 8, hp, bf16_out=A + 257, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.adam_step, A, A, A + 128, A + 192, zc.F32, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    # partial overlaps, not only equal pointers: m starts inside p; bf16_out ends inside g
    assert _status(zc.adam_step, A, A + 16, A + 128, A + 192, zc.F32, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step, A, A + 64, A + 128, A + 192, zc.F32, 8, hp, bf16_out=A + 180, stream=0) == zc.ERR_INVALID_ARG
    assert "overlap" in zc.last_error()
    assert _status(zc.adam_step, A, A + 64, A + 128, A + 192, 7, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step, A, A + 64, A + 128, A + 192, zc.F32, (1 << 40) + 1, hp, stream=0) == zc.ERR_UNSUPPORTED
    for bad in (dict(step=0), dict(beta1=1.0), dict(beta2=-0.1), dict(eps=-1.0),
                dict(lr=float("nan")), dict(mode=3), dict(grad_scale=float("inf")),
                dict(weight_decay=float("nan"))):
        kw = dict(HP, step=1)
        kw.update(bad)
        assert _status(zc.adam_step, A, A + 64, A + 128, A + 192, zc.F32, 8, zc.hparams(**kw), stream=0) == zc.ERR_INVALID_ARG
    assert "mode" in zc.last_error() or "weight_decay" in zc.last_error()
    # n == 0 is a no-op even with NULL pointers
    zc.adam_step(0, 0, 0, 0, zc.F32, 0, hp, stream=0)
    # per-range step: ranges must be sorted, disjoint and inside [0, n)
    ok = (A, A + 64, A + 128, A + 192, zc.F32, 8, hp)
    for bad in ([(4, 2, 1.0, 0.0)], [(0, 9, 1.0, 0.0)], [(0, 4, 1.0, 0.0), (3, 6, 1.0, 0.0)],
                [(0, 4, float("nan"), 0.0)], [(-1, 4, 1.0, 0.0)]):
        assert _status(zc.adam_step_groups, *ok, ranges=bad, stream=0) == zc.ERR_INVALID_ARG
    big_lr = (A, A + 64, A + 128, A + 192, zc.F32, 8, zc.hparams(step=1, **dict(HP, lr=1e10)))
    assert _status(zc.adam_step_groups, *big_lr, ranges=[(0, 4, 3e38, 0.0)], stream=0) == zc.ERR_INVALID_ARG   # lr * scale overflows
    assert _status(zc.adam_step_groups, *ok, grad_scale_dev=A + 1, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.clip_scale, 0, 1.0, 1.0, A, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.clip_scale, A, -1.0, 1.0, A + 4, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.clip_scale, A, 1.0, 0.0, A + 4, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.clip_scale, A + 2, 1.0, 1.0, A + 4, stream=0) == zc.ERR_ALIGNMENT


def test_packed_state_entry_points_reject_bad_arguments_without_a_gpu():
    hp = zc.hparams(step=1, **HP)
    G = zc.PACKED_GRANULE
    assert G == 8192
    for n in (-5, 0, 1, G - 1, G, G + 1, 7 * G + 3, 8_819_213_312):
        assert zc.packed_state_numel(n) == olayout.packed_state_numel(n, G)
    A = 0x400000                                  # fake, never dereferenced: validation fails first
    far = A + 4 * zc.packed_state_numel(8) + 4096
    ok = (A, far, zc.F32, 8, hp)
    assert _status(zc.adam_step_packed, A, far, zc.F32, -1, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step_packed, 0, far, zc.F32, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step_packed, A, 0, zc.F32, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step_packed, A + 64, far, zc.F32, 8, hp, stream=0) == zc.ERR_ALIGNMENT      # state off a 128-byte line
    assert _status(zc.adam_step_packed, A, far + 2, zc.F32, 8, hp, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.adam_step_packed, *ok, bf16_out=far + 4097, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.adam_step_packed, *ok, skip_flag=far + 8194, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.adam_step_packed, *ok, grad_scale_dev=far + 8193, stream=0) == zc.ERR_ALIGNMENT
    # the whole packed array counts, padding included: g just behind element 8 of p is still inside it
    assert _status(zc.adam_step_packed, A, A + 4 * 8, zc.F32, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step_packed, A, A + 4 * 3 * G - 4, zc.F32, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert "overlap" in zc.last_error()
    assert _status(zc.adam_step_packed, *ok, bf16_out=far + 8, stream=0) == zc.ERR_INVALID_ARG        # copy inside g
    assert _status(zc.adam_step_packed, A, far, 9, 8, hp, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.adam_step_packed, A, far, zc.F32, (1 << 40) + 1, hp, stream=0) == zc.ERR_UNSUPPORTED
    assert _status(zc.adam_step_packed, A, far, zc.F32, 8, zc.hparams(**dict(HP, step=0)), stream=0) == zc.ERR_INVALID_ARG
    for bad in ([(4, 2, 1.0, 0.0)], [(0, 9, 1.0, 0.0)], [(0, 4, 1.0, 0.0), (3, 6, 1.0, 0.0)],
                [(0, 4, 1.0, float("inf"))]):
        assert _status(zc.adam_step_packed, *ok, ranges=bad, stream=0) == zc.ERR_INVALID_ARG
    zc.adam_step_packed(0, 0, zc.F32, 0, hp, stream=0)                                                # n == 0: no-op
    # pack / unpack
    src = far + (1 << 20)
    assert _status(zc.state_pack, src, None, None, -1, A, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.state_pack, src, None, None, 8, 0, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.state_pack, src, None, None, 8, A + 16, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.state_pack, src + 2, None, None, 8, A, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.state_pack, A + 4 * G, None, None, 8, A, stream=0) == zc.ERR_INVALID_ARG          # source inside the array
    assert _status(zc.state_pack, src, src + 16, None, 8, A, stream=0) == zc.ERR_INVALID_ARG           # sources overlap
    assert _status(zc.state_pack, src, None, None, (1 << 40) + 1, A, stream=0) == zc.ERR_UNSUPPORTED
    assert _status(zc.state_unpack, A, 8, src, None, src + 8, stream=0) == zc.ERR_INVALID_ARG          # p and v overlap
    assert _status(zc.state_unpack, A + 4, 8, src, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.state_unpack, 0, 8, src, stream=0) == zc.ERR_INVALID_ARG
    zc.state_pack(0, 0, 0, 0, 0, stream=0)
    zc.state_unpack(0, 0, stream=0)
    zc.state_unpack(A, 8, stream=0)                                                                   # nothing asked for


def test_cast_and_sqnorm_reject_bad_arguments_without_a_gpu():
    A = 0x20000
    assert _status(zc.cast_bf16, A, A + 4096, -5, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.cast_bf16, 0, A, 4, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.cast_bf16, A + 1, A + 4096, 4, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.cast_bf16, A, A + 4097, 4, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.cast_bf16, A, A + 8, 16, stream=0) == zc.ERR_INVALID_ARG   # overlap
    zc.cast_bf16(0, 0, 0, stream=0)
    assert _status(zc.grad_accumulate, A, A + 4096, zc.BF16, -1, 1.0, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.grad_accumulate, 0, A + 4096, zc.BF16, 4, 1.0, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.grad_accumulate, A, A, zc.F32, 4, 1.0, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.grad_accumulate, A + 2, A + 4096, zc.F32, 4, 1.0, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.grad_accumulate, A, A + 4097, zc.BF16, 4, 1.0, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.grad_accumulate, A, A + 4096, zc.BF16, 4, float("inf"), stream=0) == zc.ERR_INVALID_ARG
    zc.grad_accumulate(0, 0, zc.F32, 0, 1.0, stream=0)
    assert _status(zc.grad_sqnorm, A, zc.BF16, -1, A + 64, A + 68, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.grad_sqnorm, A, zc.BF16, 4, 0, A + 68, stream=0) == zc.ERR_INVALID_ARG
    assert _status(zc.grad_sqnorm, A + 1, zc.BF16, 4, A + 64, A + 68, stream=0) == zc.ERR_ALIGNMENT
    assert _status(zc.grad_sqnorm, 0, zc.F32, 4, A + 64, A + 68, stream=0) == zc.ERR_INVALID_ARG


def test_unshard_plan_and_offload_reject_bad_arguments_without_a_gpu():
    A = 0x30000
    assert _status(zc.UnshardPlan, [(-1, A, 4)], 100) == zc.ERR_INVALID_ARG
    assert _status(zc.UnshardPlan, [(98, A, 4)], 100) == zc.ERR_INVALID_ARG
    assert _status(zc.UnshardPlan, [(0, A, -4)], 100) == zc.ERR_INVALID_ARG
    assert _status(zc.UnshardPlan, [(0, 0, 4)], 100) == zc.ERR_INVALID_ARG
    assert _status(zc.UnshardPlan, [(0, A + 1, 4)], 100) == zc.ERR_ALIGNMENT
    assert _status(zc.UnshardPlan, [(0, A, 4)], -1) == zc.ERR_INVALID_ARG
    assert "segment" in zc.last_error() or "gathered" in zc.last_error()
    # destinations that share bytes are refused, whatever the order they come in; touching is fine
    assert _status(zc.UnshardPlan, [(0, A, 8), (8, A + 14, 8)], 100) == zc.ERR_INVALID_ARG
    assert "overlap" in zc.last_error()
    assert _status(zc.UnshardPlan, [(8, A + 64, 8), (0, A, 40)], 100) == zc.ERR_INVALID_ARG
    assert _status(zc.UnshardPlan, [(0, A, 8), (8, A, 8)], 100) == zc.ERR_INVALID_ARG
    assert _status(zc.OffloadCtx, 1000, 3) == zc.ERR_INVALID_ARG
    assert _status(zc.OffloadCtx, 1 << 20, 0) == zc.ERR_INVALID_ARG
    assert _status(zc.OffloadCtx, 1 << 20, 9) == zc.ERR_INVALID_ARG
    assert _status(zc.OffloadCtx, 0, 3) == zc.ERR_INVALID_ARG


def test_tune_knobs():
    old = zc.tune_get("adam.rows")
    zc.tune_set("adam.rows", 4)
    assert zc.tune_get("adam.rows") == 4
    assert _status(zc.tune_set, "adam.rows", 3) == zc.ERR_INVALID_ARG
    assert _status(zc.tune_set, "adam.rows", 9) == zc.ERR_INVALID_ARG
    assert _status(zc.tune_set, "adam.block", 96) == zc.ERR_INVALID_ARG
    assert _status(zc.tune_set, "adam.block", 512) == zc.ERR_INVALID_ARG
    assert _status(zc.tune_set, "no.such.key", 1) == zc.ERR_INVALID_ARG
    assert _status(zc.tune_get, "no.such.key") == zc.ERR_INVALID_ARG
    zc.tune_set("adam.rows", old)


def test_tune_knobs_belong_to_the_calling_thread():
    """A knob set on one thread is invisible to every other thread: a sweep running beside
    production launches cannot change their kernels."""
    import threading
    default = zc.tune_get("adam.block")
    seen = {}

    def other():
        seen["before"] = zc.tune_get("adam.block")
        zc.tune_set("adam.block", 64 if default != 64 else 256)
        seen["after"] = zc.tune_get("adam.block")

    t = threading.Thread(target=other)
    t.start()
    t.join()
    assert seen["before"] == default and seen["after"] != default
    assert zc.tune_get("adam.block") == default            # this thread saw nothing
    zc.tune_set("adam.block", 256 if default != 256 else 64)
    t = threading.Thread(target=lambda: seen.__setitem__("fresh", zc.tune_get("adam.block")))
    t.start()
    t.join()
    assert seen["fresh"] == default                         # a new thread starts from the defaults
    zc.tune_set("adam.block", default)


@pytest.mark.parametrize("align", [1, 8, 4096])
def test_flat_layout_matches_oracle_layout(align):
    for numels in ([1, 3, 7, 4097], [0, 9, 0, 2], [], [4096] * 5 + [17],
                   synth.tensor_numels(synth.LLAMA3_8B), synth.tensor_numels(synth.MIXTRAL_8X7B),
                   synth.tensor_numels(synth.LLAMA3_70B)):
        offs, shard, total = zc.flat_layout(numels, 8, align)
        o_offs, o_shard, o_total = olayout.flat_layout(numels, 8, align)
        assert offs == list(o_offs) and shard == o_shard and total == o_total


@pytest.mark.parametrize("align", [1, 8, 64])
def test_per_tensor_layout_matches_oracle_layout(align):
    for numels in ([1, 3, 7, 4097], [0, 9, 0, 2], [], [16, 64, 8], [1000, 24, 333],
                   synth.tensor_numels(synth.MIXTRAL_8X7B)):
        segs, send = zc.per_tensor_layout(numels, 8, align)
        o_segs, o_send = olayout.per_tensor_segments(numels, 8, align)
        assert send == o_send
        assert len(segs) == 8 * len(numels)
        assert [s for s in segs if s[3] > 0] == [tuple(int(x) for x in s) for s in o_segs]
        assert all(s[3] == 0 or s[3] > 0 for s in segs)
    assert _status(zc.per_tensor_layout, [4, -1], 8, 1) == zc.ERR_INVALID_ARG
    assert _status(zc.per_tensor_layout, [4], 0, 1) == zc.ERR_INVALID_ARG
    assert _status(zc.per_tensor_layout, [4], 8, 0) == zc.ERR_INVALID_ARG
    assert _status(zc.per_tensor_layout, [1 << 47], 8, 1) == zc.ERR_UNSUPPORTED


def test_flat_layout_rejects_bad_input():
    assert _status(zc.flat_layout, [4, -1], 8, 1) == zc.ERR_INVALID_ARG
    assert _status(zc.flat_layout, [4], 0, 1) == zc.ERR_INVALID_ARG
    assert _status(zc.flat_layout, [4], 8, 0) == zc.ERR_INVALID_ARG
    assert _status(zc.flat_layout, [1 << 45, 1 << 45, 1 << 45], 8, 1) == zc.ERR_UNSUPPORTED


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2504_09983_amd")
    for dirpath, _dirs, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "zc_oracle" not in text and "zco_" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2504_09983_amd" not in text and "zc.h" not in text, f
