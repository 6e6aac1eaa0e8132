"""Product planner (C, host only) against the oracle planner: identical schedules."""
import numpy as np
import pytest

from oracle import planner as P
from paper_2504_09983_amd import zc
from tests.test_oracle_planner import random_case


def test_kind_codes_agree():
    assert (zc.OP_COMPUTE, zc.OP_OFFLOAD, zc.OP_SYNC_FREE, zc.OP_RELOAD, zc.OP_SYNC_RELOAD) == \
           (P.COMPUTE, P.OFFLOAD, P.SYNC_FREE, P.RELOAD, P.SYNC_RELOAD)


@pytest.mark.parametrize("seed", range(200))
def test_same_schedule_on_random_profiles(seed):
    p_mem, n_f, frags, M = random_case(np.random.default_rng(1000 + seed))
    assert zc.plan_adaptive_offload(p_mem, n_f, frags, M) == P.plan(p_mem, n_f, frags, M)


def test_hand_cases_and_large_numbers():
    assert zc.plan_adaptive_offload([10, 20, 50, 80, 60, 30], 4, [10] * 4, 100) == \
        P.plan([10, 20, 50, 80, 60, 30], 4, [10] * 4, 100)
    assert zc.plan_adaptive_offload([10, 20, 30, 95, 40], 2, [10, 10], 100) == \
        P.plan([10, 20, 30, 95, 40], 2, [10, 10], 100)
    GB = 1 << 30
    p_mem = [g * GB for g in (20, 60, 120, 180, 150, 90, 30)]
    frags = [2 * GB] * 48
    assert zc.plan_adaptive_offload(p_mem, 4, frags, 250 * GB) == P.plan(p_mem, 4, frags, 250 * GB)
    # a spike inside the forward pass: no reload before the backward pass starts
    assert zc.plan_adaptive_offload([10, 95, 20, 20, 20, 10], 4, [10, 10], 100) == \
        P.plan([10, 95, 20, 20, 20, 10], 4, [10, 10], 100)
    assert zc.plan_adaptive_offload([], 0, [], 5) == [] == P.plan([], 0, [], 5)
    assert zc.plan_adaptive_offload([1, 2], 1, [], 5) == [(0, 0), (0, 1)]


def test_errors():
    def status(*a):
        with pytest.raises(zc.ZcError) as ei:
            zc.plan_adaptive_offload(*a)
        return ei.value.status
    assert status([10, 200], 2, [10, 10], 100) == zc.ERR_UNSUPPORTED      # cannot fit
    with pytest.raises(ValueError):
        P.plan([10, 200], 2, [10, 10], 100)
    assert status([10, -1], 2, [10], 100) == zc.ERR_INVALID_ARG
    assert status([10, 20], 3, [10], 100) == zc.ERR_INVALID_ARG           # n_forward > n_ops
    assert status([10, 20], 1, [-5], 100) == zc.ERR_INVALID_ARG
    assert status([10, 20], 1, [5], -1) == zc.ERR_INVALID_ARG


def test_schedule_run_rejects_bad_schedules_without_a_gpu():
    # validation happens before any HIP call; a NULL context is refused first
    import ctypes
    L = zc.lib()
    ops = (zc.SchedOp * 1)(zc.SchedOp(0, 0))
    assert L.zc_schedule_run(None, ops, 1, None, 1, None, 0, 0, None) == zc.ERR_INVALID_ARG


# ---- proactive prefetching, Fuse, selective unsharding --------------------------------------

from tests.test_oracle_planner import SIZES, TIMES, random_prefetch_case


@pytest.mark.parametrize("seed", range(200))
def test_prefetch_same_schedule_on_random_profiles(seed):
    rng = np.random.default_rng(7000 + seed)
    is_ag, bag, p_mem, M, Mp = random_prefetch_case(rng)
    alpha = float(rng.choice([0.0, 1.2, 1.5, 2.5, 1e30]))
    sizes, times = [1, 16, 64, 256], [5.0, 6.0, 12.0, 40.0]
    want = P.plan_prefetch(is_ag, bag, p_mem, M, Mp, sizes, times, alpha)
    got = zc.plan_prefetch(is_ag, bag, p_mem, M, Mp, sizes, times, alpha)
    assert got == want


def test_prefetch_hand_case_and_errors():
    is_ag = [0, 1, 0, 1, 0, 1, 0]
    bag = [0, 30, 0, 30, 0, 30, 0]
    p_mem = [10, 10, 40, 20, 50, 30, 60]
    for M, Mp, alpha in ((1000, 1000, 1e30), (100, 1000, 1e30), (1000, 50, 1e30), (0, 1000, 1e30),
                         (1000, 1000, 0.0), (1000, 1000, 1.5)):
        assert zc.plan_prefetch(is_ag, bag, p_mem, M, Mp, SIZES, TIMES, alpha) == \
            P.plan_prefetch(is_ag, bag, p_mem, M, Mp, SIZES, TIMES, alpha)
    assert zc.plan_prefetch([], [], [], 10, 10, SIZES, TIMES, 1.5) == []
    for bad in (lambda: zc.plan_prefetch([1], [0], [5], 10, 10, SIZES, TIMES, 1.5),       # AG without size
                lambda: zc.plan_prefetch([0], [0], [-5], 10, 10, SIZES, TIMES, 1.5),
                lambda: zc.plan_prefetch([0], [0], [5], 10, 10, [4, 2], [1.0, 2.0], 1.5),  # table not increasing
                lambda: zc.plan_prefetch([0], [0], [5], 10, 10, [], [], 1.5),
                lambda: zc.plan_prefetch([0], [0], [5], 10, 10, SIZES, TIMES, -1.0)):
        with pytest.raises(zc.ZcError) as ei:
            bad()
        assert ei.value.status == zc.ERR_INVALID_ARG


@pytest.mark.parametrize("seed", range(100))
def test_select_unsharded_same_choice(seed):
    rng = np.random.default_rng(9000 + seed)
    bag = [int(x) for x in rng.integers(1, 1 << 24, int(rng.integers(0, 40)))]
    budget = int(rng.integers(0, sum(bag) + 2))
    assert zc.select_unsharded(bag, SIZES, TIMES, budget) == P.select_unsharded(bag, SIZES, TIMES, budget)


def test_select_unsharded_hand_cases():
    cases = [([200, 100, 150], [100, 200], [10.0, 20.0], 250),                        # equal ratios
             ([1 << 20, 1 << 16], [1 << 10, 1 << 16, 1 << 20], [20.0, 22.0, 400.0], 1 << 17),  # a misfit ranked first
             ([100, 7], SIZES, TIMES, 7), ([64, 64], SIZES, TIMES, 128), ([5], [8], [3.0], 5)]
    for bag, sizes, times, budget in cases:
        assert zc.select_unsharded(bag, sizes, times, budget) == P.select_unsharded(bag, sizes, times, budget)
    # Fuse tests each all-gather against the merged message built so far
    is_ag, bag = [1, 1, 1, 0], [1 << 18, 1 << 20, 1 << 22, 0]
    for alpha in (1.2, 1.5):
        assert zc.plan_prefetch(is_ag, bag, [0, 0, 0, 0], 1 << 40, 1 << 40, SIZES, TIMES, alpha) == \
            P.plan_prefetch(is_ag, bag, [0, 0, 0, 0], 1 << 40, 1 << 40, SIZES, TIMES, alpha)
    assert P.plan_prefetch(is_ag, bag, [0, 0, 0, 0], 1 << 40, 1 << 40, SIZES, TIMES, 1.2) == \
        [("allgather", [0, 1]), ("allgather", [2]), ("op", 3)]


def test_select_unsharded_on_model_shapes():
    from paper_2504_09983_amd import synth
    bag = [2 * n for n in synth.tensor_numels(synth.LLAMA3_8B)]           # bf16 buffers
    budget = 4 << 30
    got = zc.select_unsharded(bag, SIZES, TIMES, budget)
    assert got == P.select_unsharded(bag, SIZES, TIMES, budget)
    # the norm vectors (8 KiB each) come first: cheapest memory for the time saved
    assert all(bag[o] == 8192 for o in got[:65])
    assert sum(bag[o] for o in got) <= budget
