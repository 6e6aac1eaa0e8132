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
