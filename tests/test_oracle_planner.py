"""Pins for the oracle's adaptive-offloading planner (Algorithm 2 + backward reload):
a schedule worked out by hand, the memory bound, minimality of what is offloaded, and
'as late as possible' / 'as early as possible' placement checked by perturbing the plan."""
import numpy as np
import pytest

from oracle import planner as P

C, OFF, SF, RL, SR = P.COMPUTE, P.OFFLOAD, P.SYNC_FREE, P.RELOAD, P.SYNC_RELOAD


def test_hand_worked_schedule():
    # forward o0..o3 use 10, 20, 50, 80; backward o4, o5 use 60, 30; four fragments of 10; M = 100
    p_mem = [10, 20, 50, 80, 60, 30]
    S = P.plan(p_mem, 4, [10, 10, 10, 10], 100)
    # peak 80 + 40 = 120 > 100: the first two fragments leave; they are freed only when o3
    # would overflow (80 + 40 - 20 = 100 fits); both fit back right at the start of backward
    assert S == [(OFF, 0), (OFF, 1), (C, 0), (C, 1), (C, 2), (SF, 0), (SF, 1), (C, 3),
                 (RL, 0), (RL, 1), (C, 4), (C, 5), (SR, 0), (SR, 1)]
    assert P.peak_memory(S, p_mem, [10, 10, 10, 10]) == 100


def test_nothing_to_do_when_everything_fits():
    p_mem = [5, 9, 7, 3]
    S = P.plan(p_mem, 2, [4, 4], 100)
    assert S == [(C, i) for i in range(4)]


def test_reload_waits_for_memory_to_fall():
    # backward usage stays high for two operators, then drops
    p_mem = [10, 90, 90, 85, 20, 10]
    frags = [10, 10, 10]
    S = P.plan(p_mem, 2, frags, 100)
    # peak 90 + 30 = 120: two fragments leave, freed before o1
    assert S[:5] == [(OFF, 0), (OFF, 1), (C, 0), (SF, 0), (SF, 1)]
    kinds = [k for k, _ in S]
    # no reload can start before o4 (tail max 90/85 + 10 resident + 10 > 100); o4 onwards is free
    assert S.index((RL, 0)) > S.index((C, 3)) and S.index((RL, 0)) < S.index((C, 4))
    assert kinds.count(RL) == 2 and S[-2:] == [(SR, 0), (SR, 1)]
    assert P.peak_memory(S, p_mem, frags) <= 100


def test_reload_looks_ahead_to_the_end_of_the_schedule():
    # backward usage dips to 50 and spikes again to 95: a reload started in the dip would
    # overflow at the spike, so both reloads wait until the spike has passed
    p_mem = [10, 95, 50, 95, 20]
    frags = [10, 10]
    S = P.plan(p_mem, 2, frags, 100)
    assert S == [(OFF, 0), (OFF, 1), (C, 0), (SF, 0), (SF, 1), (C, 1),
                 (C, 2), (C, 3), (RL, 0), (RL, 1), (C, 4), (SR, 0), (SR, 1)]
    assert P.peak_memory(S, p_mem, frags) == 95


def test_peak_in_the_backward_pass():
    # the spike (95) sits in the backward pass: the copies still start at the very beginning,
    # the memory is only taken away right before the spike, and comes back right after it
    p_mem = [10, 20, 30, 95, 40]
    frags = [10, 10]
    S = P.plan(p_mem, 2, frags, 100)
    assert S == [(OFF, 0), (OFF, 1), (C, 0), (C, 1), (C, 2), (SF, 0), (SF, 1), (C, 3),
                 (RL, 0), (RL, 1), (C, 4), (SR, 0), (SR, 1)]
    assert P.peak_memory(S, p_mem, frags) == 95


def test_does_not_fit_is_an_error():
    with pytest.raises(ValueError):
        P.plan([10, 200], 2, [10, 10], 100)


def random_case(rng):
    n_f = int(rng.integers(2, 30))
    n_b = int(rng.integers(2, 30))
    up = np.cumsum(rng.integers(0, 20, n_f)) + rng.integers(0, 30)
    down = up[-1] - np.cumsum(rng.integers(0, 20, n_b))
    down = np.maximum(down, 0)
    if rng.random() < 0.5:                      # a bump somewhere in the backward pass
        k = int(rng.integers(0, n_b))
        down[k] = min(int(up.max()), down[k] + int(rng.integers(0, 60)))
    p_mem = [int(x) for x in np.concatenate([up, down])]
    # spikes at the loss, as in the paper's memory-trend figure
    if rng.random() < 0.5:
        p_mem[n_f - 1] += int(rng.integers(0, 40))
    if rng.random() < 0.3:                      # ... or just after it, in the backward pass
        p_mem[n_f] += int(rng.integers(0, 60))
    frags = [int(x) for x in rng.integers(1, 25, int(rng.integers(1, 12)))]
    M = max(p_mem) + int(rng.integers(0, sum(frags) + 5))
    return p_mem, n_f, frags, M


@pytest.mark.parametrize("seed", range(40))
def test_invariants_on_random_profiles(seed):
    rng = np.random.default_rng(seed)
    p_mem, n_f, frags, M = random_case(rng)
    S = P.plan(p_mem, n_f, frags, M)
    # every operator exactly once and in order
    assert [i for k, i in S if k == C] == list(range(len(p_mem)))
    # the memory limit holds everywhere (replay also checks the ordering rules)
    assert P.peak_memory(S, p_mem, frags) <= M
    offloaded = [i for k, i in S if k == OFF]
    freed = [i for k, i in S if k == SF]
    # fragments leave in order, a prefix of OS, and what leaves is what is freed and returns
    assert offloaded == list(range(len(offloaded))) and freed == offloaded
    assert sorted(i for k, i in S if k == RL) == offloaded == sorted(i for k, i in S if k == SR)
    # minimal: one fragment fewer would not fit the forward peak
    need = max(p_mem) + sum(frags) - M
    got = sum(frags[i] for i in offloaded)
    assert got >= need and (not offloaded or got - frags[offloaded[-1]] < need)
    # all offload copies start before the first forward operator (maximum overlap)
    first_compute = S.index((C, 0))
    assert all(S.index((OFF, i)) < first_compute for i in offloaded)


@pytest.mark.parametrize("seed", range(40, 70))
def test_placement_is_tight(seed):
    """Each free is as late as the limit allows, each reload as early as it allows."""
    rng = np.random.default_rng(seed)
    p_mem, n_f, frags, M = random_case(rng)
    S = P.plan(p_mem, n_f, frags, M)
    for pos, (k, i) in enumerate(S):
        if k == SF:
            # push this free (and the frees after it in the same run) behind the next operator
            nxt = next(q for q in range(pos, len(S)) if S[q][0] == C)
            later = S[:pos] + [S[nxt]] + S[pos:nxt] + S[nxt + 1:]
            assert P.peak_memory(later, p_mem, frags) > M, "a free could have waited"
        if k == RL:
            prev = [q for q in range(pos) if S[q][0] == C]
            if not prev or S[prev[-1]][1] < n_f:
                continue                      # already at the start of the backward pass
            if any(S[q2][0] == SF for q2 in range(prev[-1], pos)):
                continue                      # freed only just now: it cannot return any earlier
            q = prev[-1]
            # move this reload, together with the reloads before it in the same run, one operator up
            run_start = q + 1
            earlier = S[:q] + S[run_start:pos + 1] + [S[q]] + S[pos + 1:]
            assert P.peak_memory(earlier, p_mem, frags) > M, "a reload could have started earlier"


def test_offload_all_sync_mode():
    S = P.plan_offload_all_sync(5, 3)
    assert P.peak_memory(S, [10, 20, 30, 20, 10], [7, 7, 7]) == 30
    assert [k for k, _ in S[:6]] == [OFF] * 3 + [SF] * 3 and [k for k, _ in S[-6:]] == [RL] * 3 + [SR] * 3
