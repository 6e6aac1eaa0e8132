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


def test_no_reload_in_the_forward_pass():
    # the spike (95) sits inside the forward pass and usage is low right after it; fragments
    # come back in the backward pass only (the paper reloads there), i.e. before o4, not before o2
    p_mem = [10, 95, 20, 20, 20, 10]
    frags = [10, 10]
    S = P.plan(p_mem, 4, frags, 100)
    assert S == [(OFF, 0), (OFF, 1), (C, 0), (SF, 0), (SF, 1), (C, 1), (C, 2), (C, 3),
                 (RL, 0), (RL, 1), (C, 4), (C, 5), (SR, 0), (SR, 1)]


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


# ---- proactive prefetching, Fuse, selective unsharding ---------------------------------

SIZES = [1 << 10, 1 << 16, 1 << 20, 1 << 24, 1 << 28]
TIMES = [20.0, 22.0, 40.0, 300.0, 4000.0]            # microseconds: flat for small messages


def test_t_c_table():
    assert P.t_c(1, SIZES, TIMES) == 20.0 and P.t_c(1 << 10, SIZES, TIMES) == 20.0
    assert P.t_c(1 << 20, SIZES, TIMES) == 40.0
    mid = ((1 << 20) + (1 << 24)) // 2
    assert abs(P.t_c(mid, SIZES, TIMES) - 170.0) < 1e-9
    # beyond the table: the last slope continues
    assert abs(P.t_c(1 << 29, SIZES, TIMES) - (4000.0 + 3700.0 * (1 << 28) / ((1 << 28) - (1 << 24)))) < 1e-6
    vals = [P.t_c(v, SIZES, TIMES) for v in range(1, 1 << 22, 4099)]
    assert all(b >= a for a, b in zip(vals, vals[1:]))


def test_fuse_merges_small_messages_only():
    bag = {0: 4096, 1: 4096, 2: 4096, 3: 1 << 27, 4: 1 << 27, 5: 2048}
    # small ones: 20 + 20 > 1.5 * ~20 -> fused; large ones: 2*T(2^27) vs 1.5*T(2^28): not fused
    groups = P.fuse([0, 1, 2, 3, 4, 5], bag, SIZES, TIMES, 1.5)
    assert groups[0] == [0, 1, 2]
    assert [3] in groups and all(not (3 in g and 4 in g) for g in groups)
    assert [x for g in groups for x in g] == [0, 1, 2, 3, 4, 5]
    # the test is against the merged message built so far, not against its last member:
    # 256 KiB + 1 MiB merge (26.0 + 40.0 > 1.2 * 45.2); 4 MiB joins 1 MiB alone
    # (40.0 + 92.0 > 1.2 * 109.3) but not the 1.25 MiB message (45.2 + 92.0 < 1.2 * 114.4)
    sizes3 = {0: 1 << 18, 1: 1 << 20, 2: 1 << 22}
    assert P.fuse([0, 1, 2], sizes3, SIZES, TIMES, 1.2) == [[0, 1], [2]]
    assert P.fuse([1, 2], sizes3, SIZES, TIMES, 1.2) == [[1, 2]]
    # alpha = infinity never fuses, alpha = 0 always does
    assert P.fuse([0, 1, 2], bag, SIZES, TIMES, 1e30) == [[0], [1], [2]]
    assert P.fuse([0, 1, 5], bag, SIZES, TIMES, 0.0) == [[0, 1, 5]]


def test_prefetch_hand_worked():
    # o0 compute, o1 AG(a), o2 compute(a), o3 AG(b), o4 compute(b), o5 AG(c), o6 compute(c)
    is_ag = [0, 1, 0, 1, 0, 1, 0]
    bag = [0, 30, 0, 30, 0, 30, 0]
    p_mem = [10, 10, 40, 20, 50, 30, 60]
    big = 1e30                                       # never fuse: look at the placement only
    # plenty of memory: everything is hoisted to the front (after o0)
    S = P.plan_prefetch(is_ag, bag, p_mem, 1000, 1000, SIZES, TIMES, big)
    assert S == [("op", 0), ("allgather", [1]), ("allgather", [3]), ("allgather", [5]),
                 ("op", 2), ("op", 4), ("op", 6)]
    # M = 100: walking back, c fits before o4 (50+30 < 100); at o3, b and c together do not fit
    # before o2 (40+60 = 100), so c is placed there; b alone fits (70) and moves on; at o1, a and b
    # together fit before o0 (10+60 = 70): both go to the front
    S = P.plan_prefetch(is_ag, bag, p_mem, 100, 1000, SIZES, TIMES, big)
    assert S == [("op", 0), ("allgather", [1]), ("allgather", [3]), ("op", 2), ("allgather", [5]),
                 ("op", 4), ("op", 6)]
    # the group limit alone: at most one buffer per group (30 < 50 <= 60), so every all-gather
    # moves up past one compute operator only, until it meets the next all-gather
    for group_limit in (50, 60):                     # 60: two buffers reach the limit exactly, which is too much
        S = P.plan_prefetch(is_ag, bag, p_mem, 1000, group_limit, SIZES, TIMES, big)
        assert S == [("op", 0), ("allgather", [1]), ("allgather", [3]), ("op", 2), ("allgather", [5]),
                     ("op", 4), ("op", 6)]
    # 61 lets two travel together, not three: c and b go up to a, which stays in front of them
    S = P.plan_prefetch(is_ag, bag, p_mem, 1000, 61, SIZES, TIMES, big)
    assert S == [("op", 0), ("allgather", [1]), ("allgather", [3]), ("allgather", [5]), ("op", 2),
                 ("op", 4), ("op", 6)]
    # no memory at all: nothing moves
    S = P.plan_prefetch(is_ag, bag, p_mem, 0, 1000, SIZES, TIMES, big)
    assert S == [("op", 0), ("allgather", [1]), ("op", 2), ("allgather", [3]), ("op", 4),
                 ("allgather", [5]), ("op", 6)]


def random_prefetch_case(rng):
    layers = int(rng.integers(1, 15))
    is_ag, bag, p_mem = [], [], []
    mem = int(rng.integers(0, 50))
    for _ in range(layers):
        for _ in range(int(rng.integers(1, 3))):     # one or two parameters per layer
            is_ag.append(1); bag.append(int(rng.integers(1, 60))); p_mem.append(mem)
        for _ in range(int(rng.integers(1, 4))):
            mem += int(rng.integers(0, 25))
            is_ag.append(0); bag.append(0); p_mem.append(mem)
    M = int(rng.integers(20, max(p_mem) + 200))
    Mp = int(rng.integers(20, 300))
    return is_ag, bag, p_mem, M, Mp


@pytest.mark.parametrize("seed", range(60))
def test_prefetch_properties(seed):
    rng = np.random.default_rng(500 + seed)
    is_ag, bag, p_mem, M, Mp = random_prefetch_case(rng)
    alpha = float(rng.choice([0.0, 1.2, 1.5, 1e30]))
    table_sizes = [1, 16, 64, 256]
    table_times = [5.0, 6.0, 12.0, 40.0]
    S = P.plan_prefetch(is_ag, bag, p_mem, M, Mp, table_sizes, table_times, alpha)
    flat = []
    for kind, x in S:
        flat += x if kind == "allgather" else [x]
    # every operator exactly once
    assert sorted(flat) == list(range(len(is_ag)))
    # compute operators keep their order; all-gathers keep theirs
    assert [x for x in flat if not is_ag[x]] == [i for i in range(len(is_ag)) if not is_ag[i]]
    assert [x for x in flat if is_ag[x]] == [i for i in range(len(is_ag)) if is_ag[i]]
    # an all-gather is never later than it was: everything before it in S0's compute order that
    # used to follow it still follows it
    pos = {x: k for k, x in enumerate(flat)}
    for i in range(len(is_ag)):
        if is_ag[i]:
            assert all(pos[j] > pos[i] for j in range(i + 1, len(is_ag)) if not is_ag[j])
    # fused groups contain only all-gathers, adjacent in S0's all-gather order, and respect the cap
    for kind, x in S:
        if kind == "allgather" and len(x) > 1:
            assert all(is_ag[i] for i in x) and sum(bag[i] for i in x) < Mp
    # alpha = infinity: nothing is fused
    if alpha == 1e30:
        assert all(len(x) == 1 for kind, x in S if kind == "allgather")


def test_select_unsharded():
    bag = [1 << 12, 1 << 26, 1 << 14, 1 << 20, 1 << 12]
    # per-byte saving is largest for the smallest buffers
    chosen = P.select_unsharded(bag, SIZES, TIMES, (1 << 20) + (1 << 15))
    assert chosen[:3] == [0, 4, 2] and 1 not in chosen
    assert sum(bag[o] for o in chosen) <= (1 << 20) + (1 << 15)
    assert P.select_unsharded(bag, SIZES, TIMES, 0) == []
    assert sorted(P.select_unsharded(bag, SIZES, TIMES, 1 << 40)) == [0, 1, 2, 3, 4]
    # equal saving per byte (a table that is a line through the origin): smaller buffers first
    assert P.select_unsharded([200, 100, 150], [100, 200], [10.0, 20.0], 250) == [1, 2]
    # a table whose cost per byte rises (22 us for 64 KiB, 400 us for 1 MiB): the 1 MiB buffer
    # ranks first, does not fit, and must not stop the 64 KiB buffer behind it from being kept
    assert P.select_unsharded([1 << 20, 1 << 16], [1 << 10, 1 << 16, 1 << 20], [20.0, 22.0, 400.0], 1 << 17) == [1]
    # a candidate that fits exactly is taken
    assert P.select_unsharded([100, 7], SIZES, TIMES, 7) == [1]
    assert P.select_unsharded([64, 64], SIZES, TIMES, 128) == [0, 1]


def _select_by_repeated_argmax(b, sizes, times, budget):
    """The same choice written as its definition: again and again take, among the candidates
    not yet looked at, the one that saves the most communication time per byte (smaller
    buffer, then lower index, among equals); keep it if it still fits."""
    left, kept, room = set(range(len(b))), [], budget
    while left:
        best = None
        for o in sorted(left):
            r = P.t_c(b[o], sizes, times) / b[o]
            if best is None or r > best[0] or (r == best[0] and b[o] < b[best[1]]):
                best = (r, o)
        o = best[1]
        left.remove(o)
        if b[o] <= room:
            kept.append(o)
            room -= b[o]
    return kept


def test_select_unsharded_order_by_brute_force():
    rng = np.random.default_rng(3)
    for trial in range(200):
        k = int(rng.integers(1, 9))
        # sizes on both sides of the table's knees, with repeats so that equal ratios occur
        b = [int(x) for x in rng.choice([512, 1 << 10, 3000, 1 << 16, 1 << 18, 1 << 20, 5 << 20, 1 << 24], k)]
        budget = int(rng.integers(0, sum(b) + 2))
        ch = P.select_unsharded(b, SIZES, TIMES, budget)
        assert ch == _select_by_repeated_argmax(b, SIZES, TIMES, budget), (b, budget)
        used = sum(b[o] for o in ch)
        assert used <= budget and len(set(ch)) == len(ch)
        # chosen in non-increasing order of time saved per byte
        ratios = [P.t_c(b[o], SIZES, TIMES) / b[o] for o in ch]
        assert all(x >= y for x, y in zip(ratios, ratios[1:]))
        # an item left out did not fit at the moment its turn came: everything chosen with a
        # higher rank than it, plus the item, exceeds the budget
        rank = lambda o: (-P.t_c(b[o], SIZES, TIMES) / b[o], b[o], o)
        for o in range(k):
            if o not in ch:
                before = sum(b[c] for c in ch if rank(c) < rank(o))
                assert before + b[o] > budget, (b, budget, o)
