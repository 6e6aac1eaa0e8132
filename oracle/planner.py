"""Host-side planners of the paper, as plain Python: when optimizer-state fragments leave
and return (Adaptive offloading), where all-gathers are hoisted to and which of them are
merged (Proactive prefetching), which gathered parameters stay unsharded (Selective
unsharding).

TEST INFRASTRUCTURE (part of the CPU oracle).  Each function states the behaviour the paper
describes and computes it directly; the readings taken where the paper leaves a choice open
are listed with each function.

Inputs are profiles: `usage[i]` is the device memory in use right before operator i with the
optimizer states left out, `fragment_bytes[f]` the size of optimizer-state fragment f,
`buffer_bytes[i]` the size of the buffer all-gather i fills, and a table of measured
communication times by message size.
"""
from __future__ import annotations

from bisect import bisect_left
from collections import deque

COMPUTE, OFFLOAD, SYNC_FREE, RELOAD, SYNC_RELOAD = range(5)
KIND_NAMES = ("compute", "offload", "sync_free", "reload", "sync_reload")


def plan(usage, n_forward, fragment_bytes, limit):
    """Adaptive offloading over one iteration (paper: Adaptive offloading, Algorithm 2, and the
    paragraph on the backward pass after it).  Operators [0, n_forward) are the forward pass,
    the rest the backward pass.  Returns the schedule as a list of (kind, index).

    What the paper asks for: move out only as much optimizer state as the memory peak needs;
    start those copies at the very beginning so that they overlap the forward pass; take a
    fragment's memory away (after waiting for its copy) only when an operator would not fit
    otherwise; in the backward pass bring fragments back as soon as there is room; have
    everything back before the update.

    Readings: the peak is taken over the whole iteration (the paper's memory-trend figure has
    its spikes in the backward pass), so memory may still have to be taken away there;
    fragments leave, are released and return in list order; "room" for a reload means that the
    largest usage from that operator to the end of the iteration still fits once the fragment
    is back; fragments that found no room are reloaded after the last operator; every reload
    is waited for at the end.
    """
    usage = list(usage)
    sizes = list(fragment_bytes)
    n_ops = len(usage)
    state_bytes = sum(sizes)
    # missing[i]: optimizer-state bytes that must be off the device while operator i runs
    missing = [u + state_bytes - limit for u in usage]
    worst = (max(usage) if usage else 0) + state_bytes - limit

    # Which fragments leave: the shortest prefix of the list whose total covers the worst operator.
    leaving, covered = [], 0
    for f, b in enumerate(sizes):
        if covered >= worst:
            break
        leaving.append(f)
        covered += b
    schedule = [(OFFLOAD, f) for f in leaving]

    # missing_ahead[i]: the largest `missing` from operator i to the end
    missing_ahead = [0] * (n_ops + 1)
    for i in reversed(range(n_ops)):
        missing_ahead[i] = max(missing[i], missing_ahead[i + 1])

    copying_out = deque(leaving)     # copy started, memory still held
    away = deque()                   # memory released, copy back not started
    coming_back = []                 # copy back started
    absent = 0                       # bytes of `away`
    for i in range(n_ops):
        while missing[i] > absent:                       # operator i does not fit yet
            if not copying_out:
                raise ValueError("the schedule does not fit even with every fragment offloaded")
            f = copying_out.popleft()
            schedule.append((SYNC_FREE, f))
            absent += sizes[f]
            away.append(f)
        if i >= n_forward:
            while away and missing_ahead[i] <= absent - sizes[away[0]]:   # fits from here to the end
                f = away.popleft()
                schedule.append((RELOAD, f))
                absent -= sizes[f]
                coming_back.append(f)
        schedule.append((COMPUTE, i))
    for f in away:
        schedule.append((RELOAD, f))
        coming_back.append(f)
    schedule.extend((SYNC_RELOAD, f) for f in coming_back)
    return schedule


def plan_offload_all_sync(n_ops, nfrags):
    """The comparison mode of the paper's evaluation (Evaluation, Adaptive Offloading):
    everything is offloaded and waited for before the forward pass and reloaded
    synchronously at the end."""
    head = [(OFFLOAD, f) for f in range(nfrags)] + [(SYNC_FREE, f) for f in range(nfrags)]
    body = [(COMPUTE, i) for i in range(n_ops)]
    tail = [(RELOAD, f) for f in range(nfrags)] + [(SYNC_RELOAD, f) for f in range(nfrags)]
    return head + body + tail


def peak_memory(schedule, usage, fragment_bytes):
    """Replay a schedule: largest (profiled usage + resident optimizer bytes) seen before
    any compute operator, counting a fragment as resident from the moment its reload starts
    until its memory is freed.  Also checks the ordering rules; returns the peak."""
    resident = sum(fragment_bytes)
    state = ["resident"] * len(fragment_bytes)
    peak = 0
    for kind, idx in schedule:
        if kind == OFFLOAD:
            assert state[idx] == "resident", "offload of a fragment that is not resident"
            state[idx] = "copying_out"
        elif kind == SYNC_FREE:
            assert state[idx] == "copying_out", "free before the offload copy was started"
            state[idx] = "host"
            resident -= fragment_bytes[idx]
        elif kind == RELOAD:
            assert state[idx] == "host", "reload of a fragment that is not on the host"
            state[idx] = "copying_in"
            resident += fragment_bytes[idx]
        elif kind == SYNC_RELOAD:
            assert state[idx] == "copying_in", "wait for a reload that was never started"
            state[idx] = "resident"
        else:
            peak = max(peak, usage[idx] + resident)
    assert all(s in ("resident", "copying_out") for s in state), "a fragment is missing at the update"
    return peak


def t_c(nbytes, sizes, times):
    """Communication time of a message of `nbytes` from the profiled (sizes, times) table
    (paper: Proactive prefetching, T_c).  Reading: straight lines between neighbouring
    samples, the first sample's time for anything smaller, the last segment's slope continued
    for anything larger."""
    if nbytes <= sizes[0] or len(sizes) == 1:
        return times[0]
    hi = min(bisect_left(sizes, nbytes), len(sizes) - 1)    # first sample >= nbytes, else the last
    lo = hi - 1
    # the line through the two samples, in its two-point form
    return times[lo] + (times[hi] - times[lo]) * (nbytes - sizes[lo]) / (sizes[hi] - sizes[lo])


def fuse(gathers, buffer_bytes, sizes, times, alpha):
    """Merge neighbouring all-gathers of a prefetch group while one message is cheaper than
    two (paper: Proactive prefetching, Fuse: merge when the separate times together exceed
    alpha times the time of the merged message).  Reading: the group is walked in schedule
    order and each all-gather is tested against the merged message built so far.
    Returns a list of lists of operator indices, in schedule order."""
    merged = []          # [[indices], bytes]
    for o in gathers:
        b = buffer_bytes[o]
        if merged:
            have = merged[-1][1]
            apart = t_c(have, sizes, times) + t_c(b, sizes, times)
            if apart > alpha * t_c(have + b, sizes, times):
                merged[-1][0].append(o)
                merged[-1][1] = have + b
                continue
        merged.append([[o], b])
    return [members for members, _ in merged]


def plan_prefetch(is_allgather, buffer_bytes, usage, limit, group_limit, sizes, times, alpha):
    """Proactive prefetching (paper: Proactive prefetching, Algorithm 1).  Returns the new
    schedule as a list of ("op", i) and ("allgather", [i, j, ...]) entries.

    What the paper asks for: starting from the end of the schedule, let every all-gather
    travel towards the front together with the all-gathers met so far, for as long as the
    memory in use before the operator in front of it plus the travelling buffers stays below
    the limit and the travelling buffers stay below the group limit; where that stops, the
    travelling group is put down (and fused); nothing else changes its order.

    Readings: the all-gather at which a group is put down starts the next group when it fits
    by itself, otherwise it stays where it was; the first operator of the schedule has nothing
    in front of it, so an all-gather there joins the travelling group unless the group limit
    forbids, in which case the group is put down right behind it.
    """
    n = len(is_allgather)
    put_behind = {}      # operator index (-1: the very front) -> all-gathers put down right behind it
    stays = set()        # all-gathers that do not move
    travelling = []      # indices, latest first

    def put_down(behind):
        if travelling:
            put_behind[behind] = sorted(travelling)
            travelling.clear()

    for i in range(n - 1, 0, -1):
        if not is_allgather[i]:
            continue
        carried = sum(buffer_bytes[o] for o in travelling) + buffer_bytes[i]
        if usage[i - 1] + carried < limit and carried < group_limit:
            travelling.append(i)
            continue
        put_down(i)
        if usage[i - 1] + buffer_bytes[i] < limit and buffer_bytes[i] < group_limit:
            travelling.append(i)
        else:
            stays.add(i)
    if n:
        if not is_allgather[0]:
            put_down(0)
        else:
            if sum(buffer_bytes[o] for o in travelling) + buffer_bytes[0] >= group_limit:
                put_down(0)
            travelling.append(0)
    put_down(-1)

    schedule = []

    def emit_groups(behind):
        for members in fuse(put_behind.get(behind, []), buffer_bytes, sizes, times, alpha):
            schedule.append(("allgather", members))

    emit_groups(-1)
    for i in range(n):
        if not is_allgather[i]:
            schedule.append(("op", i))
        elif i in stays:
            schedule.append(("allgather", [i]))
        emit_groups(i)
    return schedule


def select_unsharded(buffer_bytes, sizes, times, budget):
    """Selective unsharding (paper: Selective unsharding): which gathered parameters to keep
    until the update, within `budget` bytes.  Candidates are ranked by communication time
    saved per byte kept, highest first; reading: among equal ratios the smaller buffer goes
    first, then the earlier one, and every candidate that still fits is taken (a large one
    that does not fit does not stop smaller ones after it).  Returns the indices in the order
    chosen."""
    def saving_per_byte(o):
        return t_c(buffer_bytes[o], sizes, times) / buffer_bytes[o]

    ranked = sorted(range(len(buffer_bytes)), key=lambda o: (-saving_per_byte(o), buffer_bytes[o], o))
    kept, room = [], budget
    for o in ranked:
        if buffer_bytes[o] <= room:
            kept.append(o)
            room -= buffer_bytes[o]
    return kept
