"""Adaptive offloading of optimizer-state fragments, written out step by step.

TEST INFRASTRUCTURE (part of the CPU oracle).  Plain Python in the paper's
notation: S0 / S (schedules), M (memory limit), P_mem(o) (profiled memory in
use before operator o, optimizer states not included), OS (fragments),
B_os(os) (fragment size), M_opt (total size of the optimizer states), M^-
(bytes freed so far).

Forward pass: Adaptive offloading, Algorithm 2.  Readings where the listing is
ambiguous: M_peak is taken over the whole iteration (the paper's memory-trend
figure puts the largest spikes in the backward pass), so the wait-and-free loop
also runs over the backward operators; the first loop walks the fragments in
order and stops adding as soon as the peak fits; "Pop" takes fragments in the
order they were offloaded (the copy started first finishes first).

Backward pass: the paragraph after Algorithm 2 — walk the backward operators;
wherever enough memory is free from that operator to the end of the schedule,
start the asynchronous copy back of the next fragment.  Reading: "enough" means
that the largest profiled usage from that operator on, plus the optimizer
bytes resident after the reload, stays within M; fragments return in the order
they left; whatever has not been started when the schedule ends is reloaded
there; every reload is waited for before the parameter update.
"""
from __future__ import annotations

COMPUTE, OFFLOAD, SYNC_FREE, RELOAD, SYNC_RELOAD = range(5)
KIND_NAMES = ("compute", "offload", "sync_free", "reload", "sync_reload")


def plan(p_mem, n_forward, frag_bytes, M):
    """Whole iteration: operators [0, n_forward) are the forward pass, the rest the
    backward pass.  Returns the new schedule S as a list of (kind, index)."""
    p_mem = list(p_mem)
    frag_bytes = list(frag_bytes)
    N = len(p_mem)
    S = []
    M_minus = 0
    M_peak = max(p_mem) if N else 0
    M_opt = sum(frag_bytes)
    OS_offload = []
    for i, b in enumerate(frag_bytes):
        if M_peak + M_opt - sum(frag_bytes[j] for j in OS_offload) > M:
            OS_offload.append(i)
            S.append((OFFLOAD, i))
    pending = list(OS_offload)      # copy started, memory not yet freed
    waiting = []                    # freed, reload not yet started
    started = []                    # reload started
    # largest profiled usage from operator i to the end of the schedule
    tail_max = [0] * (N + 1)
    for i in range(N - 1, -1, -1):
        tail_max[i] = max(p_mem[i], tail_max[i + 1])
    for i in range(N):
        while p_mem[i] + M_opt - M_minus > M:
            if not pending:
                raise ValueError("the schedule does not fit even with every fragment offloaded")
            os_i = pending.pop(0)
            S.append((SYNC_FREE, os_i))
            M_minus += frag_bytes[os_i]
            waiting.append(os_i)
        if i >= n_forward:
            while waiting and tail_max[i] + M_opt - M_minus + frag_bytes[waiting[0]] <= M:
                f = waiting.pop(0)
                S.append((RELOAD, f))
                M_minus -= frag_bytes[f]
                started.append(f)
        S.append((COMPUTE, i))
    for f in waiting:                 # no room before the end: bring them back now
        S.append((RELOAD, f))
        started.append(f)
    for f in started:                 # all of them must have landed before the update
        S.append((SYNC_RELOAD, f))
    return S


def plan_offload_all_sync(n_ops, nfrags):
    """The comparison mode of the paper's evaluation: everything is offloaded and
    waited for before the forward pass and reloaded synchronously at the end."""
    S = [(OFFLOAD, f) for f in range(nfrags)] + [(SYNC_FREE, f) for f in range(nfrags)]
    S += [(COMPUTE, i) for i in range(n_ops)]
    S += [(RELOAD, f) for f in range(nfrags)] + [(SYNC_RELOAD, f) for f in range(nfrags)]
    return S


def peak_memory(S, p_mem, frag_bytes):
    """Replay a schedule: largest (profiled usage + resident optimizer bytes) seen before
    any compute operator, counting a fragment as resident from the moment its reload starts
    until its memory is freed.  Also checks the ordering rules; returns the peak."""
    resident = sum(frag_bytes)
    state = ["resident"] * len(frag_bytes)
    peak = 0
    for kind, idx in S:
        if kind == OFFLOAD:
            assert state[idx] == "resident", "offload of a fragment that is not resident"
            state[idx] = "copying_out"
        elif kind == SYNC_FREE:
            assert state[idx] == "copying_out", "free before the offload copy was started"
            state[idx] = "host"
            resident -= frag_bytes[idx]
        elif kind == RELOAD:
            assert state[idx] == "host", "reload of a fragment that is not on the host"
            state[idx] = "copying_in"
            resident += frag_bytes[idx]
        elif kind == SYNC_RELOAD:
            assert state[idx] == "copying_in", "wait for a reload that was never started"
            state[idx] = "resident"
        else:
            peak = max(peak, p_mem[idx] + resident)
    assert all(s in ("resident", "copying_out") for s in state), "a fragment is missing at the update"
    return peak


# ---------------------------------------------------------------------------
# Proactive prefetching (Algorithm 1), Fuse, and the selective-unsharding choice.
#
# Notation as in the paper's Table 1: S0 initial schedule o_1..o_N, M memory
# limit, M_prefetch limit of a prefetch group, P_mem(o), B_ag(o), Fuse(U),
# T_c(V), alpha.
#
# Readings where the listing is incomplete: (1) in the branch where o_i does not
# fit, the group U is flushed and o_i then opens the next group if it fits on
# its own, otherwise it stays where it is; (2) o_1 has no predecessor to test
# against: an all-gather there joins the last group unless the group limit says no; (3) S is assembled back to
# front and reversed at the end; (4) Fuse walks the group in schedule order and
# merges the next all-gather into the current fused one while
# T_c(V1) + T_c(V2) > alpha * T_c(V1 + V2); (5) T_c(V) is the profiled table,
# linear between samples, flat below the first and continued with the last slope.
# ---------------------------------------------------------------------------

def t_c(V, sizes, times):
    """Profiled communication time for V bytes from the (sizes, times) table."""
    if V <= sizes[0]:
        return times[0]
    k = len(sizes) - 1
    for i in range(1, len(sizes)):
        if V <= sizes[i]:
            k = i
            break
    s0, s1, t0, t1 = sizes[k - 1], sizes[k], times[k - 1], times[k]
    return t0 + (t1 - t0) * (V - s0) / (s1 - s0)


def fuse(U, bag, sizes, times, alpha):
    """Fuse(U): list of groups (lists of operator indices) in schedule order."""
    groups = []
    for o in U:
        if groups:
            V1 = sum(bag[x] for x in groups[-1])
            V2 = bag[o]
            if t_c(V1, sizes, times) + t_c(V2, sizes, times) > alpha * t_c(V1 + V2, sizes, times):
                groups[-1].append(o)
                continue
        groups.append([o])
    return groups


def plan_prefetch(is_ag, bag, p_mem, M, M_prefetch, sizes, times, alpha):
    """Algorithm 1.  Returns the new schedule as a list of entries, each either
    ("op", i) or ("allgather", [i, j, ...]) for a fused group."""
    N = len(is_ag)
    S = []          # built back to front
    U = []          # unscheduled all-gathers, latest first

    def flush():
        if U:
            for grp in reversed(fuse(list(reversed(U)), bag, sizes, times, alpha)):
                S.append(("allgather", grp))
            U.clear()

    for i in range(N - 1, 0, -1):           # o_N ... o_2 (0-based N-1 ... 1)
        if is_ag[i]:
            m_U = sum(bag[o] for o in U) + bag[i]
            m_prev = p_mem[i - 1] + m_U
            if m_prev < M and m_U < M_prefetch:
                U.append(i)
            else:
                flush()
                if p_mem[i - 1] + bag[i] < M and bag[i] < M_prefetch:
                    U.append(i)
                else:
                    S.append(("allgather", [i]))
        else:
            S.append(("op", i))
    if N:
        if is_ag[0]:
            if sum(bag[o] for o in U) + bag[0] >= M_prefetch:
                flush()
            U.append(0)
        else:
            flush()
            S.append(("op", 0))
    flush()
    S.reverse()
    return S


def select_unsharded(bag, sizes, times, budget):
    """Selective unsharding: keep as many parameters gathered as fit in `budget`,
    in order of communication time saved per byte, T_c(B_ag) / B_ag (smaller
    buffers first among equals).  Returns the chosen indices in the order chosen."""
    order = sorted(range(len(bag)), key=lambda o: (-t_c(bag[o], sizes, times) / bag[o], bag[o], o))
    chosen, used = [], 0
    for o in order:
        if used + bag[o] <= budget:
            chosen.append(o)
            used += bag[o]
    return chosen
