"""The pins of the oracle's Python half must bite too: plant one plausible mistake at a time
in a copy of the source of oracle/planner.py or oracle/layout.py (text substitution, compiled
into a scratch module, its functions swapped in for the real ones) and check that at least
one pin fails.  Runs on the CPU only."""
import inspect
import types

import pytest

from oracle import layout, planner
from tests import test_oracle_cast_unshard as U
from tests import test_oracle_packed_state as K
from tests import test_oracle_planner as T

PLANNER_MUTATIONS = {
    # Algorithm 1's two tests: strict comparisons
    "prefetch_memory_test_not_strict": ("if usage[i - 1] + carried < limit and carried < group_limit:",
                                        "if usage[i - 1] + carried <= limit and carried < group_limit:"),
    "prefetch_group_test_not_strict": ("if usage[i - 1] + carried < limit and carried < group_limit:",
                                       "if usage[i - 1] + carried < limit and carried <= group_limit:"),
    "prefetch_memory_before_the_wrong_operator": ("if usage[i - 1] + carried < limit and carried < group_limit:",
                                                  "if usage[i] + carried < limit and carried < group_limit:"),
    "prefetch_blocked_gather_travels_anyway": ("            stays.add(i)", "            travelling.append(i)"),
    "prefetch_group_put_down_in_front": ("        put_down(i)\n        if usage[i - 1] + buffer_bytes[i] < limit",
                                         "        put_down(i - 1)\n        if usage[i - 1] + buffer_bytes[i] < limit"),
    # Algorithm 2: order of release and return, look-ahead, thresholds
    "fragments_released_last_in_first_out": ("f = copying_out.popleft()", "f = copying_out.pop()"),
    "fragments_return_last_in_first_out": ("f = away.popleft()\n                schedule.append((RELOAD, f))",
                                           "f = away.pop()\n                schedule.append((RELOAD, f))"),
    "reload_look_ahead_off_by_one": ("while away and missing_ahead[i] <= absent - sizes[away[0]]:",
                                     "while away and missing_ahead[i + 1] <= absent - sizes[away[0]]:"),
    "reload_ignores_the_fragment_size": ("while away and missing_ahead[i] <= absent - sizes[away[0]]:",
                                         "while away and missing_ahead[i] <= absent:"),
    "reload_allowed_in_the_forward_pass": ("        if i >= n_forward:", "        if i >= 0:"),
    "reload_one_operator_late": ("        if i >= n_forward:", "        if i > n_forward:"),
    "one_fragment_too_many_leaves": ("        if covered >= worst:", "        if covered > worst:"),
    "peak_of_the_forward_pass_only": ("worst = (max(usage) if usage else 0) + state_bytes - limit",
                                      "worst = (max(usage[:n_forward]) if usage else 0) + state_bytes - limit"),
    "memory_taken_away_too_early": ("        while missing[i] > absent:", "        while missing[i + 1 if i + 1 < n_ops else i] > absent:"),
    "reloads_not_waited_for": ("    schedule.extend((SYNC_RELOAD, f) for f in coming_back)",
                               "    schedule.extend((SYNC_RELOAD, f) for f in coming_back[:-1])"),
    # Fuse and the table
    "fuse_alpha_on_the_wrong_side": ("if apart > alpha * t_c(have + b, sizes, times):",
                                     "if alpha * apart > t_c(have + b, sizes, times):"),
    "fuse_compares_with_the_last_member_only": ("            have = merged[-1][1]", "            have = buffer_bytes[merged[-1][0][-1]]"),
    "table_flat_beyond_the_last_sample": ("    if nbytes <= sizes[0] or len(sizes) == 1:",
                                          "    if nbytes >= sizes[-1]:\n        return times[-1]\n    if nbytes <= sizes[0] or len(sizes) == 1:"),
    "table_takes_the_segment_below": ("    lo = hi - 1\n", "    hi = max(hi - 1, 1)\n    lo = hi - 1\n"),
    # selective unsharding
    "unsharded_lowest_saving_first": ("key=lambda o: (-saving_per_byte(o), buffer_bytes[o], o))",
                                      "key=lambda o: (saving_per_byte(o), buffer_bytes[o], o))"),
    "unsharded_ranked_by_time_not_per_byte": ("        return t_c(buffer_bytes[o], sizes, times) / buffer_bytes[o]",
                                              "        return t_c(buffer_bytes[o], sizes, times)"),
    "unsharded_exact_fit_refused": ("        if buffer_bytes[o] <= room:", "        if buffer_bytes[o] < room:"),
    "unsharded_stops_at_the_first_misfit": ("        if buffer_bytes[o] <= room:\n            kept.append(o)\n            room -= buffer_bytes[o]\n",
                                            "        if buffer_bytes[o] > room:\n            break\n        kept.append(o)\n        room -= buffer_bytes[o]\n"),
    "unsharded_larger_first_among_equals": ("(-saving_per_byte(o), buffer_bytes[o], o))", "(-saving_per_byte(o), -buffer_bytes[o], o))"),
}

LAYOUT_MUTATIONS = {
    "shard_size_rounded_down": ("    per_rank = -(-total // world)", "    per_rank = total // world"),
    "shard_alignment_rounded_down": ("    shard = -(-per_rank // shard_align) * shard_align",
                                     "    shard = max(1, per_rank // shard_align) * shard_align"),
    "offsets_start_at_the_first_size": ("        offsets.append(off)\n        off += n", "        off += n\n        offsets.append(off)"),
    "padding_in_front": ("    pos = 0\n    for t in tensors:\n        t = np.asarray(t, dtype=dtype).reshape(-1)",
                         "    pos = world * shard - total\n    total += pos\n    for t in tensors:\n        t = np.asarray(t, dtype=dtype).reshape(-1)"),
    "last_rank_off_by_one": ("    return offset // shard, (offset + numel - 1) // shard",
                             "    return offset // shard, (offset + numel) // shard"),
    "slice_size_rounded_down": ("        s = -(-n // world)\n", "        s = n // world\n"),
    "slice_alignment_rounded_down": ("        s = -(-s // align) * align", "        s = (s // align) * align"),
    "slices_interleaved_not_blocked": ("                i = r * s + j", "                i = j * world + r"),
    "segment_reads_the_padding": ("            k = min(s, max(0, int(n) - r * s))", "            k = s if int(n) - r * s > 0 else 0"),
    "segment_destination_ignores_the_rank": ("                segs.append((t, r * L + o, r * s, k))",
                                             "                segs.append((t, r * L + o, 0, k))"),
    "segment_source_ignores_the_tensor_offset": ("                segs.append((t, r * L + o, r * s, k))",
                                                 "                segs.append((t, r * L, r * s, k))"),
    # packed optimizer state
    "packed_length_rounded_down": ("    return 3 * (-(-int(n) // granule)) * granule", "    return 3 * (int(n) // granule) * granule"),
    "packed_length_without_padding": ("    return 3 * (-(-int(n) // granule)) * granule", "    return 3 * int(n)"),
    "packed_granules_two_apart": ("        base = 3 * k * granule", "        base = 2 * k * granule"),
    "packed_momentum_and_variance_swapped": ("        out[base + granule:base + granule + (hi - lo)] = m[lo:hi]\n        out[base + 2 * granule:base + 2 * granule + (hi - lo)] = v[lo:hi]",
                                             "        out[base + granule:base + granule + (hi - lo)] = v[lo:hi]\n        out[base + 2 * granule:base + 2 * granule + (hi - lo)] = m[lo:hi]"),
    "packed_last_granule_dropped": ("    while k * granule < n:\n        lo, hi", "    while (k + 1) * granule <= n:\n        lo, hi"),
    "unpack_reads_the_parameter_slot_twice": ("        m[first:first + count] = state[start + granule:start + granule + count]",
                                              "        m[first:first + count] = state[start:start + count]"),
    "unpack_granules_two_apart": ("        start = 3 * k * granule", "        start = 2 * k * granule"),
    "unpack_short_granule_read_whole": ("first, count = k * granule, min(granule, n - k * granule)",
                                        "first, count = k * granule, granule"),
}

PLANNER_PINS = [
    T.test_hand_worked_schedule, T.test_nothing_to_do_when_everything_fits,
    T.test_reload_waits_for_memory_to_fall, T.test_reload_looks_ahead_to_the_end_of_the_schedule,
    T.test_peak_in_the_backward_pass, T.test_no_reload_in_the_forward_pass, T.test_does_not_fit_is_an_error,
    *[(lambda s=s: T.test_invariants_on_random_profiles(s)) for s in range(40)],
    *[(lambda s=s: T.test_placement_is_tight(s)) for s in range(40, 70)],
    T.test_offload_all_sync_mode, T.test_t_c_table, T.test_fuse_merges_small_messages_only,
    T.test_prefetch_hand_worked, *[(lambda s=s: T.test_prefetch_properties(s)) for s in range(60)],
    T.test_select_unsharded, T.test_select_unsharded_order_by_brute_force,
]

LAYOUT_PINS = [
    *[(lambda n=n, a=a: U.test_layout_brute_force(n, a)) for a in (1, 8, 4096)
      for n in ([1, 3, 7, 4097], [5], [0, 9, 0, 2], [4096] * 3 + [17])],
    U.test_unshard_brute_force_ragged, U.test_unshard_hash_property_and_ranks_spanned,
    *[(lambda n=n, a=a: U.test_per_tensor_round_trip_and_ownership(n, a)) for a in (1, 8)
      for n in ([1, 3, 7, 4097], [16, 64, 8], [5], [0, 9, 0, 2], [1000, 24, 333])],
    U.test_per_tensor_divisible_case_is_a_reshape, U.test_model_shapes_match_paper_sizes,
    K.test_hand_worked_example, K.test_whole_granules_are_a_reshape, K.test_empty_and_rejected_inputs,
    *[(lambda n=n, g=g: K.test_index_formula_element_by_element(n, g))
      for n, g in ((1, 8), (7, 8), (9, 8), (37, 5), (64, 8))],
]


def failing(pins):
    failed = []
    for pin in pins:
        try:
            pin()
        except Exception as e:          # AssertionError, or a crash caused by the mistake
            failed.append((getattr(pin, "__name__", "case"), type(e).__name__))
    return failed


def swapped_in(module, old, new):
    """Context manager: the module's functions replaced by those of a mutated copy of its source."""
    class _Swap:
        def __enter__(self):
            text = inspect.getsource(module)
            assert text.count(old) == 1, "mutation anchor must occur exactly once"
            scratch = types.ModuleType(module.__name__ + "_mutated")
            exec(compile(text.replace(old, new, 1), module.__file__ + " (mutated)", "exec"), scratch.__dict__)
            self.saved = {k: v for k, v in vars(module).items() if inspect.isfunction(v)}
            for k in self.saved:
                setattr(module, k, getattr(scratch, k))

        def __exit__(self, *exc):
            for k, v in self.saved.items():
                setattr(module, k, v)
    return _Swap()


def test_unmutated_python_oracle_passes_every_pin():
    assert failing(PLANNER_PINS) == [] and failing(LAYOUT_PINS) == []


@pytest.mark.parametrize("name", sorted(PLANNER_MUTATIONS))
def test_planted_mistake_in_the_planners_is_caught(name):
    with swapped_in(planner, *PLANNER_MUTATIONS[name]):
        failed = failing(PLANNER_PINS)
    assert failed, f"no pin noticed the planted mistake '{name}'"
    assert failing(PLANNER_PINS[:7]) == []          # and the real functions are back


@pytest.mark.parametrize("name", sorted(LAYOUT_MUTATIONS))
def test_planted_mistake_in_the_layouts_is_caught(name):
    with swapped_in(layout, *LAYOUT_MUTATIONS[name]):
        failed = failing(LAYOUT_PINS)
    assert failed, f"no pin noticed the planted mistake '{name}'"
    assert failing(LAYOUT_PINS[:3]) == []
