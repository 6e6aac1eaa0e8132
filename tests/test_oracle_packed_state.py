"""Pins for the oracle's packed optimizer-state layout (granules of p, m, v following each
other).  The layout is this build's own, so the pins are its definition worked by hand, the
index formula element by element, and the special case that is a plain reshape."""
import numpy as np
import pytest

from oracle import layout


def test_hand_worked_example():
    # n = 5, granules of 2: [p0 p1][m0 m1][v0 v1][p2 p3][m2 m3][v2 v3][p4 0][m4 0][v4 0]
    p = [1, 2, 3, 4, 5]
    m = [11, 12, 13, 14, 15]
    v = [21, 22, 23, 24, 25]
    want = [1, 2, 11, 12, 21, 22, 3, 4, 13, 14, 23, 24, 5, 0, 15, 0, 25, 0]
    got = layout.pack_state(p, m, v, 2)
    assert got.dtype == np.float32 and got.tolist() == want
    assert layout.packed_state_numel(5, 2) == 18
    back = layout.unpack_state(got, 5, 2)
    assert [a.tolist() for a in back] == [p, m, v]


@pytest.mark.parametrize("n,granule", [(1, 1), (1, 8), (7, 8), (8, 8), (9, 8), (64, 8), (37, 5), (100, 32),
                                       (8192, 8192), (8193, 8192), (3 * 8192 - 1, 8192)])
def test_index_formula_element_by_element(n, granule):
    rng = np.random.default_rng(n * 131 + granule)
    p, m, v = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    packed = layout.pack_state(p, m, v, granule)
    whole = -(-n // granule)
    assert packed.size == 3 * whole * granule == layout.packed_state_numel(n, granule)
    seen = np.zeros(packed.size, dtype=bool)
    for e in range(n):
        at = (e // granule) * 3 * granule + e % granule
        assert packed[at] == p[e] and packed[at + granule] == m[e] and packed[at + 2 * granule] == v[e]
        seen[[at, at + granule, at + 2 * granule]] = True
    assert seen.sum() == 3 * n                      # no two elements share a slot
    assert not packed[~seen].any()                  # and everything else is zero padding
    back = layout.unpack_state(packed, n, granule)
    assert all(np.array_equal(a, b) for a, b in zip(back, (p, m, v)))


def test_whole_granules_are_a_reshape():
    granule, whole = 16, 5
    n = granule * whole
    rng = np.random.default_rng(7)
    p, m, v = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    want = np.stack([p.reshape(whole, granule), m.reshape(whole, granule), v.reshape(whole, granule)],
                    axis=1).reshape(-1)
    assert np.array_equal(layout.pack_state(p, m, v, granule), want)
    up, um, uv = layout.unpack_state(want, n, granule)
    cube = want.reshape(whole, 3, granule)
    assert np.array_equal(up, cube[:, 0].reshape(-1)) and np.array_equal(um, cube[:, 1].reshape(-1))
    assert np.array_equal(uv, cube[:, 2].reshape(-1))


def test_empty_and_rejected_inputs():
    assert layout.packed_state_numel(0, 8) == 0 and layout.pack_state([], [], [], 8).size == 0
    with pytest.raises(ValueError):
        layout.pack_state([1.0], [1.0, 2.0], [1.0], 8)
    with pytest.raises(ValueError):
        layout.unpack_state(np.zeros(5, np.float32), 3, 8)
    with pytest.raises(ValueError):
        layout.packed_state_numel(3, 0)
