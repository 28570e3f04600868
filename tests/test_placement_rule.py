"""The acceptance rule of the region-aware allocator (host logic; no GPU): a buffer is kept only if, at every place
looked at, neither the reference's region nor the rest of the device ends up with more traffic than allowed."""
from paper_2310_18313_amd.placement import fits

TOTAL = 12.0          # bytes per element of the update pass: v 4, copy 1, w 4, m 2, FP8 gradient 1
HERE, AWAY = 0.67 * TOTAL + 1e-9, 0.8 * TOTAL + 1e-9


def test_typical_sequence_of_a_state_allocated_upwards_from_a_region_boundary():
    K = 7
    here, away = [4.0] * K, [0.0] * K                      # v, the anchor, in one region as a whole
    inside, outside = [False] * K, [True] * K
    assert fits(here, away, 1.0, inside, HERE, AWAY)       # the copy beside v: 5 of 12
    here = [5.0] * K
    assert not fits(here, away, 4.0, inside, HERE, AWAY)   # w in the same region: 9 of 12 -> stepped over
    assert fits(here, away, 4.0, outside, HERE, AWAY)      # w in another region
    away = [4.0] * K
    assert fits(here, away, 2.0, outside, HERE, AWAY) and fits(here, away, 2.0, inside, HERE, AWAY)   # m: either side
    away = [6.0] * K
    assert fits(here, away, 1.0, outside, HERE, AWAY)      # FP8 gradient: 7 of 12 outside


def test_a_buffer_across_a_boundary_is_judged_place_by_place():
    here, away = [4.0, 4.0, 4.0, 4.0], [0.0, 0.0, 0.0, 0.0]
    assert fits(here, away, 4.0, [True, True, True, True], HERE, AWAY)
    assert fits(here, away, 4.0, [True, True, True, False], HERE, AWAY)           # 4 + 4 = 8 of 12 at the tail: allowed
    here = [5.0, 5.0, 5.0, 5.0]                                                   # one more byte there is not
    assert not fits(here, away, 4.0, [True, True, True, False], HERE, AWAY)
    assert fits(here, away, 4.0, [True, True, True, True], HERE, AWAY)


def test_the_outside_has_the_soft_limit_only():
    here, away = [4.0] * 3, [8.0] * 3
    assert fits(here, away, 1.0, [True] * 3, HERE, AWAY)          # 9 of 12 outside: allowed (stepping on rarely leads back)
    assert not fits(here, away, 2.0, [True] * 3, HERE, AWAY)      # 10 of 12: the outside would be the bottleneck
    assert fits(here, away, 2.0, [False] * 3, HERE, AWAY)
