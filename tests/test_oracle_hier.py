"""Pins for the CPU checker's hierarchical allreduce (Section 2.4: group reduce to
the master, ring allreduce among the masters, broadcast in the group)."""
import json
import os

import numpy as np
import pytest

from oracle import binding as ob

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.json")))


def _rand_halves(rng, P, L, spread=6):
    x = rng.standard_normal((P, L)) * (2.0 ** rng.integers(-spread, spread, size=(P, 1)))
    return x.astype(np.float16).view(np.uint16)


def _rand(rng, P, L, wire):
    if wire == "f16":
        return _rand_halves(rng, P, L)
    return (rng.standard_normal((P, L)) * 10.0 ** rng.integers(-3, 3, size=(P, 1))).astype(np.float32)


def _h(v):
    return np.array(v, dtype=np.float16).view(np.uint16)


@pytest.mark.parametrize("wire", ["f16", "f32"])
@pytest.mark.parametrize("P,M,L", [(4, 2, 100), (16, 4, 4099), (8, 1, 64), (8, 8, 1000), (6, 3, 17),
                                   (6, 2, 3), (12, 3, 0), (64, 8, 3000), (1, 1, 9)])
def test_message_passing_equals_the_formula_and_every_rank_ends_alike(wire, P, M, L):
    rng = np.random.default_rng(P * 100 + M * 10 + L)
    x = _rand(rng, P, L, wire)
    final, _ = ob.hier_allreduce_hops(x, M, wire)
    fold = ob.hier_fold(x, M, wire)
    for r in range(P):
        assert np.array_equal(final[r], fold)


@pytest.mark.parametrize("wire", ["f16", "f32"])
def test_groups_of_one_rank_are_the_flat_ring(wire):
    rng = np.random.default_rng(3)
    x = _rand(rng, 8, 1001, wire)
    assert np.array_equal(ob.hier_fold(x, 8, wire), ob.ring_fold(x, wire))
    final, sent = ob.hier_allreduce_hops(x, 8, wire)
    flat, flat_sent = ob.ring_allreduce_hops(x, wire)
    assert np.array_equal(final, flat) and np.array_equal(sent, flat_sent)


@pytest.mark.parametrize("P,M,L", [(4, 2, 1000), (16, 4, 4099), (12, 3, 77), (8, 1, 8)])
def test_integer_data_gives_the_exact_sum(P, M, L):
    # every partial sum is exact, so only a wrong index, group or segment can show
    rng = np.random.default_rng(P + L)
    ints = rng.integers(-8, 9, size=(P, L))
    want = ints.sum(axis=0)
    for wire, dt in (("f16", np.float16), ("f32", np.float32)):
        x = ints.astype(dt)
        x = x.view(np.uint16) if wire == "f16" else x
        got = ob.hier_fold(x, M, wire)
        got = got.view(np.float16) if wire == "f16" else got
        assert np.array_equal(got.astype(np.int64), want)
        final, _ = ob.hier_allreduce_hops(x, M, wire)
        f = final[P - 1].view(np.float16) if wire == "f16" else final[P - 1]
        assert np.array_equal(f.astype(np.int64), want)


def test_the_chain_inside_a_group_starts_after_the_master_and_ends_on_it():
    # One group of four ranks.  fp16 spacing is 2 from 2048 on: 2048 + 1 = 2048 (tie to even), so a
    # chain that started on the 2048 would stay there; started on the ones it reaches 3 and
    # 3 + 2048 = 2051 -> 2052.
    # the hand-worked values of the four positions (chain 1, 2, 3, 0):
    #   2048 on rank 0: (1+1)+1 = 3, 3+2048 = 2051 -> tie -> 2052
    #   2048 on rank 1: 2048+1 -> 2048, +1 -> 2048, +1 -> 2048
    #   2048 on rank 2: 1+2048 -> 2048, +1 -> 2048, +1 -> 2048
    #   2048 on rank 3: 1+1 = 2, 2+2048 = 2050, 2050+1 = 2051 -> tie -> 2052
    for pos, want in ((0, 2052.0), (1, 2048.0), (2, 2048.0), (3, 2052.0)):
        col = [1.0] * 4
        col[pos] = 2048.0
        x = np.repeat(_h(col)[:, None], 8, axis=1)
        assert np.all(ob.hier_fold(x, 1, "f16").view(np.float16) == np.float16(want)), pos
        final, _ = ob.hier_allreduce_hops(x, 1, "f16")
        assert np.all(final.view(np.float16) == np.float16(want)), pos


def test_masters_ring_rotates_over_group_sums():
    # Three groups of two ranks, one 8-element segment per master.  Group sums (rank 2g+1 + rank 2g)
    # are 2048, 1 and 1: exactly the three-rank example of the flat ring, whose three segments end
    # as 2048+1+1 -> 2048, 1+1+2048 = 2050 and 1+2048+1 -> 2048.
    col = [1024.0, 1024.0, 0.5, 0.5, 0.0, 1.0]
    x = np.repeat(_h(col)[:, None], 24, axis=1)
    got = ob.hier_fold(x, 3, "f16").view(np.float16)
    assert np.all(got[0:8] == np.float16(2048.0))
    assert np.all(got[8:16] == np.float16(2050.0))
    assert np.all(got[16:24] == np.float16(2048.0))


def test_group_sum_is_rounded_before_it_enters_the_masters_ring():
    # two groups of two; group 0 holds 2048 and 1 (sum rounds to 2048), group 1 holds 1 and 0.
    # Segment 0: 2048 + 1 = 2048.  A flat chain over four ranks in any order that adds the two
    # ones first would give 2050: the grouping itself is visible.
    col = [2048.0, 1.0, 1.0, 0.0]
    x = np.repeat(_h(col)[:, None], 16, axis=1)
    got = ob.hier_fold(x, 2, "f16").view(np.float16)
    assert np.all(got == np.float16(2048.0))


@pytest.mark.parametrize("P,M", [(16, 4), (8, 2), (64, 8)])
def test_message_sizes_and_traffic(P, M):
    """Section 2.4: the masters' ring sends L/M elements per message (the text's L*M/P in its
    16-rank, 4-group example), 2(M-1) times; the other ranks send the whole buffer once in the
    reduce and once in the broadcast (the last of a chain only in the reduce)."""
    G = P // M
    L = 8 * P * 5                                   # divisible: no padding in any segment
    x = _rand_halves(np.random.default_rng(1), P, L)
    _, sent = ob.hier_allreduce_hops(x, M, "f16")
    seg = ob.ring_segment(L, M, "f16")
    assert seg == L // M
    ex = GOLD["hierarchical_example"]
    if (P, M) == (ex["N"], ex["M"]):
        assert seg == L * M // P == L // 4          # the text's formula K*M/N in its own example
    for r in range(P):
        local = r % G
        if local == 0:
            want = 2 * (M - 1) * seg + (L if G > 1 else 0)          # masters' ring + first broadcast hop
        elif local == G - 1:
            want = L                                                # reduce only: last of the broadcast chain
        else:
            want = 2 * L
        assert sent[r] == want, (r, sent[r], want)


def test_iteration_drivers_take_the_order():
    from oracle import pipeline as op
    rng = np.random.default_rng(2)
    sizes = [40, 24, 100]
    pools = (rng.standard_normal((4, sum(sizes))) * 10.0 ** rng.integers(-2, 2, size=(4, 1))).astype(np.float32)
    flat = op.dense_iteration(pools, sizes, 50, 16.0)
    hier = op.dense_iteration(pools, sizes, 50, 16.0, groups=2)
    assert np.array_equal(flat["send"], hier["send"])
    for a, b in zip(hier["bucket_lo"], hier["bucket_hi"]):
        assert np.array_equal(hier["reduced"][a:b], ob.hier_fold(np.ascontiguousarray(hier["send"][:, a:b]), 2))
    st = op.new_state(4, sum(sizes))
    r = op.csc_iteration(st, pools, 16, 3, 16.0, 1.0, "immediate", groups=2)
    assert np.array_equal(r["reduced"], ob.hier_fold(r["send"], 2))
