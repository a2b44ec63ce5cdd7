"""Pins for the CPU checker's ring allreduce (Section 2.4)."""
import json
import os

import numpy as np
import pytest

from oracle import binding as ob

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.json")))


def _rand_halves(rng, P, L, spread=6):
    """Finite halves with per-rank scales a few binades apart (so order matters)."""
    x = rng.standard_normal((P, L)) * (2.0 ** rng.integers(-spread, spread, size=(P, 1)))
    return x.astype(np.float16).view(np.uint16)


@pytest.mark.parametrize("wire", ["f16", "f32"])
@pytest.mark.parametrize("P,L", [(1, 17), (2, 64), (3, 100), (4, 4096), (5, 1001), (8, 8 * 24),
                                 (16, 50), (7, 3), (4, 0), (64, 9000)])
def test_message_passing_equals_rotated_fold(wire, P, L):
    rng = np.random.default_rng(P * 1000 + L)
    x = _rand_halves(rng, P, L) if wire == "f16" else \
        (rng.standard_normal((P, L)) * 10.0 ** rng.integers(-3, 3, size=(P, 1))).astype(np.float32)
    final, sent = ob.ring_allreduce_hops(x, wire)
    fold = ob.ring_fold(x, wire)
    for r in range(P):                       # Section 3.2: afterwards all GPUs hold the same values
        assert np.array_equal(final[r], fold)


def test_one_rank_is_the_identity_and_two_ranks_add():
    rng = np.random.default_rng(5)
    x = _rand_halves(rng, 2, 999)
    assert np.array_equal(ob.ring_fold(x[:1].copy(), "f16"), x[0])
    want = (x[0].view(np.float16).astype(np.float64) + x[1].view(np.float16).astype(np.float64))
    assert np.array_equal(ob.ring_fold(x, "f16"), want.astype(np.float16).view(np.uint16))


@pytest.mark.parametrize("P,L", [(4, 1000), (8, 4099), (16, 77), (3, 8)])
def test_integer_data_gives_the_exact_sum(P, L):
    # small integers: every partial sum is exact in fp16, so any index or
    # segment mistake shows while rounding order cannot
    rng = np.random.default_rng(P + L)
    ints = rng.integers(-8, 9, size=(P, L))
    want = ints.sum(axis=0)
    for wire, dt in (("f16", np.float16), ("f32", np.float32)):
        x = ints.astype(dt)
        x = x.view(np.uint16) if wire == "f16" else x
        got = ob.ring_fold(x, wire)
        got = got.view(np.float16) if wire == "f16" else got
        assert np.array_equal(got.astype(np.int64), want)
        final, _ = ob.ring_allreduce_hops(x, wire)
        f0 = final[0].view(np.float16) if wire == "f16" else final[0]
        assert np.array_equal(f0.astype(np.int64), want)


def test_fold_starts_at_the_segment_owner_and_walks_up_the_ring():
    # Three ranks, one 8-element segment each.  In fp16, 2048 + 1 = 2048 (tie to
    # even) but 1 + 1 + 2048 = 2050, so the three rotations differ:
    #   segment 0: (x0 + x1) + x2 = (2048 + 1) + 1 = 2048
    #   segment 1: (x1 + x2) + x0 = (1 + 1) + 2048 = 2050
    #   segment 2: (x2 + x0) + x1 = (1 + 2048) + 1 = 2048
    L = 24
    x = np.stack([np.full(L, 2048.0), np.full(L, 1.0), np.full(L, 1.0)]).astype(np.float16)
    got = ob.ring_fold(x.view(np.uint16), "f16").view(np.float16)
    assert ob.ring_segment(L, 3, "f16") == 8
    assert np.all(got[0:8] == 2048) and np.all(got[8:16] == 2050) and np.all(got[16:24] == 2048)
    final, _ = ob.ring_allreduce_hops(x.view(np.uint16), "f16")
    assert np.array_equal(final[2].view(np.float16), got)


def test_fold_against_numpy_half_arithmetic():
    rng = np.random.default_rng(9)
    P, L = 6, 6 * 40
    x = _rand_halves(rng, P, L)
    seg = ob.ring_segment(L, P, "f16")
    xf = x.view(np.float16)
    want = np.empty(L, dtype=np.float16)
    for i in range(L):
        s = i // seg
        v = xf[s, i]
        for j in range(1, P):
            v = np.float16(v + xf[(s + j) % P, i])
        want[i] = v
    assert np.array_equal(ob.ring_fold(x, "f16"), want.view(np.uint16))


def test_segments_are_16_byte_multiples_and_cover_the_buffer():
    for wire, A in (("f16", 8), ("f32", 4)):
        for P in (1, 2, 3, 8, 16, 64):
            for L in (0, 1, 7, 8, 9, 1000, 4096, 262144, 6127616):
                seg = ob.ring_segment(L, P, wire)
                assert seg % A == 0 and seg * P >= L
                assert seg - A < -(-L // P) <= seg or L == 0


def test_traffic_through_each_gpu_matches_the_paper():
    # Section 2.4: K/N per message, 2(N-1) messages, 2(N-1)K/N in total
    assert GOLD["ring_traffic"]["total"] == "2*(N-1)*K/N"
    rng = np.random.default_rng(11)
    for P, per in ((4, 64), (8, 8), (16, 24)):
        L = P * per                            # divides evenly into 16-byte multiples
        x = _rand_halves(rng, P, L)
        _, sent = ob.ring_allreduce_hops(x, "f16")
        assert np.all(sent == 2 * (P - 1) * L // P)
    # Section 1: 61M fp32 parameters -> 488 MB through every GPU (2K as N grows)
    fact = GOLD["alexnet_wire"]
    K = fact["params"] * fact["bytes_per_param"]
    assert round(2 * K / 1e6) == fact["mbytes"]
    assert 2 * (512 - 1) * K / 512 / 1e6 == pytest.approx(fact["mbytes"], rel=2e-3)
