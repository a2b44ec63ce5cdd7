"""Pins for the CPU checker's fp32<->fp16 conversions and its ring-hop add
(Section 2.5: half-precision gradients go into allreduce).  numpy's float16 is
the independent library the casts are checked against; the add is checked
against the exactly computed sum rounded once."""
import numpy as np
import pytest

from oracle import binding as ob


def _f16_bits_numpy(x32: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore"):
        return x32.astype(np.float16).view(np.uint16)


def test_f16_to_f32_all_halves():
    h = np.arange(65536, dtype=np.uint16)
    mine = ob.f16_to_f32(h)
    ref = h.view(np.float16).astype(np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(mine), nan)
    assert np.array_equal(mine[~nan].view(np.uint32), ref[~nan].view(np.uint32))
    # NaNs keep sign and become fp32 NaNs with the payload in the top fraction bits
    assert np.all((mine[nan].view(np.uint32) >> 31) == (h[nan] >> 15))


def test_round_trip_every_half():
    h = np.arange(65536, dtype=np.uint16)
    back = ob.f32_to_f16(ob.f16_to_f32(h))
    nan = np.isnan(h.view(np.float16))
    assert np.array_equal(back[~nan], h[~nan])
    assert np.all(np.isnan(back[nan].view(np.float16)))


def test_f32_to_f16_random_bit_patterns():
    rng = np.random.default_rng(1)
    u = rng.integers(0, 2**32, size=1 << 22, dtype=np.uint64).astype(np.uint32)
    x = u.view(np.float32)
    mine, ref = ob.f32_to_f16(x), _f16_bits_numpy(x)
    nan = np.isnan(x)
    assert np.array_equal(mine[~nan], ref[~nan])
    assert np.all(np.isnan(mine[nan].view(np.float16)))


def test_f32_to_f16_gradient_like_values():
    rng = np.random.default_rng(2)
    for scale in (1e-8, 1e-6, 1e-4, 1e-2, 1.0, 100.0, 3e4, 7e4):
        x = (rng.standard_normal(1 << 18) * scale).astype(np.float32)
        assert np.array_equal(ob.f32_to_f16(x), _f16_bits_numpy(x))


def test_f32_to_f16_every_rounding_boundary():
    """Midpoints between neighbouring halves (ties) and the fp32 values one ulp
    either side of them, for every finite half, both signs."""
    h = np.arange(0, 0x7c00, dtype=np.uint16)          # all finite non-negative halves
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[-1] = 65536.0                                   # the step above 65504 would be 2^16
    mid = ((lo + hi) / 2).astype(np.float32)           # exact: 12 significant bits
    assert np.array_equal(mid.astype(np.float64), (lo + hi) / 2)
    below = np.nextafter(mid, np.float32(-np.inf))
    above = np.nextafter(mid, np.float32(np.inf))
    for arr in (mid, below, above):
        for sgn in (1.0, -1.0):
            x = (arr * np.float32(sgn)).astype(np.float32)
            assert np.array_equal(ob.f32_to_f16(x), _f16_bits_numpy(x))
    # a tie goes to the even neighbour
    got = ob.f32_to_f16(mid)
    assert np.all(got % 2 == 0)


def test_f32_to_f16_named_edge_cases():
    cases = [
        (0.0, 0x0000), (-0.0, 0x8000),
        (65504.0, 0x7bff), (65519.99, 0x7bff), (65520.0, 0x7c00), (1e9, 0x7c00), (-65520.0, 0xfc00),
        (np.inf, 0x7c00), (-np.inf, 0xfc00),
        (2.0 ** -24, 0x0001), (2.0 ** -25, 0x0000), (2.0 ** -25 * (1 + 2.0 ** -20), 0x0001),
        (1.5 * 2.0 ** -24, 0x0002),   # tie between 1 and 2 -> even
        (2.5 * 2.0 ** -24, 0x0002),   # tie between 2 and 3 -> even
        (2.0 ** -14, 0x0400), (2.0 ** -14 * (1 - 2.0 ** -11), 0x0400),   # rounds up into normals
        (1e-40, 0x0000), (-1e-40, 0x8000),   # fp32 subnormal inputs
        (1.0, 0x3c00), (1.0 + 2.0 ** -11, 0x3c00), (1.0 + 3 * 2.0 ** -11, 0x3c02),
    ]
    x = np.array([c[0] for c in cases], dtype=np.float32)
    want = np.array([c[1] for c in cases], dtype=np.uint16)
    assert np.array_equal(ob.f32_to_f16(x), want)


def _exact_half_sum(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Exact sum of two halves (fp64 holds it exactly) rounded once to half."""
    s = a.view(np.float16).astype(np.float64) + b.view(np.float16).astype(np.float64)
    with np.errstate(over="ignore"):
        return s.astype(np.float16).view(np.uint16)


def test_hop_add_is_the_correctly_rounded_half_sum():
    rng = np.random.default_rng(3)
    n = 1 << 21
    a = rng.integers(0, 65536, size=n, dtype=np.uint32).astype(np.uint16)
    b = rng.integers(0, 65536, size=n, dtype=np.uint32).astype(np.uint16)
    # half of the pairs: close exponents, where cancellation and ties happen
    b[: n // 2] = (a[: n // 2] ^ rng.integers(0, 1 << 12, size=n // 2, dtype=np.uint32).astype(np.uint16)
                   ^ (rng.integers(0, 2, size=n // 2, dtype=np.uint32).astype(np.uint16) << 15))
    fin = np.isfinite(a.view(np.float16)) & np.isfinite(b.view(np.float16))
    a, b = a[fin], b[fin]
    L = a.size
    x = np.stack([a, b])                               # P = 2: every segment is a + b
    got = ob.ring_fold(x, "f16")
    want = _exact_half_sum(a, b)
    nan = np.isnan(want.view(np.float16))
    assert not nan.any()
    # +0 / -0: IEEE says x + (-x) = +0 under round-to-nearest; numpy agrees
    assert np.array_equal(got, want)


def test_hop_add_scalar_examples():
    one, tiny, big = 0x3c00, 0x0001, 0x7bff
    assert ob.f16_add(one, one) == 0x4000
    assert ob.f16_add(tiny, tiny) == 0x0002            # subnormal arithmetic is exact
    assert ob.f16_add(big, big) == 0x7c00              # overflow -> inf
    assert ob.f16_add(0x6800, 0x3c00) == 0x6800        # 2048 + 1 ties to even 2048
    assert ob.f16_add(0x6801, 0x3c00) == 0x6802        # 2050 + 1 ties to even 2052
    assert ob.f16_add(0x8000, 0x0000) == 0x0000        # -0 + +0 = +0
