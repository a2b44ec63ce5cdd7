"""Pins for the CPU checker's SGD-update step of Algorithm 1 (momentum SGD correction)."""
import numpy as np

from oracle import binding as ob


def _wire(g32, S):
    return ob.f32_to_f16((g32 * np.float32(S)).astype(np.float32))


def test_all_chunks_important_is_textbook_momentum_sgd():
    # u = momentum*u + lr*g ; w = w + u, element by element in fp32 (numpy does the arithmetic here)
    rng = np.random.default_rng(0)
    N, C, S = 1000, 128, 64.0
    nc = ob.n_chunks(N, C)
    sel = np.arange(nc, dtype=np.int32)
    m, lr = np.float32(0.9), np.float32(-0.05)
    w = rng.standard_normal(N).astype(np.float32)
    hu = np.zeros(N, dtype=np.float32)
    w_ref, v_ref = w.copy(), hu.copy()
    alpha = np.float32(1) / np.float32(S)
    for t in range(5):
        red = _wire(rng.standard_normal(N).astype(np.float32) * 0.01, S)
        out = np.zeros(N, dtype=np.float32)
        ob.sgd_update(red, N, C, sel, alpha, m, lr, w, hu, out)
        g = red.view(np.float16).astype(np.float32) * alpha
        assert np.array_equal(out, g)
        v_ref = (m * v_ref).astype(np.float32) + (lr * g).astype(np.float32)
        w_ref = w_ref + v_ref
        assert np.array_equal(hu.view(np.uint32), v_ref.view(np.uint32))
        assert np.array_equal(w.view(np.uint32), w_ref.view(np.uint32))


def test_constant_gradient_closed_form():
    # powers of two: hu_T = lr*g*(1 - m^T)/(1 - m) exactly, w_T = w_0 + sum_t hu_t
    N, C = 64, 16
    sel = np.arange(4, dtype=np.int32)
    red = np.full(N, 0.125, dtype=np.float16).view(np.uint16)
    w = np.ones(N, dtype=np.float32)
    hu = np.zeros(N, dtype=np.float32)
    total = 0.0
    for T in range(1, 8):
        ob.sgd_update(red, N, C, sel, 1.0, 0.5, -0.25, w, hu)
        want = -0.25 * 0.125 * (1 - 0.5 ** T) / (1 - 0.5)
        total += want
        assert np.all(hu == np.float32(want)) and np.all(w == np.float32(1.0 + total))


def test_other_chunks_keep_their_history_and_weights():
    rng = np.random.default_rng(1)
    N, C = 1000, 100                              # 10 chunks
    w0 = rng.standard_normal(N).astype(np.float32)
    hu0 = rng.standard_normal(N).astype(np.float32)
    w, hu = w0.copy(), hu0.copy()
    sel = np.array([2, 9], dtype=np.int32)
    red = _wire(rng.standard_normal(200).astype(np.float32), 1.0)
    ob.sgd_update(red, N, C, sel, 1.0, 0.9, 0.1, w, hu)
    mask = np.zeros(N, dtype=bool)
    mask[200:300] = True
    mask[900:1000] = True
    assert np.array_equal(w[~mask], w0[~mask]) and np.array_equal(hu[~mask], hu0[~mask])
    g = red.view(np.float16).astype(np.float32)
    want_hu = (np.float32(0.9) * hu0[mask]).astype(np.float32) + (np.float32(0.1) * g).astype(np.float32)
    assert np.array_equal(hu[mask], want_hu) and np.array_equal(w[mask], w0[mask] + want_hu)
    # a chunk skipped now and important later resumes from its old history (hu_t = hu_{t-1})
    sel2 = np.array([0], dtype=np.int32)
    red2 = _wire(np.ones(100, dtype=np.float32), 1.0)
    ob.sgd_update(red2, N, C, sel2, 1.0, 0.9, 0.1, w, hu)
    assert np.array_equal(hu[:100], (np.float32(0.9) * hu0[:100]).astype(np.float32) + np.float32(0.1))


def test_momentum_zero_unit_rate_accumulates_the_gradient():
    N, C = 256, 64
    sel = np.array([1, 3], dtype=np.int32)
    red = _wire(np.arange(128, dtype=np.float32), 1.0)
    w = np.zeros(N, dtype=np.float32)
    hu = np.full(N, 7.0, dtype=np.float32)
    ob.sgd_update(red, N, C, sel, 1.0, 0.0, 1.0, w, hu)
    assert np.array_equal(w[64:128], np.arange(64, dtype=np.float32))
    assert np.array_equal(w[192:256], np.arange(64, 128, dtype=np.float32))
    assert np.all(w[:64] == 0) and np.all(hu[:64] == 7.0)


def test_half_precision_copy_of_the_weights_follows_the_updated_ones():
    """Section 2.5: the update runs on FP32 values, forward and backward use FP16 parameters.  The
    FP16 copy is the new FP32 weight rounded once (numpy's float16 does the rounding here), only
    where a weight changed; everywhere else it keeps its bits.  One conversion per updated
    parameter: with every chunk important that is N of them, the paper's count for AlexNet."""
    rng = np.random.default_rng(5)
    N, C = 1000, 96
    nc = ob.n_chunks(N, C)
    for wire in ("f16", "f32"):
        sel = np.array(sorted(rng.choice(nc, size=4, replace=False)), dtype=np.int32)
        if nc - 1 not in sel:
            sel[-1] = nc - 1                                   # the short last chunk is among them
        L = ob.packed_len(N, C, sel)
        g = (rng.standard_normal(L) * 1e-5).astype(np.float32)  # small steps: the weights keep their binades
        red = ob.f32_to_f16(g) if wire == "f16" else g
        # weights over many binades, some beyond what FP16 holds, some below its smallest normal
        w = (rng.standard_normal(N) * 10.0 ** rng.integers(-9, 7, size=N)).astype(np.float32)
        hu = (rng.standard_normal(N) * 1e-7).astype(np.float32)
        w_half = np.full(N, 0x1234, dtype=np.uint16)
        w0 = w.copy()
        ob.sgd_update(red, N, C, sel, np.float32(0.5), 0.9, -0.25, w, hu, None, wire, w_half=w_half)
        touched = np.zeros(N, dtype=bool)
        for c in sel:
            touched[c * C:(c + 1) * C] = True
        assert np.array_equal(w[~touched], w0[~touched]) and not np.array_equal(w[touched], w0[touched])
        with np.errstate(over="ignore"):
            want = w.astype(np.float16).view(np.uint16)
        assert np.array_equal(w_half[touched], want[touched])
        assert np.all(w_half[~touched] == 0x1234)
        assert np.isinf(want[touched].view(np.float16)).any() and (np.abs(w[touched]) < 6e-5).any()
    # every chunk important: exactly N conversions
    sel = np.arange(nc, dtype=np.int32)
    w_half = np.zeros(N, dtype=np.uint16)
    w = rng.standard_normal(N).astype(np.float32)
    ob.sgd_update(ob.f32_to_f16(np.ones(N, dtype=np.float32)), N, C, sel, np.float32(1), 0.0, 1.0, w,
                  np.zeros(N, dtype=np.float32), None, "f16", w_half=w_half)
    assert np.array_equal(w_half, w.astype(np.float16).view(np.uint16))
