"""Pins for the CPU checker's single-precision wire (Section 2.3: the baseline
sends fp32 gradients): every routine that branches on the wire type is checked
here on its fp32 branch against numpy's fp32 arithmetic, closed forms, and the
conservation property stated with Algorithm 1.  The fp16 branches are pinned in
test_oracle_csc.py / test_oracle_sgd.py / test_oracle_ring.py."""
import json
import os

import numpy as np
import pytest

from oracle import binding as ob, pipeline as op
from paper_1902_06855_amd import workloads as wl

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_facts.json")))
F = np.float32


def _pools(w, t, integer=False):
    g = wl.integer_gradients(w.sizes, w.P, seed=w.seed + t) if integer else wl.gradients(w, t)
    return np.stack([op.fuse([x.numpy() for x in row], w.sizes) for row in g])


def small(P=3, C=96, density=0.3, sizes=(50, 8, 700, 33, 1200, 64, 5), S=64.0):
    return wl.Workload("small32", list(sizes), P=P, chunk=C, density=density, loss_scale=S,
                       theta=1 << 40, wire="f32")


# ------------------------------------------------- pack + historical gradient

@pytest.mark.parametrize("mu", [1.0, 0.9])
@pytest.mark.parametrize("S", [64.0, 3.0])          # 3.0: acc * S is rounded, not exact
def test_pack_on_the_fp32_wire_sends_the_scaled_sum_and_clears_or_keeps_the_history(mu, S):
    w = small(S=S)
    pools = _pools(w, 0)
    hg0 = (_pools(w, 1) * 0.5).astype(F)
    acc = ob.accumulate(pools, hg0)
    nc = ob.n_chunks(w.N, w.chunk)
    sel = np.array([1, 2, 7, nc - 1], dtype=np.int32)        # includes the short last chunk
    send, hg = ob.pack_residual(acc, w.chunk, sel, S, mu, wire="f32")
    L = 3 * w.chunk + (w.N - (nc - 1) * w.chunk)
    assert send.dtype == F and send.shape == (w.P, L)
    sent = np.zeros(w.N, dtype=bool)
    slot = 0
    for c in sel:
        lo, hi = c * w.chunk, min(w.N, (c + 1) * w.chunk)
        sent[lo:hi] = True
        want = acc[:, lo:hi] * F(S)                         # one fp32 multiply, nothing else
        assert np.array_equal(send[:, slot:slot + hi - lo].view(np.uint32), want.view(np.uint32))
        slot += hi - lo
    assert slot == L
    # Algorithm 1: hg = 0 where the gradient is important (a plain +0), momentum * g elsewhere
    assert np.all(hg[:, sent].view(np.uint32) == 0)
    assert np.array_equal(hg[:, ~sent].view(np.uint32), (F(mu) * acc[:, ~sent]).view(np.uint32))
    # the fp32 wire keeps what fp16 would round away
    half, _ = ob.pack_residual(acc, w.chunk, sel, S, mu, wire="f16")
    assert not np.array_equal(ob.f16_to_f32(half), send)
    if S == 64.0 and mu == 1.0:                              # power of two: the round trip is exact
        assert np.array_equal(send / F(S), acc[:, sent])


def test_dense_cast_on_the_fp32_wire_is_one_multiply():
    rng = np.random.default_rng(5)
    g = (rng.standard_normal((3, 1001)) * 1e-2).astype(F)
    for S in (1.0, 128.0, 3.0):
        send = ob.cast_dense(g, S, wire="f32")
        assert send.dtype == F and np.array_equal(send.view(np.uint32), (g * F(S)).view(np.uint32))
    assert np.array_equal(ob.cast_dense(g, 1.0, wire="f32"), g)


# --------------------------------------------------------------------- unpack

def test_unpack_on_the_fp32_wire():
    rng = np.random.default_rng(6)
    N, C = 1000 - 30, 100                         # 10 chunks, the last one holds 70
    sel = np.array([0, 4, 9], dtype=np.int32)
    red = (rng.standard_normal(270) * 3).astype(F)
    alpha = F(1) / F(3.0)
    out = np.full(N, F(-7.0))
    norms = ob.unpack(red, N, C, sel, alpha, out, wire="f32")
    want = red * alpha
    assert np.array_equal(out[0:100].view(np.uint32), want[0:100].view(np.uint32))
    assert np.array_equal(out[400:500].view(np.uint32), want[100:200].view(np.uint32))
    assert np.array_equal(out[900:970].view(np.uint32), want[200:270].view(np.uint32))
    untouched = np.ones(N, dtype=bool)
    for a, b in ((0, 100), (400, 500), (900, 970)):
        untouched[a:b] = False
    assert np.all(out[untouched] == F(-7.0))
    for j, (a, b) in enumerate(((0, 100), (100, 200), (200, 270))):
        assert norms[j] == pytest.approx(np.abs(want[a:b].astype(np.float64)).sum(), rel=1e-6)
    # a value that fp16 cannot hold comes back unchanged
    tiny = np.array([1.0 + 2.0 ** -20] * 8, dtype=F)
    o = np.zeros(8, dtype=F)
    ob.unpack(tiny, 8, 8, np.array([0], dtype=np.int32), 1.0, o, wire="f32")
    assert np.array_equal(o, tiny)


def test_unpack_dense_on_the_fp32_wire():
    rng = np.random.default_rng(7)
    red = rng.standard_normal(513).astype(F)
    for alpha in (F(1.0), F(1) / F(128.0), F(1) / F(3.0)):
        got = ob.unpack_dense(red, alpha, wire="f32")
        assert np.array_equal(got.view(np.uint32), (red * alpha).view(np.uint32))


# ----------------------------------------------------------------- SGD update

def test_sgd_update_on_the_fp32_wire_is_textbook_momentum_sgd():
    rng = np.random.default_rng(8)
    N, C = 1000, 128
    sel = np.arange(ob.n_chunks(N, C), dtype=np.int32)
    m, lr, alpha = F(0.9), F(-0.05), F(1) / F(3.0)
    w = rng.standard_normal(N).astype(F)
    hu = np.zeros(N, dtype=F)
    w_ref, v_ref = w.copy(), hu.copy()
    for t in range(5):
        red = (rng.standard_normal(N) * 0.01).astype(F)
        out = np.zeros(N, dtype=F)
        ob.sgd_update(red, N, C, sel, alpha, m, lr, w, hu, out, wire="f32")
        g = red * alpha
        assert np.array_equal(out.view(np.uint32), g.view(np.uint32))
        v_ref = (m * v_ref).astype(F) + (lr * g).astype(F)
        w_ref = w_ref + v_ref
        assert np.array_equal(hu.view(np.uint32), v_ref.view(np.uint32))
        assert np.array_equal(w.view(np.uint32), w_ref.view(np.uint32))


def test_sgd_update_on_the_fp32_wire_closed_form_and_untouched_chunks():
    # constant gradient, powers of two: hu_T = lr*g*(1 - m^T)/(1 - m) exactly, w_T = w_0 + sum_t hu_t
    N, C = 64, 16
    sel = np.array([0, 2], dtype=np.int32)
    red = np.full(32, 0.125, dtype=F)
    w = np.ones(N, dtype=F)
    hu = np.zeros(N, dtype=F)
    total = 0.0
    for T in range(1, 8):
        ob.sgd_update(red, N, C, sel, 1.0, 0.5, -0.25, w, hu, wire="f32")
        want = -0.25 * 0.125 * (1 - 0.5 ** T) / (1 - 0.5)
        total += want
        for a in (0, 32):
            assert np.all(hu[a:a + 16] == F(want)) and np.all(w[a:a + 16] == F(1.0 + total))
        for a in (16, 48):                                  # hu_t = hu_{t-1}, no update
            assert np.all(hu[a:a + 16] == 0) and np.all(w[a:a + 16] == 1)


# ------------------------------------------------------------ whole iterations

@pytest.mark.parametrize("schedule", ["immediate", "lagged"])
def test_no_gradient_is_lost_over_iterations_on_the_fp32_wire(schedule):
    """Algorithm 1 with momentum 1 (the paper: CSC loses no learned information):
    sent + still held back = everything ever computed.  Small integers, loss
    scale 1: every sum is exact in fp32, whatever the order."""
    w = small(P=4, C=64, density=0.2)
    k = w.k_for(ob.n_chunks(w.N, w.chunk))
    st = op.new_state(w.P, w.N)
    total_in = np.zeros(w.N, dtype=np.float64)
    total_out = np.zeros(w.N, dtype=np.float64)
    for t in range(7):
        pools = _pools(w, t, integer=True)
        total_in += pools.astype(np.float64).sum(axis=0)
        out = np.zeros(w.N, dtype=F)
        r = op.csc_iteration(st, pools, w.chunk, k, 1.0, 1.0, schedule, wire="f32", out=out)
        assert r["send"].dtype == F and r["reduced"].dtype == F
        total_out += out
        held = st.hg.astype(np.float64).sum(axis=0)
        assert np.array_equal(total_out + held, total_in)
    assert np.abs(total_out).sum() > 0 and np.abs(held).sum() > 0


def test_sending_every_chunk_on_the_fp32_wire_equals_the_dense_path_and_the_plain_sum():
    w = small(P=4, C=100, density=1.0, S=1.0)
    nc = ob.n_chunks(w.N, w.chunk)
    st = op.new_state(w.P, w.N)
    pools = _pools(w, 0, integer=True)
    r = op.csc_iteration(st, pools, w.chunk, nc, 1.0, 1.0, "immediate", wire="f32")
    d = op.dense_iteration(pools, w.sizes, 1 << 40, 1.0, wire="f32")
    assert np.all(st.hg == 0)
    assert np.array_equal(r["send"], d["send"]) and np.array_equal(r["out"], d["out"])
    assert np.array_equal(d["out"], pools.sum(axis=0))       # integers: the exact sum
    # real-valued data: within fp32 rounding of the fp64 sum, far closer than the fp16 wire gets
    pools = _pools(w, 1)
    d32 = op.dense_iteration(pools, w.sizes, 1 << 40, 1.0, wire="f32")
    exact = pools.astype(np.float64).sum(axis=0)
    scale = np.abs(pools.astype(np.float64)).sum(axis=0)
    assert np.all(np.abs(d32["out"] - exact) <= scale * 4 * 2.0 ** -24)


# ----------------------------------------------- facts about the number of casts

def test_one_conversion_each_way_per_gradient():
    # Section 2.5: an iteration of mixed-precision AlexNet training needs one fp32->fp16 and one
    # fp16->fp32 conversion per parameter (60.9M each way): the dense path casts every element of
    # the pool once per worker and widens every reduced element once
    fact = GOLD["conversions"]
    a = wl.config("alexnet_dense")
    assert int(a.N / 1e5) / 10 == fact["params"] / 1e6       # 60 965 224 parameters print as 60.9M
    w = wl.scaled(a, 1024)
    pools = _pools(w, 0)
    d = op.dense_iteration(pools, w.sizes, w.theta, w.loss_scale)
    assert d["send"].shape == (w.P, w.N) and d["send"].dtype == np.uint16     # N casts per worker
    assert d["reduced"].shape == (w.N,) and d["out"].shape == (w.N,) and d["out"].dtype == F


# ------------------------------------------- rounding of the important-chunk count

def test_chunk_count_of_a_density_is_a_guarded_ceiling():
    """The number of important chunks is ceil(density * n_chunks).  The product is formed in
    double precision and can land an ulp above the integer it stands for ((1 - 0.09*2) * 1000 =
    820.0000000000001, 0.07 * 100 = 7.000000000000001); a bare ceiling would then take one chunk
    too many.  The checker subtracts 1e-9 before the ceiling.  Hand-worked values."""
    import math
    assert math.ceil((1 - 0.9 * 2 / 10) * 1000) == 821 and math.ceil((1 - 0.9 * 9 / 10) * 1000) == 191
    assert ob.warmup_k(1000, 0.1, 2, 10) == 820 and ob.warmup_k(1000, 0.1, 9, 10) == 190
    assert math.ceil(0.07 * 100) == 8 and ob.warmup_k(100, 0.07, 0, 0) == 7
    assert ob.warmup_k(700, 0.07, 5, 0) == 49 and ob.warmup_k(50, 0.14, 0, 0) == 7
    # a genuine fraction still rounds up
    assert ob.warmup_k(1861, 0.1, 0, 0) == 187 and ob.warmup_k(3120, 0.01, 0, 0) == 32
    assert ob.warmup_k(245, 0.25, 0, 0) == 62 and ob.warmup_k(1000, 0.1001, 0, 0) == 101
