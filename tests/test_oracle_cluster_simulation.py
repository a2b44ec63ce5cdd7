"""A whole job written the way the paper describes it, as a pin of the checker's whole iteration:
P separate workers, each with its own gradient tensors and historical gradients, that meet only
in two exchanges per iteration -- the chunk-norm vector and the packed buffer, the latter passed
hop by hop around a ring (Section 2.4) -- and that each decide the important chunks on their own
(Section 3.2: every GPU must arrive at the same set).  Pure Python on tiny sizes, one element at
a time, numpy only for the roundings to fp32 / fp16; nothing here comes from the checker, and
the checker's iteration driver must reproduce every buffer of every worker bit for bit.
"""
import numpy as np
import pytest

from oracle import pipeline as op

f32 = np.float32


def to_wire(x, wire):
    return np.float16(x) if wire == "f16" else f32(x)


def hop_add(a, b, wire):
    """What a rank does with a received segment element: add its own, round to the wire type."""
    return to_wire(f32(a) + f32(b), wire)


class Worker:
    def __init__(self, rank, sizes):
        self.rank = rank
        self.N = sum(sizes)
        self.hg = [f32(0.0)] * self.N

    def place(self, tensors, sizes):
        """Section 3.1: tensor m is produced first and lies first in the pool."""
        pool = []
        for j in reversed(range(len(sizes))):
            pool.extend(f32(v) for v in tensors[j])
        return pool

    def accumulate(self, pool):
        self.acc = [f32(g + h) for g, h in zip(pool, self.hg)]          # Algorithm 1: g + hg

    def local_norms(self, C):
        out = []
        for lo in range(0, self.N, C):
            s = 0.0
            for v in self.acc[lo:lo + C]:
                s += abs(float(v))
            out.append(f32(s))
        return out

    def pack(self, sel, C, S, mu, wire):
        """Important chunks go to the send buffer in ascending order; Algorithm 1's two rules
        for the historical gradient."""
        self.send = []
        chosen = set(sel)
        for c in sel:
            for v in self.acc[c * C:(c + 1) * C]:
                self.send.append(to_wire(f32(v * f32(S)), wire))
        for c in range((self.N + C - 1) // C):
            for i in range(c * C, min(self.N, (c + 1) * C)):
                self.hg[i] = f32(0.0) if c in chosen else f32(f32(mu) * self.acc[i])


def ring_allreduce(workers, lo, hi, wire):
    """The ranks in `workers` (ring order) each hold buf[lo:hi]; n-1 reduce-scatter hops, n-1
    all-gather hops.  Segments: equal cuts rounded up to 16 bytes, the trailing ones short or empty."""
    P = len(workers)
    n = hi - lo
    per = -(-n // P)
    gran = 8 if wire == "f16" else 4
    seg = -(-per // gran) * gran
    bounds = [(lo + min(n, s * seg), lo + min(n, (s + 1) * seg)) for s in range(P)]
    for step in range(P - 1):                                   # reduce-scatter
        msgs = []
        for r, w in enumerate(workers):
            s = (r - step) % P
            a, b = bounds[s]
            msgs.append(((r + 1) % P, s, list(w.buf[a:b])))
        for dst, s, data in msgs:
            a, b = bounds[s]
            for i, v in enumerate(data):
                workers[dst].buf[a + i] = hop_add(v, workers[dst].buf[a + i], wire)
    for step in range(P - 1):                                   # all-gather: copies
        msgs = []
        for r, w in enumerate(workers):
            s = (r + 1 - step) % P
            a, b = bounds[s]
            msgs.append(((r + 1) % P, s, list(w.buf[a:b])))
        for dst, s, data in msgs:
            a, b = bounds[s]
            workers[dst].buf[a:b] = data


def allreduce(workers, lo, hi, wire, groups):
    """Flat ring, or Section 2.4's hierarchical allreduce: groups of consecutive ranks, the lowest
    rank of each its master; the partial sum travels from the rank after the master along the
    group to its last rank and from there to the master; the masters run the ring; the masters
    hand the result to their groups."""
    P = len(workers)
    if groups in (0, P):
        ring_allreduce(workers, lo, hi, wire)
        return
    G = P // groups
    masters = []
    for g in range(groups):
        members = workers[g * G:(g + 1) * G]
        chain = members[1:] + members[:1]
        for src, dst in zip(chain, chain[1:]):
            dst.buf[lo:hi] = [hop_add(v, own, wire) for v, own in zip(src.buf[lo:hi], dst.buf[lo:hi])]
        masters.append(members[0])
    ring_allreduce(masters, lo, hi, wire)
    for g in range(groups):
        for w in workers[g * G + 1:(g + 1) * G]:
            w.buf[lo:hi] = list(workers[g * G].buf[lo:hi])


def top_k(score, k):
    order = sorted(range(len(score)), key=lambda c: (-float(score[c]), c))   # ties: lower index first
    return sorted(order[:k])


def exchange_sum(contributions):
    """The small allreduce of the norm vector: rank 0's value first, double precision, stored single."""
    out = []
    for c in range(len(contributions[0])):
        s = 0.0
        for p in range(len(contributions)):
            s += float(contributions[p][c])
        out.append(f32(s))
    return out


def run_cluster(grads, sizes, C, k, S, mu, theta, wire, schedule, T, groups=0, ks=None):
    """grads[t][p][j]: tensor j (ID order) of worker p at iteration t.  Returns per iteration what
    every worker ended with."""
    P = len(grads[0])
    N = sum(sizes)
    nc = (N + C - 1) // C
    workers = [Worker(p, sizes) for p in range(P)]
    sel = None
    log = []
    for t in range(T):
        # ks: the number of important chunks per iteration (warm-up changes it); the chunks of
        # iteration t + 1 are chosen at the end of iteration t, ks[t + 1] of them
        k, k_after = (ks[t], ks[t + 1]) if ks else (k, k)
        for w in workers:
            w.accumulate(w.place(grads[t][w.rank], sizes))
        norms = [w.local_norms(C) for w in workers]
        if schedule == "immediate" or sel is None:
            sel = top_k(exchange_sum(norms), k)
        for w in workers:
            w.pack(sel, C, S, mu, wire)
            w.buf = list(w.send)
        L = len(workers[0].send)
        # lazy allreduce on the packed buffer: a bucket goes out once more than theta is waiting
        start, waited, pos = 0, 0, 0
        for c in sel:
            ln = min(N, (c + 1) * C) - c * C
            pos += ln
            waited += ln
            if waited > theta:
                allreduce(workers, start, pos, wire, groups)
                start, waited = pos, 0
        if waited:
            allreduce(workers, start, pos, wire, groups)
        assert pos == L
        for w in workers[1:]:
            assert [v.tobytes() for v in w.buf] == [v.tobytes() for v in workers[0].buf], "ranks disagree"
        # unpack on every worker; each one scores the chunks it received by their norm / P
        alpha = f32(1.0) / f32(S)
        out = {}
        shares = []
        for w in workers:
            red_norm, mine = {}, {}
            for j, c in enumerate(sel):
                s = 0.0
                for i in range(min(N, (c + 1) * C) - c * C):
                    v = f32(f32(w.buf[j * C + i]) * alpha)
                    mine[c * C + i] = v
                    s += abs(float(v))
                red_norm[c] = f32(s)
            out = mine
            shares.append([float(red_norm[c]) / P if c in red_norm else float(norms[w.rank][c]) for c in range(nc)])
        entry = dict(sel=list(sel), send=[list(w.send) for w in workers], reduced=list(workers[0].buf), out=out,
                     hg=[list(w.hg) for w in workers])
        if schedule == "lagged":
            score = exchange_sum(shares)
            entry["score_post"] = score
            sel = top_k(score, k_after)
            entry["sel_next"] = list(sel)
        log.append(entry)
    return log


def bits(values, dtype):
    return np.array(values, dtype=dtype).tobytes()


@pytest.mark.parametrize("schedule", ["lagged", "immediate"])
@pytest.mark.parametrize("wire", ["f16", "f32"])
@pytest.mark.parametrize("P,sizes,C,k,S,mu,theta", [
    (3, [7, 13, 5], 4, 3, 128.0, 1.0, 1 << 60),      # 7 chunks, the last one a single element
    (4, [9, 2, 30], 8, 2, 3.0, 0.5, 1 << 60),        # loss scale that is no power of two, momentum factor
    (2, [5, 5, 5, 6], 3, 5, 1024.0, 1.0, 5),         # several packed buckets, each its own ring
    (5, [64], 16, 4, 1.0, 1.0, 16),                  # every chunk sent, more ranks than 16-byte groups per bucket
    (1, [11, 6], 4, 2, 8.0, 1.0, 1 << 60),           # one worker: the ring is the identity
])
def test_checker_iteration_equals_the_cluster_simulation(P, sizes, C, k, S, mu, theta, wire, schedule):
    rng = np.random.default_rng(P * 1000 + len(sizes))
    T = 4
    scale = [10.0 ** rng.uniform(-3, 0) for _ in sizes]
    grads = [[[(rng.standard_normal(n) * scale[j]).astype(np.float32) for j, n in enumerate(sizes)]
              for _ in range(P)] for _ in range(T)]
    log = run_cluster(grads, sizes, C, k, S, mu, theta, wire, schedule, T)

    N = sum(sizes)
    wt = np.float16 if wire == "f16" else np.float32
    st = op.new_state(P, N)
    for t in range(T):
        pools = np.stack([op.fuse(grads[t][p], sizes) for p in range(P)])
        out = np.full(N, np.float32(-7.0))
        r = op.csc_iteration(st, pools, C, k, S, mu, schedule, wire, out=out, theta=theta)
        e = log[t]
        assert list(r["sel"]) == e["sel"], f"t={t} selection"
        for p in range(P):
            assert np.ascontiguousarray(r["send"][p]).tobytes() == bits(e["send"][p], wt), f"t={t} send of worker {p}"
            assert st.hg[p].tobytes() == bits(e["hg"][p], np.float32), f"t={t} historical gradient of worker {p}"
        assert np.ascontiguousarray(r["reduced"]).tobytes() == bits(e["reduced"], wt), f"t={t} reduced"
        want = np.full(N, np.float32(-7.0))
        for i, v in e["out"].items():
            want[i] = v
        assert out.tobytes() == want.tobytes(), f"t={t} output"
        if schedule == "lagged":
            assert np.asarray(r["score_post"], dtype=np.float32).tobytes() == bits(e["score_post"], np.float32), f"t={t} scores"
            assert list(r["sel_next"]) == e["sel_next"], f"t={t} next selection"


@pytest.mark.parametrize("wire", ["f16", "f32"])
@pytest.mark.parametrize("P,groups", [(4, 2), (6, 3), (6, 2), (4, 1)])
def test_checker_iteration_with_the_hierarchical_allreduce(P, groups, wire):
    rng = np.random.default_rng(P * 10 + groups)
    sizes, C, k, S, T = [21, 9, 14], 6, 3, 64.0, 3
    grads = [[[rng.standard_normal(n).astype(np.float32) for n in sizes] for _ in range(P)] for _ in range(T)]
    log = run_cluster(grads, sizes, C, k, S, 1.0, 13, wire, "lagged", T, groups)
    wt = np.float16 if wire == "f16" else np.float32
    st = op.new_state(P, sum(sizes))
    for t in range(T):
        pools = np.stack([op.fuse(grads[t][p], sizes) for p in range(P)])
        r = op.csc_iteration(st, pools, C, k, S, 1.0, "lagged", wire, theta=13, groups=groups)
        assert list(r["sel"]) == log[t]["sel"] and list(r["sel_next"]) == log[t]["sel_next"]
        assert np.ascontiguousarray(r["reduced"]).tobytes() == bits(log[t]["reduced"], wt), f"t={t} reduced"
        for p in range(P):
            assert st.hg[p].tobytes() == bits(log[t]["hg"][p], np.float32)


@pytest.mark.parametrize("wire", ["f16", "f32"])
@pytest.mark.parametrize("theta", [0, 10, 30, 1 << 60])
def test_checker_dense_iteration_equals_the_cluster_simulation(theta, wire):
    """Lazy allreduce without sparsification (Section 3.1): tensors arrive in the order m..1, a
    bucket goes out when more than theta is waiting, every bucket a ring of its own."""
    rng = np.random.default_rng(theta % 97)
    P, sizes, S = 3, [12, 3, 20, 7, 9], 256.0
    N = sum(sizes)
    grads = [[(rng.standard_normal(n) * 0.1).astype(np.float32) for n in sizes] for _ in range(P)]
    workers = [Worker(p, sizes) for p in range(P)]
    for w in workers:
        w.buf = [to_wire(f32(v * f32(S)), wire) for v in w.place(grads[w.rank], sizes)]
    sent = [list(w.buf) for w in workers]
    start, waited, pos = 0, 0, 0
    for j in reversed(range(len(sizes))):
        pos += sizes[j]
        waited += sizes[j]
        if waited > theta:
            ring_allreduce(workers, start, pos, wire)
            start, waited = pos, 0
    if waited:
        ring_allreduce(workers, start, pos, wire)
    alpha = f32(1.0) / f32(S)
    want_out = [f32(f32(v) * alpha) for v in workers[-1].buf]

    r = op.dense_iteration(np.stack([op.fuse(grads[p], sizes) for p in range(P)]), sizes, theta, S, wire)
    wt = np.float16 if wire == "f16" else np.float32
    for p in range(P):
        assert np.ascontiguousarray(r["send"][p]).tobytes() == bits(sent[p], wt)
    assert np.ascontiguousarray(r["reduced"]).tobytes() == bits(workers[0].buf, wt)
    assert r["out"].tobytes() == bits(want_out, np.float32)


def test_checker_iterations_through_a_warm_up_ramp():
    """Warm-up dense training (Section 3.2): the sparsity ratio ramps linearly from zero, so the
    number of important chunks shrinks from all of them; the count of iteration t + 1 is what the
    selection at the end of iteration t takes."""
    from oracle import binding as ob
    rng = np.random.default_rng(11)
    P, sizes, C, S, T = 3, [30, 50, 21], 5, 32.0, 6
    nc = -(-sum(sizes) // C)
    ks = [ob.warmup_k(nc, 0.2, t, 4) for t in range(T + 1)]
    assert ks[0] == nc and ks[4] == ks[5] == -(-nc // 5) and sorted(ks, reverse=True) == ks     # dense first, then the ramp
    grads = [[[rng.standard_normal(n).astype(np.float32) for n in sizes] for _ in range(P)] for _ in range(T)]
    log = run_cluster(grads, sizes, C, None, S, 1.0, 12, "f16", "lagged", T, ks=ks)
    st = op.new_state(P, sum(sizes))
    for t in range(T):
        pools = np.stack([op.fuse(grads[t][p], sizes) for p in range(P)])
        r = op.csc_iteration(st, pools, C, ks[t], S, 1.0, "lagged", "f16", k_next=ks[t + 1], theta=12)
        assert list(r["sel"]) == log[t]["sel"] and len(r["sel"]) == ks[t], f"t={t}"
        assert list(r["sel_next"]) == log[t]["sel_next"] and len(r["sel_next"]) == ks[t + 1], f"t={t}"
        assert np.ascontiguousarray(r["reduced"]).tobytes() == bits(log[t]["reduced"], np.float16), f"t={t}"
        for p in range(P):
            assert st.hg[p].tobytes() == bits(log[t]["hg"][p], np.float32), f"t={t}"


def test_the_simulation_itself_sums_what_it_should():
    """Integers small enough that no rounding happens anywhere: after the ring every rank holds
    the plain sum, whatever the order, so a wrong segment walk or a lost hop shows."""
    P, n = 4, 37
    workers = [Worker(p, [n]) for p in range(P)]
    for w in workers:
        w.buf = [np.float16((w.rank + 1) * (i % 7)) for i in range(n)]
    ring_allreduce(workers, 3, n, "f16")
    for w in workers:
        assert [float(v) for v in w.buf[3:]] == [float(10 * (i % 7)) for i in range(3, n)]
        assert [float(v) for v in w.buf[:3]] == [float((w.rank + 1) * i) for i in range(3)]


def test_every_worker_applies_the_same_update():
    """Algorithm 1's SGD-update step inside the job: every worker updates its own copy of the
    weights from the chunks it received; the copies stay identical (they all hold the same reduced
    values) and equal the checker's, whose update runs once."""
    from oracle import binding as ob
    rng = np.random.default_rng(21)
    P, sizes, C, k, S, T = 3, [17, 40, 9], 6, 4, 16.0, 5
    N = sum(sizes)
    momentum, lr = f32(0.9), f32(-0.1)
    alpha = f32(1.0) / f32(S)
    grads = [[[rng.standard_normal(n).astype(np.float32) for n in sizes] for _ in range(P)] for _ in range(T)]
    log = run_cluster(grads, sizes, C, k, S, 1.0, 1 << 60, "f16", "lagged", T)
    w0 = rng.standard_normal(N).astype(np.float32)
    copies = [dict(w=[f32(v) for v in w0], hu=[f32(0.0)] * N) for _ in range(P)]
    w_ref, hu_ref = w0.copy(), np.zeros(N, dtype=np.float32)
    for t in range(T):
        red = np.array(log[t]["reduced"], dtype=np.float16)
        for cp in copies:                                     # what each worker does on its own
            for j, c in enumerate(log[t]["sel"]):
                for i in range(min(N, (c + 1) * C) - c * C):
                    g = f32(f32(red[j * C + i]) * alpha)
                    e = c * C + i
                    cp["hu"][e] = f32(f32(momentum * cp["hu"][e]) + f32(lr * g))
                    cp["w"][e] = f32(cp["w"][e] + cp["hu"][e])
        ob.sgd_update(red.view(np.uint16), N, C, np.array(log[t]["sel"], dtype=np.int32), alpha, momentum, lr,
                      w_ref, hu_ref)
        for cp in copies:
            assert bits(cp["w"], np.float32) == w_ref.tobytes() and bits(cp["hu"], np.float32) == hu_ref.tobytes(), f"t={t}"
    assert not np.array_equal(w_ref, w0)
