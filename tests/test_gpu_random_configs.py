"""Seeded random configurations of the whole path on the GPU against the CPU checker: tensor
counts and sizes, worker counts, chunk lengths on both sides of the sub-tile length, thresholds,
wire and gradient types, schedules, input layouts and allreduce orders drawn together, so that
combinations no hand-written case names still get exercised."""
import numpy as np
import pytest
import torch

from oracle import binding as ob, pipeline as op
from paper_1902_06855_amd import workloads as wl

from test_gpu_parity import same_bits, gfm  # noqa: F401  (gfm is a fixture)

pytestmark = pytest.mark.gpu


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    kinds = [lambda: int(rng.integers(1, 50)), lambda: int(rng.integers(100, 5000)),
             lambda: int(8192 + rng.integers(-9, 10)), lambda: int(rng.integers(20000, 70000)),
             lambda: int(rng.integers(1, 9)) * 4096]
    m = int(rng.integers(1, 13))
    sizes = [kinds[int(rng.integers(0, len(kinds)))]() for _ in range(m)]
    P = int(rng.choice([1, 2, 3, 4, 6, 8, 12]))
    groups = int(rng.choice([0] + [d for d in range(1, P + 1) if P % d == 0]))
    chunk = int(rng.choice([0, 0, 64, 1000, 4096, 8192, 8200, 20000, 32768, 50001]))
    N = sum(sizes)
    theta = int(rng.choice([0, 100, N // 3 + 1, 1 << 40]))
    cfg = dict(sizes=sizes, P=P, groups=groups, chunk=chunk, theta=theta,
               wire=str(rng.choice(["f16", "f16", "f32"])), grad=str(rng.choice(["f32", "f16"])),
               schedule=str(rng.choice(["lagged", "immediate"])), mode=str(rng.choice(["gather", "pool"])),
               S=float(rng.choice([1.0, 128.0, 1000.0])), mu=float(rng.choice([1.0, 1.0, 0.5])),
               density=float(rng.choice([0.05, 0.3, 1.0])))
    return cfg


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration(gfm, seed):
    gf, pl = gfm
    c = _draw(seed)
    w = wl.Workload(f"random{seed}", c["sizes"], P=c["P"], chunk=c["chunk"], density=c["density"],
                    loss_scale=c["S"], theta=c["theta"], mu=c["mu"], seed=seed, wire=c["wire"])
    nc = ob.n_chunks(w.N, w.chunk) if w.chunk else 0
    k = w.k_for(nc) if w.chunk else 0
    pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=k, mu=w.mu, wire=w.wire,
                       schedule=c["schedule"], grad=c["grad"], groups=c["groups"], fast=bool(seed % 2))
    st = op.new_state(w.P, w.N)
    it, nt = (torch.int16, np.int16) if w.wire == "f16" else (torch.int32, np.int32)
    what = f"seed {seed}: {c}"
    for t in range(3 if w.chunk else 1):
        g = wl.gradients(w, t)                                               # fp32, CPU
        if c["grad"] == "f16":
            g = [[x.to(torch.float16) for x in row] for row in g]
            exact = [[torch.from_numpy(ob.f16_to_f32(x.numpy().view(np.uint16))) for x in row] for row in g]
        else:
            exact = g
        pools = np.stack([op.fuse([x.numpy() for x in row], w.sizes) for row in exact])
        if c["mode"] == "gather":
            pipe.set_gradients([[x.cuda() for x in row] for row in g])
        else:
            pipe.set_pools([torch.cat([x for x in reversed(row)]).cuda() for row in g])
        pipe.out_pool.fill_(-3.0)
        pipe.step()
        torch.cuda.synchronize()
        if w.chunk:
            out = np.full(w.N, np.float32(-3.0))
            r = op.csc_iteration(st, pools, w.chunk, k, w.loss_scale, w.mu, c["schedule"], w.wire, out=out,
                                 theta=w.theta, groups=c["groups"])
            L = r["send"].shape[1]
            assert int(pipe.packed_len.item()) == ob.packed_len(w.N, w.chunk, pipe.sel.cpu().numpy()), what
            same_bits(pipe.reduced[:L].view(it), r["reduced"].view(nt), f"{what} t={t} reduced")
            same_bits(pipe.out_pool, out, f"{what} t={t} out")
            for p in range(w.P):
                same_bits(pipe.residual[p], st.hg[p], f"{what} t={t} hg[{p}]")
            nxt = r["sel_next"] if c["schedule"] == "lagged" else r["sel"]
            assert np.array_equal(pipe.sel.cpu().numpy(), nxt), f"{what} t={t} selection"
        else:
            r = op.dense_iteration(pools, w.sizes, w.theta, w.loss_scale, w.wire, groups=c["groups"])
            for p in range(w.P):
                same_bits(pipe.send[p].view(it), r["send"][p].view(nt), f"{what} send[{p}]")
            same_bits(pipe.reduced.view(it), r["reduced"].view(nt), f"{what} reduced")
            same_bits(pipe.out_pool, r["out"], f"{what} out")
