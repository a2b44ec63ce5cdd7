"""Seeded random configurations of the whole path on the GPU against the CPU checker: tensor
counts and sizes, worker counts up to 64, chunk lengths from a few elements (multiples of four or
not) to several sub-tiles, thresholds (also exactly at a bucket border), wire and gradient types,
schedules, input layouts (also tensors that are only 2- or 4-byte aligned), allreduce orders,
all-gather copies, per-tensor outputs, the SGD-update step and the warm-up ramp, drawn together,
so that combinations no hand-written case names still get exercised.  Run with -x: the first
failing draw stops the run and its message holds the whole configuration."""
import numpy as np
import pytest
import torch

from oracle import binding as ob, pipeline as op
from paper_1902_06855_amd import workloads as wl

from test_gpu_parity import same_bits, gfm  # noqa: F401  (gfm is a fixture)

N_DRAWS = 200
BUDGET = 1_500_000          # P * N elements per draw at most: the checker stays fast


def _draw(seed):
    rng = np.random.default_rng(1000 + seed)
    P = int(rng.choice([1, 2, 3, 4, 6, 8, 12, 16, 32, 64]))
    kinds = [lambda: int(rng.integers(1, 50)), lambda: int(rng.integers(100, 5000)),
             lambda: int(8192 + rng.integers(-9, 10)), lambda: int(rng.integers(20000, 70000)),
             lambda: int(rng.integers(1, 9)) * 4096]
    m = int(rng.integers(1, 13))
    sizes = [kinds[int(rng.integers(0, len(kinds)))]() for _ in range(m)]
    while P * sum(sizes) > BUDGET and max(sizes) > 64:           # shrink the largest tensor
        i = int(np.argmax(sizes))
        sizes[i] = max(64, sizes[i] // 2 + int(rng.integers(0, 5)))
    N = sum(sizes)
    groups = int(rng.choice([0] + [d for d in range(1, P + 1) if P % d == 0]))
    chunk = int(rng.choice([0, 0, 8, 13, 30, 64, 250, 1000, 1022, 4096, 8192, 8200, 20000, 32768, 50001]))
    # thresholds: none, tiny, a third of the pool, and exactly at / one short of a border of the
    # waited size (the strict "greater than" of the rule)
    edges = np.cumsum(sizes[::-1]) if chunk == 0 else np.arange(1, 6) * max(chunk, 1)
    border = int(edges[int(rng.integers(0, len(edges)))])
    theta = int(rng.choice([0, 100, N // 3 + 1, 1 << 40, border, max(0, border - 1)]))
    wire = str(rng.choice(["f16", "f16", "f32"]))
    grad = str(rng.choice(["f32", "f32", "f16"]))
    schedule = str(rng.choice(["lagged", "lagged", "immediate"]))
    cfg = dict(sizes=sizes, P=P, groups=groups, chunk=chunk, theta=theta, wire=wire, grad=grad, schedule=schedule,
               mode=str(rng.choice(["gather", "pool"])), S=float(rng.choice([1.0, 128.0, 1000.0])),
               mu=float(rng.choice([1.0, 1.0, 0.5])), density=float(rng.choice([0.05, 0.3, 0.3, 1.0])),
               allgather=bool(rng.integers(0, 2)), scatter=bool(rng.integers(0, 2)),
               sgd=bool(rng.integers(0, 3) == 0), odd_address=bool(rng.integers(0, 3) == 0),
               half=bool(seed % 3 == 0),                          # with sgd: also the FP16 copy of the weights
               boost_last=bool(rng.integers(0, 2)),              # pushes the short last chunk into the selection
               warmup=int(rng.choice([0, 0, 3])) if (chunk and schedule == "lagged") else 0,
               fast=bool(seed % 2))
    return cfg


def _on_device(t: torch.Tensor, odd: bool) -> torch.Tensor:
    """A device copy of t; with `odd` it starts one element past a 256-byte aligned address, i.e.
    it has only the natural alignment of its element type."""
    if not odd:
        return t.cuda()
    buf = torch.empty(t.numel() + 1, dtype=t.dtype, device="cuda")
    buf[1:].copy_(t)
    return buf[1:]


@pytest.mark.gpu
@pytest.mark.parametrize("seed", range(N_DRAWS))
def test_random_configuration(gfm, seed):
    gf, pl = gfm
    c = _draw(seed)
    w = wl.Workload(f"random{seed}", c["sizes"], P=c["P"], chunk=c["chunk"], density=c["density"],
                    loss_scale=c["S"], theta=c["theta"], mu=c["mu"], seed=seed, wire=c["wire"])
    what = f"seed {seed}: {c}"
    nc = ob.n_chunks(w.N, w.chunk) if w.chunk else 0
    T = 3 if w.chunk else 1
    if c["warmup"]:
        ks = [ob.warmup_k(nc, c["density"], t, c["warmup"]) for t in range(T + 1)]
    else:
        ks = [w.k_for(nc) if w.chunk else 0] * (T + 1)
    mom, lr = 0.9, -0.125
    pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=ks[0], k_max=max(ks), mu=w.mu, wire=w.wire,
                       schedule=c["schedule"], grad=c["grad"], groups=c["groups"], fast=c["fast"],
                       allgather=c["allgather"], scatter_out=c["scatter"], sgd=(mom, lr) if c["sgd"] else None,
                       half_weights=c["sgd"] and c["half"])
    st = op.new_state(w.P, w.N)
    it, nt = (torch.int16, np.int16) if w.wire == "f16" else (torch.int32, np.int32)
    alpha = np.float32(1.0) / np.float32(w.loss_scale)
    w_ref = np.random.default_rng(seed).standard_normal(w.N).astype(np.float32)
    hu_ref = np.zeros(w.N, dtype=np.float32)
    half = c["sgd"] and c["half"]
    w16_ref = np.full(w.N, 0x3C00, dtype=np.uint16) if half else None       # ones, where never updated
    if half:
        for x in (pipe.w16 if c["scatter"] else [pipe.w16]):
            x.fill_(1.0)
    if c["sgd"]:
        if c["scatter"]:
            for j, v in enumerate(op.views(w_ref, w.sizes)):
                pipe.w[j].copy_(torch.from_numpy(np.ascontiguousarray(v)))
        else:
            pipe.w.copy_(torch.from_numpy(w_ref))

    for t in range(T):
        g = wl.gradients(w, t)                                               # fp32, CPU
        if c["boost_last"]:
            for row in g:
                row[0].mul_(50.0)                                            # tensor 1 ends the pool
        if c["grad"] == "f16":
            g = [[x.to(torch.float16) for x in row] for row in g]
            exact = [[torch.from_numpy(ob.f16_to_f32(x.numpy().view(np.uint16))) for x in row] for row in g]
        else:
            exact = g
        pools = np.stack([op.fuse([x.numpy() for x in row], w.sizes) for row in exact])
        if c["mode"] == "gather":
            pipe.set_gradients([[_on_device(x, c["odd_address"]) for x in row] for row in g])
        else:
            pipe.set_pools([_on_device(torch.cat([x for x in reversed(row)]), c["odd_address"]) for row in g])
        pipe.out_pool.fill_(-3.0)
        if c["scatter"]:
            for ot in pipe.out_tensors:
                ot.fill_(-3.0)
        pipe.k_next = ks[t + 1]
        if c["warmup"] and t == 0:
            # the first iteration selects twice: for itself (k of iteration 0), then for iteration 1
            pipe.k_next = ks[0]
            pipe.accum(); pipe.select(False); pipe.pack(); pipe.ring(); pipe.unpack()
            pipe.k_next = ks[1]
            pipe.select(True)
            pipe.t = 1
        else:
            pipe.step()
        torch.cuda.synchronize()
        if w.chunk:
            out = np.full(w.N, np.float32(-3.0))
            r = op.csc_iteration(st, pools, w.chunk, ks[t], w.loss_scale, w.mu, c["schedule"], w.wire, out=out,
                                 k_next=ks[t + 1], theta=w.theta, groups=c["groups"])
            L = r["send"].shape[1]
            nxt = r["sel_next"] if c["schedule"] == "lagged" else r["sel"]
            assert np.array_equal(pipe.sel.cpu().numpy()[:len(nxt)], nxt), f"{what} t={t} selection"
            assert int(pipe.packed_len.item()) == ob.packed_len(w.N, w.chunk, nxt), what
            for p in range(w.P):
                same_bits(pipe.send[p][:L].view(it), r["send"][p].view(nt), f"{what} t={t} send[{p}]")
                same_bits(pipe.residual[p], st.hg[p], f"{what} t={t} hg[{p}]")
            same_bits(pipe.reduced[:L].view(it), r["reduced"].view(nt), f"{what} t={t} reduced")
            same_bits(pipe.out_pool, out, f"{what} t={t} out")
            sel_used, red = r["sel"], r["reduced"]
        else:
            r = op.dense_iteration(pools, w.sizes, w.theta, w.loss_scale, w.wire, groups=c["groups"])
            L = w.N
            for p in range(w.P):
                same_bits(pipe.send[p].view(it), r["send"][p].view(nt), f"{what} send[{p}]")
            same_bits(pipe.reduced.view(it), r["reduced"].view(nt), f"{what} reduced")
            same_bits(pipe.out_pool, r["out"], f"{what} out")
            out, red, sel_used = r["out"], r["reduced"], None
        if c["allgather"]:                                                   # every rank ends with the reduced buffer
            for p in (0, w.P - 1):
                same_bits(pipe.ag[p][:L].view(it), red.view(nt), f"{what} t={t} all-gather copy of rank {p}")
        if c["scatter"] and not c["sgd"]:                                    # per-tensor destinations
            for j, v in enumerate(op.views(out, w.sizes)):
                same_bits(pipe.out_tensors[j], np.ascontiguousarray(v), f"{what} t={t} out tensor {j}")
        if c["sgd"]:
            if w.chunk:
                ob.sgd_update(red, w.N, w.chunk, sel_used, alpha, mom, lr, w_ref, hu_ref, None, w.wire, w_half=w16_ref)
            else:
                ob.sgd_update(red, w.N, w.N, np.array([0], dtype=np.int32), alpha, mom, lr, w_ref, hu_ref, None, w.wire,
                              w_half=w16_ref)
            if c["scatter"]:
                for j, (wv, hv) in enumerate(zip(op.views(w_ref, w.sizes), op.views(hu_ref, w.sizes))):
                    same_bits(pipe.w[j], np.ascontiguousarray(wv), f"{what} t={t} w tensor {j}")
                    same_bits(pipe.hu[j], np.ascontiguousarray(hv), f"{what} t={t} hu tensor {j}")
                if half:
                    for j, hv in enumerate(op.views(w16_ref, w.sizes)):
                        same_bits(pipe.w16[j].view(torch.int16), np.ascontiguousarray(hv).view(np.int16),
                                  f"{what} t={t} fp16 weights of tensor {j}")
            else:
                same_bits(pipe.w, w_ref, f"{what} t={t} w")
                same_bits(pipe.hu, hu_ref, f"{what} t={t} hu")
                if half:
                    same_bits(pipe.w16.view(torch.int16), w16_ref.view(np.int16), f"{what} t={t} fp16 weights")


def test_the_draws_cover_what_they_are_meant_to():
    """Host only: the drawn set really contains the combinations named in the module docstring."""
    cs = [_draw(s) for s in range(N_DRAWS)]
    assert {16, 32, 64} <= {c["P"] for c in cs}
    assert any(0 < c["chunk"] < 64 for c in cs) and any(c["chunk"] % 4 for c in cs if c["chunk"])
    assert any(c["sgd"] and c["half"] and c["scatter"] for c in cs) and any(c["sgd"] and c["half"] and not c["scatter"] for c in cs)
    for key in ("allgather", "scatter", "sgd", "odd_address", "boost_last", "fast"):
        assert any(c[key] for c in cs) and any(not c[key] for c in cs), key
    assert any(c["warmup"] for c in cs) and any(c["sgd"] and c["chunk"] == 0 for c in cs)
    assert any(c["sgd"] and c["scatter"] and c["chunk"] for c in cs)
    assert all(c["P"] * sum(c["sizes"]) <= BUDGET or max(c["sizes"]) <= 64 for c in cs)
