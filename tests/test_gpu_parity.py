"""GPU-vs-checker parity, stage by stage and over whole iterations, through the
C ABI.  Bit-exact for every fp16 value, every fixed-order fp32 result and every
index; chunk norms and scores within 1e-5 relative; a selection may differ from
the checker's only among chunks whose scores tie with the k-th within that
tolerance (the GPU's choice is then handed to the checker so that everything
downstream stays bit-comparable)."""
import numpy as np
import pytest
import torch

from oracle import binding as ob, pipeline as op
from paper_1902_06855_amd import workloads as wl

pytestmark = pytest.mark.gpu

RTOL = 1e-5


@pytest.fixture(scope="module")
def gfm():
    from paper_1902_06855_amd import gf, pipeline
    return gf, pipeline


def bits(a: np.ndarray) -> np.ndarray:
    a = np.ascontiguousarray(a)
    return a.view({2: np.uint16, 4: np.uint32, 8: np.uint64}[a.dtype.itemsize])


def same_bits(gpu: torch.Tensor, ref: np.ndarray, what: str):
    g = gpu.detach().cpu().numpy()
    assert g.shape == ref.shape, f"{what}: shape {g.shape} vs {ref.shape}"
    bad = np.flatnonzero(bits(g).ravel() != bits(ref).ravel())
    assert bad.size == 0, f"{what}: {bad.size} of {g.size} differ, first at {bad[:5]}: " \
                          f"gpu {g.ravel()[bad[:5]]} ref {ref.ravel()[bad[:5]]}"


def close_rel(gpu: torch.Tensor, ref: np.ndarray, what: str, rtol=RTOL):
    g = gpu.detach().cpu().numpy().astype(np.float64)
    r = ref.astype(np.float64)
    err = np.abs(g - r) / np.maximum(np.abs(r), 1e-300)
    err[(r == 0) & (g == 0)] = 0
    assert err.max(initial=0) <= rtol, f"{what}: max rel err {err.max()}"


def admissible_selection(g_sel: np.ndarray, o_sel: np.ndarray, score: np.ndarray, k: int, what: str):
    assert g_sel.shape == (k,) and np.all(np.diff(g_sel) > 0), f"{what}: not k ascending indices"
    if np.array_equal(g_sel, o_sel):
        return
    kth = np.sort(score)[::-1][k - 1]
    for c in np.setxor1d(g_sel, o_sel):
        assert abs(score[c] - kth) <= RTOL * abs(kth), f"{what}: chunk {c} differs and is not tied with the k-th"


def cpu_grads(w, t):
    return wl.gradients(w, t, device="cpu")


def to_dev(grads):
    return [[x.cuda() for x in row] for row in grads]


def pools_np(grads, sizes):
    return np.stack([op.fuse([x.numpy() for x in row], sizes) for row in grads])


def odd_workload(P=3, chunk=96, wire="f16", S=64.0, density=0.3):
    # odd sizes: tensors start at unaligned pool offsets -> scalar paths, ragged tails
    return wl.Workload("odd", [50, 7, 701, 33, 1201, 64, 5, 4099], P=P, chunk=chunk, density=density,
                       loss_scale=S, theta=1000, wire=wire)


# ------------------------------------------------------------------ ring alone

def _halves(rng, P, L, special=True):
    x = (rng.standard_normal((P, L)) * 2.0 ** rng.integers(-16, 14, size=(P, 1))).astype(np.float16)
    u = x.view(np.uint16).copy()
    if special and L >= 64:
        u[:, 0:8] = rng.integers(0, 0x0400, size=(P, 8))            # subnormals
        u[:, 8:16] = 0x7bff                                          # max finite -> overflow to inf
        u[0, 16:24] = 0x8000                                         # -0
        u[:, 24:32] = rng.integers(0x7800, 0x7c00, size=(P, 8))      # large
    return u


@pytest.mark.parametrize("P,L", [(1, 100), (2, 4096), (3, 1000), (4, 253952), (8, 100003), (16, 65536),
                                 (64, 262144), (5, 7), (8, 8)])
def test_ring_single_bucket_bit_exact(gfm, P, L):
    gf, _ = gfm
    rng = np.random.default_rng(P * 7 + L)
    C = 1024
    nch = -(-L // C)
    plan = gf.Plan([nch * C], 1 << 40, C, P)
    x = _halves(rng, P, L)
    want = ob.ring_fold(x, "f16")
    send = [torch.from_numpy(x[p].view(np.float16)).cuda() for p in range(P)]
    tab = gf.ptr_table(send)
    red = torch.zeros(L, dtype=torch.float16, device="cuda")
    ag = [torch.zeros(L, dtype=torch.float16, device="cuda") for _ in range(P)]
    gf.gf_ring_reduce_sim(plan, tab, L, red, allgather_out=gf.ptr_table(ag))
    torch.cuda.synchronize()
    same_bits(red.view(torch.int16), want.view(np.int16), f"ring P={P} L={L}")
    for r in range(P):                       # every rank ends with the same buffer (all-gather)
        same_bits(ag[r].view(torch.int16), want.view(np.int16), f"allgather rank {r}")
    # the length may also come from device memory, with L only an upper bound
    cap = nch * C
    send2 = [torch.zeros(cap, dtype=torch.float16, device="cuda") for _ in range(P)]
    for p in range(P):
        send2[p][:L] = send[p]
    red2 = torch.full((cap,), 7.0, dtype=torch.float16, device="cuda")
    L_dev = torch.tensor([L], dtype=torch.int64, device="cuda")
    gf.gf_ring_reduce_sim(plan, gf.ptr_table(send2), cap, red2, L_dev=L_dev)
    torch.cuda.synchronize()
    same_bits(red2[:L].view(torch.int16), want.view(np.int16), "ring with device-side length")
    assert torch.all(red2[L:] == 7.0)        # nothing past the real length is touched


def test_ring_unaligned_buffers_and_fp32_wire(gfm):
    gf, _ = gfm
    rng = np.random.default_rng(3)
    P, L = 4, 5001
    plan = gf.Plan([8192], 1 << 40, 8192, P)
    x = _halves(rng, P, L)
    want = ob.ring_fold(x, "f16")
    raw = [torch.zeros(L + 8, dtype=torch.float16, device="cuda") for _ in range(P)]
    send = [raw[p][1 + p % 2:1 + p % 2 + L] for p in range(P)]       # 2-byte aligned only
    for p in range(P):
        send[p].copy_(torch.from_numpy(x[p].view(np.float16)))
    red = torch.zeros(L + 3, dtype=torch.float16, device="cuda")[3:]
    gf.gf_ring_reduce_sim(plan, gf.ptr_table(send), L, red)
    torch.cuda.synchronize()
    same_bits(red.view(torch.int16), want.view(np.int16), "unaligned ring")

    plan32 = gf.Plan([8192], 1 << 40, 8192, P, wire=gf.GF_WIRE_F32)
    y = (rng.standard_normal((P, L)) * 10.0 ** rng.integers(-6, 6, size=(P, 1))).astype(np.float32)
    want32 = ob.ring_fold(y, "f32")
    send32 = [torch.from_numpy(y[p]).cuda() for p in range(P)]
    red32 = torch.zeros(L, dtype=torch.float32, device="cuda")
    gf.gf_ring_reduce_sim(plan32, gf.ptr_table(send32), L, red32)
    torch.cuda.synchronize()
    same_bits(red32, want32, "fp32 ring")


# ------------------------------------------------------------------ dense path

def _run_dense(gfm, w, mode, S=None, scatter=True):
    gf, pl = gfm
    S = S or w.loss_scale
    grads = cpu_grads(w, 0)
    pools = pools_np(grads, w.sizes)
    ref = op.dense_iteration(pools, w.sizes, w.theta, S, w.wire)
    pipe = pl.Pipeline(w.sizes, w.P, 0, w.theta, S, wire=w.wire, scatter_out=scatter, allgather=True)
    if mode == "gather":
        pipe.set_gradients(to_dev(grads))
    else:
        pipe.set_pools([torch.from_numpy(pools[p]).cuda() for p in range(w.P)])
    pipe.out_pool.fill_(-77.0)
    pipe.cast_dense()
    torch.cuda.synchronize()
    for p in range(w.P):
        same_bits(pipe.send[p].view(torch.int16 if w.wire == "f16" else torch.int32),
                  ref["send"][p].view(np.int16 if w.wire == "f16" else np.int32), f"send[{p}]")
    pipe.ring()
    torch.cuda.synchronize()
    it = torch.int16 if w.wire == "f16" else torch.int32
    nt = np.int16 if w.wire == "f16" else np.int32
    same_bits(pipe.reduced.view(it), ref["reduced"].view(nt), "reduced")
    same_bits(pipe.ag[w.P - 1].view(it), ref["reduced"].view(nt), "allgather copy")
    pipe.unpack()
    torch.cuda.synchronize()
    same_bits(pipe.out_pool, ref["out"], "out pool")
    if scatter:
        for j, v in enumerate(op.views(ref["out"], w.sizes)):
            same_bits(pipe.out_tensors[j], np.ascontiguousarray(v), f"out tensor {j}")
    return pipe


@pytest.mark.parametrize("mode", ["gather", "pool"])
@pytest.mark.parametrize("wire", ["f16", "f32"])
def test_dense_odd_sizes_many_buckets(gfm, mode, wire):
    w = odd_workload(P=3, chunk=0, wire=wire)
    pipe = _run_dense(gfm, w, mode)
    assert pipe.plan.n_buckets > 1


@pytest.mark.parametrize("mode", ["gather", "pool"])
def test_dense_resnet_shaped_scaled(gfm, mode):
    w = wl.scaled(wl.config("resnet50_dense_4mb"), 16)
    pipe = _run_dense(gfm, w, mode)
    assert pipe.plan.n_buckets >= 8


def test_dense_alexnet_shaped_scaled_P8(gfm):
    _run_dense(gfm, wl.scaled(wl.config("alexnet_dense"), 32), "gather")


def test_dense_loss_scale_that_is_not_a_power_of_two(gfm):
    # acc * S is then inexact in fp32 and rounded again to fp16: both roundings must happen
    w = wl.Workload("np2", [1 << 20], P=2, chunk=0, density=1.0, loss_scale=1000.0, theta=1 << 40)
    _run_dense(gfm, w, "gather", scatter=False)


def test_cast_rounding_boundaries(gfm):
    """Every tie and near-tie between neighbouring halves, subnormals, overflow, signed zero."""
    gf, pl = gfm
    h = np.arange(0, 0x7c00, dtype=np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    hi[-1] = 65536.0
    mid = ((lo + hi) / 2).astype(np.float32)
    vals = np.concatenate([mid, np.nextafter(mid, np.float32(-np.inf)), np.nextafter(mid, np.float32(np.inf)),
                           lo.astype(np.float32),
                           np.array([0.0, -0.0, 1e-40, -1e-40, 65519.99, 65520.0, 1e9, np.inf, -np.inf],
                                    dtype=np.float32)])
    vals = np.concatenate([vals, -vals]).astype(np.float32)
    n = vals.size
    pipe = pl.Pipeline([n], 1, 0, 1 << 40, 1.0)
    g = torch.from_numpy(vals).cuda()
    pipe.set_gradients([[g]])
    pipe.cast_dense()
    torch.cuda.synchronize()
    same_bits(pipe.send[0].view(torch.int16), ob.f32_to_f16(vals).view(np.int16), "fp32->fp16 boundaries")
    # fp16 -> fp32 of every half (unpack with alpha = 1)
    allh = np.arange(65536, dtype=np.uint16)
    fin = ~np.isnan(allh.view(np.float16))
    allh = allh[fin]
    pipe2 = pl.Pipeline([allh.size], 1, 0, 1 << 40, 1.0)
    pipe2.reduced.copy_(torch.from_numpy(allh.view(np.float16)).cuda())
    pipe2.unpack()
    torch.cuda.synchronize()
    same_bits(pipe2.out_pool, ob.f16_to_f32(allh), "fp16->fp32 all halves")
    # fp32 subnormal products: loss scaling lifts them into half's range
    tiny = (np.arange(1, 4097, dtype=np.float64) * 2.0 ** -140).astype(np.float32)
    pipe3 = pl.Pipeline([tiny.size], 1, 0, 1 << 40, 2.0 ** 120)
    pipe3.set_gradients([[torch.from_numpy(tiny).cuda()]])
    pipe3.cast_dense()
    torch.cuda.synchronize()
    same_bits(pipe3.send[0].view(torch.int16), ob.cast_dense(tiny[None, :], 2.0 ** 120)[0].view(np.int16),
              "subnormal inputs")


# -------------------------------------------------------------------- selection

@pytest.mark.parametrize("nc,k", [(1, 1), (5, 1), (5, 5), (245, 62), (1861, 187), (3120, 32), (50_000, 777),
                                  (2049, 1024), (4096, 4096), (4097, 409), (8192, 1), (8199, 4100), (16384, 163),
                                  (16385, 16000), (32768, 3277), (32769, 32), (12480, 125)])
def test_select_bit_exact_including_ties(gfm, nc, k):
    gf, _ = gfm
    rng = np.random.default_rng(nc + k)
    P, C = 3, 8
    plan = gf.Plan([nc * C - 3], 1 << 40, C, P)
    l1 = rng.random((P, nc)).astype(np.float32)
    dup = rng.integers(0, nc, size=max(1, nc // 4))
    l1[:, dup] = l1[:, dup[0]][:, None]                   # exact ties, possibly at the threshold
    if nc > 100:
        l1[:, 10:40] = 0                                  # a run of zeros
    sc = ob.score(l1)
    want, wmask = ob.select(sc, k)
    d_l1 = torch.from_numpy(l1).cuda().reshape(-1)
    scores = torch.zeros(nc, dtype=torch.float32, device="cuda")
    sel = torch.zeros(k, dtype=torch.int32, device="cuda")
    mask = torch.zeros(nc, dtype=torch.uint8, device="cuda")
    plen = torch.zeros(1, dtype=torch.int64, device="cuda")
    gf.gf_chunk_score_select(plan, d_l1, k=k, scores=scores, sel_idx=sel, mask=mask, packed_len=plen,
                             workspace=plan.workspace())
    torch.cuda.synchronize()
    same_bits(scores, sc, "scores")
    assert np.array_equal(sel.cpu().numpy(), want)
    assert np.array_equal(mask.cpu().numpy(), wmask)
    assert int(plen.item()) == ob.packed_len(nc * C - 3, C, want)
    # a score vector that is only 4-byte aligned
    odd = torch.zeros(nc + 1, dtype=torch.float32, device="cuda")
    sel.fill_(-1)
    gf.gf_chunk_score_select(plan, d_l1, k=k, scores=odd[1:], sel_idx=sel, workspace=plan.workspace())
    torch.cuda.synchronize()
    same_bits(odd[1:], sc, "scores at an odd address")
    assert np.array_equal(sel.cpu().numpy(), want)
    # all-equal scores: the lowest indices win
    d_l1.fill_(1.0)
    gf.gf_chunk_score_select(plan, d_l1, k=k, sel_idx=sel, workspace=plan.workspace())
    torch.cuda.synchronize()
    assert np.array_equal(sel.cpu().numpy(), np.arange(k))


def test_select_with_scores_that_are_not_numbers(gfm):
    """Infinite and NaN norms (a worker whose gradients overflowed): NaN ranks above +inf above
    every finite score, NaNs tie, the lower index wins; the choice equals the checker's."""
    gf, _ = gfm
    rng = np.random.default_rng(77)
    P, C, nc = 2, 8, 3000
    plan = gf.Plan([nc * C], 1 << 40, C, P)
    l1 = rng.random((P, nc)).astype(np.float32)
    l1[0, rng.integers(0, nc, size=40)] = np.inf
    l1[1, rng.integers(0, nc, size=25)] = np.nan
    l1[0, 5] = np.inf; l1[1, 5] = np.nan                  # inf + nan
    sc = ob.score(l1)
    assert np.isnan(sc).sum() >= 20 and np.isinf(sc).sum() >= 30
    d_l1 = torch.from_numpy(l1).cuda().reshape(-1)
    for k in (1, 10, int(np.isnan(sc).sum()), int(np.isnan(sc).sum()) + 7, 500, nc):
        want, wmask = ob.select(sc, k)
        sel = torch.zeros(k, dtype=torch.int32, device="cuda")
        mask = torch.zeros(nc, dtype=torch.uint8, device="cuda")
        gf.gf_chunk_score_select(plan, d_l1, k=k, sel_idx=sel, mask=mask, workspace=plan.workspace())
        torch.cuda.synchronize()
        assert np.array_equal(sel.cpu().numpy(), want), f"k={k}"
        assert np.array_equal(mask.cpu().numpy(), wmask)


# up to eight workers and 8192 chunks the selecting workgroup computes the scores itself (sent chunks
# found through a table in LDS); beyond either limit a scoring kernel runs first
@pytest.mark.parametrize("P,nc,k", [(6, 500, 50), (64, 20_000, 333), (1, 3120, 312), (8, 8192, 8192), (2, 4097, 1500),
                                    (9, 4000, 400), (4, 8193, 2000), (1, 1, 1)])
def test_select_after_allreduce_scores_sent_chunks_by_their_reduced_norm(gfm, P, nc, k):
    gf, _ = gfm
    rng = np.random.default_rng(8)
    C = 16
    plan = gf.Plan([nc * C], 1 << 40, C, P)
    l1 = rng.random((P, nc)).astype(np.float32)
    prev = np.sort(rng.choice(nc, size=k, replace=False)).astype(np.int32)
    red = (rng.random(k) * 5).astype(np.float32)
    sc = ob.score(l1, prev, red)
    want, _ = ob.select(sc, k)
    scores = torch.zeros(nc, dtype=torch.float32, device="cuda")
    sel = torch.from_numpy(prev).cuda()                   # output overwrites the previous selection
    gf.gf_chunk_score_select(plan, torch.from_numpy(l1).cuda().reshape(-1), reduced_l1=torch.from_numpy(red).cuda(),
                             prev_sel=sel, k_prev=k, k=k, scores=scores, sel_idx=sel, workspace=plan.workspace())
    torch.cuda.synchronize()
    same_bits(scores, sc, "scores with sent chunks")
    assert np.array_equal(sel.cpu().numpy(), want)


# ------------------------------------------------- sparse path, stage by stage

def _run_csc(gfm, w, schedule, mode, T, k=None, scatter=False, fast=False):
    """fast: the calls hand the slot map and the unfinished chunk norms to each other through the
    workspace (what Pipeline.step() and the benchmark do); the per-worker norms are then never
    materialised, and what is checked instead is what they turn into: the scores."""
    gf, pl = gfm
    nc = ob.n_chunks(w.N, w.chunk)
    k = k or w.k_for(nc)
    pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=k, mu=w.mu, wire=w.wire,
                       schedule=schedule, scatter_out=scatter, fast=fast)
    assert pipe.n_chunks == nc
    st = op.new_state(w.P, w.N)
    it = torch.int16 if w.wire == "f16" else torch.int32
    nt = np.int16 if w.wire == "f16" else np.int32
    alpha = np.float32(1.0) / np.float32(w.loss_scale)
    sel_now = None                                        # lagged: chosen at the end of the previous iteration
    sync = torch.cuda.synchronize
    for t in range(T):
        grads = cpu_grads(w, t)
        pools = pools_np(grads, w.sizes)
        if mode == "gather":
            pipe.set_gradients(to_dev(grads))
        else:
            pipe.set_pools([torch.from_numpy(pools[p]).cuda() for p in range(w.P)])
        acc = ob.accumulate(pools, st.hg)
        l1 = ob.chunk_l1(acc, w.chunk)
        two_pass = schedule == "immediate" or t == 0
        if two_pass:
            pipe.accum(); sync()
            for p in range(w.P):
                same_bits(pipe.residual[p], acc[p], f"t={t} acc[{p}]")
            if not fast:
                close_rel(pipe.l1, l1.reshape(-1), f"t={t} chunk norms")
            pipe.select(False); sync()
            sc = ob.score(l1)
            close_rel(pipe.scores, sc, f"t={t} scores")
            o_sel, _ = ob.select(sc, k)
            sel_now = pipe.sel.cpu().numpy().copy()
            admissible_selection(sel_now, o_sel, sc, k, f"t={t} selection")
            assert np.array_equal(np.flatnonzero(pipe.mask.cpu().numpy()), sel_now)
            pipe.pack(); sync()
        else:
            assert np.array_equal(pipe.sel.cpu().numpy(), sel_now)
            pipe.fused(); sync()
            if not fast:
                close_rel(pipe.l1, l1.reshape(-1), f"t={t} chunk norms (fused)")
        L = ob.packed_len(w.N, w.chunk, sel_now)
        assert int(pipe.packed_len.item()) == L
        send, hg = ob.pack_residual(acc, w.chunk, sel_now, w.loss_scale, w.mu, w.wire)
        for p in range(w.P):
            same_bits(pipe.send[p][:L].view(it), send[p].view(nt), f"t={t} send[{p}]")
            same_bits(pipe.residual[p], hg[p], f"t={t} hg[{p}]")
        st.hg = hg
        reduced = np.empty(L, dtype=send.dtype)
        for a, b in zip(*ob.packed_buckets(w.N, w.chunk, sel_now, w.theta)):   # one ring per flushed bucket
            reduced[a:b] = ob.ring_fold(np.ascontiguousarray(send[:, a:b]), w.wire)
        pipe.ring(); sync()
        same_bits(pipe.reduced[:L].view(it), reduced.view(nt), f"t={t} reduced")
        out = np.full(w.N, np.float32(-5.0))
        pipe.out_pool.fill_(-5.0)
        red_l1 = ob.unpack(reduced, w.N, w.chunk, sel_now, alpha, out, w.wire)
        if scatter:
            for ot in pipe.out_tensors:
                ot.zero_()
        pipe.unpack(); sync()
        same_bits(pipe.out_pool, out, f"t={t} out")
        close_rel(pipe.red_l1, red_l1, f"t={t} reduced norms")
        if scatter:
            outs = op.views(out, w.sizes)
            m = np.zeros(w.N, dtype=bool)
            for c in sel_now:
                m[c * w.chunk:(c + 1) * w.chunk] = True
            for j, v in enumerate(op.views(m, w.sizes)):
                got = pipe.out_tensors[j].cpu().numpy()
                assert np.array_equal(bits(got[v]), bits(np.ascontiguousarray(outs[j][v]))), f"scatter tensor {j}"
                assert np.all(got[~v] == 0)
        if schedule == "lagged":
            sc = ob.score(l1, sel_now, red_l1)
            o_next, _ = ob.select(sc, k)
            pipe.select(True); sync()
            close_rel(pipe.scores, sc, f"t={t} scores after allreduce")
            nxt = pipe.sel.cpu().numpy().copy()
            admissible_selection(nxt, o_next, sc, k, f"t={t} next selection")
            sel_now = nxt
    return pipe


@pytest.mark.parametrize("schedule", ["immediate", "lagged"])
@pytest.mark.parametrize("mode", ["gather", "pool"])
def test_tiny_configuration(gfm, schedule, mode):
    # P=4, six tensors, C=4096, 25 % of 245 chunks, S=1024
    w = wl.config("tiny")
    pipe = _run_csc(gfm, w, schedule, mode, T=2 if schedule == "lagged" else 1)
    assert pipe.k == 62 and pipe.n_chunks == 245


@pytest.mark.parametrize("schedule", ["immediate", "lagged"])
@pytest.mark.parametrize("wire", ["f16", "f32"])
def test_csc_odd_sizes_scalar_paths(gfm, schedule, wire):
    _run_csc(gfm, odd_workload(P=3, chunk=96, wire=wire), schedule, "gather", T=3, scatter=True)
    _run_csc(gfm, odd_workload(P=2, chunk=1000, wire=wire), schedule, "pool", T=2)


@pytest.mark.parametrize("schedule", ["immediate", "lagged"])
def test_csc_momentum_below_one(gfm, schedule):
    w = odd_workload(P=3, chunk=128)
    w.mu = 0.9
    _run_csc(gfm, w, schedule, "gather", T=3)
    w2 = wl.scaled(wl.config("tiny"), 4)
    w2.mu = 0.5
    _run_csc(gfm, w2, schedule, "pool", T=3)


def test_csc_every_chunk_selected_equals_dense(gfm):
    gf, pl = gfm
    w = odd_workload(P=4, chunk=100, density=1.0)
    w.theta = 1 << 40                                 # one ring over the whole buffer on both sides
    pipe = _run_csc(gfm, w, "immediate", "gather", T=2)
    assert all(torch.all(r == 0) for r in pipe.residual)
    grads = cpu_grads(w, 1)
    d = op.dense_iteration(pools_np(grads, w.sizes), w.sizes, 1 << 40, w.loss_scale)
    # (the second iteration starts from a zero residual, so it is a dense iteration)
    same_bits(pipe.out_pool, d["out"], "k = n_chunks vs dense")


@pytest.mark.parametrize("fast", [False, True])
def test_alexnet_csc_scaled_all_iterations(gfm, fast):
    w = wl.scaled(wl.config("alexnet_csc"), 16)          # P=16, 10 iterations
    _run_csc(gfm, w, "lagged", "gather", T=w.iterations, fast=fast)


@pytest.mark.parametrize("fast", [False, True])
def test_resnet50_csc_scaled_all_iterations(gfm, fast):
    w = wl.scaled(wl.config("resnet50_csc"), 32)         # P=64, 161 tensors, 20 iterations
    _run_csc(gfm, w, "lagged", "gather", T=w.iterations, fast=fast)


@pytest.mark.parametrize("schedule", ["immediate", "lagged"])
@pytest.mark.parametrize("chunk", [96, 20000])            # one sub-tile per chunk; three, ragged
def test_hand_overs_through_the_workspace(gfm, schedule, chunk):
    """Slot map left by the selection and chunk norms finished by it (GF_PHASE_SLOTS,
    GF_PHASE_DEFER_NORMS), stage by stage, with a momentum below one (so that the pack-only
    pass of the two-pass iterations needs the slot map as well)."""
    sizes = [50, 7, 701, 33, 1201, 64, 5, 4099] if chunk == 96 else [chunk * 3 + 4, 100, chunk * 2, 5000, 12345]
    w = wl.Workload("handover", sizes, P=3, chunk=chunk, density=0.3, loss_scale=64.0, theta=1 << 40, mu=0.5)
    _run_csc(gfm, w, schedule, "gather", T=4, fast=True)
    _run_csc(gfm, w, schedule, "pool", T=3, fast=True, scatter=True)


def test_step_runs_the_same_sequence(gfm):
    """Pipeline.step() (what the benchmark times) against the stage-by-stage run."""
    gf, pl = gfm
    w = wl.scaled(wl.config("tiny"), 2)
    nc = ob.n_chunks(w.N, w.chunk)
    k = w.k_for(nc)
    for schedule, fast in (("lagged", True), ("lagged", False), ("immediate", True), ("immediate", False)):
        a = _run_csc(gfm, w, schedule, "gather", T=4)
        b = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=k, schedule=schedule, fast=fast)
        for t in range(4):
            b.set_gradients(to_dev(cpu_grads(w, t)))
            b.out_pool.fill_(-5.0)
            b.step()
        torch.cuda.synchronize()
        assert torch.equal(a.out_pool, b.out_pool) and torch.equal(a.sel, b.sel)
        for p in range(w.P):
            assert torch.equal(a.residual[p], b.residual[p])


# --------------------------------------------- SGD update fused into the unpack

@pytest.mark.parametrize("scatter", [False, True])
@pytest.mark.parametrize("wire", ["f16", "f32"])
def test_sgd_update_step_of_algorithm_1(gfm, scatter, wire):
    """Important chunks: hu = momentum*hu + lr*g, w += hu; everything else untouched; over several
    lagged iterations so that chunks go in and out of the important set."""
    gf, pl = gfm
    w_ = odd_workload(P=3, chunk=96, wire=wire) if scatter else wl.scaled(wl.config("tiny"), 4)
    w_.wire = wire
    nc = ob.n_chunks(w_.N, w_.chunk)
    k = w_.k_for(nc)
    mom, lr = 0.9, -0.125
    pipe = pl.Pipeline(w_.sizes, w_.P, w_.chunk, w_.theta, w_.loss_scale, k=k, wire=wire, schedule="lagged",
                       scatter_out=scatter, sgd=(mom, lr))
    rng = np.random.default_rng(5)
    w_ref = rng.standard_normal(w_.N).astype(np.float32)
    hu_ref = np.zeros(w_.N, dtype=np.float32)
    if scatter:
        for j, v in enumerate(op.views(w_ref, w_.sizes)):
            pipe.w[j].copy_(torch.from_numpy(np.ascontiguousarray(v)))
    else:
        pipe.w.copy_(torch.from_numpy(w_ref))
    st = op.new_state(w_.P, w_.N)
    alpha = np.float32(1.0) / np.float32(w_.loss_scale)
    for t in range(4):
        grads = cpu_grads(w_, t)
        pools = pools_np(grads, w_.sizes)
        pipe.set_gradients(to_dev(grads))
        pipe.out_pool.fill_(-3.0)
        pipe.step()
        torch.cuda.synchronize()
        out = np.full(w_.N, np.float32(-3.0))
        r = op.csc_iteration(st, pools, w_.chunk, k, w_.loss_scale, w_.mu, "lagged", wire, out=out, theta=w_.theta)
        assert np.array_equal(pipe.sel.cpu().numpy(), r["sel_next"])
        ob.sgd_update(r["reduced"], w_.N, w_.chunk, r["sel"], alpha, mom, lr, w_ref, hu_ref, None, wire)
        same_bits(pipe.out_pool, out, f"t={t} out")
        if scatter:
            for j, (wv, hv) in enumerate(zip(op.views(w_ref, w_.sizes), op.views(hu_ref, w_.sizes))):
                same_bits(pipe.w[j], np.ascontiguousarray(wv), f"t={t} w tensor {j}")
                same_bits(pipe.hu[j], np.ascontiguousarray(hv), f"t={t} hu tensor {j}")
        else:
            same_bits(pipe.w, w_ref, f"t={t} w")
            same_bits(pipe.hu, hu_ref, f"t={t} hu")
    assert np.any(hu_ref != 0) and np.any(hu_ref == 0)


def test_sgd_update_dense_plan(gfm):
    gf, pl = gfm
    w_ = odd_workload(P=3, chunk=0)
    pipe = pl.Pipeline(w_.sizes, w_.P, 0, w_.theta, w_.loss_scale, sgd=(0.5, 0.25))
    w_ref = np.linspace(-1, 1, w_.N).astype(np.float32)
    hu_ref = np.zeros(w_.N, dtype=np.float32)
    pipe.w.copy_(torch.from_numpy(w_ref))
    for t in range(2):
        grads = cpu_grads(w_, t)
        d = op.dense_iteration(pools_np(grads, w_.sizes), w_.sizes, w_.theta, w_.loss_scale)
        pipe.set_gradients(to_dev(grads))
        pipe.step()
        torch.cuda.synchronize()
        g = d["out"]
        hu_ref = (np.float32(0.5) * hu_ref).astype(np.float32) + (np.float32(0.25) * g).astype(np.float32)
        w_ref = w_ref + hu_ref
        same_bits(pipe.out_pool, g, "dense out")
        same_bits(pipe.hu, hu_ref, "dense hu")
        same_bits(pipe.w, w_ref, "dense w")


def test_warmup_changes_the_number_of_important_chunks_every_iteration(gfm):
    """Lagged schedule with the dense-to-sparse warm-up ramp: k differs between consecutive iterations."""
    gf, pl = gfm
    w = wl.scaled(wl.config("tiny"), 4)
    nc = ob.n_chunks(w.N, w.chunk)
    T_w, final = 4, 0.25
    pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=nc, k_max=nc, schedule="lagged")
    ks = [pipe.plan.warmup_k(final, t, T_w) for t in range(8)]
    assert ks[0] == nc and ks[-1] == w.k_for(nc) and len(set(ks)) >= 4
    st = op.new_state(w.P, w.N)
    for t in range(7):
        grads = cpu_grads(w, t)
        pipe.set_gradients(to_dev(grads))
        pipe.k_next = ks[t] if t == 0 else ks[t + 1]     # iteration 0 selects twice: for itself, then for t = 1
        pipe.out_pool.fill_(-2.0)
        if t == 0:
            pipe.accum(); pipe.select(False); pipe.pack(); pipe.ring(); pipe.unpack()
            pipe.k_next = ks[1]
            pipe.select(True)
            pipe.t = 1
        else:
            pipe.step()
        torch.cuda.synchronize()
        out = np.full(w.N, np.float32(-2.0))
        r = op.csc_iteration(st, pools_np(grads, w.sizes), w.chunk, ks[t], w.loss_scale, w.mu, "lagged",
                             out=out, k_next=ks[t + 1])
        assert pipe.k == ks[t + 1]
        assert np.array_equal(pipe.sel[:pipe.k].cpu().numpy(), r["sel_next"]), f"t={t} next selection"
        assert int(pipe.packed_len.item()) == ob.packed_len(w.N, w.chunk, r["sel_next"])
        same_bits(pipe.out_pool, out, f"t={t} out")
        for p in range(w.P):
            same_bits(pipe.residual[p], st.hg[p], f"t={t} hg[{p}]")


@pytest.mark.parametrize("wire", ["f16", "f32"])
def test_packed_buffer_is_reduced_bucket_by_bucket(gfm, wire):
    """theta below the packed length: several rings over the packed buffer, incl. a short last bucket."""
    w = wl.scaled(wl.config("tiny"), 4)                  # C = 1024, 245 chunks, k = 62
    w.wire = wire
    w.theta = 5 * 1024 + 17                              # a bucket every 6 chunks
    pipe = _run_csc(gfm, w, "lagged", "gather", T=3)
    w2 = odd_workload(P=4, chunk=100, wire=wire)         # odd chunk length: unaligned bucket starts
    w2.theta = 250
    _run_csc(gfm, w2, "immediate", "gather", T=2)


# ------------------------------------------------------- fp16 gradients as input

def _half_grads(w, t):
    """fp16 gradients (as a mixed-precision backward would hand them over) and their exact fp32 values."""
    g16 = [[x.to(torch.float16) for x in row] for row in cpu_grads(w, t)]
    g32 = [[torch.from_numpy(ob.f16_to_f32(x.numpy().view(np.uint16))) for x in row] for row in g16]
    return g16, g32


@pytest.mark.parametrize("mode", ["gather", "pool"])
@pytest.mark.parametrize("wire", ["f16", "f32"])
def test_fp16_gradients_csc(gfm, mode, wire):
    gf, pl = gfm
    for w in (odd_workload(P=3, chunk=96, wire=wire), wl.scaled(wl.config("tiny"), 4)):
        w.wire = wire
        w.theta = 1 << 40
        nc = ob.n_chunks(w.N, w.chunk)
        k = w.k_for(nc)
        pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=k, wire=wire, schedule="lagged", grad="f16",
                           fast=False)                  # the norms are compared below
        st = op.new_state(w.P, w.N)
        for t in range(3):
            g16, g32 = _half_grads(w, t)
            if mode == "gather":
                pipe.set_gradients(to_dev(g16))
            else:
                pipe.set_pools([torch.cat([x for x in reversed(row)]).cuda() for row in g16])
            pipe.out_pool.fill_(-4.0)
            pipe.step()
            torch.cuda.synchronize()
            out = np.full(w.N, np.float32(-4.0))
            r = op.csc_iteration(st, pools_np(g32, w.sizes), w.chunk, k, w.loss_scale, w.mu, "lagged", wire, out=out)
            assert np.array_equal(pipe.sel.cpu().numpy(), r["sel_next"]), f"t={t} selection"
            same_bits(pipe.out_pool, out, f"t={t} out")
            close_rel(pipe.l1, r["l1"].reshape(-1), f"t={t} norms")
            for p in range(w.P):
                same_bits(pipe.residual[p], st.hg[p], f"t={t} hg[{p}]")


@pytest.mark.parametrize("mode", ["gather", "pool"])
def test_fp16_gradients_dense(gfm, mode):
    gf, pl = gfm
    w = odd_workload(P=3, chunk=0)
    g16, g32 = _half_grads(w, 0)
    ref = op.dense_iteration(pools_np(g32, w.sizes), w.sizes, w.theta, w.loss_scale)
    pipe = pl.Pipeline(w.sizes, w.P, 0, w.theta, w.loss_scale, grad="f16")
    if mode == "gather":
        pipe.set_gradients(to_dev(g16))
    else:
        pipe.set_pools([torch.cat([x for x in reversed(row)]).cuda() for row in g16])
    pipe.step()
    torch.cuda.synchronize()
    for p in range(w.P):
        same_bits(pipe.send[p].view(torch.int16), ref["send"][p].view(np.int16), f"send[{p}]")
    same_bits(pipe.out_pool, ref["out"], "out")


@pytest.mark.parametrize("theta", [1 << 40, 700, 0])
def test_fp16_pools_reduced_in_place(gfm, theta):
    """fp16 pools on an fp16 wire: no cast pass, each bucket of the pools is ring-reduced where it lies."""
    gf, pl = gfm
    w = odd_workload(P=5, chunk=0)
    g16, _ = _half_grads(w, 0)
    pools = [torch.cat([x for x in reversed(row)]) for row in g16]
    h = np.stack([x.numpy().view(np.uint16) for x in pools])
    lo, hi = ob.buckets(w.sizes, theta)
    reduced = np.empty(w.N, dtype=np.uint16)
    for a, b in zip(lo, hi):
        reduced[a:b] = ob.ring_fold(np.ascontiguousarray(h[:, a:b]), "f16")
    out = ob.unpack_dense(reduced, np.float32(1.0) / np.float32(w.loss_scale), "f16")
    pipe = pl.Pipeline(w.sizes, w.P, 0, theta, w.loss_scale, grad="f16", zero_copy=True)
    assert pipe.send is None and pipe.plan.n_buckets == len(lo)
    dev = [x.cuda() for x in pools]
    pipe.set_pools(dev)
    pipe.step()
    torch.cuda.synchronize()
    same_bits(pipe.reduced.view(torch.int16), reduced.view(np.int16), "reduced")
    same_bits(pipe.out_pool, out, "out")
    for p in range(w.P):                                   # the pools themselves are only read
        assert torch.equal(dev[p].cpu().view(torch.int16), pools[p].view(torch.int16))
    with pytest.raises(ValueError):
        pl.Pipeline(w.sizes, w.P, 0, theta, w.loss_scale, grad="f32", zero_copy=True)


# ------------------------------------------------- hierarchical allreduce order (Section 2.4)

@pytest.mark.parametrize("P,M,L", [(4, 2, 4096), (16, 4, 100003), (8, 1, 70000), (64, 8, 262144), (6, 3, 1000),
                                   (12, 2, 7), (64, 16, 33333), (9, 3, 8), (20, 4, 50001)])
def test_hierarchical_order_single_bucket_bit_exact(gfm, P, M, L):
    gf, _ = gfm
    rng = np.random.default_rng(P * 7 + M + L)
    C = 1024
    nch = -(-L // C)
    plan = gf.Plan([nch * C], 1 << 40, C, P, groups=M)
    assert plan.ring_segment(L) == ob.ring_segment(L, M)
    x = _halves(rng, P, L)
    want = ob.hier_fold(x, M, "f16")
    send = [torch.from_numpy(x[p].view(np.float16)).cuda() for p in range(P)]
    red = torch.zeros(L, dtype=torch.float16, device="cuda")
    ag = [torch.zeros(L, dtype=torch.float16, device="cuda") for _ in range(P)]
    L_dev = torch.tensor([L], dtype=torch.int64, device="cuda")
    gf.gf_ring_reduce_sim(plan, gf.ptr_table(send), L, red, L_dev=L_dev, allgather_out=gf.ptr_table(ag))
    torch.cuda.synchronize()
    same_bits(red.view(torch.int16), want.view(np.int16), f"hier P={P} M={M} L={L}")
    for r in (0, P - 1):                     # the broadcast leaves every rank with the same buffer
        same_bits(ag[r].view(torch.int16), want.view(np.int16), f"broadcast rank {r}")


def test_hierarchical_order_unaligned_and_fp32_wire(gfm):
    gf, _ = gfm
    rng = np.random.default_rng(4)
    P, M, L = 6, 2, 5001
    plan = gf.Plan([8192], 1 << 40, 8192, P, groups=M)
    x = _halves(rng, P, L)
    want = ob.hier_fold(x, M, "f16")
    raw = [torch.zeros(L + 8, dtype=torch.float16, device="cuda") for _ in range(P)]
    send = [raw[p][1 + p % 2:1 + p % 2 + L] for p in range(P)]       # 2-byte aligned only: scalar path
    for p in range(P):
        send[p].copy_(torch.from_numpy(x[p].view(np.float16)))
    red = torch.zeros(L, dtype=torch.float16, device="cuda")
    gf.gf_ring_reduce_sim(plan, gf.ptr_table(send), L, red)
    torch.cuda.synchronize()
    same_bits(red.view(torch.int16), want.view(np.int16), "unaligned hierarchical")

    plan32 = gf.Plan([8192], 1 << 40, 8192, P, wire=gf.GF_WIRE_F32, groups=M)
    y = (rng.standard_normal((P, L)) * 10.0 ** rng.integers(-6, 6, size=(P, 1))).astype(np.float32)
    want32 = ob.hier_fold(y, M, "f32")
    red32 = torch.zeros(L, dtype=torch.float32, device="cuda")
    gf.gf_ring_reduce_sim(plan32, gf.ptr_table([torch.from_numpy(y[p]).cuda() for p in range(P)]), L, red32)
    torch.cuda.synchronize()
    same_bits(red32, want32, "fp32 hierarchical")


@pytest.mark.parametrize("wire", ["f16", "f32"])
def test_hierarchical_order_dense_buckets(gfm, wire):
    gf, pl = gfm
    w = odd_workload(P=6, chunk=0, wire=wire)
    for M, theta in ((2, 1000), (3, 0), (1, 1 << 40), (6, 64)):
        grads = cpu_grads(w, 0)
        pools = pools_np(grads, w.sizes)
        ref = op.dense_iteration(pools, w.sizes, theta, w.loss_scale, wire, groups=M)
        pipe = pl.Pipeline(w.sizes, w.P, 0, theta, w.loss_scale, wire=wire, groups=M)
        pipe.set_gradients(to_dev(grads))
        pipe.step()
        torch.cuda.synchronize()
        it, nt = (torch.int16, np.int16) if wire == "f16" else (torch.int32, np.int32)
        same_bits(pipe.reduced.view(it), ref["reduced"].view(nt), f"reduced M={M} theta={theta}")
        same_bits(pipe.out_pool, ref["out"], f"out M={M}")


@pytest.mark.parametrize("schedule", ["lagged", "immediate"])
def test_hierarchical_order_csc_iterations(gfm, schedule):
    """Several sparse iterations with the packed buffer reduced hierarchically, bucket-wise."""
    gf, pl = gfm
    for w, M, theta in ((odd_workload(P=4, chunk=96), 2, 1 << 40), (wl.scaled(wl.config("tiny"), 4), 2, 3000),
                        (odd_workload(P=6, chunk=64, density=0.5), 3, 200)):
        nc = ob.n_chunks(w.N, w.chunk)
        k = w.k_for(nc)
        pipe = pl.Pipeline(w.sizes, w.P, w.chunk, theta, w.loss_scale, k=k, schedule=schedule, groups=M)
        st = op.new_state(w.P, w.N)
        for t in range(3):
            grads = cpu_grads(w, t)
            pipe.set_gradients(to_dev(grads))
            pipe.out_pool.fill_(-4.0)
            pipe.step()
            torch.cuda.synchronize()
            out = np.full(w.N, np.float32(-4.0))
            r = op.csc_iteration(st, pools_np(grads, w.sizes), w.chunk, k, w.loss_scale, w.mu, schedule,
                                 out=out, theta=theta, groups=M)
            L = r["send"].shape[1]
            same_bits(pipe.reduced[:L].view(torch.int16), r["reduced"].view(np.int16), f"t={t} reduced")
            same_bits(pipe.out_pool, out, f"t={t} out")
            nxt = r["sel_next"] if schedule == "lagged" else r["sel"]
            assert np.array_equal(pipe.sel.cpu().numpy(), nxt), f"t={t} selection"


# ------------------------------------------------------------- iterations replayed as HIP graphs

@pytest.mark.parametrize("kind", ["csc", "dense"])
def test_graph_replays_match_eager_iterations(gfm, kind):
    """A captured iteration, replayed several times with eager work and synchronisations in
    between, gives what the same iterations give when launched one call at a time."""
    gf, pl = gfm
    w = wl.scaled(wl.config("tiny"), 4) if kind == "csc" else odd_workload(P=3, chunk=0)
    k = w.k_for(ob.n_chunks(w.N, w.chunk)) if w.chunk else 0
    mk = lambda: pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=k, schedule="lagged")
    eager, graphed = mk(), mk()
    dev = [to_dev(cpu_grads(w, t)) for t in range(3)]
    for pipe in (eager, graphed):                          # iteration 0 (the lagged bootstrap) runs eagerly
        pipe.set_gradients(dev[0])
        pipe.step()
    torch.cuda.synchronize()
    graphs = []
    for t in (1, 2):                                       # one graph per gradient set: tables are baked in
        graphed.set_gradients(dev[t])
        graphs.append((graphed.grads_tab, graphed.capture()))
    for it in range(6):
        t = 1 + it % 2
        eager.set_gradients(dev[t])
        eager.step()
        graphs[t - 1][1].replay()
        torch.cuda.synchronize()
        scratch = torch.randn(1 << 16, device="cuda").sum().item()          # unrelated eager work in between
        assert scratch == scratch
        same_bits(graphed.out_pool, eager.out_pool.cpu().numpy(), f"replay {it} out")
        same_bits(graphed.reduced.view(torch.int16), eager.reduced.view(torch.int16).cpu().numpy(), f"replay {it} reduced")
        if w.chunk:
            assert torch.equal(graphed.sel, eager.sel), f"replay {it} selection"
            for p in range(w.P):
                same_bits(graphed.residual[p], eager.residual[p].cpu().numpy(), f"replay {it} hg[{p}]")


# ------------------------------------------- buckets issued one by one on side streams (overlap)

@pytest.mark.parametrize("mode", ["gather", "pool"])
@pytest.mark.parametrize("wire", ["f16", "f32"])
def test_buckets_issued_on_side_streams_equal_the_single_pass(gfm, mode, wire):
    gf, pl = gfm
    for w, theta in ((odd_workload(P=3, chunk=0, wire=wire), 1000), (odd_workload(P=4, chunk=0, wire=wire), 0),
                     (wl.Workload("even", [4096, 64, 8192, 1000, 24, 16384], P=2, chunk=0, density=1.0,
                                  loss_scale=32.0, theta=5000, wire=wire), 5000)):
        grads = cpu_grads(w, 0)
        pools = pools_np(grads, w.sizes)
        ref = op.dense_iteration(pools, w.sizes, theta, w.loss_scale, wire)
        ov = pl.OverlappedDense(w.sizes, w.P, theta, w.loss_scale, wire=wire, n_streams=3)
        assert ov.n_buckets == len(ref["bucket_lo"]) and ov.lo == list(ref["bucket_lo"])
        dev = to_dev(grads)
        dev_pools = [torch.from_numpy(pools[p]).cuda() for p in range(w.P)]
        if mode == "gather":
            ov.set_gradients(dev)
        else:
            ov.set_pools(dev_pools)
        ready = [torch.cuda.Event() for _ in range(ov.n_buckets)]    # one arrival event per bucket
        ov.step(ready=None)
        torch.cuda.synchronize()
        it, nt = (torch.int16, np.int16) if wire == "f16" else (torch.int32, np.int32)
        for p in range(w.P):
            same_bits(ov.send[p].view(it), ref["send"][p].view(nt), f"send[{p}] theta={theta}")
        same_bits(ov.reduced.view(it), ref["reduced"].view(nt), f"reduced theta={theta}")
        same_bits(ov.out_pool, ref["out"], f"out theta={theta}")
        ov.out_pool.fill_(-1.0)
        for e in reversed(ready):
            e.record()
        ov.step(ready=ready)
        torch.cuda.synchronize()
        same_bits(ov.out_pool, ref["out"], f"out with arrival events theta={theta}")


def test_a_bucket_waits_for_its_own_gradients_only(gfm):
    """Gradients are written bucket by bucket on a producer stream (as backward would), each bucket
    followed by its arrival event; the buckets' own streams must not read them earlier."""
    gf, pl = gfm
    sizes = [1 << 20, 1 << 18, 3000, 1 << 20, 1 << 16]
    w = wl.Workload("arrive", sizes, P=2, chunk=0, density=1.0, loss_scale=16.0, theta=1 << 17)
    grads = cpu_grads(w, 0)
    ref = op.dense_iteration(pools_np(grads, w.sizes), w.sizes, w.theta, w.loss_scale)
    ov = pl.OverlappedDense(w.sizes, w.P, w.theta, w.loss_scale, n_streams=2)
    assert ov.n_buckets >= 3
    staged = to_dev(grads)
    live = [[torch.zeros_like(x) for x in row] for row in staged]        # what the buckets read
    ov.set_gradients(live)
    torch.cuda.synchronize()
    producer = torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(ov.n_buckets)]
    with torch.cuda.stream(producer):
        for b, mem in enumerate(ov.members):                              # generation order
            for _ in range(20):                                           # make the producer slow
                for p in range(w.P):
                    for j in mem:
                        live[p][j].copy_(staged[p][j], non_blocking=True)
            ready[b].record(producer)
    ov.step(ready=ready)
    torch.cuda.synchronize()
    same_bits(ov.reduced.view(torch.int16), ref["reduced"].view(np.int16), "reduced")
    same_bits(ov.out_pool, ref["out"], "out")


def test_bucket_wise_iteration_replayed_as_a_graph(gfm):
    """Fork to the side streams and join back inside one captured graph; replays with eager work in
    between equal the single pass."""
    gf, pl = gfm
    w = odd_workload(P=3, chunk=0)
    ref = [op.dense_iteration(pools_np(cpu_grads(w, t), w.sizes), w.sizes, 300, w.loss_scale) for t in range(2)]
    ov = pl.OverlappedDense(w.sizes, w.P, 300, w.loss_scale, n_streams=3)
    assert ov.n_buckets > 3
    graphs, keep = [], []
    for t in range(2):
        dev = to_dev(cpu_grads(w, t))
        ov.set_gradients(dev)
        keep.append((dev, ov.grad_tabs))
        graphs.append(ov.capture())
    for it in range(6):
        t = it % 2
        ov.out_pool.fill_(-2.0)
        graphs[t].replay()
        torch.cuda.synchronize()
        torch.randn(1 << 14, device="cuda").sum().item()                     # unrelated eager work in between
        same_bits(ov.reduced.view(torch.int16), ref[t]["reduced"].view(np.int16), f"replay {it} reduced")
        same_bits(ov.out_pool, ref[t]["out"], f"replay {it} out")


# ------------------------------------------- one host call per steady-state iteration

@pytest.mark.parametrize("wire", ["f16", "f32"])
@pytest.mark.parametrize("mode", ["gather", "pool"])
def test_one_call_iteration_equals_the_four_calls(gfm, mode, wire):
    """gf_csc_iteration against the same iteration made of the four calls (two pipelines fed the
    same gradients), over iterations whose chunk count changes, with all-gather copies and
    per-tensor outputs, the slot map rebuilt (modifiers 0) or handed over; and against the checker."""
    gf, pl = gfm
    w = odd_workload(P=3, chunk=250, wire=wire, density=0.3)
    nc = ob.n_chunks(w.N, w.chunk)
    ks = [w.k_for(nc), w.k_for(nc), max(1, nc // 2), 2, nc, 3, 3]     # the first iteration keeps its count
    raw = lambda x: x.contiguous().view(torch.uint8)
    mk = lambda fast: pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=ks[0], k_max=nc, mu=0.75, wire=wire,
                                  scatter_out=True, allgather=True, fast=fast)
    one, four = mk(True), mk(False)                       # `four` never takes the one-call route
    st = op.new_state(w.P, w.N)
    for t in range(len(ks) - 1):
        grads = cpu_grads(w, t)
        pools = pools_np(grads, w.sizes)
        for pipe in (one, four):
            if mode == "gather":
                pipe.set_gradients(to_dev(grads))
            else:
                pipe.set_pools([torch.from_numpy(pools[p]).cuda() for p in range(w.P)])
            pipe.k_next = ks[t + 1]
            pipe.out_pool.fill_(-2.0)
        four.step()
        if t == 0:
            one.step()                                    # the first iteration is made of the single calls
        elif t % 2:
            one.step()                                    # gf_csc_iteration with the slot map handed over
        else:
            gf.gf_csc_iteration(one.plan, 0, grads=one.grads_tab, pools=one.pools_tab, residual=one.residual_tab,
                                sel_idx=one.sel, k=one.k, k_next=one.k_next, packed_len=one.packed_len,
                                loss_scale=one.S, mu=one.mu, sendbuf=one.send_tab, reduced=one.reduced,
                                allgather_out=one.ag_tab, alpha=one.alpha, out_pool=one.out_pool,
                                out_tensors=one.out_tab, reduced_l1=one.red_l1, workspace=one.ws)   # no scores, no mask
            one.k = one.k_next
            one.t += 1
        torch.cuda.synchronize()
        out = np.full(w.N, np.float32(-2.0))
        r = op.csc_iteration(st, pools, w.chunk, ks[t], w.loss_scale, 0.75, "lagged", wire, out=out, k_next=ks[t + 1],
                             theta=w.theta)
        L = r["send"].shape[1]
        what = f"{mode} {wire} t={t}"
        assert np.array_equal(one.sel.cpu().numpy()[:ks[t + 1]], r["sel_next"]), what
        assert torch.equal(one.sel[:ks[t + 1]], four.sel[:ks[t + 1]]) and torch.equal(one.packed_len, four.packed_len), what
        same_bits(one.out_pool, out, what + " out")
        for a, b in ((one.reduced[:L], four.reduced[:L]), (one.red_l1[:ks[t]], four.red_l1[:ks[t]]),
                     (one.out_pool, four.out_pool), (one.scores, four.scores) if t % 2 or t == 0 else (one.mask[:0], four.mask[:0])):
            assert torch.equal(raw(a), raw(b)), what
        for p in range(w.P):
            assert torch.equal(raw(one.residual[p]), raw(four.residual[p])), what
            assert torch.equal(raw(one.send[p][:L]), raw(four.send[p][:L])), what
            assert torch.equal(raw(one.ag[p][:L]), raw(four.ag[p][:L])), what
        for a, b in zip(one.out_tensors, four.out_tensors):
            assert torch.equal(raw(a), raw(b)), what


def test_the_call_sequence_of_a_training_loop(gfm):
    """The sequence a training loop makes (first iteration from the single calls, every later one
    with gf_csc_iteration), through the binding alone, against the checker."""
    gf, _ = gfm
    w = odd_workload(P=2, chunk=512, density=0.25)
    P, N, C, S = w.P, w.N, w.chunk, w.loss_scale
    plan = gf.Plan(w.sizes, w.theta, C, P)
    nc = plan.n_chunks
    k = w.k_for(nc)
    ws = plan.workspace()
    dev = lambda n, dt: torch.zeros(n, dtype=dt, device="cuda")
    hg = [dev(N, torch.float32) for _ in range(P)]
    send = [dev(k * C, torch.float16) for _ in range(P)]
    hg_tab, send_tab = gf.ptr_table(hg), gf.ptr_table(send)
    sel, L_dev, rl1 = dev(k, torch.int32), dev(1, torch.int64), dev(k, torch.float32)
    reduced, out = dev(k * C, torch.float16), dev(N, torch.float32)
    alpha = float(np.float32(1.0) / np.float32(S))
    st = op.new_state(P, N)
    for t in range(4):
        grads = cpu_grads(w, t)
        g_dev = to_dev(grads)
        grads_tab = gf.ptr_table([x for row in g_dev for x in row])
        out.fill_(-1.0)
        if t == 0:
            gf.gf_fuse_pack(plan, gf.GF_PHASE_ACCUM | gf.GF_PHASE_DEFER_NORMS, grads=grads_tab, residual=hg_tab,
                            workspace=ws)
            gf.gf_chunk_score_select(plan, None, k=k, sel_idx=sel, packed_len=L_dev, workspace=ws)
            gf.gf_fuse_pack(plan, gf.GF_PHASE_PACK | gf.GF_PHASE_SLOTS, residual=hg_tab, sel_idx=sel, k=k,
                            loss_scale=S, sendbuf=send_tab, workspace=ws)
            gf.gf_ring_reduce_sim(plan, send_tab, k * C, reduced, L_dev=L_dev)
            gf.gf_unpack_apply(plan, reduced, k * C, sel_idx=sel, k=k, alpha=alpha, out_pool=out, reduced_l1=rl1)
            gf.gf_chunk_score_select(plan, None, reduced_l1=rl1, prev_sel=sel, k_prev=k, k=k, sel_idx=sel,
                                     packed_len=L_dev, workspace=ws)
        else:
            gf.gf_csc_iteration(plan, gf.GF_PHASE_SLOTS, grads=grads_tab, residual=hg_tab, sel_idx=sel, k=k,
                                packed_len=L_dev, loss_scale=S, sendbuf=send_tab, reduced=reduced, alpha=alpha,
                                out_pool=out, reduced_l1=rl1, workspace=ws)
        torch.cuda.synchronize()
        want = np.full(N, np.float32(-1.0))
        r = op.csc_iteration(st, pools_np(grads, w.sizes), C, k, S, w.mu, "lagged", out=want, theta=w.theta)
        L = r["send"].shape[1]
        assert np.array_equal(sel.cpu().numpy(), r["sel_next"]), f"t={t}"
        same_bits(out, want, f"t={t} out")
        same_bits(reduced[:L].view(torch.int16), r["reduced"].view(np.int16), f"t={t} reduced")
        for p in range(P):
            same_bits(hg[p], st.hg[p], f"t={t} hg[{p}]")
