"""Degenerate and extreme cases of the path on the GPU, against the CPU checker."""
import numpy as np
import pytest
import torch

from oracle import binding as ob, pipeline as op
from paper_1902_06855_amd import workloads as wl

from test_gpu_parity import _run_csc, _run_dense, cpu_grads, pools_np, same_bits, gfm  # noqa: F401  (gfm is a fixture)

pytestmark = pytest.mark.gpu


def _wl(sizes, P, chunk, density, S=32.0, theta=1 << 40, wire="f16"):
    return wl.Workload("edge", list(sizes), P=P, chunk=chunk, density=density, loss_scale=S, theta=theta, wire=wire)


@pytest.mark.parametrize("schedule", ["immediate", "lagged"])
def test_one_worker(gfm, schedule):
    # P = 1: the ring is the identity and both scoring rules coincide
    _run_csc(gfm, _wl([4096, 1000, 24], 1, 256, 0.2), schedule, "gather", T=3)


@pytest.mark.parametrize("schedule", ["immediate", "lagged"])
def test_a_single_important_chunk_and_a_single_chunk_pool(gfm, schedule):
    _run_csc(gfm, _wl([3000, 5000], 3, 512, 0.0001), schedule, "gather", T=3, k=1)     # k = 1: argmax
    _run_csc(gfm, _wl([300, 500], 3, 4096, 1.0), schedule, "pool", T=2)                # C > N: one short chunk


@pytest.mark.parametrize("groups", [0, 64])
def test_the_largest_worker_count(gfm, groups):
    # P = 4096, the most a plan takes: every per-worker table, the 4096-term folds of the ring
    # (flat, and 64 groups of 64) and the column sum over 4096 norm rows, on a small pool
    gf, pl = gfm
    w = _wl([40, 24, 130], 4096, 16, 0.3, theta=50)
    nc = ob.n_chunks(w.N, w.chunk)
    k = w.k_for(nc)
    pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=k, mu=w.mu, wire=w.wire, groups=groups)
    st = op.new_state(w.P, w.N)
    for t in range(3):
        pools = pools_np(cpu_grads(w, t), w.sizes)
        pipe.set_pools([torch.from_numpy(pools[p]).cuda() for p in range(w.P)])
        pipe.out_pool.fill_(-3.0)
        pipe.step()
        torch.cuda.synchronize()
        out = np.full(w.N, np.float32(-3.0))
        r = op.csc_iteration(st, pools, w.chunk, k, w.loss_scale, w.mu, "lagged", w.wire, out=out, theta=w.theta,
                             groups=groups)
        L = r["send"].shape[1]
        assert np.array_equal(pipe.sel.cpu().numpy(), r["sel_next"]), f"t={t} selection"
        same_bits(pipe.reduced[:L].view(torch.int16), r["reduced"].view(np.int16), f"t={t} reduced")
        same_bits(pipe.out_pool, out, f"t={t} out")
        for p in (0, 1, 63, 64, 2047, 4095):
            same_bits(pipe.send[p][:L].view(torch.int16), r["send"][p].view(np.int16), f"t={t} send[{p}]")
            same_bits(pipe.residual[p], st.hg[p], f"t={t} hg[{p}]")


def test_chunks_of_eight_elements(gfm):
    w = _wl([1000, 24, 8], 2, 8, 0.1)
    pipe = _run_csc(gfm, w, "lagged", "gather", T=2)
    assert pipe.n_chunks == 129


def test_one_element_tensors_and_chunks_that_span_hundreds_of_tensors(gfm):
    # 300 tensors of 1..24 elements inside 4096-element chunks: more pieces per tile than the
    # LDS piece table holds, unaligned everywhere
    rng = np.random.default_rng(0)
    sizes = [int(s) for s in rng.integers(1, 25, size=300)] + [5000]
    _run_csc(gfm, _wl(sizes, 2, 4096, 0.5), "lagged", "gather", T=2, scatter=True)
    _run_dense(gfm, _wl(sizes, 2, 0, 1.0, theta=64), "gather")
    # a few dozen aligned pieces per tile: the LDS piece table path
    sizes = [64] * 40 + [8, 8, 16, 4096]
    _run_csc(gfm, _wl(sizes, 3, 2048, 0.5), "lagged", "gather", T=2, scatter=True)
    _run_dense(gfm, _wl(sizes, 3, 0, 1.0, theta=500), "gather")


def test_gradient_tensors_at_odd_addresses(gfm):
    """Scattered tensors that are only 4-byte aligned (views one element into their storage)."""
    gf, pl = gfm
    w = _wl([4096, 8192, 512], 2, 1024, 0.25)
    nc = ob.n_chunks(w.N, w.chunk)
    k = w.k_for(nc)
    grads = wl.gradients(w, 0)
    dev = [[torch.cat([torch.zeros(1 + (j + p) % 3), g]).cuda()[1 + (j + p) % 3:] for j, g in enumerate(row)]
           for p, row in enumerate(grads)]
    assert any(t.data_ptr() % 16 for row in dev for t in row)
    pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=k, schedule="immediate")
    pipe.set_gradients(dev)
    pipe.step()
    torch.cuda.synchronize()
    pools = np.stack([op.fuse([x.numpy() for x in row], w.sizes) for row in grads])
    st = op.new_state(w.P, w.N)
    r = op.csc_iteration(st, pools, w.chunk, k, w.loss_scale, 1.0, "immediate")
    assert np.array_equal(pipe.sel.cpu().numpy(), r["sel"])
    same_bits(pipe.out_pool, r["out"], "out")
    for p in range(w.P):
        same_bits(pipe.residual[p], st.hg[p], f"hg[{p}]")


def test_pool_beyond_two_to_the_31_elements(gfm):
    """64-bit offsets: one worker, a 2^31 + 12 345 element pool, dense path, sampled against the checker."""
    gf, pl = gfm
    free, _ = torch.cuda.mem_get_info()
    if free < 40 << 30:
        pytest.skip("needs about 36 GB of free device memory")
    big = (1 << 31) + 12_345
    sizes = [1000, big - 1000 - 4096, 4096]
    w = _wl(sizes, 1, 0, 1.0, S=8.0, theta=1 << 30)
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    grads = [[torch.randn(s, generator=g, device="cuda", dtype=torch.float32) for s in sizes]]
    pipe = pl.Pipeline(w.sizes, 1, 0, w.theta, w.loss_scale)
    assert pipe.N == big and pipe.plan.n_buckets == 2
    pipe.set_gradients(grads)
    pipe.step()
    torch.cuda.synchronize()
    off, N = ob.layout(sizes)
    rng = np.random.default_rng(1)
    idx = np.unique(np.concatenate([np.arange(0, 5000), np.arange(big - 5000, big),
                                    np.arange((1 << 31) - 3000, (1 << 31) + 3000),
                                    rng.integers(0, big, size=20000)]))
    tens = np.searchsorted(-np.asarray(off), -idx, side="left")        # offsets descend with the ID index
    gs = np.empty(idx.size, dtype=np.float32)
    for j in range(len(sizes)):
        m = tens == j
        if m.any():
            gs[m] = grads[0][j][torch.from_numpy(idx[m] - off[j]).cuda()].cpu().numpy()
    send = ob.cast_dense(gs[None, :], w.loss_scale)[0]
    tidx = torch.from_numpy(idx).cuda()
    assert np.array_equal(pipe.send[0][tidx].cpu().numpy().view(np.uint16), send)
    assert np.array_equal(pipe.reduced[tidx].cpu().numpy().view(np.uint16), send)      # P = 1: identity
    out = ob.unpack_dense(send, np.float32(1) / np.float32(w.loss_scale))
    assert np.array_equal(pipe.out_pool[tidx].cpu().numpy().view(np.uint32), out.view(np.uint32))


@pytest.mark.parametrize("chunk", [1024, 2048, 4096, 8192, 16384])
@pytest.mark.parametrize("mode", ["gather", "pool"])
def test_power_of_two_chunks_around_the_sub_tile_length(gfm, chunk, mode):
    """Chunks of 1024 ... 16384 elements (an eighth of a sub-tile, one, two: each launch shape of the
    sweep); mixes plain chunks with chunks that hold tensor borders, an unaligned tensor, and the
    ragged pool end."""
    sizes = [chunk * 5, 100, chunk * 2 + 4, 5000, chunk * 9, 7, chunk * 3]
    w = _wl(sizes, 3, chunk, 0.3)
    for schedule in ("lagged", "immediate"):
        _run_csc(gfm, w, schedule, mode, T=3)
    w32 = _wl(sizes, 2, chunk, 0.3, wire="f32")
    _run_csc(gfm, w32, "lagged", mode, T=2)


@pytest.mark.parametrize("chunk", [20000, 32000, 8200, 40001])
@pytest.mark.parametrize("mode", ["gather", "pool"])
def test_long_chunks_cut_into_sub_tiles(gfm, chunk, mode):
    """Chunks longer than a workgroup's share are swept by several workgroups: ragged last
    sub-tiles, tensor borders and unaligned tensors inside sub-tiles, a short last chunk that
    ends before some of its sub-tiles begin, chunk lengths that are no multiple of four."""
    sizes = [chunk * 2 + 4, 100, 7, chunk + 8192, 33, 5000, chunk * 3, 9000, 8192 * 3, 50]
    w = _wl(sizes, 3, chunk, 0.4)
    for schedule in ("lagged", "immediate"):
        _run_csc(gfm, w, schedule, mode, T=3)
    w16 = _wl([s // 4 * 4 for s in sizes], 2, chunk, 0.4, wire="f32")
    _run_csc(gfm, w16, "lagged", mode, T=2)


def test_fp16_gradients_at_two_byte_addresses_and_in_long_chunks(gfm):
    """fp16 gradient tensors that are only 2-byte aligned (element-wise path), and fp16 gradients in
    chunks long enough to be cut into sub-tiles."""
    gf, pl = gfm
    for sizes, chunk, shift in (([4096, 8192, 520], 1024, True), ([20000 * 2 + 8, 36, 9000, 20000], 20000, False)):
        w = _wl(sizes, 2, chunk, 0.3)
        nc = ob.n_chunks(w.N, w.chunk)
        k = w.k_for(nc)
        pipe = pl.Pipeline(w.sizes, w.P, w.chunk, w.theta, w.loss_scale, k=k, schedule="lagged", grad="f16")
        st = op.new_state(w.P, w.N)
        for t in range(2):
            g16 = [[x.to(torch.float16) for x in row] for row in wl.gradients(w, t)]
            g32 = [[torch.from_numpy(ob.f16_to_f32(x.numpy().view(np.uint16))) for x in row] for row in g16]
            if shift:
                dev = [[torch.cat([torch.zeros(1 + (j + p) % 3, dtype=torch.float16), g]).cuda()[1 + (j + p) % 3:]
                        for j, g in enumerate(row)] for p, row in enumerate(g16)]
                assert any(x.data_ptr() % 8 for row in dev for x in row)
            else:
                dev = [[x.cuda() for x in row] for row in g16]
            pipe.set_gradients(dev)
            pipe.out_pool.fill_(-4.0)
            pipe.step()
            torch.cuda.synchronize()
            out = np.full(w.N, np.float32(-4.0))
            pools = np.stack([op.fuse([x.numpy() for x in row], w.sizes) for row in g32])
            r = op.csc_iteration(st, pools, w.chunk, k, w.loss_scale, w.mu, "lagged", out=out)
            assert np.array_equal(pipe.sel.cpu().numpy(), r["sel_next"]), f"t={t} selection"
            same_bits(pipe.out_pool, out, f"t={t} out")
            for p in range(w.P):
                same_bits(pipe.residual[p], st.hg[p], f"t={t} hg[{p}]")


def test_reduce_groups_are_fixed_once_the_tables_are_on_the_device(gfm):
    gf, _ = gfm
    plan = gf.Plan([4096], 1 << 40, 0, 8)                  # uploaded by the constructor
    with pytest.raises(gf.GfError) as e:
        plan.set_reduce_groups(2)
    assert e.value.status == gf.GF_ESTATE
    plan.set_grad_type(gf.GF_WIRE_F16)                      # host-side only: allowed at any time


def test_hierarchical_order_with_one_rank_and_with_one_group(gfm):
    gf, _ = gfm
    rng = np.random.default_rng(9)
    for P, M in ((1, 1), (5, 1), (5, 5)):
        L = 3001
        x = (rng.standard_normal((P, L)) * 2.0 ** rng.integers(-6, 6, size=(P, 1))).astype(np.float16).view(np.uint16)
        plan = gf.Plan([4096], 1 << 40, 4096, P, groups=M)
        red = torch.zeros(L, dtype=torch.float16, device="cuda")
        gf.gf_ring_reduce_sim(plan, gf.ptr_table([torch.from_numpy(x[p].view(np.float16)).cuda() for p in range(P)]), L, red)
        torch.cuda.synchronize()
        same_bits(red.view(torch.int16), ob.hier_fold(x, M).view(np.int16), f"P={P} M={M}")
