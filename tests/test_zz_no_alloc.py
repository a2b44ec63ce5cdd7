"""gf_fuse_pack_static (the entry point that allocates nothing: its scratch is a
fixed device array inside the library) against gf_fuse_pack with a caller's
workspace, through the C ABI: bit-identical send buffers, historical gradients
and chunk norms, on two calls in a row, the second on a smaller problem, plus
the size limit."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _problem(gf, sizes, P, chunk, k, seed):
    """Inputs for one fused pass (accumulate + norms + pack with a known selection)."""
    plan = gf.Plan(sizes, 1 << 40, chunk, P)
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    N, nc = plan.N, plan.n_chunks
    pools = [torch.randn(N, generator=g, device="cuda") * 1e-2 for _ in range(P)]
    hg = [torch.randn(N, generator=g, device="cuda") * 1e-3 for _ in range(P)]
    sel = torch.sort(torch.randperm(nc, generator=g, device="cuda")[:k]).values.to(torch.int32)
    return plan, pools, hg, sel


def _run(gf, plan, pools, hg, sel, k, static, phase):
    P, N, nc = plan.P, plan.N, plan.n_chunks
    res = [h.clone() for h in hg]
    send = [torch.full((k * plan.chunk,), 9.0, dtype=torch.float16, device="cuda") for _ in range(P)]
    l1 = torch.full((P * nc,), -1.0, device="cuda")
    args = dict(pools=gf.ptr_table(pools), residual=gf.ptr_table(res), chunk_l1=l1)
    if phase & gf.GF_PHASE_PACK:
        args.update(sel_idx=sel, k=k, loss_scale=128.0, mu=0.9, sendbuf=gf.ptr_table(send))
    if static:
        gf.gf_fuse_pack_static(plan, phase, **args)
    else:
        gf.gf_fuse_pack(plan, phase, workspace=plan.workspace(), **args)
    torch.cuda.synchronize()
    return res, send, l1


def _same(a, b, what):
    assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a.view(torch.int16),
                       b.view(torch.int32) if b.dtype == torch.float32 else b.view(torch.int16)), what


def test_static_scratch_variant_equals_the_workspace_variant_on_two_calls_in_a_row():
    from paper_1902_06855_amd import gf
    torch.cuda.set_device(0)
    # first a larger problem (chunks of three sub-tiles: partial norms and the slot map are both in
    # use), then a smaller one (two sub-tiles, fewer workers) that finds the first call's leftovers
    cases = [([150_000, 64, 90_001, 7, 33_000, 40_960], 3, 20_000, 5, 1),
             ([30_000, 8, 50_000, 1_000], 2, 9_000, 3, 2)]
    for sizes, P, chunk, k, seed in cases:
        plan, pools, hg, sel = _problem(gf, sizes, P, chunk, k, seed)
        assert plan.workspace_bytes() <= gf.GF_STATIC_SCRATCH_BYTES
        for phase in (gf.GF_PHASE_ACCUM | gf.GF_PHASE_PACK, gf.GF_PHASE_ACCUM):
            want = _run(gf, plan, pools, hg, sel, k, False, phase)
            got = _run(gf, plan, pools, hg, sel, k, True, phase)
            for p in range(P):
                _same(got[0][p], want[0][p], f"historical gradient of worker {p}, phase {phase}")
                _same(got[1][p], want[1][p], f"send buffer of worker {p}, phase {phase}")
            _same(got[2], want[2], f"chunk norms, phase {phase}")
            assert torch.all(want[2] >= 0)                       # the norms were written at all
        plan.close()


def test_static_scratch_variant_rejects_a_plan_that_needs_more_than_its_array():
    from paper_1902_06855_amd import gf
    torch.cuda.set_device(0)
    # 64 workers x 5000 chunks x 2 sub-tiles x 8 bytes of partial norms > 4 MiB; the call must
    # refuse before it touches any pointer (the tables below are never dereferenced)
    plan = gf.Plan([5000 * 8200], 1 << 40, 8200, 64)
    assert plan.workspace_bytes() > gf.GF_STATIC_SCRATCH_BYTES
    dummy = torch.zeros(64, dtype=torch.int64, device="cuda")
    l1 = torch.zeros(64 * 5000, device="cuda")
    with pytest.raises(gf.GfError) as e:
        gf.gf_fuse_pack_static(plan, gf.GF_PHASE_ACCUM, pools=dummy, residual=dummy, chunk_l1=l1)
    assert e.value.status == gf.GF_ELIMIT
    plan.close()
