"""CPU-side checks of the C-ABI library: it loads, exports what include/gf.h
declares, plans exactly like the CPU checker, and rejects bad calls with
status codes.  No kernel is launched here."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import binding as ob
from paper_1902_06855_amd import build as gf_build, workloads as wl

if not os.path.exists(gf_build.LIB):          # nothing built yet: compile once (hipcc cross-compiles without a GPU)
    gf_build.build()
from paper_1902_06855_amd import gf  # noqa: E402  (fails loudly if the library cannot be loaded)

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "gf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gf_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert len(names) >= 14 and {"gf_fuse_pack", "gf_chunk_score_select", "gf_ring_reduce_sim",
                                 "gf_unpack_apply"} <= set(names)
    lib = ctypes.CDLL(gf.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in gf.h but not exported"
    assert set(names) == set(gf.EXPORTS)


def test_status_strings():
    for code in range(6):
        assert gf.gf_status_string(code).startswith("GF_")
    assert "unknown" in gf.gf_status_string(99)


@pytest.mark.parametrize("name", ["tiny", "alexnet_dense", "resnet50_dense_4mb", "resnet50_dense_64mb",
                                  "alexnet_csc", "resnet50_csc"])
def test_plan_matches_the_checker(name):
    w = wl.config(name)
    plan = gf.Plan(w.sizes, min(w.theta, 1 << 60), w.chunk, w.P, to_device=False)
    off, lo, hi = plan.layout()
    o_off, o_N = ob.layout(w.sizes)
    o_lo, o_hi = ob.buckets(w.sizes, w.theta)
    assert plan.N == o_N and off == list(o_off)
    assert lo == list(o_lo) and hi == list(o_hi) and plan.n_buckets == len(o_lo)
    if w.chunk:
        assert plan.n_chunks == ob.n_chunks(w.N, w.chunk) == plan.tiles()
    else:
        assert plan.n_chunks == 0
    for L in (0, 1, 7, 8, 1000, w.N // 3, w.N):
        assert plan.ring_segment(L) == ob.ring_segment(L, w.P, "f16")
    plan.close()


def _buckets_by_cumsum(sizes, theta):
    """Section 3.1's rule stated without a running counter: a bucket that starts at pool offset
    `start` ends at the first tensor border that lies more than theta beyond it (tensors in
    generation order, the last ID first); what is left at the end is one more bucket."""
    edges = np.concatenate([[0], np.cumsum(list(sizes)[::-1])])
    out, start = [], 0
    while start < edges[-1]:
        beyond = edges[edges - start > theta]
        end = int(beyond[0]) if len(beyond) else int(edges[-1])
        out.append((start, end))
        start = end
    return out


def test_plan_buckets_follow_the_threshold_rule_stated_on_cumulative_sizes():
    rng = np.random.default_rng(11)
    cases = [([5, 3, 4, 2], th) for th in (0, 1, 5, 6, 13, 14)]
    cases += [([int(s) for s in rng.integers(1, 5000, size=int(rng.integers(1, 60)))], int(rng.integers(0, 12000)))
              for _ in range(40)]
    for name in ("alexnet_dense", "resnet50_dense_4mb", "resnet50_dense_64mb"):
        w = wl.config(name)
        cases.append((w.sizes, w.theta))
    for sizes, theta in cases:
        plan = gf.Plan(sizes, theta, 0, 2, to_device=False)
        _, lo, hi = plan.layout()
        assert list(zip(lo, hi)) == _buckets_by_cumsum(sizes, theta), (sizes[:8], theta)
        plan.close()
    # hand-worked (generation order 2, 4, 3, 5): theta 5 -> 6 | 8; theta 6 -> 9 | 5; strict ">"
    for theta, want in ((5, [6, 8]), (6, [9, 5]), (13, [14]), (0, [2, 4, 3, 5]), (1, [2, 4, 3, 5])):
        plan = gf.Plan([5, 3, 4, 2], theta, 0, 2, to_device=False)
        _, lo, hi = plan.layout()
        assert [b - a for a, b in zip(lo, hi)] == want
        plan.close()


def test_warmup_chunk_counts_hand_worked():
    # sparsity ramps linearly: k = 1000 * (1 - 0.09 t); the double-precision product sits an ulp
    # above 820 and 190 at t = 2 and t = 9 and must not round up to 821 / 191
    plan = gf.Plan([1000 * 64], 1 << 40, 64, 2, to_device=False)
    assert [plan.warmup_k(0.1, t, 10) for t in range(12)] == [1000, 910, 820, 730, 640, 550, 460, 370, 280, 190, 100, 100]
    small = gf.Plan([100 * 8], 1 << 40, 8, 2, to_device=False)
    assert small.warmup_k(0.07, 0, 0) == 7 and small.warmup_k(0.071, 0, 0) == 8
    plan.close(); small.close()


def test_warmup_schedule_matches_the_checker():
    plan = gf.Plan([1000 * 64], 1 << 40, 64, 2, to_device=False)
    for d, T in ((0.1, 10), (0.25, 4), (0.15, 7), (1.0, 5), (0.01, 0)):
        for t in range(0, 14):
            assert plan.warmup_k(d, t, T) == ob.warmup_k(plan.n_chunks, d, t, T)
    dense = gf.Plan([100], 1 << 40, 0, 2, to_device=False)
    for bad in (lambda: dense.warmup_k(0.1, 0, 1), lambda: plan.warmup_k(0.0, 0, 1), lambda: plan.warmup_k(1.5, 0, 1),
                lambda: plan.warmup_k(0.1, -1, 1), lambda: plan.warmup_k(0.1, 0, -1)):
        with pytest.raises(gf.GfError):
            bad()


def test_ring_segment_fp32_wire():
    plan = gf.Plan([100, 200], 1 << 40, 0, 6, wire=gf.GF_WIRE_F32, to_device=False)
    for L in (0, 1, 5, 24, 25, 300):
        assert plan.ring_segment(L) == ob.ring_segment(L, 6, "f32")
    assert plan.ring_segment(-1) == -1


def test_reduce_groups_change_the_ring_size_and_reject_bad_counts():
    plan = gf.Plan([100, 200], 1 << 40, 0, 12, to_device=False)
    for M in (1, 2, 3, 4, 6, 12, 0):
        plan.set_reduce_groups(M)
        for L in (0, 1, 5, 24, 25, 300):
            assert plan.ring_segment(L) == ob.ring_segment(L, M or 12, "f16")
    for M in (5, 7, 13, -1, 24):
        with pytest.raises(gf.GfError) as e:
            plan.set_reduce_groups(M)
        assert e.value.status == gf.GF_EINVAL
    assert plan.ring_segment(300) == ob.ring_segment(300, 12, "f16")       # a refused count changes nothing


@pytest.mark.parametrize("sizes,chunk", [([7, 1, 64, 333, 2, 1024, 5], 96), ([50, 8, 700, 33, 1200, 64, 5], 0),
                                         (wl.resnet50_sizes(), 8192), ([5], 3), ([3, 3, 3], 3)])
def test_tile_pieces_tile_the_pool_in_generation_order(sizes, chunk):
    plan = gf.Plan(sizes, 1 << 40, chunk, 2, to_device=False)
    off, N = ob.layout(sizes)
    owner = np.empty(N, dtype=np.int64)        # which tensor / element each pool slot holds
    elem = np.empty(N, dtype=np.int64)
    for j, s in enumerate(sizes):
        owner[off[j]:off[j] + s] = j
        elem[off[j]:off[j] + s] = np.arange(s)
    T = chunk if chunk else 8192
    assert plan.tiles() == -(-N // T)
    pos = 0
    for t in range(plan.tiles()):
        assert pos == t * T
        for (tensor, src, ln) in plan.tile_pieces(t):
            assert ln >= 1
            assert np.all(owner[pos:pos + ln] == tensor)
            assert np.array_equal(elem[pos:pos + ln], np.arange(src, src + ln))
            pos += ln
        assert pos == min(N, (t + 1) * T)
    assert pos == N


def test_plan_create_rejects_bad_arguments():
    bad = [
        dict(tensor_numel=[], theta_elems=1, chunk_elems=0, P=1),
        dict(tensor_numel=[4, 0], theta_elems=1, chunk_elems=0, P=1),
        dict(tensor_numel=[4], theta_elems=-1, chunk_elems=0, P=1),
        dict(tensor_numel=[4], theta_elems=1, chunk_elems=-2, P=1),
        dict(tensor_numel=[4], theta_elems=1, chunk_elems=0, P=0),
        dict(tensor_numel=[4], theta_elems=1, chunk_elems=0, P=5000),
        dict(tensor_numel=[4], theta_elems=1, chunk_elems=0, P=1, wire=7),
    ]
    for kw in bad:
        with pytest.raises(gf.GfError) as e:
            gf.Plan(to_device=False, **kw)
        assert e.value.status == gf.GF_EINVAL


def test_compute_calls_validate_before_touching_the_gpu():
    csc = gf.Plan([4096, 4096], 1 << 40, 1024, 2, to_device=False)
    dense = gf.Plan([4096, 4096], 1 << 40, 0, 2, to_device=False)
    fake = 0x1000                     # never dereferenced: validation fails first
    E, S = gf.GF_EINVAL, gf.GF_ESTATE

    def status(fn, *a, **kw):
        with pytest.raises(gf.GfError) as e:
            fn(*a, stream=0, **kw)
        return e.value.status

    # fuse_pack
    assert status(gf.gf_fuse_pack, csc, 0, pools=fake, residual=fake, sendbuf=fake) == E
    assert status(gf.gf_fuse_pack, csc, 3, residual=fake, sendbuf=fake) == E               # no gradients
    assert status(gf.gf_fuse_pack, csc, 3, grads=fake, pools=fake, residual=fake, sendbuf=fake) == E
    assert status(gf.gf_fuse_pack, csc, 3, pools=fake, residual=fake) == E                 # no send buffer
    assert status(gf.gf_fuse_pack, csc, 1, pools=fake) == E                                # dense needs both phases
    assert status(gf.gf_fuse_pack, csc, 3, pools=fake, sel_idx=fake, k=1, sendbuf=fake) == E  # sparse needs hg
    assert status(gf.gf_fuse_pack, dense, 3, pools=fake, residual=fake, sel_idx=fake, k=1, sendbuf=fake) == E
    assert status(gf.gf_fuse_pack, dense, 3, pools=fake, residual=fake, chunk_l1=fake, sendbuf=fake) == E
    assert status(gf.gf_fuse_pack, csc, 3, pools=fake, residual=fake, sel_idx=fake, k=0, sendbuf=fake,
                  workspace=0x100) == E
    assert status(gf.gf_fuse_pack, csc, 3, pools=fake, residual=fake, sel_idx=fake, k=9, sendbuf=fake,
                  workspace=0x100) == E
    assert status(gf.gf_fuse_pack, csc, 3, pools=fake, residual=fake, sel_idx=fake, k=2, sendbuf=fake) == E  # no workspace
    assert status(gf.gf_fuse_pack, csc, 3, pools=fake, residual=fake, sel_idx=fake, k=2, sendbuf=fake,
                  workspace=0x104) == E                                                    # misaligned workspace
    assert status(gf.gf_fuse_pack, csc, 3, pools=fake, residual=fake, sel_idx=fake, k=2, sendbuf=fake,
                  workspace=0x100) == S                                                    # valid, but not uploaded
    assert status(gf.gf_fuse_pack, dense, 3, pools=fake, sendbuf=fake) == S
    # select
    assert status(gf.gf_chunk_score_select, csc, fake, k=0, sel_idx=fake, scores=fake) == E
    assert status(gf.gf_chunk_score_select, csc, fake, k=9, sel_idx=fake, scores=fake) == E
    assert status(gf.gf_chunk_score_select, dense, fake, k=1, sel_idx=fake, scores=fake) == E
    assert status(gf.gf_chunk_score_select, csc, fake, k=1, sel_idx=fake, prev_sel=fake, k_prev=1, scores=fake) == E
    assert status(gf.gf_chunk_score_select, csc, fake, k=1, sel_idx=fake) == E             # scores need workspace
    assert status(gf.gf_chunk_score_select, csc, fake, k=1, sel_idx=fake, scores=fake) == S
    # ring
    assert status(gf.gf_ring_reduce_sim, csc, fake, -1, fake) == E
    assert status(gf.gf_ring_reduce_sim, csc, fake, 8193, fake) == E
    assert status(gf.gf_ring_reduce_sim, dense, fake, 100, fake) == E                      # dense reduces all N
    assert status(gf.gf_ring_reduce_sim, dense, fake, 8192, fake, L_dev=fake) == E
    assert status(gf.gf_ring_reduce_sim, dense, fake, 8192, fake) == S
    assert status(gf.gf_ring_reduce_sim, csc, fake, 2048, fake, L_dev=fake) == S
    # unpack
    assert status(gf.gf_unpack_apply, csc, fake, 1024, sel_idx=fake, k=1) == E             # nowhere to write
    assert status(gf.gf_unpack_apply, csc, fake, 1025, sel_idx=fake, k=1, out_pool=fake) == E
    assert status(gf.gf_unpack_apply, csc, fake, 1024, sel_idx=fake, k=2, out_pool=fake) == E
    assert status(gf.gf_unpack_apply, dense, fake, 8192, reduced_l1=fake, out_pool=fake) == E
    assert status(gf.gf_unpack_apply, dense, fake, 8000, out_pool=fake) == E
    assert status(gf.gf_unpack_apply, csc, fake, 2000, sel_idx=fake, k=2, out_pool=fake) == S
    # unpack + SGD update: weights and history in exactly one form
    upd = dict(momentum=0.9, learning_rate=0.1)
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1024, sel_idx=fake, k=1, **upd) == E
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1024, sel_idx=fake, k=1, w_pool=fake, **upd) == E
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1024, sel_idx=fake, k=1, w_pool=fake, hu_pool=fake,
                  w_tensors=fake, hu_tensors=fake, **upd) == E
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1024, sel_idx=fake, k=1, w_pool=fake, hu_tensors=fake, **upd) == E
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1025, sel_idx=fake, k=1, w_pool=fake, hu_pool=fake, **upd) == E
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1024, sel_idx=fake, k=1, w_pool=fake, hu_pool=fake, **upd) == S
    assert status(gf.gf_unpack_sgd_update, dense, fake, 8192, w_tensors=fake, hu_tensors=fake, **upd) == S
    # the FP16 copy of the weights comes in the same form as the weights
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1024, sel_idx=fake, k=1, w_pool=fake, hu_pool=fake,
                  w_half_tensors=fake, **upd) == E
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1024, sel_idx=fake, k=1, w_tensors=fake, hu_tensors=fake,
                  w_half_pool=fake, **upd) == E
    assert status(gf.gf_unpack_sgd_update, csc, fake, 1024, sel_idx=fake, k=1, w_pool=fake, hu_pool=fake,
                  w_half_pool=fake, **upd) == S


def test_modifier_bits_and_range_calls_validate_before_touching_the_gpu():
    csc = gf.Plan([4096, 4096], 1 << 40, 1024, 2, to_device=False)        # 8 chunks
    dense = gf.Plan([4096, 4096], 1 << 40, 0, 2, to_device=False)
    fake, ws = 0x1000, 0x100
    E, S, Lim = gf.GF_EINVAL, gf.GF_ESTATE, gf.GF_ELIMIT
    A, K, SL, DF = gf.GF_PHASE_ACCUM, gf.GF_PHASE_PACK, gf.GF_PHASE_SLOTS, gf.GF_PHASE_DEFER_NORMS

    def status(fn, *a, **kw):
        with pytest.raises(gf.GfError) as e:
            fn(*a, stream=0, **kw)
        return e.value.status

    sparse = dict(pools=fake, residual=fake, sel_idx=fake, k=2, sendbuf=fake)
    # modifier bits need what they modify
    assert status(gf.gf_fuse_pack, csc, SL, **sparse, workspace=ws) == E                 # no phase at all
    assert status(gf.gf_fuse_pack, csc, 16 | A, pools=fake, residual=fake, workspace=ws) == E   # unknown bit
    assert status(gf.gf_fuse_pack, csc, A | SL, pools=fake, residual=fake, workspace=ws) == E   # slots without a pack
    assert status(gf.gf_fuse_pack, csc, A | K | SL, pools=fake, residual=fake, sendbuf=fake, workspace=ws) == E  # no selection
    assert status(gf.gf_fuse_pack, csc, K | DF, residual=fake, sel_idx=fake, k=2, sendbuf=fake, workspace=ws) == E  # no norms in a pack
    assert status(gf.gf_fuse_pack, dense, A | K | DF, pools=fake, sendbuf=fake, workspace=ws) == E
    assert status(gf.gf_fuse_pack, csc, A | DF, pools=fake, residual=fake) == E               # nowhere to leave them
    assert status(gf.gf_fuse_pack, csc, A | K | SL | DF, **sparse, workspace=ws) == S         # valid, not uploaded
    assert status(gf.gf_fuse_pack, csc, A | DF, pools=fake, residual=fake, workspace=ws) == S
    # a selection that takes its norms from the workspace needs one
    assert status(gf.gf_chunk_score_select, csc, None, k=1, sel_idx=fake, scores=fake) == E
    assert status(gf.gf_chunk_score_select, csc, None, k=1, sel_idx=fake, scores=fake, workspace=0x104) == E
    assert status(gf.gf_chunk_score_select, csc, None, k=1, sel_idx=fake, workspace=ws) == S
    # chunk ranges
    rng = dict(pools=fake, residual=fake, workspace=ws)
    assert status(gf.gf_fuse_pack_range, csc, A, -1, 4, **rng) == E
    assert status(gf.gf_fuse_pack_range, csc, A, 5, 4, **rng) == E
    assert status(gf.gf_fuse_pack_range, csc, A, 0, 9, **rng) == E
    assert status(gf.gf_fuse_pack_range, dense, A | K, 0, 1, pools=fake, sendbuf=fake) == E      # chunks needed
    assert status(gf.gf_fuse_pack_range, csc, K, 2, 4, residual=fake, sel_idx=fake, k=2, sendbuf=fake, workspace=ws) == E
    assert status(gf.gf_fuse_pack_range, csc, A | K, 2, 4, **sparse, workspace=ws) == S
    assert status(gf.gf_ring_reduce_range, csc, fake, 2048, fake, None, 2, 0, 4) == E              # no selection
    assert status(gf.gf_ring_reduce_range, csc, fake, 2000, fake, fake, 2, 0, 4) == E              # L is the capacity k*C
    assert status(gf.gf_ring_reduce_range, csc, fake, 2048, fake, fake, 2, 3, 2) == E
    assert status(gf.gf_ring_reduce_range, csc, fake, 2048, fake, fake, 9, 0, 4) == E
    assert status(gf.gf_ring_reduce_range, dense, fake, 8192, fake, fake, 1, 0, 1) == E
    assert status(gf.gf_ring_reduce_range, csc, fake, 2048, fake, fake, 2, 0, 4) == S
    assert status(gf.gf_unpack_range, csc, fake, 2048, None, 2, 0, 4, out_pool=fake) == E
    assert status(gf.gf_unpack_range, csc, fake, 2048, fake, 2, 0, 9, out_pool=fake) == E
    assert status(gf.gf_unpack_range, csc, fake, 2048, fake, 2, 0, 4) == E                         # nowhere to write
    assert status(gf.gf_unpack_range, dense, fake, 8192, fake, 1, 0, 1, out_pool=fake) == E
    assert status(gf.gf_unpack_range, csc, fake, 2048, fake, 2, 0, 4, out_pool=fake) == S
    gf.gf_ring_reduce_range(csc, fake, 2048, fake, fake, 2, 3, 3, stream=0)                        # empty range: nothing to do
    gf.gf_unpack_range(csc, fake, 2048, fake, 2, 3, 3, out_pool=fake, stream=0)
    # the variant with its own scratch takes neither hand-over and has a size limit
    assert status(gf.gf_fuse_pack_static, csc, A | K | SL, **sparse) == E
    assert status(gf.gf_fuse_pack_static, csc, A | DF, pools=fake, residual=fake) == E
    big = gf.Plan([5000 * 8200], 1 << 40, 8200, 64, to_device=False)
    assert big.workspace_bytes() > gf.GF_STATIC_SCRATCH_BYTES
    assert status(gf.gf_fuse_pack_static, big, A, pools=fake, residual=fake, chunk_l1=fake) == Lim


def test_the_one_call_iteration_validates_everything_before_the_first_launch():
    csc = gf.Plan([4096, 4096], 1 << 40, 1024, 2, to_device=False)        # 8 chunks
    dense = gf.Plan([4096, 4096], 1 << 40, 0, 2, to_device=False)
    fake, ws = 0x1000, 0x100
    E, S = gf.GF_EINVAL, gf.GF_ESTATE

    def status(plan, modifiers=0, **change):
        kw = dict(pools=fake, residual=fake, sel_idx=fake, k=2, k_next=3, packed_len=fake, sendbuf=fake,
                  reduced=fake, out_pool=fake, reduced_l1=fake, workspace=ws)
        kw.update(change)
        with pytest.raises(gf.GfError) as e:
            gf.gf_csc_iteration(plan, modifiers, stream=0, **kw)
        return e.value.status

    assert status(csc) == S                                               # valid, but not uploaded
    assert status(csc, gf.GF_PHASE_SLOTS, scores=fake, mask=fake, allgather_out=fake) == S
    assert status(dense) == E                                             # needs chunks
    assert status(csc, gf.GF_PHASE_DEFER_NORMS) == E                      # the only modifier is the slot map's
    assert status(csc, 16) == E
    assert status(csc, grads=fake) == E                                   # both gradient forms
    assert status(csc, pools=None) == E                                   # neither
    for missing in ("residual", "sel_idx", "packed_len", "sendbuf", "reduced", "reduced_l1", "workspace"):
        assert status(csc, **{missing: None}) == E, missing
    assert status(csc, out_pool=None) == E                                # nowhere to write
    assert status(csc, out_pool=None, out_tensors=fake) == S
    assert status(csc, k=0) == E
    assert status(csc, k=9) == E
    assert status(csc, k_next=0) == E
    assert status(csc, k_next=9) == E
    assert status(csc, workspace=0x104) == E


def test_the_header_is_plain_c(tmp_path):
    """include/gf.h is the boundary for C callers: it must compile as C99 on its own, and a C
    program must link against the library and reach a host-only call."""
    import subprocess
    src = tmp_path / "use_gf.c"
    src.write_text(
        '#include "gf.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "    int64_t numel[3] = {5, 7, 11}, N = 0; int32_t nc = 0, nb = 0; gf_plan *p = 0;\n"
        "    if (gf_plan_create(&p, numel, 3, 6, 4, 2, GF_WIRE_F16) != GF_OK) return 1;\n"
        "    if (gf_plan_info(p, &N, &nc, &nb) != GF_OK) return 2;\n"
        '    printf("%lld %d %d %s\\n", (long long)N, nc, nb, gf_status_string(GF_ELIMIT));\n'
        "    gf_plan_destroy(p);\n    return 0;\n}\n")
    exe = tmp_path / "use_gf"
    inc = os.path.join(ROOT, "include")
    libdir = os.path.dirname(gf_build.LIB)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                    os.path.join(inc, "gf.h")], check=True)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", inc, str(src), "-o", str(exe), "-L", libdir,
                    "-l:libgf.so", "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert out[:3] == ["23", "6", "3"]          # 23 elements, 6 chunks of 4, buckets {11}, {7} (7 > 6), {5}
