"""Whole iterations of the path, assembled from the CPU checker's steps
(test infrastructure; see gf_oracle.c for the arithmetic of each step).

Order of one iteration with coarse-grained sparse communication on
(Section 3.2 and Algorithm 1 of the paper):

  acc = g + hg                       allreduce preprocess
  l1[p][c] = ||acc_p[chunk c]||_1    local chunk norms
  pack important chunks as fp16(acc*S); hg = 0 there, hg = momentum*acc elsewhere
  ring allreduce of the packed buffer (Section 2.4), fp16 rounded at every hop
  unpack: out[chunk] = fp32(reduced) / S at the important chunks
  score, select the important chunks of the next iteration

Two schedules of the selection are provided.  "lagged" is the paper's: the
chunks used at iteration t were chosen at the end of iteration t-1 from the
state after the allreduce (sent chunks scored by the norm of their reduced
values, each GPU dividing by the GPU count before the norms are summed).
Iteration 0 has no predecessor and picks from its own accumulated gradients.
"immediate" picks, in every iteration, from that iteration's accumulated
gradients before packing.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

from . import binding as ob


def fuse(tensors: Sequence[np.ndarray], sizes: Sequence[int]) -> np.ndarray:
    """Place ID-ordered tensors in the pool (Section 3.1: tensor m first)."""
    off, N = ob.layout(sizes)
    pool = np.empty(N, dtype=np.float32)
    for j, t in enumerate(tensors):
        assert t.size == sizes[j]
        pool[off[j]:off[j] + sizes[j]] = np.asarray(t, dtype=np.float32).ravel()
    return pool


def views(pool: np.ndarray, sizes: Sequence[int]) -> List[np.ndarray]:
    off, _ = ob.layout(sizes)
    return [pool[off[j]:off[j] + sizes[j]] for j in range(len(sizes))]


def dense_iteration(pools: np.ndarray, sizes: Sequence[int], theta: int, S: float,
                    wire: str = "f16", groups: int = 0) -> Dict[str, np.ndarray]:
    """pools [P, N] fp32.  Lazy allreduce without sparsification: cast, one
    allreduce per bucket (flat ring, or hierarchical with `groups` groups), cast
    back (times 1/S)."""
    P, N = pools.shape
    lo, hi = ob.buckets(sizes, theta)
    send = ob.cast_dense(pools, S, wire)
    reduced = np.empty(N, dtype=send.dtype)
    for a, b in zip(lo, hi):
        reduced[a:b] = ob.allreduce(np.ascontiguousarray(send[:, a:b]), wire, groups)
    out = ob.unpack_dense(reduced, np.float32(1.0) / np.float32(S), wire)
    return dict(send=send, reduced=reduced, out=out, bucket_lo=lo, bucket_hi=hi)


@dataclass
class CscState:
    hg: np.ndarray                       # [P, N] historical gradients
    sel: Optional[np.ndarray] = None     # lagged schedule: chunks to send next


def new_state(P: int, N: int) -> CscState:
    return CscState(hg=np.zeros((P, N), dtype=np.float32))


def csc_iteration(state: CscState, pools: np.ndarray, C: int, k: int, S: float, mu: float,
                  schedule: str = "lagged", wire: str = "f16",
                  out: Optional[np.ndarray] = None, k_next: Optional[int] = None,
                  theta: int = 1 << 60,
                  choose: Optional[Callable[[str, np.ndarray, np.ndarray], np.ndarray]] = None,
                  groups: int = 0) -> Dict[str, np.ndarray]:
    """One iteration; updates `state` in place and returns every intermediate.

    k is the number of important chunks of this iteration; k_next (default k)
    is how many the lagged schedule picks for the next one (warm-up changes it
    from iteration to iteration).  theta is the lazy-allreduce threshold on the
    packed buffer: each bucket of it is reduced by an allreduce of its own
    (the flat ring, or the hierarchical one with `groups` groups).

    choose(stage, score, sel) may replace a selection (stage is "pre" for one
    taken before packing, "post" for one taken after the allreduce); tests use
    it to impose an equally valid choice when scores tie within tolerance.
    """
    assert schedule in ("lagged", "immediate")
    P, N = pools.shape
    r: Dict[str, np.ndarray] = {}
    acc = ob.accumulate(pools, state.hg)
    l1 = ob.chunk_l1(acc, C)
    r["acc"], r["l1"] = acc, l1

    if schedule == "immediate" or state.sel is None:
        sc = ob.score(l1)
        sel, _ = ob.select(sc, k)
        if choose is not None:
            sel = choose("pre", sc, sel)
        r["score_pre"] = sc
    else:
        sel = state.sel
    r["sel"] = sel

    send, hg = ob.pack_residual(acc, C, sel, S, mu, wire)
    state.hg = hg
    reduced = np.empty(send.shape[1], dtype=send.dtype)
    b_lo, b_hi = ob.packed_buckets(N, C, sel, theta)
    for a, b in zip(b_lo, b_hi):
        reduced[a:b] = ob.allreduce(np.ascontiguousarray(send[:, a:b]), wire, groups)
    r["packed_bucket_lo"], r["packed_bucket_hi"] = b_lo, b_hi
    if out is None:
        out = np.zeros(N, dtype=np.float32)
    red_l1 = ob.unpack(reduced, N, C, sel, np.float32(1.0) / np.float32(S), out, wire)
    r.update(send=send, hg=hg, reduced=reduced, out=out, red_l1=red_l1)

    if schedule == "lagged":
        sc = ob.score(l1, sel, red_l1)
        nxt, _ = ob.select(sc, k if k_next is None else k_next)
        if choose is not None:
            nxt = choose("post", sc, nxt)
        state.sel = nxt
        r["score_post"], r["sel_next"] = sc, nxt
    return r


def csc_iteration_in_ranges(state: CscState, pools: np.ndarray, C: int, k: int, S: float, mu: float,
                            boundaries: Sequence[int], theta: int, wire: str = "f16",
                            out: Optional[np.ndarray] = None, k_next: Optional[int] = None,
                            groups: int = 0) -> Dict[str, np.ndarray]:
    """A steady-state iteration of the lagged schedule the way Section 3.2 describes it running
    while backward is still filling the pool (the enable-overlap setting of Section 3.1).

    The pool fills in generation order, that is by ascending chunk index.  `boundaries` are
    ascending chunk indices ending with n_chunks: the pool is swept range by range,
    [0, b_0), [b_0, b_1), ...  A sweep accumulates, takes the norms of and packs the chunks of its
    range only (an important chunk that is filled is copied to the buffer).  After each sweep
    every bucket of the packed buffer that has just become complete (the waiting chunks exceed
    theta, or the pool's last important chunk is in) is allreduced and unpacked.  Selection
    follows once the pool is done.  Nothing here depends on how the pool is cut into ranges, so
    the result must equal csc_iteration(theta=theta) bit for bit; the tests check that.
    """
    assert state.sel is not None, "the first iteration chooses from its own gradients: nothing to overlap"
    P, N = pools.shape
    nc = ob.n_chunks(N, C)
    bounds = [int(b) for b in boundaries]
    assert bounds == sorted(set(bounds)) and bounds[-1] == nc and bounds[0] > 0
    sel = state.sel
    L = ob.packed_len(N, C, sel)
    wdt = ob.WIRE_DTYPE[wire]
    send = np.zeros((P, L), dtype=wdt)
    reduced = np.zeros(L, dtype=wdt)
    hg = state.hg.copy()
    acc = np.empty_like(pools)
    l1 = np.empty((P, nc), dtype=np.float32)
    if out is None:
        out = np.zeros(N, dtype=np.float32)
    red_l1 = np.zeros(len(sel), dtype=np.float32)
    slot_of = {int(c): j for j, c in enumerate(sel)}           # rank of a chunk in the selection
    slot_start = np.concatenate([[0], np.cumsum([min(N, (int(c) + 1) * C) - int(c) * C for c in sel])])
    b_lo, b_hi = ob.packed_buckets(N, C, sel, theta)
    # chunks (by rank in the selection) of every packed bucket
    members = [[j for j in range(len(sel)) if a <= slot_start[j] < b] for a, b in zip(b_lo, b_hi)]
    packed = np.zeros(len(sel), dtype=bool)
    done = np.zeros(len(b_lo), dtype=bool)
    alpha = np.float32(1.0) / np.float32(S)
    lo = 0
    for hi in bounds:
        e_lo, e_hi = lo * C, min(N, hi * C)
        a_r = ob.accumulate(np.ascontiguousarray(pools[:, e_lo:e_hi]), np.ascontiguousarray(hg[:, e_lo:e_hi]))
        acc[:, e_lo:e_hi] = a_r
        l1[:, lo:hi] = ob.chunk_l1(a_r, C)
        mine = np.array([c - lo for c in sel if lo <= c < hi], dtype=np.int32)
        s_r, hg_r = ob.pack_residual(a_r, C, mine, S, mu, wire)
        hg[:, e_lo:e_hi] = hg_r
        if len(mine):
            j0 = slot_of[int(mine[0]) + lo]
            send[:, slot_start[j0]:slot_start[j0] + s_r.shape[1]] = s_r
            packed[j0:j0 + len(mine)] = True
        for b, mem in enumerate(members):                       # buckets this sweep completed
            if done[b] or not (lo <= sel[mem[-1]] < hi):
                continue
            assert packed[mem].all(), "a bucket is reduced only when all its chunks are in the buffer"
            a, e = int(b_lo[b]), int(b_hi[b])
            reduced[a:e] = ob.allreduce(np.ascontiguousarray(send[:, a:e]), wire, groups)
            red_l1[mem] = ob.unpack(reduced[a:e], N, C, sel[mem], alpha, out, wire)
            done[b] = True
        lo = hi
    assert done.all() and packed.all()
    state.hg = hg
    sc = ob.score(l1, sel, red_l1)
    nxt, _ = ob.select(sc, k if k_next is None else k_next)
    state.sel = nxt
    return dict(acc=acc, l1=l1, sel=sel, send=send, hg=hg, reduced=reduced, out=out, red_l1=red_l1,
                score_post=sc, sel_next=nxt, packed_bucket_lo=b_lo, packed_bucket_hi=b_hi)
