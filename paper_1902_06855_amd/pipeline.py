"""One simulated iteration of the path, as calls into the C-ABI library.

`Pipeline` owns the device buffers of a run (through PyTorch, used only as an
allocator) and strings the four entry points together in the order of
Sections 3.1-3.2 of the paper.  It computes nothing itself.

Schedules for a plan with chunks (coarse-grained sparse communication):
  "lagged"     the paper's: the chunks sent at iteration t were chosen at the
               end of iteration t-1, so accumulate, norms, pack and the
               historical-gradient rule are one pass (gf_fuse_pack with both
               phases).  Iteration 0 chooses from its own accumulated gradients.
  "immediate"  every iteration chooses from its own accumulated gradients:
               accumulate pass, select, pack pass.
A dense plan (chunk = 0) runs cast -> per-bucket ring -> cast back.  With fp16
pools as input and `zero_copy` set, the cast pass is dropped: the ring reads
the workers' pools in place (the memory pool of Section 3.1 holding fp16
gradients, reduced bucket by bucket with no copy).
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np
import torch

from . import gf


class Pipeline:
    def __init__(self, sizes: Sequence[int], P: int, chunk: int, theta: int, loss_scale: float,
                 k: int = 0, mu: float = 1.0, wire: str = "f16", schedule: str = "lagged",
                 scatter_out: bool = False, allgather: bool = False, device: str = "cuda",
                 sgd: Optional[tuple] = None, k_max: Optional[int] = None, grad: str = "f32",
                 zero_copy: bool = False, groups: int = 0, fast: bool = True, half_weights: bool = False):
        assert schedule in ("lagged", "immediate")
        # fast: the calls of an iteration hand the slot map and the unfinished chunk norms to each
        # other through the workspace (two small launches fewer per iteration; `self.l1` is then
        # never written).  The results are the same bit for bit.
        self.fast = bool(fast)
        if zero_copy and not (chunk == 0 and grad == "f16" and wire == "f16"):
            raise ValueError("zero_copy needs a dense plan with fp16 pools on an fp16 wire")
        self.zero_copy = bool(zero_copy)
        self.sizes, self.P, self.chunk, self.mu = list(sizes), int(P), int(chunk), float(mu)
        self.S, self.schedule, self.device = float(loss_scale), schedule, device
        self.alpha = float(np.float32(1.0) / np.float32(loss_scale))   # 1/S rounded once to fp32
        self.wire = gf.GF_WIRE_F16 if wire == "f16" else gf.GF_WIRE_F32
        self.wdtype = torch.float16 if wire == "f16" else torch.float32
        # groups: hierarchical allreduce with that many groups (Section 2.4); 0 = flat ring
        self.plan = gf.Plan(self.sizes, min(int(theta), 1 << 60), self.chunk, self.P, self.wire, groups=groups)
        if grad == "f16":                      # gradients arrive as fp16 (mixed-precision backward)
            self.plan.set_grad_type(gf.GF_WIRE_F16)
        self.N, self.n_chunks, self.m = self.plan.N, self.plan.n_chunks, len(self.sizes)
        # k: important chunks in the current selection; k_next: how many the next selection
        # takes (warm-up changes it between iterations); buffers are sized for k_max
        self.k = self.k_next = int(k) if self.chunk else 0
        self.k_max = max(int(k_max or 0), self.k)
        self.ws = self.plan.workspace()
        self.t = 0
        new = lambda n, dt: torch.zeros(n, dtype=dt, device=device)
        if self.chunk:
            assert 1 <= self.k <= self.k_max <= self.n_chunks
            self.cap_max = self.k_max * self.chunk              # packed-buffer capacity, elements
            self.residual = [new(self.N, torch.float32) for _ in range(self.P)]
            self.residual_tab = gf.ptr_table(self.residual, device)
            self.l1 = new(self.P * self.n_chunks, torch.float32)
            self.scores = new(self.n_chunks, torch.float32)
            self.sel = new(self.k_max, torch.int32)
            self.mask = new(self.n_chunks, torch.uint8)
            self.packed_len = new(1, torch.int64)
            self.red_l1 = new(self.k_max, torch.float32)
        else:
            self.cap_max = self.N
            self.residual = None
        self.send, self.send_tab = None, None
        if not self.zero_copy:
            self.send = [new(self.cap_max, self.wdtype) for _ in range(self.P)]
            self.send_tab = gf.ptr_table(self.send, device)
        self.reduced = new(self.cap_max, self.wdtype)
        self.out_pool = new(self.N, torch.float32)
        self.out_tensors = self.out_tab = None
        if scatter_out:
            self.out_tensors = [new(s, torch.float32) for s in self.sizes]
            self.out_tab = gf.ptr_table(self.out_tensors, device)
        self.ag = self.ag_tab = None
        if allgather:
            self.ag = [new(self.cap_max, self.wdtype) for _ in range(self.P)]
            self.ag_tab = gf.ptr_table(self.ag, device)
        # sgd = (momentum, learning_rate): unpack also applies Algorithm 1's update step to
        # weight and historical-update pools (or per-tensor buffers when scatter_out is set)
        self.sgd = sgd
        self.w = self.hu = self.w_tab = self.hu_tab = None
        if sgd is not None:
            if scatter_out:
                self.w = [new(s, torch.float32) for s in self.sizes]
                self.hu = [new(s, torch.float32) for s in self.sizes]
                self.w_tab, self.hu_tab = gf.ptr_table(self.w, device), gf.ptr_table(self.hu, device)
            else:
                self.w, self.hu = new(self.N, torch.float32), new(self.N, torch.float32)
        # half_weights: the update also maintains the FP16 copy of the weights that forward and
        # backward use under mixed precision (Section 2.5), in the same form as the weights
        self.w16 = self.w16_tab = None
        if half_weights:
            if sgd is None:
                raise ValueError("half_weights belongs to the SGD-update step: pass sgd=(momentum, learning_rate)")
            if scatter_out:
                self.w16 = [new(s, torch.float16) for s in self.sizes]
                self.w16_tab = gf.ptr_table(self.w16, device)
            else:
                self.w16 = new(self.N, torch.float16)
        self.grads_tab = self.pools_tab = None
        self._keep = None
        self.probe = None            # list to collect (stage, start event, end event) per launch
        self.probe_only = None       # bracket only this stage (fewer event packets between kernels)

    @property
    def cap(self) -> int:
        """Upper bound of the packed length for the current selection (elements)."""
        return self.k * self.chunk if self.chunk else self.N

    # ------------------------------------------------------------- inputs
    def set_gradients(self, grads: List[List[torch.Tensor]]) -> None:
        """grads[p][l]: scattered fp32 device tensors in ID order (fusion happens in the read)."""
        flat = [t for row in grads for t in row]
        assert len(flat) == self.P * self.m
        self._keep = grads
        self.grads_tab, self.pools_tab = gf.ptr_table(flat, self.device), None

    def set_pools(self, pools: List[torch.Tensor]) -> None:
        """pools[p]: N-element fp32 pools already in generation order (zero-copy lazy allreduce)."""
        assert len(pools) == self.P and all(p.numel() == self.N for p in pools)
        self._keep = pools
        self.pools_tab, self.grads_tab = gf.ptr_table(pools, self.device), None

    def use_tables(self, grads_tab: Optional[torch.Tensor], pools_tab: Optional[torch.Tensor]) -> None:
        """Switch to pointer tables prepared earlier (no allocation, no copy)."""
        self.grads_tab, self.pools_tab = grads_tab, pools_tab

    # ------------------------------------------------------------- stages
    def accum(self) -> None:
        defer = gf.GF_PHASE_DEFER_NORMS if self.fast else 0
        gf.gf_fuse_pack(self.plan, gf.GF_PHASE_ACCUM | defer, grads=self.grads_tab, pools=self.pools_tab,
                        residual=self.residual_tab, chunk_l1=None if self.fast else self.l1, workspace=self.ws)

    def select(self, after_allreduce: bool) -> None:
        """Choose self.sel (in place); after_allreduce scores the chunks just sent by their reduced norm."""
        l1 = None if self.fast else self.l1          # fast: the norms are still in the workspace
        if after_allreduce:
            gf.gf_chunk_score_select(self.plan, l1, reduced_l1=self.red_l1, prev_sel=self.sel, k_prev=self.k,
                                     k=self.k_next, scores=self.scores, sel_idx=self.sel, mask=self.mask,
                                     packed_len=self.packed_len, workspace=self.ws)
        else:
            gf.gf_chunk_score_select(self.plan, l1, k=self.k_next, scores=self.scores, sel_idx=self.sel,
                                     mask=self.mask, packed_len=self.packed_len, workspace=self.ws)
        self.k = self.k_next

    def pack(self) -> None:
        # self.sel always comes from the last select() on this workspace, which left its slot map there
        slots = gf.GF_PHASE_SLOTS if self.fast else 0
        gf.gf_fuse_pack(self.plan, gf.GF_PHASE_PACK | slots, residual=self.residual_tab, sel_idx=self.sel, k=self.k,
                        loss_scale=self.S, mu=self.mu, sendbuf=self.send_tab, workspace=self.ws)

    def fused(self) -> None:
        extra = (gf.GF_PHASE_SLOTS | gf.GF_PHASE_DEFER_NORMS) if self.fast else 0
        gf.gf_fuse_pack(self.plan, gf.GF_PHASE_ACCUM | gf.GF_PHASE_PACK | extra, grads=self.grads_tab,
                        pools=self.pools_tab, residual=self.residual_tab, sel_idx=self.sel, k=self.k,
                        loss_scale=self.S, mu=self.mu, sendbuf=self.send_tab,
                        chunk_l1=None if self.fast else self.l1, workspace=self.ws)

    def cast_dense(self) -> None:
        gf.gf_fuse_pack(self.plan, gf.GF_PHASE_ACCUM | gf.GF_PHASE_PACK, grads=self.grads_tab,
                        pools=self.pools_tab, loss_scale=self.S, sendbuf=self.send_tab, workspace=self.ws)

    def ring(self) -> None:
        if self.chunk:   # the packed length stays on the device
            gf.gf_ring_reduce_sim(self.plan, self.send_tab, self.cap, self.reduced, L_dev=self.packed_len,
                                  allgather_out=self.ag_tab, workspace=self.ws)
        else:
            src = self.pools_tab if self.zero_copy else self.send_tab
            if src is None:
                raise ValueError("zero_copy reduces pools in place: call set_pools first")
            gf.gf_ring_reduce_sim(self.plan, src, self.N, self.reduced, allgather_out=self.ag_tab,
                                  workspace=self.ws)

    def unpack(self) -> None:
        if self.sgd is not None:
            pooled = self.w_tab is None
            gf.gf_unpack_sgd_update(self.plan, self.reduced, self.cap, sel_idx=self.sel if self.chunk else None,
                                    k=self.k, alpha=self.alpha, momentum=self.sgd[0], learning_rate=self.sgd[1],
                                    w_pool=self.w if pooled else None, hu_pool=self.hu if pooled else None,
                                    w_tensors=self.w_tab, hu_tensors=self.hu_tab,
                                    w_half_pool=self.w16 if (pooled and self.w16 is not None) else None,
                                    w_half_tensors=self.w16_tab, out_pool=self.out_pool,
                                    reduced_l1=self.red_l1 if self.chunk else None, workspace=self.ws)
            return
        if self.chunk:
            gf.gf_unpack_apply(self.plan, self.reduced, self.cap, sel_idx=self.sel, k=self.k, alpha=self.alpha,
                               out_pool=self.out_pool, out_tensors=self.out_tab, reduced_l1=self.red_l1,
                               workspace=self.ws)
        else:
            gf.gf_unpack_apply(self.plan, self.reduced, self.N, alpha=self.alpha, out_pool=self.out_pool,
                               out_tensors=self.out_tab, workspace=self.ws)

    # ---------------------------------------------------------- iteration
    def _run(self, name: str, fn, after: bool = False) -> None:
        """Run one stage; with a probe list attached, bracket it with events on the launch stream."""
        if self.probe is None or (self.probe_only is not None and name != self.probe_only):
            fn(after) if name == "select" else fn()
            return
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn(after) if name == "select" else fn()
        e1.record()
        self.probe.append((name, e0, e1))

    def capture(self) -> "torch.cuda.CUDAGraph":
        """Record one steady-state iteration, with the gradient tables and the k in use now, as a
        HIP graph; `replay()` on the result then launches the whole iteration at once.  Every
        launch of an iteration depends on the one before it, so the graph saves only the host's
        share of the gaps between kernels.  Not for the bootstrap iteration of the lagged
        schedule, nor while warm-up still changes k."""
        if self.chunk and self.schedule == "lagged" and self.t == 0:
            raise ValueError("the first iteration of the lagged schedule is not a steady-state one")
        if self.probe is not None:
            raise ValueError("event probes cannot be recorded into a graph")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step()
        return graph

    def step(self) -> None:
        """One whole iteration on the current stream; returns without synchronising."""
        if not self.chunk:
            if not self.zero_copy:
                self._run("cast", self.cast_dense)
            self._run("ring", self.ring); self._run("unpack", self.unpack)
        elif self.schedule == "immediate" or self.t == 0:
            self._run("accum", self.accum); self._run("select", self.select, False)
            self._run("pack", self.pack); self._run("ring", self.ring); self._run("unpack", self.unpack)
            if self.schedule == "lagged":
                self._run("select", self.select, True)
        elif self.fast and self.sgd is None and self.probe is None:
            self.iteration()
        else:
            self._run("fused", self.fused); self._run("ring", self.ring); self._run("unpack", self.unpack)
            self._run("select", self.select, True)
        self.t += 1

    def iteration(self) -> None:
        """A steady-state lagged iteration as one call into the library (the same four launches)."""
        gf.gf_csc_iteration(self.plan, gf.GF_PHASE_SLOTS, grads=self.grads_tab, pools=self.pools_tab,
                            residual=self.residual_tab, sel_idx=self.sel, k=self.k, k_next=self.k_next,
                            packed_len=self.packed_len, loss_scale=self.S, mu=self.mu, sendbuf=self.send_tab,
                            reduced=self.reduced, allgather_out=self.ag_tab, alpha=self.alpha,
                            out_pool=self.out_pool, out_tensors=self.out_tab, reduced_l1=self.red_l1,
                            scores=self.scores, mask=self.mask, workspace=self.ws)
        self.k = self.k_next


class OverlappedDense:
    """The enable-overlap setting of lazy allreduce (Sections 2.6 and 3.1): every bucket is cast,
    reduced and cast back on its own, on side streams, in the order backward produces the
    buckets (tensor m first), each as soon as its gradients are there, instead of one pass over
    the whole pool after backward.

    A bucket holds whole tensors and is one contiguous range of the pool, so it is a dense plan of
    its own over those tensors; the same entry points are called with pointers that start at the
    bucket.  The results are those of the single-pass `Pipeline` bit for bit (every bucket is its
    own ring there as well).  It computes nothing itself."""

    def __init__(self, sizes: Sequence[int], P: int, theta: int, loss_scale: float, wire: str = "f16",
                 n_streams: int = 2, device: str = "cuda", grad: str = "f32", groups: int = 0):
        self.sizes, self.P, self.S, self.device = list(sizes), int(P), float(loss_scale), device
        self.alpha = float(np.float32(1.0) / np.float32(loss_scale))
        self.wire = gf.GF_WIRE_F16 if wire == "f16" else gf.GF_WIRE_F32
        self.wdtype = torch.float16 if wire == "f16" else torch.float32
        whole = gf.Plan(self.sizes, min(int(theta), 1 << 60), 0, self.P, self.wire, to_device=False)
        self.N, self.m = whole.N, len(self.sizes)
        self.off, self.lo, self.hi = whole.layout()
        whole.close()
        new = lambda n, dt: torch.zeros(n, dtype=dt, device=device)
        self.send = [new(self.N, self.wdtype) for _ in range(self.P)]
        self.reduced = new(self.N, self.wdtype)
        self.out_pool = new(self.N, torch.float32)
        # tensors of bucket b, ID order: those whose pool offset lies in [lo, hi)
        self.members = [[j for j in range(self.m) if lo <= self.off[j] < hi] for lo, hi in zip(self.lo, self.hi)]
        self.plans = []
        for mem in self.members:
            plan = gf.Plan([self.sizes[j] for j in mem], 1 << 60, 0, self.P, self.wire, groups=groups)
            if grad == "f16":
                plan.set_grad_type(gf.GF_WIRE_F16)
            self.plans.append(plan)
        self.send_tabs = [gf.ptr_table([s[lo:] for s in self.send], device) for lo in self.lo]
        self.streams = [torch.cuda.Stream(device=device) for _ in range(max(1, int(n_streams)))]   # default priority
        self.grad_tabs = self.pool_tabs = None
        self._keep = None

    @property
    def n_buckets(self) -> int:
        return len(self.lo)

    def set_gradients(self, grads: List[List[torch.Tensor]]) -> None:
        """grads[p][l]: scattered device tensors in ID order."""
        self._keep = grads
        self.grad_tabs = [gf.ptr_table([grads[p][j] for p in range(self.P) for j in mem], self.device)
                          for mem in self.members]
        self.pool_tabs = None

    def set_pools(self, pools: List[torch.Tensor]) -> None:
        """pools[p]: N-element pools in generation order (read in place, bucket by bucket)."""
        self._keep = pools
        self.pool_tabs = [gf.ptr_table([q[lo:] for q in pools], self.device) for lo in self.lo]
        self.grad_tabs = None

    def step(self, ready: Optional[Sequence[torch.cuda.Event]] = None) -> None:
        """Issue every bucket in generation order.  ready[b], if given, is an event recorded once
        the gradients of bucket b exist (by whatever produces them); bucket b waits for it alone.
        Returns without synchronising; the current stream waits for all buckets."""
        cur = torch.cuda.current_stream()
        start = torch.cuda.Event()
        start.record(cur)
        for b, plan in enumerate(self.plans):
            s = self.streams[b % len(self.streams)]
            s.wait_event(start)
            if ready is not None:
                s.wait_event(ready[b])
            lo, hi = self.lo[b], self.hi[b]
            with torch.cuda.stream(s):
                gf.gf_fuse_pack(plan, gf.GF_PHASE_ACCUM | gf.GF_PHASE_PACK,
                                grads=self.grad_tabs[b] if self.grad_tabs else None,
                                pools=self.pool_tabs[b] if self.pool_tabs else None,
                                loss_scale=self.S, sendbuf=self.send_tabs[b])
                gf.gf_ring_reduce_sim(plan, self.send_tabs[b], hi - lo, self.reduced[lo:])
                gf.gf_unpack_apply(plan, self.reduced[lo:], hi - lo, alpha=self.alpha, out_pool=self.out_pool[lo:])
        for s in self.streams:
            cur.wait_stream(s)

    def capture(self) -> "torch.cuda.CUDAGraph":
        """The whole bucket-by-bucket iteration (side streams forked from and joined to the current
        one, no arrival events) as one HIP graph: takes the host's launch rate out of the picture."""
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step()
        return graph


class OverlappedCsc:
    """Coarse-grained sparse communication with the enable-overlap setting (Section 3.2: an important
    chunk goes into the packed buffer as soon as backward has filled it, and the buffer goes to
    allreduce whenever what waits in it exceeds the threshold; Section 3.1): the pool is swept range by
    range in generation order, each range as soon as its gradients exist, and every bucket of the
    packed buffer is reduced and unpacked right after the sweep that completed it, while the next
    ranges are still being swept.

    Two side streams: one runs the sweeps (gf_fuse_pack_range) in order, the other the
    allreduce and unpack of the buckets each sweep completed (gf_ring_reduce_range,
    gf_unpack_range), which decide on the device, from the selection, which buckets those are.
    The host therefore never reads the selection, and a whole iteration can be recorded in a graph.
    Iteration 0 (the selection needs every norm first) and the selection at the end of every
    iteration run as in `Pipeline`.  The results are those of `Pipeline` bit for bit.  It
    computes nothing itself."""

    def __init__(self, sizes: Sequence[int], P: int, chunk: int, theta: int, loss_scale: float, k: int,
                 boundaries: Sequence[int], mu: float = 1.0, wire: str = "f16", device: str = "cuda",
                 grad: str = "f32", groups: int = 0, scatter_out: bool = False, allgather: bool = False):
        if not chunk:
            raise ValueError("a plan with chunks is needed (dense plans: OverlappedDense)")
        self.pipe = Pipeline(sizes, P, chunk, theta, loss_scale, k=k, mu=mu, wire=wire, schedule="lagged",
                             scatter_out=scatter_out, allgather=allgather, device=device, grad=grad, groups=groups,
                             fast=True)
        nc = self.pipe.n_chunks
        self.bounds = [int(b) for b in boundaries]
        if not self.bounds or self.bounds != sorted(set(self.bounds)) or self.bounds[0] < 1 or self.bounds[-1] != nc:
            raise ValueError("boundaries: ascending chunk indices, the last one n_chunks")
        self.sweep_stream = torch.cuda.Stream(device=device)       # default priority
        self.reduce_stream = torch.cuda.Stream(device=device)

    @property
    def n_ranges(self) -> int:
        return len(self.bounds)

    def step(self, ready: Optional[Sequence[torch.cuda.Event]] = None) -> None:
        """One iteration.  ready[r], if given, is an event recorded once the gradients of chunk
        range r exist; the sweep of that range waits for it (and for the sweeps before it).
        Returns without synchronising; the current stream waits for everything."""
        p = self.pipe
        if p.t == 0:
            if ready is not None:
                torch.cuda.current_stream().wait_event(ready[-1])
            p.step()
            return
        cur = torch.cuda.current_stream()
        start = torch.cuda.Event()
        start.record(cur)
        self.sweep_stream.wait_event(start)
        self.reduce_stream.wait_event(start)
        phase = gf.GF_PHASE_ACCUM | gf.GF_PHASE_PACK | gf.GF_PHASE_SLOTS | gf.GF_PHASE_DEFER_NORMS
        lo = 0
        for r, hi in enumerate(self.bounds):
            if ready is not None:
                self.sweep_stream.wait_event(ready[r])
            with torch.cuda.stream(self.sweep_stream):
                gf.gf_fuse_pack_range(p.plan, phase, lo, hi, grads=p.grads_tab, pools=p.pools_tab,
                                      residual=p.residual_tab, sel_idx=p.sel, k=p.k, loss_scale=p.S, mu=p.mu,
                                      sendbuf=p.send_tab, workspace=p.ws)
                swept = torch.cuda.Event()
                swept.record(self.sweep_stream)
            self.reduce_stream.wait_event(swept)
            with torch.cuda.stream(self.reduce_stream):
                gf.gf_ring_reduce_range(p.plan, p.send_tab, p.cap, p.reduced, p.sel, p.k, lo, hi,
                                        L_dev=p.packed_len, allgather_out=p.ag_tab, workspace=p.ws)
                gf.gf_unpack_range(p.plan, p.reduced, p.cap, p.sel, p.k, lo, hi, alpha=p.alpha, out_pool=p.out_pool,
                                   out_tensors=p.out_tab, reduced_l1=p.red_l1, workspace=p.ws)
            lo = hi
        cur.wait_stream(self.sweep_stream)
        cur.wait_stream(self.reduce_stream)
        p.select(True)
        p.t += 1

    def capture(self) -> "torch.cuda.CUDAGraph":
        """A steady-state iteration (both side streams forked from and joined to the current one, no
        arrival events) as one HIP graph.  The graph stays valid from iteration to iteration: which
        buckets a call reduces is decided on the device."""
        if self.pipe.t == 0:
            raise ValueError("the first iteration is not a steady-state one")
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.step()
        return graph
