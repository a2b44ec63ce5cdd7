"""Thin ctypes binding over the C-ABI library (include/gf.h).

Argument marshalling only: every step of the path runs in the HIP kernels of
libgf.so.  There is no fallback: if the library has not been built this module
raises on import, and every non-OK status raises GfError.

PyTorch appears here only as the owner of device memory and streams: tensors
are turned into raw device addresses, pointer tables are int64 tensors on the
device, and kernels are enqueued on torch's current stream unless told
otherwise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Optional, Sequence, Tuple

import torch  # loaded first so that the HIP runtime in the process is torch's

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgf.so")

if not os.path.exists(LIB_PATH):
    raise ImportError(
        f"{LIB_PATH} is missing: build it with `python -m paper_1902_06855_amd.build` "
        "(or __graft_entry__.build()); there is no fallback path")

_lib = C.CDLL(LIB_PATH)

GF_OK, GF_EINVAL, GF_ENOMEM, GF_EHIP, GF_ESTATE, GF_ELIMIT = 0, 1, 2, 3, 4, 5
GF_STATIC_SCRATCH_BYTES = 4 << 20
GF_WIRE_F16, GF_WIRE_F32 = 0, 1
GF_PHASE_ACCUM, GF_PHASE_PACK, GF_PHASE_SLOTS, GF_PHASE_DEFER_NORMS = 1, 2, 4, 8

EXPORTS = (
    "gf_status_string", "gf_plan_create", "gf_plan_set_grad_type", "gf_plan_set_reduce_groups",
    "gf_plan_to_device", "gf_plan_destroy", "gf_plan_info",
    "gf_plan_layout", "gf_plan_ring_segment", "gf_plan_tiles", "gf_plan_tile_pieces",
    "gf_plan_workspace_bytes", "gf_plan_warmup_k", "gf_fuse_pack", "gf_fuse_pack_range", "gf_fuse_pack_static",
    "gf_chunk_score_select", "gf_ring_reduce_sim", "gf_ring_reduce_range", "gf_unpack_apply", "gf_unpack_range",
    "gf_unpack_sgd_update", "gf_csc_iteration",
)

_vp, _i32, _i64, _u32, _f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_float


def _sig(name, restype, *argtypes):
    f = getattr(_lib, name)
    f.restype = restype
    f.argtypes = list(argtypes)
    return f


_status_string = _sig("gf_status_string", C.c_char_p, C.c_int)
_plan_create = _sig("gf_plan_create", C.c_int, C.POINTER(_vp), C.POINTER(_i64), _i32, _i64, _i32, _i32, C.c_int)
_plan_to_device = _sig("gf_plan_to_device", C.c_int, _vp)
_plan_set_grad_type = _sig("gf_plan_set_grad_type", C.c_int, _vp, C.c_int)
_plan_set_reduce_groups = _sig("gf_plan_set_reduce_groups", C.c_int, _vp, _i32)
_plan_destroy = _sig("gf_plan_destroy", None, _vp)
_plan_info = _sig("gf_plan_info", C.c_int, _vp, C.POINTER(_i64), C.POINTER(_i32), C.POINTER(_i32))
_plan_layout = _sig("gf_plan_layout", C.c_int, _vp, C.POINTER(_i64), C.POINTER(_i64), C.POINTER(_i64))
_plan_ring_segment = _sig("gf_plan_ring_segment", _i64, _vp, _i64)
_plan_tiles = _sig("gf_plan_tiles", _i32, _vp)
_plan_tile_pieces = _sig("gf_plan_tile_pieces", _i32, _vp, _i32, _i32, C.POINTER(_i32), C.POINTER(_i64),
                         C.POINTER(_i32))
_plan_workspace_bytes = _sig("gf_plan_workspace_bytes", C.c_size_t, _vp)
_plan_warmup_k = _sig("gf_plan_warmup_k", _i32, _vp, C.c_double, _i64, _i64)
_fuse_pack = _sig("gf_fuse_pack", C.c_int, _vp, _u32, _vp, _vp, _vp, _vp, _i32, _f32, _f32, _vp, _vp, _vp, _vp)
_fuse_pack_range = _sig("gf_fuse_pack_range", C.c_int, _vp, _u32, _vp, _vp, _vp, _vp, _i32, _f32, _f32, _vp, _vp, _i32, _i32,
                        _vp, _vp)
_fuse_pack_static = _sig("gf_fuse_pack_static", C.c_int, _vp, _u32, _vp, _vp, _vp, _vp, _i32, _f32, _f32, _vp, _vp, _vp)
_chunk_score_select = _sig("gf_chunk_score_select", C.c_int, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _vp, _vp,
                           _vp, _vp, _vp)
_ring_reduce_sim = _sig("gf_ring_reduce_sim", C.c_int, _vp, _vp, _i64, _vp, _vp, _vp, _vp, _vp)
_ring_reduce_range = _sig("gf_ring_reduce_range", C.c_int, _vp, _vp, _i64, _vp, _vp, _i32, _i32, _i32, _vp, _vp, _vp, _vp)
_unpack_range = _sig("gf_unpack_range", C.c_int, _vp, _vp, _i64, _vp, _i32, _i32, _i32, _f32, _vp, _vp, _vp, _vp, _vp)
_unpack_apply = _sig("gf_unpack_apply", C.c_int, _vp, _vp, _i64, _vp, _i32, _f32, _vp, _vp, _vp, _vp, _vp)
_unpack_sgd_update = _sig("gf_unpack_sgd_update", C.c_int, _vp, _vp, _i64, _vp, _i32, _f32, _f32, _f32, _vp, _vp, _vp,
                          _vp, _vp, _vp, _vp, _vp, _vp, _vp)
_csc_iteration = _sig("gf_csc_iteration", C.c_int, _vp, _u32, _vp, _vp, _vp, _vp, _i32, _i32, _vp, _f32, _f32, _vp,
                      _vp, _vp, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _vp)


class GfError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {gf_status_string(status)}")


def gf_status_string(status: int) -> str:
    return _status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != GF_OK:
        raise GfError(status, where)


def _dptr(x) -> Optional[int]:
    """Device address of a tensor (or a raw int address, or None)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    assert isinstance(x, torch.Tensor) and x.is_cuda and x.is_contiguous(), "need a contiguous device tensor"
    return x.data_ptr()


def _stream(stream) -> Optional[int]:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream or None
    return int(stream) or None


def ptr_table(tensors: Sequence, device="cuda") -> torch.Tensor:
    """Device array of the device addresses of `tensors` (flat list)."""
    addrs = [t if isinstance(t, int) else t.data_ptr() for t in tensors]
    return torch.tensor(addrs, dtype=torch.int64).to(device)


class Plan:
    """Owner of a gf_plan handle."""

    def __init__(self, tensor_numel: Sequence[int], theta_elems: int, chunk_elems: int, P: int,
                 wire: int = GF_WIRE_F16, to_device: bool = True, groups: int = 0):
        m = len(tensor_numel)
        arr = (_i64 * m)(*[int(s) for s in tensor_numel])
        h = _vp()
        _check(_plan_create(C.byref(h), arr, m, int(theta_elems), int(chunk_elems), int(P), int(wire)),
               "gf_plan_create")
        self.handle = h
        self.m, self.P, self.chunk, self.wire = m, int(P), int(chunk_elems), int(wire)
        N, nc, nb = _i64(), _i32(), _i32()
        _check(_plan_info(h, C.byref(N), C.byref(nc), C.byref(nb)), "gf_plan_info")
        self.N, self.n_chunks, self.n_buckets = N.value, nc.value, nb.value
        self._workspace = None
        if groups:
            self.set_reduce_groups(groups)
        if to_device:
            self.to_device()

    def to_device(self) -> None:
        _check(_plan_to_device(self.handle), "gf_plan_to_device")

    def set_grad_type(self, wire: int) -> None:
        """GF_WIRE_F16: the gradients given to gf_fuse_pack are fp16; GF_WIRE_F32 (default): fp32."""
        _check(_plan_set_grad_type(self.handle, int(wire)), "gf_plan_set_grad_type")

    def set_reduce_groups(self, M: int) -> None:
        """Hierarchical allreduce with M groups (0 or P: the flat ring); before to_device only."""
        _check(_plan_set_reduce_groups(self.handle, int(M)), "gf_plan_set_reduce_groups")

    def layout(self) -> Tuple[List[int], List[int], List[int]]:
        off = (_i64 * self.m)()
        lo = (_i64 * self.n_buckets)()
        hi = (_i64 * self.n_buckets)()
        _check(_plan_layout(self.handle, off, lo, hi), "gf_plan_layout")
        return list(off), list(lo), list(hi)

    def ring_segment(self, L: int) -> int:
        return int(_plan_ring_segment(self.handle, int(L)))

    def tiles(self) -> int:
        return int(_plan_tiles(self.handle))

    def tile_pieces(self, tile: int) -> List[Tuple[int, int, int]]:
        n = _plan_tile_pieces(self.handle, int(tile), 0, None, None, None)
        if n < 0:
            raise GfError(GF_EINVAL, "gf_plan_tile_pieces")
        t, s, l = (_i32 * n)(), (_i64 * n)(), (_i32 * n)()
        _plan_tile_pieces(self.handle, int(tile), n, t, s, l)
        return [(t[i], s[i], l[i]) for i in range(n)]

    def warmup_k(self, final_density: float, iteration: int, warmup_iterations: int) -> int:
        k = int(_plan_warmup_k(self.handle, float(final_density), int(iteration), int(warmup_iterations)))
        if k < 0:
            raise GfError(GF_EINVAL, "gf_plan_warmup_k")
        return k

    def workspace_bytes(self) -> int:
        return int(_plan_workspace_bytes(self.handle))

    def workspace(self) -> torch.Tensor:
        """A device scratch buffer of the required size (allocated once)."""
        if self._workspace is None:
            self._workspace = torch.empty(self.workspace_bytes() + 256, dtype=torch.uint8, device="cuda")
            assert self._workspace.data_ptr() % 256 == 0
        return self._workspace

    def close(self) -> None:
        if getattr(self, "handle", None):
            _plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def gf_fuse_pack(plan: Plan, phase: int, *, grads=None, pools=None, residual=None, sel_idx=None, k: int = 0,
                 loss_scale: float = 1.0, mu: float = 1.0, sendbuf=None, chunk_l1=None, workspace=None,
                 stream=None) -> None:
    """grads / pools / residual / sendbuf are device pointer tables (see ptr_table)."""
    _check(_fuse_pack(plan.handle, int(phase), _dptr(grads), _dptr(pools), _dptr(residual), _dptr(sel_idx),
                      int(k), float(loss_scale), float(mu), _dptr(sendbuf), _dptr(chunk_l1), _dptr(workspace),
                      _stream(stream)), "gf_fuse_pack")


def gf_fuse_pack_range(plan: Plan, phase: int, chunk_lo: int, chunk_hi: int, *, grads=None, pools=None, residual=None,
                       sel_idx=None, k: int = 0, loss_scale: float = 1.0, mu: float = 1.0, sendbuf=None, chunk_l1=None,
                       workspace=None, stream=None) -> None:
    """gf_fuse_pack over the chunks [chunk_lo, chunk_hi) only."""
    _check(_fuse_pack_range(plan.handle, int(phase), _dptr(grads), _dptr(pools), _dptr(residual), _dptr(sel_idx),
                            int(k), float(loss_scale), float(mu), _dptr(sendbuf), _dptr(chunk_l1), int(chunk_lo),
                            int(chunk_hi), _dptr(workspace), _stream(stream)), "gf_fuse_pack_range")


def gf_fuse_pack_static(plan: Plan, phase: int, *, grads=None, pools=None, residual=None, sel_idx=None, k: int = 0,
                        loss_scale: float = 1.0, mu: float = 1.0, sendbuf=None, chunk_l1=None, stream=None) -> None:
    """gf_fuse_pack with the library's own fixed scratch instead of a workspace (allocates nothing)."""
    _check(_fuse_pack_static(plan.handle, int(phase), _dptr(grads), _dptr(pools), _dptr(residual), _dptr(sel_idx),
                             int(k), float(loss_scale), float(mu), _dptr(sendbuf), _dptr(chunk_l1),
                             _stream(stream)), "gf_fuse_pack_static")


def gf_chunk_score_select(plan: Plan, chunk_l1=None, *, reduced_l1=None, prev_sel=None, k_prev: int = 0, k: int,
                          scores=None, sel_idx, mask=None, packed_len=None, workspace=None, stream=None) -> None:
    _check(_chunk_score_select(plan.handle, _dptr(chunk_l1), _dptr(reduced_l1), _dptr(prev_sel), int(k_prev),
                               int(k), _dptr(scores), _dptr(sel_idx), _dptr(mask), _dptr(packed_len),
                               _dptr(workspace), _stream(stream)), "gf_chunk_score_select")


def gf_ring_reduce_sim(plan: Plan, sendbuf, L: int, reduced, *, L_dev=None, allgather_out=None, workspace=None,
                       stream=None) -> None:
    _check(_ring_reduce_sim(plan.handle, _dptr(sendbuf), int(L), _dptr(L_dev), _dptr(reduced),
                            _dptr(allgather_out), _dptr(workspace), _stream(stream)), "gf_ring_reduce_sim")


def gf_ring_reduce_range(plan: Plan, sendbuf, L: int, reduced, sel_idx, k: int, chunk_lo: int, chunk_hi: int, *,
                         L_dev=None, allgather_out=None, workspace=None, stream=None) -> None:
    """The packed buckets completed by the sweep over chunks [chunk_lo, chunk_hi)."""
    _check(_ring_reduce_range(plan.handle, _dptr(sendbuf), int(L), _dptr(L_dev), _dptr(sel_idx), int(k), int(chunk_lo),
                              int(chunk_hi), _dptr(reduced), _dptr(allgather_out), _dptr(workspace), _stream(stream)),
           "gf_ring_reduce_range")


def gf_unpack_range(plan: Plan, reduced, L: int, sel_idx, k: int, chunk_lo: int, chunk_hi: int, *, alpha: float = 1.0,
                    out_pool=None, out_tensors=None, reduced_l1=None, workspace=None, stream=None) -> None:
    _check(_unpack_range(plan.handle, _dptr(reduced), int(L), _dptr(sel_idx), int(k), int(chunk_lo), int(chunk_hi),
                         float(alpha), _dptr(out_pool), _dptr(out_tensors), _dptr(reduced_l1), _dptr(workspace),
                         _stream(stream)), "gf_unpack_range")


def gf_unpack_apply(plan: Plan, reduced, L: int, *, sel_idx=None, k: int = 0, alpha: float = 1.0, out_pool=None,
                    out_tensors=None, reduced_l1=None, workspace=None, stream=None) -> None:
    _check(_unpack_apply(plan.handle, _dptr(reduced), int(L), _dptr(sel_idx), int(k), float(alpha),
                         _dptr(out_pool), _dptr(out_tensors), _dptr(reduced_l1), _dptr(workspace),
                         _stream(stream)), "gf_unpack_apply")


def gf_unpack_sgd_update(plan: Plan, reduced, L: int, *, sel_idx=None, k: int = 0, alpha: float = 1.0,
                         momentum: float, learning_rate: float, w_pool=None, hu_pool=None, w_tensors=None,
                         hu_tensors=None, w_half_pool=None, w_half_tensors=None, out_pool=None, reduced_l1=None,
                         workspace=None, stream=None) -> None:
    _check(_unpack_sgd_update(plan.handle, _dptr(reduced), int(L), _dptr(sel_idx), int(k), float(alpha),
                              float(momentum), float(learning_rate), _dptr(w_pool), _dptr(hu_pool),
                              _dptr(w_tensors), _dptr(hu_tensors), _dptr(w_half_pool), _dptr(w_half_tensors),
                              _dptr(out_pool), _dptr(reduced_l1), _dptr(workspace), _stream(stream)),
           "gf_unpack_sgd_update")


def gf_csc_iteration(plan: Plan, modifiers: int = 0, *, grads=None, pools=None, residual, sel_idx, k: int,
                     k_next: Optional[int] = None, packed_len, loss_scale: float = 1.0, mu: float = 1.0, sendbuf,
                     reduced, allgather_out=None, alpha: float = 1.0, out_pool=None, out_tensors=None, reduced_l1,
                     scores=None, mask=None, workspace, stream=None) -> None:
    """One steady-state lagged iteration (fuse-pack, allreduce, unpack, select) in one call."""
    _check(_csc_iteration(plan.handle, int(modifiers), _dptr(grads), _dptr(pools), _dptr(residual), _dptr(sel_idx),
                          int(k), int(k if k_next is None else k_next), _dptr(packed_len), float(loss_scale),
                          float(mu), _dptr(sendbuf), _dptr(reduced), _dptr(allgather_out), float(alpha),
                          _dptr(out_pool), _dptr(out_tensors), _dptr(reduced_l1), _dptr(scores), _dptr(mask),
                          _dptr(workspace), _stream(stream)), "gf_csc_iteration")
