"""ctypes access to the CPU checker in gf_oracle.c (test infrastructure).

Arrays are numpy, C-contiguous; fp16 data travels as uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

from . import build as _build

# GF_ORACLE_LIB: another build of the same source (the sanitizer build the tests make)
_lib = C.CDLL(os.environ.get("GF_ORACLE_LIB") or _build.build())

_i32, _i64, _f32 = C.c_int32, C.c_int64, C.c_float
_vp = C.c_void_p


def _ptr(a: Optional[np.ndarray]):
    if a is None:
        return None
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(_vp)


def _sig(name, restype, *argtypes):
    f = getattr(_lib, name)
    f.restype = restype
    f.argtypes = list(argtypes)
    return f


_set_threads = _sig("gfo_set_threads", None, C.c_int)
_get_threads = _sig("gfo_get_threads", C.c_int)
_f2h = _sig("gfo_f32_to_f16_array", None, _vp, _vp, _i64)
_h2f = _sig("gfo_f16_to_f32_array", None, _vp, _vp, _i64)
_hadd = _sig("gfo_f16_add", C.c_uint16, C.c_uint16, C.c_uint16)
_layout = _sig("gfo_layout", _i64, _vp, _i32, _vp)
_buckets = _sig("gfo_buckets", _i32, _vp, _i32, _i64, _vp, _vp)
_n_chunks = _sig("gfo_n_chunks", _i64, _i64, _i64)
_packed_len = _sig("gfo_packed_len", _i64, _i64, _i64, _vp, _i32)
_packed_buckets = _sig("gfo_packed_buckets", _i32, _i64, _i64, _vp, _i32, _i64, _vp, _vp)
_warmup_k = _sig("gfo_warmup_k", _i64, _i64, C.c_double, _i64, _i64)
_accumulate_w = _sig("gfo_accumulate_workers", None, _vp, _vp, _vp, _i32, _i64)
_chunk_l1 = _sig("gfo_chunk_l1", None, _vp, _i64, _i64, _vp)
_chunk_l1_w = _sig("gfo_chunk_l1_workers", None, _vp, _i32, _i64, _i64, _vp)
_score = _sig("gfo_score", None, _vp, _i32, _i64, _vp, _i32, _vp, _vp)
_select = _sig("gfo_select", None, _vp, _i64, _i32, _vp, _vp)
_pack_w = _sig("gfo_pack_residual_workers", None, _i32, _vp, _i32, _i64, _i64, _vp, _i32,
               _f32, _f32, _vp, _vp)
_cast_w = _sig("gfo_cast_dense_workers", None, _i32, _vp, _i32, _i64, _f32, _vp)
_ring_seg = _sig("gfo_ring_segment", _i64, _i64, _i32, C.c_int)
_ring_hops = _sig("gfo_ring_allreduce_hops", None, C.c_int, _vp, _i64, _i32, _vp)
_ring_fold = _sig("gfo_ring_fold", None, C.c_int, _vp, _i64, _i32, _vp)
_hier_hops = _sig("gfo_hier_allreduce_hops", None, C.c_int, _vp, _i64, _i32, _i32, _vp)
_hier_fold = _sig("gfo_hier_fold", None, C.c_int, _vp, _i64, _i32, _i32, _vp)
_unpack = _sig("gfo_unpack", None, C.c_int, _vp, _i64, _i64, _vp, _i32, _f32, _vp, _vp)
_sgd_update = _sig("gfo_sgd_update", None, C.c_int, _vp, _i64, _i64, _vp, _i32, _f32, _f32, _f32, _vp, _vp, _vp, _vp)
_unpack_dense = _sig("gfo_unpack_dense", None, C.c_int, _vp, _i64, _f32, _vp)

WIRE = {"f16": 0, "f32": 1}
WIRE_DTYPE = {"f16": np.uint16, "f32": np.float32}


def set_threads(n: int) -> None:
    _set_threads(int(n))


def get_threads() -> int:
    return int(_get_threads())


def f32_to_f16(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    h = np.empty(x.shape, dtype=np.uint16)
    _f2h(_ptr(x), _ptr(h), x.size)
    return h


def f16_to_f32(h: np.ndarray) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16)
    x = np.empty(h.shape, dtype=np.float32)
    _h2f(_ptr(h), _ptr(x), h.size)
    return x


def f16_add(a: int, b: int) -> int:
    return int(_hadd(int(a), int(b)))


def layout(sizes: Sequence[int]) -> Tuple[np.ndarray, int]:
    s = np.asarray(sizes, dtype=np.int64)
    off = np.empty(len(s), dtype=np.int64)
    n = _layout(_ptr(s), len(s), _ptr(off))
    return off, int(n)


def buckets(sizes: Sequence[int], theta: int) -> Tuple[np.ndarray, np.ndarray]:
    s = np.asarray(sizes, dtype=np.int64)
    lo = np.empty(len(s), dtype=np.int64)
    hi = np.empty(len(s), dtype=np.int64)
    nb = _buckets(_ptr(s), len(s), int(theta), _ptr(lo), _ptr(hi))
    return lo[:nb].copy(), hi[:nb].copy()


def n_chunks(N: int, Cc: int) -> int:
    return int(_n_chunks(int(N), int(Cc)))


def packed_len(N: int, Cc: int, sel: np.ndarray) -> int:
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    return int(_packed_len(int(N), int(Cc), _ptr(sel), len(sel)))


def packed_buckets(N: int, Cc: int, sel: np.ndarray, theta: int) -> Tuple[np.ndarray, np.ndarray]:
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    lo = np.empty(len(sel), dtype=np.int64)
    hi = np.empty(len(sel), dtype=np.int64)
    nb = _packed_buckets(int(N), int(Cc), _ptr(sel), len(sel), int(theta), _ptr(lo), _ptr(hi))
    return lo[:nb].copy(), hi[:nb].copy()


def warmup_k(nc: int, final_density: float, t: int, warmup: int) -> int:
    return int(_warmup_k(int(nc), float(final_density), int(t), int(warmup)))


def accumulate(g: np.ndarray, hg: np.ndarray) -> np.ndarray:
    """g, hg: [P, N] fp32 -> acc [P, N]."""
    assert g.dtype == np.float32 and hg.dtype == np.float32 and g.shape == hg.shape
    acc = np.empty_like(g)
    P, N = g.shape
    _accumulate_w(_ptr(g), _ptr(hg), _ptr(acc), P, N)
    return acc


def chunk_l1_f64(acc1: np.ndarray, Cc: int) -> np.ndarray:
    """One worker's pool [N] -> fp64 norms [n_chunks]."""
    assert acc1.dtype == np.float32 and acc1.ndim == 1
    out = np.empty(n_chunks(acc1.size, Cc), dtype=np.float64)
    _chunk_l1(_ptr(acc1), acc1.size, int(Cc), _ptr(out))
    return out


def chunk_l1(acc: np.ndarray, Cc: int) -> np.ndarray:
    """acc [P, N] -> norms [P, n_chunks] stored in single precision."""
    assert acc.dtype == np.float32 and acc.ndim == 2
    P, N = acc.shape
    out = np.empty((P, n_chunks(N, Cc)), dtype=np.float32)
    _chunk_l1_w(_ptr(acc), P, N, int(Cc), _ptr(out))
    return out


def score(l1f: np.ndarray, sent: Optional[np.ndarray] = None,
          red_l1: Optional[np.ndarray] = None) -> np.ndarray:
    assert l1f.dtype == np.float32 and l1f.ndim == 2
    P, nc = l1f.shape
    out = np.empty(nc, dtype=np.float32)
    if sent is None or len(sent) == 0:
        _score(_ptr(l1f), P, nc, None, 0, None, _ptr(out))
    else:
        sent = np.ascontiguousarray(sent, dtype=np.int32)
        red_l1 = np.ascontiguousarray(red_l1, dtype=np.float32)
        assert len(sent) == len(red_l1)
        _score(_ptr(l1f), P, nc, _ptr(sent), len(sent), _ptr(red_l1), _ptr(out))
    return out


def select(sc: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray]:
    sc = np.ascontiguousarray(sc, dtype=np.float32)
    assert 1 <= k <= sc.size
    sel = np.empty(k, dtype=np.int32)
    mask = np.empty(sc.size, dtype=np.uint8)
    _select(_ptr(sc), sc.size, int(k), _ptr(sel), _ptr(mask))
    return sel, mask


def pack_residual(acc: np.ndarray, Cc: int, sel: np.ndarray, S: float, mu: float,
                  wire: str = "f16") -> Tuple[np.ndarray, np.ndarray]:
    """acc [P, N] -> (send [P, L] wire dtype, hg [P, N])."""
    assert acc.dtype == np.float32 and acc.ndim == 2
    P, N = acc.shape
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    L = packed_len(N, Cc, sel)
    send = np.empty((P, L), dtype=WIRE_DTYPE[wire])
    hg = np.empty_like(acc)
    _pack_w(WIRE[wire], _ptr(acc), P, N, int(Cc), _ptr(sel), len(sel), float(S), float(mu),
            _ptr(send), _ptr(hg))
    return send, hg


def cast_dense(g: np.ndarray, S: float, wire: str = "f16") -> np.ndarray:
    assert g.dtype == np.float32 and g.ndim == 2
    P, N = g.shape
    send = np.empty((P, N), dtype=WIRE_DTYPE[wire])
    _cast_w(WIRE[wire], _ptr(g), P, N, float(S), _ptr(send))
    return send


def ring_segment(L: int, P: int, wire: str = "f16") -> int:
    return int(_ring_seg(int(L), int(P), WIRE[wire]))


def ring_allreduce_hops(x: np.ndarray, wire: str = "f16") -> Tuple[np.ndarray, np.ndarray]:
    """x [P, L] -> (all ranks' final buffers [P, L], elements sent per rank [P])."""
    assert x.dtype == WIRE_DTYPE[wire] and x.ndim == 2
    buf = x.copy()
    P, L = buf.shape
    sent = np.zeros(P, dtype=np.int64)
    _ring_hops(WIRE[wire], _ptr(buf), L, P, _ptr(sent))
    return buf, sent


def ring_fold(x: np.ndarray, wire: str = "f16") -> np.ndarray:
    assert x.dtype == WIRE_DTYPE[wire] and x.ndim == 2
    x = np.ascontiguousarray(x)
    P, L = x.shape
    out = np.empty(L, dtype=x.dtype)
    _ring_fold(WIRE[wire], _ptr(x), L, P, _ptr(out))
    return out


def hier_allreduce_hops(x: np.ndarray, M: int, wire: str = "f16") -> Tuple[np.ndarray, np.ndarray]:
    """Hierarchical allreduce with M groups of consecutive ranks, message by message:
    x [P, L] -> (all ranks' final buffers [P, L], elements sent per rank [P])."""
    assert x.dtype == WIRE_DTYPE[wire] and x.ndim == 2
    buf = x.copy()
    P, L = buf.shape
    assert 1 <= M <= P and P % M == 0
    sent = np.zeros(P, dtype=np.int64)
    _hier_hops(WIRE[wire], _ptr(buf), L, P, int(M), _ptr(sent))
    return buf, sent


def hier_fold(x: np.ndarray, M: int, wire: str = "f16") -> np.ndarray:
    assert x.dtype == WIRE_DTYPE[wire] and x.ndim == 2
    x = np.ascontiguousarray(x)
    P, L = x.shape
    assert 1 <= M <= P and P % M == 0
    out = np.empty(L, dtype=x.dtype)
    _hier_fold(WIRE[wire], _ptr(x), L, P, int(M), _ptr(out))
    return out


def allreduce(x: np.ndarray, wire: str = "f16", groups: int = 0) -> np.ndarray:
    """The reduced buffer [L] of x [P, L]: flat ring, or hierarchical with `groups` groups."""
    return hier_fold(x, groups, wire) if groups else ring_fold(x, wire)


def unpack(reduced: np.ndarray, N: int, Cc: int, sel: np.ndarray, alpha: float,
           out: np.ndarray, wire: str = "f16") -> np.ndarray:
    """Writes the important chunks of `out` [N] in place; returns their norms [k]."""
    assert reduced.dtype == WIRE_DTYPE[wire] and out.dtype == np.float32 and out.size == N
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    assert reduced.size == packed_len(N, Cc, sel)
    red_l1 = np.empty(len(sel), dtype=np.float32)
    _unpack(WIRE[wire], _ptr(reduced), int(N), int(Cc), _ptr(sel), len(sel), float(alpha),
            _ptr(out), _ptr(red_l1))
    return red_l1


def sgd_update(reduced: np.ndarray, N: int, Cc: int, sel: np.ndarray, alpha: float, momentum: float,
               lr: float, w: np.ndarray, hu: np.ndarray, out: Optional[np.ndarray] = None,
               wire: str = "f16", w_half: Optional[np.ndarray] = None) -> None:
    """Algorithm 1's update step on the important chunks; w, hu (and out, and the FP16 copy of the
    weights w_half, uint16 bit patterns) [N] are updated in place."""
    assert reduced.dtype == WIRE_DTYPE[wire] and w.dtype == np.float32 and hu.dtype == np.float32
    assert w.size == N and hu.size == N and (out is None or (out.dtype == np.float32 and out.size == N))
    assert w_half is None or (w_half.dtype == np.uint16 and w_half.size == N)
    sel = np.ascontiguousarray(sel, dtype=np.int32)
    assert reduced.size == packed_len(N, Cc, sel)
    _sgd_update(WIRE[wire], _ptr(reduced), int(N), int(Cc), _ptr(sel), len(sel), float(alpha),
                float(momentum), float(lr), _ptr(w), _ptr(hu), _ptr(out), _ptr(w_half))


def unpack_dense(reduced: np.ndarray, alpha: float, wire: str = "f16") -> np.ndarray:
    assert reduced.dtype == WIRE_DTYPE[wire]
    out = np.empty(reduced.size, dtype=np.float32)
    _unpack_dense(WIRE[wire], _ptr(reduced), reduced.size, float(alpha), _ptr(out))
    return out
