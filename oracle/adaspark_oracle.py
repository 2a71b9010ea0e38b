"""ctypes front end of the fp64 C oracle (``adaspark_oracle.c``).

TEST INFRASTRUCTURE, NOT PRODUCT CODE: argument marshalling only, every number
is produced by the C file next to this one.  Arrays are numpy; bf16 tensors are
passed as their uint16 bit patterns.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "adaspark_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


class _CShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int) for n in ("T", "H", "W", "ct", "ch", "cw", "Hq", "Hkv", "D", "text", "lead")]


@dataclass(frozen=True)
class Shape:
    """Token grid (frames, height, width), cube shape and head geometry."""

    T: int
    H: int
    W: int
    ct: int
    ch: int
    cw: int
    Hq: int
    Hkv: int
    D: int
    text: int = 0  # text tokens that follow the video tokens
    lead: int = 0  # text tokens that precede the video tokens

    @property
    def S(self) -> int:
        return self.lead + self.T * self.H * self.W + self.text

    def _c(self) -> _CShape:
        return _CShape(self.T, self.H, self.W, self.ct, self.ch, self.cw, self.Hq, self.Hkv, self.D, self.text,
                       self.lead)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP over rows, no fast-math)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"]
        )
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_num_cubes.restype = ctypes.c_int
        _lib.oracle_top_p.restype = ctypes.c_int
        _lib.oracle_top_k.restype = ctypes.c_int
    return _lib


def _p(a, typ):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(typ))


def _u16(a) -> np.ndarray:
    """bf16 torch tensor or uint16 array -> contiguous uint16 numpy array."""
    if isinstance(a, np.ndarray):
        assert a.dtype == np.uint16
        return np.ascontiguousarray(a)
    import torch  # only to view a CPU bf16 tensor's bits

    assert a.dtype == torch.bfloat16 and a.device.type == "cpu"
    return a.contiguous().view(torch.int16).numpy().view(np.uint16)


def num_threads() -> int:
    """Threads the OpenMP loops will use (OMP_NUM_THREADS or the affinity mask)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    return len(os.sched_getaffinity(0))


def num_cubes(shape: Shape) -> int:
    cs = shape._c()
    return int(_load().oracle_num_cubes(ctypes.byref(cs)))


def cube_map(shape: Shape):
    """-> (cube_of[S], rank_of[S], size_of[N], start[N+1])  (Sec. 3.1)."""
    lib, cs, N = _load(), shape._c(), num_cubes(shape)
    cube_of = np.empty(shape.S, np.int32)
    rank_of = np.empty(shape.S, np.int32)
    size_of = np.empty(N, np.int32)
    start = np.empty(N + 1, np.int64)
    lib.oracle_cube_map(ctypes.byref(cs), _p(cube_of, ctypes.c_int32), _p(rank_of, ctypes.c_int32),
                        _p(size_of, ctypes.c_int32), _p(start, ctypes.c_int64))
    return cube_of, rank_of, size_of, start


def cube_pool(shape: Shape, K) -> np.ndarray:
    """Mean key per (cube, KV head): fp64 [N, Hkv, D]  (Eq. 1)."""
    lib, cs, N = _load(), shape._c(), num_cubes(shape)
    k = _u16(K)
    assert k.size == shape.S * shape.Hkv * shape.D
    kbar = np.empty((N, shape.Hkv, shape.D), np.float64)
    lib.oracle_cube_pool(ctypes.byref(cs), _p(k, ctypes.c_uint16), _p(kbar, ctypes.c_double))
    return kbar


def relevance(q: np.ndarray, kbar_rows: np.ndarray):
    """One row's logits and softmax over the given mean keys [n, D]  (Eq. 1)."""
    lib = _load()
    q = np.ascontiguousarray(q, np.float64)
    kb = np.ascontiguousarray(kbar_rows, np.float64)
    n, D = kb.shape
    logits = np.empty(n, np.float64)
    probs = np.empty(n, np.float64)
    lib.oracle_relevance(_p(q, ctypes.c_double), _p(kb, ctypes.c_double), ctypes.c_int64(D),
                         ctypes.c_int(n), ctypes.c_int(D), _p(logits, ctypes.c_double), _p(probs, ctypes.c_double))
    return logits, probs


def top_p(probs: np.ndarray, p: float):
    """Nucleus rule on one distribution -> (keep[n] bool, order[n], cum[n])  (Eq. 2)."""
    lib = _load()
    pr = np.ascontiguousarray(probs, np.float64)
    n = pr.size
    keep = np.zeros(n, np.uint8)
    order = np.zeros(n, np.int32)
    cum = np.zeros(n, np.float64)
    lib.oracle_top_p(_p(pr, ctypes.c_double), ctypes.c_int(n), ctypes.c_double(p), _p(keep, ctypes.c_uint8),
                     _p(order, ctypes.c_int32), _p(cum, ctypes.c_double))
    return keep.astype(bool), order, cum


def _rows(rows):
    if rows is None:
        return None
    return np.ascontiguousarray(rows, np.int64)


def cube_select(shape: Shape, Q, kbar: np.ndarray, p: float, rows=None, eps: float = 1e-5, causal: bool = True):
    """Selection for the given rows (all if None).

    -> (sel_mask uint32 [nrows, ceil(N/32)], sel_count int32 [nrows], near_cut bool [nrows])
    """
    lib, cs, N = _load(), shape._c(), num_cubes(shape)
    q = _u16(Q)
    assert q.size == shape.S * shape.Hq * shape.D
    kb = np.ascontiguousarray(kbar, np.float64)
    assert kb.shape == (N, shape.Hkv, shape.D)
    r = _rows(rows)
    nrows = shape.S * shape.Hq if r is None else r.size
    words = (N + 31) // 32
    mask = np.zeros((nrows, words), np.uint32)
    count = np.zeros(nrows, np.int32)
    near = np.zeros(nrows, np.uint8)
    fn = lib.oracle_cube_select if causal else lib.oracle_cube_select_noncausal
    fn(ctypes.byref(cs), _p(q, ctypes.c_uint16), _p(kb, ctypes.c_double), ctypes.c_double(p),
       _p(r, ctypes.c_int64), ctypes.c_int64(nrows), _p(mask, ctypes.c_uint32),
       _p(count, ctypes.c_int32), _p(near, ctypes.c_uint8), ctypes.c_double(eps))
    return mask, count, near.astype(bool)


def top_k(probs: np.ndarray, k: int):
    """Fixed Top-K rule on one distribution -> (keep[n] bool, order[n])."""
    lib = _load()
    pr = np.ascontiguousarray(probs, np.float64)
    n = pr.size
    keep = np.zeros(n, np.uint8)
    order = np.zeros(n, np.int32)
    lib.oracle_top_k(_p(pr, ctypes.c_double), ctypes.c_int(n), ctypes.c_int(k), _p(keep, ctypes.c_uint8),
                     _p(order, ctypes.c_int32))
    return keep.astype(bool), order


def cube_select_topk(shape: Shape, Q, kbar: np.ndarray, k: int, rows=None, eps: float = 1e-5):
    """Top-K selection for the given rows (all if None); outputs as cube_select."""
    lib, cs, N = _load(), shape._c(), num_cubes(shape)
    q = _u16(Q)
    assert q.size == shape.S * shape.Hq * shape.D
    kb = np.ascontiguousarray(kbar, np.float64)
    assert kb.shape == (N, shape.Hkv, shape.D)
    r = _rows(rows)
    nrows = shape.S * shape.Hq if r is None else r.size
    words = (N + 31) // 32
    mask = np.zeros((nrows, words), np.uint32)
    count = np.zeros(nrows, np.int32)
    near = np.zeros(nrows, np.uint8)
    lib.oracle_cube_select_topk(ctypes.byref(cs), _p(q, ctypes.c_uint16), _p(kb, ctypes.c_double), ctypes.c_int(int(k)),
                                _p(r, ctypes.c_int64), ctypes.c_int64(nrows), _p(mask, ctypes.c_uint32),
                                _p(count, ctypes.c_int32), _p(near, ctypes.c_uint8), ctypes.c_double(eps))
    return mask, count, near.astype(bool)


def sparse_attn(shape: Shape, Q, K, V, sel_mask: np.ndarray, rows=None, causal: bool = True):
    """Eq. 3 on the given rows -> (out fp64 [nrows, D], n_keys int64 [nrows]).  causal False: the own cube is
    attended in full and selected cubes may lie after it."""
    lib, cs, N = _load(), shape._c(), num_cubes(shape)
    q, k, v = _u16(Q), _u16(K), _u16(V)
    r = _rows(rows)
    nrows = shape.S * shape.Hq if r is None else r.size
    words = (N + 31) // 32
    m = np.ascontiguousarray(sel_mask, np.uint32)
    assert m.shape == (nrows, words)
    out = np.empty((nrows, shape.D), np.float64)
    nk = np.empty(nrows, np.int64)
    fn = lib.oracle_sparse_attn if causal else lib.oracle_sparse_attn_noncausal
    fn(ctypes.byref(cs), _p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
       _p(r, ctypes.c_int64), ctypes.c_int64(nrows), _p(m, ctypes.c_uint32),
       _p(out, ctypes.c_double), _p(nk, ctypes.c_int64))
    return out, nk


def dense_attn(shape: Shape, Q, K, V, rows=None, causal: bool = True) -> np.ndarray:
    """Causal attention in cube-major order on the given rows -> fp64 [nrows, D]; causal False: attention over all
    tokens."""
    lib, cs = _load(), shape._c()
    q, k, v = _u16(Q), _u16(K), _u16(V)
    r = _rows(rows)
    nrows = shape.S * shape.Hq if r is None else r.size
    out = np.empty((nrows, shape.D), np.float64)
    fn = lib.oracle_dense_attn if causal else lib.oracle_dense_attn_noncausal
    fn(ctypes.byref(cs), _p(q, ctypes.c_uint16), _p(k, ctypes.c_uint16), _p(v, ctypes.c_uint16),
       _p(r, ctypes.c_int64), ctypes.c_int64(nrows), _p(out, ctypes.c_double))
    return out


def bf16_round(x32: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even (NaN inputs are not expected here)."""
    u = np.ascontiguousarray(x32, np.float32).view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(np.uint16)


def group_mean_query(shape: Shape, Q) -> np.ndarray:
    """The query that scores the cubes for a whole GQA group: bf16 bit patterns [S, Hkv, D].

    The precision is part of the definition (a selection is decided by it, so both sides compute it alike): the
    group's queries are added in head order in float32, the sum is multiplied by float32(1)/float32(G), and the
    product is rounded to bf16 (nearest even)."""
    q = _u16(Q).reshape(shape.S, shape.Hkv, shape.Hq // shape.Hkv, shape.D)
    q32 = (q.astype(np.uint32) << 16).view(np.float32)
    acc = np.zeros((shape.S, shape.Hkv, shape.D), np.float32)
    for g in range(shape.Hq // shape.Hkv):
        acc = acc + q32[:, :, g, :]
    inv = np.float32(1.0) / np.float32(shape.Hq // shape.Hkv)
    return bf16_round(acc * inv)


def cube_select_shared(shape: Shape, Q, kbar: np.ndarray, p: float, eps: float = 1e-5):
    """Group-shared selection (a variant, not in the paper): Eqs. 1-2 applied once per (token, KV head) to the
    group's mean query (group_mean_query), the kept set shared by all query heads of the group.
    -> (sel_mask uint32 [S*Hq, words], sel_count int32 [S*Hq], near_cut bool [S*Hq]), rows n*Hq + a."""
    G = shape.Hq // shape.Hkv
    one = Shape(shape.T, shape.H, shape.W, shape.ct, shape.ch, shape.cw, shape.Hkv, shape.Hkv, shape.D, shape.text,
                shape.lead)
    mask, count, near = cube_select(one, group_mean_query(shape, Q), kbar, p, eps=eps)
    rows = np.arange(shape.S * shape.Hq)
    src = (rows // shape.Hq) * shape.Hkv + (rows % shape.Hq) // G
    return mask[src], count[src], near[src]
