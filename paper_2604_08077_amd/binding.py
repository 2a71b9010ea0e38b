"""Thin ctypes binding of ``libadaspark.so`` (see ``include/adaspark.h``).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  torch is used for device memory (outputs and workspaces are torch
tensors) and for the current HIP stream.  There is no CPU fallback: if the
library has not been built, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

from .build import lib_path

CALL_CUBE_POOL, CALL_CUBE_SELECT, CALL_SPARSE_ATTN, CALL_DENSE_ATTN, CALL_ATTN_BWD, CALL_CUBE_SELECT_SHARED = 0, 1, 2, 3, 4, 5
CALL_SPARSE_ATTN_CSR = 6
ECAPACITY = -5  # ADASPARK_ECAPACITY: what a selection call leaves in its device status word on list overflow


class _CShape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in (
        "frames", "height", "width", "cube_t", "cube_h", "cube_w", "q_heads", "kv_heads", "head_dim", "text_tokens",
        "prefix_tokens")]


@dataclass(frozen=True)
class Shape:
    """Mirror of ``adaspark_shape``."""

    frames: int
    height: int
    width: int
    cube_t: int
    cube_h: int
    cube_w: int
    q_heads: int
    kv_heads: int
    head_dim: int
    text_tokens: int = 0    # text tokens that follow the video tokens
    prefix_tokens: int = 0  # text tokens that precede the video tokens

    @property
    def tokens(self) -> int:
        return self.prefix_tokens + self.frames * self.height * self.width + self.text_tokens

    @property
    def rows(self) -> int:
        return self.tokens * self.q_heads

    def _c(self) -> _CShape:
        return _CShape(self.frames, self.height, self.width, self.cube_t, self.cube_h, self.cube_w,
                       self.q_heads, self.kv_heads, self.head_dim, self.text_tokens, self.prefix_tokens)

    @staticmethod
    def of(w) -> "Shape":
        """From a ``synth.Workload``."""
        return Shape(w.T, w.H, w.W, w.ct, w.ch, w.cw, w.Hq, w.Hkv, w.D, w.text, w.lead)


class _CFfnDims(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32)]


class AdasparkError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


_lib = None

EXPORTS = (
    "adaspark_num_cubes",
    "adaspark_workspace_bytes",
    "adaspark_status_string",
    "adaspark_pairs_workspace_bytes",
    "adaspark_cube_pool",
    "adaspark_cube_select",
    "adaspark_select_status_offset",
    "adaspark_cube_select_noalloc",
    "adaspark_cube_select_topk",
    "adaspark_cube_select_shared",
    "adaspark_sparse_attn",
    "adaspark_sparse_attn_csr",
    "adaspark_dense_attn",
    "adaspark_kv_pack",
    "adaspark_sparse_attn_packed",
    "adaspark_sparse_attn_packed_with",
    "adaspark_dense_attn_packed",
    "adaspark_sparse_attn_bwd",
    "adaspark_ffn_workspace_bytes",
    "adaspark_ffn_select",
    "adaspark_ffn_sparse",
    "adaspark_probe_copy",
    "adaspark_probe_mfma",
)

SPARSE_AUTO, SPARSE_COMPACT, SPARSE_MASKED, SPARSE_PAIRS = 0, 1, 2, 3
NOALLOC_SCRATCH_BYTES = 4 << 20  # ADASPARK_NOALLOC_SCRATCH_BYTES


def load():
    """dlopen the library; raises if it was not built (no fallback)."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(
                f"{path} is missing: build it first (python -m paper_2604_08077_amd.build); "
                "this package has no CPU or eager fallback")
        lib = ctypes.CDLL(path)
        vp, sp = ctypes.c_void_p, ctypes.POINTER(_CShape)
        lib.adaspark_num_cubes.argtypes = [sp, ctypes.POINTER(ctypes.c_int32)]
        lib.adaspark_workspace_bytes.argtypes = [sp, ctypes.c_int, ctypes.POINTER(ctypes.c_size_t)]
        lib.adaspark_status_string.argtypes = [ctypes.c_int]
        lib.adaspark_status_string.restype = ctypes.c_char_p
        lib.adaspark_pairs_workspace_bytes.argtypes = [sp, ctypes.c_int64, ctypes.POINTER(ctypes.c_size_t)]
        lib.adaspark_cube_pool.argtypes = [sp, vp, vp, vp]
        lib.adaspark_cube_select.argtypes = [sp, vp, vp, ctypes.c_float, ctypes.c_int, vp, vp, vp, vp,
                                             ctypes.c_int64, vp, ctypes.c_size_t, vp]
        lib.adaspark_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        lib.adaspark_probe_mfma.argtypes = [vp, ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_double), vp]
        lib.adaspark_select_status_offset.argtypes = [sp, ctypes.POINTER(ctypes.c_size_t)]
        lib.adaspark_sparse_attn_csr.argtypes = [sp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, vp, ctypes.c_size_t, vp]
        lib.adaspark_cube_select_noalloc.argtypes = [sp, vp, vp, ctypes.c_float, ctypes.c_int, vp, vp, vp, vp,
                                                     ctypes.c_int64, vp]
        lib.adaspark_cube_select_topk.argtypes = [sp, vp, vp, ctypes.c_int32, ctypes.c_int, vp, vp, vp, vp,
                                                  ctypes.c_int64, vp, ctypes.c_size_t, vp]
        lib.adaspark_cube_select_shared.argtypes = [sp, vp, vp, ctypes.c_float, ctypes.c_int, vp, vp, vp, ctypes.c_size_t,
                                                    vp]
        lib.adaspark_sparse_attn.argtypes = [sp, vp, vp, vp, vp, ctypes.c_int, vp, vp, vp, ctypes.c_size_t, vp]
        lib.adaspark_dense_attn.argtypes = [sp, vp, vp, vp, ctypes.c_int, vp, vp, vp, ctypes.c_size_t, vp]
        lib.adaspark_kv_pack.argtypes = [sp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.adaspark_sparse_attn_packed.argtypes = [sp, vp, vp, ctypes.c_size_t, vp, ctypes.c_int, vp, vp, vp]
        lib.adaspark_sparse_attn_packed_with.argtypes = [sp, vp, vp, ctypes.c_size_t, vp, ctypes.c_int, ctypes.c_int,
                                                         vp, vp, vp]
        lib.adaspark_dense_attn_packed.argtypes = [sp, vp, vp, ctypes.c_size_t, ctypes.c_int, vp, vp, vp]
        lib.adaspark_sparse_attn_bwd.argtypes = [sp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, vp, vp, vp, vp,
                                                 ctypes.c_size_t, vp]
        dp = ctypes.POINTER(_CFfnDims)
        lib.adaspark_ffn_workspace_bytes.argtypes = [sp, dp, ctypes.POINTER(ctypes.c_size_t)]
        lib.adaspark_ffn_select.argtypes = [sp, dp, vp, ctypes.c_float, ctypes.c_float, vp, vp, vp, vp]
        lib.adaspark_ffn_sparse.argtypes = [sp, dp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        for name in EXPORTS:
            if name != "adaspark_status_string":
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().adaspark_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != 0:
        raise AdasparkError(status, what)


def _dev(t: torch.Tensor, dtype, numel: int, name: str) -> int:
    if not isinstance(t, torch.Tensor) or t.device.type != "cuda":
        raise ValueError(f"{name} must be a GPU tensor (this package has no CPU path)")
    if t.dtype != dtype or not t.is_contiguous() or t.numel() != numel:
        raise ValueError(f"{name}: expected contiguous {dtype} with {numel} elements, got {t.dtype} {tuple(t.shape)}")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def num_cubes(shape: Shape) -> int:
    n = ctypes.c_int32(0)
    cs = shape._c()
    _check(load().adaspark_num_cubes(ctypes.byref(cs), ctypes.byref(n)), "adaspark_num_cubes")
    return n.value


def workspace_bytes(shape: Shape, which_call: int) -> int:
    b = ctypes.c_size_t(0)
    cs = shape._c()
    _check(load().adaspark_workspace_bytes(ctypes.byref(cs), which_call, ctypes.byref(b)), "adaspark_workspace_bytes")
    return b.value


def pairs_workspace_bytes(shape: Shape, max_selected: int) -> int:
    """Attention workspace size that lets the key-stationary kernel run for up to ``max_selected`` selected
    (row, cube) pairs in total."""
    b = ctypes.c_size_t(0)
    cs = shape._c()
    _check(load().adaspark_pairs_workspace_bytes(ctypes.byref(cs), int(max_selected), ctypes.byref(b)),
           "adaspark_pairs_workspace_bytes")
    return b.value


def alloc_workspace(shape: Shape, which_call: int, device="cuda", pairs_capacity: int | None = None) -> torch.Tensor:
    """``pairs_capacity``: size an attention workspace for that many selected (row, cube) pairs as well."""
    n = workspace_bytes(shape, which_call)
    if pairs_capacity is not None:
        n = max(n, pairs_workspace_bytes(shape, pairs_capacity))
    return torch.empty(max(n, 16), dtype=torch.uint8, device=device)


def cube_pool(shape: Shape, K: torch.Tensor, kbar: torch.Tensor | None = None) -> torch.Tensor:
    """Eq. 1 mean keys: K bf16 [S,Hkv,D] -> kbar fp32 [N,Hkv,D]."""
    N = num_cubes(shape)
    if kbar is None:
        kbar = torch.empty((N, shape.kv_heads, shape.head_dim), dtype=torch.float32, device=K.device)
    cs = shape._c()
    _check(load().adaspark_cube_pool(
        ctypes.byref(cs), _dev(K, torch.bfloat16, shape.tokens * shape.kv_heads * shape.head_dim, "K"),
        _dev(kbar, torch.float32, N * shape.kv_heads * shape.head_dim, "kbar"), _stream()), "adaspark_cube_pool")
    return kbar


def cube_select(shape: Shape, Q: torch.Tensor, kbar: torch.Tensor, top_p: float, causal: bool = True,
                sel_mask=None, sel_count=None, csr_capacity: int | None = None, workspace=None):
    """Eqs. 1-2: -> (sel_mask int32-viewed-u32 [R, words], sel_count int32 [R], row_ptr|None, cube_idx|None)."""
    return _cube_select("adaspark_cube_select", ctypes.c_float(top_p), shape, Q, kbar, causal, sel_mask, sel_count,
                        csr_capacity, workspace)


def select_status(shape: Shape, workspace: torch.Tensor) -> int:
    """The device status word a selection call left in its workspace (0, or ECAPACITY if the compact list did not
    fit): a 4-byte copy to the host, which waits for the stream."""
    off = ctypes.c_size_t(0)
    cs = shape._c()
    _check(load().adaspark_select_status_offset(ctypes.byref(cs), ctypes.byref(off)), "adaspark_select_status_offset")
    return int(workspace[off.value: off.value + 4].view(torch.int32).item())


def sparse_attn_csr(shape: Shape, Q, K, V, row_ptr, cube_idx, causal: bool = True, O=None, lse=None, workspace=None,
                    return_lse: bool = False):
    """adaspark_sparse_attn_csr: Eq. 3 + own-cube rule over the cubes each row's compact list names."""
    R = shape.rows
    dev = Q.device
    if O is None:
        O = torch.empty((shape.tokens, shape.q_heads, shape.head_dim), dtype=torch.bfloat16, device=dev)
    if lse is None and return_lse:
        lse = torch.empty((R,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = alloc_workspace(shape, CALL_SPARSE_ATTN_CSR, dev)
    kvn = shape.tokens * shape.kv_heads * shape.head_dim
    if cube_idx.dtype != torch.int32 or not cube_idx.is_contiguous() or cube_idx.device.type != "cuda":
        raise ValueError("cube_idx must be a contiguous int32 GPU tensor")
    cs = shape._c()
    _check(load().adaspark_sparse_attn_csr(
        ctypes.byref(cs), _dev(Q, torch.bfloat16, R * shape.head_dim, "Q"), _dev(K, torch.bfloat16, kvn, "K"),
        _dev(V, torch.bfloat16, kvn, "V"), _dev(row_ptr, torch.int64, R + 1, "row_ptr"), cube_idx.data_ptr(),
        int(bool(causal)), _dev(O, torch.bfloat16, R * shape.head_dim, "O"),
        None if lse is None else _dev(lse, torch.float32, R, "lse"), workspace.data_ptr(), workspace.numel(),
        _stream()), "adaspark_sparse_attn_csr")
    return (O, lse) if return_lse else O


def cube_select_noalloc(shape: Shape, Q: torch.Tensor, kbar: torch.Tensor, top_p: float, sel_mask: torch.Tensor,
                        sel_count: torch.Tensor, row_ptr=None, cube_idx=None, causal: bool = True):
    """adaspark_cube_select_noalloc: the selection with the library's own scratch array instead of a workspace.
    Every output tensor is the caller's; nothing is allocated here or in the library."""
    N = num_cubes(shape)
    words = (N + 31) // 32
    R = shape.rows
    rp = ci = None
    cap = 0
    if row_ptr is not None:
        rp, ci, cap = _dev(row_ptr, torch.int64, R + 1, "row_ptr"), cube_idx.data_ptr(), cube_idx.numel()
    cs = shape._c()
    _check(load().adaspark_cube_select_noalloc(
        ctypes.byref(cs), _dev(Q, torch.bfloat16, R * shape.head_dim, "Q"),
        _dev(kbar, torch.float32, N * shape.kv_heads * shape.head_dim, "kbar"), ctypes.c_float(top_p),
        int(bool(causal)), _dev(sel_mask, torch.int32, R * words, "sel_mask"),
        _dev(sel_count, torch.int32, R, "sel_count"), rp, ci, cap, _stream()), "adaspark_cube_select_noalloc")
    return sel_mask, sel_count, row_ptr, cube_idx


def cube_select_topk(shape: Shape, Q: torch.Tensor, kbar: torch.Tensor, top_k: int, causal: bool = True,
                     sel_mask=None, sel_count=None, csr_capacity: int | None = None, workspace=None):
    """Fixed Top-K selection (the paper's ablation baseline); outputs as cube_select."""
    return _cube_select("adaspark_cube_select_topk", ctypes.c_int32(int(top_k)), shape, Q, kbar, causal, sel_mask,
                        sel_count, csr_capacity, workspace)


def _cube_select(fn_name, rule_arg, shape, Q, kbar, causal, sel_mask, sel_count, csr_capacity, workspace):
    N = num_cubes(shape)
    words = (N + 31) // 32
    R = shape.rows
    dev = Q.device
    if sel_mask is None:
        sel_mask = torch.empty((R, words), dtype=torch.int32, device=dev)
    if sel_count is None:
        sel_count = torch.empty((R,), dtype=torch.int32, device=dev)
    row_ptr = cube_idx = None
    rp = ci = None
    cap = 0
    if csr_capacity is not None:
        cap = int(csr_capacity)
        row_ptr = torch.empty((R + 1,), dtype=torch.int64, device=dev)
        cube_idx = torch.empty((max(cap, 4),), dtype=torch.int32, device=dev)
        rp, ci = row_ptr.data_ptr(), cube_idx.data_ptr()
    if workspace is None:
        workspace = alloc_workspace(shape, CALL_CUBE_SELECT, dev)
    cs = shape._c()
    _check(getattr(load(), fn_name)(
        ctypes.byref(cs), _dev(Q, torch.bfloat16, R * shape.head_dim, "Q"),
        _dev(kbar, torch.float32, N * shape.kv_heads * shape.head_dim, "kbar"),
        rule_arg, int(bool(causal)),
        _dev(sel_mask, torch.int32, R * words, "sel_mask"), _dev(sel_count, torch.int32, R, "sel_count"),
        rp, ci, cap, workspace.data_ptr(), workspace.numel(), _stream()), fn_name)
    return sel_mask, sel_count, row_ptr, cube_idx


def _attn(fn_name, shape, Q, K, V, sel_mask, causal, O, lse, workspace, want_lse):
    R = shape.rows
    dev = Q.device
    if O is None:
        O = torch.empty((shape.tokens, shape.q_heads, shape.head_dim), dtype=torch.bfloat16, device=dev)
    if lse is None and want_lse:
        lse = torch.empty((R,), dtype=torch.float32, device=dev)
    if workspace is None:
        workspace = alloc_workspace(shape, CALL_SPARSE_ATTN, dev)
    kvn = shape.tokens * shape.kv_heads * shape.head_dim
    cs = shape._c()
    args = [ctypes.byref(cs), _dev(Q, torch.bfloat16, R * shape.head_dim, "Q"), _dev(K, torch.bfloat16, kvn, "K"),
            _dev(V, torch.bfloat16, kvn, "V")]
    if fn_name == "adaspark_sparse_attn":
        words = (num_cubes(shape) + 31) // 32
        args.append(_dev(sel_mask, torch.int32, R * words, "sel_mask"))
    args += [int(bool(causal)), _dev(O, torch.bfloat16, R * shape.head_dim, "O"),
             None if lse is None else _dev(lse, torch.float32, R, "lse"),
             workspace.data_ptr(), workspace.numel(), _stream()]
    _check(getattr(load(), fn_name)(*args), fn_name)
    return (O, lse) if want_lse else O


def sparse_attn(shape: Shape, Q, K, V, sel_mask, causal: bool = True, O=None, lse=None, workspace=None,
                return_lse: bool = False):
    """Eq. 3 + own-cube rule over the cubes set in ``sel_mask`` -> O bf16 [S,Hq,D]."""
    return _attn("adaspark_sparse_attn", shape, Q, K, V, sel_mask, causal, O, lse, workspace, return_lse)


def dense_attn(shape: Shape, Q, K, V, causal: bool = True, O=None, lse=None, workspace=None,
               return_lse: bool = False):
    """Dense causal attention in cube-major order -> O bf16 [S,Hq,D]."""
    return _attn("adaspark_dense_attn", shape, Q, K, V, None, causal, O, lse, workspace, return_lse)


def kv_pack(shape: Shape, K, V, workspace=None) -> torch.Tensor:
    """Gather K,V into the cube-major tiled copy the attention kernels read; returns the workspace."""
    if workspace is None:
        workspace = alloc_workspace(shape, CALL_SPARSE_ATTN, K.device)
    kvn = shape.tokens * shape.kv_heads * shape.head_dim
    cs = shape._c()
    _check(load().adaspark_kv_pack(ctypes.byref(cs), _dev(K, torch.bfloat16, kvn, "K"), _dev(V, torch.bfloat16, kvn, "V"),
                                   workspace.data_ptr(), workspace.numel(), _stream()), "adaspark_kv_pack")
    return workspace


def _attn_packed(fn_name, shape, Q, packed, sel_mask, causal, O, lse, want_lse, kernel=None):
    R = shape.rows
    if O is None:
        O = torch.empty((shape.tokens, shape.q_heads, shape.head_dim), dtype=torch.bfloat16, device=Q.device)
    if lse is None and want_lse:
        lse = torch.empty((R,), dtype=torch.float32, device=Q.device)
    if packed.device.type != "cuda":
        raise ValueError("packed must be a GPU tensor")
    cs = shape._c()
    args = [ctypes.byref(cs), _dev(Q, torch.bfloat16, R * shape.head_dim, "Q"), packed.data_ptr(), packed.numel()]
    if fn_name.startswith("adaspark_sparse_attn_packed"):
        words = (num_cubes(shape) + 31) // 32
        args.append(_dev(sel_mask, torch.int32, R * words, "sel_mask"))
    args.append(int(bool(causal)))
    if kernel is not None:
        args.append(int(kernel))
    args += [_dev(O, torch.bfloat16, R * shape.head_dim, "O"),
             None if lse is None else _dev(lse, torch.float32, R, "lse"), _stream()]
    _check(getattr(load(), fn_name)(*args), fn_name)
    return (O, lse) if want_lse else O


def sparse_attn_packed(shape: Shape, Q, packed, sel_mask, causal: bool = True, O=None, lse=None,
                       return_lse: bool = False, kernel: int | None = None):
    """``kernel``: None/SPARSE_AUTO lets the library choose, SPARSE_COMPACT / SPARSE_MASKED / SPARSE_PAIRS force
    one (SPARSE_PAIRS needs a workspace from ``alloc_workspace(..., pairs_capacity=...)``)."""
    if kernel is None:
        return _attn_packed("adaspark_sparse_attn_packed", shape, Q, packed, sel_mask, causal, O, lse, return_lse)
    return _attn_packed("adaspark_sparse_attn_packed_with", shape, Q, packed, sel_mask, causal, O, lse, return_lse,
                        kernel)


def dense_attn_packed(shape: Shape, Q, packed, causal: bool = True, O=None, lse=None, return_lse: bool = False):
    return _attn_packed("adaspark_dense_attn_packed", shape, Q, packed, None, causal, O, lse, return_lse)


def ffn_workspace_bytes(shape: Shape, d_model: int, d_ff: int) -> int:
    n = ctypes.c_size_t(0)
    cs, cd = shape._c(), _CFfnDims(d_model, d_ff)
    _check(load().adaspark_ffn_workspace_bytes(ctypes.byref(cs), ctypes.byref(cd), ctypes.byref(n)),
           "adaspark_ffn_workspace_bytes")
    return int(n.value)


def ffn_select(shape: Shape, X: torch.Tensor, d_ff: int, top_p: float, eps: float = 1e-6):
    """Sec. 3.3, Eqs. 4-5: X bf16 [S, d_model] -> (keep uint8 [S], score fp32 [S], keep_count int32 [cubes])."""
    d_model = X.shape[-1]
    S, N = shape.tokens, num_cubes(shape)
    keep = torch.empty(S, dtype=torch.uint8, device=X.device)
    score = torch.empty(S, dtype=torch.float32, device=X.device)
    count = torch.empty(N, dtype=torch.int32, device=X.device)
    cs, cd = shape._c(), _CFfnDims(d_model, d_ff)
    _check(load().adaspark_ffn_select(
        ctypes.byref(cs), ctypes.byref(cd), _dev(X, torch.bfloat16, S * d_model, "X"), ctypes.c_float(top_p),
        ctypes.c_float(eps), _dev(keep, torch.uint8, S, "keep"), _dev(score, torch.float32, S, "score"),
        _dev(count, torch.int32, N, "keep_count"), _stream()), "adaspark_ffn_select")
    return keep, score, count


def ffn_sparse(shape: Shape, X, W_gate, W_up, W_down, keep=None, Y=None, workspace=None) -> torch.Tensor:
    """Sec. 3.3, Eqs. 6-7: the gated FFN on the activated tokens, mean compensation for the others.
    keep None: every token takes the layer (the dense layer)."""
    S, d_model, d_ff = shape.tokens, X.shape[-1], W_gate.shape[0]
    if Y is None:
        Y = torch.empty_like(X)
    if workspace is None:
        workspace = torch.empty(ffn_workspace_bytes(shape, d_model, d_ff), dtype=torch.uint8, device=X.device)
    cs, cd = shape._c(), _CFfnDims(d_model, d_ff)
    _check(load().adaspark_ffn_sparse(
        ctypes.byref(cs), ctypes.byref(cd), _dev(X, torch.bfloat16, S * d_model, "X"),
        _dev(W_gate, torch.bfloat16, d_ff * d_model, "W_gate"), _dev(W_up, torch.bfloat16, d_ff * d_model, "W_up"),
        _dev(W_down, torch.bfloat16, d_ff * d_model, "W_down"),
        None if keep is None else _dev(keep, torch.uint8, S, "keep"), _dev(Y, torch.bfloat16, S * d_model, "Y"),
        _dev(workspace, torch.uint8, workspace.numel(), "workspace"), workspace.numel(), _stream()),
        "adaspark_ffn_sparse")
    return Y


def sparse_attn_bwd(shape: Shape, Q, K, V, O, lse, dO, sel_mask=None, causal: bool = True, workspace=None,
                    dQ=None, dK=None, dV=None):
    """Backward of the attention entries with the selection held constant -> (dQ, dK, dV) bf16.
    sel_mask None: dense causal attention."""
    R, D = shape.rows, shape.head_dim
    kvn = shape.tokens * shape.kv_heads * D
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    if workspace is None:
        workspace = alloc_workspace(shape, CALL_ATTN_BWD, device=Q.device)
    words = (num_cubes(shape) + 31) // 32
    cs = shape._c()
    _check(load().adaspark_sparse_attn_bwd(
        ctypes.byref(cs), _dev(Q, torch.bfloat16, R * D, "Q"), _dev(K, torch.bfloat16, kvn, "K"),
        _dev(V, torch.bfloat16, kvn, "V"), _dev(O, torch.bfloat16, R * D, "O"), _dev(lse, torch.float32, R, "lse"),
        _dev(dO, torch.bfloat16, R * D, "dO"),
        None if sel_mask is None else _dev(sel_mask, torch.int32, R * words, "sel_mask"), int(bool(causal)),
        _dev(dQ, torch.bfloat16, R * D, "dQ"), _dev(dK, torch.bfloat16, kvn, "dK"), _dev(dV, torch.bfloat16, kvn, "dV"),
        _dev(workspace, torch.uint8, workspace.numel(), "workspace"), workspace.numel(), _stream()),
        "adaspark_sparse_attn_bwd")
    return dQ, dK, dV


def cube_select_shared(shape: Shape, Q: torch.Tensor, kbar: torch.Tensor, top_p: float, causal: bool = True):
    """Group-shared selection: one Top-p set per (token, KV head) from the group's mean query, copied to the rows
    of all its query heads -> (sel_mask int32-viewed-u32 [R, words], sel_count int32 [R])."""
    R, N = shape.rows, num_cubes(shape)
    words = (N + 31) // 32
    sel_mask = torch.empty((R, words), dtype=torch.int32, device=Q.device)
    sel_count = torch.empty((R,), dtype=torch.int32, device=Q.device)
    workspace = alloc_workspace(shape, CALL_CUBE_SELECT_SHARED, Q.device)
    cs = shape._c()
    _check(load().adaspark_cube_select_shared(
        ctypes.byref(cs), _dev(Q, torch.bfloat16, R * shape.head_dim, "Q"),
        _dev(kbar, torch.float32, N * shape.kv_heads * shape.head_dim, "kbar"), ctypes.c_float(top_p), int(bool(causal)),
        _dev(sel_mask, torch.int32, R * words, "sel_mask"), _dev(sel_count, torch.int32, R, "sel_count"),
        workspace.data_ptr(), workspace.numel(), _stream()), "adaspark_cube_select_shared")
    return sel_mask, sel_count


def probe_copy(dst: torch.Tensor, src: torch.Tensor) -> int:
    """adaspark_probe_copy: src -> dst (same size, GPU, no overlap); returns the bytes moved (read + written)."""
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != n or dst.device.type != "cuda" or src.device.type != "cuda":
        raise ValueError("probe_copy: two GPU tensors of the same size")
    _check(load().adaspark_probe_copy(dst.data_ptr(), src.data_ptr(), n, _stream()), "adaspark_probe_copy")
    return 2 * n


def probe_mfma(out: torch.Tensor, workgroups: int, trips: int) -> float:
    """adaspark_probe_mfma: enqueue the back-to-back MFMA probe; returns the floating-point operations it performs."""
    if out.numel() < workgroups:
        raise ValueError("probe_mfma: out needs one float per workgroup")
    flops = ctypes.c_double(0.0)
    _check(load().adaspark_probe_mfma(_dev(out, torch.float32, out.numel(), "out"), workgroups, trips,
                                      ctypes.byref(flops), _stream()), "adaspark_probe_mfma")
    return flops.value
