"""CPU-only checks of the C-ABI boundary: the library loads, exports every
function the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

from paper_2604_08077_amd import binding, build, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(build.lib_path()):
        build.build()
    return binding.load()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "adaspark.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(adaspark_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_num_cubes_and_workspace_sizes(lib):
    expect = {"C1": 64, "C2": 64, "C3": 256, "C4": 1024, "C5": 150}
    for name, n in expect.items():
        sh = binding.Shape.of(synth.WORKLOADS[name])
        assert binding.num_cubes(sh) == n
        assert binding.workspace_bytes(sh, binding.CALL_CUBE_POOL) == 0
        assert binding.workspace_bytes(sh, binding.CALL_CUBE_SELECT) > 0
        ws = binding.workspace_bytes(sh, binding.CALL_SPARSE_ATTN)
        assert ws == binding.workspace_bytes(sh, binding.CALL_DENSE_ATTN)
        w = synth.WORKLOADS[name]
        assert ws >= 2 * w.S * w.Hkv * w.D * 2          # room for a packed copy of K and V


def test_status_strings(lib):
    assert binding.status_string(0) == "ok"
    for code in (-1, -2, -3, -4, -5):
        assert binding.status_string(code) not in ("ok", "unknown status")
    assert binding.status_string(-99) == "unknown status"


def _raw_shape(**kw):
    base = dict(frames=4, height=8, width=8, cube_t=2, cube_h=4, cube_w=4, q_heads=4, kv_heads=2, head_dim=64)
    base.update(kw)
    return binding.Shape(**base)


@pytest.mark.parametrize("kw,code", [
    (dict(frames=0), -1), (dict(cube_w=0), -1), (dict(q_heads=3), -1), (dict(kv_heads=0), -1),
    (dict(head_dim=96), -2), (dict(frames=4096, height=64, width=64, cube_t=1, cube_h=1, cube_w=1), -2),
    (dict(text_tokens=-1), -1), (dict(prefix_tokens=-1), -1), (dict(prefix_tokens=32 * 2048), -2), (dict(text_tokens=32 * 2048), -2),
])
def test_bad_shapes_are_rejected(lib, kw, code):
    with pytest.raises(binding.AdasparkError) as e:
        binding.num_cubes(_raw_shape(**kw))
    assert e.value.status == code


def test_bad_pointers_and_arguments_are_rejected_before_launch(lib):
    cs = _raw_shape()._c()
    ok_ptr = ctypes.c_void_p(4096)      # never dereferenced: validation fails first
    assert lib.adaspark_cube_pool(ctypes.byref(cs), None, ok_ptr, None) == -1
    assert lib.adaspark_cube_pool(ctypes.byref(cs), ctypes.c_void_p(4097), ok_ptr, None) == -1
    args = [ctypes.byref(cs), ok_ptr, ok_ptr, ctypes.c_float(1.5), 1, ok_ptr, ok_ptr, None, None, 0, ok_ptr, 1 << 30, None]
    assert lib.adaspark_cube_select(*args) == -1                       # top_p outside [0,1]
    args[3] = ctypes.c_float(float("nan"))
    assert lib.adaspark_cube_select(*args) == -1
    args[3] = ctypes.c_float(0.9)
    # non-causal mode runs on the masked-walk kernel only: the other two sparse kernels refuse it
    nc = lambda kernel: lib.adaspark_sparse_attn_packed_with(
        ctypes.byref(cs), ok_ptr, ok_ptr, 1 << 30, ok_ptr, 0, kernel, ok_ptr, None, None)
    assert nc(binding.SPARSE_COMPACT) == -2 and nc(binding.SPARSE_PAIRS) == -2
    args[11] = 8
    assert lib.adaspark_cube_select(*args) == -3                       # workspace too small
    args[11] = 1 << 30
    args[7] = ok_ptr
    assert lib.adaspark_cube_select(*args) == -1                       # row_ptr without cube_idx
    assert lib.adaspark_sparse_attn(ctypes.byref(cs), ok_ptr, ok_ptr, ok_ptr, None, 1, ok_ptr, None, ok_ptr, 1 << 30, None) == -1
    assert lib.adaspark_dense_attn(ctypes.byref(cs), ok_ptr, ok_ptr, ok_ptr, 1, ok_ptr, None, None, 0, None) == -3
    assert lib.adaspark_dense_attn(None, ok_ptr, ok_ptr, ok_ptr, 1, ok_ptr, None, ok_ptr, 1 << 30, None) == -1
    # packed sparse entry with an explicit kernel: unknown choice, workspace too small, missing selection
    pw = lambda kernel, nbytes, mask: lib.adaspark_sparse_attn_packed_with(
        ctypes.byref(cs), ok_ptr, ok_ptr, nbytes, mask, 1, kernel, ok_ptr, None, None)
    assert pw(7, 1 << 30, ok_ptr) == -1
    assert pw(-1, 1 << 30, ok_ptr) == -1
    assert pw(binding.SPARSE_COMPACT, 8, ok_ptr) == -3
    assert pw(binding.SPARSE_MASKED, 1 << 30, None) == -1
    # the key-stationary kernel needs scratch memory beyond the minimum workspace
    need = ctypes.c_size_t(0)
    assert lib.adaspark_workspace_bytes(ctypes.byref(cs), binding.CALL_SPARSE_ATTN, ctypes.byref(need)) == 0
    assert pw(binding.SPARSE_PAIRS, need.value, ok_ptr) == -3
    big = ctypes.c_size_t(0)
    assert lib.adaspark_pairs_workspace_bytes(ctypes.byref(cs), 1000, ctypes.byref(big)) == 0
    assert big.value > need.value + 1000 * (2 * cs.head_dim + 24)
    assert lib.adaspark_pairs_workspace_bytes(ctypes.byref(cs), -1, ctypes.byref(big)) == -1
    assert lib.adaspark_pairs_workspace_bytes(ctypes.byref(cs), 1, None) == -1
    huge = binding.Shape(4, 32, 32, 4, 32, 32, 4, 4, 64)._c()      # a cube of 4096 tokens does not fit on chip
    assert lib.adaspark_pairs_workspace_bytes(ctypes.byref(huge), 1, ctypes.byref(big)) == -2


def test_backward_arguments_are_validated_before_launch(lib):
    cs = _raw_shape()._c()
    ok_ptr = ctypes.c_void_p(4096)      # never dereferenced: validation fails first
    need = ctypes.c_size_t(0)
    assert lib.adaspark_workspace_bytes(ctypes.byref(cs), binding.CALL_ATTN_BWD, ctypes.byref(need)) == 0
    fwd = ctypes.c_size_t(0)
    assert lib.adaspark_workspace_bytes(ctypes.byref(cs), binding.CALL_SPARSE_ATTN, ctypes.byref(fwd)) == 0
    rows, D = 4 * 8 * 8 * 4, 64
    assert need.value >= 2 * fwd.value + 4 * rows * D * 2 + 2 * rows * 4      # two K/V packs, four row packs, two vectors
    run = lambda q=ok_ptr, mask=ok_ptr, causal=1, ws=ok_ptr, nbytes=1 << 30, dq=ok_ptr: lib.adaspark_sparse_attn_bwd(
        ctypes.byref(cs), q, ok_ptr, ok_ptr, ok_ptr, ok_ptr, ok_ptr, mask, causal, dq, ok_ptr, ok_ptr, ws, nbytes, None)
    assert run(q=None) == -1 and run(dq=ctypes.c_void_p(4097)) == -1 and run(mask=ctypes.c_void_p(4100)) == -1
    assert run(causal=0) == -2
    assert run(ws=None) == -3 and run(nbytes=need.value - 1) == -3


def test_ffn_arguments_are_validated_before_launch(lib):
    cs = _raw_shape()._c()
    ok_ptr = ctypes.c_void_p(4096)      # never dereferenced: validation fails first
    dims = lambda m, f: ctypes.byref(binding._CFfnDims(m, f))
    n = ctypes.c_size_t(0)
    assert lib.adaspark_ffn_workspace_bytes(ctypes.byref(cs), dims(256, 384), ctypes.byref(n)) == 0
    tokens, rows = 4 * 8 * 8, 256
    assert n.value >= rows * 384 * 2 + rows * 256 * 4 + 2 * tokens * 4     # hidden activations, FFN values, tables
    assert lib.adaspark_ffn_workspace_bytes(ctypes.byref(cs), dims(256, 384), None) == -1
    assert lib.adaspark_ffn_workspace_bytes(ctypes.byref(cs), None, ctypes.byref(n)) == -1
    for m, f, code in ((0, 384, -1), (256, -128, -1), (200, 384, -2), (256, 100, -2), (32768, 384, -2), (256, 1 << 17, -2)):
        assert lib.adaspark_ffn_workspace_bytes(ctypes.byref(cs), dims(m, f), ctypes.byref(n)) == code
    big_cube = binding.Shape(8, 32, 32, 8, 32, 32, 4, 4, 64)._c()           # a cube of 8192 tokens
    assert lib.adaspark_ffn_workspace_bytes(ctypes.byref(big_cube), dims(256, 384), ctypes.byref(n)) == -2
    long_video = binding.Shape(4096, 16, 16, 4, 8, 8, 4, 4, 64)._c()        # tokens * d_model does not fit 2^30
    assert lib.adaspark_ffn_workspace_bytes(ctypes.byref(long_video), dims(4096, 384), ctypes.byref(n)) == -2
    sel = lambda p, eps, x=ok_ptr, keep=ok_ptr: lib.adaspark_ffn_select(
        ctypes.byref(cs), dims(256, 384), x, ctypes.c_float(p), ctypes.c_float(eps), keep, None, None, None)
    assert sel(1.5, 1e-6) == -1 and sel(float("nan"), 1e-6) == -1 and sel(0.7, -1.0) == -1
    assert sel(0.7, 1e-6, x=None) == -1 and sel(0.7, 1e-6, keep=ctypes.c_void_p(4097)) == -1
    xbytes = tokens * 256 * 2
    run = lambda ws, nbytes, x=ok_ptr, y=ctypes.c_void_p(4096 + xbytes): lib.adaspark_ffn_sparse(
        ctypes.byref(cs), dims(256, 384), x, ok_ptr, ok_ptr, ok_ptr, None, y, ws, nbytes, None)
    assert run(None, 1 << 30) == -3 and run(ok_ptr, 64) == -3                # Y right behind X: no overlap
    assert run(ok_ptr, 1 << 30, y=ok_ptr) == -1                              # Y aliases X
    assert run(ok_ptr, 1 << 30, y=ctypes.c_void_p(4096 + xbytes - 16)) == -1  # Y starts inside X
    assert run(ok_ptr, 1 << 30, x=ctypes.c_void_p(4096 + xbytes), y=ctypes.c_void_p(4096 + 512)) == -1  # X starts inside Y
    assert run(ok_ptr, 1 << 30, x=None) == -1


def test_binding_refuses_cpu_tensors(lib):
    import torch
    w = synth.TEST_WORKLOADS["T_tiny"]
    _, K, _ = synth.generate(w)
    with pytest.raises(ValueError):
        binding.cube_pool(binding.Shape.of(w), K)


def test_shared_selection_arguments_are_validated(lib):
    cs = _raw_shape()._c()
    ok_ptr = ctypes.c_void_p(4096)      # never dereferenced: validation fails first
    need, plain = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert lib.adaspark_workspace_bytes(ctypes.byref(cs), binding.CALL_CUBE_SELECT_SHARED, ctypes.byref(need)) == 0
    assert lib.adaspark_workspace_bytes(ctypes.byref(cs), binding.CALL_CUBE_SELECT, ctypes.byref(plain)) == 0
    tokens, kv, D = 4 * 8 * 8, 2, 64
    assert need.value >= tokens * kv * D * 2 + tokens * kv * 8          # the mean queries and their selection
    run = lambda p=0.9, causal=1, ws=ok_ptr, nbytes=1 << 30, q=ok_ptr: lib.adaspark_cube_select_shared(
        ctypes.byref(cs), q, ok_ptr, ctypes.c_float(p), causal, ok_ptr, ok_ptr, ws, nbytes, None)
    assert run(p=1.5) == -1 and run(p=float("nan")) == -1 and run(q=None) == -1
    assert run(ws=None) == -3 and run(nbytes=need.value - 1) == -3


def test_allocation_free_selection_refuses_what_its_array_cannot_hold(lib):
    """adaspark_cube_select_noalloc keeps its workspace in an array of the library (ADASPARK_NOALLOC_SCRATCH_BYTES):
    a shape that needs more is refused before anything is asked of the runtime, and so are a bad top_p or shape."""
    ok_ptr = ctypes.c_void_p(4096)
    call = lambda cs, p: lib.adaspark_cube_select_noalloc(ctypes.byref(cs), ok_ptr, ok_ptr, ctypes.c_float(p), 1,
                                                          ok_ptr, ok_ptr, None, None, 0, None)
    big = binding.Shape(2048, 16, 16, 1, 16, 16, 8, 8, 128)            # 2,048 cubes, 8 KV heads of 128
    assert binding.workspace_bytes(big, binding.CALL_CUBE_SELECT) > binding.NOALLOC_SCRATCH_BYTES
    assert call(big._c(), 0.9) == -3
    for name in ("C1", "C2", "C3", "C4", "C5"):                        # every benchmark configuration fits
        assert binding.workspace_bytes(binding.Shape.of(synth.WORKLOADS[name]), binding.CALL_CUBE_SELECT) \
            <= binding.NOALLOC_SCRATCH_BYTES
    assert call(_raw_shape()._c(), 1.5) == -1
    assert call(_raw_shape(head_dim=96)._c(), 0.5) == -2
    header = open(os.path.join(ROOT, "include", "adaspark.h")).read()
    assert "#define ADASPARK_NOALLOC_SCRATCH_BYTES (4u << 20)" in header and binding.NOALLOC_SCRATCH_BYTES == 4 << 20


def test_compact_list_entries_validate_before_launch(lib):
    cs = _raw_shape()._c()
    ok_ptr = ctypes.c_void_p(4096)
    off = ctypes.c_size_t(0)
    assert lib.adaspark_select_status_offset(ctypes.byref(cs), ctypes.byref(off)) == 0
    need = ctypes.c_size_t(0)
    assert lib.adaspark_workspace_bytes(ctypes.byref(cs), binding.CALL_CUBE_SELECT, ctypes.byref(need)) == 0
    assert off.value % 256 == 0 and off.value + 4 <= need.value
    assert lib.adaspark_select_status_offset(ctypes.byref(cs), None) == -1
    csr = lambda rp, ci, ws, n: lib.adaspark_sparse_attn_csr(ctypes.byref(cs), ok_ptr, ok_ptr, ok_ptr, rp, ci, 1, ok_ptr,
                                                             None, ws, n, None)
    assert csr(None, ok_ptr, ok_ptr, 1 << 30) == -1
    assert csr(ok_ptr, None, ok_ptr, 1 << 30) == -1
    assert csr(ok_ptr, ok_ptr, None, 0) == -3
    plain, with_mask = ctypes.c_size_t(0), ctypes.c_size_t(0)
    assert lib.adaspark_workspace_bytes(ctypes.byref(cs), binding.CALL_SPARSE_ATTN, ctypes.byref(plain)) == 0
    assert lib.adaspark_workspace_bytes(ctypes.byref(cs), binding.CALL_SPARSE_ATTN_CSR, ctypes.byref(with_mask)) == 0
    rows, words = 4 * 8 * 8 * 4, 1
    assert with_mask.value >= plain.value + rows * words * 4
    assert csr(ok_ptr, ok_ptr, ok_ptr, plain.value) == -3           # room for the K/V copy but not for the mask rows
