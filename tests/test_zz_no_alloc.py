"""The allocation-free selection entry (adaspark_cube_select_noalloc) against adaspark_cube_select, through the C ABI:
same masks, counts and compact lists bit for bit, on two calls in a row, the second on a smaller input -- both use the
one scratch array the library keeps per GPU, which still holds what the first call left."""
import numpy as np
import pytest
import torch

from paper_2604_08077_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2604_08077_amd import binding

    binding.load()
    return binding


def run_both(B, w, p):
    sh = B.Shape.of(w)
    Q, K, _ = synth.generate(w)
    Qg, Kg = Q.cuda(), K.cuda()
    kbar = B.cube_pool(sh, Kg)
    p32 = float(np.float32(p))
    mask, count, row_ptr, cube_idx = B.cube_select(sh, Qg, kbar, p32, csr_capacity=0)
    torch.cuda.synchronize()
    cap = int(row_ptr[-1].item())
    mask, count, row_ptr, cube_idx = B.cube_select(sh, Qg, kbar, p32, csr_capacity=cap)
    # outputs of the allocation-free call: allocated here, before it, and poisoned
    m2 = torch.full_like(mask, -1)
    c2 = torch.full_like(count, -1)
    rp2 = torch.full_like(row_ptr, -1)
    ci2 = torch.full_like(cube_idx, -1)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    B.cube_select_noalloc(sh, Qg, kbar, p32, m2, c2, rp2, ci2)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    print(f"[{w.name}] p={p} rows={sh.rows} selected pairs={cap}", flush=True)
    assert differences({"sel_mask": (m2, mask), "sel_count": (c2, count), "row_ptr": (rp2, row_ptr),
                        "cube_idx": (ci2[:cap], cube_idx[:cap])}) == {}
    # without the compact list
    m3, c3 = torch.full_like(mask, -1), torch.full_like(count, -1)
    B.cube_select_noalloc(sh, Qg, kbar, p32, m3, c3)
    torch.cuda.synchronize()
    assert differences({"sel_mask, no list": (m3, mask), "sel_count, no list": (c3, count)}) == {}


def differences(pairs):
    """{name: (number of differing elements, first differing flat index, the two values there)} for the pairs that
    differ: what a failure report needs to name the output and the place."""
    out = {}
    for name, (got, want) in pairs.items():
        if not torch.equal(got, want):
            ne = (got != want).reshape(-1)
            first = int(torch.nonzero(ne)[0].item())
            out[name] = (int(ne.sum().item()), first, int(got.reshape(-1)[first].item()), int(want.reshape(-1)[first].item()))
    return out


def test_two_calls_in_a_row_the_second_smaller(B):
    run_both(B, synth.WORKLOADS["C2"], 0.9)            # 16,384 tokens, 64 cubes, 28/4 heads
    run_both(B, synth.TEST_WORKLOADS["T_ragged"], 0.7)  # 1,080 tokens, ragged, 6/2 heads
    run_both(B, synth.TEST_WORKLOADS["T_cubes280"], 0.7)  # more than 256 cubes: the wide kernel


def test_shape_beyond_the_scratch_array_is_refused(B):
    """2,048 cubes x 8 KV heads of 128 need more than the array holds: refused before anything runs."""
    sh = B.Shape(2048, 16, 16, 1, 16, 16, 8, 8, 128)
    assert B.workspace_bytes(sh, B.CALL_CUBE_SELECT) > B.NOALLOC_SCRATCH_BYTES
    z = torch.zeros(16, dtype=torch.int32, device="cuda")
    import ctypes
    cs = sh._c()
    rc = B.load().adaspark_cube_select_noalloc(ctypes.byref(cs), z.data_ptr(), z.data_ptr(), ctypes.c_float(0.5), 1,
                                               z.data_ptr(), z.data_ptr(), None, None, 0, None)
    assert rc == -3
