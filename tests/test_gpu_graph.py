"""The library's entries under HIP graph capture: they allocate nothing, clear their own counters with kernels and
launch only on the caller's stream, so a whole step can be recorded once and replayed.  A graph is replayed several
times with eager work, new inputs and synchronisations in between, and every replay is compared with what the same
entries give when launched eagerly on the same inputs (bit for bit: no result depends on the order of atomics).
"""
import pytest
import torch

from paper_2604_08077_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2604_08077_amd import binding

    binding.load()  # raises if the HIP library was not built: there is no fallback
    return binding


def inputs(w, variant):
    """Two input sets of the same workload: the seeded one, and the same with Q and V in reversed token order."""
    Q, K, V = synth.generate(w)
    if variant:
        Q = Q.flip(0).contiguous()
        V = V.flip(0).contiguous()
    return Q, K, V


@pytest.mark.parametrize("name,p", [("T_ragged", 0.9), ("T_text64", 0.6), ("C2", 0.5)])
def test_forward_step_replays(B, name, p):
    w = synth.TEST_WORKLOADS.get(name) or synth.WORKLOADS[name]
    sh = B.Shape.of(w)
    N, R = B.num_cubes(sh), sh.rows
    words = (N + 31) // 32
    dev = "cuda"
    Qg, Kg, Vg = (torch.empty_like(t, device=dev) for t in inputs(w, 0))
    kbar = torch.empty((N, w.Hkv, w.D), dtype=torch.float32, device=dev)
    mask = torch.empty((R, words), dtype=torch.int32, device=dev)
    count = torch.empty((R,), dtype=torch.int32, device=dev)
    O = torch.empty((w.S, w.Hq, w.D), dtype=torch.bfloat16, device=dev)
    lse = torch.empty((R,), dtype=torch.float32, device=dev)
    ws_sel = B.alloc_workspace(sh, B.CALL_CUBE_SELECT)
    cap = None
    try:  # room for the key-stationary kernel too, where the geometry is one it covers
        B.pairs_workspace_bytes(sh, R * N)
        cap = R * N
    except B.AdasparkError:
        pass
    ws_att = B.alloc_workspace(sh, B.CALL_SPARSE_ATTN, pairs_capacity=cap)

    def step():
        B.cube_pool(sh, Kg, kbar)
        B.cube_select(sh, Qg, kbar, p, sel_mask=mask, sel_count=count, workspace=ws_sel)
        B.kv_pack(sh, Kg, Vg, ws_att)
        B.sparse_attn_packed(sh, Qg, ws_att, mask, O=O, lse=lse)

    def load(variant):
        for dst, src in zip((Qg, Kg, Vg), inputs(w, variant)):
            dst.copy_(src)

    eager = []
    for variant in (0, 1):
        load(variant)
        step()
        torch.cuda.synchronize()
        eager.append((mask.clone(), count.clone(), O.clone(), lse.clone()))
    assert not torch.equal(eager[0][2], eager[1][2])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()  # every kernel has run once on this stream before the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    for rep, variant in enumerate((1, 0, 0, 1)):
        load(variant)
        for t in (kbar, mask, count, O, lse):  # eager work between replays; outputs start dirty
            t.fill_(1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want, what in zip((mask, count, O, lse), eager[variant], ("sel_mask", "sel_count", "O", "lse")):
            assert torch.equal(got, want), f"replay {rep} (inputs {variant}): {what} differs from the eager launch"
    print(f"[{name} p={p}] 4 replays of pool+select+pack+attention equal the eager results", flush=True)


def test_ffn_and_backward_replay(B):
    w = synth.TEST_WORKLOADS["T_ragged"]
    sh = B.Shape.of(w)
    d_model, d_ff, pf, p = 256, 384, 0.6, 0.9
    X, Wg, Wu, Wd = (t.cuda() for t in synth.generate_ffn(w, d_model, d_ff))
    Q, K, V = (t.cuda() for t in synth.generate(w))
    g = torch.Generator(device="cpu")
    g.manual_seed(synth.BASE_SEED + 31 * w.config_id)
    dO = torch.randn((w.S, w.Hq, w.D), generator=g, dtype=torch.float32).to(torch.bfloat16).cuda()
    kbar = B.cube_pool(sh, K)
    mask, _, _, _ = B.cube_select(sh, Q, kbar, p)
    O, lse = B.sparse_attn(sh, Q, K, V, mask, return_lse=True)
    keep, _, _ = B.ffn_select(sh, X, d_ff, pf)
    Y = torch.empty_like(X)
    dQ, dK, dV = torch.empty_like(Q), torch.empty_like(K), torch.empty_like(V)
    ws_ffn = torch.empty(B.ffn_workspace_bytes(sh, d_model, d_ff), dtype=torch.uint8, device="cuda")
    ws_bwd = B.alloc_workspace(sh, B.CALL_ATTN_BWD)

    def step():
        B.ffn_sparse(sh, X, Wg, Wu, Wd, keep=keep, Y=Y, workspace=ws_ffn)
        B.sparse_attn_bwd(sh, Q, K, V, O, lse, dO, sel_mask=mask, dQ=dQ, dK=dK, dV=dV, workspace=ws_bwd)

    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in (Y, dQ, dK, dV)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in (Y, dQ, dK, dV):
            t.fill_(1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, want, what in zip((Y, dQ, dK, dV), eager, ("Y", "dQ", "dK", "dV")):
            assert torch.equal(got, want), f"replay {rep}: {what} differs from the eager launch"
    print("[T_ragged] 3 replays of the sparse FFN + attention backward equal the eager results", flush=True)
