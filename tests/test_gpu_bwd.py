"""GPU parity of the attention backward pass (selection held constant): the HIP library through its C ABI against
the fp64 oracle on the same seeded bf16 inputs.

The GPU takes O and the log-sum-exp from its own forward (as a training step does), rebuilds the probabilities in
fp32, rounds P and dS to bf16 for the MFMA products, sums in fp32 and rounds the gradients to bf16.  A gradient
element is therefore a sum of terms each off by up to 2^-9 of itself, independently (standard deviation
2^-9/sqrt(3) of the root-sum-square T of its terms, which the oracle reports), plus the output rounding:
    |g_gpu - g_oracle| <= 2^-8 |g_oracle| + 2^-7 T + 1e-4          (2^-7 T is about seven standard deviations),
and the mean error must stay below a fifth of the mean bound.  Terms may cancel (rows that attend few keys with
large scores), so T, not |g|, is the unit.  delta = dO.O is a function of the O the caller hands over: the oracle is
given the same bf16 O (the oracle's own pins use the exact one).
"""
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

    binding.load()  # raises if the HIP library was not built: there is no fallback
    return binding


def oshape(o, w):
    return o.Shape(w.T, w.H, w.W, w.ct, w.ch, w.cw, w.Hq, w.Hkv, w.D, w.text, w.lead)


def f64(t):
    return t.to(torch.float64).numpy()


def check_grad(name, got, want, terms):
    got, want, terms = (x.reshape(-1, x.shape[-1]) for x in (got, want, terms))
    err = np.abs(got - want)
    bound = 2.0 ** -8 * np.abs(want) + 2.0 ** -7 * terms + 1e-4
    print(f"[{name}] elements={err.size} max-abs={err.max():.3e} mean-abs={err.mean():.3e} "
          f"worst err/bound={np.max(err / bound):.3f} mean err/mean bound={err.mean() / bound.mean():.3f}", flush=True)
    assert np.isfinite(got).all()
    assert (err <= bound).all()
    assert err.mean() <= 0.2 * bound.mean()


def workload(name):
    return synth.TEST_WORKLOADS.get(name) or synth.SAMPLED_WORKLOADS.get(name) or synth.WORKLOADS[name]


def run_case(B, oracle, name, p, dense=False):
    w = workload(name)
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    Q, K, V = synth.generate(w)
    g = torch.Generator(device="cpu")
    g.manual_seed(synth.BASE_SEED + 31 * w.config_id)
    dO = torch.randn((w.S, w.Hq, w.D), generator=g, dtype=torch.float32).to(torch.bfloat16)
    kbar = oracle.cube_pool(osh, K)
    mask = oracle.cube_select(osh, Q, kbar, 1.0 if dense else p)[0]
    Qg, Kg, Vg, dOg = Q.cuda(), K.cuda(), V.cuda(), dO.cuda()
    mg = torch.from_numpy(mask.view(np.int32)).cuda()
    print(f"[{name}] forward p={p} dense={dense}", flush=True)
    if dense:
        O, lse = B.dense_attn(sh, Qg, Kg, Vg, return_lse=True)
    else:
        O, lse = B.sparse_attn(sh, Qg, Kg, Vg, mg, return_lse=True)
    torch.cuda.synchronize()
    print(f"[{name}] backward", flush=True)
    dQ, dK, dV = B.sparse_attn_bwd(sh, Qg, Kg, Vg, O, lse, dOg, sel_mask=None if dense else mg)
    torch.cuda.synchronize()
    T = {}
    rq, rk, rv, _ = oracle.bwd.sparse_attn_bwd(osh, f64(Q), f64(K), f64(V), mask, f64(dO).reshape(-1, w.D),
                                               O=f64(O.cpu()).reshape(-1, w.D), scales=T)
    check_grad(f"{name} dV", f64(dV.cpu()), rv, T["dV"])
    check_grad(f"{name} dQ", f64(dQ.cpu()), rq, T["dQ"])
    check_grad(f"{name} dK", f64(dK.cpu()), rk, T["dK"])


@pytest.mark.parametrize("name,p", [("T_tiny", 0.8), ("T_mha64", 0.7), ("T_ragged", 0.9), ("T_text64", 0.8),
                                    ("T_lead64", 0.8), ("T_manycubes", 0.6), ("T_lead128", 0.9), ("C1", 0.9),
                                    ("M_bwd256", 0.8), ("T_cube2048", 0.9)])
def test_backward_matches_oracle(B, oracle, name, p):
    run_case(B, oracle, name, p)


@pytest.mark.parametrize("name,p", [("T_tiny", 0.8), ("T_ragged", 0.9), ("T_lead64", 0.8), ("M_bwd256", 0.8)])
def test_backward_matches_the_exact_gradient(B, oracle, name, p):
    """Against the oracle's own gradient: delta = dO.o from the exact fp64 forward, not from the bf16 O the GPU
    backward is handed.  What the forward's rounding of O does to the gradients enters through delta alone (dS_j =
    p_j (dO.v_j - delta)), so the bound of the other tests grows by the oracle's `dQ_delta` / `dK_delta`: the
    element's sensitivity to delta times the row's delta_error_bound (dV does not depend on delta).  The forward's
    O itself must be within that model too: |dO.O_gpu - dO.o| <= delta_error_bound, row by row."""
    w = workload(name)
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    Q, K, V = synth.generate(w)
    g = torch.Generator(device="cpu")
    g.manual_seed(synth.BASE_SEED + 31 * w.config_id)
    dO = torch.randn((w.S, w.Hq, w.D), generator=g, dtype=torch.float32).to(torch.bfloat16)
    mask = oracle.cube_select(osh, Q, oracle.cube_pool(osh, K), p)[0]
    Qg, Kg, Vg, dOg = Q.cuda(), K.cuda(), V.cuda(), dO.cuda()
    mg = torch.from_numpy(mask.view(np.int32)).cuda()
    print(f"[{name}] forward + backward, exact-delta comparison", flush=True)
    O, lse = B.sparse_attn(sh, Qg, Kg, Vg, mg, return_lse=True)
    dQ, dK, dV = B.sparse_attn_bwd(sh, Qg, Kg, Vg, O, lse, dOg, sel_mask=mg)
    torch.cuda.synchronize()
    T = {}
    q, k, v, do = f64(Q), f64(K), f64(V), f64(dO).reshape(-1, w.D)
    rq, rk, rv, delta = oracle.bwd.sparse_attn_bwd(osh, q, k, v, mask, do, O=None, scales=T)
    # the forward's effect on delta, row by row, against the model the extra tolerance is built from
    tables = oracle.bwd.cube_tables(osh)
    d_gpu = (do * f64(O.cpu()).reshape(-1, w.D)).sum(axis=1)
    worst = 0.0
    for r in synth.sample_rows(w, 200):
        att, _, _, _, _, _, pr = oracle.bwd.row_backward(osh, q, k, v, mask[r], r, do[r], None, tables)
        n, a = divmod(int(r), w.Hq)
        gk = a // (w.Hq // w.Hkv)
        absdot = (np.abs(k[att, gk]) @ np.abs(q[n, a])).max() / np.sqrt(w.D)
        worst = max(worst, abs(d_gpu[r] - delta[r]) / oracle.bwd.delta_error_bound(do[r], pr @ v[att, gk], pr, v[att, gk], absdot))
    print(f"[{name}] |delta_gpu - delta_exact| / bound, worst of the sampled rows: {worst:.3f}", flush=True)
    assert worst <= 1.0
    for nm, got, want in (("dV", dV, rv), ("dQ", dQ, rq), ("dK", dK, rk)):
        got, want_, terms = (x.reshape(-1, w.D) for x in (f64(got.cpu()), want, T[nm]))
        extra = T[nm + "_delta"].reshape(-1, w.D) if nm != "dV" else 0.0
        err = np.abs(got - want_)
        bound = 2.0 ** -8 * np.abs(want_) + 2.0 ** -7 * terms + 1e-4 + extra
        print(f"[{name} {nm} vs exact] max-abs={err.max():.3e} worst err/bound={np.max(err / bound):.3f} "
              f"share of the bound that is the delta term: {np.mean(extra / bound):.2f}", flush=True)
        assert (err <= bound).all()


@pytest.mark.parametrize("name", ["T_ragged", "T_mha64"])
def test_dense_backward_matches_oracle(B, oracle, name):
    run_case(B, oracle, name, 1.0, dense=True)


def test_backward_with_nothing_selected(B, oracle):
    """p = 0: every row attends the causal part of its own cube only (and earlier text cubes, if any)."""
    run_case(B, oracle, "T_ragged", 0.0)
    run_case(B, oracle, "T_lead64", 0.0)


def test_backward_full_size_sampled(B, oracle):
    """65,536 tokens, p = 0.9, the launch configuration the benchmark times.  dQ: sampled rows recomputed by the
    oracle.  dK, dV: the last eight tokens of the last cube of one KV head (few rows attend them: the oracle takes
    them all), and two identities that hold at any size because every row's probabilities sum to one and its dS to
    zero: sum over tokens of dV = sum over the group's rows of dO, sum over tokens of dK = 0."""
    w = synth.WORKLOADS["C3"]
    p = 0.9
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    Q, K, V = synth.generate(w)
    g = torch.Generator(device="cpu")
    g.manual_seed(synth.BASE_SEED + 31 * w.config_id)
    dO = torch.randn((w.S, w.Hq, w.D), generator=g, dtype=torch.float32).to(torch.bfloat16)
    Qg, Kg, Vg, dOg = Q.cuda(), K.cuda(), V.cuda(), dO.cuda()
    kbar = B.cube_pool(sh, Kg)
    mask_g, _, _, _ = B.cube_select(sh, Qg, kbar, p)
    print("[C3] forward", flush=True)
    O, lse = B.sparse_attn(sh, Qg, Kg, Vg, mask_g, return_lse=True)
    torch.cuda.synchronize()
    print("[C3] backward", flush=True)
    dQ, dK, dV = B.sparse_attn_bwd(sh, Qg, Kg, Vg, O, lse, dOg, sel_mask=mask_g)
    torch.cuda.synchronize()
    mask = mask_g.cpu().numpy().view(np.uint32)
    q, k, v, do = f64(Q), f64(K), f64(V), f64(dO).reshape(-1, w.D)
    o = f64(O.cpu()).reshape(-1, w.D)
    tables = oracle.bwd.cube_tables(osh)
    G, c = w.Hq // w.Hkv, 1.0 / np.sqrt(w.D)

    rows = synth.sample_rows(w, 24, seed=5)
    want, terms = [], []
    for r in rows:
        att, dq, _, _, _, ds, _ = oracle.bwd.row_backward(osh, q, k, v, mask[r], r, do[r], o[r], tables)
        want.append(dq)
        terms.append(c * np.sqrt((ds * ds) @ (k[att, (r % w.Hq) // G] ** 2)))
    got = f64(dQ.reshape(-1, w.D)[torch.as_tensor(rows).cuda()].cpu())
    check_grad("C3 dQ sampled rows", got, np.array(want), np.array(terms))

    # keys: the last eight tokens (in cube order) of the last cube, KV head 1; the rows that attend them are the
    # rows of those tokens themselves and of the later ones among them
    members = tables[2][-1]
    toks = members[-8:]
    gk = 1
    wk, wv = np.zeros((8, w.D)), np.zeros((8, w.D))
    tk, tv = np.zeros((8, w.D)), np.zeros((8, w.D))
    for x, n in enumerate(toks):
        for a in range(gk * G, (gk + 1) * G):
            r = n * w.Hq + a
            att, _, dk_t, dv_t, _, _, _ = oracle.bwd.row_backward(osh, q, k, v, mask[r], r, do[r], o[r], tables)
            for y in range(x + 1):                      # this row attends toks[0..x]
                pos = int(np.nonzero(att == toks[y])[0][0])
                wk[y] += dk_t[pos]
                wv[y] += dv_t[pos]
                tk[y] += dk_t[pos] ** 2
                tv[y] += dv_t[pos] ** 2
    idx = torch.as_tensor(toks).cuda()
    check_grad("C3 dK last tokens", f64(dK[idx, gk].cpu()), wk, np.sqrt(tk))
    check_grad("C3 dV last tokens", f64(dV[idx, gk].cpu()), wv, np.sqrt(tv))

    dVs = dV.to(torch.float64).sum(dim=0).cpu().numpy()                      # [Hkv, D]
    dKs = dK.to(torch.float64).sum(dim=0).cpu().numpy()
    dOs = f64(dO).reshape(w.S, w.Hkv, G, w.D).sum(axis=(0, 2))
    # every element of dV, dK carries its own bf16 rounding (relative 2^-9) and the noise of its rounded terms, which
    # cancel in part (measured: about 7 x 2^-9 of the column's root-sum-square); over 65,536 tokens these add up like
    # a random walk
    tol_v = 16.0 * 2.0 ** -9 * np.sqrt((f64(dV.cpu()) ** 2).sum(axis=0)) + 1e-3 * np.abs(dOs)
    tol_k = 16.0 * 2.0 ** -9 * np.sqrt((f64(dK.cpu()) ** 2).sum(axis=0))
    print(f"[C3] sum dV - sum dO: max {np.abs(dVs - dOs).max():.3e} (tolerance {tol_v.min():.3e}..{tol_v.max():.3e}); "
          f"sum dK: max {np.abs(dKs).max():.3e} (tolerance {tol_k.min():.3e}..{tol_k.max():.3e})", flush=True)
    assert (np.abs(dVs - dOs) <= tol_v).all()
    assert (np.abs(dKs) <= tol_k).all()


def test_backward_quarter_million_tokens(B, oracle):
    """262,144 tokens (1,024 cubes, the largest configuration): offsets and tables at full scale.  A few dQ rows
    against the oracle, and the identities sum(dV) = sum(dO) per KV head, sum(dK) = 0."""
    w = synth.WORKLOADS["C4"]
    p = 0.9
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    Q, K, V = synth.generate(w)
    g = torch.Generator(device="cpu")
    g.manual_seed(synth.BASE_SEED + 31 * w.config_id)
    dO = torch.randn((w.S, w.Hq, w.D), generator=g, dtype=torch.float32).to(torch.bfloat16)
    Qg, Kg, Vg, dOg = Q.cuda(), K.cuda(), V.cuda(), dO.cuda()
    kbar = B.cube_pool(sh, Kg)
    mask_g, _, _, _ = B.cube_select(sh, Qg, kbar, p)
    print("[C4] forward", flush=True)
    O, lse = B.sparse_attn(sh, Qg, Kg, Vg, mask_g, return_lse=True)
    torch.cuda.synchronize()
    print("[C4] backward", flush=True)
    dQ, dK, dV = B.sparse_attn_bwd(sh, Qg, Kg, Vg, O, lse, dOg, sel_mask=mask_g)
    torch.cuda.synchronize()
    G, c = w.Hq // w.Hkv, 1.0 / np.sqrt(w.D)
    q, k, v = f64(Q), f64(K), f64(V)
    tables = oracle.bwd.cube_tables(osh)
    rows = np.array([0, w.Hq * 4097 + 3, w.Hq * (w.S // 2) + 11, w.Hq * (w.S - 300) + 27, w.S * w.Hq - 1])
    idx = torch.as_tensor(rows).cuda()
    mrows = mask_g[idx].cpu().numpy().view(np.uint32)
    do_rows, o_rows = f64(dO.reshape(-1, w.D)[rows]), f64(O.reshape(-1, w.D)[idx].cpu())
    want, terms = [], []
    for x, r in enumerate(rows):
        att, dq, _, _, _, ds, _ = oracle.bwd.row_backward(osh, q, k, v, mrows[x], r, do_rows[x], o_rows[x], tables)
        want.append(dq)
        terms.append(c * np.sqrt((ds * ds) @ (k[att, (r % w.Hq) // G] ** 2)))
    check_grad("C4 dQ sampled rows", f64(dQ.reshape(-1, w.D)[idx].cpu()), np.array(want), np.array(terms))
    dVs = dV.to(torch.float64).sum(dim=0).cpu().numpy()
    dKs = dK.to(torch.float64).sum(dim=0).cpu().numpy()
    dOs = dOg.view(w.S, w.Hkv, G, w.D).to(torch.float64).sum(dim=(0, 2)).cpu().numpy()
    tol_v = 16.0 * 2.0 ** -9 * torch.sqrt((dV.to(torch.float64) ** 2).sum(dim=0)).cpu().numpy() + 1e-3 * np.abs(dOs)
    tol_k = 16.0 * 2.0 ** -9 * torch.sqrt((dK.to(torch.float64) ** 2).sum(dim=0)).cpu().numpy()
    print(f"[C4] sum dV - sum dO: max {np.abs(dVs - dOs).max():.3e} (tolerance {tol_v.min():.3e}..{tol_v.max():.3e}); "
          f"sum dK: max {np.abs(dKs).max():.3e} (tolerance {tol_k.min():.3e}..{tol_k.max():.3e})", flush=True)
    assert np.isfinite(dVs).all() and np.isfinite(dKs).all()
    assert (np.abs(dVs - dOs) <= tol_v).all()
    assert (np.abs(dKs) <= tol_k).all()
