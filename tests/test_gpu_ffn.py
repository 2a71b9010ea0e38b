"""GPU parity of the token-selective FFN (Sec. 3.3): the HIP library through its C ABI against the fp64 oracle on the
same seeded bf16 inputs.

Bars:
  * importance scores: fp32 against fp64, relative 2e-5;
  * activated-token sets: bit-exact, except in cubes the oracle flags as sitting within 1e-5 of the Top-p boundary
    (counted and printed);
  * outputs: the selection is the oracle's, so only arithmetic differs.  The GPU rounds the hidden activations to
    bf16 once (relative 2^-9 each, independent: the second product's error is a random sum of about that size
    relative to its own terms) and the output to bf16 (relative 2^-8 of |y| at most):
        |y_gpu - y_oracle| <= 2^-8 |y_oracle| + 2^-6 rms_over_the_token(y_oracle - x),
    (the second term: fourteen standard deviations of the sum of d_ff terms, each off by up to 2^-9 of itself)
    and the mean error must stay below a fifth of the mean bound.
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


def check_outputs(name, got, want, x):
    err = np.abs(got - want)
    move = np.sqrt(np.mean((want - x) ** 2, axis=1, keepdims=True))
    bound = 2.0 ** -8 * np.abs(want) + 2.0 ** -6 * move + 1e-30
    print(f"[{name}] elements={err.size} max-abs={err.max():.3e} mean-abs={err.mean():.3e} "
          f"worst err/bound={np.max(err / bound):.3f} mean err/mean bound={err.mean() / bound.mean():.3f}", flush=True)
    assert np.isfinite(got).all()
    assert (err <= bound).all()
    assert err.mean() <= 0.2 * bound.mean()


# (workload, d_model, d_ff, p): ragged cubes, text on either side, 256-token cubes, several row and weight tiles,
# several reduction depths
CASES = [
    ("T_tiny", 256, 128, 0.7),
    ("T_ragged", 256, 384, 0.6),
    ("T_text64", 512, 256, 0.7),
    ("T_lead64", 256, 640, 0.5),
    ("T_gqa128", 768, 1152, 0.7),
    ("T_cube2048", 256, 256, 0.6),      # 2,048 tokens per cube: more tokens than threads in every per-cube kernel
]


def workload(name):
    return synth.TEST_WORKLOADS.get(name) or synth.WORKLOADS[name]


@pytest.mark.parametrize("name,d_model,d_ff,p", CASES)
def test_ffn_select_matches_oracle(B, oracle, name, d_model, d_ff, p):
    w = workload(name)
    X = synth.generate_ffn(w, d_model, d_ff)[0]
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    cube_of = oracle.cube_map(osh)[0]
    for top_p in (p, 0.0, 1.0, 0.25, 0.95):
        print(f"[{name}] ffn_select d_model={d_model} p={top_p}", flush=True)
        keep, score, count = B.ffn_select(sh, X.cuda(), d_ff, top_p, eps=1e-6)
        torch.cuda.synchronize()
        rk, rs, near = oracle.ffn.ffn_select(osh, f64(X), top_p, eps=1e-6)
        np.testing.assert_allclose(score.cpu().numpy(), rs, rtol=2e-5, atol=1e-12)
        k = keep.cpu().numpy()
        assert set(np.unique(k).tolist()) <= {0, 1}
        differ = np.unique(cube_of[k != rk])
        bad = [c for c in differ if not near[c]]
        print(f"[{name}] p={top_p} cubes={near.size} near-boundary(exempt)={int(near.sum())} "
              f"differing cubes={differ.size} kept={int(k.sum())}/{k.size}", flush=True)
        assert not bad, f"cubes {bad} differ from the oracle away from the Top-p boundary"
        assert np.array_equal(count.cpu().numpy(), np.bincount(cube_of, weights=k, minlength=near.size).astype(np.int32))


@pytest.mark.parametrize("name,d_model,d_ff,p", CASES)
def test_ffn_sparse_matches_oracle(B, oracle, name, d_model, d_ff, p):
    w = workload(name)
    X, Wg, Wu, Wd = synth.generate_ffn(w, d_model, d_ff)
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    x64, g64, u64, d64 = (f64(t) for t in (X, Wg, Wu, Wd))
    dev = [t.cuda() for t in (X, Wg, Wu, Wd)]
    for top_p in (p, 0.2):
        keep = oracle.ffn.ffn_select(osh, x64, top_p)[0]
        want = oracle.ffn.ffn_sparse(osh, x64, g64, u64, d64, keep)
        print(f"[{name}] ffn_sparse d_model={d_model} d_ff={d_ff} p={top_p} activated={int(keep.sum())}/{keep.size}",
              flush=True)
        Y = B.ffn_sparse(sh, *dev, keep=torch.from_numpy(keep).cuda())
        torch.cuda.synchronize()
        check_outputs(f"{name} p={top_p}", f64(Y.cpu()), want, x64)
    print(f"[{name}] dense layer", flush=True)
    Y = B.ffn_sparse(sh, *dev, keep=None)
    torch.cuda.synchronize()
    check_outputs(f"{name} dense", f64(Y.cpu()), oracle.ffn.ffn_dense(x64, g64, u64, d64), x64)


def test_ffn_degenerate_masks(B, oracle):
    """No token activated: the input comes back bit for bit.  One activated token per cube: every other token of
    the cube moves by that token's FFN value.  Stale workspace contents must not matter."""
    w = workload("T_ragged")
    d_model, d_ff = 256, 384
    X, Wg, Wu, Wd = synth.generate_ffn(w, d_model, d_ff)
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    x64, g64, u64, d64 = (f64(t) for t in (X, Wg, Wu, Wd))
    dev = [t.cuda() for t in (X, Wg, Wu, Wd)]
    ws = torch.full((B.ffn_workspace_bytes(sh, d_model, d_ff),), 0xFF, dtype=torch.uint8, device="cuda")
    print("[T_ragged] no token activated", flush=True)
    Y = B.ffn_sparse(sh, *dev, keep=torch.zeros(w.S, dtype=torch.uint8, device="cuda"), workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(Y.cpu(), X)
    cube_of, rank_of, size_of, _ = oracle.cube_map(osh)
    keep = (rank_of == (size_of[cube_of] - 1)).astype(np.uint8)      # the last token of every cube
    print("[T_ragged] one token per cube", flush=True)
    Y = B.ffn_sparse(sh, *dev, keep=torch.from_numpy(keep).cuda(), workspace=ws)
    torch.cuda.synchronize()
    check_outputs("T_ragged one per cube", f64(Y.cpu()), oracle.ffn.ffn_sparse(osh, x64, g64, u64, d64, keep), x64)


def test_ffn_full_size_sampled(B, oracle):
    """65,536 tokens, the backbone's widths (3584 / 18944), the launch configuration the benchmark times: two whole
    cubes and a sample of activated tokens elsewhere are recomputed by the oracle; the selection is checked in full."""
    w = synth.WORKLOADS["C3"]
    d_model, d_ff, p = 3584, 18944, 0.7
    X, Wg, Wu, Wd = synth.generate_ffn(w, d_model, d_ff)
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    Xg = X.cuda()
    print("[C3] ffn_select", flush=True)
    keep, score, count = B.ffn_select(sh, Xg, d_ff, p)
    torch.cuda.synchronize()
    x64 = f64(X)
    rk, rs, near = oracle.ffn.ffn_select(osh, x64, p)
    cube_of = oracle.cube_map(osh)[0]
    k = keep.cpu().numpy()
    np.testing.assert_allclose(score.cpu().numpy(), rs, rtol=2e-5, atol=1e-12)
    differ = np.unique(cube_of[k != rk])
    print(f"[C3] cubes={near.size} near-boundary(exempt)={int(near.sum())} differing={differ.size} "
          f"activated share={k.mean():.3f}", flush=True)
    assert all(near[c] for c in differ)
    print("[C3] ffn_sparse", flush=True)
    dev = [t.cuda() for t in (Wg, Wu, Wd)]
    Y = B.ffn_sparse(sh, Xg, *dev, keep=torch.from_numpy(rk).cuda())
    torch.cuda.synchronize()
    g64, u64, d64 = (f64(t) for t in (Wg, Wu, Wd))
    rng = np.random.default_rng(11)
    picks = rng.choice(np.nonzero(rk)[0], 48, replace=False)
    F = oracle.ffn.ffn(x64[picks], g64, u64, d64)
    check_outputs("C3 activated sample", f64(Y[torch.from_numpy(picks).cuda()].cpu()), x64[picks] + F, x64[picks])
    for c in (0, 171):
        toks = np.nonzero(cube_of == c)[0]
        act, rest = toks[rk[toks] != 0], toks[rk[toks] == 0]
        Fc = oracle.ffn.ffn(x64[act], g64, u64, d64)
        want = np.concatenate([x64[act] + Fc, x64[rest] + Fc.mean(axis=0)])
        got = f64(Y[torch.from_numpy(np.concatenate([act, rest])).cuda()].cpu())
        check_outputs(f"C3 cube {c} ({act.size} activated, {rest.size} bypassed)", got, want,
                      x64[np.concatenate([act, rest])])


def test_ffn_zero_tokens_and_zero_cube(B, oracle):
    """Tokens of norm zero rank last; a cube whose tokens are all zero has an all-zero distribution, whose mass never
    reaches p: every token is activated (and FFN(0) = 0 leaves them unchanged)."""
    w = workload("T_ragged")
    d_model, d_ff = 256, 384
    X, Wg, Wu, Wd = synth.generate_ffn(w, d_model, d_ff)
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    cube_of = oracle.cube_map(osh)[0]
    X = X.clone()
    X[cube_of == 3] = 0                                  # a whole cube
    X[torch.from_numpy(np.nonzero(cube_of == 5)[0][::3])] = 0   # every third token of another
    x64 = f64(X)
    for p, eps in ((0.6, 1e-6), (0.999, 1e-6), (0.6, 0.0)):   # eps = 0: the all-zero cube's 0/0 scores are 0, not NaN
        print(f"[T_ragged zeros] ffn_select p={p} eps={eps}", flush=True)
        keep, score, _ = B.ffn_select(sh, X.cuda(), d_ff, p, eps=eps)
        torch.cuda.synchronize()
        assert torch.isfinite(score).all()
        rk, rs, near = oracle.ffn.ffn_select(osh, x64, p, eps=eps)
        k = keep.cpu().numpy()
        differ = np.unique(cube_of[k != rk])
        assert all(near[c] for c in differ)
        assert k[cube_of == 3].all() and (score.cpu().numpy()[cube_of == 3] == 0).all()
        if p == 0.6:
            assert not k[np.nonzero(cube_of == 5)[0][::3]].any()
    keep = oracle.ffn.ffn_select(osh, x64, 0.6)[0]
    Y = B.ffn_sparse(sh, X.cuda(), Wg.cuda(), Wu.cuda(), Wd.cuda(), keep=torch.from_numpy(keep).cuda())
    torch.cuda.synchronize()
    check_outputs("T_ragged zeros", f64(Y.cpu()), oracle.ffn.ffn_sparse(osh, x64, f64(Wg), f64(Wu), f64(Wd), keep), x64)
    assert (Y.cpu()[cube_of == 3] == 0).all()


def test_ffn_full_size_every_token(B, oracle):
    """The benchmark's configuration (65,536 tokens, 3584 / 18944, p = 0.7) compared on EVERY output element: cube by
    cube, the oracle's layer on the activated tokens and its mean on the others."""
    w = synth.WORKLOADS["C3"]
    d_model, d_ff, p = 3584, 18944, 0.7
    X, Wg, Wu, Wd = synth.generate_ffn(w, d_model, d_ff)
    sh, osh = B.Shape.of(w), oshape(oracle, w)
    x64 = f64(X)
    rk, _, _ = oracle.ffn.ffn_select(osh, x64, p)
    Y = B.ffn_sparse(sh, X.cuda(), Wg.cuda(), Wu.cuda(), Wd.cuda(), keep=torch.from_numpy(rk).cuda())
    torch.cuda.synchronize()
    got_all = Y.cpu()
    g64, u64, d64 = (f64(t) for t in (Wg, Wu, Wd))
    cube_of = oracle.cube_map(osh)[0]
    worst, err_sum, bound_sum, n = 0.0, 0.0, 0.0, 0
    for c in range(int(cube_of.max()) + 1):
        toks = np.nonzero(cube_of == c)[0]
        act, rest = toks[rk[toks] != 0], toks[rk[toks] == 0]
        order = np.concatenate([act, rest])
        Fc = oracle.ffn.ffn(x64[act], g64, u64, d64)
        want = np.concatenate([x64[act] + Fc, x64[rest] + Fc.mean(axis=0)])
        err = np.abs(f64(got_all[torch.from_numpy(order)]) - want)
        move = np.sqrt(np.mean((want - x64[order]) ** 2, axis=1, keepdims=True))
        bound = 2.0 ** -8 * np.abs(want) + 2.0 ** -6 * move + 1e-30
        assert (err <= bound).all(), f"cube {c}"
        worst = max(worst, float(np.max(err / bound)))
        err_sum, bound_sum, n = err_sum + float(err.sum()), bound_sum + float(bound.sum()), n + err.size
        if c % 16 == 15:
            print(f"[C3 ffn every token] cubes 0..{c}: worst err/bound so far {worst:.3f}", flush=True)
    print(f"[C3 ffn every token] elements={n} worst err/bound={worst:.3f} mean err/mean bound={err_sum / bound_sum:.3f}",
          flush=True)
    assert err_sum <= 0.2 * bound_sum
