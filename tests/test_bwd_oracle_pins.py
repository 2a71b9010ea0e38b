"""Pins for the fp64 oracle of the attention backward pass: its forward agrees with the C oracle's (an independent
implementation of Eq. 3), its gradients agree with central finite differences of that forward and with torch
autograd on the case that reduces to dense causal attention, and the identities softmax gradients obey hold."""
import numpy as np
import pytest
import torch

from paper_2604_08077_amd import synth


def shape_of(o, w):
    return o.Shape(w.T, w.H, w.W, w.ct, w.ch, w.cw, w.Hq, w.Hkv, w.D, w.text, w.lead)


def setup(oracle, name, p=None, seed=3):
    w = synth.TEST_WORKLOADS[name]
    sh = shape_of(oracle, w)
    Q, K, V = synth.generate(w)
    kbar = oracle.cube_pool(sh, K)
    mask, _, _ = oracle.cube_select(sh, Q, kbar, w.top_p[0] if p is None else p)
    q, k, v = (t.to(torch.float64).numpy() for t in (Q, K, V))
    dO = np.random.default_rng(seed).standard_normal((w.S * w.Hq, w.D))
    return w, sh, (Q, K, V), (q, k, v), mask, dO


def test_forward_agrees_with_the_c_oracle(oracle):
    w, sh, bf, (q, k, v), mask, _ = setup(oracle, "T_tiny")
    ref, _ = oracle.sparse_attn(sh, *bf, mask)
    np.testing.assert_allclose(oracle.bwd.sparse_attn_fwd(sh, q, k, v, mask), ref, rtol=1e-11, atol=1e-12)
    w, sh, bf, (q, k, v), mask, _ = setup(oracle, "T_lead64")
    rows = synth.sample_rows(w, 64)
    ref, _ = oracle.sparse_attn(sh, *bf, mask[rows], rows=rows)
    np.testing.assert_allclose(oracle.bwd.sparse_attn_fwd(sh, q, k, v, mask[rows], rows=rows), ref, rtol=1e-11, atol=1e-12)


def test_gradients_match_finite_differences(oracle):
    """L = sum(O * G).  Central differences of the forward in every input, on a sample of coordinates."""
    w, sh, _, (q, k, v), mask, G = setup(oracle, "T_tiny")
    dQ, dK, dV, _ = oracle.bwd.sparse_attn_bwd(sh, q, k, v, mask, G)
    loss = lambda q_, k_, v_: float((oracle.bwd.sparse_attn_fwd(sh, q_, k_, v_, mask) * G).sum())
    rng = np.random.default_rng(0)
    h = 1e-5
    for which, grad in (("q", dQ), ("k", dK), ("v", dV)):
        base_arr = {"q": q, "k": k, "v": v}[which]
        for _ in range(6):
            idx = tuple(int(rng.integers(0, s)) for s in base_arr.shape)
            plus, minus = base_arr.copy(), base_arr.copy()
            plus[idx] += h
            minus[idx] -= h
            args_p = {"q": (plus, k, v), "k": (q, plus, v), "v": (q, k, plus)}[which]
            args_m = {"q": (minus, k, v), "k": (q, minus, v), "v": (q, k, minus)}[which]
            fd = (loss(*args_p) - loss(*args_m)) / (2 * h)
            assert grad[idx] == pytest.approx(fd, rel=2e-6, abs=2e-8), (which, idx)


def test_everything_selected_is_dense_causal_attention_under_autograd(oracle):
    """p = 1: every preceding cube attended.  Tokens reordered cube-major make it plain causal attention, whose
    gradient torch computes by automatic differentiation."""
    w, sh, _, (q, k, v), mask, G = setup(oracle, "T_mha64", p=1.0)
    dQ, dK, dV, _ = oracle.bwd.sparse_attn_bwd(sh, q, k, v, mask, G)
    cube_of, rank_of, _, start = oracle.cube_map(sh)
    pos = start[cube_of] + rank_of                          # position of every token in cube-major order
    order = np.argsort(pos)
    tq, tk, tv = (torch.tensor(x[order], requires_grad=True) for x in (q, k, v))     # [S, H, D], MHA
    s = torch.einsum("nhd,mhd->hnm", tq, tk) / np.sqrt(w.D)
    causal = torch.tril(torch.ones(w.S, w.S, dtype=torch.bool))
    o = torch.einsum("hnm,mhd->nhd", torch.softmax(s.masked_fill(~causal, -np.inf), dim=-1), tv)
    tG = torch.tensor(G.reshape(w.S, w.Hq, w.D)[order])
    (o * tG).sum().backward()
    for mine, theirs in ((dQ, tq.grad), (dK, tk.grad), (dV, tv.grad)):
        np.testing.assert_allclose(mine[order], theirs.numpy(), rtol=1e-9, atol=1e-11)


def test_softmax_gradient_identities(oracle):
    """GQA case.  With dO = 1 every row hands out probabilities that sum to one, so dV summed over the keys is the
    number of rows of the KV head; delta = dO.O; the ds of a row sum to zero, so shifting every key by one vector u
    (which moves all scores of a row by q.u and leaves the softmax alone) changes neither dK nor dQ."""
    w, sh, _, (q, k, v), mask, _ = setup(oracle, "T_tiny")
    ones = np.ones((w.S * w.Hq, w.D))
    _, _, dV, delta = oracle.bwd.sparse_attn_bwd(sh, q, k, v, mask, ones)
    # with dO = 1, sum_j dv_j over keys = sum over rows of (sum_j p_j) * 1 = number of rows of the KV head
    G = w.Hq // w.Hkv
    np.testing.assert_allclose(dV.sum(axis=0), np.full((w.Hkv, w.D), w.S * G), rtol=1e-12)
    # delta = do.o, and o is a convex combination of values
    O = oracle.bwd.sparse_attn_fwd(sh, q, k, v, mask)
    np.testing.assert_allclose(delta, O.sum(axis=1), rtol=1e-12)
    rng = np.random.default_rng(2)
    dO = rng.standard_normal((w.S * w.Hq, w.D))
    dQ, dK, _, _ = oracle.bwd.sparse_attn_bwd(sh, q, k, v, mask, dO)
    u = rng.standard_normal(w.D)
    dQ2, dK2, _, _ = oracle.bwd.sparse_attn_bwd(sh, q, k + u, v, mask, dO)
    # softmax is invariant to adding q.u to every score of a row, so p and ds do not change: dK is unchanged and
    # dQ changes by c * (sum_j ds_j) u = 0
    np.testing.assert_allclose(dK2, dK, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(dQ2, dQ, rtol=1e-9, atol=1e-11)
