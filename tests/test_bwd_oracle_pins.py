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


def _explicit_row(oracle, sh, w, q, k, v, mask, r, do):
    """One row's attended tokens, probabilities and dS written out from scratch: the attended set from nested loops
    over the token grid (no use of the backward oracle's tables), a plain-Python softmax, scalar arithmetic."""
    cube_of, rank_of, _, _ = oracle.cube_map(sh)
    n, a = divmod(int(r), w.Hq)
    g = a // (w.Hq // w.Hkv)
    att = []
    for m in range(w.S):
        j = int(cube_of[m])
        if j < cube_of[n] and (int(mask[r, j >> 5]) >> (j & 31)) & 1:
            att.append(m)
        elif j == cube_of[n] and rank_of[m] <= rank_of[n]:
            att.append(m)
    s = [sum(float(q[n, a, d]) * float(k[m, g, d]) for d in range(w.D)) / w.D ** 0.5 for m in att]
    top = max(s)
    e = [np.exp(x - top) for x in s]
    z = sum(e)
    p = [x / z for x in e]
    o = [sum(p[x] * float(v[m, g, d]) for x, m in enumerate(att)) for d in range(w.D)]
    delta = sum(float(do[d]) * o[d] for d in range(w.D))
    ds = [p[x] * (sum(float(do[d]) * float(v[m, g, d]) for d in range(w.D)) - delta) for x, m in enumerate(att)]
    return n, a, g, att, s, p, o, ds


def test_error_scales_are_the_root_sum_square_of_the_terms(oracle):
    """The `scales` output is the unit of every backward tolerance: per gradient element, the root of the sum of the
    squares of the terms that add up to it.  Recomputed here for sampled elements from explicit per-term lists --
    dQ[r,d]: c dS_j k_jd over the row's attended tokens j; dK[m,g,d]: c dS_rm q_rd and dV[m,g,d]: p_rm dO_rd over
    the rows r (of the KV head's group) that attend token m."""
    w, sh, _, (q, k, v), mask, dO = setup(oracle, "T_tiny")
    T = {}
    oracle.bwd.sparse_attn_bwd(sh, q, k, v, mask, dO, scales=T)
    c = 1.0 / w.D ** 0.5
    R = w.S * w.Hq
    rows = {r: _explicit_row(oracle, sh, w, q, k, v, mask, r, dO[r]) for r in range(R)}
    rng = np.random.default_rng(11)
    for r in rng.choice(R, 12, replace=False):
        n, a, g, att, _, p, _, ds = rows[int(r)]
        for d in rng.choice(w.D, 3, replace=False):
            want = np.sqrt(sum((c * ds[x] * float(k[m, g, d])) ** 2 for x, m in enumerate(att)))
            assert T["dQ"][n, a, d] == pytest.approx(want, rel=1e-12, abs=1e-300)
    G = w.Hq // w.Hkv
    for m in [0, 1, w.S // 2, w.S - 1] + list(rng.choice(w.S, 6, replace=False)):
        for g in range(w.Hkv):
            d = int(rng.integers(0, w.D))
            tk, tv, count = 0.0, 0.0, 0
            for r in range(R):
                n, a, gr, att, _, p, _, ds = rows[r]
                if gr != g or m not in att:
                    continue
                x = att.index(m)
                tk += (c * ds[x] * float(q[n, a, d])) ** 2
                tv += (p[x] * float(dO[r, d])) ** 2
                count += 1
            assert count >= G                       # at least the token's own rows attend it
            assert T["dK"][m, g, d] == pytest.approx(np.sqrt(tk), rel=1e-12)
            assert T["dV"][m, g, d] == pytest.approx(np.sqrt(tv), rel=1e-12)


def test_delta_sensitivity_diagnostics(oracle):
    """`dQ_delta`, `dK_delta`: how far a gradient element moves when a row's delta is off by that row's
    delta_error_bound.  Pinned two ways: the bound itself from its explicit terms, and the sensitivity against an
    actual perturbation -- handing the oracle an O that moves every row's delta by exactly its bound (with either
    sign) must move dQ by exactly dQ_delta and dK by no more than dK_delta."""
    w, sh, _, (q, k, v), mask, dO = setup(oracle, "T_tiny")
    T = {}
    dQ0, dK0, dV0, delta0 = oracle.bwd.sparse_attn_bwd(sh, q, k, v, mask, dO, scales=T)
    R = w.S * w.Hq
    c = 1.0 / w.D ** 0.5
    derr = np.zeros(R)
    O_exact = oracle.bwd.sparse_attn_fwd(sh, q, k, v, mask)
    for r in range(R):
        n, a, g, att, s, p, o, ds = _explicit_row(oracle, sh, w, q, k, v, mask, r, dO[r])
        absdot = max(sum(abs(float(q[n, a, d]) * float(k[m, g, d])) for d in range(w.D)) for m in att) * c
        derr[r] = sum(abs(float(dO[r, d])) * (2.0 ** -8 * abs(o[d]) + 2.0 ** -7 * (1.0 + absdot / 8.0) *
                                              np.sqrt(sum((p[x] * float(v[m, g, d])) ** 2 for x, m in enumerate(att))))
                      for d in range(w.D))
        if r % 37 == 0:
            pk = [sum(p[x] * float(k[m, g, d]) for x, m in enumerate(att)) for d in range(w.D)]
            np.testing.assert_allclose(T["dQ_delta"][n, a], c * derr[r] * np.abs(pk), rtol=1e-11)
    # an O whose delta is off by sign_r * derr[r]: O + dO * (sign * derr / |dO|^2)
    sign = np.where(np.random.default_rng(5).random(R) < 0.5, -1.0, 1.0)
    O_off = O_exact + dO * (sign * derr / (dO * dO).sum(axis=1))[:, None]
    dQ1, dK1, dV1, delta1 = oracle.bwd.sparse_attn_bwd(sh, q, k, v, mask, dO, O=O_off)
    np.testing.assert_allclose(delta1 - delta0, sign * derr, rtol=1e-9, atol=1e-14)
    np.testing.assert_allclose(np.abs(dQ1 - dQ0), T["dQ_delta"], rtol=1e-8, atol=1e-15)
    assert (np.abs(dK1 - dK0) <= T["dK_delta"] * (1 + 1e-9) + 1e-15).all()
    # all signs equal: the rows' contributions to dK no longer cancel in the parts that have one sign
    assert np.abs(dK1 - dK0).max() > 0.05 * T["dK_delta"].max()
    np.testing.assert_array_equal(dV1, dV0)


def test_log_sum_exp_of_the_attended_scores(oracle):
    """lse_rows: against scipy's logsumexp of scores written out term by term, against the forward (the weights
    exp(s - lse) are the row's probabilities), and the companion value max_j sum_d |q_d k_jd| / sqrt(D)."""
    from scipy.special import logsumexp

    w, sh, _, (q, k, v), mask, dO = setup(oracle, "T_ragged")
    rows = synth.sample_rows(w, 10)
    lse, absdot = oracle.bwd.lse_rows(sh, q, k, mask[rows], rows)
    out = oracle.bwd.sparse_attn_fwd(sh, q, k, v, mask[rows], rows=rows)
    for x, r in enumerate(rows):
        n, a, g, att, s, p, o, _ = _explicit_row(oracle, sh, w, q, k, v, mask, r, dO[r])
        assert lse[x] == pytest.approx(logsumexp(np.array(s)), rel=1e-13, abs=1e-13)
        np.testing.assert_allclose(np.exp(np.array(s) - lse[x]), p, rtol=1e-11)
        np.testing.assert_allclose(out[x], o, rtol=1e-10, atol=1e-13)
        want = max(sum(abs(float(q[n, a, d]) * float(k[m, g, d])) for d in range(w.D)) for m in att) / w.D ** 0.5
        assert absdot[x] == pytest.approx(want, rel=1e-13)
