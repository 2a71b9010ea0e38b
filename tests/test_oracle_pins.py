"""Pins for the fp64 oracle: every check here compares the oracle with something
other than itself -- a closed form, an invariant of the rule, brute force on tiny
inputs, or a library routine (numpy / scipy / torch CPU) on a case that reduces
to it.  The paper prints no worked numeric example, so there is no printed value
to compare with; tests/golden/ holds hand-derived closed-form cases.
"""
import itertools
import json
import math
import os

import numpy as np
import pytest
import torch
from scipy.special import softmax as sp_softmax

from paper_2604_08077_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def shape_of(o, w):
    return o.Shape(w.T, w.H, w.W, w.ct, w.ch, w.cw, w.Hq, w.Hkv, w.D, w.text, w.lead)


def widen(x):
    return x.to(torch.float64).numpy()


def brute_cube_table(w):
    """Independent cube map: leading text in runs of one full cube's length, then the video cubes walked in
    (tb,hb,wb) order and inside each cube in local (t,h,w) order, handing out ranks as tokens are met, then the
    trailing text in runs."""
    T, H, W = w.grid
    ct, ch, cw = w.cube
    full = ct * ch * cw
    S = w.lead + T * H * W + w.text
    cube_of = -np.ones(S, np.int64)
    rank_of = -np.ones(S, np.int64)
    sizes = []
    c = 0

    def text_span(first, count):
        nonlocal c
        done = 0
        while done < count:
            take = min(full, count - done)
            cube_of[first + done: first + done + take] = c
            rank_of[first + done: first + done + take] = np.arange(take)
            sizes.append(take)
            c += 1
            done += take

    text_span(0, w.lead)
    for t0 in range(0, T, ct):
        for h0 in range(0, H, ch):
            for w0 in range(0, W, cw):
                r = 0
                for t in range(t0, min(t0 + ct, T)):
                    for h in range(h0, min(h0 + ch, H)):
                        for x in range(w0, min(w0 + cw, W)):
                            n = w.lead + (t * H + h) * W + x
                            cube_of[n], rank_of[n] = c, r
                            r += 1
                sizes.append(r)
                c += 1
    text_span(w.lead + T * H * W, w.text)
    assert (cube_of >= 0).all()
    return cube_of, rank_of, np.array(sizes)


def video_cubes(w):
    T, H, W = w.grid
    ct, ch, cw = w.cube
    return -(-T // ct) * -(-H // ch) * -(-W // cw)


def lead_cubes(w):
    return -(-w.lead // (w.ct * w.ch * w.cw))


ALL_SMALL = list(synth.TEST_WORKLOADS.values())


# --------------------------------------------------------------------------- cube map
@pytest.mark.parametrize("w", ALL_SMALL + [synth.WORKLOADS["C1"], synth.WORKLOADS["C5"]], ids=lambda w: w.name)
def test_cube_map_matches_brute_force_and_is_bijection(oracle, w):
    cube_of, rank_of, size_of, start = oracle.cube_map(shape_of(oracle, w))
    bc, br, bs = brute_cube_table(w)
    assert np.array_equal(cube_of, bc)
    assert np.array_equal(rank_of, br)
    assert np.array_equal(size_of, bs)
    assert size_of.sum() == w.S and start[-1] == w.S
    pos = start[cube_of] + rank_of
    assert np.array_equal(np.sort(pos), np.arange(w.S))


def test_cube_counts_of_benchmark_configs(oracle):
    expect = {"C1": 64, "C2": 64, "C3": 256, "C4": 1024, "C5": 150}
    for name, n in expect.items():
        assert oracle.num_cubes(shape_of(oracle, synth.WORKLOADS[name])) == n
    _, _, size_of, _ = oracle.cube_map(shape_of(oracle, synth.WORKLOADS["C5"]))
    # 15x20 frames with 8x8 faces: faces of 8x8, 8x4, 7x8, 7x4 tokens, 4 frames deep
    assert sorted(set(size_of.tolist())) == [112, 128, 224, 256]
    for name in ("C2", "C3"):
        _, _, size_of, _ = oracle.cube_map(shape_of(oracle, synth.WORKLOADS[name]))
        assert set(size_of.tolist()) == {256}


def test_whole_frame_cubes_make_cube_major_equal_raster(oracle):
    sh = oracle.Shape(8, 4, 6, 2, 4, 6, 1, 1, 64)
    cube_of, rank_of, _, start = oracle.cube_map(sh)
    assert np.array_equal(start[cube_of] + rank_of, np.arange(sh.S))


# --------------------------------------------------------------------------- pool
@pytest.mark.parametrize("w", ALL_SMALL, ids=lambda w: w.name)
def test_pool_equals_numpy_mean_over_members(oracle, w):
    _, K, _ = synth.generate(w)
    kbar = oracle.cube_pool(shape_of(oracle, w), K)
    bc, _, _ = brute_cube_table(w)
    Kd = widen(K)
    for c in range(kbar.shape[0]):
        ref = Kd[np.nonzero(bc == c)[0]].mean(axis=0)
        np.testing.assert_allclose(kbar[c], ref, rtol=0, atol=1e-13)


def test_pool_constant_and_indicator(oracle):
    w = synth.TEST_WORKLOADS["T_tiny"]
    sh = shape_of(oracle, w)
    N = oracle.num_cubes(sh)
    K = torch.full((w.S, w.Hkv, w.D), 1.5, dtype=torch.bfloat16)
    assert np.all(oracle.cube_pool(sh, K) == 1.5)
    bc, _, _ = brute_cube_table(w)
    assert N <= w.D
    K = torch.zeros((w.S, w.Hkv, w.D), dtype=torch.bfloat16)
    K[torch.arange(w.S), :, torch.from_numpy(bc)] = 1.0
    kbar = oracle.cube_pool(sh, K)
    for g in range(w.Hkv):
        np.testing.assert_allclose(kbar[:, g, :N], np.eye(N), atol=1e-15)


# --------------------------------------------------------------------------- relevance (Eq. 1)
def test_relevance_closed_form_golden(oracle):
    with open(os.path.join(GOLDEN, "relevance_closed_form.json")) as f:
        case = json.load(f)
    q = np.array(case["q"], np.float64)
    kb = np.array(case["kbar"], np.float64)
    logits, probs = oracle.relevance(q, kb)
    np.testing.assert_allclose(logits, case["logits"], rtol=0, atol=1e-15)
    e = math.e
    closed = np.array([1.0, e, e * e]) / (1.0 + e + e * e)
    np.testing.assert_allclose(probs, closed, rtol=1e-15)
    np.testing.assert_allclose(probs, case["probs"], rtol=1e-12)


def test_relevance_zero_query_is_uniform_and_matches_scipy(oracle):
    rng = np.random.default_rng(3)
    kb = rng.standard_normal((9, 64))
    _, probs = oracle.relevance(np.zeros(64), kb)
    np.testing.assert_allclose(probs, np.full(9, 1 / 9), rtol=1e-15)
    q = rng.standard_normal(64)
    logits, probs = oracle.relevance(q, kb)
    np.testing.assert_allclose(logits, kb @ q / 8.0, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(probs, sp_softmax(kb @ q / 8.0), rtol=1e-12)


# --------------------------------------------------------------------------- Top-p (Eq. 2)
def brute_top_p(probs, p):
    """Set definition of the nucleus: smallest cardinality with mass >= p; among
    those the largest mass; among those the lexicographically smallest index set."""
    n = len(probs)
    if p <= 0:
        return set()
    for k in range(1, n + 1):
        best = None
        for sub in itertools.combinations(range(n), k):
            mass = sum(probs[j] for j in sub)
            key = (-mass, sub)
            if best is None or key < best:
                best = key
        # masses are compared exactly: test distributions are dyadic rationals
        if -best[0] >= p:
            return set(best[1])
    return set(range(n))


def dyadic_distribution(rng, n, denom=1 << 12):
    cuts = np.sort(rng.choice(np.arange(1, denom), size=n - 1, replace=False))
    parts = np.diff(np.concatenate([[0], cuts, [denom]]))
    return parts / denom


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 11])
def test_top_p_equals_subset_enumeration(oracle, n):
    rng = np.random.default_rng(100 + n)
    for trial in range(12):
        probs = dyadic_distribution(rng, n) if n > 1 else np.array([1.0])
        if trial % 3 == 0 and n > 2:           # plant ties
            probs[1] = probs[0] = (probs[0] + probs[1]) / 2
        for p in (1 / 8, 0.5, 0.6875, 0.9375, 4095 / 4096):
            keep, _, _ = oracle.top_p(probs, p)
            assert set(np.nonzero(keep)[0].tolist()) == brute_top_p(probs.tolist(), p), (probs, p)


def test_top_p_uniform_one_hot_and_limits(oracle):
    for n, p in ((8, 0.5), (16, 0.6875), (64, 0.9375), (32, 1 / 32), (32, 1 / 32 + 1 / 1024)):
        keep, _, _ = oracle.top_p(np.full(n, 1.0 / n), p)
        k = math.ceil(p * n)
        assert keep.sum() == k and keep[:k].all()      # ties resolved toward low cube index
    onehot = np.zeros(10)
    onehot[7] = 1.0
    keep, _, _ = oracle.top_p(onehot, 0.9)
    assert keep.tolist() == [j == 7 for j in range(10)]
    probs = np.array([0.5, 0.25, 0.125, 0.125])
    assert oracle.top_p(probs, 0.0)[0].sum() == 0
    assert oracle.top_p(probs, 1.0)[0].all()
    # the element on which the cumulative mass reaches p exactly is the last one kept
    assert oracle.top_p(probs, 0.75)[0].tolist() == [True, True, False, False]
    assert oracle.top_p(probs, 0.75 + 2 ** -20)[0].tolist() == [True, True, True, False]


def unpack(mask, N):
    bits = (mask[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1
    return bits.reshape(mask.shape[0], -1)[:, :N].astype(bool)


@pytest.mark.parametrize("w", ALL_SMALL, ids=lambda w: w.name)
def test_select_invariants_and_independent_recomputation(oracle, w):
    sh = shape_of(oracle, w)
    N = oracle.num_cubes(sh)
    Q, K, _ = synth.generate(w)
    kbar = oracle.cube_pool(sh, K)
    bc, _, _ = brute_cube_table(w)
    Qd = widen(Q)
    G = w.Hq // w.Hkv
    prev = None
    for p in (0.3, 0.6, w.top_p[0], 0.97):
        mask, count, _ = oracle.cube_select(sh, Q, kbar, p)
        sel = unpack(mask, N)
        assert np.array_equal(sel.sum(1), count)
        if prev is not None:                      # nesting in p
            assert not (prev & ~sel).any()
        prev = sel
        rng = np.random.default_rng(5)
        nv, npre = video_cubes(w), lead_cubes(w)
        picks = rng.choice(w.S * w.Hq, size=60, replace=False).tolist()
        picks += list(range(w.S * w.Hq - min(w.text, 3) * w.Hq, w.S * w.Hq))   # the last text rows, if any
        picks += list(range(0, min(w.lead, 3) * w.Hq))                         # the first text rows, if any
        for r in picks:
            n, a = divmod(int(r), w.Hq)
            own = bc[n]
            assert not sel[r, own:].any()         # own and later cubes never selected
            lo, hi = npre, max(npre, min(own, npre + nv))   # candidates: the video cubes before the own cube
            i = hi - lo
            # text cubes before the own cube are always attended
            assert sel[r, :min(own, npre)].all() and sel[r, npre + nv:own].all()
            assert count[r] == sel[r, lo:hi].sum() + min(own, npre) + max(own - npre - nv, 0)
            if i == 0:
                continue
            probs = sp_softmax(kbar[lo:hi, a // G] @ Qd[n, a] / math.sqrt(w.D))
            s = sel[r, lo:hi]
            mass = probs[s].sum()
            assert mass >= p - 1e-12
            assert mass - probs[s].min() < p + 1e-12         # minimal prefix
            if (~s).any():
                assert probs[s].min() >= probs[~s].max() - 1e-15
            if i <= 10:
                # independent brute force; masses are not dyadic here, so allow the
                # enumeration to differ only if two masses tie within rounding
                bf = brute_top_p(probs.tolist(), p)
                assert bf == set(np.nonzero(s)[0].tolist())


def test_select_heads_differ_and_p_limits(oracle):
    w = synth.TEST_WORKLOADS["T_gqa128"]
    sh = shape_of(oracle, w)
    N = oracle.num_cubes(sh)
    Q, K, _ = synth.generate(w)
    kbar = oracle.cube_pool(sh, K)
    bc, _, _ = brute_cube_table(w)
    m1, c1, _ = oracle.cube_select(sh, Q, kbar, 1.0)
    assert np.array_equal(c1, np.repeat(bc, w.Hq))           # every preceding cube
    m0, c0, _ = oracle.cube_select(sh, Q, kbar, 0.0)
    assert not c0.any() and not m0.any()
    m, c, _ = oracle.cube_select(sh, Q, kbar, 0.9)
    sel = unpack(m, N).reshape(w.S, w.Hq, N)
    last = sel[-1]
    assert any(not np.array_equal(last[0], last[a]) for a in range(1, w.Hq))  # per query head
    rows = np.array([5, 77, w.S * w.Hq - 1], np.int64)
    ms, cs, _ = oracle.cube_select(sh, Q, kbar, 0.9, rows=rows)
    assert np.array_equal(ms, m[rows]) and np.array_equal(cs, c[rows])


# --------------------------------------------------------------------------- fixed Top-K (ablation baseline)
def brute_top_k(probs, k):
    """Set definition: the subset of min(k, n) elements of largest total mass; among subsets of equal mass the
    lexicographically smallest index set (ties go to the lower cube index)."""
    n = len(probs)
    m = min(k, n)
    best = None
    for sub in itertools.combinations(range(n), m):
        key = (-sum(probs[j] for j in sub), sub)      # dyadic masses: exact sums
        if best is None or key < best:
            best = key
    return set(best[1])


@pytest.mark.parametrize("n", [1, 2, 3, 5, 8, 10])
def test_top_k_equals_subset_enumeration_and_stable_argsort(oracle, n):
    rng = np.random.default_rng(300 + n)
    for trial in range(10):
        probs = dyadic_distribution(rng, n) if n > 1 else np.array([1.0])
        if trial % 3 == 0 and n > 3:               # plant a three-way tie straddling typical cuts
            probs[1] = probs[2] = probs[3] = (probs[1] + probs[2] + probs[3]) / 3 if n > 3 else probs[1]
        for k in (0, 1, 2, n // 2, n - 1, n, n + 3):
            if k < 0:
                continue
            keep, order = oracle.top_k(probs, k)
            got = set(np.nonzero(keep)[0].tolist())
            assert len(got) == min(k, n)
            # library routine: a stable sort of the negated values ranks ties by ascending index
            ref_order = np.argsort(-probs, kind="stable")
            assert order.tolist() == ref_order.tolist()
            assert got == set(ref_order[:k].tolist())
            if n <= 8 and abs(probs.sum() - 1.0) < 1e-15 and trial % 3 != 0:
                assert got == brute_top_k(probs.tolist(), k)


def test_top_k_ties_prefer_low_index_and_nesting(oracle):
    probs = np.array([0.125, 0.25, 0.25, 0.125, 0.25])
    assert oracle.top_k(probs, 2)[0].tolist() == [False, True, True, False, False]
    assert oracle.top_k(probs, 3)[0].tolist() == [False, True, True, False, True]
    assert oracle.top_k(probs, 4)[0].tolist() == [True, True, True, False, True]
    prev = np.zeros(5, bool)
    for k in range(0, 7):
        keep, _ = oracle.top_k(probs, k)
        assert not (prev & ~keep).any() and keep.sum() == min(k, 5)
        prev = keep


@pytest.mark.parametrize("w", [synth.TEST_WORKLOADS[k] for k in ("T_ragged", "T_gqa128", "T_manycubes")],
                         ids=lambda w: w.name)
def test_select_topk_invariants(oracle, w):
    sh = shape_of(oracle, w)
    N = oracle.num_cubes(sh)
    Q, K, _ = synth.generate(w)
    kbar = oracle.cube_pool(sh, K)
    bc, _, _ = brute_cube_table(w)
    Qd = widen(Q)
    G = w.Hq // w.Hkv
    cubes_of_row = np.repeat(bc, w.Hq)
    prev = None
    for k in (0, 1, 3, 7, N):
        mask, count, _ = oracle.cube_select_topk(sh, Q, kbar, k)
        sel = unpack(mask, N)
        assert np.array_equal(sel.sum(1), count)
        assert np.array_equal(count, np.minimum(k, cubes_of_row))     # exactly min(k, #preceding cubes)
        if prev is not None:
            assert not (prev & ~sel).any()                            # nesting in k
        prev = sel
        rng = np.random.default_rng(9)
        for r in rng.choice(w.S * w.Hq, size=60, replace=False):
            n, a = divmod(int(r), w.Hq)
            i = bc[n]
            assert not sel[r, i:].any()
            if i == 0 or k == 0:
                continue
            logits = kbar[:i, a // G] @ Qd[n, a] / math.sqrt(w.D)
            s = sel[r, :i]
            if (~s).any():
                assert logits[s].min() >= logits[~s].max()            # nothing dropped outranks a kept cube
            assert set(np.nonzero(s)[0].tolist()) == set(np.argsort(-logits, kind="stable")[:k].tolist())
    # k >= number of cubes is the p = 1 selection: every preceding cube
    m_all, _, _ = oracle.cube_select_topk(sh, Q, kbar, N)
    m_p1, _, _ = oracle.cube_select(sh, Q, kbar, 1.0)
    assert np.array_equal(m_all, m_p1)


# --------------------------------------------------------------------------- attention (Eq. 3)
def torch_dense_reference(w, Q, K, V, pos):
    """scaled_dot_product_attention (CPU, fp64, is_causal) on cube-major ordered,
    GQA-expanded tensors; result returned in raster token order."""
    order = np.argsort(pos)
    G = w.Hq // w.Hkv
    q = Q.to(torch.float64)[order].permute(1, 0, 2)
    k = K.to(torch.float64)[order].repeat_interleave(G, dim=1).permute(1, 0, 2)
    v = V.to(torch.float64)[order].repeat_interleave(G, dim=1).permute(1, 0, 2)
    o = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True)
    out = torch.empty_like(o)
    out[:, order] = o
    return out.permute(1, 0, 2).reshape(w.S * w.Hq, w.D).numpy()


@pytest.mark.parametrize("w", ALL_SMALL, ids=lambda w: w.name)
def test_p_one_equals_dense_and_torch_sdpa(oracle, w):
    sh = shape_of(oracle, w)
    Q, K, V = synth.generate(w)
    kbar = oracle.cube_pool(sh, K)
    mask, _, _ = oracle.cube_select(sh, Q, kbar, 1.0)
    sparse, nk = oracle.sparse_attn(sh, Q, K, V, mask)
    dense = oracle.dense_attn(sh, Q, K, V)
    np.testing.assert_allclose(sparse, dense, rtol=0, atol=1e-12)
    bc, br, bs = brute_cube_table(w)
    start = np.concatenate([[0], np.cumsum(bs)])
    pos = start[bc] + br
    assert np.array_equal(nk, np.repeat(pos + 1, w.Hq))
    np.testing.assert_allclose(dense, torch_dense_reference(w, Q, K, V, pos), rtol=0, atol=1e-12)


@pytest.mark.parametrize("w", ALL_SMALL[:3], ids=lambda w: w.name)
def test_p_zero_is_block_diagonal_causal_and_first_cube_ignores_p(oracle, w):
    sh = shape_of(oracle, w)
    N = oracle.num_cubes(sh)
    Q, K, V = synth.generate(w)
    kbar = oracle.cube_pool(sh, K)
    m0, _, _ = oracle.cube_select(sh, Q, kbar, 0.0)
    out0, nk0 = oracle.sparse_attn(sh, Q, K, V, m0)
    bc, br, _ = brute_cube_table(w)
    Qd, Kd, Vd = widen(Q), widen(K), widen(V)
    G = w.Hq // w.Hkv
    ref = np.zeros_like(out0)
    for n in range(w.S):
        keys = np.nonzero((bc == bc[n]) & (br <= br[n]))[0]
        for a in range(w.Hq):
            pr = sp_softmax(Kd[keys, a // G] @ Qd[n, a] / math.sqrt(w.D))
            ref[n * w.Hq + a] = pr @ Vd[keys, a // G]
    np.testing.assert_allclose(out0, ref, rtol=0, atol=1e-12)
    assert np.array_equal(nk0, np.repeat(br + 1, w.Hq))
    mp, _, _ = oracle.cube_select(sh, Q, kbar, 0.9)
    outp, _ = oracle.sparse_attn(sh, Q, K, V, mp)
    first = np.repeat(bc == 0, w.Hq)
    assert np.array_equal(outp[first], out0[first])
    assert N > 1 and not np.allclose(outp[~first], out0[~first])


@pytest.mark.parametrize("name", ["T_text64", "T_text128", "T_lead64", "T_lead128"])
def test_rows_of_text_and_video_recomputed_from_explicit_token_lists(oracle, name):
    """End of Sec. 3.2, recomputed in numpy from an explicit token list for rows of all three spans: every
    earlier text token (leading and trailing), the video tokens of the cubes the nucleus rule keeps among the
    video cubes before the own cube (a trailing-text query: among ALL video cubes), and the causal part of the
    own cube.  Without leading text, video rows give what they give with the trailing text cut off."""
    w = synth.TEST_WORKLOADS[name]
    sh = shape_of(oracle, w)
    N, nv, npre, Sv = oracle.num_cubes(sh), video_cubes(w), lead_cubes(w), w.S_video
    Q, K, V = synth.generate(w)
    Qd, Kd, Vd = widen(Q), widen(K), widen(V)
    kbar = oracle.cube_pool(sh, K)
    bc, br, _ = brute_cube_table(w)
    G = w.Hq // w.Hkv
    p = w.top_p[0]
    is_text = np.ones(w.S, bool)
    is_text[w.lead: w.lead + Sv] = False
    rows = np.unique(np.concatenate([np.arange(0, w.lead * w.Hq, 3), np.arange(w.lead * w.Hq, w.S * w.Hq, 41),
                                     np.arange((w.lead + Sv) * w.Hq, w.S * w.Hq, 5)])).astype(np.int64)
    mask, count, _ = oracle.cube_select(sh, Q, kbar, p, rows=rows)
    out, nk = oracle.sparse_attn(sh, Q, K, V, mask, rows=rows)
    sel = unpack(mask, N)
    for x, r in enumerate(rows):
        n, a = divmod(int(r), w.Hq)
        kvh = a // G
        own = bc[n]
        ncand = max(min(own, npre + nv) - npre, 0)
        keep_cube = np.zeros(N, bool)
        if ncand:
            probs = sp_softmax(kbar[npre:npre + ncand, kvh] @ Qd[n, a] / math.sqrt(w.D))
            keep, _, _ = oracle.top_p(probs, p)       # the nucleus rule itself is pinned by enumeration above
            keep_cube[npre:npre + ncand] = keep
        assert np.array_equal(sel[x, npre:npre + nv], keep_cube[npre:npre + nv])
        attended = (keep_cube[bc] & ~is_text) | (is_text & (bc < own)) | ((bc == own) & (br <= br[n]))
        toks = np.nonzero(attended)[0]
        assert nk[x] == toks.size
        ref = sp_softmax(Kd[toks, kvh] @ Qd[n, a] / math.sqrt(w.D)) @ Vd[toks, kvh]
        assert np.abs(out[x] - ref).max() < 1e-10
    if w.lead == 0:
        # video rows do not see text that follows them: same selection and output as for the video alone
        wv = synth.Workload(**{**w.__dict__, "text": 0})
        shv = shape_of(oracle, wv)
        vrows = np.arange(0, Sv * w.Hq, 37)
        kbar_v = oracle.cube_pool(shv, K[:Sv])
        assert np.array_equal(kbar_v, kbar[:nv])
        m1, c1, _ = oracle.cube_select(sh, Q, kbar, p, rows=vrows)
        m2, c2, _ = oracle.cube_select(shv, Q[:Sv], kbar_v, p, rows=vrows)
        assert np.array_equal(unpack(m1, N)[:, :nv], unpack(m2, nv)) and not unpack(m1, N)[:, nv:].any()
        assert np.array_equal(c1, c2)
        o1, _ = oracle.sparse_attn(sh, Q, K, V, m1, rows=vrows)
        o2, _ = oracle.sparse_attn(shv, Q[:Sv], K[:Sv], V[:Sv], m2, rows=vrows)
        assert np.array_equal(o1, o2)


def test_attention_special_inputs(oracle):
    w = synth.TEST_WORKLOADS["T_mha64"]
    sh = shape_of(oracle, w)
    N = oracle.num_cubes(sh)
    Q, K, V = synth.generate(w)
    kbar = oracle.cube_pool(sh, K)
    mask, count, _ = oracle.cube_select(sh, Q, kbar, 0.7)
    # constant V -> constant output
    Vc = torch.full_like(V, -0.75)
    out, _ = oracle.sparse_attn(sh, Q, K, Vc, mask)
    np.testing.assert_allclose(out, -0.75, rtol=0, atol=1e-14)
    # V[n] = indicator of cube(n): output column j = attention mass on cube j
    bc, br, bs = brute_cube_table(w)
    assert N <= w.D
    Vi = torch.zeros_like(V)
    Vi[torch.arange(w.S), :, torch.from_numpy(bc)] = 1.0
    out, nk = oracle.sparse_attn(sh, Q, K, Vi, mask)
    sel = unpack(mask, N)
    own = np.zeros_like(sel)
    own[np.arange(w.S * w.Hq), np.repeat(bc, w.Hq)] = True
    attended = sel | own
    assert np.all(out[:, :N][~attended] == 0.0)
    assert np.all(out[:, :N][attended] > 0.0)
    np.testing.assert_allclose(out[:, :N].sum(1), 1.0, rtol=0, atol=1e-13)
    expect_keys = (sel * bs[None, :]).sum(1) + np.repeat(br + 1, w.Hq)
    assert np.array_equal(nk, expect_keys)
    # zero queries -> plain mean of the attended values
    Qz = torch.zeros_like(Q)
    out, _ = oracle.sparse_attn(sh, Qz, K, V, mask)
    Vd = widen(V)
    for r in (0, 37, w.S * w.Hq - 1):
        n, a = divmod(r, w.Hq)
        keys = np.nonzero((sel[r][bc] & (bc != bc[n])) | ((bc == bc[n]) & (br <= br[n])))[0]
        np.testing.assert_allclose(out[r], Vd[keys, a].mean(0), rtol=0, atol=1e-13)


def test_gqa_equals_mha_with_repeated_kv_heads(oracle):
    w = synth.TEST_WORKLOADS["T_ragged"]
    sh = shape_of(oracle, w)
    Q, K, V = synth.generate(w)
    G = w.Hq // w.Hkv
    sh_mha = oracle.Shape(w.T, w.H, w.W, w.ct, w.ch, w.cw, w.Hq, w.Hq, w.D)
    Kr, Vr = K.repeat_interleave(G, dim=1), V.repeat_interleave(G, dim=1)
    kbar, kbar_r = oracle.cube_pool(sh, K), oracle.cube_pool(sh_mha, Kr)
    np.testing.assert_array_equal(np.repeat(kbar, G, axis=1), kbar_r)
    m, c, _ = oracle.cube_select(sh, Q, kbar, 0.9)
    mr, cr, _ = oracle.cube_select(sh_mha, Q, kbar_r, 0.9)
    assert np.array_equal(m, mr) and np.array_equal(c, cr)
    o, _ = oracle.sparse_attn(sh, Q, K, V, m)
    orr, _ = oracle.sparse_attn(sh_mha, Q, Kr, Vr, mr)
    np.testing.assert_array_equal(o, orr)


def test_near_cut_flag_marks_rows_at_the_boundary(oracle):
    # two candidate cubes with equal mean keys -> equal logits -> flagged
    sh = oracle.Shape(3, 2, 2, 1, 2, 2, 1, 1, 64)
    K = torch.ones((sh.S, 1, 64), dtype=torch.bfloat16)
    Q = torch.ones((sh.S, 1, 64), dtype=torch.bfloat16)
    kbar = oracle.cube_pool(sh, K)
    _, count, near = oracle.cube_select(sh, Q, kbar, 0.6)
    assert count[-1] == 2 and near[-1]
    # a clearly separated row is not flagged
    K2 = K.clone()
    K2[:4] = 3.0
    kbar2 = oracle.cube_pool(sh, K2)
    _, count2, near2 = oracle.cube_select(sh, Q, kbar2, 0.6)
    assert count2[-1] == 1 and not near2[-1]


def test_group_shared_selection_reduces_to_per_head_selection(oracle):
    """The group-shared variant: with one query head per KV head the mean query is the query itself, so the variant
    is Eq. 2 unchanged; with the heads of every group made identical (groups of 2 and 4: halving and quartering are
    exact in float32 and bf16) it equals the per-head selection of that query, copied to the group; and rows of one
    group always share their set."""
    w = synth.TEST_WORKLOADS["T_mha64"]                       # 3 query heads, 3 KV heads
    sh = shape_of(oracle, w)
    Q, K, _ = synth.generate(w)
    kbar = oracle.cube_pool(sh, K)
    a, b = oracle.cube_select_shared(sh, Q, kbar, 0.7), oracle.cube_select(sh, Q, kbar, 0.7)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    for name in ("T_tiny", "T_text64"):                       # 4 query heads, 2 KV heads: groups of 2
        w = synth.TEST_WORKLOADS[name]
        sh = shape_of(oracle, w)
        Q, K, _ = synth.generate(w)
        kbar = oracle.cube_pool(sh, K)
        G = w.Hq // w.Hkv
        Qs = Q.clone()
        Qs[:, 1::2] = Qs[:, 0::2]                             # both heads of a group carry the first one's query
        m, c, _ = oracle.cube_select_shared(sh, Qs, kbar, 0.8)
        pm, pc, _ = oracle.cube_select(sh, Qs, kbar, 0.8)
        assert np.array_equal(m, pm) and np.array_equal(c, pc)
        m, c, _ = oracle.cube_select_shared(sh, Q, kbar, 0.8)
        m3 = m.reshape(w.S, w.Hkv, G, -1)
        assert (m3 == m3[:, :, :1]).all()
        # the mean of two bf16 values: exact in float32, then one rounding -- against exact rational arithmetic
        q = widen(Q).reshape(w.S, w.Hkv, G, w.D)
        mean = q.mean(axis=2)
        got = (oracle.group_mean_query(sh, Q).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        assert np.all(np.abs(got - mean) <= np.abs(mean) * 2.0 ** -8 + 1e-30)       # within half a bf16 step
    # the rounding itself against torch's own float32 -> bfloat16 conversion (round to nearest even), ties included
    x = np.concatenate([np.random.default_rng(1).standard_normal(4096).astype(np.float32),
                        np.array([1.00390625, 1.01171875, -1.00390625, 3.0e38, 1e-40, 0.0], np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.adaspark_oracle.bf16_round(x), want)


def test_noncausal_mode_against_library_softmax_and_brute_force(oracle):
    """causal = 0: (1) every cube selected = plain attention over all tokens, against scipy's softmax; (2) the dense
    non-causal entry likewise; (3) the selection takes all other video cubes as candidates: brute force per row on
    a tiny grid; text cubes other than the own one are always set; (4) the attended set of a row = selected cubes
    + its whole own cube (key counts)."""
    w = synth.TEST_WORKLOADS["T_tiny"]
    sh = shape_of(oracle, w)
    Q, K, V = synth.generate(w)
    q, k, v = widen(Q), widen(K), widen(V)
    G = w.Hq // w.Hkv
    N = oracle.num_cubes(sh)
    kbar = oracle.cube_pool(sh, K)
    full, cnt, _ = oracle.cube_select(sh, Q, kbar, 1.0, causal=False)
    assert (cnt == N - 1).all()
    out, nk = oracle.sparse_attn(sh, Q, K, V, full, causal=False)
    assert (nk == w.S).all()
    want = np.zeros_like(out)
    for n in range(w.S):
        for a in range(w.Hq):
            p = sp_softmax(k[:, a // G] @ q[n, a] / math.sqrt(w.D))
            want[n * w.Hq + a] = p @ v[:, a // G]
    np.testing.assert_allclose(out, want, rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(oracle.dense_attn(sh, Q, K, V, causal=False), want, rtol=1e-11, atol=1e-12)
    # brute-force selection
    bc, _, sizes = brute_cube_table(w)
    mask, count, _ = oracle.cube_select(sh, Q, kbar, 0.6, causal=False)
    for r in range(0, w.S * w.Hq, 7):
        n, a = divmod(r, w.Hq)
        own = bc[n]
        cand = [j for j in range(N) if j != own]
        logits = np.array([kbar[j, a // G] @ q[n, a] / math.sqrt(w.D) for j in cand])
        probs = sp_softmax(logits)
        order = sorted(range(len(cand)), key=lambda t: (-probs[t], t))
        kept, before = set(), 0.0
        for t in order:
            if before < 0.6:
                kept.add(cand[t])
            before += probs[t]
        got = {j for j in range(N) if (mask[r, j >> 5] >> (j & 31)) & 1}
        assert got == kept and count[r] == len(kept) and own not in got
    out2, nk2 = oracle.sparse_attn(sh, Q, K, V, mask, causal=False)
    for r in range(0, w.S * w.Hq, 11):
        own = bc[r // w.Hq]
        sel = [j for j in range(N) if (mask[r, j >> 5] >> (j & 31)) & 1]
        assert nk2[r] == sizes[own] + sum(sizes[j] for j in sel)
    # with text on both sides: every text cube except the own one is set, whatever p
    w = synth.TEST_WORKLOADS["T_lead64"]
    sh = shape_of(oracle, w)
    Q, K, _ = synth.generate(w)
    bc, _, _ = brute_cube_table(w)
    N = oracle.num_cubes(sh)
    full_c = w.ct * w.ch * w.cw
    Np, Nt = -(-w.lead // full_c), -(-w.text // full_c)
    mask, count, _ = oracle.cube_select(sh, Q, oracle.cube_pool(sh, K), 0.0, causal=False)
    text_cubes = list(range(Np)) + list(range(N - Nt, N))
    for r in range(0, w.S * w.Hq, 5):
        own = bc[r // w.Hq]
        got = {j for j in range(N) if (mask[r, j >> 5] >> (j & 31)) & 1}
        assert got == {j for j in text_cubes if j != own}
