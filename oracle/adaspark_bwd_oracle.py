"""fp64 oracle of the backward pass of cube-selective attention (Eq. 3 differentiated, selection held constant).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Plain numpy in float64, one query row at a time, no blocking or fusion; it
shares nothing with the GPU path.  The paper trains through the operator (supplementary material, "AdaSpark
Training Algorithm") and states no gradient of its own: the gradient here is the textbook derivative of softmax
attention restricted to each row's attended keys, with the selected set S_r treated as a constant (the Top-p rule is
piecewise constant in Q and K, so its derivative is zero wherever it exists).

For row r = (token n, head a) with attended keys A_r (tokens of the selected cubes, and the tokens of the own cube
up to n's rank), scale c = 1/sqrt(D), KV head g = a / (Hq / Hkv):
    s_j = c q.k_j,  p = softmax(s),  o = sum_j p_j v_j                      (forward, Eq. 3)
    dv_j += p_j do,  dp_j = do.v_j,  delta = do.o,  ds_j = p_j (dp_j - delta),
    dq = c sum_j ds_j k_j,  dk_j += c ds_j q                                  (backward)
"""
from __future__ import annotations

import numpy as np

from . import adaspark_oracle as base


def attended_tokens(shape: base.Shape, sel_mask_row: np.ndarray, token: int, tables):
    """Token indices row attends, in cube-major order: selected cubes in full, then the own cube up to the row's rank."""
    cube_of, rank_of, members = tables
    own = cube_of[token]
    parts = [members[j] for j in range(own) if (sel_mask_row[j >> 5] >> (j & 31)) & 1]
    parts.append(members[own][: rank_of[token] + 1])
    return np.concatenate(parts)


def cube_tables(shape: base.Shape):
    cube_of, rank_of, size_of, _ = base.cube_map(shape)
    members = [np.zeros(int(n), np.int64) for n in size_of]
    for n in range(shape.S):
        members[cube_of[n]][rank_of[n]] = n
    return cube_of, rank_of, members


def forward_row(q, Ka, Va, D):
    """Eq. 3 for one row on its attended keys -> (o, p)."""
    s = (Ka @ q) / np.sqrt(D)
    e = np.exp(s - s.max())
    p = e / e.sum()
    return p @ Va, p


def lse_rows(shape: base.Shape, Q, K, sel_mask, rows):
    """Natural-log sum-exp of Eq. 3's scaled scores over each row's attended keys, and next to it the largest
    sum_d |q_d k_d| / sqrt(D) among those keys: the size of a score's products, which bounds how far a relative
    perturbation of q's elements can move any score of the row -- and hence the log-sum-exp, a weighted mean of the
    scores' movements.  Q [S,Hq,D], K [S,Hkv,D] float64; sel_mask the rows' mask words.  -> (lse, absdot), [nrows]."""
    tables = cube_tables(shape)
    G = shape.Hq // shape.Hkv
    lse, absdot = np.zeros(len(rows)), np.zeros(len(rows))
    for x, r in enumerate(rows):
        n, a = divmod(int(r), shape.Hq)
        Ka = K[attended_tokens(shape, sel_mask[x], n, tables), a // G]
        s = (Ka @ Q[n, a]) / np.sqrt(shape.D)
        lse[x] = s.max() + np.log(np.exp(s - s.max()).sum())
        absdot[x] = (np.abs(Ka) @ np.abs(Q[n, a])).max() / np.sqrt(shape.D)
    return lse, absdot


def sparse_attn_fwd(shape: base.Shape, Q, K, V, sel_mask, rows=None):
    """Forward in numpy on float64 inputs Q [S,Hq,D], K, V [S,Hkv,D] -> O [nrows, D] (rows: row ids n*Hq + a)."""
    tables = cube_tables(shape)
    G = shape.Hq // shape.Hkv
    rows = np.arange(shape.S * shape.Hq) if rows is None else np.asarray(rows)
    out = np.zeros((rows.size, shape.D))
    for x, r in enumerate(rows):
        n, a = divmod(int(r), shape.Hq)
        att = attended_tokens(shape, sel_mask[x], n, tables)
        out[x], _ = forward_row(Q[n, a], K[att, a // G], V[att, a // G], shape.D)
    return out


def row_backward(shape: base.Shape, Q, K, V, sel_mask_row, r: int, do, o_given, tables):
    """One query row r = n*Hq + a.  -> (att, dq, dk_terms [len(att), D], dv_terms [len(att), D], delta, ds, p):
    the tokens it attends, its dQ row, and what it adds to dK and dV of those tokens."""
    G, D = shape.Hq // shape.Hkv, shape.D
    c = 1.0 / np.sqrt(D)
    n, a = divmod(int(r), shape.Hq)
    g = a // G
    att = attended_tokens(shape, sel_mask_row, n, tables)
    Ka, Va = K[att, g], V[att, g]
    o, p = forward_row(Q[n, a], Ka, Va, D)
    delta = do @ (o if o_given is None else o_given)
    ds = p * (Va @ do - delta)
    return att, c * (ds @ Ka), c * np.outer(ds, Q[n, a]), np.outer(p, do), delta, ds, p


def delta_error_bound(do, o, p, Va, absdot):
    """Tolerance model, not part of the gradient: how far delta = do.O can lie from the exact do.o when O comes from a
    forward that rounds every probability and the output to bf16 and whose scores carry a relative perturbation of
    2^-12 in every product q_d k_d -- a query operand rounded to fp16 -- (`absdot`: the row's largest
    sum_d |q_d k_d| / sqrt(D)).  Element d of such an O is a sum of terms p_j v_jd, each off by about
    2^-9 (1 + absdot / 8) of itself, independently: about seven standard deviations of that,
    2^-7 (1 + absdot / 8) sqrt(sum_j p_j^2 v_jd^2), plus the output's own rounding 2^-8 |o_d|; the elements' bounds are
    added up with the weights |do_d|."""
    t_o = np.sqrt((p * p) @ (Va * Va))
    return float(np.abs(do) @ (2.0 ** -8 * np.abs(o) + 2.0 ** -7 * (1.0 + absdot / 8.0) * t_o))


def sparse_attn_bwd(shape: base.Shape, Q, K, V, sel_mask, dO, O=None, scales=None):
    """All rows.  Q [S,Hq,D], K, V [S,Hkv,D], dO [S*Hq, D] float64; sel_mask uint32 [S*Hq, words].
    O (optional, [S*Hq, D]): the forward output as the caller stored it; delta = dO.O is then taken from it, as an
    implementation that is handed a rounded O does, instead of from the exact o recomputed here.
    scales (optional dict): filled with diagnostics for tolerances; they do not influence the gradients.
      'dQ', 'dK', 'dV': arrays of the gradients' shapes holding, per element, the root of the sum of squares of the
      terms that add up to it -- the natural unit for the error of an implementation that rounds every term;
      'dQ_delta', 'dK_delta': per element, how far it can move when every row's delta is off by up to that row's
      delta_error_bound: dQ[r] depends on delta_r through -c delta_r sum_j p_j k_j, dK_j through -c p_j delta_r q
      (dV does not depend on delta); the rows' contributions to a dK element are added in absolute value.
    -> (dQ [S,Hq,D], dK [S,Hkv,D], dV [S,Hkv,D], delta [S*Hq])."""
    tables = cube_tables(shape)
    G, D = shape.Hq // shape.Hkv, shape.D
    c = 1.0 / np.sqrt(D)
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    delta = np.zeros(shape.S * shape.Hq)
    if scales is not None:
        scales.update(dQ=np.zeros_like(Q), dK=np.zeros_like(K), dV=np.zeros_like(V),
                      dQ_delta=np.zeros_like(Q), dK_delta=np.zeros_like(K))
    for r in range(shape.S * shape.Hq):
        n, a = divmod(r, shape.Hq)
        g = a // G
        att, dq, dk_terms, dv_terms, delta[r], ds, p = row_backward(
            shape, Q, K, V, sel_mask[r], r, dO[r], None if O is None else O[r], tables)
        dQ[n, a] = dq
        dK[att, g] += dk_terms   # a row's attended tokens are distinct
        dV[att, g] += dv_terms
        if scales is not None:
            Ka, Va = K[att, g], V[att, g]
            scales["dQ"][n, a] = c * np.sqrt((ds * ds) @ (Ka * Ka))
            scales["dK"][att, g] += dk_terms ** 2
            scales["dV"][att, g] += dv_terms ** 2
            absdot = (np.abs(Ka) @ np.abs(Q[n, a])).max() * c
            derr = delta_error_bound(dO[r], p @ Va, p, Va, absdot)
            scales["dQ_delta"][n, a] = c * derr * np.abs(p @ Ka)
            scales["dK_delta"][att, g] += c * derr * np.outer(p, np.abs(Q[n, a]))
    if scales is not None:
        scales["dK"], scales["dV"] = np.sqrt(scales["dK"]), np.sqrt(scales["dV"])
    return dQ, dK, dV, delta
