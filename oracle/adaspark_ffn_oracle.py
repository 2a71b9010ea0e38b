"""fp64 oracle of the Adaptive Token-Selective FFN (AdaS-FFN, Sec. 3.3).

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Plain numpy in float64, one function per
equation, no blocking or fusion; it shares nothing with the GPU path.  Cube
membership (Sec. 3.1) comes from the C oracle's cube map.

Readings of the paper fixed here:
  * FFN(x) is the gated MLP of the Qwen2.5 backbone the paper builds on (Sec. 4,
    implementation details): W_down . (silu(W_gate x) * (W_up x)), no biases; the
    supplementary FLOP count speaks of a generic two-matrix FFN.
  * Top-p on the importance distribution S_i (Eq. 5) is the rule of Eq. 2: rank the
    tokens of the cube by s_j descending (ties: lower rank inside the cube first)
    and keep a token iff the mass of the tokens ranked before it is below p;
    p >= 1 keeps every token, p = 0 none.
  * A cube with no activated token (p = 0) has no mean transformation: its tokens
    keep their value (m-bar = 0).
  * Text tokens all take the dense FFN (last paragraph of Sec. 3.3).
  * Eq. 4 with a zero denominator (every token of the cube has norm 0 and eps = 0): all
    scores are 0.
"""
from __future__ import annotations

import numpy as np

from . import adaspark_oracle as base


def widen(x_bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly."""
    return (x_bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def token_norms(X: np.ndarray) -> np.ndarray:
    """||x_j||_2 of every token; X float64 [S, d_model]  (numerator of Eq. 4)."""
    return np.sqrt((X * X).sum(axis=1))


def importance(norms: np.ndarray, eps: float) -> np.ndarray:
    """s_j = ||x_j|| / (sum_k ||x_k|| + eps) over the tokens of ONE cube  (Eq. 4).  The epsilon is there for a cube
    whose tokens all have zero norm; with eps = 0 as well the quotient 0/0 is read as 0: such a cube has no
    importance to hand out, every score is 0, and the Top-p rule then keeps every token for p > 0 (nothing is
    ranked before anybody with positive mass) and none for p = 0."""
    total = norms.sum() + eps
    if total == 0.0:
        return np.zeros_like(norms)
    return norms / total


def top_p_tokens(s: np.ndarray, p: float):
    """Eq. 5 on one cube's distribution -> (keep[n] bool, order[n], mass_before[n] in ranked order)."""
    n = s.size
    order = np.array(sorted(range(n), key=lambda j: (-s[j], j)), dtype=np.int64)
    before = np.concatenate([[0.0], np.cumsum(s[order])[:-1]]) if n else np.zeros(0)
    keep = np.zeros(n, bool)
    keep[order] = True if p >= 1.0 else (before < p)
    return keep, order, before


def cube_members(shape: base.Shape):
    """List, per cube, of its token indices in rank order, and the flag 'is a text cube'."""
    cube_of, rank_of, size_of, _ = base.cube_map(shape)
    N = size_of.size
    members = [np.zeros(int(size_of[i]), np.int64) for i in range(N)]
    for n in range(shape.S):
        members[cube_of[n]][rank_of[n]] = n
    video = shape.T * shape.H * shape.W
    is_text = [bool(len(m)) and not (shape.lead <= m[0] < shape.lead + video) for m in members]
    return members, is_text


def ffn_select(shape: base.Shape, X: np.ndarray, p: float, eps: float = 1e-6, near: float = 1e-5):
    """Activated-token mask of Eq. 5 for every cube.

    X float64 [S, d_model].  Returns (keep uint8 [S], score float64 [S], near_cut uint8 [cubes]).
    Text tokens are always kept.  near_cut[i] = 1 iff the decision in cube i sits within `near`
    of the boundary (mass before the last kept or the first dropped token within `near` of p, or
    their scores closer than `near` relative): there a float32 implementation may legitimately
    differ; the flag does not influence the selection.
    """
    members, is_text = cube_members(shape)
    norms = token_norms(X)
    keep = np.zeros(shape.S, np.uint8)
    score = np.zeros(shape.S, np.float64)
    near_cut = np.zeros(len(members), np.uint8)
    for i, m in enumerate(members):
        if len(m) == 0:
            continue
        s = importance(norms[m], eps)
        score[m] = s
        if is_text[i]:
            keep[m] = 1
            continue
        k, order, before = top_p_tokens(s, p)
        keep[m] = k
        kept = int(k.sum())
        if 0.0 < p < 1.0 and 0 < kept:
            flag = abs(before[kept - 1] - p) < near
            if kept < len(m):
                flag |= abs(before[kept] - p) < near
                a, b = s[order[kept - 1]], s[order[kept]]
                flag |= (a - b) < near * max(a, 1e-300)
            near_cut[i] = flag
    return keep, score, near_cut


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def ffn(X: np.ndarray, Wg: np.ndarray, Wu: np.ndarray, Wd: np.ndarray) -> np.ndarray:
    """Gated MLP on rows of X: [n, d_model] -> [n, d_model]; Wg, Wu [d_ff, d_model], Wd [d_model, d_ff]."""
    return (silu(X @ Wg.T) * (X @ Wu.T)) @ Wd.T


def ffn_sparse(shape: base.Shape, X: np.ndarray, Wg, Wu, Wd, keep: np.ndarray) -> np.ndarray:
    """Eqs. 6-7: y = x + FFN(x) on kept tokens, y = x + mean of the cube's kept FFN(x) on the others."""
    members, _ = cube_members(shape)
    Y = X.copy()
    for m in members:
        if len(m) == 0:
            continue
        act = m[keep[m] != 0]
        rest = m[keep[m] == 0]
        if len(act) == 0:
            continue
        F = ffn(X[act], Wg, Wu, Wd)
        Y[act] = X[act] + F
        Y[rest] = X[rest] + F.mean(axis=0)
    return Y


def ffn_dense(X: np.ndarray, Wg, Wu, Wd) -> np.ndarray:
    """The standard layer every token of which takes the FFN: y = x + FFN(x)."""
    return X + ffn(X, Wg, Wu, Wd)
