"""Seeded synthetic workloads (shapes and value distributions only).

This module serves both the HIP path and the CPU oracle and therefore holds
none of the method's arithmetic: no pooling, scoring, selection or attention,
and no token->cube index function.  The per-cube key mean is laid onto the
token grid by repeating a [cubes_t, cubes_h, cubes_w] field along each axis and
cropping it to the grid.

All tensors are drawn in fp32 on the CPU with ``torch.Generator`` and rounded to
bf16 once; the bf16 buffers are the single source of truth for both sides.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Tuple

import torch

BASE_SEED = 20260408


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    T: int
    H: int
    W: int
    ct: int
    ch: int
    cw: int
    Hq: int
    Hkv: int
    D: int
    top_p: Tuple[float, ...]
    # scale of the per-cube key mean, one entry per KV head
    k_mean_scale: Tuple[float, ...]
    # text tokens appended after the video tokens (no per-cube key mean: plain noise keys)
    text: int = 0
    # text tokens placed before the video tokens (the same)
    lead: int = 0

    @property
    def S(self) -> int:
        return self.lead + self.T * self.H * self.W + self.text

    @property
    def S_video(self) -> int:
        return self.T * self.H * self.W

    @property
    def grid(self):
        return (self.T, self.H, self.W)

    @property
    def cube(self):
        return (self.ct, self.ch, self.cw)


def _wl(name, cid, grid, cube, hq, hkv, d, top_p, scale, text=0, lead=0):
    if not isinstance(scale, tuple):
        scale = (float(scale),) * hkv
    if not isinstance(top_p, tuple):
        top_p = (float(top_p),)
    return Workload(name, cid, *grid, *cube, hq, hkv, d, top_p, scale, text, lead)


# The five benchmark configurations (token grid, cube, heads, head_dim, Top-p).
WORKLOADS = {
    "C1": _wl("C1", 1, (8, 16, 16), (2, 4, 4), 4, 4, 64, 0.9, 0.0),
    "C2": _wl("C2", 2, (64, 16, 16), (4, 8, 8), 28, 4, 128, 0.9, 1.0),
    "C3": _wl("C3", 3, (256, 16, 16), (4, 8, 8), 28, 4, 128, (0.5, 0.7, 0.9, 0.99), 1.0),
    "C4": _wl("C4", 4, (1024, 16, 16), (4, 8, 8), 28, 4, 128, 0.9, 0.5),
    # entropy stress: KV heads 0-3 flat scores, 4-7 sharply peaked scores
    "C5": _wl("C5", 5, (100, 15, 20), (4, 8, 8), 32, 8, 128, 0.9, (0.0,) * 4 + (4.0,) * 4),
}

# Small cases for tests: ragged in every axis, GQA, both head dims.
TEST_WORKLOADS = {
    "T_tiny": _wl("T_tiny", 11, (3, 5, 6), (2, 2, 4), 4, 2, 64, 0.8, 1.0),
    "T_ragged": _wl("T_ragged", 12, (9, 10, 12), (4, 4, 8), 6, 2, 128, 0.9, (0.0, 2.0)),
    "T_mha64": _wl("T_mha64", 13, (6, 8, 8), (2, 4, 4), 3, 3, 64, 0.7, 0.5),
    "T_gqa128": _wl("T_gqa128", 14, (12, 16, 16), (4, 8, 8), 14, 2, 128, 0.9, 1.0),
    "T_manycubes": _wl("T_manycubes", 15, (40, 4, 4), (1, 2, 2), 4, 2, 64, 0.6, 1.0),
    # more than 256 and more than 1024 cubes: a row's candidate cubes are spread over several wavefronts
    "T_cubes280": _wl("T_cubes280", 16, (70, 4, 4), (1, 2, 2), 4, 2, 64, 0.7, 1.0),
    "T_cubes1100": _wl("T_cubes1100", 17, (275, 4, 4), (1, 2, 2), 2, 1, 128, 0.8, 0.5),
    # video followed by text tokens: 100 = three full text cubes of 32 and one of 4; 37 = a single short text cube
    "T_text64": _wl("T_text64", 18, (6, 8, 8), (2, 4, 4), 4, 2, 64, 0.8, 1.0, text=100),
    "T_text128": _wl("T_text128", 19, (5, 10, 12), (4, 4, 8), 6, 2, 128, 0.9, (0.0, 2.0), text=37),
    # text on both sides of the video: 70 leading tokens (two full text cubes and one of 6), 45 trailing
    "T_lead64": _wl("T_lead64", 21, (6, 8, 8), (2, 4, 4), 4, 2, 64, 0.8, 1.0, text=45, lead=70),
    # two cubes of 2,048 tokens: 32 key tiles per cube, several key blocks per cube in the key-stationary kernels
    "T_cube2048": _wl("T_cube2048", 25, (8, 16, 32), (4, 16, 32), 2, 1, 64, 0.9, 1.0),
    # a short leading prompt only (a single text cube of 50), ragged video grid, D 128
    "T_lead128": _wl("T_lead128", 22, (5, 10, 12), (4, 4, 8), 6, 2, 128, 0.9, (0.0, 2.0), lead=50),
}

# Mid-sized cases, checked on sampled rows only.
SAMPLED_WORKLOADS = {
    # a 16,384-token video with a 1,000-token prompt after it: 64 video cubes, 4 text cubes
    "M_text16k": _wl("M_text16k", 20, (64, 16, 16), (4, 8, 8), 28, 4, 128, 0.9, 1.0, text=1000),
    # a 300-token system prompt, an 8,192-token video, a 500-token question
    "M_lead8k": _wl("M_lead8k", 23, (32, 16, 16), (4, 8, 8), 28, 4, 128, 0.9, 1.0, text=500, lead=300),
    # a slice of the quarter-million-token geometry: 300 cubes of 256 tokens (more than one wavefront's 256 candidate
    # cubes per row), the same heads and key statistics; small enough for every sparse kernel's scratch to fit a test
    "M_c4slice": _wl("M_c4slice", 26, (300, 16, 16), (4, 8, 8), 28, 4, 128, 0.5, 0.5),
    # 256-token cubes (four key tiles each, the last cube half as long), a GQA group of seven: small enough for the
    # backward oracle to take every row
    "M_bwd256": _wl("M_bwd256", 24, (6, 16, 16), (4, 8, 8), 7, 1, 128, 0.8, 1.0),
}


def _randn(shape, seed):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32)


def generate(w: Workload, query_corr: float = 0.0):
    """-> (Q [S,Hq,D], K [S,Hkv,D], V [S,Hkv,D]) CPU bf16 tensors.

    Q, V ~ N(0,1).  K = N(0,1) + scale[g] * mu, mu ~ N(0, I) drawn once per
    (cube, KV head) and shared by all tokens of that cube.  Text tokens (the first
    ``w.lead`` and the last ``w.text`` rows) have plain N(0,1) keys.

    ``query_corr`` = rho > 0 (a variant, not one of the listed configurations): the
    queries of the video tokens of a cube share a component per query head,
    q = sqrt(1 - rho^2) * N(0,1) + rho * c[cube, head], still of unit variance, the way
    neighbouring video tokens resemble each other; rho = 0 is the listed recipe.
    """
    seed = BASE_SEED + 1000 * w.config_id
    S, Sv = w.S, w.S_video
    Q = _randn((S, w.Hq, w.D), seed + 0)
    if query_corr > 0.0:
        nt, nh, nw = -(-w.T // w.ct), -(-w.H // w.ch), -(-w.W // w.cw)
        c = _randn((nt, nh, nw, w.Hq, w.D), seed + 4)
        field = c.repeat_interleave(w.ct, 0).repeat_interleave(w.ch, 1).repeat_interleave(w.cw, 2)
        field = field[: w.T, : w.H, : w.W].reshape(Sv, w.Hq, w.D)
        Q[w.lead : w.lead + Sv] = (1.0 - query_corr ** 2) ** 0.5 * Q[w.lead : w.lead + Sv] + query_corr * field
    Q = Q.to(torch.bfloat16)
    V = _randn((S, w.Hkv, w.D), seed + 2).to(torch.bfloat16)
    K = _randn((S, w.Hkv, w.D), seed + 1)
    if any(s != 0.0 for s in w.k_mean_scale):
        nt, nh, nw = -(-w.T // w.ct), -(-w.H // w.ch), -(-w.W // w.cw)
        mu = _randn((nt, nh, nw, w.Hkv, w.D), seed + 3)
        mu = mu * torch.tensor(w.k_mean_scale, dtype=torch.float32).view(1, 1, 1, w.Hkv, 1)
        field = mu.repeat_interleave(w.ct, 0).repeat_interleave(w.ch, 1).repeat_interleave(w.cw, 2)
        field = field[: w.T, : w.H, : w.W].reshape(Sv, w.Hkv, w.D)
        K[w.lead : w.lead + Sv] = K[w.lead : w.lead + Sv] + field
    return Q, K.to(torch.bfloat16), V


def generate_ffn(w: Workload, d_model: int, d_ff: int, norm_sigma: float = 0.6):
    """-> (X [S,d_model], W_gate [d_ff,d_model], W_up [d_ff,d_model], W_down [d_model,d_ff]) CPU bf16 tensors.

    Token embeddings are N(0,1) vectors, each multiplied by its own log-normal factor exp(norm_sigma * N(0,1)), so
    that token norms inside a cube are spread like a layer's hidden states rather than all alike; weights are
    N(0, 1/fan_in) like a freshly initialised layer.
    """
    seed = BASE_SEED + 1000 * w.config_id + 500
    X = _randn((w.S, d_model), seed + 0) * torch.exp(norm_sigma * _randn((w.S, 1), seed + 1))
    Wg = _randn((d_ff, d_model), seed + 2) * d_model ** -0.5
    Wu = _randn((d_ff, d_model), seed + 3) * d_model ** -0.5
    Wd = _randn((d_model, d_ff), seed + 4) * d_ff ** -0.5
    return tuple(t.to(torch.bfloat16) for t in (X, Wg, Wu, Wd))


def sample_rows(w: Workload, n: int, seed: int = 7):
    """A seeded sample of query row ids (row = token * Hq + head), sorted.

    Always contains the first and last token's rows so that both ends of the
    sequence are covered; the rest is uniform without replacement.  With text
    tokens, an eighth as many rows again are drawn from the text rows alone.
    """
    R = w.S * w.Hq
    g = torch.Generator(device="cpu")
    g.manual_seed(BASE_SEED + 77 * w.config_id + seed)
    n = min(n, R)
    picks = torch.randperm(R, generator=g)[:n]
    fixed = torch.tensor([0, w.Hq - 1, R - w.Hq, R - 1], dtype=torch.int64)
    parts = [picks, fixed]
    if w.text:
        first = (w.lead + w.S_video) * w.Hq
        parts.append(first + torch.randperm(R - first, generator=g)[: max(8, n // 8)])
        parts.append(torch.tensor([first, first + w.Hq - 1], dtype=torch.int64))
    if w.lead:
        end = w.lead * w.Hq
        parts.append(torch.randperm(end, generator=g)[: max(8, n // 8)])
        parts.append(torch.tensor([end - 1, end, end + w.Hq - 1], dtype=torch.int64))
    rows = torch.unique(torch.cat(parts))
    return rows.numpy()
