#!/usr/bin/env python3
"""Benchmark of the AdaS-Attn hot path on one MI355X.

A "step" is one pass of the whole path over one synthetic batch already resident
in HBM: cube mean-pool -> relevance scoring + Top-p selection -> KV pack ->
sparse attention.  The default workload is the 64K-token configuration the
headline metric is quoted on (256 frames x 16x16 tokens, cube 4x8x8, 28 query /
4 KV heads, head_dim 128, Top-p 0.9).

Prints ONE JSON line (see the field list in main()).  Besides the contract
fields it carries
  roofline     -- the dominant kernel (sparse attention) against bf16 MFMA peak:
                  algorithmic FLOPs = 4 * head_dim * (attended keys summed over
                  all query rows, from the selection actually produced) divided
                  by the kernel's mean duration, timed with HIP events on the
                  stream the kernels are launched on;
  cpu_baseline -- the fp64 oracle timed on this machine's host cores on a bounded
                  sample of the same workload (a reported baseline, not a target).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2604_08077_amd import synth  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# HBM traffic of one sparse-attention launch (bytes), from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# scaled by a copy kernel of known size; keyed by (workload, top_p).  See profiles/.
# (C3, 0.9): attn_walk_kernel<128, true>; (C3, 0.5): the key-stationary kernels together (pairs, own cubes, merge).
MEASURED_TRAFFIC_BYTES = {("C3", 0.9): 5.235e9, ("C3", 0.5): 3.767e10}


def cube_tables(w):
    """Host-side sizes of all cubes and rank of every token (measurement bookkeeping only)."""
    t, h, x = np.meshgrid(np.arange(w.T), np.arange(w.H), np.arange(w.W), indexing="ij")
    nH, nW = -(-w.H // w.ch), -(-w.W // w.cw)
    tb, hb, wb = t // w.ct, h // w.ch, x // w.cw
    cube = ((tb * nH + hb) * nW + wb).reshape(-1)
    eh = np.minimum(w.ch, w.H - hb * w.ch)
    ew = np.minimum(w.cw, w.W - wb * w.cw)
    rank = (((t - tb * w.ct) * eh + (h - hb * w.ch)) * ew + (x - wb * w.cw)).reshape(-1)
    sizes = np.bincount(cube)
    return cube, rank, sizes


def attended_keys_total(w, mask, sizes, rank):
    """Sum over all query rows of the number of attended keys, from the GPU's own selection mask."""
    R, words = mask.shape
    shifts = torch.arange(32, device=mask.device, dtype=torch.int32).view(1, 1, 32)
    colsum = torch.zeros(words * 32, dtype=torch.int64, device=mask.device)
    chunk = max(1, (1 << 25) // (words * 32))
    for r0 in range(0, R, chunk):
        bits = (mask[r0:r0 + chunk].unsqueeze(-1) >> shifts) & 1
        colsum += bits.sum(dim=0, dtype=torch.int64).reshape(-1)
    colsum = colsum[: len(sizes)].cpu().numpy()
    selected_keys = int((colsum * sizes.astype(np.int64)).sum())
    own_keys = int((rank.astype(np.int64) + 1).sum()) * w.Hq
    return selected_keys + own_keys, int(colsum.sum())


def timed(fn, n):
    """Mean duration in ms of fn() over n launches, HIP events on the current stream."""
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(n):
        fn()
    ev1.record()
    ev1.synchronize()
    return ev0.elapsed_time(ev1) / n


def measured_ceilings(B):
    """What this GPU sustains, from the library's two probes (outside every timed region): a plain 1 GiB streaming
    copy (bytes read + written per second) and back-to-back bf16 MFMAs on every SIMD.  The roofline fractions are
    given against the datasheet peaks and, as *_measured, against these."""
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    src.zero_()
    B.probe_copy(dst, src)
    moved = [0]

    def copy():
        moved[0] = B.probe_copy(dst, src)

    copy_ms = timed(copy, 5)
    del src, dst
    out = torch.empty(1024, dtype=torch.float32, device="cuda")
    flops = [0.0]

    def mfma():
        flops[0] = B.probe_mfma(out, 1024, 8192)

    mfma()
    mfma_ms = timed(mfma, 3)
    torch.cuda.empty_cache()
    return {"copy_gbs": moved[0] / (copy_ms * 1e-3) / 1e9, "mfma_bf16_tflops": flops[0] / (mfma_ms * 1e-3) / 1e12}


def cpu_baseline(w, p, Q, K, V, budget_rows_sel=262144, budget_rows_attn=24576):
    """The fp64 oracle on a bounded row sample of the same workload, extrapolated to tokens/s."""
    import oracle

    osh = oracle.Shape(w.T, w.H, w.W, w.ct, w.ch, w.cw, w.Hq, w.Hkv, w.D, w.text, w.lead)
    R = w.S * w.Hq
    t0 = time.perf_counter()
    kbar = oracle.cube_pool(osh, K)
    t_pool = time.perf_counter() - t0
    rows_sel = synth.sample_rows(w, budget_rows_sel, seed=101)
    t0 = time.perf_counter()
    mask, _, _ = oracle.cube_select(osh, Q, kbar, p, rows=rows_sel)
    t_sel = time.perf_counter() - t0
    rows_att = synth.sample_rows(w, budget_rows_attn, seed=102)
    mask_att, _, _ = oracle.cube_select(osh, Q, kbar, p, rows=rows_att)
    t0 = time.perf_counter()
    oracle.sparse_attn(osh, Q, K, V, mask_att, rows=rows_att)
    t_att = time.perf_counter() - t0
    total = t_pool + t_sel / len(rows_sel) * R + t_att / len(rows_att) * R
    return {
        "value": w.S / total,
        "unit": "tokens/s",
        "cores": oracle.num_threads(),
        "kind": "oracle",
        "sample": (f"pool on all {w.S} tokens ({t_pool:.2f}s) + select on {len(rows_sel)} of {R} rows ({t_sel:.2f}s) "
                   f"+ attention on {len(rows_att)} of {R} rows ({t_att:.2f}s), uniform seeded row samples, "
                   f"per-row cost scaled to all rows"),
    }


# Widths of the token-selective FFN leg: the 7B backbone the 28-head attention configurations correspond to
# (28 heads x 128 = 3584 model width, 18944 hidden width).
FFN_D_MODEL, FFN_D_FF, FFN_TOP_P = 3584, 18944, 0.7
# Bytes the two matrix-product kernels of one adaspark_ffn_sparse call move between the L2 caches and the fabric
# (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy of known size; see profiles/), keyed by workload.
FFN_MEASURED_TRAFFIC_BYTES = {"C3": 2.237e10}


def ffn_leg(B, w, steps, dense=True):
    """AdaS-FFN (Sec. 3.3) on the same token grid: selection + sparse layer at the paper's default p = 0.7, timed
    with HIP events on the launch stream; the dense layer (every token activated) beside it."""
    sh = B.Shape.of(w)
    X, Wg, Wu, Wd = (t.cuda() for t in synth.generate_ffn(w, FFN_D_MODEL, FFN_D_FF))
    ws = torch.empty(B.ffn_workspace_bytes(sh, FFN_D_MODEL, FFN_D_FF), dtype=torch.uint8, device="cuda")
    Y = torch.empty_like(X)
    keep, _, _ = B.ffn_select(sh, X, FFN_D_FF, FFN_TOP_P)
    share = float(keep.float().mean().item())
    B.ffn_sparse(sh, X, Wg, Wu, Wd, keep=keep, Y=Y, workspace=ws)  # untimed first launch
    t_sel = timed(lambda: B.ffn_select(sh, X, FFN_D_FF, FFN_TOP_P), steps)
    t_sparse = timed(lambda: B.ffn_sparse(sh, X, Wg, Wu, Wd, keep=keep, Y=Y, workspace=ws), steps)
    t_dense = timed(lambda: B.ffn_sparse(sh, X, Wg, Wu, Wd, keep=None, Y=Y, workspace=ws), max(2, steps // 3)) if dense else None
    flops = 6.0 * share * w.S * FFN_D_MODEL * FFN_D_FF  # three matrix products on the activated tokens
    tf = flops / (t_sparse * 1e-3) / 1e12
    return {
        "workload": f"{w.name} token grid, d_model {FFN_D_MODEL}, d_ff {FFN_D_FF}, gated MLP, top_p {FFN_TOP_P}, "
                    "synthetic bf16 embeddings with log-normal norms",
        "tokens_per_s": w.S / ((t_sel + t_sparse) * 1e-3),
        "activated_share": share,
        "ms": {"ffn_select": t_sel, "ffn_sparse": t_sparse, "ffn_dense": t_dense},
        "speedup_vs_dense": None if t_dense is None else t_dense / (t_sel + t_sparse),
        "roofline": {"kernel": "ffn_gemm_kernel<true> + ffn_gemm_kernel<false> (whole adaspark_ffn_sparse call)",
                     "bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": tf / PEAK_BF16_TFLOPS, "traffic": FFN_MEASURED_TRAFFIC_BYTES.get(w.name)},
        "dense_tflops": None if t_dense is None else 6.0 * w.S * FFN_D_MODEL * FFN_D_FF / (t_dense * 1e-3) / 1e12,
        "select_hbm_gbs": w.S * FFN_D_MODEL * 2 / (t_sel * 1e-3) / 1e9,
    }


# Bytes the three backward kernels of one call move between the L2 caches and the fabric (rocprofv3 --pmc FETCH_SIZE /
# WRITE_SIZE, scaled by a copy of known size; see profiles/), keyed by (workload, top_p).
BWD_MEASURED_TRAFFIC_BYTES = {("C3", 0.9): 4.58e10}


def bwd_leg(B, w, sh, Qg, Kg, Vg, ws_att, mask, eff_flops, dense_flops, steps, top_p):
    """Backward of the sparse attention (selection constant) on the headline inputs: O and the log-sum-exp from the
    library's forward, a seeded dO; the whole adaspark_sparse_attn_bwd call timed with HIP events."""
    O, lse = B.sparse_attn_packed(sh, Qg, ws_att, mask, return_lse=True)
    g = torch.Generator(device="cpu")
    g.manual_seed(synth.BASE_SEED + 31 * w.config_id)
    dO = torch.randn((w.S, w.Hq, w.D), generator=g, dtype=torch.float32).to(torch.bfloat16).cuda()
    ws = B.alloc_workspace(sh, B.CALL_ATTN_BWD)
    B.sparse_attn_bwd(sh, Qg, Kg, Vg, O, lse, dO, sel_mask=mask, workspace=ws)  # untimed first launch
    ms = timed(lambda: B.sparse_attn_bwd(sh, Qg, Kg, Vg, O, lse, dO, sel_mask=mask, workspace=ws), max(2, steps // 2))
    # five matrix products on the attended keys against the forward's two; the kernels execute eight on every
    # preceding cube (S three times, dP twice, dV, dK, dQ), with the selection as a mask
    tf = 2.5 * eff_flops / (ms * 1e-3) / 1e12
    return {
        "ms": ms,
        "roofline": {"kernel": "attn_bwd_dq_kernel + attn_bwd_dkv_kernel<dV> + attn_bwd_dkv_kernel<dK> (whole call)",
                     "bound": "mfma", "achieved": tf, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": tf / PEAK_BF16_TFLOPS, "traffic": BWD_MEASURED_TRAFFIC_BYTES.get((w.name, top_p)),
                     "executed_tflops": 4.0 * dense_flops / (ms * 1e-3) / 1e12},
    }


def workload_line(B, w, steps, query_corr=0.0, top_p=None):
    """One of the configuration's other workloads at its first Top-p value (or top_p), measured like the headline
    step (pool + select + pack + sparse attention, host clock; dense entry beside it) but reported in a few figures
    only.  query_corr > 0: synth.generate's variant with queries that neighbouring tokens share."""
    p = float(np.float32(w.top_p[0] if top_p is None else top_p))
    sh = B.Shape.of(w)
    N = B.num_cubes(sh)
    Q, K, V = synth.generate(w, query_corr=query_corr)
    Qg, Kg, Vg = Q.cuda(), K.cuda(), V.cuda()
    del Q, K, V
    R, words = sh.rows, (N + 31) // 32
    kbar = torch.empty((N, w.Hkv, w.D), dtype=torch.float32, device="cuda")
    mask = torch.empty((R, words), dtype=torch.int32, device="cuda")
    count = torch.empty((R,), dtype=torch.int32, device="cuda")
    O = torch.empty((w.S, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")
    ws_sel = B.alloc_workspace(sh, B.CALL_CUBE_SELECT)
    cube, rank, sizes = cube_tables(w)
    preceding = int(cube.astype(np.int64).sum()) * w.Hq
    pairs_capacity = int(0.41 * preceding)
    free_bytes, _ = torch.cuda.mem_get_info()
    try:
        if B.pairs_workspace_bytes(sh, pairs_capacity) > 0.4 * free_bytes:
            pairs_capacity = None
    except B.AdasparkError:
        pairs_capacity = None
    ws_att = B.alloc_workspace(sh, B.CALL_SPARSE_ATTN, pairs_capacity=pairs_capacity)

    def step():
        B.cube_pool(sh, Kg, kbar)
        B.cube_select(sh, Qg, kbar, p, sel_mask=mask, sel_count=count, workspace=ws_sel)
        B.kv_pack(sh, Kg, Vg, ws_att)
        B.sparse_attn_packed(sh, Qg, ws_att, mask, O=O)

    step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    graph_ms = None
    if ms < 10.0:  # short steps are launch-bound: the same step recorded as a HIP graph and replayed
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
    att_ms = timed(lambda: B.sparse_attn_packed(sh, Qg, ws_att, mask, O=O), steps)
    pack_ms = timed(lambda: B.kv_pack(sh, Kg, Vg, ws_att), steps)
    B.dense_attn_packed(sh, Qg, ws_att, O=O)
    dense_ms = timed(lambda: B.dense_attn_packed(sh, Qg, ws_att, O=O), max(1, min(steps, 3)))
    keys_total, pairs = attended_keys_total(w, mask, sizes, rank)
    dense_keys = int((np.cumsum(np.concatenate([[0], sizes[:-1]]))[cube] + rank + 1).sum()) * w.Hq
    tf = 4.0 * w.D * keys_total / (att_ms * 1e-3) / 1e12
    return {"workload": f"{w.T}x{w.H}x{w.W} tokens={w.S}, cube {w.ct}x{w.ch}x{w.cw} ({N} cubes), {w.Hq}q/{w.Hkv}kv "
                        f"heads, head_dim {w.D}, top_p {p:g}" + (f", query correlation {query_corr:g}" if query_corr else ""),
            "ms_per_step": ms, "tokens_per_s": w.S / (ms * 1e-3), "graph_replay_ms_per_step": graph_ms,
            "sparse_attn_ms": att_ms,
            "selected_fraction_of_preceding_cubes": pairs / max(1, preceding),
            "effective_tflops": tf, "frac_of_mfma_peak": tf / PEAK_BF16_TFLOPS,
            "dense_attn_ms": dense_ms, "dense_tflops": 4.0 * w.D * dense_keys / (dense_ms * 1e-3) / 1e12,
            "speedup_vs_dense": (pack_ms + dense_ms) / ms}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="C3", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--top-p", type=float, default=0.9)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--shared-selection", action="store_true",
                    help="select once per (token, KV head) from the group's mean query (adaspark_cube_select_shared) "
                         "instead of per query head; a variant, not the headline configuration")
    ap.add_argument("--query-corr", type=float, default=0.0,
                    help="a variant, not the headline: queries of a cube's video tokens share a component per head "
                         "(synth.generate's query_corr), as neighbouring video tokens do; the masked walk then "
                         "leaves out the cubes that no row of a workgroup selected")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-ffn", action="store_true", help="skip the token-selective FFN leg (Sec. 3.3)")
    ap.add_argument("--no-bwd", action="store_true", help="skip the attention backward leg")
    ap.add_argument("--no-sweep", action="store_true",
                    help="do not time the workload's other Top-p values (C3: 0.5, 0.7, 0.99; the top_p_sweep object) "
                         "nor, in a default C3 run, the four other workloads (the other_workloads object)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch one plain 1 GiB device copy after the timed region: the known-size "
                         "reference the HBM counters of a rocprofv3 --pmc run are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)

    from paper_2604_08077_amd import binding as B

    B.load()
    w = synth.WORKLOADS[args.workload]
    p = float(np.float32(args.top_p))
    sh = B.Shape.of(w)
    N = B.num_cubes(sh)
    Q, K, V = synth.generate(w, query_corr=args.query_corr)
    Qg, Kg, Vg = Q.cuda(), K.cuda(), V.cuda()
    R, words = sh.rows, (N + 31) // 32
    kbar = torch.empty((N, w.Hkv, w.D), dtype=torch.float32, device="cuda")
    mask = torch.empty((R, words), dtype=torch.int32, device="cuda")
    count = torch.empty((R,), dtype=torch.int32, device="cuda")
    O = torch.empty((w.S, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")
    ws_sel = B.alloc_workspace(sh, B.CALL_CUBE_SELECT)
    # Attention workspace: the packed K/V copy plus, where HBM allows, scratch for the key-stationary kernel up to
    # the selected share below which the library prefers it (attn_walk.hip: 40 % of the candidate cubes).
    cube, rank, sizes = cube_tables(w)
    preceding = int(cube.astype(np.int64).sum()) * w.Hq
    pairs_capacity = int(0.41 * preceding)
    free_bytes, _ = torch.cuda.mem_get_info()
    try:
        if B.pairs_workspace_bytes(sh, pairs_capacity) > 0.4 * free_bytes:
            pairs_capacity = None
    except B.AdasparkError:
        pairs_capacity = None  # geometry outside what that kernel covers
    ws_att = B.alloc_workspace(sh, B.CALL_SPARSE_ATTN, pairs_capacity=pairs_capacity)

    def f_pool():
        B.cube_pool(sh, Kg, kbar)

    def f_select():
        nonlocal mask, count
        if args.shared_selection:
            mask, count = B.cube_select_shared(sh, Qg, kbar, p)
        else:
            B.cube_select(sh, Qg, kbar, p, sel_mask=mask, sel_count=count, workspace=ws_sel)

    def f_pack():
        B.kv_pack(sh, Kg, Vg, ws_att)

    def f_attn():
        B.sparse_attn_packed(sh, Qg, ws_att, mask, O=O)

    def f_dense():
        B.dense_attn_packed(sh, Qg, ws_att, O=O)

    # the sparse entry picks one of its kernels from the share of selected cubes (on the device); for the roofline
    # line the same kernel is launched alone, so that the HIP events bracket exactly one kernel
    def f_attn_kernel(kernel):
        B.sparse_attn_packed(sh, Qg, ws_att, mask, O=O, kernel=kernel)

    def step():
        f_pool()
        f_select()
        f_pack()
        f_attn()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-kernel means (HIP events on the launch stream), same inputs, same launch configuration
    k_ms = {name: timed(fn, args.steps) for name, fn in
            (("cube_pool", f_pool), ("cube_select", f_select), ("kv_pack", f_pack), ("sparse_attn", f_attn))}
    dense_ms = None
    if not args.no_dense:
        f_dense()
        torch.cuda.synchronize()
        dense_ms = timed(f_dense, max(1, min(args.steps, 3)))

    if args.copy_probe:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")  # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    ceilings = measured_ceilings(B)
    keys_total, pairs = attended_keys_total(w, mask, sizes, rank)
    eff_flops = 4.0 * w.D * keys_total
    dense_keys = int((np.cumsum(np.concatenate([[0], sizes[:-1]]))[cube] + rank + 1).sum()) * w.Hq
    dense_flops = 4.0 * w.D * dense_keys
    share = pairs / max(1, preceding)
    # the library's own rule (attn_walk.hip, attn_pairs.hip), restated to name the kernel(s) that ran: per KV head
    # the key-stationary kernel below 40 % selected cubes (if its records fit), else one of the row-stationary ones
    G = w.Hq // w.Hkv
    sel_per_kv = count.view(w.S, w.Hkv, G).sum(dim=(0, 2), dtype=torch.int64).cpu().numpy()
    pairs_heads = [kv for kv in range(w.Hkv) if pairs_capacity is not None
                   and int(sel_per_kv[kv]) * 1000 < (preceding // w.Hkv) * 400]
    if pairs_heads and int(sum(sel_per_kv[kv] for kv in pairs_heads)) > pairs_capacity:
        pairs_heads = []
    row_kernel, row_name = ((B.SPARSE_MASKED, f"attn_walk_kernel<{w.D}, true>") if share * 1000.0 > 15.0
                            else (B.SPARSE_COMPACT, f"attn_compact_kernel<{w.D}>"))
    pairs_name = f"attn_pairs_kernel<{w.D}> + pairs_merge_kernel<{w.D}>"
    if len(pairs_heads) == w.Hkv:
        chosen, chosen_name = B.SPARSE_PAIRS, pairs_name
    elif not pairs_heads:
        chosen, chosen_name = row_kernel, row_name
    else:  # heads differ: the entry's own mix, timed as a whole
        chosen, chosen_name = B.SPARSE_AUTO, f"{pairs_name} (KV heads {pairs_heads}), {row_name} (the others)"
    if args.query_corr > 0.0:
        # the library also weighs the share of cubes a masked-walk workgroup can leave out (estimated on the device):
        # the rule restated above does not say which kernel ran, so the entry's own choice is timed as a whole
        chosen, chosen_name = B.SPARSE_AUTO, "the library's choice among its sparse kernels"
    masked_walk = chosen == B.SPARSE_MASKED
    attn_kernel_ms = timed(lambda: f_attn_kernel(chosen), args.steps)
    attn_tflops = eff_flops / (attn_kernel_ms * 1e-3) / 1e12
    # the masked walk computes every preceding cube that some row of a workgroup selected: with the listed recipe
    # (rows selecting independently) that is every preceding cube
    executed_flops = dense_flops if masked_walk and args.query_corr == 0.0 else None

    hbm_bytes = {
        "cube_pool": w.S * w.Hkv * w.D * 2 + N * w.Hkv * w.D * 4,
        "cube_select": R * w.D * 2 + R * words * 4 + R * 4,
        "kv_pack": 2 * w.S * w.Hkv * w.D * 2 + B.workspace_bytes(sh, B.CALL_SPARSE_ATTN),
    }
    out = {
        "metric": ("AdaS-Attn tokens/s at 64K video tokens" if args.workload == "C3" else f"AdaS-Attn tokens/s ({w.name})")
                  + (f" (variant: query correlation {args.query_corr})" if args.query_corr > 0.0 else ""),
        "value": w.S / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{w.name}: {w.T}x{w.H}x{w.W} tokens={w.S}, cube {w.ct}x{w.ch}x{w.cw} ({N} cubes), "
                        f"{w.Hq}q/{w.Hkv}kv heads, head_dim {w.D}, top_p {args.top_p}, causal, batch 1",
            "top_p": args.top_p,
            "selection": "shared by the GQA group" if args.shared_selection else "per query head",
            "arithmetic": "bf16 in and out; q.k products fp16 x fp16 -> fp32 (MFMA), p.v products bf16 x bf16 -> fp32, "
                          "softmax fp32; selection logits fp32-accurate (three bf16 MFMA terms)",
            "query_corr": args.query_corr,
        },
        "effective_tflops": attn_tflops,
        "effective_flops_per_step": eff_flops,
        "dense_flops": dense_flops,
        "selected_fraction_of_preceding_cubes": share,
        "kernel_ms": k_ms,
        "kernel_hbm_gbs": {k: hbm_bytes[k] / (k_ms[k] * 1e-3) / 1e9 for k in hbm_bytes},
        "kernel_hbm_frac": {k: hbm_bytes[k] / (k_ms[k] * 1e-3) / 1e9 / PEAK_HBM_GBS for k in hbm_bytes},
        "kernel_hbm_frac_measured": {k: hbm_bytes[k] / (k_ms[k] * 1e-3) / 1e9 / ceilings["copy_gbs"] for k in hbm_bytes},
        "measured_ceilings": ceilings,
        "dense_attn_ms": dense_ms,
        "dense_tflops": None if dense_ms is None else dense_flops / (dense_ms * 1e-3) / 1e12,
        "speedup_vs_dense": None if dense_ms is None else (k_ms["kv_pack"] + dense_ms) / ms_per_step,
        "roofline": {
            "kernel": chosen_name,
            "kernel_ms": attn_kernel_ms,
            "bound": "mfma",
            "achieved": attn_tflops,
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": attn_tflops / PEAK_BF16_TFLOPS,
            "peak_measured": ceilings["mfma_bf16_tflops"],
            "frac_measured": attn_tflops / ceilings["mfma_bf16_tflops"],
            "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, args.top_p)),
            "traffic_source": "stored figure from the rocprofv3 --pmc summaries under profiles/ (not counted in this run)",
            "executed_tflops": None if executed_flops is None else executed_flops / (attn_kernel_ms * 1e-3) / 1e12,
        },
    }
    if not args.no_sweep and not args.shared_selection and len(w.top_p) > 1:
        # the workload's other Top-p values (the configuration names the sweep): same inputs, same workspaces; step =
        # pool + select + pack + sparse attention, host clock around `steps` steps; effective FLOPs from the selection
        sweep = {}
        for ps in w.top_p:
            psf = float(np.float32(ps))
            if abs(psf - p) < 1e-6:
                continue
            B.cube_select(sh, Qg, kbar, psf, sel_mask=mask, sel_count=count, workspace=ws_sel)

            def step_p():
                B.cube_pool(sh, Kg, kbar)
                B.cube_select(sh, Qg, kbar, psf, sel_mask=mask, sel_count=count, workspace=ws_sel)
                B.kv_pack(sh, Kg, Vg, ws_att)
                B.sparse_attn_packed(sh, Qg, ws_att, mask, O=O)

            step_p()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(max(2, args.steps // 2)):
                step_p()
            torch.cuda.synchronize()
            ms_p = (time.perf_counter() - t0) * 1e3 / max(2, args.steps // 2)
            keys_p, pairs_p = attended_keys_total(w, mask, sizes, rank)
            att_p = timed(f_attn, max(2, args.steps // 2))
            sweep[str(ps)] = {"ms_per_step": ms_p, "tokens_per_s": w.S / (ms_p * 1e-3), "sparse_attn_ms": att_p,
                              "selected_fraction_of_preceding_cubes": pairs_p / max(1, preceding),
                              "effective_tflops": 4.0 * w.D * keys_p / (att_p * 1e-3) / 1e12,
                              "speedup_vs_dense": None if dense_ms is None else (k_ms["kv_pack"] + dense_ms) / ms_p}
        out["top_p_sweep"] = sweep
        B.cube_select(sh, Qg, kbar, p, sel_mask=mask, sel_count=count, workspace=ws_sel)  # back to the headline p
    if not args.no_bwd and w.S * w.Hq * words < (1 << 30) and w.S <= 131072:
        out["attn_bwd"] = bwd_leg(B, w, sh, Qg, Kg, Vg, ws_att, mask, eff_flops, dense_flops, args.steps, args.top_p)
    if not args.no_ffn and w.S * FFN_D_MODEL < (1 << 30):
        del ws_att, mask, count, O
        torch.cuda.empty_cache()
        out["adas_ffn"] = ffn_leg(B, w, args.steps, dense=not args.no_dense)
    if not args.no_cpu_baseline and not args.shared_selection and args.query_corr == 0.0:
        out["cpu_baseline"] = cpu_baseline(w, p, Q, K, V)
    if (not args.no_sweep and not args.shared_selection and args.workload == "C3" and abs(p - 0.9) < 1e-6
            and args.query_corr == 0.0):
        # the four other workloads of the configuration list, one after the other on the emptied device
        del Qg, Kg, Vg, kbar, Q, K, V
        torch.cuda.empty_cache()
        out["other_workloads"] = {}
        for name in sorted(synth.WORKLOADS):
            if name != "C3":
                out["other_workloads"][name] = workload_line(B, synth.WORKLOADS[name], 3 if name == "C4" else args.steps)
                torch.cuda.empty_cache()
        # The headline workload once more with queries that the video tokens of a cube share a component of
        # (synth.generate's query_corr: a variant outside the configuration's recipe, whose rows select independently
        # of each other -- the hardest case for a kernel that can only leave out what a whole group of rows skips).
        # The selected share per row stays what it is; what changes is how much neighbouring rows agree.
        out["correlated_queries"] = {
            str(rho): workload_line(B, synth.WORKLOADS["C3"], max(2, args.steps // 2), query_corr=rho, top_p=p)
            for rho in (0.9, 0.99)}
        torch.cuda.empty_cache()
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
