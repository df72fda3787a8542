#!/usr/bin/env python3
"""Benchmark of the SharePrefill per-layer prefill attention path on one MI355X.

A "step" is one fused sp_prefill_layer call (K/V packing -> dense pivots + block
scores -> mask builder -> block-sparse heads) on one layer of seeded synthetic
input that is already resident in HBM.  Prints ONE JSON line.

  value        effective TFLOP/s = flops a dense causal layer would need / time of the
               sparse-prefill layer (so it grows with both kernel speed and sparsity)
  ms_per_step  sparse-prefill attention ms per layer
  roofline     dense-pivot kernel (the dominant one): tiles x 4*B^2*d flops / its average
               launch time (HIP events recorded by the library on the launch stream)
               against the bf16 dense MFMA peak
  cpu_baseline the CPU oracle timed on a bounded sample of query-block rows of the same
               workload, in the same unit
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0
# HBM/fabric bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes (counters scaled by a
# 1 GiB copy).  A benchmark run cannot collect counters itself, so the figures are carried here per workload and
# kernel together with the profile summary they come from and the digest of the kernel sources that summary was
# made with (kernel_source_digest() below); a run whose sources differ reports null.
MEASURED_TRAFFIC = {
    "llama8b_128k": {"profile": "profiles/prefill_layer_llama8b_128k.md", "source_digest": "f8cce53a0630691d",
                     "dense_bytes": 14.30e9, "sparse_bytes": 45.25e9},
}


def kernel_source_digest() -> str:
    """sha256 (first 16 hex digits) over the library's sources: names the build a counter figure belongs to."""
    import hashlib
    h = hashlib.sha256()
    src = os.path.join(ROOT, "paper_2505_19578_amd", "csrc")
    # the files that define the two attention kernels, their K/V images and their launch
    for name in ["attn_kernel.h", "pack_kernel.h", "sp_common.h", "shareprefill.hip", "../../include/shareprefill.h"]:
        with open(os.path.join(src, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def bench_dict(args, sp, torch, np, CONFIGS, make_layer) -> int:
    """L layers of one prompt through the dictionary; a "step" is the whole stack of layers."""
    nl = args.dict_layers
    delta, tau = (float(x) for x in (args.gate or "10,0.2").split(","))
    score_mode = sp.SP_SCORE_MEAN_LOGIT if args.score_mode == "mean-logit" else sp.SP_SCORE_BLOCK_MASS
    select_mode = sp.SP_SELECT_GLOBAL if args.select_mode == "global" else sp.SP_SELECT_PER_ROW
    t0 = time.time()
    Ls = [make_layer(CONFIGS[args.config], layer=l, seq=args.seq, structure_layer=0) for l in range(nl)]
    gen_s = time.time() - t0
    cfg = Ls[0]["cfg"]
    B, d, N, Hq, C = cfg.block, cfg.head_dim, cfg.seq, cfg.n_q_heads, cfg.n_clusters
    nqb = N // B
    dev = [{x: torch.from_numpy(L[x].view(np.int16)).view(torch.bfloat16).unsqueeze(0).cuda() for x in "qkv"} for L in Ls]
    h2c = [int(x) for x in Ls[0]["head_to_cluster"]]
    shape = sp.shape_of(dev[0]["q"], dev[0]["k"], None, B)
    outs = [torch.zeros_like(dv["q"]) for dv in dev]
    vs = args.fallback == "vs"
    vst = args.fallback == "vs-token"
    ws = torch.empty(sp.sp_workspace_bytes(shape, C) + (sp.sp_vs_workspace_bytes(shape, Hq) if vs else 0)
                     + (sp.sp_vs_token_workspace_bytes(shape, Hq) if vst else 0), dtype=torch.uint8, device="cuda")
    vs_idx = torch.empty((1, Hq, nqb, nqb), dtype=torch.int32, device="cuda") if vs else None
    vs_cnt = torch.zeros((1, Hq, nqb), dtype=torch.int32, device="cuda") if vs else None
    scores = torch.empty((1, C, nqb, nqb), dtype=torch.float32, device="cuda")
    valid = torch.zeros((1, C), dtype=torch.int32, device="cuda")
    a_tilde = torch.empty((1, C, nqb), dtype=torch.float32, device="cuda")
    kb_idx = torch.empty((1, C, nqb, nqb), dtype=torch.int32, device="cuda")
    kb_cnt = torch.empty((1, C, nqb), dtype=torch.int32, device="cuda")
    pd = sp.pattern_dict_of(valid, a_tilde, kb_idx, kb_cnt)
    roles = [torch.empty((1, Hq), dtype=torch.int32, device="cuda") for _ in range(nl)]
    a_hat = torch.empty((1, Hq, nqb), dtype=torch.float32, device="cuda")
    dist = torch.empty((1, Hq, 2), dtype=torch.float32, device="cuda")

    def step():
        valid.zero_()                      # a new prefill starts with an empty dictionary
        for l in range(nl):
            sp.sp_prefill_layer_dict(shape, dev[l]["q"], dev[l]["k"], dev[l]["v"], h2c, cfg.gamma, delta, tau,
                                     score_mode, select_mode, pd, outs[l], scores, roles[l], a_hat, dist, ws,
                                     fallback_mode=(sp.SP_FALLBACK_VERTICAL_SLASH if vs else
                                                    sp.SP_FALLBACK_VERTICAL_SLASH_TOKEN if vst else sp.SP_FALLBACK_DENSE),
                                     vs_idx=vs_idx, vs_cnt=vs_cnt)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    sp.sp_profile_enable(True)          # per-kernel durations from a second, separately bracketed pass
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    prof = sp.sp_profile_read(reset=True)
    sp.sp_profile_enable(False)
    ms_step = wall * 1e3 / args.steps
    role_h = [r.cpu().numpy()[0] for r in roles]
    cnt = kb_cnt.cpu().numpy()[0].astype(np.int64)
    tile_flops = 4.0 * B * B * d
    dense_tiles_per_head = nqb * (nqb + 1) // 2
    tiles = 0
    vs_last = vs_cnt.cpu().numpy()[0].astype(np.int64) if vs else None   # lists of the last layer's fallback heads
    for l, r in enumerate(role_h):
        for h in range(Hq):
            if r[h] >= 0:
                tiles += int(cnt[r[h]].sum())
            elif r[h] == -1 and vs and l == nl - 1:
                tiles += int(vs_last[h].sum())
            elif r[h] == -1 and vs:
                tiles += -1 << 60        # unknown for earlier layers (their lists were overwritten): flagged below
            else:
                tiles += dense_tiles_per_head
    dense_equiv_flops = nl * Hq * 4.0 * d * (N * (N + 1) / 2.0)
    # token-level fallback: the pattern's size (pairs kept / causal pairs) of the last layer's fallback heads, from
    # one stand-alone call outside the timed region
    pair_frac = None
    if vst:
        fb = [h for h in range(Hq) if role_h[-1][h] == -1]
        if fb:
            pairs = torch.zeros((1, len(fb)), dtype=torch.int64, device="cuda")
            sp.sp_vertical_slash_attn(shape, dev[-1]["q"], dev[-1]["k"], dev[-1]["v"], fb, cfg.gamma, True,
                                      torch.zeros_like(outs[-1]), None, pairs, ws)
            torch.cuda.synchronize()
            pair_frac = float(pairs.sum().item() / (len(fb) * (N * (N + 1) / 2.0)))
    out = {
        "metric": "sparse-prefill attention ms/layer at 128K + effective TFLOP/s vs dense",
        "value": dense_equiv_flops / (ms_step * 1e-3) / 1e12,
        "unit": "effective TFLOP/s (dense-causal-equivalent flops / sparse-prefill layer time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {nl} layers of one prompt through the cross-layer pattern dictionary, "
                               f"batch 1, {Hq}q/{cfg.n_kv_heads}kv heads, d{d}, seq {N}, block {B}, {C} clusters spanning "
                               f"the layers, gamma {cfg.gamma}, delta {delta}, tau {tau}",
                   "density": float(cnt.sum() / (C * dense_tiles_per_head))},
        "ms_per_layer": ms_step / nl,
        "computed_tflops": tiles * tile_flops / (ms_step * 1e-3) / 1e12 if tiles >= 0 else None,
        "fallback": args.fallback,
        "vs_token_pair_fraction_last_layer": pair_frac,
        "vs_block_density_last_layer": (float(sum(vs_last[h].sum() for h in range(Hq) if role_h[-1][h] == -1)
                                              / max(1, int((role_h[-1] == -1).sum()) * dense_tiles_per_head))
                                        if vs else None),
        "roles_per_layer": [{"pivot": int((r == -2).sum()), "shared": int((r >= 0).sum()),
                             "fallback": int((r == -1).sum())} for r in role_h],
        "kernel_ms_per_step": {kk: prof[kk][0] / args.steps for kk in prof},
        "pattern": {"score_mode": args.score_mode, "select_mode": args.select_mode},
        "input_gen_s": gen_s,
    }
    print(json.dumps(out))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="llama8b_128k")
    ap.add_argument("--seq", type=int, default=None, help="override the sequence length (debug)")
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--score-mode", choices=["mass", "mean-logit"], default="mass",
                    help="pivot score map: exact block mass (default) or the paper's row softmax of block-mean logits")
    ap.add_argument("--select-mode", choices=["row", "global"], default="row",
                    help="Alg. 2 per query-block row (default) or once over the flattened map as printed")
    ap.add_argument("--gate", default=None, metavar="DELTA,TAU",
                    help="run Alg. 3's gate in front of the sharing (sp_prefill_layer_gated), e.g. 0.3,0.2")
    ap.add_argument("--dict-layers", type=int, default=0, metavar="L",
                    help="time L layers of one prompt through the cross-layer pattern dictionary "
                         "(sp_prefill_layer_dict; thresholds from --gate, default 10,0.2) and print that line instead")
    ap.add_argument("--fallback", choices=["dense", "vs", "vs-token"], default="dense",
                    help="with --dict-layers: what heads that fail Alg. 3 run: dense, the vertical-slash pattern of "
                         "Alg. 5 widened to whole key blocks (vs), or that pattern token by token (vs-token)")
    ap.add_argument("--graph", action="store_true",
                    help="capture the step into a HIP graph and time replays (the calls enqueue kernels only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dense-all", action="store_true")
    ap.add_argument("--sparse-one-per-cluster", action="store_true",
                    help="after the timed steps, also launch the block-sparse kernel twice on one sharing head per "
                         "cluster (for counter runs: how much of the K/V traffic the heads of a cluster share)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (a known-size reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU (no sharding, no collectives); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2505_19578_amd as sp
    from synth import CONFIGS, make_layer

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.dict_layers > 0:
        return bench_dict(args, sp, torch, np, CONFIGS, make_layer)
    t0 = time.time()
    L = make_layer(CONFIGS[args.config], layer=args.layer, seq=args.seq)
    cfg = L["cfg"]
    gen_s = time.time() - t0
    dev = {x: torch.from_numpy(L[x].view(np.int16)).view(torch.bfloat16).unsqueeze(0).cuda() for x in "qkv"}
    q, k, v = dev["q"], dev["k"], dev["v"]
    B, d, N, Hq = cfg.block, cfg.head_dim, cfg.seq, cfg.n_q_heads
    nqb = N // B
    C = cfg.n_clusters
    h2c, piv = [int(x) for x in L["head_to_cluster"]], [int(x) for x in L["pivot_heads"]]
    shape = sp.shape_of(q, k, None, B)
    o = torch.zeros_like(q)
    ws = torch.empty(sp.sp_workspace_bytes(shape, C), dtype=torch.uint8, device="cuda")
    scores = torch.empty((1, C, nqb, nqb), dtype=torch.float32, device="cuda")
    kb_idx = torch.empty((1, C, nqb, nqb), dtype=torch.int32, device="cuda")
    kb_cnt = torch.empty((1, C, nqb), dtype=torch.int32, device="cuda")

    score_mode = sp.SP_SCORE_MEAN_LOGIT if args.score_mode == "mean-logit" else sp.SP_SCORE_BLOCK_MASS
    select_mode = sp.SP_SELECT_GLOBAL if args.select_mode == "global" else sp.SP_SELECT_PER_ROW
    default_modes = args.score_mode == "mass" and args.select_mode == "row"

    gate = None
    if args.gate:
        gate = tuple(float(x) for x in args.gate.split(","))
        a_hat = torch.empty((1, Hq, nqb), dtype=torch.float32, device="cuda")
        dist = torch.empty((1, Hq, 2), dtype=torch.float32, device="cuda")
        pattern = torch.empty((1, Hq), dtype=torch.int32, device="cuda")

    def step():
        if gate:
            sp.sp_prefill_layer_gated(shape, q, k, v, h2c, piv, cfg.gamma, gate[0], gate[1], score_mode, select_mode,
                                      o, scores, kb_idx, kb_cnt, a_hat, dist, pattern, ws)
        elif default_modes:
            sp.sp_prefill_layer(shape, q, k, v, h2c, piv, cfg.gamma, o, scores, kb_idx, kb_cnt, ws)
        else:
            sp.sp_prefill_layer_modes(shape, q, k, v, h2c, piv, cfg.gamma, score_mode, select_mode, o, scores,
                                      kb_idx, kb_cnt, ws)

    if args.graph:
        eager_step = step
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            eager_step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            eager_step()
        step = graph.replay

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").fill_(1.0)   # 1 GiB
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps, nothing else on the stream (no per-kernel events)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # same stream as the launches
    t0 = time.perf_counter()
    marks[0].record()
    for n in range(args.steps):
        step()
        marks[n + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    per_step = sorted(marks[n].elapsed_time(marks[n + 1]) for n in range(args.steps))
    ms_step = wall * 1e3 / args.steps
    # a second pass of the same steps with every kernel bracketed by HIP events on the launch stream:
    # the per-kernel durations behind the roofline objects (not part of ms_per_step)
    prof = None
    if not args.graph:
        sp.sp_profile_enable(True)
        for n in range(args.steps):
            step()
        torch.cuda.synchronize()
        prof = sp.sp_profile_read(reset=True)
        sp.sp_profile_enable(False)
    if prof is None:
        prof = {kk: (0.0, 0) for kk in ("pack", "dense", "mask", "sparse", "score", "vs")}

    # work actually done
    cnt = kb_cnt.cpu().numpy()[0].astype(np.int64)            # [C][nqb]
    tile_flops = 4.0 * B * B * d
    n_free = sum(1 for h in range(Hq) if h2c[h] < 0)
    fell_back = []          # clustered heads the gate sent to the dense fallback
    if gate:
        pat_h = pattern.cpu().numpy()[0]
        fell_back = [h for h in range(Hq) if h2c[h] >= 0 and h not in piv and pat_h[h] < 0]
    dense_tiles_per_head = nqb * (nqb + 1) // 2
    pivot_tiles = (C + n_free) * dense_tiles_per_head
    sparse_tiles = int(sum(cnt[h2c[h]].sum() for h in range(Hq)
                           if h2c[h] >= 0 and h not in piv and h not in fell_back))
    sparse_tiles += len(fell_back) * dense_tiles_per_head
    density = float(cnt.sum() / (C * dense_tiles_per_head))
    dense_equiv_flops = Hq * 4.0 * d * (N * (N + 1) / 2.0)    # exact causal pair count
    computed_flops = (pivot_tiles + sparse_tiles) * tile_flops

    # dominant kernel: dense pivots
    dense_ms, dense_n = prof["dense"]
    dense_avg_ms = dense_ms / max(dense_n, 1)
    dense_flops_per_launch = pivot_tiles * tile_flops if n_free == 0 else C * dense_tiles_per_head * tile_flops
    if n_free:
        dense_avg_ms = dense_ms / args.steps          # two dense launches per step: report them together
        dense_flops_per_launch = pivot_tiles * tile_flops
    dense_tflops = dense_flops_per_launch / (dense_avg_ms * 1e-3) / 1e12 if dense_avg_ms > 0 else 0.0
    sparse_ms, sparse_n = prof["sparse"]
    sparse_avg_ms = sparse_ms / max(sparse_n, 1)
    sparse_per_step = max(sparse_n // max(args.steps, 1), 1)     # sparse launches per step (2 with the gate)
    sparse_tflops = (sparse_tiles * tile_flops / sparse_per_step / (sparse_avg_ms * 1e-3) / 1e12
                     if sparse_avg_ms > 0 else 0.0)

    if args.sparse_one_per_cluster:
        sub = []
        for c in range(C):
            sub.append(next(h for h in range(Hq) if h2c[h] == c and h not in piv))
        for _ in range(2):
            sp.sp_block_sparse_attn(shape, q, k, v, sub, [h2c[h] for h in sub], kb_idx, kb_cnt, C, o, ws)
        torch.cuda.synchronize()

    # the "vs dense" denominator: this library's own dense kernel on every head, no scores
    dense_all_ms = None
    if not args.no_dense_all:
        heads = list(range(Hq))
        sp.sp_dense_attn_with_block_scores(shape, q, k, v, heads, o, None, ws)
        torch.cuda.synchronize()
        reps = 5
        dm = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
        dm[0].record()
        for n in range(reps):
            sp.sp_dense_attn_with_block_scores(shape, q, k, v, heads, o, None, ws)
            dm[n + 1].record()
        torch.cuda.synchronize()
        dense_all_ms = dm[0].elapsed_time(dm[reps]) / reps

    # counter figures carried from a profile: only for the workload and the build they were taken on
    digest = kernel_source_digest()
    rec = MEASURED_TRAFFIC.get(cfg.name) if (args.seq is None and default_modes and not gate) else None
    traffic, traffic_source = {}, None
    if rec is not None:
        traffic_source = {"profile": rec["profile"], "source_digest": rec["source_digest"],
                          "matches_this_build": rec["source_digest"] == digest}
        if rec["source_digest"] == digest:
            traffic = rec
    out = {
        "metric": "sparse-prefill attention ms/layer at 128K + effective TFLOP/s vs dense",
        "value": dense_equiv_flops / (ms_step * 1e-3) / 1e12,
        "unit": "effective TFLOP/s (dense-causal-equivalent flops / sparse-prefill layer time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: 1 layer, batch 1, {Hq}q/{cfg.n_kv_heads}kv heads, d{d}, "
                               f"seq {N}, block {B}, {C} clusters x {cfg.cluster_size} heads, "
                               f"1 pivot each, gamma {cfg.gamma}",
                   "seed": L["seed"], "density": density},
        "ms_per_layer": ms_step,
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "hip_graph": bool(args.graph),
        "pattern": {"score_mode": args.score_mode, "select_mode": args.select_mode,
                    "gate": None if not gate else {"delta": gate[0], "tau": gate[1], "heads_fallen_back": len(fell_back)}},
        "computed_tflops": computed_flops / (ms_step * 1e-3) / 1e12,
        "computed_frac_of_bf16_peak": computed_flops / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        # the same with each diagonal tile counted by its B(B+1)/2 existing pairs instead of as a full tile
        "computed_tflops_causal_exact": (computed_flops - Hq * nqb * 4.0 * d * (B * (B - 1) / 2.0))
        / (ms_step * 1e-3) / 1e12,
        "tiles": {"pivot": int(pivot_tiles), "sparse": int(sparse_tiles),
                  "dense_layer": int(Hq * dense_tiles_per_head)},
        "kernel_ms": {kk: (prof[kk][0] / max(prof[kk][1], 1)) for kk in prof},
        "sparse_kernel_tflops": sparse_tflops,
        "dense_all_heads_ms": dense_all_ms,
        "speedup_vs_dense": (dense_all_ms / ms_step) if dense_all_ms else None,
        "roofline": {"kernel": "attn_kernel<dense> (pivot heads + block scores)", "bound": "mfma",
                     "achieved": dense_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": dense_tflops / PEAK_BF16_TFLOPS,
                     "traffic": traffic.get("dense_bytes"),
                     "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE+WRITE_SIZE, scaled)",
                     "traffic_source": traffic_source,
                     "traffic_gbs": (traffic["dense_bytes"] / (dense_avg_ms * 1e-3) / 1e9
                                     if traffic.get("dense_bytes") and dense_avg_ms > 0 else None),
                     "hbm_peak_gbs": PEAK_HBM_GBS,
                     "algorithmic_flops_per_launch": dense_flops_per_launch,
                     "launch_ms": dense_avg_ms, "launches_timed": dense_n},
        "roofline_sparse": {"kernel": "attn_kernel<block-sparse> (heads sharing their cluster's lists)", "bound": "mfma",
                            "achieved": sparse_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                            "frac": sparse_tflops / PEAK_BF16_TFLOPS,
                            "traffic": traffic.get("sparse_bytes"),
                            "traffic_unit": "bytes per launch (rocprofv3 FETCH_SIZE+WRITE_SIZE, scaled)",
                            "traffic_source": traffic_source,
                            "traffic_gbs": (traffic["sparse_bytes"] / (sparse_avg_ms * 1e-3) / 1e9
                                            if traffic.get("sparse_bytes") and sparse_avg_ms > 0 else None),
                            "algorithmic_flops_per_launch": sparse_tiles * tile_flops / sparse_per_step,
                            "tiles_from_kb_cnt": int(sparse_tiles),
                            "launch_ms": sparse_avg_ms, "launches_timed": sparse_n},
        "kernel_source_digest": digest,
        "input_gen_s": gen_s,
    }
    # the published peak next to what this board's CU count and maximum engine clock give
    props = torch.cuda.get_device_properties(0)
    clock_mhz = 0.0
    try:    # rocminfo lists every agent; the GPU agents are the ones with a gfx name
        import re
        import subprocess
        txt = subprocess.run(["rocminfo"], capture_output=True, text=True, timeout=60).stdout
        for agent in txt.split("*******")[1:]:
            if re.search(r"Name:\s+gfx9", agent):
                m = re.search(r"Max Clock Freq\. \(MHz\):\s+(\d+)", agent)
                if m:
                    clock_mhz = float(m.group(1))
                    break
    except Exception:
        pass
    out["roofline"]["peak_source"] = "published MI355X dense bf16 MFMA figure (256 CUs x 4096 flop/clk x 2.4 GHz)"
    out["roofline"]["board"] = {"name": props.name, "cus": props.multi_processor_count,
                                "max_engine_clock_mhz": clock_mhz,
                                "derived_peak_tflops": props.multi_processor_count * 4096 * clock_mhz * 1e6 / 1e12}

    if not args.no_cpu_baseline:
        import oracle
        from synth import bf16_bits_to_f32
        rows = sorted({nqb // 4, nqb // 2}) if nqb >= 8 else [nqb - 1]
        # bounded sample: every head, a couple of mid-length query-block rows
        idx_h, cnt_h = kb_idx.cpu().numpy()[0], kb_cnt.cpu().numpy()[0]
        hq = bf16_bits_to_f32(L["q"][: (max(rows) + 1) * B])
        hk = bf16_bits_to_f32(L["k"][: (max(rows) + 1) * B])
        hv = bf16_bits_to_f32(L["v"][: (max(rows) + 1) * B])
        t0 = time.perf_counter()
        oracle.prefill_layer(hq, hk, hv, B, h2c, piv, cfg.gamma, rows=rows)
        cpu_s = time.perf_counter() - t0
        pairs = sum(B * (i * B) + B * (B + 1) / 2 for i in rows)
        cpu_equiv = Hq * 4.0 * d * pairs
        out["cpu_baseline"] = {
            "value": cpu_equiv / cpu_s / 1e12, "unit": out["unit"], "cores": oracle.num_threads(),
            "kind": "oracle", "seconds": cpu_s,
            "sample": f"all {Hq} heads, query-block rows {rows} of {nqb} (sequence prefix of "
                      f"{(max(rows) + 1) * B} tokens), same inputs",
        }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
