#!/usr/bin/env python3
"""Benchmark of the SpecVLM hot path on one MI355X.

One "step" is one pass of the whole path over the 72B-verifier full-stack
workload (64 frames x 196 video tokens + 256 text tokens, 64/8 heads, d 128,
80 verifier layers; draft 14/2 heads, d 64, 24 layers; keep 10 %, gamma 5):

  score (80 layers, accumulated) -> select -> gather (24 draft layers)
  -> gamma x 24 draft decode attentions over the pruned cache
  -> 80 verify attentions (gamma+1 queries, full cache) -> accept

All inputs are synthetic and resident in HBM before the timed region.  The
headline value is the verify-step attention's achieved HBM bandwidth (its
algorithmic bytes / its time); the other stages are reported beside it.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per verify-attention launch (split + merge) from the rocprofv3 PMC runs summarised in
# profiles/bench_72b-full_hbm_traffic.md (FETCH_SIZE and WRITE_SIZE, scaled by the copy-kernel factors).
# Only valid for the default launch shape of that workload.
MEASURED_TRAFFIC_BYTES = {("72b-full", "head-major", 0): 62.18e6}
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="72b-full")
    ap.add_argument("--layout", default=None, choices=["head-major", "token-major"],
                    help="KV layout; default head-major ([H_kv][tokens][d], for a batch over the packed token axis)")
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sampling", action="store_true", help="rejection-sampling accept instead of greedy")
    ap.add_argument("--eager", action="store_true", help="launch from Python instead of replaying HIP graphs")
    ap.add_argument("--score-lse", action="store_true",
                    help="hand the score call each row's softmax normaliser (as a prefill attention would "
                         "have saved it), so scoring is one sweep per layer")
    ap.add_argument("--frames", type=int, default=0, help="override the frame count (with --attn-only)")
    ap.add_argument("--attn-only", action="store_true",
                    help="time only the verify attention of --workload (32b-long, ragged-x8, ...): extra context "
                         "numbers, not the headline line")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2508_16201_amd import binding as B, synth

    B.lib()                                    # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.attn_only:
        return attn_only(args, torch, B, synth)
    if args.layout is None:
        args.layout = "head-major"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.WORKLOADS[args.workload]
    L, V, T = w.n_layers, w.n_video, w.n_text
    hq, hkv, d, g1 = w.n_q_heads, w.n_kv_heads, w.head_dim, w.q_len
    kv_len, n_ctx = w.kv_len, w.n_ctx
    dq, dkv, dd, dl = w.draft_q_heads, w.draft_kv_heads, w.draft_head_dim, w.draft_layers
    scale, dscale = w.softmax_scale, 1.0 / float(np.sqrt(dd))
    budget, k_top = w.keep_budget, w.k_top
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED_BASE + 1000 * w.index)

    def randn_bf16(shape):
        out = torch.empty(shape, dtype=torch.bfloat16, device=dev)
        flat = out.view(-1)
        step = 1 << 26
        for o in range(0, flat.numel(), step):
            n = min(step, flat.numel() - o)
            flat[o:o + n] = torch.randn(n, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
        return out

    # ---- verifier cache: layer 0 is the seeded host layer (the one the parity
    # tests and the CPU baseline use), the rest is drawn on the device ----
    if args.layout == "head-major":
        k_all = randn_bf16((L, hkv, kv_len, d)).permute(0, 2, 1, 3)       # view [L, S, H, d]
        v_all = randn_bf16((L, hkv, kv_len, d)).permute(0, 2, 1, 3)
    else:
        k_all = randn_bf16((L, kv_len, hkv, d))
        v_all = randn_bf16((L, kv_len, hkv, d))
    host0 = synth.make_layer(w, 0)

    def dev_bits(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    k_all[0].copy_(dev_bits(host0["k"]))
    v_all[0].copy_(dev_bits(host0["v"]))
    q_text = randn_bf16((L, T, hq, d))
    q_text[0].copy_(dev_bits(host0["q_text"]))
    q_block = randn_bf16((L, g1, hq, d))
    q_block[0].copy_(dev_bits(host0["q_block"]))
    # plant the high-attention keys of layer 0's recipe in every layer (2 % of the video)
    planted = torch.from_numpy(host0["planted"]).to(dev)
    for l in range(1, L):
        k_all[l, planted] = k_all[0, planted]

    # ---- draft cache (full, draft-shaped) and its pruned destination ----
    draft_k = randn_bf16((dl, n_ctx, dkv, dd))
    draft_v = randn_bf16((dl, n_ctx, dkv, dd))
    n_pruned = n_ctx - V + budget
    pruned_k = torch.zeros((dl, n_pruned + g1, dkv, dd), dtype=torch.bfloat16, device=dev)
    pruned_v = torch.zeros_like(pruned_k)
    draft_q = randn_bf16((dl, 1, dq, dd))

    # ---- accept inputs ----
    acc = synth.make_accept_inputs(1, w.gamma, w.vocab, synth.SEED_BASE + 77, greedy=not args.sampling)
    t_logits = torch.from_numpy(acc["target_logits"]).to(dev)
    d_logits = torch.from_numpy(acc["draft_logits"]).to(dev) if args.sampling else None
    d_tokens = torch.from_numpy(acc["draft_tokens"]).to(dev)
    uniforms = torch.from_numpy(acc["uniforms"]).to(dev) if args.sampling else None

    # ---- workspaces and outputs, allocated once ----
    ws_score = B.new_workspace(B.score_workspace_bytes(T, n_ctx, V, hq, hkv, d), dev)
    ws_attn = B.new_workspace(B.decode_attn_workspace_bytes(1, g1, kv_len, hq, hkv, d, args.num_splits), dev)
    ws_dattn = B.new_workspace(B.decode_attn_workspace_bytes(1, 1, n_pruned + g1, dq, dkv, dd, 0), dev)
    ws_acc = B.new_workspace(B.accept_workspace_bytes(1, w.gamma, w.vocab, args.sampling), dev)
    scores = torch.zeros(V, dtype=torch.float32, device=dev)
    k_top_d = torch.tensor([k_top], dtype=torch.int32, device=dev)
    budget_d = torch.tensor([budget], dtype=torch.int32, device=dev)
    out_v = torch.empty((g1, hq, d), dtype=torch.bfloat16, device=dev)
    out_d = torch.empty((1, dq, dd), dtype=torch.bfloat16, device=dev)
    torch.cuda.synchronize()

    stages = ["score", "select", "gather", "draft_attn", "verify_attn", "accept"]
    keep = torch.zeros(budget, dtype=torch.int32, device=dev)
    n_acc = torch.zeros(1, dtype=torch.int32, device=dev)
    out_tok = torch.zeros((1, g1), dtype=torch.int32, device=dev)

    # Row normalisers of the text queries, as the verifier's prefill attention would have saved them
    # (set-up only: plain torch, outside the timed region).
    row_lse = None
    if args.score_lse:
        row_lse = torch.empty((L, T, hq), dtype=torch.float32, device=dev)
        hidden = torch.arange(n_ctx, device=dev)[None, :] > (V + torch.arange(T, device=dev))[:, None]
        for l in range(L):
            qf = q_text[l].float().permute(1, 0, 2)                                       # [hq, T, d]
            kf = k_all[l, :n_ctx].float().permute(1, 0, 2).repeat_interleave(hq // hkv, dim=0)
            logits = torch.bmm(qf, kf.transpose(1, 2)) * scale                           # [hq, T, n_ctx]
            logits.masked_fill_(hidden[None], float("-inf"))
            row_lse[l] = torch.logsumexp(logits, dim=-1).transpose(0, 1)
        del qf, kf, logits

    def st_score():
        for l in range(L):
            B.score(q_text[l], k_all[l, :n_ctx], 0, V, V, scale, beta=(1.0 if l else 0.0),
                    row_lse=None if row_lse is None else row_lse[l], scores=scores, workspace=ws_score)

    def st_select():
        B.select(scores, k_top_d, budget_d, budget, want_flags=False, keep_idx=keep)

    def st_gather():
        B.gather_kv(draft_k, draft_v, 0, V, keep, k_dst=pruned_k[:, :n_pruned], v_dst=pruned_v[:, :n_pruned])

    def st_draft():
        for t in range(w.gamma):
            for l in range(dl):
                B.decode_attn(draft_q[l], pruned_k[l, :n_pruned + t + 1], pruned_v[l, :n_pruned + t + 1],
                              dscale, out=out_d, workspace=ws_dattn)

    def st_verify():
        for l in range(L):
            B.decode_attn(q_block[l], k_all[l], v_all[l], scale, out=out_v,
                          num_splits=args.num_splits, workspace=ws_attn)

    def st_accept():
        B.accept(t_logits, d_tokens, draft_logits=d_logits, uniforms=uniforms, workspace=ws_acc,
                 n_accepted=n_acc, out_tokens=out_tok)

    stage_fns = [st_score, st_select, st_gather, st_draft, st_verify, st_accept]
    for fn in stage_fns:                       # eager pass: first-use set-up happens outside any capture
        fn()
    torch.cuda.synchronize()

    # Each stage is a launch-bound sequence of short kernels: capture it once in
    # a HIP graph (kernel nodes only) and replay it, so the GPU, not the Python
    # launch loop, sets the pace.
    graphs = []
    if args.eager:
        runners = stage_fns
    else:
        for fn in stage_fns:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fn()
            graphs.append(g)
        runners = [g.replay for g in graphs]
    torch.cuda.synchronize()

    def one_step(ev=None):
        for i, run in enumerate(runners):
            if ev is not None:
                ev[i].record()
            run()
        if ev is not None:
            ev[len(runners)].record()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(7)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(events[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    stage_ms = {name: float(np.mean([events[s][i].elapsed_time(events[s][i + 1]) for s in range(args.steps)]))
                for i, name in enumerate(stages)}

    # ---- verify attention: algorithmic bytes = K and V once + q in + o out ----
    attn_bytes = 2 * kv_len * hkv * d * 2 + 2 * g1 * hq * d * 2
    t_layer_us = stage_ms["verify_attn"] * 1e3 / L
    attn_gbs = attn_bytes / (t_layer_us * 1e-6) / 1e9
    # a second timing of the verify stage alone, replayed back to back
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(5, args.steps)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        runners[4]()
    e1.record()
    torch.cuda.synchronize()
    t_layer_us2 = e0.elapsed_time(e1) * 1e3 / (reps * L)
    attn_gbs2 = attn_bytes / (t_layer_us2 * 1e-6) / 1e9

    # The short stages (one or two kernels): inside a step each is a graph launch of its own, and an
    # event pair around a lone launch mostly times the launch.  Their GPU time is taken from a graph
    # that holds the stage ten times over, replayed back to back.
    def repeated_us(fn, inner=10, outer=5):
        if args.eager:
            run = lambda: [fn() for _ in range(inner)]
        else:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(inner):
                    fn()
            run = g.replay
        run()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(outer):
            run()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e3 / (inner * outer)
    short_us = {"select": repeated_us(st_select), "gather": repeated_us(st_gather), "accept": repeated_us(st_accept)}

    score_flops = 2.0 * T * hq * d * (V + (T + 1) / 2.0)          # one sweep of the contraction
    score_tflops = score_flops * L / (stage_ms["score"] * 1e-3) / 1e12
    draft_bytes = 2 * (n_pruned + 3) * dkv * dd * 2
    gather_bytes = 2 * 2 * dl * n_pruned * dkv * dd * 2
    decode_steps_per_s = 1e3 / (stage_ms["draft_attn"] + stage_ms["verify_attn"] + stage_ms["accept"])   # as timed inside the step

    result = {
        "metric": "verify-step attn HBM GB/s (% peak); prune+gather us; decode steps/s",
        "value": round(attn_gbs2, 1),
        "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_frames}x{w.grid_h * w.grid_w} video + {T} text tokens, "
                               f"{hq}/{hkv} heads d{d}, {L} verifier layers, gamma {w.gamma}, keep {w.keep_percent}%, "
                               f"draft {dq}/{dkv} d{dd} x{dl} layers",
                   "kv_layout": args.layout, "num_splits": args.num_splits,
                   "accept": "sampling" if args.sampling else "greedy",
                   "score_row_lse": "supplied" if args.score_lse else "computed",
                   "launch": "eager" if args.eager else "hip-graph per stage"},
        "pct_of_hbm_peak": round(100.0 * attn_gbs2 / HBM_PEAK_GBS, 1),
        "prune_gather_us": round(short_us["select"] + short_us["gather"], 1),
        "prune_gather_us_in_step": round((stage_ms["select"] + stage_ms["gather"]) * 1e3, 1),
        "select_us": round(short_us["select"], 2), "gather_us": round(short_us["gather"], 2),
        "accept_us": round(short_us["accept"], 2),
        "decode_steps_per_s": round(decode_steps_per_s, 1),
        "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()},
        "verify_attn_us_per_layer": round(t_layer_us2, 3),
        "verify_attn_us_per_layer_in_step": round(t_layer_us, 3),
        "verify_attn_gbs_in_step": round(attn_gbs, 1),
        "score_tflops_one_sweep_counted": round(score_tflops, 1),
        "score_pct_mfma_peak": round(100.0 * score_tflops / MFMA_BF16_PEAK_TFLOPS, 2),
        "draft_attn_us_per_layer": round(stage_ms["draft_attn"] * 1e3 / (w.gamma * dl), 3),
        "gather_gbs": round(gather_bytes / (short_us["gather"] * 1e-6) / 1e9, 1),
        "n_accepted": int(n_acc.item()),
        "score_mass_on_video": round(float(scores.sum().item()), 4),
        "roofline": {"kernel": "specvlm_decode_attn (verify, split + merge)", "bound": "hbm",
                     "achieved": round(attn_gbs2, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(attn_gbs2 / HBM_PEAK_GBS, 4),
                     "traffic": MEASURED_TRAFFIC_BYTES.get((w.name, args.layout, args.num_splits)),
                     "algorithmic_bytes_per_launch": attn_bytes},
    }

    if not args.no_cpu_baseline:
        # The fp64 oracle as it stands, on the host cores, over the same layer-0
        # inputs: repeated whole-layer passes for about 10 s (at most 30 s).
        import oracle
        cores = len(os.sched_getaffinity(0))
        passes, t0 = 0, time.perf_counter()
        while True:
            oracle.decode_attn(host0["q_block"], host0["k"], host0["v"], scale, want_lse=False)
            passes += 1
            dt = time.perf_counter() - t0
            if dt >= 10.0 or (passes >= 1 and dt * (passes + 1) / passes > 30.0):
                break
        result["cpu_baseline"] = {"value": round(attn_bytes * passes / dt / 1e9, 4), "unit": "GB/s",
                                  "cores": cores, "kind": "oracle",
                                  "sample": f"{passes} passes of the verify attention of layer 0 of {L} "
                                            f"(fp64 oracle, {dt:.1f} s, OpenMP over query rows)"}
    print(json.dumps(result))


def attn_only(args, torch, B, synth):
    """Verify attention alone on another workload: `layers` distinct caches
    (more than the 256 MB Infinity Cache holds) replayed from one HIP graph."""
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.WORKLOADS[args.workload]
    if args.frames:
        w = synth.scaled(w, n_frames=args.frames)
    hq, hkv, d, g1 = w.n_q_heads, w.n_kv_heads, w.head_dim, w.q_len
    if w.name == "ragged-x8":
        lens = [int(f) * 196 + w.n_text + g1 for f in synth.ragged_frames()]
    else:
        lens = [w.kv_len]
    batch, total = len(lens), sum(lens)
    attn_bytes = 2 * total * hkv * d * 2 + 2 * batch * g1 * hq * d * 2
    layers = max(2, min(w.n_layers if w.n_layers > 1 else 8, int(1.5e9 // attn_bytes) + 1))
    gen = torch.Generator(device=dev)
    gen.manual_seed(synth.SEED_BASE + 1000 * w.index)

    def randn_bf16(shape):
        return torch.randn(shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)

    # head-major: [H_kv][sum kv_len][d] (the requests packed along the token axis), viewed as
    # [sum kv_len, H_kv, d]; token-major: [sum kv_len][H_kv][d]
    if args.layout is None:
        args.layout = "head-major"
    if args.layout == "head-major":
        k = [randn_bf16((hkv, total, d)).permute(1, 0, 2) for _ in range(layers)]
        v = [randn_bf16((hkv, total, d)).permute(1, 0, 2) for _ in range(layers)]
    else:
        k = [randn_bf16((total, hkv, d)) for _ in range(layers)]
        v = [randn_bf16((total, hkv, d)) for _ in range(layers)]
    q = [randn_bf16((batch * g1, hq, d)) for _ in range(layers)]
    out = torch.empty((batch * g1, hq, d), dtype=torch.bfloat16, device=dev)
    import numpy as np
    cu_q = torch.tensor(np.arange(batch + 1) * g1, dtype=torch.int32, device=dev) if batch > 1 else None
    cu_kv = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev) if batch > 1 else None
    ws = B.new_workspace(B.decode_attn_workspace_bytes(batch, g1, max(lens), hq, hkv, d, args.num_splits), dev)

    def stage():
        for l in range(layers):
            B.decode_attn(q[l], k[l], v[l], w.softmax_scale, cu_q=cu_q, cu_kv=cu_kv, max_q_len=g1,
                          max_kv_len=max(lens), out=out, num_splits=args.num_splits, workspace=ws)

    stage()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stage()
    for _ in range(args.warmup):
        graph.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(args.steps):
        graph.replay()
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / (args.steps * layers)
    gbs = attn_bytes / (us * 1e-6) / 1e9
    print(json.dumps({
        "metric": "verify-step attn HBM GB/s (% peak)", "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us * layers / 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name} (verify attention only): batch {batch}, {total} keys, {hq}/{hkv} heads "
                               f"d{d}, gamma {w.gamma}, {layers} distinct layers",
                   "kv_layout": args.layout,
                   "num_splits": args.num_splits},
        "verify_attn_us_per_layer": round(us, 2),
        "roofline": {"kernel": "specvlm_decode_attn (verify, split + merge)", "bound": "hbm",
                     "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": attn_bytes}}))


if __name__ == "__main__":
    main()
