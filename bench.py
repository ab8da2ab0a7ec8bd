#!/usr/bin/env python3
"""Benchmark of the SpecVLM hot path on one MI355X.

One "step" is one pass of the whole path over the 72B-verifier full-stack
workload (64 frames x 196 video tokens + 256 text tokens, 64/8 heads, d 128,
80 verifier layers; draft 14/2 heads, d 64, 24 layers; keep 10 %, gamma 5):

  score (80 layers, accumulated) -> select -> gather (24 draft layers)
  -> gamma x 24 draft decode attentions over the pruned cache
  -> 80 verify attentions (gamma+1 queries, full cache) -> accept

All inputs are synthetic and resident in HBM before the timed region.  The
headline value is the verify-step attention's achieved HBM bandwidth: its
algorithmic bytes over its time INSIDE the timed steps (HIP events around the
stage in every step; mean over the steps, median and minimum beside it).
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "bench_72b-full_hbm_traffic.md")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="72b-full")
    ap.add_argument("--layout", default=None, choices=["head-major", "token-major"],
                    help="KV layout; default head-major ([H_kv][tokens][d], for a batch over the packed token axis)")
    ap.add_argument("--num-splits", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true",
                    help="skip the extra measurements (other attention shapes, sampling accept, large gather)")
    ap.add_argument("--sampling", action="store_true", help="rejection-sampling accept instead of greedy")
    ap.add_argument("--eager", action="store_true", help="launch from Python instead of replaying HIP graphs")
    ap.add_argument("--score-lse", action="store_true",
                    help="hand the score call each row's softmax normaliser (as a prefill attention would "
                         "have saved it), so scoring is one sweep per layer")
    ap.add_argument("--score-per-layer", action="store_true",
                    help="score with one specvlm_score call per verifier layer (4 launches each) instead of one "
                         "specvlm_score_layers call for all layers (4 launches in all)")
    ap.add_argument("--frames", type=int, default=0, help="override the frame count (with --attn-only)")
    ap.add_argument("--attn-only", action="store_true",
                    help="time only the verify attention of --workload (32b-long, ragged-x8, ...): extra context "
                         "numbers, not the headline line")
    return ap.parse_args()


def stats(xs):
    xs = np.asarray(xs, dtype=np.float64)
    return {"mean": float(xs.mean()), "median": float(np.median(xs)), "min": float(xs.min())}


def timed_replays(torch, run, reps):
    """HIP events (on the stream the work is launched on) around `reps` back-to-back runs; us per run."""
    run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        run()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e3 / reps


def graph_of(torch, fn, eager=False):
    fn()                                       # first-use set-up happens outside any capture
    torch.cuda.synchronize()
    if eager:
        return fn
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    return g.replay


def measured_traffic(workspace_bytes):
    """HBM bytes per verify-attention launch from the committed rocprofv3 counter summary, if it was taken
    with the split plan that runs now (identified by the workspace size, which is splits x padded rows)."""
    try:
        text = open(TRAFFIC_PROFILE).read()
        m = re.search(r"traffic_bytes_per_launch:\s*(\d+)\s+workspace_bytes:\s*(\d+)", text)
        if m and int(m.group(2)) == int(workspace_bytes):
            return int(m.group(1))
    except OSError:
        pass
    return None


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
        print(json.dumps(attn_only(args, torch, B, synth, args.workload, args.layout or "head-major",
                                   args.frames, args.steps, args.warmup)))
        return
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

    # ---- accept inputs: 64 seeded draws; the step uses the one whose accepted length is nearest the mean ----
    n_draws = 64
    acc = synth.make_accept_inputs(n_draws, w.gamma, w.vocab, synth.SEED_BASE + 77, greedy=not args.sampling)
    t_all = torch.from_numpy(acc["target_logits"]).to(dev)
    dl_all = torch.from_numpy(acc["draft_logits"]).to(dev) if args.sampling else None
    tok_all = torch.from_numpy(acc["draft_tokens"]).to(dev)
    u_all = torch.from_numpy(acc["uniforms"]).to(dev) if args.sampling else None
    n_all, _ = B.accept(t_all, tok_all, draft_logits=dl_all, uniforms=u_all)
    torch.cuda.synchronize()
    n_all = n_all.cpu().numpy().astype(np.float64)
    tokens_per_step = float(n_all.mean() + 1.0)
    pick = int(np.argmin(np.abs(n_all - n_all.mean())))
    t_logits = t_all[pick:pick + 1].contiguous()
    d_logits = dl_all[pick:pick + 1].contiguous() if args.sampling else None
    d_tokens = tok_all[pick:pick + 1].contiguous()
    uniforms = u_all[pick:pick + 1].contiguous() if args.sampling else None
    del t_all, dl_all, tok_all, u_all

    # ---- workspaces and outputs, allocated once ----
    ws_attn_bytes = B.decode_attn_workspace_bytes(1, g1, kv_len, hq, hkv, d, args.num_splits)
    ws_score = B.new_workspace(max(B.score_workspace_bytes(T, n_ctx, V, hq, hkv, d),
                                   B.score_layers_workspace_bytes(L, T, n_ctx, V, hq, hkv, d)), dev)
    ws_attn = B.new_workspace(ws_attn_bytes, dev)
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
        if not args.score_per_layer:
            # every verifier layer in one call: the text queries of all layers are kept until the prefill ends
            B.score_layers(q_text, k_all[:, :n_ctx], 0, V, V, scale, row_lse=row_lse, scores=scores,
                           workspace=ws_score)
            return
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
    # Each stage is a launch-bound sequence of short kernels: capture it once in
    # a HIP graph (kernel nodes only) and replay it, so the GPU, not the Python
    # launch loop, sets the pace.
    runners = [graph_of(torch, fn, args.eager) for fn in stage_fns]
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
    stage_ms_all = {name: [events[s][i].elapsed_time(events[s][i + 1]) for s in range(args.steps)]
                    for i, name in enumerate(stages)}
    stage_ms = {k: stats(v) for k, v in stage_ms_all.items()}

    # ---- verify attention: algorithmic bytes = K and V once + q in + o out; time = the stage inside the steps ----
    attn_bytes = 2 * kv_len * hkv * d * 2 + 2 * g1 * hq * d * 2
    layer_us = {k: v * 1e3 / L for k, v in stage_ms["verify_attn"].items()}
    attn_gbs = {k: attn_bytes / (v * 1e-6) / 1e9 for k, v in layer_us.items()}
    # beside it: the verify stage alone, replayed back to back (no other stage between the replays)
    isolated_us = timed_replays(torch, runners[4], max(5, args.steps // 5)) / L
    # and what merely reading one layer's K and V costs in one launch on this machine
    read_fn = graph_of(torch, lambda: [B.probe_read(k_all[l], v_all[l]) for l in range(L)], args.eager)
    read_ceiling_us = timed_replays(torch, read_fn, 5) / L

    # The short stages (one or two kernels): inside a step each is a graph launch of its own, and an
    # event pair around a lone launch mostly times the launch.  Their GPU time is taken from a graph
    # that holds the stage ten times over, replayed back to back.
    def repeated_us(fn, inner=10, outer=10):
        return timed_replays(torch, graph_of(torch, lambda: [fn() for _ in range(inner)], args.eager), outer) / inner
    short_us = {"select": repeated_us(st_select), "gather": repeated_us(st_gather), "accept": repeated_us(st_accept)}

    score_flops = 2.0 * T * hq * d * (V + (T + 1) / 2.0)          # one sweep of the contraction
    score_tflops = score_flops * L / (stage_ms["score"]["mean"] * 1e-3) / 1e12
    gather_bytes = 2 * 2 * dl * n_pruned * dkv * dd * 2
    decode_ms = stage_ms["draft_attn"]["mean"] + stage_ms["verify_attn"]["mean"] + stage_ms["accept"]["mean"]
    decode_steps_per_s = 1e3 / decode_ms                                     # as timed inside the step

    result = {
        "metric": "verify-step attn HBM GB/s (% peak); prune+gather us; decode steps/s",
        "value": round(attn_gbs["mean"], 1),
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
                   "score_row_lse": "supplied (torch logsumexp at set-up, untimed)" if args.score_lse else "computed",
                   "score_call": "one call per layer" if args.score_per_layer else "one call for all layers",
                   "launch": "eager" if args.eager else "hip-graph per stage"},
        "value_source": "verify_attn stage inside the timed steps (mean over steps)",
        "in_step_note": "inside a step the verify stage is the first pass over the 4.2 GB cache after the other stages ran; a "
                        "pass that follows another pass over the same cache (the isolated figure beside it) is 0.5-1 us "
                        "per layer faster; an idle gap after the score stage changes neither",
        "pct_of_hbm_peak": round(100.0 * attn_gbs["mean"] / HBM_PEAK_GBS, 1),
        "verify_attn_us_per_layer": {k: round(v, 3) for k, v in layer_us.items()},
        "verify_attn_gbs": {k: round(v, 1) for k, v in attn_gbs.items()},
        "verify_attn_us_per_layer_isolated_replays": round(isolated_us, 3),
        "verify_attn_gbs_isolated_replays": round(attn_bytes / (isolated_us * 1e-6) / 1e9, 1),
        "prune_gather_us": round(short_us["select"] + short_us["gather"], 1),
        "prune_gather_us_in_step": round((stage_ms["select"]["mean"] + stage_ms["gather"]["mean"]) * 1e3, 1),
        "select_us": round(short_us["select"], 2), "gather_us": round(short_us["gather"], 2),
        "accept_us": round(short_us["accept"], 2),
        "decode_steps_per_s": round(decode_steps_per_s, 1),
        "tokens_per_step_mean": round(tokens_per_step, 3),
        "tokens_per_step_sample": f"mean(n_accepted)+1 over {n_draws} seeded accept inputs; the step uses draw {pick}",
        "decode_tokens_per_s": round(decode_steps_per_s * tokens_per_step, 1),
        "stage_ms": {k: {kk: round(vv, 4) for kk, vv in v.items()} for k, v in stage_ms.items()},
        "score_tflops_one_sweep_counted": round(score_tflops, 1),
        "score_pct_mfma_peak": round(100.0 * score_tflops / MFMA_BF16_PEAK_TFLOPS, 2),
        "score_us_per_layer": round(stage_ms["score"]["mean"] * 1e3 / L, 2),
        "draft_attn_us_per_layer": round(stage_ms["draft_attn"]["mean"] * 1e3 / (w.gamma * dl), 3),
        "gather_gbs": round(gather_bytes / (short_us["gather"] * 1e-6) / 1e9, 1),
        "n_accepted": int(n_acc.item()),
        "score_mass_on_video": round(float(scores.sum().item()), 4),
        "roofline": {"kernel": "specvlm_decode_attn (verify: attn_split_kernel + attn_merge_kernel per layer)",
                     "bound": "hbm", "achieved": round(attn_gbs["mean"], 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(attn_gbs["mean"] / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(ws_attn_bytes),
                     "algorithmic_bytes_per_launch": attn_bytes,
                     "avg_launch_us": round(layer_us["mean"], 3),
                     "read_ceiling_us": round(read_ceiling_us, 3),
                     "read_ceiling_note": "one plain-read launch over the same layer's K and V (specvlm_probe_read), "
                                          "timed the same way"},
    }

    if not args.no_other_workloads:
        other = {}
        for name, layout in (("32b-long", "head-major"), ("ragged-x8", "head-major"), ("ragged-x8", "token-major")):
            r = attn_only(args, torch, B, synth, name, layout, 0, 10, 2)
            other[f"verify_attn {name} {layout}"] = {
                "us_per_layer": r["verify_attn_us_per_layer"], "gbs": r["value"],
                "pct_of_hbm_peak": round(100.0 * r["value"] / HBM_PEAK_GBS, 1), "shape": r["config"]["workload"]}
        # tree verification at the 72B shape: a seeded 26-node static tree (208 query rows per kv head, four
        # row groups) whose nodes are the last 26 rows of the same caches
        n_nodes = 26
        tmask = torch.from_numpy(synth.ancestor_masks(synth.make_tree(n_nodes, seed=synth.SEED_BASE + 26))
                                 .view(np.int64)).to(dev)
        q_tree = randn_bf16((L, n_nodes, hq, d))
        out_t = torch.empty((n_nodes, hq, d), dtype=torch.bfloat16, device=dev)
        ws_t = B.new_workspace(B.decode_attn_workspace_bytes(1, n_nodes, kv_len, hq, hkv, d, 0), dev)
        us_t = timed_replays(torch, graph_of(torch, lambda: [B.tree_attn(q_tree[l], k_all[l], v_all[l], scale, tmask,
                                                                         out=out_t, workspace=ws_t)
                                                             for l in range(L)], args.eager), 5) / L
        tree_bytes = 2 * kv_len * hkv * d * 2 + 2 * n_nodes * hq * d * 2
        other["tree verify 26 nodes, 72b-full caches"] = {
            "us_per_layer": round(us_t, 2), "gbs": round(tree_bytes / (us_t * 1e-6) / 1e9, 1),
            "pct_of_hbm_peak": round(100.0 * tree_bytes / (us_t * 1e-6) / 1e9 / HBM_PEAK_GBS, 1),
            "note": "algorithmic bytes count K and V once; the four row groups of a head re-read them (L2)"}
        del q_tree
        # rejection-sampling accept at the long-video configuration's size (gamma 7, vocab 152 064)
        w3 = synth.scaled(synth.WORKLOADS["32b-long"], gamma=7)
        a3 = synth.make_accept_inputs(1, w3.gamma, w3.vocab, synth.SEED_BASE + 3077, greedy=False)
        a3 = {k: torch.from_numpy(v).to(dev) for k, v in a3.items()}
        ws3 = B.new_workspace(B.accept_workspace_bytes(1, w3.gamma, w3.vocab, True), dev)
        n3 = torch.zeros(1, dtype=torch.int32, device=dev)
        o3 = torch.zeros((1, w3.gamma + 1), dtype=torch.int32, device=dev)
        us3 = repeated_us(lambda: B.accept(a3["target_logits"], a3["draft_tokens"], draft_logits=a3["draft_logits"],
                                           uniforms=a3["uniforms"], workspace=ws3, n_accepted=n3, out_tokens=o3))
        acc_bytes = (2 * w3.gamma + 1) * w3.vocab * 4
        other["accept sampling gamma 7 vocab 152064"] = {"us": round(us3, 2), "bytes": acc_bytes,
                                                         "gbs": round(acc_bytes / (us3 * 1e-6) / 1e9, 1)}
        # Stage I sized by cumulative score mass (Eq. 6) on the step's own scores
        cnt = torch.empty(1, dtype=torch.int32, device=dev)
        us_tp = repeated_us(lambda: B.top_p_count(scores, 0.3, count=cnt))
        other[f"top_p_count lambda 0.3 over {V} video tokens"] = {"us": round(us_tp, 2), "count": int(cnt.item())}
        # gather at the self-speculation shape: the verifier's own cache (all layers, 8 kv heads, d 128), keep 10 %
        if args.layout == "head-major":
            big_k = torch.empty((L, hkv, n_pruned, d), dtype=torch.bfloat16, device=dev).permute(0, 2, 1, 3)
        else:
            big_k = torch.empty((L, n_pruned, hkv, d), dtype=torch.bfloat16, device=dev)
        big_v = torch.empty_like(big_k)
        us_g = timed_replays(torch, graph_of(torch, lambda: B.gather_kv(k_all[:, :n_ctx], v_all[:, :n_ctx], 0, V, keep,
                                                                         k_dst=big_k, v_dst=big_v), args.eager), 10)
        big_bytes = 2 * 2 * L * n_pruned * hkv * d * 2
        # beside it: the runtime's own contiguous device-to-device copy of as many bytes (K onto V), the yardstick
        # for "a copy on this machine"
        us_copy = timed_replays(torch, graph_of(torch, lambda: [big_v.copy_(big_k), big_v.copy_(big_k)], args.eager), 10)
        other[f"gather self-speculation shape ({L} layers x {n_pruned} kept rows x {hkv} kv heads d{d})"] = {
            "us": round(us_g, 1), "bytes_read_plus_written": big_bytes,
            "gbs": round(big_bytes / (us_g * 1e-6) / 1e9, 1),
            "pct_of_hbm_peak": round(100.0 * big_bytes / (us_g * 1e-6) / 1e9 / HBM_PEAK_GBS, 1),
            "plain_copy_of_as_many_bytes_us": round(us_copy, 1),
            "plain_copy_gbs": round(big_bytes / (us_copy * 1e-6) / 1e9, 1)}
        del big_k, big_v
        # gather at the long-video configuration's sizes: 64 layers x 8 kv heads x d 128, 32 768 video + 256 text
        # tokens, keep 10 / 25 / 50 % (1.85 / 4.4 / 8.7 GB read + written); uninitialised buffers (a row copy does
        # not look at the values), kept rows = a seeded random subset in ascending order
        w3g = synth.WORKLOADS["32b-long"]
        L3, h3, d3, V3, n3ctx = w3g.n_layers, w3g.n_kv_heads, w3g.head_dim, w3g.n_video, w3g.n_ctx
        src_k = torch.empty((L3, h3, n3ctx, d3), dtype=torch.bfloat16, device=dev).permute(0, 2, 1, 3)
        src_v = torch.empty_like(src_k)
        gen3 = torch.Generator(device=dev); gen3.manual_seed(synth.SEED_BASE + 3100)
        for pct in (10, 25, 50):
            b3 = (V3 * pct + 50) // 100
            keep3 = torch.randperm(V3, generator=gen3, device=dev)[:b3].sort().values.to(torch.int32)
            rows3 = n3ctx - V3 + b3
            dst_k = torch.empty((L3, h3, rows3, d3), dtype=torch.bfloat16, device=dev).permute(0, 2, 1, 3)
            dst_v = torch.empty_like(dst_k)
            us3g = timed_replays(torch, graph_of(torch, lambda: B.gather_kv(src_k, src_v, 0, V3, keep3, k_dst=dst_k,
                                                                            v_dst=dst_v), args.eager), 5)
            bytes3 = 2 * 2 * L3 * rows3 * h3 * d3 * 2
            other[f"gather 32b-long shape keep {pct}% ({L3} layers x {rows3} rows x {h3} kv heads d{d3})"] = {
                "us": round(us3g, 1), "bytes_read_plus_written": bytes3,
                "gbs": round(bytes3 / (us3g * 1e-6) / 1e9, 1),
                "pct_of_hbm_peak": round(100.0 * bytes3 / (us3g * 1e-6) / 1e9 / HBM_PEAK_GBS, 1)}
            del dst_k, dst_v, keep3
        del src_k, src_v
        result["other_workloads"] = other

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, host0, scores, keep, draft_k, acc, pick, attn_bytes, L, scale)
    print(json.dumps(result))


def cpu_baseline(w, host0, scores, keep, draft_k, acc, pick, attn_bytes, L, scale):
    """The fp64 oracle as it stands, on the host cores, over the same seeded layer-0 inputs: a bounded
    sample per stage (about 25 s in all), extrapolated to the step where the sample is a part of it."""
    import torch
    import oracle
    cores = len(os.sched_getaffinity(0))
    passes, t0 = 0, time.perf_counter()
    while True:
        oracle.decode_attn(host0["q_block"], host0["k"], host0["v"], scale, want_lse=False)
        passes += 1
        dt = time.perf_counter() - t0
        if dt >= 8.0 or dt * (passes + 1) / passes > 20.0:
            break
    base = {"value": round(attn_bytes * passes / dt / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "sample": f"{passes} passes of the verify attention of layer 0 of {L} "
                      f"(fp64 oracle, {dt:.1f} s, OpenMP over query rows)"}
    stages = {"verify_attn": {"ms_per_layer": round(dt * 1e3 / passes, 2),
                              "ms_per_step_extrapolated": round(dt * 1e3 / passes * L, 1)}}
    # score: one kv-head group of layer 0 (its q heads against its one kv head), extrapolated x groups x layers
    group = w.n_q_heads // w.n_kv_heads
    t0 = time.perf_counter()
    oracle.score(host0["q_text"][:, :group], host0["k"][:w.n_ctx, :1], 0, w.n_video, w.n_video, scale)
    dt_s = time.perf_counter() - t0
    stages["score"] = {"sample": f"one kv-head group ({group} q heads) of layer 0",
                       "s_sample": round(dt_s, 2),
                       "ms_per_layer_extrapolated": round(dt_s * 1e3 * w.n_kv_heads, 1),
                       "s_per_step_extrapolated": round(dt_s * w.n_kv_heads * L, 1)}
    s_host = scores.cpu().numpy()
    t0 = time.perf_counter()
    for _ in range(20):
        okeep, _ = oracle.select(s_host, w.k_top, w.keep_budget)
    stages["select"] = {"us": round((time.perf_counter() - t0) / 20 * 1e6, 1), "sample": "20 calls, the step's own scores",
                        "matches_gpu": bool(np.array_equal(okeep, keep.cpu().numpy()))}
    d0 = draft_k[0].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    t0 = time.perf_counter()
    for _ in range(5):
        oracle.gather_kv(d0, 0, w.n_video, okeep)
    dt_g = (time.perf_counter() - t0) / 5
    stages["gather"] = {"us_per_layer_one_of_K_V": round(dt_g * 1e6, 1),
                        "us_per_step_extrapolated": round(dt_g * 1e6 * 2 * w.draft_layers, 1),
                        "sample": "5 calls on draft layer 0's K (single thread memcpy loop)"}
    t0 = time.perf_counter()
    for _ in range(5):
        oracle.accept_greedy(acc["target_logits"][pick], acc["draft_tokens"][pick])
    stages["accept"] = {"us": round((time.perf_counter() - t0) / 5 * 1e6, 1), "sample": "5 greedy calls on the step's draw"}
    base["stages"] = stages
    return base


def attn_only(args, torch, B, synth, workload, layout, frames, steps, warmup):
    """Verify attention alone on another workload: `layers` distinct caches
    (more than the 256 MB Infinity Cache holds) replayed from one HIP graph."""
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.WORKLOADS[workload]
    if frames:
        w = synth.scaled(w, n_frames=frames)
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
    if layout == "head-major":
        k = [randn_bf16((hkv, total, d)).permute(1, 0, 2) for _ in range(layers)]
        v = [randn_bf16((hkv, total, d)).permute(1, 0, 2) for _ in range(layers)]
    else:
        k = [randn_bf16((total, hkv, d)) for _ in range(layers)]
        v = [randn_bf16((total, hkv, d)) for _ in range(layers)]
    q = [randn_bf16((batch * g1, hq, d)) for _ in range(layers)]
    out = torch.empty((batch * g1, hq, d), dtype=torch.bfloat16, device=dev)
    cu_q = torch.tensor(np.arange(batch + 1) * g1, dtype=torch.int32, device=dev) if batch > 1 else None
    cu_kv = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=dev) if batch > 1 else None
    ws = B.new_workspace(B.decode_attn_workspace_bytes(batch, g1, max(lens), hq, hkv, d, args.num_splits), dev)

    def stage():
        for l in range(layers):
            B.decode_attn(q[l], k[l], v[l], w.softmax_scale, cu_q=cu_q, cu_kv=cu_kv, max_q_len=g1,
                          max_kv_len=max(lens), out=out, num_splits=args.num_splits, workspace=ws)

    run = graph_of(torch, stage, args.eager)
    for _ in range(warmup):
        run()
    us = timed_replays(torch, run, steps) / layers
    gbs = attn_bytes / (us * 1e-6) / 1e9
    return {
        "metric": "verify-step attn HBM GB/s (% peak)", "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": round(us * layers / 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name} (verify attention only): batch {batch}, {total} keys, {hq}/{hkv} heads "
                               f"d{d}, gamma {w.gamma}, {layers} distinct layers",
                   "kv_layout": layout,
                   "num_splits": args.num_splits},
        "verify_attn_us_per_layer": round(us, 2),
        "roofline": {"kernel": "specvlm_decode_attn (verify, split + merge)", "bound": "hbm",
                     "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": attn_bytes}}


if __name__ == "__main__":
    main()
