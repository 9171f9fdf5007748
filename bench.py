#!/usr/bin/env python3
"""Benchmark of the DREAM decode-step hot path on one MI355X.

One step = one decode round on one batch of synthetic input:
  n_layers x dream_tree_verify_attn (one call per target layer, each over its own K/V cache)
  + 6 x dream_draft_xattn (one call per drafted tree level)
  + dream_accept_path.
dream_visual_compress (scores over all prefill rows, top-k keep, row gather) runs once per request, after the
prefill, not once per step: it is timed separately (`per_request_us`) and is not part of `value`.
All inputs are resident in HBM before the timed region.  The timed step is ONE HIP graph holding the three
phases (no memset nodes), replayed K times.  After the timed region the same work runs once more as one
graph per phase with HIP events between the graph launches, on the launching stream: that gives the phase
breakdown and the time of the verification block, from which the roofline figure of the dominant kernel
is derived.

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
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PAPER_TAU = {"llava": 5.51, "pixtral": 3.78, "gemma3": 2.36, "smolvlm_b1": 3.09, "smolvlm_b8": 3.09, "smolvlm_b32": 3.09}
PLANT_DEPTH = 4   # accepted drafted tokens per step in the synthetic logits (5 tokens a step with the bonus)


def verify_bytes_per_launch(cfg) -> int:
    """Algorithmic bytes of one dream_tree_verify_attn call: K and V rows once, Q in, O out."""
    S = cfg.prefix + cfg.n_tree
    e = cfg.elem_bytes
    return 2 * cfg.batch * cfg.n_kv_heads * S * cfg.head_dim * e + 2 * cfg.batch * cfg.n_q_heads * cfg.n_tree * cfg.head_dim * e


def read_traffic(name: str, plan: str):
    """HBM traffic per launch of the verification kernel, from the committed summary of the two rocprofv3 --pmc runs
    (FETCH_SIZE, WRITE_SIZE; counters cannot be read from inside this process).  Returns (bytes or None, where the
    figure comes from: file, the kernel it was measured on and the date of that measurement).  A figure measured on
    another kernel than the one the launch plan names now is stale: it is dropped and the source says so."""
    rel = os.path.join("profiles", f"attn_verify_{name}_traffic.txt")
    traffic, kernel, date = None, "?", "?"
    try:
        for line in open(os.path.join(ROOT, rel)):
            key, _, val = line.partition(":")
            if key == "traffic_bytes_per_launch":
                traffic = float(val)
            elif key == "kernel":
                kernel = val.strip()
            elif key == "measured":
                date = val.strip()
    except OSError:
        return None, "no rocprofv3 summary committed for this configuration"
    if kernel != plan.split(" ")[0]:
        return None, f"{rel} is stale: measured on {kernel} ({date}), the plan now names {plan.split(' ')[0]}"
    return traffic, f"{rel} (rocprofv3 --pmc FETCH_SIZE/WRITE_SIZE, kernel {kernel}, measured {date})"


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="llava")
    ap.add_argument("--layers", type=int, default=0, help="target layers per step (0 = the configuration's)")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-configs", action="store_true", help="skip the short runs of the other configurations")
    ap.add_argument("--splits", type=int, default=0, help="force the number of key-range splits (0 = automatic)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run plain device copies of a known size (reference for scaling rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        return 2

    import torch
    import dream_inputs as di
    import paper_2505_19201_amd as dream

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    dream.load()
    torch.cuda.set_device(0)
    dream.dream_init()
    if args.copy_calibration:
        return copy_calibration(torch)
    if args.splits:
        dream.dream_set_kv_splits(args.splits)
    cfg = di.CONFIGS[args.config]
    out = run_config(torch, dream, di, args, cfg, args.steps, args.warmup, full=True)
    if not args.no_configs:
        # the other measurement shapes: a short run each (same step, same graph replay), the figures the report asks for
        out["configs"] = {}
        for name in ("llava", "pixtral", "gemma3", "smolvlm_b1", "smolvlm_b8", "smolvlm_b32"):
            if name == cfg.name:
                continue
            torch.cuda.empty_cache()
            r = run_config(torch, dream, di, args, di.CONFIGS[name], steps=max(5, min(args.steps, 20)), warmup=3, full=False)
            if di.CONFIGS[name].batch == 1:
                torch.cuda.empty_cache()
                r["streaming_regime"] = streaming_regime(torch, dream, di, di.CONFIGS[name])
            out["configs"][name] = {"step_latency_us": r["step_latency_us"], "tokens_per_s": r["value"], "streaming_regime": r.get("streaming_regime"),
                                    "tokens_per_s_at_paper_tau": r["tokens_per_s_at_paper_tau"], "phase_us": r["phase_us"],
                                    "per_request_us": r["per_request_us"], "per_call_us": r["per_call_us"], "roofline": r["roofline"], "read_ceiling": r["read_ceiling"],
                                    "workload": r["config"]["workload"]}
    if not args.no_cpu:
        out["cpu_baseline"] = cpu_baseline(cfg, args.layers or cfg.n_layers, out["config"]["tokens_per_step"])
    print(json.dumps(out))
    return 0


def run_config(torch, dream, di, args, cfg, steps, warmup, full):
    """Allocates one configuration's resident inputs, times `steps` replays of the step graph and the per-phase
    breakdown, and returns the result line as a dict (full=True adds the legs that are reported once)."""
    L = args.layers or cfg.n_layers
    dev = torch.device("cuda:0")
    B, T, Hq, Hkv, D, P = cfg.batch, cfg.n_tree, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.prefix
    S = P + T
    s_max = S
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)

    def randn(*shape):
        return torch.randn(*shape, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)

    # ---- resident inputs -------------------------------------------------------------------------
    parents_np = np.stack([di.config_tree(cfg, b) for b in range(B)])
    parent = dream.to_device(parents_np)
    prefix_len = torch.full((B,), P, dtype=torch.int32, device=dev)
    vq = [randn(B, T, Hq, D) for _ in range(L)]
    vk = [randn(B, Hkv, s_max, D) for _ in range(L)]
    vv = [randn(B, Hkv, s_max, D) for _ in range(L)]
    vout = [torch.empty(B, T, Hq, D, dtype=torch.bfloat16, device=dev) for _ in range(L)]
    desc = dream.attn_desc(B, Hq, Hkv, D, dream.BF16, s_max)
    ws_v = dream.alloc_workspace(dream.dream_tree_verify_attn_workspace(desc, T, S))

    levels = [np.stack([di.tree_levels(parents_np[b])[lv] for b in range(B)]) for lv in range(cfg.depth)]
    xk, xv = randn(B, Hkv, s_max, D), randn(B, Hkv, s_max, D)
    xq = [randn(B, lv.shape[1], Hq, D) for lv in levels]
    xnode = [dream.to_device(np.ascontiguousarray(lv, dtype=np.int32)) for lv in levels]
    xout = [torch.empty_like(t) for t in xq]
    ws_x = dream.alloc_workspace(max(dream.dream_draft_xattn_workspace(desc, lv.shape[1], S) for lv in levels))

    pq = randn(B, P, Hq, D)
    rows = randn(B, P, cfg.hidden)
    k_keep = (cfg.n_visual * cfg.keep_num + cfg.keep_den // 2) // cfg.keep_den
    kept = torch.empty(B, k_keep, dtype=torch.int32, device=dev)
    gathered = torch.empty(B, k_keep, cfg.hidden, dtype=torch.bfloat16, device=dev)
    scores = torch.empty(B, cfg.n_visual, dtype=torch.float32, device=dev)
    ws_c = dream.alloc_workspace(dream.dream_visual_compress_workspace(desc, P, cfg.n_visual))

    lg_np, tok_np, par_np, _ = di.accept_inputs(cfg, plant_depths=[PLANT_DEPTH] * B)
    logits = dream.to_device(lg_np, "bf16")
    token = dream.to_device(tok_np)
    node_argmax = torch.empty(B, T, dtype=torch.int32, device=dev)
    accept_len = torch.empty(B, dtype=torch.int32, device=dev)
    accept_path = torch.empty(B, cfg.depth + 1, dtype=torch.int32, device=dev)
    bonus = torch.empty(B, dtype=torch.int32, device=dev)
    ws_a = dream.alloc_workspace(dream.dream_accept_path_workspace(B, T, cfg.vocab))

    def phase_verify():
        for l in range(L):
            dream.dream_tree_verify_attn(desc, vq[l], vk[l], vv[l], prefix_len, T, parent, None, S, vout[l], None, ws_v)

    def phase_xattn():
        for i in range(len(levels)):
            dream.dream_draft_xattn(desc, xq[i], xk, xv, prefix_len, T, parent, levels[i].shape[1], xnode[i], S, xout[i], ws_x)

    def phase_accept():
        dream.dream_accept_path(logits, dream.BF16, B, T, cfg.vocab, token, parent, cfg.depth, node_argmax, accept_len,
                                accept_path, bonus, ws_a)

    def per_request_compress():
        dream.dream_visual_compress(desc, pq, None, P, vk[L - 1], P, 0, cfg.n_visual, cfg.keep_num, cfg.keep_den, None,
                                    scores, kept, rows, P, gathered, cfg.hidden, ws_c)

    # A step is one decode round: the verification attention of every target layer, the cross-attention of every drafted
    # level and the acceptance.  The visual-token compression runs once per request (after the prefill), not per step:
    # it is timed on its own below and is not part of `value`.
    phases = [("verify", phase_verify), ("xattn", phase_xattn), ("accept", phase_accept)]
    for _, f in phases:      # eager warm-up before any capture
        f()
    per_request_compress()
    torch.cuda.synchronize()

    stream = torch.cuda.Stream()
    runners = []
    if args.no_graph:
        runners = [f for _, f in phases]

        def whole_step():
            for f in runners:
                f()
    else:
        for _, f in phases:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                f()
            runners.append(g.replay)
        # the timed step is ONE graph holding all phases; the per-phase graphs above only serve the breakdown
        step_graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(step_graph, stream=stream):
            for _, f in phases:
                f()
        whole_step = step_graph.replay
    torch.cuda.synchronize()

    def one_step(evs):
        for i, r in enumerate(runners):
            evs[i].record()
            r()
        evs[len(runners)].record()

    with torch.cuda.stream(stream):
        for _ in range(warmup):
            whole_step()
        stream.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            whole_step()
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        # phase breakdown (outside the timed region): the same work as one graph per phase with events between
        all_evs = [[torch.cuda.Event(enable_timing=True) for _ in range(len(runners) + 1)] for _ in range(steps)]
        for s in range(steps):
            one_step(all_evs[s])
        stream.synchronize()
        torch.cuda.synchronize()

    ms_per_step = (t1 - t0) * 1e3 / steps
    phase_ms = [float(np.mean([all_evs[s][i].elapsed_time(all_evs[s][i + 1]) for s in range(steps)]))
                for i in range(len(runners))]
    tokens_per_step = int((accept_len + 1).sum().item())
    assert tokens_per_step == B * (PLANT_DEPTH + 1), "accept_path did not return the planted path"
    value = tokens_per_step / (ms_per_step * 1e-3)
    compress_us = graph_time_us(torch, lambda: [per_request_compress() for _ in range(4)], reps=5) / 4
    # the same call when the caller brings the rows' log-sum-exps (what the prefill attention leaves): one score pass
    row_lse = torch.zeros(B, Hq, P, dtype=torch.float32, device=dev)

    def compress_with_lse():
        dream.dream_visual_compress(desc, pq, None, P, vk[L - 1], P, 0, cfg.n_visual, cfg.keep_num, cfg.keep_den, None,
                                    scores, kept, rows, P, gathered, cfg.hidden, ws_c, row_lse_in=row_lse)
    compress_with_lse()
    torch.cuda.synchronize()
    compress_lse_us = graph_time_us(torch, lambda: [compress_with_lse() for _ in range(4)], reps=5) / 4

    accept_call_us = graph_time_us(torch, lambda: [phase_accept() for _ in range(8)], reps=5) / 8
    xattn_call_us = graph_time_us(torch, lambda: [phase_xattn() for _ in range(2)], reps=5) / (2 * len(levels))
    launch_us = phase_ms[0] * 1e3 / L
    bytes_launch = verify_bytes_per_launch(cfg)
    achieved = bytes_launch / (launch_us * 1e-6) / 1e9
    plan = dream.dream_attn_plan_describe(desc, T, S)
    traffic, traffic_source = read_traffic(cfg.name, plan)
    roofline = {"bound": "hbm", "kernel": "dream_tree_verify_attn: " + plan, "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "traffic_source": traffic_source, "bytes_per_launch": bytes_launch,
                "launch_us": round(launch_us, 3), "launches_per_step": L}

    out = {
        "metric": "verify+draft step throughput (tokens/s) and latency on 1 MI355X",
        "value": round(value, 1), "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_per_step, 5), "step_latency_us": round(ms_per_step * 1e3, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: B={B} Hq={Hq} Hkv={Hkv} D={D} prefix={cfg.n_visual}+{cfg.n_text} tree={T} "
                               f"depth={cfg.depth} layers={L} vocab={cfg.vocab} keep={cfg.keep_num}/{cfg.keep_den}",
                   "step": f"{L} x dream_tree_verify_attn + {len(levels)} x dream_draft_xattn + dream_accept_path, one HIP graph",
                   "tokens_per_step": tokens_per_step, "hip_graph": not args.no_graph,
                   "kv_splits": args.splits or "auto"},
        "phase_us": {n: round(ms * 1e3, 2) for (n, _), ms in zip(phases, phase_ms)},
        "per_request_us": {"visual_compress": round(compress_us, 2), "visual_compress_given_row_lse": round(compress_lse_us, 2)},
        # the phases above are one graph each, so each carries a graph launch (several us); per call inside a graph:
        "per_call_us": {"accept_path": round(accept_call_us, 2), "draft_xattn_level": round(xattn_call_us, 2)},
        "step_with_compress_us": round(ms_per_step * 1e3 + compress_us, 2),
        "tokens_per_s_at_paper_tau": round(B * PAPER_TAU.get(cfg.name, 0.0) / (ms_per_step * 1e-3), 1),
        "roofline": roofline,
    }
    out["read_ceiling"] = read_ceiling(torch, dream, bytes_launch, L)
    if full:
        out["next_rows"] = {"spec_accept": spec_accept_leg(torch, dream, logits, token, parent, cfg),
                            "attention_entropy": entropy_leg(torch, dream, desc, pq, vk[L - 1], P),
                            "tree_build": tree_build_leg(torch, dream, di, cfg),
                            "project": project_leg(torch, dream, desc, xk, xv, prefix_len, xnode[1], cfg),
                            "kv_commit": kv_commit_leg(torch, dream, desc, vk + vv, prefix_len, T, accept_path, accept_len, cfg)}
        out["streaming_regime"] = streaming_regime(torch, dream, di, cfg)
    return out


def graph_time_us(torch, body, reps=20, warm=3):
    """Capture `body()` (library calls only) into one HIP graph on a side stream and return the mean time of
    one replay in microseconds, by HIP events on that stream.  `body` must have run eagerly once before."""
    stream = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=stream):
        body()
    with torch.cuda.stream(stream):
        for _ in range(warm):
            g.replay()
        stream.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        stream.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps


def read_ceiling(torch, dream, bytes_launch, L):
    """What a launch that only READS the verification kernel's algorithmic bytes costs: L back-to-back launches
    of the library's plain 16-byte-load read kernel over L distinct buffers, replayed as a HIP graph like the
    verification phase.  The attention kernel cannot beat this; it is the ceiling the roofline fraction of a
    single-sequence launch should be read against."""
    n = (bytes_launch + 15) // 16 * 16
    buf = torch.empty(L * n, dtype=torch.uint8, device="cuda").random_(0, 255)
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")

    def run():
        for l in range(L):
            dream.dream_stream_read(buf, n, sink, offset_bytes=l * n)
    run()
    torch.cuda.synchronize()
    us = graph_time_us(torch, run) / L
    gbs = n / (us * 1e-6) / 1e9
    return {"kernel": "stream_read_kernel (16-byte loads, no writes)", "bytes_per_launch": n, "launch_us": round(us, 3),
            "achieved": round(gbs, 1), "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4)}


def spec_accept_leg(torch, dream, logits, token, parent, cfg):
    """Acceptance at temperature 1 over the same tree and target logits as the greedy phase (not part of `value`),
    with draft logits = target logits + noise and seeded uniforms; 4 calls per graph."""
    B, T, V = logits.shape
    g = torch.Generator(device="cuda")
    g.manual_seed(cfg.seed)
    dlogits = (logits.float() + 0.7 * torch.randn(B, T, V, device="cuda", generator=g)).to(torch.bfloat16)
    ua = torch.rand(B, T, device="cuda", generator=g)
    ub = torch.rand(B, device="cuda", generator=g)
    alen = torch.empty(B, dtype=torch.int32, device="cuda")
    path = torch.empty(B, cfg.depth + 1, dtype=torch.int32, device="cuda")
    bonus = torch.empty(B, dtype=torch.int32, device="cuda")
    ws = dream.alloc_workspace(dream.dream_spec_accept_workspace(B, T, V))

    def run():
        dream.dream_spec_accept(logits, dlogits, dream.BF16, B, T, V, token, parent, ua, ub, cfg.depth, 1.0, alen, path, bonus, ws)
    run()
    torch.cuda.synchronize()
    us = graph_time_us(torch, lambda: [run() for _ in range(4)]) / 4
    return {"temperature": 1.0, "us": round(us, 2), "mean_accept_len": round(float(alen.float().mean().item()), 3)}


def entropy_leg(torch, dream, desc, pq, k_cache, P):
    """Eq. 2's attention entropy of one layer over all prefill rows (not part of `value`): the log-sum-exp pass
    with one more running sum plus a small reduction, 4 calls per graph."""
    B, Hq = pq.shape[0], pq.shape[2]
    row = torch.empty(B, Hq, P, dtype=torch.float32, device="cuda")
    ae = torch.empty(B, dtype=torch.float32, device="cuda")
    ws = dream.alloc_workspace(dream.dream_attention_entropy_workspace(desc, P))
    dream.dream_attention_entropy(desc, pq, None, P, k_cache, P, row, ae, ws)
    torch.cuda.synchronize()
    us = graph_time_us(torch, lambda: [dream.dream_attention_entropy(desc, pq, None, P, k_cache, P, row, ae, ws) for _ in range(4)]) / 4
    return {"rows": P, "us": round(us, 2), "ae": [round(float(x), 4) for x in ae.cpu().tolist()[:4]]}


def tree_build_leg(torch, dream, di, cfg):
    """The step before verification (not part of `value`): the draft tree of the benchmarked shape is grown
    level by level (root top-10, then the 10 best candidates of a level expand 10 children each: 60 nodes of
    at most 510 candidates at depth 6) from synthetic draft logits already resident in HBM: `depth`
    dream_tree_expand_level calls and one dream_tree_finalize, replayed as one HIP graph."""
    B, V, depth, k = cfg.batch, cfg.vocab, cfg.depth, 10
    budget = cfg.n_tree - 1
    dev = "cuda"
    levels = []
    for lv in range(depth):
        F = 1 if lv == 0 else k
        lg, cum = di.draft_level_inputs(B, F, V, "bf16", cfg.seed, level=lv)
        levels.append((dream.to_device(lg, "bf16"), dream.to_device(cum), F,
                       torch.empty(B, F, k, dtype=torch.int32, device=dev), torch.empty(B, F, k, dtype=torch.float32, device=dev),
                       torch.empty(B, min(k, F * k), dtype=torch.int32, device=dev)))
    ws = dream.alloc_workspace(dream.dream_tree_expand_workspace(B, k, V, k))
    n_pool = 1 + k + (depth - 1) * k * k
    pool_score = torch.randn(B, n_pool, device=dev).abs().neg().cumsum(1)    # decreasing scores: any ranking works for timing
    pool_parent = torch.arange(-1, n_pool - 1, dtype=torch.int32, device=dev).clamp(min=0).repeat(B, 1)
    pool_parent[:, 0] = -1
    pool_token = torch.randint(0, V, (B, n_pool), dtype=torch.int32, device=dev)
    T = 1 + min(budget, n_pool - 1)
    tp, tt, ti = (torch.empty(B, T, dtype=torch.int32, device=dev) for _ in range(3))

    def run():
        for lg, cum, F, tok, sc, nxt in levels:
            dream.dream_tree_expand_level(lg, dream.BF16, B, F, V, cum, k, tok, sc, nxt, ws)
        dream.dream_tree_finalize(pool_score, pool_parent, pool_token, B, n_pool, budget, tp, tt, ti)
    run()
    torch.cuda.synchronize()
    us = graph_time_us(torch, lambda: [run() for _ in range(4)]) / 4
    nbytes = sum(lv[0].numel() * 2 for lv in levels)
    return {"levels": depth, "k": k, "budget": budget, "launches": 2 * depth + 1, "us": round(us, 2), "logit_bytes": nbytes,
            "achieved_GBs": round(nbytes / (us * 1e-6) / 1e9, 1), "bound": "hbm (launch latency at one sequence)"}


def project_leg(torch, dream, desc, xk, xv, prefix_len, frontier, cfg):
    """Eq. 1's three linear maps for one draft level (not part of `value`): the frontier rows' queries
    (W_Q: hidden -> Hq D, dense output) and the same rows' keys and values written into the draft cache at
    prefix_len + node (W_K, W_V: hidden -> Hkv D).  The weights are read once per call and dominate the bytes;
    One launch per level carries all three maps; 4 levels per graph, each with its own weights (more than the
    last-level cache holds together), so every launch streams from HBM."""
    B, R = frontier.shape
    Hq, Hkv, D, hid = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.hidden
    per_graph = 4

    def rnd(*shape):
        return torch.randn(*shape, dtype=torch.float32, device="cuda").mul_(hid ** -0.5).to(torch.bfloat16)
    wq = [rnd(Hq * D, hid) for _ in range(per_graph)]
    wk = [rnd(Hkv * D, hid) for _ in range(per_graph)]
    wv = [rnd(Hkv * D, hid) for _ in range(per_graph)]
    e = torch.randn(B, R, hid, dtype=torch.float32, device="cuda").to(torch.bfloat16)
    s = torch.randn(B, R, hid, dtype=torch.float32, device="cuda").to(torch.bfloat16)
    q = torch.empty(B, R, Hq, D, dtype=torch.bfloat16, device="cuda")

    def run(i):
        dream.dream_project_rows_multi(desc, [(e, wq[i], Hq, None, None, q), (s, wk[i], Hkv, prefix_len, frontier, xk),
                                              (s, wv[i], Hkv, prefix_len, frontier, xv)], R, hid)
    run(0)
    torch.cuda.synchronize()
    us = graph_time_us(torch, lambda: [run(i) for i in range(per_graph)]) / per_graph
    nbytes = 2 * hid * (Hq + 2 * Hkv) * D + 2 * B * R * hid * 2 + 2 * B * R * (Hq + 2 * Hkv) * D
    return {"rows": B * R, "us_per_level": round(us, 2), "bytes": nbytes, "achieved_GBs": round(nbytes / (us * 1e-6) / 1e9, 1),
            "bound": "hbm"}


def kv_commit_leg(torch, dream, desc, caches, prefix_len, T, accept_path, accept_len, cfg):
    """The step that follows acceptance (not part of `value`): one dream_kv_commit launch moves the accepted
    path's rows in the K and V caches of every layer.  Timed as a replayed graph; it runs last because it
    rewrites the tree rows of the caches."""
    new_len = torch.empty_like(prefix_len)
    dream.dream_kv_commit(desc, caches, prefix_len, T, accept_path, accept_len, new_len)
    torch.cuda.synchronize()
    per_graph = 16   # a lone kernel per graph would time the graph launch, not the kernel
    us = graph_time_us(torch, lambda: [dream.dream_kv_commit(desc, caches, prefix_len, T, accept_path, accept_len, new_len)
                                       for _ in range(per_graph)]) / per_graph
    rows = int((accept_len + 1).sum().item())
    nbytes = 2 * len(caches) * cfg.n_kv_heads * rows * cfg.head_dim * 2   # read + write of the path rows
    assert new_len.cpu().tolist() == (prefix_len + accept_len + 1).cpu().tolist()
    return {"caches": len(caches), "launch_us": round(us, 3), "bytes": nbytes,
            "achieved_GBs": round(nbytes / (us * 1e-6) / 1e9, 1), "bound": "hbm"}


def copy_calibration(torch):
    """Plain device-to-device copies of 256 MiB: each launch reads 256 MiB and writes 256 MiB, which is what
    rocprofv3's FETCH_SIZE / WRITE_SIZE should report for it; the ratio scales the counters of other kernels."""
    n = 256 << 20
    src = torch.empty(n, dtype=torch.uint8, device="cuda")
    src.random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(5):
        dst.copy_(src)
    torch.cuda.synchronize()
    print(json.dumps({"copy_calibration": True, "bytes_read_per_launch": n, "bytes_written_per_launch": n, "launches": 5}))
    return 0


def streaming_regime(torch, dream, di, cfg, batch=32, iters=80, warm=320):
    """The same verification kernel on the same shape with `batch` sequences per launch: one launch then
    moves hundreds of MB, so its duration measures streaming efficiency rather than launch latency.
    Two cache sets are alternated so that nothing is served from the last-level cache; the launches are replayed as a
    HIP graph of 8.  The warm-up is 320 launches (about 25 ms): the launch time keeps falling for the first 15-20 ms of
    sustained load (5-10 % in all) while the clocks settle."""
    big = cfg.with_batch(batch) if cfg.batch < batch else cfg
    B, T, Hq, Hkv, D, P = big.batch, big.n_tree, big.n_q_heads, big.n_kv_heads, big.head_dim, big.prefix
    S = P + T
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(big.seed + 77)
    rn = lambda *s: torch.randn(*s, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)  # noqa: E731
    import numpy as np
    parent = dream.to_device(np.stack([di.config_tree(big, b) for b in range(B)]))
    pl = torch.full((B,), P, dtype=torch.int32, device=dev)
    sets = [(rn(B, T, Hq, D), rn(B, Hkv, S, D), rn(B, Hkv, S, D)) for _ in range(2)]
    out = torch.empty(B, T, Hq, D, dtype=torch.bfloat16, device=dev)
    desc = dream.attn_desc(B, Hq, Hkv, D, dream.BF16, S)
    ws = dream.alloc_workspace(dream.dream_tree_verify_attn_workspace(desc, T, S))

    def run(i):
        q, k, v = sets[i & 1]
        dream.dream_tree_verify_attn(desc, q, k, v, pl, T, parent, None, S, out, None, ws)

    run(0)
    torch.cuda.synchronize()
    per_graph = 8   # replayed as a graph, so that the host's launch path cannot be what is timed
    us = graph_time_us(torch, lambda: [run(i) for i in range(per_graph)], reps=max(1, iters // per_graph), warm=max(1, warm // per_graph)) / per_graph
    nbytes = verify_bytes_per_launch(big)
    gbs = nbytes / us / 1e3
    tflops = 4.0 * B * Hq * T * S * D / us / 1e6   # QK^T and PV, 2 flops per multiply-add, over all (row, key) pairs
    return {"workload": f"{big.name}: same shape, {B} sequences per launch", "bytes_per_launch": nbytes,
            "kernel": dream.dream_attn_plan_describe(desc, T, S),
            "launch_us": round(us, 2), "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(gbs / HBM_PEAK_GBS, 4), "mfma_tflops": round(tflops, 1), "mfma_frac_of_2500": round(tflops / 2500.0, 4)}


def cpu_baseline(cfg, L, tokens_per_step):
    """The float64 oracle, as it stands, timed on this host, once on all the threads it can use (at most 16) and once
    single-threaded: one verification layer (scaled by the layer count), the six cross-attention calls and the
    acceptance call, i.e. the same step as `value`; the per-request compression is timed beside it."""
    import dream_inputs as di
    import oracle

    x = di.verify_inputs(cfg)
    nb = min(cfg.batch, 2)   # bounded sample of the batch
    scale_b = cfg.batch / nb
    lg, tok, par, _ = di.accept_inputs(cfg, plant_depths=[PLANT_DEPTH] * cfg.batch)
    pq = np.ascontiguousarray(di.prefill_q(cfg)[:nb])
    feats = di.feature_rows(cfg)[:nb]

    def sub(a):
        return np.ascontiguousarray(a[:nb])

    def repeat(f, min_s):
        """Mean time of f() over as many calls as it takes to fill min_s seconds (at least 2)."""
        n, t0 = 0, time.perf_counter()
        while n < 2 or time.perf_counter() - t0 < min_s:
            f()
            n += 1
        return (time.perf_counter() - t0) / n, n

    reps = {}

    def timed(threads, with_compress, min_s):
        oracle.set_threads(threads)
        t_verify, reps["verify_layer"] = repeat(
            lambda: oracle.tree_attn(sub(x.q), sub(x.k), sub(x.v), cfg.dtype, x.prefix_len[:nb], x.parent[:nb], True), min_s)
        t_verify *= scale_b

        def all_levels():
            for lv in range(cfg.depth):
                rows = np.stack([di.tree_levels(x.parent[b])[lv] for b in range(nb)])
                qsel = np.stack([x.q[b, rows[b]] for b in range(nb)])
                oracle.tree_attn(qsel, sub(x.k), sub(x.v), cfg.dtype, x.prefix_len[:nb], x.parent[:nb], False, q_node=rows)
        t_xattn, reps["xattn"] = repeat(all_levels, min_s)
        t_xattn *= scale_b
        t_acc, reps["accept"] = repeat(
            lambda: oracle.accept_path(np.ascontiguousarray(lg[:nb]), cfg.dtype, tok[:nb], par[:nb], cfg.depth), min_s / 4)
        t_acc *= scale_b
        t_comp = None
        if with_compress:
            def compress():
                sc = oracle.visual_scores(pq, sub(x.k), cfg.dtype, 0, cfg.n_visual)
                kept = oracle.topk_keep(sc, 0, cfg.keep_num, cfg.keep_den)
                oracle.gather_rows(feats, cfg.dtype, kept)
            t_comp, reps["compress"] = repeat(compress, min_s)
            t_comp *= scale_b
        oracle.set_threads(1)
        step_s = L * t_verify + t_xattn + t_acc
        return step_s, {"verify_layer": round(t_verify, 4), "xattn": round(t_xattn, 4), "accept": round(t_acc, 5),
                        "per_request_compress": None if t_comp is None else round(t_comp, 4)}

    threads = min(16, oracle.hw_threads())
    step_s, parts = timed(threads, True, 2.0)
    reps_threaded = dict(reps)
    # the other reading of Section 3.3's score (a token's own attention weight left out): how many kept indices change
    oracle.set_threads(threads)
    sc_a = oracle.visual_scores(pq, sub(x.k), cfg.dtype, 0, cfg.n_visual)
    sc_b = oracle.visual_scores(pq, sub(x.k), cfg.dtype, 0, cfg.n_visual, include_diag=False)
    oracle.set_threads(1)
    kept_a, kept_b = oracle.topk_keep(sc_a, 0, cfg.keep_num, cfg.keep_den), oracle.topk_keep(sc_b, 0, cfg.keep_num, cfg.keep_den)
    diag_report = {"sequences": nb, "kept_per_sequence": int(kept_a.shape[1]),
                   "kept_indices_that_change": int(sum(len(set(kept_a[b]) - set(kept_b[b])) for b in range(nb)))}
    step_1, parts_1 = timed(1, cfg.batch == 1, 2.0)    # (the single-threaded compression of a batch would take minutes)
    return {"value": round(tokens_per_step / step_s, 3), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "step_s": round(step_s, 3), "host_nproc": os.cpu_count(), "host_hw_threads_seen_by_openmp": oracle.hw_threads(),
            "sample": f"{nb} of {cfg.batch} sequences; 1 of {L} verification layers timed and scaled by {L}; "
                      f"6 cross-attention calls and acceptance timed in full; compression (per request) timed beside the step; "
                      f"every part repeated for about 2 s and averaged (calls: {reps_threaded})",
            "parts_s": parts,
            "exclude_diagonal_reading": diag_report,
            "single_thread": {"value": round(tokens_per_step / step_1, 3), "unit": "tokens/s", "cores": 1, "step_s": round(step_1, 3),
                              "parts_s": parts_1}}


if __name__ == "__main__":
    sys.exit(main())
