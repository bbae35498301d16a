#!/usr/bin/env python3
"""Benchmark: draft-tree rounds per second at the LLaMA3-8B shape on one MI355X.

A step is one whole draft-plus-verify round of the hot path on seeded synthetic
inputs that are already resident in HBM: D x eagle2_expand, eagle2_rerank,
eagle2_tree_attn (one layer), eagle2_accept.  Prints ONE JSON line with the
throughput, the HBM roofline of the dominant kernel (the LM-head stream, timed
with HIP events on the launch stream) and the CPU oracle's speed on the same
round as a reported baseline.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
PROFILE_SUMMARY = {3: "profiles/round_cfg3_llama3_8b.md"}


def recorded_traffic(cfg_index):
    """HBM bytes per LM-head launch (fetch + write) as RECORDED in the kept rocprofv3 counter summary of this
    workload (two --pmc runs, FETCH_SIZE and WRITE_SIZE, scaled by a plain copy; the summary states the
    command).  It is read from that file, not measured by this run: the line that carries it is
    `lm-head HBM traffic per launch: <bytes> B`.  None when no summary is kept or the line is missing."""
    import re
    path = PROFILE_SUMMARY.get(cfg_index)
    if path is None:
        return None, None
    try:
        text = open(os.path.join(ROOT, path)).read()
    except OSError:
        return None, None
    m = re.search(r"lm-head HBM traffic per launch:\s*([0-9][0-9,]*)\s*B", text)
    return (int(m.group(1).replace(",", "")) if m else None), path


def algorithmic_bytes(cfg, plens):
    """LM head: one pass streams W once (H and the partials are negligible).  Attention, per
    layer: K and V of prefix + tree once, Q read and O written once."""
    el = 4 if cfg.dtype == "fp32" else 2
    lm = cfg.vocab * cfg.hidden * el
    attn = sum(2 * (P + cfg.n_tree) * cfg.n_kv_heads * cfg.head_dim * el
               + 2 * cfg.n_tree * cfg.n_q_heads * cfg.head_dim * el for P in plens)
    return lm, attn


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--with-draft-model", action="store_true",
                    help="also run the draft model's decoder layer before every LM-head pass (not the headline metric)")
    ap.add_argument("--fp8-kv", action="store_true",
                    help="keep the prefix KV cache as 8-bit E4M3 codes (eagle2_tree_attn_fp8kv; a variant, not the headline metric)")
    ap.add_argument("--attn-layers", type=int, default=0,
                    help="run eagle2_tree_attn over this many independent seeded KV layers per round instead of the "
                         "configuration's own count (secondary measurement: --config 3 --attn-layers 32)")
    ap.add_argument("--hip-graph", action="store_true",
                    help="capture the round once into a HIP graph and time replays instead of eager launches")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device copy five times (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures the one-GPU hot path only; --gpus must be 1 "
              "(no collectives or sharding exist in this repository).", file=sys.stderr)
        sys.exit(2)

    import torch
    import workloads as wl
    from paper_2406_16858_amd import DraftRound, eagle2_kernel_timing_enable, eagle2_kernel_timing_read

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    dev = "cuda"
    if args.calibrate_copy:
        n = 1 << 30
        src = torch.full((n,), 7, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes": n, "copies": 5}))
        return
    cfg = wl.get_config(args.config)
    if args.attn_layers > 0:
        cfg = cfg.scaled(n_layers=args.attn_layers)
    B, D, k, N, V = cfg.batch, cfg.depth, cfg.topk, cfg.n_tree, cfg.vocab

    # ---- inputs, resident in HBM -------------------------------------------------
    W = wl.make_lm_head(cfg, dev)
    H_all = wl.make_hidden_states(cfg, dev)
    plens = wl.make_prefix_lengths(cfg)
    modes_l = {"greedy": [0] * B, "sample": [1] * B, "mixed": [b % 2 for b in range(B)]}[cfg.accept]
    rnd = DraftRound(B, V, cfg.hidden, D, k, N, cfg.dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                     total_prefix=sum(plens), keep_draft_logits=any(modes_l), device=dev)
    layers = [wl.make_attention_inputs(cfg, dev, layer=l, prefix_lens=plens) for l in range(cfg.n_layers)]
    O = torch.empty_like(layers[0][0])
    if args.fp8_kv:
        if cfg.dtype != "bf16":
            sys.exit("bench.py: --fp8-kv needs a bf16 configuration")
        layers8 = []
        for (Q, Kp, Vp, Kt, Vt, off) in layers:
            K8, V8, ks, vs = wl.make_fp8_prefix(Kp, Vp)
            layers8.append((Q, K8, V8, ks, vs, Kt, Vt, off))
        del layers
    tl, _ = wl.make_target_logits(cfg, dev)
    ua, ub = wl.make_uniforms(cfg, dev)
    temp = torch.full((B,), cfg.temperature, dtype=torch.float32, device=dev)
    mode_t = torch.tensor(modes_l, dtype=torch.int32, device=dev)
    root = (torch.arange(B, dtype=torch.int32) * 3 + 7).to(dev)
    plen_t = torch.tensor(plens, dtype=torch.int32, device=dev)

    dm = None
    if args.with_draft_model:
        from paper_2406_16858_amd import DraftModel
        if cfg.name not in wl.DRAFT_LAYERS:
            sys.exit(f"bench.py: no draft-layer shape is defined for {cfg.name}; --with-draft-model works with "
                     f"{', '.join(wl.DRAFT_LAYERS)}")
        dl = wl.DRAFT_LAYERS[cfg.name]
        dcfg = wl.RoundConfig(**{**cfg.__dict__, "n_q_heads": dl.n_q_heads, "n_kv_heads": dl.n_kv_heads, "head_dim": dl.head_dim})
        dm = DraftModel(rnd, wl.make_draft_weights(cfg, dl, dev), dl.n_q_heads, dl.n_kv_heads, dl.head_dim, dl.intermediate,
                        dl.eps, dl.rope_theta, sum(plens))
        _, dKp, dVp, _, _, doff = wl.make_attention_inputs(dcfg, dev, layer=97, prefix_lens=plens)
        root_feat = H_all[:, 0, 0].contiguous()

    def one_round():
        if dm is None:
            rnd.expand_all(H_all, W)
        else:
            for d in range(D):
                dm.forward(d, root, root_feat, plen_t, dKp, dVp, doff)
                dm.expand(d, W)
        rnd.rerank(root, plen_t)
        if args.fp8_kv:
            for (Q, K8, V8, ks, vs, Kt, Vt, off) in layers8:
                rnd.tree_attn_fp8kv(Q, K8, V8, ks, vs, off, Kt, Vt, O, None)
        else:
            for (Q, Kp, Vp, Kt, Vt, off) in layers:
                rnd.tree_attn(Q, Kp, Vp, off, Kt, Vt, O, None)
        rnd.accept(mode_t, tl, temp, ua, ub)

    step = one_round
    if args.hip_graph:
        # every entry point only enqueues kernels on the current stream: the round records as it is
        one_round()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            one_round()
        step = graph.replay
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    rounds_per_s = B * 1e3 / ms_per_step

    # ---- spread of single rounds: an event pair around each of a few rounds (outside the timed region) ----
    n_single = max(3, min(20, args.steps))
    pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_single)]
    for e0, e1 in pairs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    singles = sorted(e0.elapsed_time(e1) for e0, e1 in pairs)

    # ---- dominant kernel: LM-head stream, HIP events on the launch stream --------
    eagle2_kernel_timing_enable(True)
    reps = max(3, min(10, args.steps))
    for _ in range(reps):
        one_round()
    torch.cuda.synchronize()
    lm_ms, lm_n = eagle2_kernel_timing_read(0)
    at_ms, at_n = eagle2_kernel_timing_read(1)
    eagle2_kernel_timing_enable(False)
    lm_bytes, attn_bytes = algorithmic_bytes(cfg, plens)
    if args.fp8_kv:                                    # the prefix rows are one byte per element
        attn_bytes -= sum(2 * P * cfg.n_kv_heads * cfg.head_dim for P in plens)
    lm_avg_ms = lm_ms / max(lm_n, 1)
    achieved = lm_bytes / (lm_avg_ms * 1e-3) / 1e9
    round_bytes = D * lm_bytes + cfg.n_layers * attn_bytes
    traffic, traffic_src = recorded_traffic(cfg.index)
    if traffic_src is not None:
        traffic_src = f"recorded counter run, {traffic_src} (not measured by this run)"
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic, "traffic_source": traffic_src,
                "kernel": "lmhead_kernel" if B * k <= 16 else "lmhead_gemm128_kernel (passes 1..D-1), lmhead_kernel (pass 0)",
                "bytes_per_launch": lm_bytes, "avg_launch_ms": round(lm_avg_ms, 5),
                "launches_timed": lm_n}
    extra = {"round_algorithmic_bytes": round_bytes,
             "round_hbm_roofline_frac": round(round_bytes / (ms_per_step * 1e-3) / (HBM_PEAK_GBS * 1e9), 4),
             "attn_kernel_avg_ms": round(at_ms / max(at_n, 1), 5),
             "single_round_ms": {"median": round(singles[len(singles) // 2], 4), "min": round(singles[0], 4), "rounds": n_single},
             "launch": "hip graph replay" if args.hip_graph else "eager"}

    # ---- the oracle on the host cores, same round, bounded sample ------------------
    cpu = None
    if not args.no_cpu_baseline and not args.fp8_kv:
        import numpy as np
        from oracle import eagle2_oracle as orc
        from tests.parity_utils import f64
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        W_h, H_h = W.float().cpu().numpy(), f64(H_all)
        Q, Kp, Vp, Kt, Vt, off = [t.float().cpu().numpy() if t.dtype != torch.int64 else t.cpu().numpy() for t in layers[0]]
        tl_h = tl[0].cpu().numpy()
        ua_h, ub_h = ua[0].cpu().numpy(), ub[0].cpu().numpy()
        def oracle_round():
            st = orc.DraftState(D, k)
            dl = np.zeros((orc.n_draft_rows(D, k), V))
            for d in range(D):
                orc.expand(st, d, H_h[0, d, : (1 if d == 0 else k)], W_h, draft_logits=dl)
            tree = orc.rerank(st, N, 7, plens[0])
            orc.tree_attn(Q[0], Kp[: plens[0]], Vp[: plens[0]], Kt[0], Vt[0], tree.mask)
            if modes_l[0] == 0:
                orc.accept_greedy(tl_h, tree.token, tree.parent)
            else:
                orc.accept_sample(tl_h, dl, cfg.temperature, ua_h, ub_h, tree.token, tree.parent, tree.cand, k)

        # repeat the round of sequence 0 until about 10 s of host time have passed (at most 16 rounds)
        c0 = time.perf_counter()
        n_rounds = 0
        while n_rounds < 16 and (n_rounds == 0 or time.perf_counter() - c0 < 10.0):
            oracle_round()
            n_rounds += 1
        c1 = time.perf_counter()
        cpu = {"value": round(n_rounds / (c1 - c0), 5), "unit": "rounds/s", "cores": int(cores), "kind": "oracle",
               "sample": f"{n_rounds} full rounds of sequence 0 of {cfg.name} (all {D} passes, 1 attention layer, accept), "
                         f"{c1 - c0:.1f} s of host time"}

    name = "draft_tree_rounds_per_sec_llama3_8b_shape" if cfg.index == 3 else f"draft_tree_rounds_per_sec_{cfg.name}"
    if dm is not None:
        name += "_with_draft_model"
    if args.fp8_kv:
        name += "_fp8_prefix_kv"
    if args.attn_layers > 0:
        name += f"_attn_layers_{args.attn_layers}"
    if args.hip_graph:
        name += "_hip_graph"
    out = {"metric": name,
           "value": round(rounds_per_s, 2), "unit": "rounds/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
           "config": {"workload": f"cfg{cfg.index} {cfg.name}: V={V} Hd={cfg.hidden} D={D} k={k} N={N} B={B} "
                                  f"Hq/Hkv={cfg.n_q_heads}/{cfg.n_kv_heads} dh={cfg.head_dim} P={cfg.prefix_lo}"
                                  f"{'' if cfg.prefix_lo == cfg.prefix_hi else '..' + str(cfg.prefix_hi)} "
                                  f"layers={cfg.n_layers} accept={cfg.accept}",
                      "global_batch": B, "round": ("6x (draft layer + expand)" if dm is not None else "6x expand") + " + rerank + tree_attn + accept"},
           "roofline": roofline, "cpu_baseline": cpu, **extra}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
