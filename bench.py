#!/usr/bin/env python3
"""Benchmark of the block-sparse global-attention layer on one MI355X.

A step is one pass of the whole hot path over one synthetic batch that is already resident in
HBM: block pooling of Q and K, block scoring + selection, block-sparse attention.
The default workload is the headline shape: 100 frames x 1374 tokens = 137,400 tokens, 16 heads,
head dim 64, bf16, block 128, tau = 0.9.  The dense kernel is timed on the same inputs.

Prints ONE JSON line.  `value` is the kept-block throughput of the
whole layer: FLOPs of the kept (query block, key block) pairs, counting valid tokens only,
divided by the layer time.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0


def kept_flops(kv_idx, kv_cnt, n_tokens: int, block: int, block_k: int = 0) -> float:
    """4 * n_I * n_J * 64 summed over kept pairs, with n_I, n_J the valid tokens of each block
    (query blocks of `block` tokens, key blocks of `block_k`, default the same)."""
    import torch
    block_k = block_k or block
    H, nb, _ = kv_idx.shape
    nbk = -(-n_tokens // block_k)
    tail_k = n_tokens - (nbk - 1) * block_k
    cnt = kv_cnt.to(torch.int64)
    ar = torch.arange(kv_idx.shape[-1], device=kv_idx.device)[None, None, :]
    has_last = ((kv_idx == nbk - 1) & (ar < cnt[..., None])).any(-1)
    keys = cnt * block_k - has_last.to(torch.int64) * (block_k - tail_k)     # valid keys per row
    rows = torch.full((nb,), block, device=kv_idx.device, dtype=torch.int64)
    rows[-1] = n_tokens - (nb - 1) * block
    return float((keys * rows[None, :]).sum().item()) * 4.0 * 64.0


def measured_traffic(cfg_id: int):
    """HBM bytes per launch of the attention kernel, from the committed rocprofv3 --pmc summary
    (profiles/attention_hbm_traffic.txt, written from FETCH_SIZE / WRITE_SIZE runs); None if that
    workload has not been profiled."""
    path = os.path.join(ROOT, "profiles", "attention_hbm_traffic.txt")
    key = f"cfg{cfg_id}.hbm_bytes_per_launch"
    try:
        with open(path) as f:
            for line in f:
                if line.split("=")[0].strip() == key:
                    return float(line.split("=")[1])
    except (OSError, ValueError, IndexError):
        pass
    return None


def cpu_baseline(cfg, tau: float, budget_s: float = 20.0):
    """Times the fp64 numpy oracle on a bounded sample of the same workload: one head's mask
    prediction over the full sequence, then masked attention for query blocks of that head until
    the time budget is used.  Returns kept-block TFLOP/s of the sampled work."""
    import numpy as np
    from oracle import bsga_oracle as O
    from workload import generate_head

    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    q, k, v = generate_head(cfg, 0)
    q, k, v = q[None], k[None], v[None]
    b, N = cfg.block, cfg.n_tokens
    t0 = time.perf_counter()
    mask = O.predict_mask(q, k, b, tau, 1.0)
    t_mask = time.perf_counter() - t0
    nb = mask.shape[-1]
    tail = N - (nb - 1) * b
    flops = 0.0
    done = 0
    t1 = time.perf_counter()
    order = [0, nb - 1] + list(range(1, nb - 1))
    for I in order:
        O.sparse_attention(q, k, v, mask, b, q_blocks=[I])
        n_i = tail if I == nb - 1 else b
        keys = int(mask[0, I].sum()) * b - (b - tail if mask[0, I, nb - 1] else 0)
        flops += 4.0 * 64.0 * n_i * keys
        done += 1
        if time.perf_counter() - t1 > budget_s:
            break
    t_attn = time.perf_counter() - t1
    # the mask prediction covers all nb rows of the head; charge the sampled rows their share
    t_total = t_attn + t_mask * done / nb
    return {
        "value": flops / t_total / 1e12,
        "unit": "TFLOP/s",
        "cores": int(threads),
        "kind": "oracle",
        "sample": f"head 0: mask prediction for all {nb} query blocks ({t_mask:.2f} s, charged pro rata) + masked "
                  f"attention of {done} query blocks over the full key range ({t_attn:.1f} s), fp64 numpy",
        "layer_seconds_extrapolated": t_total / done * nb * cfg.heads,
    }


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--cfg", type=int, default=4, help="workload id (1-5); 4 is the headline 100-frame shape")
    ap.add_argument("--tau", type=float, default=0.9)
    ap.add_argument("--rho", type=float, default=1.0)
    ap.add_argument("--dense-steps", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--sweep", action="store_true", help="also time the (tau, rho) sweep; rows go to stderr and into the JSON")
    ap.add_argument("--block", action="store_true",
                    help="also time one whole transformer block (projections + this layer + MLP, d_model 1024, random "
                         "weights) dense and sparse; goes into the JSON")
    ap.add_argument("--asym", action="store_true",
                    help="also time the layer with query blocks of 128 and key blocks of 64; goes into the JSON")
    ap.add_argument("--special", action="store_true",
                    help="also time the layer with the special-token split (gathers included); goes into the JSON")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run one 1 GiB device-to-device copy first (reference dispatch for scaling the "
                         "FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding or collectives are implemented); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2509_07120_amd as B
    from paper_2509_07120_amd.flop_model import attention_only_speedup, theoretical_speedup
    from workload import CONFIGS, generate

    cfg = CONFIGS[args.cfg]
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    t0 = time.time()
    q, k, v = generate(cfg)
    tq, tk, tv = (torch.from_numpy(x).to(dt).cuda() for x in (q, k, v))
    del q, k, v
    print(f"[bench] generated cfg {cfg.cfg_id} ({cfg.name}) in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)
    H, N, d = tq.shape
    b = cfg.block
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ws_bytes = B.bsga_attn_workspace_bytes(dt, H, N, d)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device="cuda")
    sel_ws = torch.empty(B.bsga_select_workspace_bytes(H, cfg.n_blocks, cfg.n_blocks), dtype=torch.uint8, device="cuda")
    out = torch.empty_like(tq)

    def layer(tau, rho, events=None):
        if events:
            events[0].record()
        qp, kp = B.bsga_pool_qk(tq, tk, b)
        if events:
            events[1].record()
        bits, idx, cnt = B.bsga_select_blocks(qp, kp, tau, rho, want_bits=False, workspace=sel_ws)
        if events:
            events[2].record()
        B.bsga_sparse_attn(tq, tk, tv, b, idx, cnt, out=out, workspace=ws)
        if events:
            events[3].record()
        return idx, cnt

    def run(tau, rho, steps, warmup):
        for _ in range(warmup):
            idx, cnt = layer(tau, rho)
        torch.cuda.synchronize()
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        t0 = time.perf_counter()
        for s in range(steps):
            idx, cnt = layer(tau, rho, evs[s])
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        stage = [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / steps for i in range(3)]
        print("[bench] attention ms per step: " + ", ".join(f"{e[2].elapsed_time(e[3]):.2f}" for e in evs), file=sys.stderr,
              flush=True)
        flops = kept_flops(idx, cnt, N, b)
        kept_frac = float(cnt.to(torch.float64).sum().item()) / (H * cfg.n_blocks * cfg.n_blocks)
        return wall_ms, stage, flops, kept_frac

    wall_ms, stage, flops, kept_frac = run(args.tau, args.rho, args.steps, args.warmup)

    # dense baseline on the same inputs
    dense_ms = None
    if args.dense_steps > 0:
        B.bsga_dense_attn(tq, tk, tv, out=out, workspace=ws)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.dense_steps):
            B.bsga_dense_attn(tq, tk, tv, out=out, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        dense_ms = e0.elapsed_time(e1) / args.dense_steps
    dense_flops = 4.0 * H * float(N) * float(N) * d

    sweep_rows = []
    if args.sweep:
        for tau, rho in [(0.8, 1.0), (0.9, 1.0), (0.95, 1.0), (0.0, 0.5), (0.0, 0.75), (0.0, 0.9)]:
            w, st, fl, kf = run(tau, rho, max(2, args.steps // 2), 1)
            row = {"tau": tau, "rho": rho, "kept_fraction": kf, "layer_ms": w, "pool_ms": st[0], "select_ms": st[1],
                   "attention_ms": st[2], "kept_tflops_layer": fl / (w * 1e-3) / 1e12,
                   "kept_tflops_attention": fl / (st[2] * 1e-3) / 1e12,
                   "speedup_vs_dense": (dense_ms / w) if dense_ms else None,
                   # upper bounds from the appendix's FLOP model: the attention kernel alone, and a whole
                   # VGGT-sized network at this sparsity
                   "bound_attention_speedup": attention_only_speedup(1.0 - kf),
                   "bound_end_to_end_speedup": theoretical_speedup(cfg.frames, cfg.tokens_per_frame, 1.0 - kf)}
            sweep_rows.append(row)
            print("[sweep] " + json.dumps(row), file=sys.stderr, flush=True)

    block_rows = []
    if args.block:
        flags = torch.arange(N) % cfg.tokens_per_frame < 5
        gx = torch.Generator().manual_seed(1)
        x = torch.randn(N, 1024, generator=gx).to(torch.bfloat16).cuda()
        for name, tau, rho, sp in [("dense", 1.0, 1.0, None), ("tau=0.9", 0.9, 1.0, None), ("tau=0.9, special split", 0.9, 1.0, flags),
                                   ("top-k rho=0.75, special split", 0.0, 0.75, flags)]:
            blk = B.GlobalAttentionBlock(1024, H, b, tau, rho, special=sp)
            blk(x)
            torch.cuda.synchronize()
            e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
            e0.record()
            a = blk.attention(x)
            e1.record()
            blk(x)
            e2.record()
            torch.cuda.synchronize()
            row = {"variant": name, "attention_with_projections_ms": e0.elapsed_time(e1), "block_ms": e1.elapsed_time(e2)}
            block_rows.append(row)
            print("[block] " + json.dumps(row), file=sys.stderr, flush=True)
            del blk, a
        del x

    asym_rows = []
    if args.asym and b == 128:
        nbk64 = -(-N // 64)
        ws64 = torch.empty(B.bsga_select_workspace_bytes(H, cfg.n_blocks, nbk64), dtype=torch.uint8, device="cuda")
        for tau, rho in [(args.tau, args.rho), (0.0, 0.5), (0.0, 0.75), (0.0, 0.9)]:
            def asym_layer(ev=None):
                if ev:
                    ev[0].record()
                qp, kp = B.bsga_pool(tq, 128), B.bsga_pool(tk, 64)
                _, idx, cnt = B.bsga_select_blocks(qp, kp, tau, rho, want_bits=False, workspace=ws64)
                if ev:
                    ev[1].record()
                B.bsga_sparse_attn(tq, tk, tv, 128, idx, cnt, out=out, workspace=ws, block_k=64)
                if ev:
                    ev[2].record()
                return idx, cnt
            asym_layer()
            torch.cuda.synchronize()
            steps = max(2, args.steps // 2)
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
            t0 = time.perf_counter()
            for s_ in range(steps):
                idx, cnt = asym_layer(evs[s_])
            torch.cuda.synchronize()
            w = (time.perf_counter() - t0) * 1e3 / steps
            st = [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / steps for i in range(2)]
            fl = kept_flops(idx, cnt, N, 128, 64)
            kf = float(cnt.to(torch.float64).sum().item()) / (H * cfg.n_blocks * nbk64)
            row = {"tau": tau, "rho": rho, "block_q": 128, "block_k": 64, "kept_fraction": kf, "layer_ms": w,
                   "pool_select_ms": st[0], "attention_ms": st[1], "kept_tflops_layer": fl / (w * 1e-3) / 1e12,
                   "speedup_vs_dense": (dense_ms / w) if dense_ms else None}
            asym_rows.append(row)
            print("[asym] " + json.dumps(row), file=sys.stderr, flush=True)
        del ws64

    special_rec = None
    if args.special:
        # Sec. 4.2: patch tokens first, special tokens last; block map on the pure patch blocks only
        import numpy as np
        flags = torch.from_numpy((np.arange(N) % cfg.tokens_per_frame) < 5)
        plan = B.SpecialTokenPlan(flags, b, "cuda")
        gq, gk, gv, go = (torch.empty_like(tq) for _ in range(4))
        out_sp = torch.empty_like(tq)

        def special_layer(tau, rho, ev=None):
            if ev:
                ev[0].record()
            for src, dst in ((tq, gq), (tk, gk), (tv, gv)):
                B.bsga_gather_tokens(src, plan.perm, out=dst)
            if ev:
                ev[1].record()
            qp, kp = B.bsga_pool_qk(gq, gk, b)
            _, idx, cnt = B.bsga_select_blocks(qp, kp, tau, rho, want_bits=False, workspace=sel_ws,
                                               force_q=plan.force_q, force_k=plan.force_k)
            if ev:
                ev[2].record()
            B.bsga_sparse_attn(gq, gk, gv, b, idx, cnt, out=go, workspace=ws)
            if ev:
                ev[3].record()
            B.bsga_gather_tokens(go, plan.inverse, out=out_sp)
            if ev:
                ev[4].record()
            return idx, cnt

        rows_sp = []
        for tau, rho in [(args.tau, args.rho), (0.0, 0.5), (0.0, 0.75), (0.0, 0.9)]:
            special_layer(tau, rho)
            torch.cuda.synchronize()
            steps = max(2, args.steps // 2)
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
            t0 = time.perf_counter()
            for s_ in range(steps):
                idx, cnt = special_layer(tau, rho, evs[s_])
            torch.cuda.synchronize()
            w = (time.perf_counter() - t0) * 1e3 / steps
            st = [sum(e[i].elapsed_time(e[i + 1]) for e in evs) / steps for i in range(4)]
            fl = kept_flops(idx, cnt, N, b)
            kf = float(cnt.to(torch.float64).sum().item()) / (H * cfg.n_blocks * cfg.n_blocks)
            row = {"tau": tau, "rho": rho, "kept_fraction": kf, "layer_ms": w, "gather_in_ms": st[0],
                   "pool_select_ms": st[1], "attention_ms": st[2], "gather_out_ms": st[3],
                   "gather_gbs": (2.0 * 4 * H * N * d * 2) / ((st[0] + st[3]) * 1e-3) / 1e9,
                   "kept_tflops_layer": fl / (w * 1e-3) / 1e12,
                   "speedup_vs_dense": (dense_ms / w) if dense_ms else None}
            rows_sp.append(row)
            print("[special] " + json.dumps(row), file=sys.stderr, flush=True)
        special_rec = {"n_patch_blocks": plan.n_patch_blocks, "n_blocks": cfg.n_blocks, "rows": rows_sp}

    attn_ms = stage[2]
    achieved = flops / (attn_ms * 1e-3) / 1e12
    value = flops / (wall_ms * 1e-3) / 1e12
    rec = {
        "metric": "global-attn layer ms + kept-block TFLOP/s (% bf16 peak) at 100 frames vs dense",
        "value": value,
        "unit": "TFLOP/s (kept-block FLOPs / whole layer time)",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall_ms,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": f"cfg{cfg.cfg_id}: {cfg.frames} frames x {cfg.tokens_per_frame} tokens = {N} tokens, "
                               f"{H} heads, d={d}, {cfg.dtype}, block {b}, tau={args.tau}, rho={args.rho}"},
        "layer_ms": wall_ms,
        "stage_ms": {"pool": stage[0], "select": stage[1], "attention": stage[2]},
        "pool_gbs": (2.0 * H * N * d * (2 if cfg.dtype == "bf16" else 4)) / (stage[0] * 1e-3) / 1e9,
        "kept_fraction": kept_frac,
        "pct_of_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "dense_ms": dense_ms,
        "dense_tflops": (dense_flops / (dense_ms * 1e-3) / 1e12) if dense_ms else None,
        "speedup_vs_dense": (dense_ms / wall_ms) if dense_ms else None,
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_traffic(cfg.cfg_id),
                     "kernel": f"attn_bf16_kernel<{b}> (block-sparse attention, one launch per step)",
                     "flops_per_launch": flops, "launch_ms": attn_ms},
    }
    if sweep_rows:
        rec["sweep"] = sweep_rows
    if special_rec:
        rec["special_token_split"] = special_rec
    if asym_rows:
        rec["query128_key64_blocks"] = asym_rows
    if block_rows:
        rec["transformer_block"] = block_rows
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(cfg, args.tau, args.cpu_budget)
    print(json.dumps(rec), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
