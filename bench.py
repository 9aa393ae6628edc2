#!/usr/bin/env python3
"""Benchmark of the block-sparse global-attention layer on one MI355X.

A step is one pass of the whole hot path over one synthetic batch that is already resident in
HBM: block pooling of Q and K, block scoring + selection (bit mask, index lists and counts),
block-sparse attention.  The headline workload is 100 frames x 1374 tokens = 137,400 tokens,
16 heads, head dim 64, bf16, block 128, tau = 0.9; the dense kernel is timed on the same inputs.

Prints ONE JSON line.  `value` is the kept-block throughput of the whole layer: FLOPs of the kept
(query block, key block) pairs, counting valid tokens only, divided by the layer time.  Besides
the headline the line carries `rows`: the same measurement at the other thresholds of the
100-frame shape, with top-k selection, with the special-token split, and at the other frame
counts / resolutions, each with its dense time on the same inputs.  Every buffer the layer writes
is allocated before the timed region; stage times are medians over the timed steps.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0
ATTN_SOURCE = os.path.join(ROOT, "paper_2509_07120_amd", "csrc", "attn_bf16.hip")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "attention_hbm_traffic.txt")


def kept_flops(kv_idx, kv_cnt, n_tokens: int, block: int, block_k: int = 0, n_first=None) -> float:
    """4 * n_I * n_J * 64 summed over kept pairs, with n_I, n_J the valid tokens of each block
    (query blocks of `block` tokens, key blocks of `block_k`, default the same; n_first: the
    sequence is split there and each part blocked separately)."""
    import torch
    block_k = block_k or block
    n_first = n_tokens if n_first is None else n_first

    def sizes(b):
        out = []
        for lo, hi in ((0, n_first), (n_first, n_tokens)):
            n = hi - lo
            full, rest = divmod(n, b)
            out += [b] * full + ([rest] if rest else [])
        return torch.tensor(out, dtype=torch.int64, device=kv_idx.device)

    q_sizes, k_sizes = sizes(block), sizes(block_k)
    H, nbq, stride = kv_idx.shape
    assert nbq == q_sizes.numel()
    ar = torch.arange(stride, device=kv_idx.device)[None, None, :]
    valid = ar < kv_cnt.to(torch.int64)[..., None]
    keys = (k_sizes[kv_idx.clamp(0, k_sizes.numel() - 1).to(torch.int64)] * valid).sum(-1)  # valid keys per row
    return float((keys * q_sizes[None, :]).sum().item()) * 4.0 * 64.0


def file_sha(path: str) -> str:
    with open(path, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def measured_traffic(cfg_id: int):
    """HBM-side bytes per launch of the attention kernel from the committed rocprofv3 --pmc summary
    (profiles/attention_hbm_traffic.txt, written by paper_2509_07120_amd/profile_summary.py from
    FETCH_SIZE / WRITE_SIZE runs).  The file names the hash of the kernel source it was measured
    with; for any other source the figure is stale and None is returned."""
    vals = {}
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                if "=" in line and not line.lstrip().startswith("#"):
                    k, v = line.split("=", 1)
                    vals[k.strip()] = v.strip()
        if vals.get("kernel_source_sha256_16") != file_sha(ATTN_SOURCE):
            return None
        return float(vals[f"cfg{cfg_id}.hbm_bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        return None


def cpu_baseline(cfg, tau: float, budget_s: float = 20.0):
    """Times the fp64 numpy oracle on a bounded sample of the same workload: one head's mask
    prediction over the full sequence, then masked attention for query blocks of that head until
    the time budget is used.  Returns kept-block TFLOP/s of the sampled work."""
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


class Workload:
    """One configuration resident on the GPU with every buffer the layer needs."""

    def __init__(self, B, torch, cfg):
        from workload import generate
        self.B, self.torch, self.cfg = B, torch, cfg
        dt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
        t0 = time.time()
        q, k, v = generate(cfg)
        self.q, self.k, self.v = (torch.from_numpy(x).to(dt).cuda() for x in (q, k, v))
        del q, k, v
        print(f"[bench] generated cfg {cfg.cfg_id} ({cfg.name}) in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)
        self.H, self.N, self.d = self.q.shape
        self.b = cfg.block
        self.elem = 2 if cfg.dtype == "bf16" else 4
        self.ws = torch.empty(max(B.bsga_attn_workspace_bytes(dt, self.H, self.N, self.d), 16), dtype=torch.uint8, device="cuda")
        self.out = torch.empty_like(self.q)
        self.dense_ms = None
        self._bufs = {}

    def buffers(self, nb):
        """Pooled vectors, selection workspace, mask bits, index lists and counts for nb blocks."""
        if nb not in self._bufs:
            t, H = self.torch, self.H
            self._bufs[nb] = {
                "pool": (t.empty((H, nb, 64), dtype=t.float64, device="cuda"), t.empty((H, nb, 64), dtype=t.float64, device="cuda")),
                "sel_ws": t.empty(self.B.bsga_select_workspace_bytes(H, nb, nb), dtype=t.uint8, device="cuda"),
                "sel": (t.empty((H, nb, (nb + 31) // 32), dtype=t.int32, device="cuda"),
                        t.empty((H, nb, nb), dtype=t.int32, device="cuda"), t.empty((H, nb), dtype=t.int32, device="cuda")),
            }
        return self._bufs[nb]

    # ---- the layer, uniform blocking (every token in one sequence of blocks) ------------------------
    def layer(self, tau, rho, ev=None):
        B, bufs = self.B, self.buffers(self.cfg.n_blocks)
        if ev:
            ev[0].record()
        qp, kp = B.bsga_pool_qk(self.q, self.k, self.b, out=bufs["pool"])
        if ev:
            ev[1].record()
        bits, idx, cnt = B.bsga_select_blocks(qp, kp, tau, rho, want_bits=True, workspace=bufs["sel_ws"], out=bufs["sel"])
        if ev:
            ev[2].record()
        B.bsga_sparse_attn(self.q, self.k, self.v, self.b, idx, cnt, out=self.out, workspace=self.ws)
        if ev:
            ev[3].record()
        return idx, cnt

    STAGES = ("pool", "select", "attention")

    # ---- the layer with the special-token split (Sec. 4.2): gathers in, split blocking, gather out -----
    def prepare_special(self):
        import numpy as np
        torch, B = self.torch, self.B
        flags = torch.from_numpy((np.arange(self.N) % self.cfg.tokens_per_frame) < 5)
        self.plan = B.SpecialTokenPlan(flags, self.b, "cuda")
        self.g = [torch.empty_like(self.q) for _ in range(4)]  # gathered q, k, v and the output before the gather back
        self.out_sp = torch.empty_like(self.q)

    def layer_special(self, tau, rho, ev=None):
        B, plan = self.B, self.plan
        bufs = self.buffers(plan.n_blocks)
        gq, gk, gv, go = self.g
        if ev:
            ev[0].record()
        for src, dst in ((self.q, gq), (self.k, gk), (self.v, gv)):
            B.bsga_gather_tokens(src, plan.perm, out=dst)
        if ev:
            ev[1].record()
        qp, kp = B.bsga_pool_qk_split(gq, gk, self.b, plan.n_patch, out=bufs["pool"])
        if ev:
            ev[2].record()
        bits, idx, cnt = B.bsga_select_blocks(qp, kp, tau, rho, want_bits=True, workspace=bufs["sel_ws"], out=bufs["sel"],
                                              force_q=plan.force_q, force_k=plan.force_k)
        if ev:
            ev[3].record()
        B.bsga_sparse_attn_split(gq, gk, gv, self.b, plan.n_patch, idx, cnt, out=go, workspace=self.ws)
        if ev:
            ev[4].record()
        B.bsga_gather_tokens(go, plan.inverse, out=self.out_sp)
        if ev:
            ev[5].record()
        return idx, cnt

    STAGES_SPECIAL = ("gather_in", "pool", "select", "attention", "gather_out")

    # ---- timing -----------------------------------------------------------------------------------
    def time_layer(self, fn, stages, tau, rho, steps, warmup):
        """Runs fn(tau, rho) `warmup` + `steps` times; returns wall ms per step over the timed steps
        (bracketed by synchronisations), per-stage event times of every step, and the lists."""
        torch = self.torch
        for _ in range(warmup):
            idx, cnt = fn(tau, rho)
        torch.cuda.synchronize()
        n_ev = len(stages) + 1
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(n_ev)] for _ in range(steps)]
        t0 = time.perf_counter()
        for s in range(steps):
            idx, cnt = fn(tau, rho, evs[s])
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        per_stage = {name: [e[i].elapsed_time(e[i + 1]) for e in evs] for i, name in enumerate(stages)}
        per_step = [e[0].elapsed_time(e[-1]) for e in evs]
        return wall_ms, per_stage, per_step, idx, cnt

    def time_dense(self, steps):
        if self.dense_ms is None:
            torch, B = self.torch, self.B
            B.bsga_dense_attn(self.q, self.k, self.v, out=self.out, workspace=self.ws)
            torch.cuda.synchronize()
            times = []
            for _ in range(steps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                B.bsga_dense_attn(self.q, self.k, self.v, out=self.out, workspace=self.ws)
                e1.record()
                torch.cuda.synchronize()
                times.append(e0.elapsed_time(e1))
            self.dense_ms = statistics.median(times)
        return self.dense_ms

    def row(self, tau, rho, steps, warmup, special=False, dense_steps=2):
        """One measured row: medians over `steps` timed steps."""
        from paper_2509_07120_amd.flop_model import attention_only_speedup, theoretical_speedup
        cfg, H, N = self.cfg, self.H, self.N
        if special and not hasattr(self, "plan"):
            self.prepare_special()
        fn, stages = (self.layer_special, self.STAGES_SPECIAL) if special else (self.layer, self.STAGES)
        wall_ms, per_stage, per_step, idx, cnt = self.time_layer(fn, stages, tau, rho, steps, warmup)
        nb = self.plan.n_blocks if special else cfg.n_blocks
        flops = kept_flops(idx, cnt, N, self.b, n_first=self.plan.n_patch if special else None)
        kept = float(cnt.to(self.torch.float64).sum().item())
        med = {k: statistics.median(v) for k, v in per_stage.items()}
        layer_ms = statistics.median(per_step)
        dense_ms = self.time_dense(dense_steps) if dense_steps > 0 else None
        dense_flops = 4.0 * H * float(N) * float(N) * self.d
        # bytes the selection stage reads and writes: pooled q and k in, fp64 block logits out and in
        # again, mask words, index lists (kept entries only) and counts out
        sel_bytes = 2.0 * H * nb * 64 * 8 + 2.0 * H * nb * nb * 8 + H * nb * ((nb + 31) // 32) * 4 + 4.0 * kept + 4.0 * H * nb
        row = {
            "workload": f"cfg{cfg.cfg_id}: {cfg.frames} frames x {cfg.tokens_per_frame} tokens = {N}, block {self.b}",
            "variant": "special-token split" if special else "all tokens in one block map",
            "tau": tau, "rho": rho, "steps": steps,
            "kept_fraction": kept / (H * nb * nb),
            "layer_ms": layer_ms,
            "stage_ms": med,
            "kept_tflops_layer": flops / (layer_ms * 1e-3) / 1e12,
            "frac_of_bf16_peak": flops / (layer_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
            "kept_tflops_attention": flops / (med["attention"] * 1e-3) / 1e12,
            "pool_gbs": (2.0 * H * N * self.d * self.elem) / (med["pool"] * 1e-3) / 1e9,
            "select_gbs": sel_bytes / (med["select"] * 1e-3) / 1e9,
            "dense_ms": dense_ms,
            "dense_tflops": (dense_flops / (dense_ms * 1e-3) / 1e12) if dense_ms else None,
            "speedup_vs_dense": (dense_ms / layer_ms) if dense_ms else None,
            # upper bounds from the appendix's FLOP model: the attention kernel alone, and a whole
            # network of the paper's size at this sparsity
            "bound_attention_speedup": attention_only_speedup(1.0 - kept / (H * nb * nb)),
            "bound_end_to_end_speedup": theoretical_speedup(cfg.frames, cfg.tokens_per_frame, 1.0 - kept / (H * nb * nb)),
        }
        if special:
            row["gather_gbs"] = (2.0 * 4 * H * N * self.d * self.elem) / ((med["gather_in"] + med["gather_out"]) * 1e-3) / 1e9
        extra = {"wall_ms": wall_ms, "flops": flops, "per_stage": per_stage, "per_step": per_step}
        return row, extra


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--cfg", type=int, default=4, help="headline workload id (1-6); 4 is the 100-frame shape")
    ap.add_argument("--tau", type=float, default=0.9)
    ap.add_argument("--rho", type=float, default=1.0)
    ap.add_argument("--dense-steps", type=int, default=3)
    ap.add_argument("--rows", choices=("all", "headline-config", "none"), default="all",
                    help="which further rows to measure: every threshold / variant / frame count (default), only those "
                         "on the headline configuration, or none (profiling runs)")
    ap.add_argument("--row-steps", type=int, default=5, help="timed steps per further row")
    ap.add_argument("--no-probe", action="store_true", help="skip the MFMA instruction-rate probe")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-budget", type=float, default=20.0)
    ap.add_argument("--block", action="store_true",
                    help="also time one whole transformer block (projections + this layer + MLP, d_model 1024, random "
                         "weights) dense and sparse; goes into the JSON")
    ap.add_argument("--asym", action="store_true",
                    help="also time the layer with query blocks of 128 and key blocks of 64; goes into the JSON")
    ap.add_argument("--locality", action="store_true",
                    help="also time the attention kernel on short rows (10 %% of the key blocks) whose lists are random per "
                         "row / identical within a head / a band around the row: separates tile locality from per-row "
                         "overhead; goes into the JSON")
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
    from workload import CONFIGS

    cfg = CONFIGS[args.cfg]
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").zero_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    w = Workload(B, torch, cfg)
    H, N, d, b = w.H, w.N, w.d, w.b

    # ---- headline: exactly --steps timed steps of the whole layer -------------------------------------
    head, extra = w.row(args.tau, args.rho, args.steps, args.warmup, dense_steps=args.dense_steps)
    print("[bench] attention ms per step: " + ", ".join(f"{x:.2f}" for x in extra["per_stage"]["attention"]), file=sys.stderr,
          flush=True)
    wall_ms, flops = extra["wall_ms"], extra["flops"]
    attn_mean_ms = statistics.fmean(extra["per_stage"]["attention"])

    # ---- what the matrix pipes sustain on this machine with no memory traffic (the part clocks down with
    # the switching activity of the operands; the attention kernel is to be read against these).  After
    # the headline, so that the headline is measured on a part in the state the driver hands over. ------
    probe = None
    if not args.no_probe:
        probe = {"what": "v_mfma_f32_32x32x16_bf16 only, registers only, 2 workgroups x 4 waves per CU; 'softmax' adds, "
                         "per MFMA, 2 exp2 + 1 bf16 pack and the row sum of the two weights (by 2 fp32 adds, or, as the "
                         "attention kernel does it, by one 16x16x32 MFMA per 4 products): the mix of head dim 64; the "
                         "FLOPs counted are those of the 32x32x16 products only",
                 "unit": "TFLOP/s",
                 "zero_operands": B.bsga_probe_mfma(0, 0),
                 "random_operands": B.bsga_probe_mfma(1, 0),
                 "random_operands_softmax_adds": B.bsga_probe_mfma(1, 1),
                 "zero_operands_softmax": B.bsga_probe_mfma(0, 2),
                 "random_operands_softmax": B.bsga_probe_mfma(1, 2)}
        print("[bench] mfma probe: " + json.dumps({k: v for k, v in probe.items() if k not in ("what", "unit")}),
              file=sys.stderr, flush=True)

    rows = []

    def add(wl, tau, rho, special=False):
        r, _ = wl.row(tau, rho, args.row_steps, 1, special=special, dense_steps=max(1, min(2, args.dense_steps)))
        rows.append(r)
        print("[row] " + json.dumps(r), file=sys.stderr, flush=True)

    if args.rows != "none":
        for tau in cfg.taus:
            if tau != args.tau and tau < 1.0:
                add(w, tau, 1.0)
        for rho in (0.5, 0.75, 0.9):  # top-k only: the regime the paper operates in (50-90 % sparsity)
            add(w, 0.0, rho)
        add(w, args.tau, args.rho, special=True)
        add(w, 0.0, 0.75, special=True)

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

    locality_rows = []
    if args.locality:
        import numpy as np
        nbk = cfg.n_blocks
        kc = max(1, nbk // 10)
        rng = np.random.default_rng(0)
        cnt_l = torch.full((H, nbk), kc, dtype=torch.int32, device="cuda")
        dense_ms = w.time_dense(2)
        for kind in ("random per row", "identical within a head", "band around the row"):
            a = np.zeros((H, nbk, nbk), np.int32)
            for h_ in range(H):
                if kind == "identical within a head":
                    a[h_, :, :kc] = np.sort(rng.choice(nbk - 1, kc, replace=False))
                else:
                    for I in range(nbk):
                        if kind == "random per row":
                            a[h_, I, :kc] = np.sort(rng.choice(nbk - 1, kc, replace=False))
                        else:
                            lo = min(max(I - kc // 2, 0), nbk - 1 - kc)
                            a[h_, I, :kc] = np.arange(lo, lo + kc)
            idx_l = torch.from_numpy(a).cuda()
            ts = []
            for _ in range(args.row_steps + 1):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                B.bsga_sparse_attn(w.q, w.k, w.v, b, idx_l, cnt_l, out=w.out, workspace=w.ws)
                e1.record()
                torch.cuda.synchronize()
                ts.append(e0.elapsed_time(e1))
            ms = statistics.median(ts[1:])
            fl = kept_flops(idx_l, cnt_l, N, b)
            row = {"lists": kind, "blocks_per_row": kc, "attention_ms": ms, "kept_tflops_attention": fl / (ms * 1e-3) / 1e12,
                   "dense_tflops": 4.0 * H * float(N) * float(N) * d / (dense_ms * 1e-3) / 1e12}
            locality_rows.append(row)
            print("[locality] " + json.dumps(row), file=sys.stderr, flush=True)
            del idx_l

    asym_rows = []
    if args.asym and b == 128:
        nbk64 = -(-N // 64)
        ws64 = torch.empty(B.bsga_select_workspace_bytes(H, cfg.n_blocks, nbk64), dtype=torch.uint8, device="cuda")
        dense_ms = w.time_dense(2)
        for tau, rho in [(args.tau, args.rho), (0.0, 0.5), (0.0, 0.75), (0.0, 0.9)]:
            def asym_layer(ev=None):
                if ev:
                    ev[0].record()
                qp, kp = B.bsga_pool(w.q, 128), B.bsga_pool(w.k, 64)
                _, idx, cnt = B.bsga_select_blocks(qp, kp, tau, rho, want_bits=False, workspace=ws64)
                if ev:
                    ev[1].record()
                B.bsga_sparse_attn(w.q, w.k, w.v, 128, idx, cnt, out=w.out, workspace=w.ws, block_k=64)
                if ev:
                    ev[2].record()
                return idx, cnt
            asym_layer()
            torch.cuda.synchronize()
            steps = max(2, args.row_steps)
            evs = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(steps)]
            for s_ in range(steps):
                idx, cnt = asym_layer(evs[s_])
            torch.cuda.synchronize()
            st = [statistics.median(e[i].elapsed_time(e[i + 1]) for e in evs) for i in range(2)]
            ms = statistics.median(e[0].elapsed_time(e[2]) for e in evs)
            fl = kept_flops(idx, cnt, N, 128, 64)
            kf = float(cnt.to(torch.float64).sum().item()) / (H * cfg.n_blocks * nbk64)
            row = {"tau": tau, "rho": rho, "block_q": 128, "block_k": 64, "kept_fraction": kf, "layer_ms": ms,
                   "pool_select_ms": st[0], "attention_ms": st[1], "kept_tflops_layer": fl / (ms * 1e-3) / 1e12,
                   "speedup_vs_dense": dense_ms / ms}
            asym_rows.append(row)
            print("[asym] " + json.dumps(row), file=sys.stderr, flush=True)
        del ws64

    # ---- the other frame counts / resolutions, tau = 0.9, each with its own dense time ------------------
    if args.rows == "all":
        del w
        torch.cuda.empty_cache()
        for other in (2, 3, 6, 5):
            if other == cfg.cfg_id:
                continue
            wl = Workload(B, torch, CONFIGS[other])
            add(wl, 0.9, 1.0)
            if other == 6:
                add(wl, 0.9, 1.0, special=True)
            del wl
            torch.cuda.empty_cache()

    achieved = flops / (attn_mean_ms * 1e-3) / 1e12
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
        "layer_ms": head["layer_ms"],
        "stage_ms": head["stage_ms"],
        "pool_gbs": head["pool_gbs"],
        "select_gbs": head["select_gbs"],
        "kept_fraction": head["kept_fraction"],
        "pct_of_bf16_peak": 100.0 * value / PEAK_BF16_TFLOPS,
        "dense_ms": head["dense_ms"],
        "dense_tflops": head["dense_tflops"],
        "speedup_vs_dense": (head["dense_ms"] / wall_ms) if head["dense_ms"] else None,
        "timing": "ms_per_step = wall clock over the timed steps / steps; layer_ms, stage_ms, dense_ms and every row are "
                  "medians of per-step HIP event times",
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_traffic(cfg.cfg_id),
                     "kernel": f"attn_bf16_kernel<{b}> (block-sparse attention, one launch per step)",
                     "flops_per_launch": flops, "launch_ms": attn_mean_ms,
                     "launch_ms_median": head["stage_ms"]["attention"]},
    }
    if probe:
        probe["attention_kernel_vs_random_operands_softmax"] = achieved / probe["random_operands_softmax"]
        rec["mfma_probe"] = probe
    if rows:
        rec["rows"] = rows
    if locality_rows:
        rec["short_row_locality"] = locality_rows
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
