"""Turns rocprofv3 output folders of `bench.py` runs into the short summaries kept under profiles/.

Usage (from the repository root, after the rocprofv3 runs listed in each summary's header):

    python -m paper_2509_07120_amd.profile_summary stats   <dir of --kernel-trace --stats run> <bench json of that run>
    python -m paper_2509_07120_amd.profile_summary traffic <dir FETCH_SIZE run> <dir WRITE_SIZE run> <dir TCC run>
    python -m paper_2509_07120_amd.profile_summary pipes   <dir of counter run A> <dir of counter run B> ...
    python -m paper_2509_07120_amd.profile_summary topk    <dir TCC run at rho 0.9> <dir pipe-counter run at rho 0.9>

Each sub-command reads the `*_kernel_stats.csv`, `*_kernel_trace.csv` or `*_counter_collection.csv`
files rocprofv3 wrote with `--output-format csv`, prints what it found, and rewrites the matching
file under profiles/.  The traffic summary also writes profiles/attention_hbm_traffic.txt, which
bench.py reads for `roofline.traffic`; that file names the hash of the attention kernel's source, so
a figure measured with another kernel is never reported.
"""
from __future__ import annotations

import collections
import csv
import glob
import hashlib
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PROFILES = os.path.join(ROOT, "profiles")
ATTN_SOURCE = os.path.join(ROOT, "paper_2509_07120_amd", "csrc", "attn_bf16.hip")
KERNELS = ("attn_bf16_kernel", "select_kernel", "logits_kernel", "pool_kernel", "order_hist", "order_merge", "order_scan",
           "order_place", "gather_kernel", "probe_kernel")


def short(name: str):
    for k in KERNELS:
        if k in name:
            return k
    return None


def one(folder: str, suffix: str) -> str:
    hits = sorted(glob.glob(os.path.join(folder, "**", f"*{suffix}"), recursive=True))
    if not hits:
        raise SystemExit(f"no *{suffix} under {folder}")
    return hits[-1]


def source_sha() -> str:
    with open(ATTN_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def dispatches(folder: str):
    """Per dispatch: kernel name, grid, duration in ms and every counter collected in that run."""
    out = collections.OrderedDict()
    for r in csv.DictReader(open(one(folder, "counter_collection.csv"))):
        d = out.setdefault(int(r["Dispatch_Id"]), {"name": r["Kernel_Name"], "grid": int(r["Grid_Size"])})
        d[r["Counter_Name"]] = d.get(r["Counter_Name"], 0.0) + float(r["Counter_Value"])
        d["ms"] = (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6
    return [out[k] for k in sorted(out)]


# --------------------------------------------------------------------------------------------- stats
def cmd_stats(folder: str, bench_json: str) -> None:
    bench = json.loads(open(bench_json).read().strip().splitlines()[-1])
    rows = []
    for r in csv.DictReader(open(one(folder, "kernel_stats.csv"))):
        n = short(r["Name"])
        if n:
            rows.append((n, int(r["Calls"]), float(r["AverageNs"]) / 1e6, float(r["MinNs"]) / 1e6, float(r["MaxNs"]) / 1e6,
                         float(r["Percentage"])))
    trace = [(r["Kernel_Name"], (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e6)
             for r in csv.DictReader(open(one(folder, "kernel_trace.csv")))]
    attn = [ms for n, ms in trace if "attn_bf16" in n]
    steps, warmup = bench["steps"], bench["warmup"]
    sparse_timed = attn[warmup:warmup + steps]
    rest = attn[warmup + steps:]
    mean = sum(sparse_timed) / len(sparse_timed)
    path = os.path.join(PROFILES, "layer_cfg4_tau0.9_kernel_stats.md")
    with open(path, "w") as f:
        f.write(f"""# Kernel time of the whole layer, 100-frame workload (cfg4), tau = 0.9

Command (from the repository root, on one MI355X; the summary below is written by
`python -m paper_2509_07120_amd.profile_summary stats <out>/prof_stats <out>/prof_stats_bench.json`):

    cd /tmp && export TMPDIR=/tmp && rocprofv3 --kernel-trace --stats -d <out>/prof_stats -o stats --output-format csv -- python3 <repo>/bench.py --no-cpu-baseline --no-probe --rows none --steps {steps} --warmup {warmup} > <out>/prof_stats_bench.json

Workload: 100 frames x 1374 tokens = 137,400 tokens, 16 heads, d = 64, bf16, block 128, tau = 0.9, rho = 1
(kept fraction {bench['kept_fraction']:.4f}).  Kernel source hash (attn_bf16.hip, sha256/16): {source_sha()}.
The run launches the sparse layer {warmup + steps} times ({warmup} warm-up + {steps} timed) and then the dense baseline
{len(rest)} times; both use the same attention kernel, so the `attn_bf16_kernel` row of `stats_kernel_stats.csv` mixes the
two.  The per-dispatch trace (`stats_kernel_trace.csv`) separates them.

## stats_kernel_stats.csv (library kernels only; the rest are torch helpers of bench.py, < 0.1 %)

| kernel | calls | avg ms | min ms | max ms | % of GPU time |
|---|---|---|---|---|---|
""")
        for n, c, a, mn, mx, p in rows:
            f.write(f"| {n} | {c} | {a:.4f} | {mn:.4f} | {mx:.4f} | {p:.3f} |\n")
        f.write(f"""
`pool_kernel` runs twice per step (Q and K); the four `order_*` kernels build the launch order of the sparse
attention kernel and run once per sparse launch.

## attn_bf16_kernel per dispatch (stats_kernel_trace.csv), ms

- sparse, the {steps} timed launches: {', '.join(f'{x:.3f}' for x in sparse_timed)}  -> mean {mean:.3f}
- dense launches after them: {', '.join(f'{x:.3f}' for x in rest)}

## bench.py line of the same run (timed with events inside bench.py)

- stage_ms (medians): pool {bench['stage_ms']['pool']:.4f}, select {bench['stage_ms']['select']:.4f}, attention {bench['stage_ms']['attention']:.3f}
- roofline.launch_ms (attention stage, mean of the {steps} timed sparse launches, order kernels included): {bench['roofline']['launch_ms']:.3f}
  (trace mean of the attention kernel alone: {mean:.3f}; ratio {bench['roofline']['launch_ms'] / mean:.4f})
- roofline.achieved {bench['roofline']['achieved']:.1f} TFLOP/s of 2500 (frac {bench['roofline']['frac']:.4f}); dense {bench['dense_ms']:.3f} ms = {bench['dense_tflops']:.1f} TFLOP/s
- layer {bench['layer_ms']:.3f} ms (median), {bench['ms_per_step']:.3f} ms per step by the wall clock; value {bench['value']:.1f} TFLOP/s; speed-up vs dense {bench['speedup_vs_dense']:.4f}
- selection stage: {bench['select_gbs']:.0f} GB/s on the bytes it reads and writes; pooling: {bench['pool_gbs']:.0f} GB/s

The event-timed stages include launch gaps between the small kernels.
""")
    print(open(path).read())


# ------------------------------------------------------------------------------------------- traffic
def cmd_traffic(d_fetch: str, d_write: str, d_tcc: str) -> None:
    F, W, T = dispatches(d_fetch), dispatches(d_write), dispatches(d_tcc)
    copy_f = [x["FETCH_SIZE"] for x in F if "copyBuffer" in x["name"] and x["grid"] == 131072][0]
    copy_w = [x["WRITE_SIZE"] for x in W if "copyBuffer" in x["name"] and x["grid"] == 131072][0]
    sf, sw = 1048576.0 / copy_f, 1048576.0 / copy_w
    aF = [x for x in F if "attn_bf16" in x["name"]]
    aW = [x for x in W if "attn_bf16" in x["name"]]
    n_sparse = 3  # bench.py --steps 2 --warmup 1: three sparse launches, then the dense ones
    sparse_f = sum(x["FETCH_SIZE"] for x in aF[1:n_sparse]) / (n_sparse - 1)
    sparse_w = sum(x["WRITE_SIZE"] for x in aW[1:n_sparse]) / (n_sparse - 1)
    dense_f = sum(x["FETCH_SIZE"] for x in aF[n_sparse:]) / max(1, len(aF[n_sparse:]))
    dense_w = sum(x["WRITE_SIZE"] for x in aW[n_sparse:]) / max(1, len(aW[n_sparse:]))
    hbm = (sparse_f * sf + sparse_w * sw) * 1024.0
    hbm_dense = (dense_f * sf + dense_w * sw) * 1024.0

    def mean_of(rows, key, counter):
        v = [x[counter] for x in rows if key in x["name"]]
        return sum(v) / len(v)

    cmd = ("cd /tmp && export TMPDIR=/tmp && rocprofv3 --pmc {c} -d <out>/{d} -o {o} --output-format csv -- python3 "
           "<repo>/bench.py --no-cpu-baseline --no-probe --rows none --copy-calibration --steps 2 --warmup 1 --dense-steps 1")
    path = os.path.join(PROFILES, "attention_cfg4_hbm_traffic.md")
    with open(path, "w") as f:
        f.write(f"""# Memory traffic per launch (FETCH_SIZE / WRITE_SIZE, L2 hit rate), 100-frame workload (cfg4), tau = 0.9

Commands (one run per counter set; the summary is written by
`python -m paper_2509_07120_amd.profile_summary traffic <out>/prof_fetch <out>/prof_write <out>/prof_tcc`):

    {cmd.format(c='FETCH_SIZE', d='prof_fetch', o='fetch')}
    {cmd.format(c='WRITE_SIZE', d='prof_write', o='write')}
    {cmd.format(c='TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum', d='prof_tcc', o='tcc')}

Kernel source hash (attn_bf16.hip, sha256/16): {source_sha()}.
`--copy-calibration` issues one 1 GiB device-to-device copy (`__amd_rocclr_copyBuffer`, grid 131072) before the
layer.  It reads and writes 1,048,576 KiB; the counters report

| counter | copy kernel reads (KiB) | scale = 1,048,576 / reading |
|---|---|---|
| FETCH_SIZE | {copy_f:.1f} | {sf:.4f} |
| WRITE_SIZE | {copy_w:.1f} | {sw:.4f} |

Counter values per dispatch (KiB, unscaled):

| kernel | FETCH_SIZE | WRITE_SIZE |
|---|---|---|
| pool_kernel (one tensor) | {mean_of(F, 'pool_kernel', 'FETCH_SIZE'):.1f} | {mean_of(W, 'pool_kernel', 'WRITE_SIZE'):.1f} |
| logits_kernel | {mean_of(F, 'logits_kernel', 'FETCH_SIZE'):.1f} | {mean_of(W, 'logits_kernel', 'WRITE_SIZE'):.1f} |
| select_kernel | {mean_of(F, 'select_kernel', 'FETCH_SIZE'):.1f} | {mean_of(W, 'select_kernel', 'WRITE_SIZE'):.1f} |
| attn_bf16_kernel, sparse launches (1 warm-up + 2 timed) | {', '.join(f"{x['FETCH_SIZE']:.0f}" for x in aF[:n_sparse])} | {', '.join(f"{x['WRITE_SIZE']:.0f}" for x in aW[:n_sparse])} |
| attn_bf16_kernel, dense launches | {', '.join(f"{x['FETCH_SIZE']:.0f}" for x in aF[n_sparse:])} | {', '.join(f"{x['WRITE_SIZE']:.0f}" for x in aW[n_sparse:])} |

Scaled, per launch of the sparse attention kernel (mean of the two timed launches):
fetch {sparse_f * sf * 1024 / 1e9:.2f} GB + write {sparse_w * sw * 1024 / 1e9:.3f} GB = **{hbm / 1e9:.2f} GB**
(dense launch: {hbm_dense / 1e9:.2f} GB).  Algorithmic bytes (Q, K, V, O once): 1.13 GB.

Selection stage (logits_kernel + select_kernel), scaled: reads {(mean_of(F, 'logits_kernel', 'FETCH_SIZE') + mean_of(F, 'select_kernel', 'FETCH_SIZE')) * sf * 1024 / 1e6:.0f} MB,
writes {(mean_of(W, 'logits_kernel', 'WRITE_SIZE') + mean_of(W, 'select_kernel', 'WRITE_SIZE')) * sw * 1024 / 1e6:.0f} MB per call (the fp64 block logits are 148 MB each way, the outputs 69 MB).

L2 (TCC) requests of the attention kernel per launch:

| launch | TCC_REQ | TCC_HIT | TCC_MISS | hit rate | ms |
|---|---|---|---|---|---|
""")
        for i, x in enumerate(y for y in T if "attn_bf16" in y["name"]):
            kind = "sparse" if i < n_sparse else "dense"
            f.write(f"| {kind} {i} | {x['TCC_REQ_sum']:.4g} | {x['TCC_HIT_sum']:.4g} | {x['TCC_MISS_sum']:.4g} | "
                    f"{x['TCC_HIT_sum'] / x['TCC_REQ_sum']:.3f} | {x['ms']:.2f} |\n")
        f.write("""
Reading.  The write side equals the output tensor (137,400 x 16 x 64 x 2 B = 274,805 KiB).  The fetch side is what the
eight L2 caches request from the fabric (Infinity Cache hits included; the counter sits at the L2 boundary): Q, K, V
are 0.84 GB, and every workgroup streams its ~966 kept K and V tiles (31 MB) through LDS: L2 requests of 128 B, none of
them absorbed by the CUs' own caches.  The 64 workgroups resident on one XCD walk the same head's keys; they start
together and have rows of nearly equal length, so they stay roughly in step and most requests hit in L2.  If they were
exactly in step each tile would be fetched once per XCD per round (about 9.4 GB per launch).  The 4 MB L2 cannot hold
the 35 MB of one head's K and V, so workgroups that fall more than about 64 tiles behind miss; the misses are served by
the Infinity Cache (one head fits it), not by HBM.
""")
    with open(os.path.join(PROFILES, "attention_hbm_traffic.txt"), "w") as f:
        f.write("# HBM-side bytes per launch of the attention kernel, read by bench.py for roofline.traffic.\n"
                "# Written by `python -m paper_2509_07120_amd.profile_summary traffic ...` (see attention_cfg4_hbm_traffic.md);\n"
                "# valid only for the kernel source whose hash is given here.\n"
                f"kernel_source_sha256_16 = {source_sha()}\n"
                f"cfg4.hbm_bytes_per_launch = {hbm:.0f}\n"
                f"cfg4.fetch_kib_unscaled = {sparse_f:.1f}\n"
                f"cfg4.write_kib_unscaled = {sparse_w:.1f}\n"
                f"cfg4.fetch_scale = {sf:.4f}\n"
                f"cfg4.write_scale = {sw:.4f}\n")
    print(open(path).read())


# --------------------------------------------------------------------------------------------- pipes
def cmd_pipes(*folders: str) -> None:
    """Pipe utilisation, clock and where the waves' time goes, from several --pmc runs of the same
    bench command.  Counters of different runs are merged per dispatch position of the attention kernel."""
    merged = None
    for d in folders:
        attn = [x for x in dispatches(d) if "attn_bf16" in x["name"]]
        if merged is None:
            merged = [dict(x) for x in attn]
        else:
            for m, x in zip(merged, attn):
                for k, v in x.items():
                    if k not in ("name", "grid"):
                        m[k if k != "ms" else f"ms_{os.path.basename(d.rstrip('/'))}"] = v
    n_sparse = 3
    cols = [k for k in merged[0] if k not in ("name", "grid") and not k.startswith("ms")]
    path = os.path.join(PROFILES, "attention_cfg4_mfma_utilisation.md")
    cmd = ("cd /tmp && export TMPDIR=/tmp && rocprofv3 --pmc {c} -d <out>/{d} -o pmc --output-format csv -- python3 "
           "<repo>/bench.py --no-cpu-baseline --no-probe --rows none --copy-calibration --steps 2 --warmup 1 --dense-steps 1")
    sets = {
        "pipes_a": "SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_VALU_MFMA_COEXEC_CYCLES SQ_INSTS_VALU SQ_INSTS_SALU SQ_INSTS_LDS SQ_INSTS_MFMA GRBM_GUI_ACTIVE",
        "pipes_b": "SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY SQ_WAIT_INST_LDS SQ_ACTIVE_INST_ANY SQ_ACTIVE_INST_VALU SQ_ACTIVE_INST_LDS",
        "pipes_c": "SQ_ACTIVE_INST_SCA SQ_ACTIVE_INST_VMEM SQ_ACTIVE_INST_MISC SQ_INST_CYCLES_SALU SQ_LDS_IDX_ACTIVE SQ_LDS_BANK_CONFLICT SQ_THREAD_CYCLES_VALU SQ_INSTS_VALU_TRANS_F32",
    }
    with open(path, "w") as f:
        f.write("# Pipe utilisation, clock and wave time of the attention kernel, 100-frame workload (cfg4), tau = 0.9\n\n"
                "Commands (one run per counter set; the summary is written by\n"
                "`python -m paper_2509_07120_amd.profile_summary pipes <out>/pipes_a <out>/pipes_b <out>/pipes_c`):\n\n")
        for d, c in sets.items():
            f.write("    " + cmd.format(c=c, d=d) + "\n")
        f.write(f"\nKernel source hash (attn_bf16.hip, sha256/16): {source_sha()}.  Per dispatch of `attn_bf16_kernel` "
                f"({n_sparse} sparse launches, then the dense ones):\n\n")
        f.write("| launch | ms | " + " | ".join(cols) + " |\n|---|---|" + "---|" * len(cols) + "\n")
        for i, m in enumerate(merged):
            kind = "sparse" if i < n_sparse else "dense"
            f.write(f"| {kind} {i} | {m['ms']:.2f} | " + " | ".join(f"{m.get(c, float('nan')):.4g}" for c in cols) + " |\n")
        f.write("\n## Derived (per launch)\n\n| launch | clock GHz | MFMA pipe busy | co-execution | VALU instr per MFMA | SALU instr per MFMA | LDS instr per MFMA |"
                " wave time waiting | waiting for issue | of which LDS | wave time issuing VALU | issuing LDS | issuing scalar |\n"
                "|---|---|---|---|---|---|---|---|---|---|---|---|---|\n")

        def g(m, k):
            return m.get(k, float("nan"))

        for i, m in enumerate(merged):
            kind = "sparse" if i < n_sparse else "dense"
            clock = g(m, "GRBM_GUI_ACTIVE") / 8.0 / (m["ms"] * 1e-3) / 1e9
            util = g(m, "SQ_VALU_MFMA_BUSY_CYCLES") / (4.0 * g(m, "SQ_BUSY_CU_CYCLES"))
            coex = g(m, "SQ_VALU_MFMA_COEXEC_CYCLES") / g(m, "SQ_VALU_MFMA_BUSY_CYCLES")
            nm = g(m, "SQ_INSTS_MFMA")
            wc = g(m, "SQ_WAVE_CYCLES")
            f.write(f"| {kind} {i} | {clock:.3f} | {util:.3f} | {coex:.3f} | {(g(m, 'SQ_INSTS_VALU') - nm) / nm:.2f} | "
                    f"{g(m, 'SQ_INSTS_SALU') / nm:.2f} | {g(m, 'SQ_INSTS_LDS') / nm:.2f} | {g(m, 'SQ_WAIT_ANY') / wc:.3f} | "
                    f"{g(m, 'SQ_WAIT_INST_ANY') / wc:.3f} | {g(m, 'SQ_WAIT_INST_LDS') / wc:.3f} | "
                    f"{g(m, 'SQ_ACTIVE_INST_VALU') / wc:.3f} | {g(m, 'SQ_ACTIVE_INST_LDS') / wc:.3f} | "
                    f"{g(m, 'SQ_ACTIVE_INST_SCA') / wc:.3f} |\n")
        f.write("""
How to read it.  GRBM_GUI_ACTIVE counts busy cycles summed over the 8 XCDs, so divided by 8 and by the kernel's
duration it gives the clock the kernel ran at.  SQ_VALU_MFMA_BUSY_CYCLES is summed over the four SIMDs of a CU and
SQ_BUSY_CU_CYCLES is per CU, hence the factor 4.  Fraction of the 2.5 PFLOP/s peak = (clock / 2.4) x MFMA pipe busy.
SQ_WAVE_CYCLES counts, in units of 4 cycles, the time waves are resident; the "wave time" columns are shares of it
(a wave can be waiting for one thing while another of its instructions executes, so they need not add up to 1).
""")
    print(open(path).read())


# ---------------------------------------------------------------------------------------------- topk
def cmd_topk(d_tcc: str, d_pipes: str) -> None:
    """Counters of the short-row regime (top-k only, rho = 0.9) next to the dense launch of the same run."""
    T = [x for x in dispatches(d_tcc) if "attn_bf16" in x["name"]]
    P = [x for x in dispatches(d_pipes) if "attn_bf16" in x["name"]]
    n_sparse = 3
    cmd = ("cd /tmp && export TMPDIR=/tmp && rocprofv3 --pmc {c} -d <out>/{d} -o pmc --output-format csv -- python3 "
           "<repo>/bench.py --no-cpu-baseline --no-probe --rows none --tau 0 --rho 0.9 --copy-calibration --steps 2 "
           "--warmup 1 --dense-steps 1")
    path = os.path.join(PROFILES, "attention_cfg4_topk0.9_counters.md")
    with open(path, "w") as f:
        f.write("# Short rows: top-k only, rho = 0.9 (107 of 1074 key blocks per row), 100-frame workload (cfg4)\n\n"
                "Commands (the summary is written by `python -m paper_2509_07120_amd.profile_summary topk <out>/tcc <out>/pipes`):\n\n"
                "    " + cmd.format(c="TCC_HIT_sum TCC_MISS_sum TCC_REQ_sum", d="tcc") + "\n"
                "    " + cmd.format(c="SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_WAVE_CYCLES SQ_WAIT_ANY SQ_WAIT_INST_ANY "
                                      "SQ_INSTS_MFMA SQ_ACTIVE_INST_VALU SQ_BUSY_CYCLES GRBM_GUI_ACTIVE", d="pipes") + "\n\n"
                f"Kernel source hash (attn_bf16.hip, sha256/16): {source_sha()}.  Per dispatch of `attn_bf16_kernel` "
                f"({n_sparse} sparse launches at rho = 0.9, then the dense launches of the same inputs):\n\n"
                "| launch | ms | L2 requests | L2 hit rate | L2 misses x 128 B | clock GHz | MFMA pipe busy (of CU-busy time) | CUs busy (of the launch) | waves ready but not issued |\n"
                "|---|---|---|---|---|---|---|---|---|\n")
        for i, (t, m) in enumerate(zip(T, P)):
            kind = "rho 0.9" if i < n_sparse else "dense"
            clock = m["GRBM_GUI_ACTIVE"] / 8.0 / (m["ms"] * 1e-3) / 1e9
            cu_busy = m["SQ_BUSY_CU_CYCLES"] / 256.0 / (m["ms"] * 1e-3 * clock * 1e9)
            f.write(f"| {kind} {i} | {t['ms']:.2f} | {t['TCC_REQ_sum']:.4g} | {t['TCC_HIT_sum'] / t['TCC_REQ_sum']:.3f} | "
                    f"{t['TCC_MISS_sum'] * 128 / 1e9:.1f} GB | {clock:.3f} | "
                    f"{m['SQ_VALU_MFMA_BUSY_CYCLES'] / (4.0 * m['SQ_BUSY_CU_CYCLES']):.3f} | {cu_busy:.3f} | "
                    f"{m['SQ_WAIT_INST_ANY'] / m['SQ_WAVE_CYCLES']:.3f} |\n")
        f.write("""
Reading.  With rows of 107 tiles the matrix pipes are as busy, while a CU is busy, as with rows of 966 tiles; what
is lost is clock (the L2 misses are served by the Infinity Cache at several TB/s, and that traffic takes power from
the core clock) and CU time (every row pays its start-up and end merge, and the launch ends with a partly filled
round of workgroups).  The L2 hit rate is low because the generator's kept sets are nearly random subsets of the
key blocks: the 64 workgroups of an XCD walk their lists in ascending order, but a block that six of them need is
needed over a window of about +-50 tiles, many times what 4 MB of L2 hold.
""")
    print(open(path).read())


def main(argv) -> int:
    if len(argv) >= 4 and argv[1] == "stats":
        cmd_stats(argv[2], argv[3])
    elif len(argv) >= 5 and argv[1] == "traffic":
        cmd_traffic(argv[2], argv[3], argv[4])
    elif len(argv) >= 3 and argv[1] == "pipes":
        cmd_pipes(*argv[2:])
    elif len(argv) >= 4 and argv[1] == "topk":
        cmd_topk(argv[2], argv[3])
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
