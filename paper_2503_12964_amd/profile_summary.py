"""Turns the rocprofv3 output of the profiling runs of bench.py into the short text summaries
under profiles/ (host only; reads CSV and log files, touches no GPU).

    python -m paper_2503_12964_amd.profile_summary RUN_DIR [--workload C4] [--out profiles/NAME.txt]

RUN_DIR holds what these commands wrote (run from the repository root, after
`cd /tmp && export TMPDIR=/tmp && cd <repo>`; P = rocprofv3, B = python3 bench.py --workload W):

    B                                                               > RUN_DIR/bench_default.log
    P --kernel-trace --stats -d RUN_DIR -o stats --output-format csv -- B --steps 5 --warmup 2 \
        --no-cpu-baseline --no-mfma-ceiling                         > RUN_DIR/stats.log
    P --pmc FETCH_SIZE  -d RUN_DIR -o fetch  --output-format csv -- B --steps 2 --warmup 1 ...
    P --pmc WRITE_SIZE  -d RUN_DIR -o write  --output-format csv -- B --steps 2 --warmup 1 ...
    P --pmc FETCH_SIZE  -d RUN_DIR -o cal_fetch --output-format csv -- python3 bench.py --calibrate-copy
    P --pmc WRITE_SIZE  -d RUN_DIR -o cal_write --output-format csv -- python3 bench.py --calibrate-copy
    P --pmc <MFMA_COUNTERS> -d RUN_DIR -o sq  --output-format csv -- B --steps 2 --warmup 1 ...
    P --pmc <LDS_COUNTERS>  -d RUN_DIR -o lds --output-format csv -- B --steps 2 --warmup 1 ...

("..." = --no-cpu-baseline --no-mfma-ceiling; each counter set is a run of its own.)  Missing
files leave their section out.  Besides the summary the module rewrites the workload's lines of
profiles/attention_hbm_traffic.txt, which bench.py reads for `roofline.traffic`.
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "attention_hbm_traffic.txt")

MFMA_COUNTERS = ("SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CU_CYCLES SQ_INSTS_VALU_MFMA_MOPS_BF16 SQ_INSTS_MFMA "
                 "SQ_WAVE_CYCLES SQ_INSTS_VALU SQ_LDS_BANK_CONFLICT SQ_BUSY_CYCLES")
LDS_COUNTERS = ("SQ_LDS_IDX_ACTIVE SQ_ACTIVE_INST_LDS SQ_WAIT_INST_LDS SQ_INSTS_LDS SQ_INSTS_VALU_TRANS_F32 "
                "SQ_ACTIVE_INST_VALU SQ_WAVE_CYCLES SQ_BUSY_CYCLES")

# kernel-name fragment -> short label, most specific first
KERNELS = (("tattn_fwd", "tattn_fwd_kernel"), ("tattn_bwd", "tattn_bwd_kernel"),
           ("attn_bwd_both", "attn_bwd_both_kernel"), ("attn_bwd_dkdv", "attn_bwd_dkdv_kernel"), ("attn_bwd_dq2", "attn_bwd_dq2_kernel"),
           ("attn_bwd_dq", "attn_bwd_dq_kernel"), ("attn_fwd_fp8", "attn_fwd_fp8_kernel"),
           ("attn_fwd", "attn_fwd_kernel"), ("qknorm_rope3d_bwd", "qknorm_rope3d_bwd_kernel (outside the step)"),
           ("qknorm_rope3d", "qknorm_rope3d_kernel (outside the step)"), ("rope3d", "rope3d_kernel"),
           ("bwd_prepare", "bwd_prepare_kernel"), ("bwd_short_delta", "bwd_short_delta_kernel"),
           ("copyBuffer", "copy kernel (1 GiB)"))
ATTENTION = ("attn_bwd_dkdv_kernel", "attn_bwd_dq2_kernel", "attn_bwd_both_kernel", "attn_fwd_kernel")
N_SIMD, N_CU, N_SE = 1024, 256, 32      # MI355X: 256 CUs x 4 SIMDs, 8 XCDs x 4 shader engines


def _label(name: str):
    return next((lab for frag, lab in KERNELS if frag in name), None)


def _bench_line(path: str):
    if not os.path.exists(path):
        return None
    lines = [l for l in open(path) if l.startswith("{")]
    return json.loads(lines[-1]) if lines else None


def _pmc(run_dir: str, name: str):
    """Mean counter value per dispatch, keyed (kernel label, counter)."""
    path = os.path.join(run_dir, f"{name}_counter_collection.csv")
    if not os.path.exists(path):
        return None
    acc = collections.defaultdict(lambda: [0, 0.0])
    for r in csv.DictReader(open(path)):
        lab = _label(r["Kernel_Name"])
        if lab:
            a = acc[(lab, r["Counter_Name"])]
            a[0] += 1
            a[1] += float(r["Counter_Value"])
    return {k: v[1] / v[0] for k, v in acc.items()}


def _write_traffic(workload: str, entries: dict) -> None:
    keep = []
    if os.path.exists(TRAFFIC_FILE):
        keep = [l for l in open(TRAFFIC_FILE) if l.startswith("#") or (l.split() and l.split()[0] != workload)]
    if not any(l.startswith("#") for l in keep):
        keep.insert(0, "# workload  what  HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy of known size)\n"
                       "# written by python -m paper_2503_12964_amd.profile_summary; read by bench.py (roofline.traffic)\n")
    keep += [f"{workload} {key} {val:.6e}\n" for key, val in entries.items()]
    os.makedirs(os.path.dirname(TRAFFIC_FILE), exist_ok=True)
    open(TRAFFIC_FILE, "w").writelines(keep)


def summarise(run_dir: str, workload: str, out_path: str) -> str:
    L = []
    P = L.append
    rel = os.path.relpath(run_dir, ROOT)
    bench = f"python3 bench.py --workload {workload}"
    quiet = "--no-cpu-baseline --no-mfma-ceiling"
    d = _bench_line(os.path.join(run_dir, "bench_default.log"))
    b = _bench_line(os.path.join(run_dir, "stats.log"))
    cfg = (d or b or {}).get("config", {}).get("workload", workload)
    if len(cfg) > 240:                      # packs of hundreds of clips: the list of grids is cut
        cfg = cfg[:cfg.index("(") + 48] + " ... " + cfg[cfg.index("] ->"):]
    P(f"rocprofv3 summary: packed 3D-RoPE attention, workload {cfg}")
    P("device: AMD Instinct MI355X (gfx950), 256 CUs, 2.4 GHz; all commands run from the repository root after")
    P("  cd /tmp && export TMPDIR=/tmp && cd <repo>;   summarised by: python -m paper_2503_12964_amd.profile_summary " + rel)
    P("")
    if d:
        bd, rf = d["breakdown"], d["roofline"]
        P(f"[0] {bench}        (default run: {d['steps']} timed steps after {d['warmup']} warm-ups, HIP events, no profiler)")
        P(f"    value={d['value']:.1f} TFLOP/s ({d['config']['pct_of_bf16_mfma_peak']:.1f}% of the 2500 TFLOP/s bf16 peak) "
          f"ms_per_step={d['ms_per_step']:.2f} (median; min {bd['step_ms_min']:.2f})")
        line = f"    rope_ms={bd['rope_ms']:.3f} ({bd['rope_gbs']:.0f} GB/s) fwd_ms={bd['fwd_ms']:.2f} ({bd['fwd_tflops']:.0f} TFLOP/s)"
        if bd.get("bwd_tflops"):
            line += f" bwd_ms={bd['bwd_ms']:.2f} ({bd['bwd_tflops']:.0f} TFLOP/s)"
        P(line)
        mc = rf.get("mfma_only_measured")
        if mc:
            P(f"    MFMA-only loop (paper_2503_12964_amd/mfma_ceiling, {mc['seconds_each']} s each): constant operands "
              f"{mc['constant_operands_tflops']:.0f} TFLOP/s, random operands {mc['random_operands_tflops']:.0f} TFLOP/s")
            P(f"    dominant call = {rf['achieved']:.0f} TFLOP/s = {rf['frac']:.3f} of the published peak, "
              f"{mc['frac_of_random_operand_ceiling']:.3f} of the random-operand MFMA-only ceiling")
        cs = rf.get("clock_power_sample")
        if cs:
            pw = f", power median {cs['power_w_median']:.0f} W" if cs.get("power_w_median") else ""
            P(f"    shader clock while the timed steps ran (rocm-smi, {cs['samples']} samples): median {cs['sclk_mhz_median']:.0f} MHz, "
              f"min {cs['sclk_mhz_min']:.0f}, max {cs['sclk_mhz_max']:.0f}{pw}")
        cb = d.get("cpu_baseline")
        if cb:
            P(f"    cpu_baseline: {cb['value'] * 1e3:.2f} GFLOP/s on {cb['cores']} threads ({cb['sample']})")
        P("")
    avg = {}
    stats_csv = os.path.join(run_dir, "stats_kernel_stats.csv")
    if os.path.exists(stats_csv):
        P(f"[1] rocprofv3 --kernel-trace --stats -d {rel} -o stats --output-format csv -- {bench} --steps 5 --warmup 2 {quiet}")
        if b:
            P(f"    bench line: value={b['value']:.1f} TFLOP/s ms_per_step={b['ms_per_step']:.2f} fwd_ms={b['breakdown']['fwd_ms']:.2f} "
              f"bwd_ms={b['breakdown']['bwd_ms']:.2f} rope_ms={b['breakdown']['rope_ms']:.3f}")
            P(f"    roofline: achieved={b['roofline']['achieved']:.1f} TFLOP/s frac={b['roofline']['frac']:.4f} "
              f"({b['roofline']['kernel']}, HIP events)")
        P(f"    {'kernel':46s} {'calls':>5s} {'avg_ms':>10s} {'min_ms':>10s} {'max_ms':>10s} {'pct':>7s}")
        for r in csv.DictReader(open(stats_csv)):
            lab = _label(r["Name"])
            if lab and "copy" not in lab:
                avg[lab] = float(r["AverageNs"]) / 1e6
                P(f"    {lab:46s} {r['Calls']:>5s} {float(r['AverageNs']) / 1e6:10.3f} {float(r['MinNs']) / 1e6:10.3f} "
                  f"{float(r['MaxNs']) / 1e6:10.3f} {float(r['Percentage']):7.3f}")
        bwd_sum = sum(avg.get(x, 0.0) for x in ("attn_bwd_dkdv_kernel", "attn_bwd_dq2_kernel", "attn_bwd_both_kernel",
                                                "bwd_prepare_kernel"))
        if b and bwd_sum:
            P(f"    backward kernels summed: {bwd_sum:.3f} ms (bench.py's HIP-event time for the vfm_attn_bwd call: "
              f"{b['breakdown']['bwd_ms']:.3f} ms)")
        P("")
    f, w, cf, cw = (_pmc(run_dir, n) for n in ("fetch", "write", "cal_fetch", "cal_write"))
    if f and w and cf and cw:
        P("[2] HBM traffic, one counter per run (KiB per dispatch, mean over dispatches):")
        P(f"    rocprofv3 --pmc FETCH_SIZE -d {rel} -o fetch --output-format csv -- {bench} --steps 2 --warmup 1 {quiet}")
        P(f"    rocprofv3 --pmc WRITE_SIZE -d {rel} -o write --output-format csv -- {bench} --steps 2 --warmup 1 {quiet}")
        P(f"    rocprofv3 --pmc FETCH_SIZE|WRITE_SIZE -d {rel} -o cal_fetch|cal_write --output-format csv -- python3 bench.py --calibrate-copy")
        cfv, cwv = cf[("copy kernel (1 GiB)", "FETCH_SIZE")], cw[("copy kernel (1 GiB)", "WRITE_SIZE")]
        kf, kw = 1048576.0 / cfv, 1048576.0 / cwv
        P(f"    copy kernel: FETCH_SIZE reads {cfv:.0f} KiB for 1,048,576 KiB read  -> scale {kf:.4f}")
        P(f"                 WRITE_SIZE reads {cwv:.0f} KiB for 1,048,576 KiB written -> scale {kw:.4f}")
        P(f"    {'kernel':46s} {'FETCH_SIZE':>12s} {'WRITE_SIZE':>12s} {'scaled read GB':>15s} {'scaled write GB':>16s}")
        bwd_total, fwd_total = 0.0, 0.0
        for lab in ("attn_bwd_dkdv_kernel", "attn_bwd_dq2_kernel", "attn_bwd_both_kernel", "attn_bwd_dq_kernel",
                    "attn_fwd_kernel", "rope3d_kernel",
                    "bwd_prepare_kernel", "bwd_short_delta_kernel"):
            fv, wv = f.get((lab, "FETCH_SIZE")), w.get((lab, "WRITE_SIZE"))
            if fv is None and wv is None:
                continue
            fv, wv = fv or 0.0, wv or 0.0
            rg, wg = fv * kf * 1024 / 1e9, wv * kw * 1024 / 1e9
            if "bwd" in lab:
                bwd_total += (rg + wg) * 1e9
            if lab == "attn_fwd_kernel":
                fwd_total = (rg + wg) * 1e9
            P(f"    {lab:46s} {fv:12.0f} {wv:12.0f} {rg:15.3f} {wg:16.3f}")
        P(f"    backward call (all its kernels) scaled traffic: {bwd_total / 1e9:.2f} GB per launch; forward call "
          f"{fwd_total / 1e9:.2f} GB   <- bench.py roofline.traffic (profiles/attention_hbm_traffic.txt)")
        _write_traffic(workload, {"backward_call": bwd_total, "forward_call": fwd_total})
        P("")
    sq = _pmc(run_dir, "sq")
    if sq and avg:
        P(f"[3] rocprofv3 --pmc {MFMA_COUNTERS}")
        P(f"        -d {rel} -o sq --output-format csv -- {bench} --steps 2 --warmup 1 {quiet}")
        P(f"    {'kernel':30s} {'MFMA insts':>11s} {'MFMA busy cyc':>14s} {'clock GHz':>10s} {'busy @2.4GHz':>13s} {'busy @clock':>12s} "
          f"{'VALU insts':>11s} {'LDS bank confl':>15s}")
        for lab in ATTENTION:
            if (lab, "SQ_VALU_MFMA_BUSY_CYCLES") not in sq or lab not in avg:
                continue
            busy = sq[(lab, "SQ_VALU_MFMA_BUSY_CYCLES")]
            cyc = sq.get((lab, "SQ_BUSY_CYCLES"), 0.0) / N_SE               # cycles the kernel was resident, per shader engine
            clock = cyc / (avg[lab] * 1e-3) / 1e9 if cyc else float("nan")
            P(f"    {lab:30s} {sq.get((lab, 'SQ_INSTS_MFMA'), 0):11.4g} {busy:14.4g} {clock:10.2f} "
              f"{busy / (avg[lab] * 1e-3 * 2.4e9 * N_SIMD):13.3f} {busy / (cyc * N_SIMD) if cyc else float('nan'):12.3f} "
              f"{sq.get((lab, 'SQ_INSTS_VALU'), 0):11.4g} {sq.get((lab, 'SQ_LDS_BANK_CONFLICT'), 0):15.0f}")
        P("    MFMA busy = SQ_VALU_MFMA_BUSY_CYCLES / (cycles x 1024 SIMDs); each v_mfma_f32_32x32x16_bf16 is 32 busy cycles.")
        P("    clock = SQ_BUSY_CYCLES / 32 shader engines / kernel time of [1]: the cycles the chip really clocked while the kernel ran.")
        P("    'busy @2.4GHz' prices the kernel time at the nominal clock, 'busy @clock' at the measured one.")
        P("")
    lds = _pmc(run_dir, "lds")
    if lds:
        P(f"[4] rocprofv3 --pmc {LDS_COUNTERS}")
        P(f"        -d {rel} -o lds --output-format csv -- {bench} --steps 2 --warmup 1 {quiet}")
        P(f"    {'kernel':30s} {'LDS insts':>11s} {'LDS idx active':>15s} {'LDS pipe busy':>14s} {'wait LDS':>10s} {'exp insts':>11s} "
          f"{'VALU active':>12s} {'wave cycles':>12s}")
        for lab in ATTENTION:
            if (lab, "SQ_LDS_IDX_ACTIVE") not in lds:
                continue
            cyc = lds.get((lab, "SQ_BUSY_CYCLES"), 0.0) / N_SE
            act = lds[(lab, "SQ_LDS_IDX_ACTIVE")]
            wave = lds.get((lab, "SQ_WAVE_CYCLES"), 0.0)
            P(f"    {lab:30s} {lds.get((lab, 'SQ_INSTS_LDS'), 0):11.4g} {act:15.4g} {act / (cyc * N_CU) if cyc else float('nan'):14.3f} "
              f"{lds.get((lab, 'SQ_WAIT_INST_LDS'), 0) / wave if wave else float('nan'):10.3f} "
              f"{lds.get((lab, 'SQ_INSTS_VALU_TRANS_F32'), 0):11.4g} "
              f"{lds.get((lab, 'SQ_ACTIVE_INST_VALU'), 0) / wave if wave else float('nan'):12.3f} {wave:12.4g}")
        P("    LDS pipe busy = SQ_LDS_IDX_ACTIVE / (cycles x 256 CUs): share of the clocked cycles a CU's LDS pipe was working.")
        P("    wait LDS, VALU active = SQ_WAIT_INST_LDS, SQ_ACTIVE_INST_VALU as a share of SQ_WAVE_CYCLES (all three in units of 4 cycles).")
        P("")
    text = "\n".join(L) + "\n"
    os.makedirs(os.path.dirname(os.path.abspath(out_path)), exist_ok=True)
    open(out_path, "w").write(text)
    return text


WIDENED = (("C2", "2 x 4,096 tokens, 16 heads (classifier-free-guidance batch), rope+fwd+bwd"),
           ("C3", "8 mixed clips packed, 28,704 tokens, 24 heads, rope+fwd+bwd"),
           ("C5", "130,560 tokens, 40 heads, rope+fwd (inference step)"),
           ("C4-spatial", "spatial view of the headline latent: 16 sequences of 3,520 tokens, rope+fwd+bwd"),
           ("P288", "288 images of 256 tokens packed (73,728 tokens), 32 heads, rope+fwd+bwd"),
           ("C4-cross", "cross-attention: 56,320 queries x 512 text keys/values, fwd+bwd"),
           ("C4-temporal", "temporal attention: 3,520 pixels x 16 frames, 32 heads, fwd+bwd"),
           ("L64-temporal", "temporal attention: 3,520 pixels x 64 frames, 8 heads, fwd+bwd (block-walking kernels)"),
           ("C4-fp8", "FP8 (E4M3, per-tile scales) forward at the headline shape: pack + attention"),
           ("C5-fp8", "FP8 forward at the 130,560-token inference shape: pack + attention"))


def _short_kernel(name: str):
    import re
    m = re.match(r"(?:void )?(?:vfm::)?(\w+)<", name) or re.match(r"_ZN3vfm\d+(\w+?_kernel)I", name)
    if not m:
        return None
    k = m.group(1)
    if k == "tattnL_fwd_kernel":        # two instances: the forward pass, and the backward's statistics pass
        k += " (bwd stats)" if ("Lb1E" in name or ", true>" in name) else " (forward)"
    return k


def summarise_widened(run_dir: str, out_path: str) -> str:
    """Per-kernel times of the workloads beyond the headline: RUN_DIR/<W>.log and <W>_kernel_stats.csv from
    rocprofv3 --kernel-trace --stats -d RUN_DIR -o <W> --output-format csv -- python3 bench.py --workload <W> ..."""
    rel = os.path.relpath(run_dir, ROOT)
    L = ["rocprofv3 summary: the workloads beyond the headline run (bf16 unless noted), one MI355X (gfx950)",
         "commands run from the repository root after  cd /tmp && export TMPDIR=/tmp && cd <repo>;  summarised by:",
         f"  python -m paper_2503_12964_amd.profile_summary {rel} --widened",
         "kernel names are shortened (template arguments dropped); a call with more than 256 clips launches a kernel once per run of clips"]
    P = L.append
    for w, what in WIDENED:
        b = _bench_line(os.path.join(run_dir, f"{w}.log"))
        stats = os.path.join(run_dir, f"{w}_kernel_stats.csv")
        if not b or not os.path.exists(stats):
            continue
        br, rf = b["breakdown"], b["roofline"]
        P("")
        P(f"[{w}] {what}")
        P(f"    rocprofv3 --kernel-trace --stats -d {rel} -o {w} --output-format csv -- python3 bench.py --workload {w} "
          f"--steps {b['steps']} --warmup {b['warmup']} --no-cpu-baseline --no-mfma-ceiling --no-constant-run")
        parts = [f"value={b['value']:.1f} {b['unit']}", f"ms_per_step={b['ms_per_step']:.3f}"]
        parts += [f"{k}={br[k]:.3f}" for k in ("rope_ms", "pack_ms", "fwd_ms", "bwd_ms") if isinstance(br.get(k), float) and br[k] > 0]
        P("    bench line: " + " ".join(parts) + f"; roofline {rf['bound']} achieved={rf['achieved']:.1f} {rf['unit']} frac={rf['frac']:.3f}")
        P(f"    {'kernel':32s} {'calls':>5s} {'avg_ms':>9s} {'min_ms':>9s} {'max_ms':>9s}")
        for r in csv.DictReader(open(stats)):
            k = _short_kernel(r["Name"])
            if k and float(r["Percentage"]) >= 0.05 and "qknorm" not in k:
                P(f"    {k:32s} {r['Calls']:>5s} {float(r['AverageNs']) / 1e6:9.3f} {float(r['MinNs']) / 1e6:9.3f} {float(r['MaxNs']) / 1e6:9.3f}")
    tf, tw = _pmc(run_dir, "temporal_fetch"), _pmc(run_dir, "temporal_write")
    if tf and tw:
        P("")
        P(f"[C4-temporal HBM traffic]  rocprofv3 --pmc FETCH_SIZE (then WRITE_SIZE) -d {rel} -o temporal_fetch (temporal_write) --output-format csv")
        P("        -- python3 bench.py --workload C4-temporal --steps 2 --warmup 1 --no-cpu-baseline --no-mfma-ceiling")
        P("    counter scale factors from the plain-copy calibration in attention_C4_56k_rocprofv3.txt: FETCH_SIZE x 2.0, WRITE_SIZE x 1.0 (KiB)")
        tensor_gb = 56320 * 32 * 128 * 2 / 1e9
        for kname, nt_r, nt_w in (("tattn_fwd_kernel", 3, 1), ("tattn_bwd_kernel", 4, 3)):
            rg = sum(v for (k, c), v in tf.items() if c == "FETCH_SIZE" and kname.split("_kernel")[0] in k) * 2.0 * 1024 / 1e9
            wg = sum(v for (k, c), v in tw.items() if c == "WRITE_SIZE" and kname.split("_kernel")[0] in k) * 1024 / 1e9
            P(f"    {kname:20s} read {rg:.3f} GB (algorithmic {nt_r * tensor_gb:.3f}), written {wg:.3f} GB (algorithmic {nt_w * tensor_gb:.3f})")
    text = "\n".join(L) + "\n"
    os.makedirs(os.path.dirname(os.path.abspath(out_path)), exist_ok=True)
    open(out_path, "w").write(text)
    return text


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("run_dir")
    ap.add_argument("--workload", default="C4")
    ap.add_argument("--out", default=None)
    ap.add_argument("--widened", action="store_true", help="summarise the workloads beyond the headline run")
    args = ap.parse_args(argv)
    if args.widened:
        out = args.out or os.path.join(ROOT, "profiles", "widened_rows_rocprofv3.txt")
        sys.stdout.write(summarise_widened(os.path.abspath(args.run_dir), out))
        return 0
    out = args.out or os.path.join(ROOT, "profiles", f"attention_{args.workload}_rocprofv3.txt")
    sys.stdout.write(summarise(os.path.abspath(args.run_dir), args.workload, out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
