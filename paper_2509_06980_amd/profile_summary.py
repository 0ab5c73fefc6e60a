#!/usr/bin/env python3
"""Summarise rocprofv3 counter runs of bench.py for the decode-attention kernel.

Usage (after the two counter runs named in the summary it writes):
    python -m paper_2509_06980_amd.profile_summary FETCH.csv WRITE.csv [STATS.csv] > profiles/<name>.md

FETCH.csv / WRITE.csv are rocprofv3 `--pmc FETCH_SIZE` / `--pmc WRITE_SIZE` counter_collection
files (KiB per dispatch).  Both counters are calibrated against the largest device-to-device
copy of the run (the embedding table that rl_model_load copies: vocab x hidden x 2 bytes read
and written once).  Prints a markdown summary whose `traffic_bytes_per_launch` line bench.py
reads back, together with the hash of the kernel source the counters belong to.
"""
import csv
import hashlib
import os
import sys
from collections import defaultdict

HERE = os.path.dirname(os.path.abspath(__file__))
KERNEL_SRC = os.path.join(HERE, "csrc", "kernels_mfma.hip")


def kernel_source_hash():
    return hashlib.sha256(open(KERNEL_SRC, "rb").read()).hexdigest()[:16]


def read_counter(path, counter):
    """-> {kernel name: {grid size: [values]}}"""
    out = defaultdict(lambda: defaultdict(list))
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] != counter:
                continue
            name = r["Kernel_Name"].split("(")[0]
            name = name[5:] if name.startswith("void ") else name
            out[name][int(r["Grid_Size"])].append(float(r["Counter_Value"]))
    return out


def trace_summary(path):
    """Average duration of attention_mfma_kernel per grid size from a rocprofv3 kernel trace CSV
    (decode launches have grid = trajectories x kv heads x 256 threads)."""
    acc = defaultdict(lambda: [0, 0.0])
    with open(path, newline="") as f:
        for r in csv.DictReader(f):
            if "attention_mfma_kernel<false>" not in r["Kernel_Name"]:
                continue
            g = int(r.get("Grid_Size_X") or r.get("Grid_Size"))
            a = acc[g]
            a[0] += 1
            a[1] += float(r["End_Timestamp"]) - float(r["Start_Timestamp"])
    print("| attention_mfma_kernel grid (threads) | launches | avg us |\n|---|---|---|")
    for g, (n, t) in sorted(acc.items(), key=lambda kv: -kv[1][0])[:6]:
        print(f"| {g} | {n} | {t / n / 1e3:.2f} |")


def decode_step_table(fetch_path, write_path):
    """Per kernel and launch shape: mean HBM bytes fetched / written per dispatch (calibrated like
    the attention summary), for every shape with at least 100 dispatches.  With the Qwen3-4B shape
    and 128 trajectories the decode GEMM shapes are: QKV 240 workgroups (31.5 MB of weights), O and
    down 160 workgroups each (21.0 and 49.8 MB; same launch shape, so they average to 35.4 MB),
    gate-up 152 workgroups (99.6 MB), lm-head 1187 workgroups (777.9 MB)."""
    fetch = read_counter(fetch_path, "FETCH_SIZE")
    write = read_counter(write_path, "WRITE_SIZE")
    copy_bytes = 151936 * 2560 * 2

    def calib(tab):
        best = max((max(v) for v in tab.get("__amd_rocclr_copyBuffer", {}).values()), default=None)
        return copy_bytes / (best * 1024.0) if best else float("nan")

    kf, kw = calib(fetch), calib(write)
    expect = {("gemm_mfma_kernel<0, 2, 4, 4>", 240 * 256): "QKV: 31.5 MB weights + 5 x 3.1 MB partial sums written",
              ("gemm_mfma_kernel<0, 2, 4, 4>", 160 * 256): "O / down mixed: 35.4 MB weights + 8 x 1.3 MB written",
              ("gemm_mfma_kernel<2, 2, 4, 4>", 152 * 256): "gate-up: 99.6 MB weights, 2.5 MB written",
              ("gemm_mfma_kernel<0, 2, 4, 4>", 1187 * 256): "lm-head: 777.9 MB weights, 77.8 MB logits written"}
    print("# HBM traffic per dispatch of the decode-step kernels (Qwen3-4B shape, 128 trajectories)\n")
    print("Commands (MI355X box, repository root; one counter per run; the rollout is shortened, the "
          "decode launch shapes are those of the full workload):\n")
    print("    rocprofv3 --pmc FETCH_SIZE --output-format csv -d out/pmc_fetch_all -o f -- python3 bench.py "
          "--warmup 0 --no-cpu-baseline --scale 0.1")
    print("    rocprofv3 --pmc WRITE_SIZE --output-format csv -d out/pmc_write_all -o w -- python3 bench.py "
          "--warmup 0 --no-cpu-baseline --scale 0.1")
    print("    python -m paper_2509_06980_amd.profile_summary --decode-step <f_counter_collection.csv> <w_counter_collection.csv>\n")
    print(f"FETCH_SIZE factor {kf:.4f}, WRITE_SIZE factor {kw:.4f} (embedding-table copy of {copy_bytes} bytes).\n")
    print("| kernel | grid (threads) | dispatches | fetched MB | written MB | algorithmic |\n|---|---|---|---|---|---|")
    rows = []
    for k, grids in fetch.items():
        for g, vals in grids.items():
            if len(vals) < 100:
                continue
            wv = write.get(k, {}).get(g, [])
            rows.append((k, g, len(vals), sum(vals) / len(vals) * 1024 * kf / 1e6,
                         sum(wv) / len(wv) * 1024 * kw / 1e6 if wv else float("nan")))
    for k, g, n, fm, wm in sorted(rows, key=lambda r: -r[2] * (r[3] + r[4])):
        print(f"| {k[:60]} | {g} | {n} | {fm:.2f} | {wm:.2f} | {expect.get((k, g), '')} |")


def mfma_table(counter_path, trace_path):
    """Matrix-core work per kernel and launch shape: bf16 MFMA operations the hardware counted
    (SQ_INSTS_VALU_MFMA_MOPS_BF16, 512 flops each) against the kernel's duration from a kernel trace
    of the same command, for every shape with at least 20 dispatches."""
    mops = read_counter(counter_path, "SQ_INSTS_VALU_MFMA_MOPS_BF16")
    dur = defaultdict(lambda: defaultdict(list))
    with open(trace_path, newline="") as f:
        for r in csv.DictReader(f):
            name = r["Kernel_Name"].split("(")[0]
            name = name[5:] if name.startswith("void ") else name
            if r.get("Grid_Size_X"):    # the counter file gives the total number of threads of a launch
                g = int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y") or 1) * int(r.get("Grid_Size_Z") or 1)
            else:
                g = int(r["Grid_Size"])
            dur[name][g].append(float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
    peak = 2500.0
    print("# Matrix-core (MFMA) utilisation of the chunked-prefill kernels and the decode GEMMs "
          "(Qwen3-4B shape, 128 trajectories)\n")
    print("Commands (MI355X box, repository root; counters and durations in separate runs of the same command):\n")
    print("    rocprofv3 --pmc SQ_INSTS_VALU_MFMA_MOPS_BF16 --kernel-include-regex 'gemm|attention' "
          "--output-format csv -d out/pmc_mfma -o m -- python3 bench.py --warmup 0 --no-cpu-baseline --scale 0.5")
    print("    rocprofv3 --kernel-trace --output-format csv -d out/trace_half -o t -- python3 bench.py --warmup 0 "
          "--no-cpu-baseline --scale 0.5")
    print("    python -m paper_2509_06980_amd.profile_summary --mfma <m_counter_collection.csv> <t_kernel_trace.csv>\n")
    print("MFMA flops = counter x 512 (the counter includes the padded columns and rows a kernel "
          "multiplies: decode attention fills 4 of 16 MFMA columns, a 128-row decode GEMM all of them); "
          f"peak {peak:.0f} TFLOP/s dense bf16.\n")
    print("| kernel | grid (threads) | dispatches | avg us | MFMA GFLOP per dispatch | TFLOP/s | of peak |\n|---|---|---|---|---|---|---|")
    rows = []
    for k, grids in mops.items():
        for g, vals in grids.items():
            d = dur.get(k, {}).get(g, [])
            if len(vals) < 20 or not d:
                continue
            fl = sum(vals) / len(vals) * 512.0
            us = sum(d) / len(d) / 1e3
            rows.append((k, g, len(vals), us, fl))
    for k, g, n, us, fl in sorted(rows, key=lambda r: -r[2] * r[3]):
        tf = fl / (us * 1e-6) / 1e12 if us > 0 else 0.0
        print(f"| {k[:64]} | {g} | {n} | {us:.1f} | {fl / 1e9:.1f} | {tf:.0f} | {tf / peak:.3f} |")


def rollout_summary(trace_path, stats_path, bench_log):
    """Kernel summary of a profiled bench.py run: the decode-attention launches by shape (kernel
    trace), rocprofv3's own per-kernel statistics, and the figures bench.py printed in that run
    (`bench_log`: its captured output; the last line starting with {"metric" is used)."""
    import json
    line = [l for l in open(bench_log).read().splitlines() if l.startswith('{"metric"')][-1]
    b = json.loads(line)
    r = b["roofline"]
    print("# rocprofv3 kernel summary: attention_mfma_kernel and the rest of the cfg3 rollout "
          "(Qwen3-4B shape, 128 trajectories)\n")
    print("Commands (on the MI355X box, from the repository root):\n")
    print("    cd /tmp && export TMPDIR=/tmp && cd <repository root> && rocprofv3 --kernel-trace --stats "
          "--output-format csv -d out/prof_full -o cfg3 -- python3 bench.py --no-cpu-baseline > out/bench.log")
    print("    python -m paper_2509_06980_amd.profile_summary --rollout out/prof_full/<host>/cfg3_kernel_trace.csv "
          "out/prof_full/<host>/cfg3_kernel_stats.csv out/bench.log\n")
    print("The run covers one warm-up rollout plus one timed rollout (2 x 2048 decode steps, 2 x 5 appends).\n")
    print(f"bench.py line of the same run: value {b['value']} tokens/s, decode-only "
          f"{b['decode_only_tokens_per_s']} tokens/s, decode-step HBM fraction {b['decode_step_hbm']['frac']} "
          f"(distinct pages; {b['decode_step_hbm'].get('achieved_counting_shared_pages_per_trajectory')} GB/s when "
          f"every trajectory is charged its whole context); roofline: {r['achieved']} GB/s over distinct pages "
          f"({r['achieved_counting_shared_pages_per_trajectory']} GB/s counting shared prompt pages per trajectory), "
          f"{r['avg_launch_us']} us per decode launch (HIP events around attention + merge, every 16th step), "
          f"{r['bytes_per_launch']} bytes per launch; measured streaming-read ceiling of the box "
          f"{b['measured_stream_read_GBs']} GB/s.\n")
    print("attention_mfma_kernel<false> (the bf16-cache instance; decode launches: one workgroup per "
          "trajectory x kv head) by launch shape, from the kernel trace:\n")
    trace_summary(trace_path)
    print("\nThe decode average agrees with the HIP-event figure of bench.py (the profiler adds a little "
          "per-launch overhead to the event bracket). Chunked prefill runs in attention_prefill_lds_kernel.\n")
    print("| kernel | calls | total ms | avg us | % |\n|---|---|---|---|---|")
    with open(stats_path, newline="") as f:
        for x in csv.DictReader(f):
            n = x["Name"][5:] if x["Name"].startswith("void ") else x["Name"]
            print(f"| {n.split('(')[0]} | {x['Calls']} | {float(x['TotalDurationNs']) / 1e6:.1f} | "
                  f"{float(x['AverageNs']) / 1e3:.2f} | {float(x['Percentage']):.2f} |")


def stall_table(path_a, path_b):
    """Where the GEMM and attention kernels spend their cycles, per kernel and launch shape, from
    two counter runs of the same command (a: wave / MFMA / wait counters of the SQ block,
    b: GRBM_GUI_ACTIVE, texture-addresser and L1 stall counters).  Ratios:
      MFMA busy   = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 XCDs x 1024 SIMDs)
      waves wait  = SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES (share of resident wave time spent waiting)
      ... on LDS  = SQ_WAIT_INST_LDS / SQ_WAVE_CYCLES
      TA busy     = TA_TA_BUSY_sum / (GRBM_GUI_ACTIVE / 8 x 256 CUs)
      L1 pending  = TCP_PENDING_STALL_CYCLES_sum / (GRBM_GUI_ACTIVE / 8 x 256 CUs)
      clock       = GRBM_GUI_ACTIVE / 8 / kernel duration"""
    def read_all(path):
        out = defaultdict(lambda: defaultdict(lambda: defaultdict(list)))
        dur = defaultdict(lambda: defaultdict(list))
        with open(path, newline="") as f:
            for r in csv.DictReader(f):
                name = r["Kernel_Name"].split("(")[0]
                name = name[5:] if name.startswith("void ") else name
                g = int(r["Grid_Size"])
                out[name][g][r["Counter_Name"]].append(float(r["Counter_Value"]))
                if r["Counter_Name"] == "GRBM_GUI_ACTIVE":
                    dur[name][g].append(float(r["End_Timestamp"]) - float(r["Start_Timestamp"]))
        return out, dur
    a, _ = read_all(path_a)
    b, dur = read_all(path_b)
    mean = lambda v: sum(v) / len(v) if v else float("nan")
    print("# Stall profile of the GEMM and attention kernels (Qwen3-4B shape, 128 trajectories, half lengths)\n")
    print("Commands (MI355X box, repository root; two counter sets, one run each):\n")
    print("    rocprofv3 --pmc SQ_WAVE_CYCLES SQ_BUSY_CYCLES SQ_VALU_MFMA_BUSY_CYCLES SQ_WAIT_INST_LDS SQ_WAIT_INST_ANY "
          "SQ_LDS_BANK_CONFLICT SQ_LDS_IDX_ACTIVE --kernel-include-regex 'gemm|attention' --output-format csv "
          "-d out/pmc_sq_a -o a -- python3 bench.py --warmup 0 --no-cpu-baseline --scale 0.5")
    print("    rocprofv3 --pmc GRBM_GUI_ACTIVE SQ_LDS_DATA_FIFO_FULL SQ_LDS_CMD_FIFO_FULL TA_TA_BUSY_sum "
          "TA_ADDR_STALLED_BY_TC_CYCLES_sum TCP_PENDING_STALL_CYCLES_sum TCP_TCP_TA_DATA_STALL_CYCLES_sum "
          "--kernel-include-regex 'gemm|attention' --output-format csv -d out/pmc_sq_b -o b -- python3 bench.py "
          "--warmup 0 --no-cpu-baseline --scale 0.5")
    print("    python -m paper_2509_06980_amd.profile_summary --stalls <a_counter_collection.csv> <b_counter_collection.csv>\n")
    print("GRBM_GUI_ACTIVE is summed over the 8 XCDs; durations are those of the counter run (kernels run one at a "
          "time there).  MFMA busy counts issue cycles of the matrix pipes against 1024 SIMDs.  The clock column is "
          "GRBM_GUI_ACTIVE over the kernel's duration: meaningful for the long kernels only (for kernels of a few "
          "tens of microseconds the counter window includes the launch, and the figure reads high).\n")
    print("| kernel | grid (threads) | dispatches | avg us | clock GHz | MFMA busy | waves wait | ... on LDS | LDS bank conflicts | TA busy | L1 pending-miss stall |")
    print("|---|---|---|---|---|---|---|---|---|---|---|")
    rows = []
    for k, grids in b.items():
        for g, cb in grids.items():
            ca = a.get(k, {}).get(g)
            if not ca or len(cb.get("GRBM_GUI_ACTIVE", [])) < 20:
                continue
            gui = mean(cb["GRBM_GUI_ACTIVE"]) / 8.0
            us = mean(dur[k][g]) / 1e3
            wave = mean(ca["SQ_WAVE_CYCLES"])
            rows.append((k, g, len(cb["GRBM_GUI_ACTIVE"]), us, gui / (us * 1e3),
                         mean(ca["SQ_VALU_MFMA_BUSY_CYCLES"]) / (gui * 1024.0),
                         mean(ca["SQ_WAIT_INST_ANY"]) / wave, mean(ca["SQ_WAIT_INST_LDS"]) / wave,
                         mean(ca["SQ_LDS_BANK_CONFLICT"]),
                         mean(cb["TA_TA_BUSY_sum"]) / (gui * 256.0),
                         mean(cb["TCP_PENDING_STALL_CYCLES_sum"]) / (gui * 256.0)))
    for r in sorted(rows, key=lambda r: -r[2] * r[3]):
        print(f"| {r[0][:56]} | {r[1]} | {r[2]} | {r[3]:.1f} | {r[4]:.2f} | {r[5]:.2f} | {r[6]:.2f} | {r[7]:.2f} | "
              f"{r[8]:.0f} | {r[9]:.2f} | {r[10]:.2f} |")


def main():
    if sys.argv[1] == "--stalls":
        return stall_table(sys.argv[2], sys.argv[3])
    if sys.argv[1] == "--rollout":
        return rollout_summary(sys.argv[2], sys.argv[3], sys.argv[4])
    if sys.argv[1] == "--trace":
        return trace_summary(sys.argv[2])
    if sys.argv[1] == "--mfma":
        return mfma_table(sys.argv[2], sys.argv[3])
    if sys.argv[1] == "--decode-step":
        return decode_step_table(sys.argv[2], sys.argv[3])
    fetch = read_counter(sys.argv[1], "FETCH_SIZE")
    write = read_counter(sys.argv[2], "WRITE_SIZE")
    vocab, hidden, n_traj, n_kv = 151936, 2560, 128, 8
    copy_bytes = vocab * hidden * 2

    def calib(tab):
        best = max((max(v) for g in tab.get("__amd_rocclr_copyBuffer", {}).values() for v in [g]), default=None)
        return copy_bytes / (best * 1024.0) if best else float("nan")

    kf, kw = calib(fetch), calib(write)
    grid = n_traj * n_kv * 256                      # decode launches: one workgroup per (trajectory, kv head)
    name = "attention_mfma_kernel<false>"           # the bf16-cache instance of the decode kernel
    fa = fetch[name][grid]
    wa = write[name][grid]
    f_bytes = sum(fa) / len(fa) * 1024.0 * kf
    w_bytes = sum(wa) / len(wa) * 1024.0 * kw
    print("# HBM traffic of attention_mfma_kernel, cfg3 rollout (Qwen3-4B shape, 128 trajectories)\n")
    print("Commands (MI355X box, repository root; one counter per run):\n")
    print("    rocprofv3 --pmc FETCH_SIZE --kernel-include-regex 'attention_mfma_kernel|copyBuffer' "
          "--output-format csv -d out/pmc_fetch -o f -- python3 bench.py --warmup 0 --no-cpu-baseline")
    print("    rocprofv3 --pmc WRITE_SIZE --kernel-include-regex 'attention_mfma_kernel|copyBuffer' "
          "--output-format csv -d out/pmc_write -o w -- python3 bench.py --warmup 0 --no-cpu-baseline")
    print("    python -m paper_2509_06980_amd.profile_summary <f_counter_collection.csv> <w_counter_collection.csv>\n")
    print(f"Calibration copy: embedding table, {copy_bytes} bytes read and written by `__amd_rocclr_copyBuffer`; "
          f"FETCH_SIZE factor {kf:.4f}, WRITE_SIZE factor {kw:.4f} (expected bytes / counter KiB x 1024).\n")
    print(f"Decode launches (grid {grid} threads): {len(fa)} with FETCH_SIZE, {len(wa)} with WRITE_SIZE.\n")
    print(f"- fetched from HBM per launch: {f_bytes / 1e6:.1f} MB")
    print(f"- written to HBM per launch: {w_bytes / 1e6:.1f} MB")
    print(f"- traffic_bytes_per_launch: {f_bytes + w_bytes:.0f}")
    print(f"- kernel_source_sha256_16: {kernel_source_hash()}")


if __name__ == "__main__":
    main()
