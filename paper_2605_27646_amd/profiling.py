"""Turns raw rocprofv3 output of bench.py runs into the short text summaries kept under profiles/.

    python -m paper_2605_27646_amd.profiling <raw_dir> <workload>

<raw_dir> holds what these commands wrote (each run from /tmp with TMPDIR=/tmp, <repo> = the repository):

    python3 <repo>/bench.py --workload W --stream-ceiling > <raw_dir>/bench.json
    rocprofv3 --kernel-trace --stats --output-format csv -d <raw_dir> -o trace -- \
        python3 <repo>/bench.py --workload W --steps 3 --warmup 1 --no-cpu-baseline
    rocprofv3 --pmc FETCH_SIZE --output-format csv -d <raw_dir> -o fetch -- \
        python3 <repo>/bench.py --workload W --steps 1 --warmup 0 --layers 2 --no-cpu-baseline --no-append --calibrate-copy
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d <raw_dir> -o write -- (the same bench.py arguments)
    rocprofv3 --pmc SQ_WAVES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_ACTIVE_INST_VALU SQ_BUSY_CYCLES SQ_WAVE_CYCLES \
        SQ_INSTS_SALU SQ_INSTS_LDS --output-format csv -d <raw_dir> -o insts -- \
        python3 <repo>/bench.py --workload W --steps 1 --warmup 0 --layers 1 --no-cpu-baseline --no-append --q-heads-per-kv 0

Writes profiles/hot_path_kernels_W.txt, profiles/hbm_traffic_W.txt and profiles/instruction_counters_W.txt.  The
lines `figure <kernel> <name> <value>` at the end of the last two are what bench.py reads back for the
`traffic` and `executed` parts of its JSON line.  Nothing here touches a GPU."""
from __future__ import annotations

import collections
import csv
import json
import os
import re
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
N_SIMD = 256 * 4
CLOCK_GHZ = 2.4


def short(name: str) -> str:
    m = re.search(r"hqmq::(k_[a-z_]+(?:<[^>]*>)?)", name)
    return "hqmq::" + (m.group(1) if m else name)


def base(name: str) -> str:
    m = re.search(r"hqmq::(k_[a-z_]+)", name)
    return m.group(1) if m else name


def counters(path: str) -> dict:
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        acc[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in acc.items()}


def main(raw: str, wl: str) -> None:
    d = json.loads(open(f"{raw}/bench.json").read().strip().split("\n")[-1])
    cfg = d["config"]
    nt = cfg["tensors_per_step"]
    groups = (nt + 31) // 32
    per_launch = nt / groups
    shape = f"[{cfg['B']}, {cfg['kv_heads']}, {cfg['T']}, {cfg['D']}]"
    n_c = (cfg["D"] + 3) // 4
    chunks = cfg["B"] * cfg["kv_heads"] * cfg["T"] * n_c
    has_att = "attend" in d
    rf, rd = d["roofline"], d["roofline_decode"]
    os.makedirs(f"{ROOT}/profiles", exist_ok=True)

    # ---- kernel trace ----------------------------------------------------------------------------------
    rows = [r for r in csv.DictReader(open(f"{raw}/trace_kernel_stats.csv")) if "hqmq" in r["Name"]]
    out = [f"""Kernel-trace summary of the whole hot path, workload {wl} ({cfg['layers']} layers, K and V,
{shape} fp16 each, S = {cfg['S']}, b_r = {cfg['b_r']}, C = {cfg['C']:g}), MI355X, 4 steps (1 warm-up + 3 timed) of {nt} tensors.
A step is {groups} hqmq_encode_batch call(s) and one hqmq_decode_batch call; every kernel launch covers {per_launch:g} tensors
(blockIdx.z = tensor).""" + ("""  After the timed steps bench.py runs its fused-attention extra (6 passes of one
hqmq_attend per layer, 4 query heads per kv head).""" if has_att else "") + ("""  Then its appended-token extra: 53 encodes of the
one-token tensors of a generation step with supplied thresholds (the fused search kernel `k_search<.., true, ..>` or
`k_search_flat<.., true, ..>` and `k_list_small`, two launches of 32 tensors each per encode).""" if "append" in d else "") + f"""

command (run from /tmp with TMPDIR=/tmp):
  rocprofv3 --kernel-trace --stats --output-format csv -d <out> -o trace -- python3 bench.py --workload {wl} --steps 3 --warmup 1 --no-cpu-baseline

kernel ({per_launch:g} tensors per launch unless noted)       calls     avg (us)   min (us)   max (us)   % time   avg per tensor (us)"""]
    for r in rows:
        nm = short(r["Name"])
        per = "" if "attend" in nm else f"{float(r['AverageNs']) / 1e3 / per_launch:10.1f}"
        if "attend" in nm:
            nm += " (per layer)"
        out.append(f"{nm:48s} {r['Calls']:>6s} {float(r['AverageNs']) / 1e3:12.1f} {float(r['MinNs']) / 1e3:10.1f} "
                   f"{float(r['MaxNs']) / 1e3:10.1f} {float(r['Percentage']):8.2f} {per}")
    ex, fe32 = rf["executed_mfma"], rf["fp32_equivalent"]
    out.append(f"""
(% time is of all GPU kernels in the process, including torch's generators for the synthetic inputs.)

bench.py line of the same build (python bench.py --workload {wl}; {d['warmup']} warm-up + {d['steps']} timed steps; HIP-event times on the launch stream):
  search kernel: avg launch {rf['avg_launch_ms'] * 1e3:.1f} us for {per_launch:g} tensors (median {rf['median_launch_ms'] * 1e3:.1f}, min {rf['min_launch_ms'] * 1e3:.1f}; {rf['avg_launch_ms'] * 1e3 / per_launch:.1f} us per tensor)  ->  bound by VALU issue:
      closed-form scoring, {rf['flops_per_chunk']:g} VALU lane-operations per chunk ({chunks:,} chunks per tensor): {rf['achieved']:.1f} T op/s of the {rf['peak']:.1f} the chip issues = {rf['frac'] * 100:.1f} %;
      fp32-equivalent ({fe32['flops_per_chunk']:g} flop per chunk): {fe32['achieved']:.1f} TFLOP/s = {fe32['ratio_to_fp32_peak']:.3f} x the 157.3 fp32 peak (the metric's yardstick, not a roofline fraction: the contraction runs as fp16 products);
      executed on the matrix cores: {ex['instruction']}, {ex['achieved']:.0f} TFLOP/s of 2500 = {ex['frac'] * 100:.1f} %
  decode kernel: avg launch {rd['avg_launch_ms'] * 1e3:.1f} us for {rd['tensors_per_launch']:g} tensors (median {rd['median_launch_ms'] * 1e3:.1f}, min {rd['min_launch_ms'] * 1e3:.1f}; {rd['avg_launch_ms'] * 1e3 / rd['tensors_per_launch']:.1f} us per tensor)  ->  {rd['achieved']:.0f} GB/s of 8000 = {rd['frac'] * 100:.1f} % ({rd['bytes_per_chunk']:.2f} B per chunk)
  encode {d['encode_elems_per_s']:.3e} elems/s, decode {d['decode_elems_per_s']:.3e} elems/s, encode+decode {d['value']:.3e} elems/s ({d['ms_per_step']:.1f} ms per step)
  encode phases per tensor: median select {d['encode_phase_ms_per_tensor']['median_select'] * 1e3:.1f} us ({d['median_select_GBs']:.0f} GB/s over the {d['median_select_reads']:.4g} reads of the tensor it makes), search + quantise + pack {d['encode_phase_ms_per_tensor']['search_quantise_pack'] * 1e3:.1f} us, outlier scan + gather {d['encode_phase_ms_per_tensor']['outlier_scan_gather'] * 1e3:.1f} us
  outlier fraction {d['outlier_fraction']:.4f}, stored bits per element {d['bits_per_element_stored']:.3f}""")
    if has_att:
        at = d["attend"]
        out.append(f"  fused attention extra: {at['us_per_layer']:.1f} us per layer (k_attend_joint or k_attend_partial, then k_attend_merge) for {cfg['T']} cached "
                   f"tokens x {cfg['kv_heads'] * at['q_heads_per_kv_head']} query heads, reading {at['packed_bytes_per_layer'] / 1e6:.1f} MB of "
                   f"packed K and V (fp16 cache: {at['fp16_cache_bytes_per_layer'] / 1e6:.1f} MB)")
    if "append" in d:
        apd = d["append"]
        out.append(f"  appended-token extra: {apd['us_per_step']:.1f} us for the {apd['tensors']} tensors {apd['shape']} of one generation step "
                   f"(hqmq_encode_batch with supplied thresholds: the fused search kernel and k_list_small, one launch each per 32 tensors)")
    if "cpu_baseline" in d:
        cb = d["cpu_baseline"]
        out.append(f"  cpu_baseline (the oracle, {cb['cores']} threads, {cb['sample']}): {cb['value']:.3e} elems/s; "
                   f"one thread ({cb['single_thread']['sample']}): {cb['single_thread']['value']:.3e} elems/s")
    if "stream_ceiling" in d:
        sc = d["stream_ceiling"]
        out.append(f"  streaming kernels on the same box (bench.py --stream-ceiling: {sc['what']}): fill {sc['fill_GBs']:.0f} GB/s, "
                   f"copy {sc['copy_GBs']:.0f} GB/s (read + written)")
    if "parity_sample" in d:
        ps = d["parity_sample"]
        out.append(f"  parity on the oracle's sample of layer 0 K: {ps['chunks_compared']:,} chunks compared, {ps['near_ties']} near-ties "
                   f"(gap < 1e-6), {ps['index_mismatches_in_near_ties']} of them resolved differently, "
                   f"{ps['index_mismatches_elsewhere']} mismatches elsewhere, {ps['radius_code_mismatches']} radius-code mismatches, "
                   f"masks / offsets / payload / scales identical: {ps['masks_offsets_payload_scales_identical']}")
    open(f"{ROOT}/profiles/hot_path_kernels_{wl}.txt", "w").write("\n".join(out) + "\n")

    # ---- HBM traffic ------------------------------------------------------------------------------------
    if os.path.exists(f"{raw}/fetch_counter_collection.csv") and os.path.exists(f"{raw}/write_counter_collection.csv"):
        fe, wr = counters(f"{raw}/fetch_counter_collection.csv"), counters(f"{raw}/write_counter_collection.csv")
        cal_f = [v["FETCH_SIZE"] for k, v in fe.items() if "vectorized_elementwise_kernel<8" in k][0]
        cal_w = [v["WRITE_SIZE"] for k, v in wr.items() if "vectorized_elementwise_kernel<8" in k][0]
        tensor_kib = cfg["B"] * cfg["kv_heads"] * cfg["T"] * cfg["D"] * 2 / 1024
        ff, fw = tensor_kib / cal_f, tensor_kib / cal_w
        lines = [f"""HBM traffic per launch from rocprofv3 PMC counters, workload {wl} ({shape} fp16 tensors,
S = {cfg['S']}, b_r = {cfg['b_r']}), MI355X.  FETCH_SIZE and WRITE_SIZE are reported in KiB per dispatch; each was collected in a run of
its own and scaled by what the same counter reads for a plain copy of known size in the same run
(torch.add(x, 0, out=y) on one tensor: {tensor_kib:g} KiB read, {tensor_kib:g} KiB written).  This 2-layer run has 4 tensors:
every encode / decode kernel is ONE launch over the 4 tensors""" + ("; the attention kernels run once per layer." if has_att else ".") + f"""

commands (run from /tmp with TMPDIR=/tmp):
  rocprofv3 --pmc FETCH_SIZE --output-format csv -d <out> -o fetch -- python3 bench.py --workload {wl} --steps 1 --warmup 0 --layers 2 --no-cpu-baseline --no-append --calibrate-copy
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d <out> -o write -- python3 bench.py --workload {wl} --steps 1 --warmup 0 --layers 2 --no-cpu-baseline --no-append --calibrate-copy

calibration copy: FETCH_SIZE reads {cal_f:.1f} KiB for {tensor_kib:g} KiB  -> factor {ff:.3f};  WRITE_SIZE reads {cal_w:.1f} KiB -> factor {fw:.3f}

kernel                                      FETCH (KiB)    WRITE (KiB)   read MB scaled written MB scaled   per tensor (read + written MB)"""]
        per = {}
        for k in fe:
            if "hqmq" not in k or k not in wr:
                continue
            f, w = fe[k]["FETCH_SIZE"], wr[k]["WRITE_SIZE"]
            r_mb, w_mb = f * ff * 1024 / 1e6, w * fw * 1024 / 1e6
            nt_l = 1 if "attend" in k else 4
            per[base(k)] = (r_mb / nt_l, w_mb / nt_l)
            lines.append(f"{short(k):42s} {f:12.1f} {w:14.1f} {r_mb:16.2f} {w_mb:16.2f}   {r_mb / nt_l:8.2f} + {w_mb / nt_l:.2f}"
                         + (" (per layer)" if nt_l == 1 else ""))
        skey = "k_search" if "k_search" in per else "k_search_flat"
        dkey = "k_decode" if "k_decode" in per else "k_decode_rows"
        s, dk = per[skey], per[dkey]
        info_w = rd["bytes_per_chunk"] - 8.0
        x_mb = chunks * 8 / 1e6
        lines.append(f"""
algorithmic bytes for comparison, per tensor: the search kernel reads the tensor, {x_mb:.1f} MB (8 B per chunk; the flat kernel for
head dimensions other than 128 reads it twice, the second time from L2) and writes codes, flags, scales and offsets,
{chunks * (info_w - 8 * d['outlier_fraction']) / 1e6:.1f} MB; the decode kernel reads {chunks * info_w / 1e6:.1f} MB (codes, flags, scales, offsets, payload) and writes {x_mb:.1f} MB.
measured per tensor: search {s[0] + s[1]:.1f} MB ({s[0]:.1f} read + {s[1]:.1f} written); decode {dk[0] + dk[1]:.1f} MB ({dk[0]:.1f} read + {dk[1]:.1f} written).""")
        akey = "k_attend_joint" if "k_attend_joint" in per else "k_attend_partial"
        if has_att and akey in per:
            ak = per[akey]
            lines.append(f"{akey} {ak[0]:.1f} MB read + {ak[1]:.1f} MB written per layer (algorithmic: the packed K and V of a layer, "
                         f"{d['attend']['packed_bytes_per_layer'] / 1e6:.1f} MB).")
        lines.append("\nfigures read back by bench.py (bytes per tensor, read + written):")
        lines.append(f"figure {skey} traffic_bytes_per_tensor {(s[0] + s[1]) * 1e6:.0f}")
        lines.append(f"figure {dkey} traffic_bytes_per_tensor {(dk[0] + dk[1]) * 1e6:.0f}")
        open(f"{ROOT}/profiles/hbm_traffic_{wl}.txt", "w").write("\n".join(lines) + "\n")

    # ---- instruction counters ---------------------------------------------------------------------------
    if os.path.exists(f"{raw}/insts_counter_collection.csv"):
        ic = counters(f"{raw}/insts_counter_collection.csv")
        lines = [f"""Instruction counters of the hot-path kernels, workload {wl} ({shape} fp16 tensors, S = {cfg['S']}, b_r = {cfg['b_r']}), MI355X:
one rocprofv3 PMC pass over a 1-layer run (2 tensors: every encode / decode kernel is ONE launch over both).  Counters are
sums over the launch.  SQ_ACTIVE_INST_VALU counts in units of 4 cycles; with {N_SIMD} SIMDs and a nominal {CLOCK_GHZ} GHz clock
"VALU busy" below is 4 x SQ_ACTIVE_INST_VALU / {N_SIMD} cycles, i.e. the time every SIMD's vector ALU would be busy if the work
were spread evenly; "launch" is the kernel's average duration in the kernel trace of the same build (32 tensors per launch),
scaled to the 2 tensors of this run.

command (run from /tmp with TMPDIR=/tmp):
  rocprofv3 --pmc SQ_WAVES SQ_INSTS_VALU SQ_INSTS_MFMA SQ_ACTIVE_INST_VALU SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_SALU SQ_INSTS_LDS --output-format csv -d <out> -o insts -- python3 bench.py --workload {wl} --steps 1 --warmup 0 --layers 1 --no-cpu-baseline --no-append --q-heads-per-kv 0

kernel                              waves   VALU/wave   MFMA/wave   SALU/wave    LDS/wave   VALU busy (us)   launch (us, 2 tensors)   busy / launch"""]
        trace_us = {short(r["Name"]): float(r["AverageNs"]) / 1e3 / per_launch * 2 for r in rows}
        figs = []
        for k, c in ic.items():
            if "hqmq" not in k or not c.get("SQ_WAVES"):
                continue
            wv = c["SQ_WAVES"]
            busy_us = 4 * c["SQ_ACTIVE_INST_VALU"] / N_SIMD / (CLOCK_GHZ * 1e3)
            t = trace_us.get(short(k))
            lines.append(f"{short(k):32s} {wv:8.0f} {c['SQ_INSTS_VALU'] / wv:11.1f} {c['SQ_INSTS_MFMA'] / wv:11.2f} "
                         f"{c['SQ_INSTS_SALU'] / wv:11.1f} {c['SQ_INSTS_LDS'] / wv:11.1f} {busy_us:16.1f} "
                         + (f"{t:24.1f} {busy_us / t:15.2f}" if t else ""))
            m = re.search(r"(k_search(?:_flat)?)<(\d+), (\d+)(?:, \w+)*>", k)
            if m:
                waves_wg, rows_wg = int(m.group(2)), int(m.group(3))
                # passes of 64 chunks per wave: two rows of 32 chunks per pass in k_search; in k_search_flat the
                # workgroup's rows as one flat list of chunks shared by its waves
                passes = rows_wg / (2 * waves_wg) if m.group(1) == "k_search" else -(-rows_wg * n_c // (64 * waves_wg))
                figs.append((m.group(1), c["SQ_INSTS_VALU"] / wv / passes, c["SQ_INSTS_MFMA"] / wv / passes, passes))
        lines.append("")
        for name, v, mf, passes in figs:
            s16 = (cfg["S"] + 15) // 16
            lines.append(f"{name}: {passes:g} passes of 64 chunks per wave -> {v:.1f} VALU and {mf:.2f} MFMA instructions per pass; the closed form "
                         f"alone is 5.5 x 16 x {s16} = {5.5 * 16 * s16:g} VALU instructions per pass ({5.5 * 16 * s16 / v * 100:.1f} % of the executed ones), "
                         f"the analytic MFMA count 4 x {s16} + 1 = {4 * s16 + 1}.")
        lines.append("\nfigures read back by bench.py:")
        for name, v, mf, passes in figs:
            lines.append(f"figure {name} valu_instructions_per_pass {v:.1f}")
            lines.append(f"figure {name} mfma_instructions_per_pass {mf:.2f}")
        open(f"{ROOT}/profiles/instruction_counters_{wl}.txt", "w").write("\n".join(lines) + "\n")
    print("wrote profiles for", wl)


if __name__ == "__main__":
    main(sys.argv[1], sys.argv[2])
