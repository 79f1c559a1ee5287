"""Summarises two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, WRITE_SIZE; csv output) into the HBM-side traffic of
the MFMA GEMM kernel per launch, scaled by what the same counters read for the plain 256 MiB device copy that
`bench.py --copy-calibration` issues.  Also records the hash of the kernel source so that bench.py can tell
whether the figure still belongs to the kernel it times.

usage: python -m paper_2011_13635_amd.pmc_summary <fetch_counter_collection.csv> <write_counter_collection.csv> <steps_in_run>
       python -m paper_2011_13635_amd.pmc_summary --mfma <counter_collection.csv> <steps_in_run>
       python -m paper_2011_13635_amd.pmc_summary --rowwise <fetch_counter_collection.csv> <write_counter_collection.csv> <last_steps>
The second form summarises a run with SQ_VALU_MFMA_BUSY_CYCLES and SQ_INSTS_VALU_MFMA_MOPS_BF16: the FLOPs the
matrix cores executed (512 per counted operation) and the fraction of the kernels' duration their pipes were busy.
The third form gives, for every kernel that is not a GEMM, the HBM-side bytes per launch (FETCH_SIZE + WRITE_SIZE,
scaled by the copy) over the last <last_steps> steps of the run (the event-timing pass of bench.py, in which every
kernel runs alone), its average duration there and the resulting GB/s.
"""
from __future__ import annotations

import csv
import hashlib
import os
import re
import sys

CSRC = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
KERNEL_SOURCES = [os.path.join(CSRC, f) for f in ("gemm_ring.hip", "gemm_mfma.hip", "gemm_epilogue.h", "common.h")]
ROWWISE_SOURCES = [os.path.join(CSRC, f) for f in ("rowwise.hip", "attention_mfma.hip", "common.h")]
GEMM_KERNELS = ("k_gemm_mfma", "k_gemm_ring")
COPY_BYTES = 256 * 1024 * 1024


def rowwise_source_hash() -> str:
    return kernel_source_hash(ROWWISE_SOURCES)


def kernel_source_hash(sources=None) -> str:
    """Hash of the kernels' code: comments and blank space do not count."""
    h = hashlib.sha256()
    for path in (sources or KERNEL_SOURCES):
        text = open(path, encoding="utf-8").read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        for line in text.splitlines():
            line = re.sub(r"//.*", "", line)
            line = "".join(line.split())
            if line:
                h.update(line.encode() + b"\n")
    return h.hexdigest()


def read_counter(path):
    copy_kib, gemm = 0.0, {}
    for r in csv.DictReader(open(path)):
        name, v = r["Kernel_Name"], float(r["Counter_Value"])
        if "copyBuffer" in name:
            copy_kib = max(copy_kib, v)
        elif any(g in name for g in GEMM_KERNELS):
            n, s = gemm.get(name, (0, 0.0))
            gemm[name] = (n + 1, s + v)
    return copy_kib, gemm


SIMDS = 256 * 4            # compute units x SIMDs
CLOCK_HZ = 2.4e9           # the clock the published peak is quoted at


def mfma_main(path, steps):
    per = {}
    for r in csv.DictReader(open(path)):
        name = r["Kernel_Name"]
        if "mfma" not in name and "attn" not in name and "k_gemm" not in name:
            continue
        key = name.split("(")[0].replace("void ", "")
        e = per.setdefault(key, {"ids": set(), "ns": 0, "busy": 0.0, "mops": 0.0})
        if r["Dispatch_Id"] not in e["ids"]:
            e["ids"].add(r["Dispatch_Id"])
            e["ns"] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
        if r["Counter_Name"] == "SQ_VALU_MFMA_BUSY_CYCLES":
            e["busy"] += float(r["Counter_Value"])
        elif r["Counter_Name"] == "SQ_INSTS_VALU_MFMA_MOPS_BF16":
            e["mops"] += float(r["Counter_Value"])
    out = ["kernel: dispatches, executed bf16 MFMA GFLOP per step, avg duration, MFMA-pipe busy cycles per SIMD and launch, "
           "busy fraction of the duration at 2.4 GHz"]
    tot_flop = tot_busy = tot_ns = 0.0
    for key, e in sorted(per.items()):
        n = len(e["ids"])
        busy_per_simd = e["busy"] / SIMDS / n
        frac = busy_per_simd / (e["ns"] / n * 1e-9 * CLOCK_HZ)
        out.append(f"  {key}: {n}, {e['mops'] * 512 / steps / 1e9:.1f} GFLOP, {e['ns'] / n / 1e3:.1f} us, "
                   f"{busy_per_simd:.0f} cycles, {frac:.3f}")
        if any(g in key for g in GEMM_KERNELS):
            tot_flop += e["mops"] * 512
            tot_busy += e["busy"] / SIMDS
            tot_ns += e["ns"]
    out.append(f"GEMM kernels, all variants: {tot_flop / steps / 1e9:.1f} GFLOP executed per step, "
               f"busy fraction {tot_busy / (tot_ns * 1e-9 * CLOCK_HZ):.3f}")
    sys.stdout.write("\n".join(out) + "\n")


def short_name(name):
    name = name.replace("void ", "").replace("mslt::", "")
    return re.sub(r"\(.*", "", name)


def rowwise_main(fetch_csv, write_csv, last_steps):
    """Per non-GEMM kernel over the last `last_steps` steps: launches per step, HBM-side bytes per launch, average
    duration, GB/s.  A step starts at its k_batch_scan dispatch."""
    per = {}
    out = [f"kernel_source_sha256: {rowwise_source_hash()}"]
    for label, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        rows = list(csv.DictReader(open(path)))
        copy_kib = max((float(r["Counter_Value"]) for r in rows if "copyBuffer" in r["Kernel_Name"]), default=0.0)
        factor = COPY_BYTES / (copy_kib * 1024.0)
        out.append(f"{label}: 256 MiB copy reads {copy_kib:.0f} KiB -> scale factor {factor:.4f}")
        scans = sorted(int(r["Start_Timestamp"]) for r in rows if "k_batch_scan" in r["Kernel_Name"])
        t0 = scans[-last_steps]
        for r in rows:
            name = r["Kernel_Name"]
            if int(r["Start_Timestamp"]) < t0 or any(g in name for g in GEMM_KERNELS) or "copyBuffer" in name:
                continue
            e = per.setdefault(short_name(name), {"FETCH_SIZE": [0, 0.0, 0], "WRITE_SIZE": [0, 0.0, 0]})[label]
            e[0] += 1
            e[1] += float(r["Counter_Value"]) * 1024.0 * factor
            e[2] += int(r["End_Timestamp"]) - int(r["Start_Timestamp"])
    out.append(f"last_steps: {last_steps}")
    out.append("# kernel <name>: launches per step, fetched MB per launch, written MB per launch, avg duration us, GB/s (HBM side)")
    for key, e in sorted(per.items(), key=lambda kv: -(kv[1]["FETCH_SIZE"][2])):
        nf, bf, tf = e["FETCH_SIZE"]
        nw, bw, tw = e["WRITE_SIZE"]
        if not nf or not nw:
            continue
        dur_us = (tf / nf + tw / nw) / 2e3
        mb_f, mb_w = bf / nf / 1e6, bw / nw / 1e6
        out.append(f"kernel {key}: {nf / last_steps:.1f} launches/step, fetch {mb_f:.2f} MB, write {mb_w:.2f} MB, "
                   f"{dur_us:.1f} us, {(mb_f + mb_w) / dur_us * 1e3:.0f} GB/s")
    sys.stdout.write("\n".join(out) + "\n")


def main():
    if sys.argv[1] == "--mfma":
        return mfma_main(sys.argv[2], int(sys.argv[3]))
    if sys.argv[1] == "--rowwise":
        return rowwise_main(sys.argv[2], sys.argv[3], int(sys.argv[4]))
    fetch_csv, write_csv, steps = sys.argv[1], sys.argv[2], int(sys.argv[3])
    out = [f"kernel_source_sha256: {kernel_source_hash()}"]
    total = 0.0
    launches = 0
    for label, path in (("FETCH_SIZE", fetch_csv), ("WRITE_SIZE", write_csv)):
        copy_kib, gemm = read_counter(path)
        factor = COPY_BYTES / (copy_kib * 1024.0)
        out.append(f"{label}: 256 MiB copy reads {copy_kib:.0f} KiB -> scale factor {factor:.4f}")
        n_all = 0
        for name, (n, s) in sorted(gemm.items()):
            out.append(f"  {name}: {n} dispatches, {s:.0f} KiB raw, {s * 1024 * factor / steps / 1e9:.4f} GB per step")
            total += s * 1024 * factor
            n_all += n
        launches = n_all
    per_step = total / steps
    out.append(f"steps_in_run: {steps}")
    out.append(f"gemm_launches_per_step: {launches / steps:.1f}")
    out.append(f"traffic_bytes_per_step: {per_step:.0f}")
    out.append(f"traffic_bytes_per_launch: {per_step / (launches / steps):.0f}")
    sys.stdout.write("\n".join(out) + "\n")


if __name__ == "__main__":
    main()
