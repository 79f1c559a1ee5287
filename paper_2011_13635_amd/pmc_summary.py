"""Summarises two rocprofv3 --pmc runs of bench.py (FETCH_SIZE, WRITE_SIZE; csv output) into the HBM-side traffic of
the MFMA GEMM kernel per launch, scaled by what the same counters read for the plain 256 MiB device copy that
`bench.py --copy-calibration` issues.  Also records the hash of the kernel source so that bench.py can tell
whether the figure still belongs to the kernel it times.

usage: python -m paper_2011_13635_amd.pmc_summary <fetch_counter_collection.csv> <write_counter_collection.csv> <steps_in_run>
       python -m paper_2011_13635_amd.pmc_summary --mfma <counter_collection.csv> <steps_in_run>
The second form summarises a run with SQ_VALU_MFMA_BUSY_CYCLES and SQ_INSTS_VALU_MFMA_MOPS_BF16: the FLOPs the
matrix cores executed (512 per counted operation) and the fraction of the kernels' duration their pipes were busy.
"""
from __future__ import annotations

import csv
import hashlib
import os
import re
import sys

CSRC = os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc")
KERNEL_SOURCES = [os.path.join(CSRC, "gemm_mfma.hip"), os.path.join(CSRC, "common.h")]   # kernel + its epilogue helpers
COPY_BYTES = 256 * 1024 * 1024


def kernel_source_hash() -> str:
    """Hash of the kernel's code: comments and blank space do not count."""
    h = hashlib.sha256()
    for path in KERNEL_SOURCES:
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
        elif "k_gemm_mfma" in name:
            n, s = gemm.get(name, (0, 0.0))
            gemm[name] = (n + 1, s + v)
    return copy_kib, gemm


SIMDS = 256 * 4            # compute units x SIMDs
CLOCK_HZ = 2.4e9           # the clock the published peak is quoted at


def mfma_main(path, steps):
    per = {}
    for r in csv.DictReader(open(path)):
        name = r["Kernel_Name"]
        if "mfma" not in name and "attn" not in name:
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
        if "k_gemm_mfma" in key:
            tot_flop += e["mops"] * 512
            tot_busy += e["busy"] / SIMDS
            tot_ns += e["ns"]
    out.append(f"k_gemm_mfma, all variants: {tot_flop / steps / 1e9:.1f} GFLOP executed per step, "
               f"busy fraction {tot_busy / (tot_ns * 1e-9 * CLOCK_HZ):.3f}")
    sys.stdout.write("\n".join(out) + "\n")


def main():
    if sys.argv[1] == "--mfma":
        return mfma_main(sys.argv[2], int(sys.argv[3]))
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
