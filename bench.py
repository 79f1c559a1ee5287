#!/usr/bin/env python3
"""Benchmark of one MSLT stage step (stage_step + apply_update) on one MI355X.

Headline workload: the final stage of the BERT-Large schedule (Section 4.1): 24 encoder layers, the
bottom 18 frozen (forward only), the top 6 and the masked-LM head trainable, batch 64 x sequence 128,
bf16 compute with fp32 master weights, LAMB.  Inputs are seeded and synthetic (Zipf token ids, 15 %
masking, N(0, 0.02) weights); they are resident in HBM before the timed region starts.

Prints ONE JSON line.  `value` is tokens/s of the whole step.  `roofline` covers the dominant
kernels, the bf16 MFMA GEMMs: algorithmic FLOPs of all their launches in a step divided by their
summed duration, measured with HIP events on the library's stream in a second pass over the same
steps directly after the timed region (event recording would disturb the step timing itself).
`cpu_baseline` times the float64 numpy oracle on the host cores on a bounded sample of the same
workload.  Further keys of the same line (unless --no-compare): the same kernels with every layer
trainable, BERT-Base stage 2 and final stage, and the BERT-Large schedule sweep at 32 x 512 with the
stack grown between stages.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2516.6   # 256 CU x 2.4 GHz x 4096 FLOP/clk/CU, dense
PEAK_HBM_GBS = 8000.0


def run_steps(model, cbatches, f, k, emb, opt, n, stamps=None, dropout=0.0):
    loss = None
    for i in range(n):
        if dropout > 0.0:
            model.mslt_set_dropout(dropout, 20201127, i)    # a new step number: new masks
        # one call = stage step + optimizer update (the same work as mslt_stage_step + mslt_apply_update);
        # it returns once the loss is on the host, i.e. after the step's kernels (the update may still run)
        loss = model.mslt_train_step(f, k, emb, cbatches[i % len(cbatches)], opt)
        if stamps is not None:
            stamps.append(time.perf_counter())
    return loss


def time_steps(torch, model, cbatches, f, k, emb, opt, steps, warmup, dropout=0.0):
    run_steps(model, cbatches, f, k, emb, opt, warmup, dropout=dropout)
    model.mslt_sync()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    stamps = [t0]
    loss = run_steps(model, cbatches, f, k, emb, opt, steps, stamps, dropout=dropout)
    if dropout > 0.0:
        model.mslt_set_dropout(0.0, 0, 0)
    model.mslt_sync()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    time_steps.per_step_ms = sorted((b - a) * 1e3 for a, b in zip(stamps, stamps[1:]))
    return dt / steps, loss


def profile_steps(model, cbatches, f, k, emb, opt, steps):
    model.mslt_profile_enable(True)
    run_steps(model, cbatches, f, k, emb, opt, steps)
    prof = model.mslt_profile_read()
    model.mslt_profile_enable(False)
    for v in prof.values():
        for key in ("launches", "ms", "flops", "bytes"):
            v[key] = v[key] / steps
    return prof


def clocks_under_load(model, cbatches, f, k, emb, opt):
    """Clock and power state while the step runs: rocm-smi is queried from a second thread during a burst of about a
    second and a half of steps (the library calls release the interpreter lock).  None if the tool is not there."""
    import re
    import shutil
    import subprocess
    import threading
    if shutil.which("rocm-smi") is None:
        return None
    got = {}

    def query():
        time.sleep(0.4)
        try:
            got["text"] = subprocess.run(["rocm-smi", "--showclocks", "--showperflevel", "--showpower", "--showmaxpower"],
                                         capture_output=True, text=True, timeout=20).stdout
        except (OSError, subprocess.SubprocessError):
            pass

    th = threading.Thread(target=query)
    th.start()
    t_end = time.perf_counter() + 1.5
    while time.perf_counter() < t_end or th.is_alive():
        run_steps(model, cbatches, f, k, emb, opt, 10)
    th.join()
    model.mslt_sync()
    text = got.get("text")
    if not text:
        return None

    def find(pattern, cast=float):
        m = re.search(pattern, text)
        return cast(m.group(1)) if m else None

    return {"sclk_mhz": find(r"sclk clock level: \d+: \((\d+)Mhz\)"), "mclk_mhz": find(r"mclk clock level: \d+: \((\d+)Mhz\)"),
            "perf_level": find(r"Performance Level: (\w+)", str), "power_w": find(r"(?:Average|Current Socket) Graphics Package Power \(W\): ([\d.]+)"),
            "power_cap_w": find(r"Max Graphics Package Power \(W\): ([\d.]+)"),
            "sampled": "rocm-smi, once, while the benchmark step was running back to back"}


PMC_TRAFFIC_FILE = os.path.join(ROOT, "profiles", "gemm_kernels_large_18f6t_64x128_pmc_traffic.txt")
PMC_ROWWISE_FILE = os.path.join(ROOT, "profiles", "non_gemm_kernels_large_18f6t_64x128_pmc_traffic.txt")


def _summary_fields(path):
    return dict(line.split(":", 1) for line in open(path) if ":" in line and not line.startswith((" ", "#")))


def recorded_gemm_traffic():
    """HBM-side bytes per GEMM launch from the committed rocprofv3 --pmc summary, or None if the kernel
    source has changed since those counters were taken (or no summary exists)."""
    from paper_2011_13635_amd.pmc_summary import kernel_source_hash
    try:
        fields = _summary_fields(PMC_TRAFFIC_FILE)
        if fields["kernel_source_sha256"].strip() != kernel_source_hash():
            return None
        return float(fields["traffic_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


def recorded_rowwise_traffic():
    """Counter-measured HBM-side GB/s of the non-GEMM kernels (committed rocprofv3 --pmc summary), or None when
    their source has changed since (or no summary exists)."""
    from paper_2011_13635_amd.pmc_summary import rowwise_source_hash
    try:
        fields = _summary_fields(PMC_ROWWISE_FILE)
        if fields["kernel_source_sha256"].strip() != rowwise_source_hash():
            return None
        return {key[len("kernel "):]: v.strip() for key, v in fields.items() if key.startswith("kernel ")}
    except (OSError, KeyError, ValueError):
        return None


def gemm_roofline(prof):
    gemm = [v for n, v in prof.items() if n.startswith("gemm_mfma")]
    flops, ms = sum(v["flops"] for v in gemm), sum(v["ms"] for v in gemm)
    tf = flops / (ms * 1e-3) / 1e12 if ms > 0 else 0.0
    return {"achieved_TFLOPs": round(tf, 1), "frac_of_peak": round(tf / PEAK_BF16_TFLOPS, 4), "gemm_ms": round(ms, 4)}


def extra_workloads(torch, binding, synth, steps):
    """The other configurations of the stage step (parity-test cases, timed here for the record): each MSLT step
    next to the same kernels with every layer and the embeddings trainable."""
    res = {}
    cases = [
        # the paper's own training settings (Section 4.1): both objectives of BERT and its dropout of 0.1
        ("base_final_64x128_nsp_dropout", synth.ModelShape(n_layers=12, hidden=768, n_heads=12, ffn=3072, vocab=30522,
                                                           nsp=True), 64, 128, [(9, 3, False)], binding.adam(lr=1e-4), 0.1),
        ("base_final_16x512", synth.bert_base_shape(12), 16, 512, [(9, 3, False)], binding.adam(lr=1e-4)),
        # grouped variant (Section 3.3): 12 layers in 4 groups of 3 that share their parameters
        ("base_grouped_4x3_final_64x128", synth.ModelShape(n_layers=12, hidden=768, n_heads=12, ffn=3072, vocab=30522,
                                                           layers_per_group=3), 64, 128, [(9, 3, False)], binding.adam(lr=1e-4)),
    ]
    for name, shape, B, S, stages, opt, *rest in cases:
        dropout = rest[0] if rest else 0.0
        W = synth.make_weights(shape, seed=0)
        batches = [synth.make_batch(shape, B, S, seed=1 + i) for i in range(2)]
        n_pred = max(len(b["masked_positions"]) for b in batches)
        m = binding.Model(binding.make_config(shape, B, S, 1, max_predictions=n_pred + 64))
        m.mslt_load_params(synth.pack_weights(shape, W))
        del W
        cb = [m.device_batch(b) for b in batches]
        tokens = B * S
        entry = {"tokens_per_step": tokens, "stages": []}
        for f, k, emb in stages:
            sec, loss = time_steps(torch, m, cb, f, k, emb, opt, steps, 2, dropout=dropout)
            prof = profile_steps(m, cb, f, k, emb, opt, min(steps, 4))
            entry["stages"].append({"frozen": f, "trainable": k, "train_embeddings": emb, "ms_per_step": round(sec * 1e3, 4),
                                    "tokens_per_s": round(tokens / sec, 1), **gemm_roofline(prof)})
        sec_full, _ = time_steps(torch, m, cb, 0, shape.n_layers, True, opt, steps, 2, dropout=dropout)
        entry["full_step_ms"] = round(sec_full * 1e3, 4)
        entry["full_tokens_per_s"] = round(tokens / sec_full, 1)
        entry["speedup_last_stage_vs_full"] = round(sec_full / (entry["stages"][-1]["ms_per_step"] * 1e-3), 3)
        if len(stages) > 1:   # schedule: equal step counts per stage against the same number of full steps
            total = sum(st["ms_per_step"] for st in entry["stages"])
            entry["schedule_time_ratio_full_over_mslt"] = round(len(stages) * sec_full * 1e3 / total, 3)
        res[name] = entry
        m.close()
        del m
        torch.cuda.empty_cache()
    return res


def build_model(binding, synth, shape, B, S, batches, opt_pred_extra=64):
    n_pred = max(len(b["masked_positions"]) for b in batches)
    W = synth.make_weights(shape, seed=0)
    model = binding.Model(binding.make_config(shape, B, S, 1, max_predictions=n_pred + opt_pred_extra))
    model.mslt_load_params(synth.pack_weights(shape, W))
    return model, W, [model.device_batch(b) for b in batches]


def class_table(prof):
    classes = {}
    for n, v in sorted(prof.items(), key=lambda kv: -kv[1]["ms"]):
        e = {"ms": round(v["ms"], 4), "launches": round(v["launches"], 1)}
        if v["flops"] > 0 and n.startswith(("gemm", "attention")):
            e["TFLOP/s"] = round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 1)
        if v["bytes"] > 0:
            e["GB/s"] = round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1)
        classes[n] = e
    return classes


def large_schedule_sweep(torch, binding, synth, steps):
    """Section 3.2's schedule at BERT-Large width, batch 32 x seq 512: stages of 6 layers (the first one trains
    everything it has, embeddings included), the stack grown by copying its top 6 layers between stages, `steps`
    training steps per stage, then the same number of steps with all 24 layers and the embeddings trainable."""
    shape, B, S = synth.bert_large_shape(24), 32, 512
    batches = [synth.make_batch(shape, B, S, seed=1 + i) for i in range(2)]
    m, W, cb = build_model(binding, synth, shape, B, S, batches)
    del W
    opt = binding.lamb()
    tokens = B * S
    res = {"workload": "BERT-Large, batch 32 x seq 512, LAMB, stages of 6 layers with growth between them",
           "steps_per_stage": steps, "stages": []}
    present = 6
    for stage in range(4):
        f, k, emb = present - 6, 6, stage == 0
        sec, loss = time_steps(torch, m, cb, f, k, emb, opt, steps, 2)
        res["stages"].append({"layers_present": present, "frozen": f, "trainable": k, "train_embeddings": emb,
                              "ms_per_step": round(sec * 1e3, 4), "tokens_per_s": round(tokens / sec, 1)})
        if present < shape.n_layers:
            m.mslt_grow(present, 6)
            present += 6
    sec_full, _ = time_steps(torch, m, cb, 0, shape.n_layers, True, opt, steps, 2)
    res["full_step_ms"] = round(sec_full * 1e3, 4)
    res["full_tokens_per_s"] = round(tokens / sec_full, 1)
    total = sum(st["ms_per_step"] for st in res["stages"])
    res["schedule_time_ratio_full_over_mslt"] = round(len(res["stages"]) * sec_full * 1e3 / total, 3)
    m.close()
    del m
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-compare", action="store_true",
                    help="only the headline workload: skip the full-step comparison, BERT-Base and the schedule sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-clocks", action="store_true",
                    help="skip the burst of steps during which rocm-smi is queried (keeps a profiler run short)")
    ap.add_argument("--all-configs", action="store_true",
                    help="also time the remaining configurations (both objectives with dropout, grouped variant, "
                         "BERT-Base at 16x512; several minutes)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 256 MiB device copy (reference dispatch for scaling FETCH_SIZE/WRITE_SIZE "
                         "counters when this script runs under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch
    from paper_2011_13635_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        return 2

    # headline: final stage of the BERT-Large schedule (Section 4.1: 24 layers, stages of 6, LAMB)
    B, S = 64, 128
    f, k = 18, 6
    shape = synth.bert_large_shape(24)
    batches = [synth.make_batch(shape, B, S, seed=1 + i) for i in range(4)]
    n_pred = max(len(b["masked_positions"]) for b in batches)
    model, W, cb = build_model(binding, synth, shape, B, S, batches)
    opt = binding.lamb()

    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0")   # 256 MiB read + 256 MiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        # the counters are read per launch: keep every step of this run in the form the per-launch timing below
        # uses (one stream, one launch per product) so that the launches of the two runs correspond
        model.mslt_profile_enable(True)

    sec, loss = time_steps(torch, model, cb, f, k, False, opt, args.steps, args.warmup)
    if args.copy_calibration:
        model.mslt_profile_read()
    tokens = B * S
    ps = time_steps.per_step_ms     # host time between consecutive step returns
    step_quantiles = [round(ps[len(ps) // 2], 4), round(ps[len(ps) // 10], 4), round(ps[(len(ps) * 9) // 10], 4)]
    prof = profile_steps(model, cb, f, k, False, opt, min(args.steps, 10))

    gemm = [v for n, v in prof.items() if n.startswith("gemm_mfma")]
    g_flops = sum(v["flops"] for v in gemm)
    g_ms = sum(v["ms"] for v in gemm)
    g_launch = sum(v["launches"] for v in gemm)
    achieved = g_flops / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0

    out = {
        "metric": "MSLT stage-step tokens/sec at BERT-Base/Large; MFMA util % vs bf16 peak",
        "value": round(tokens / sec, 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec * 1e3, 4),
        "ms_per_step_median_p10_p90": step_quantiles,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "BERT-Large MSLT final stage: 24 layers, bottom 18 frozen, top 6 + MLM head trainable, "
                               "batch 64 x seq 128, LAMB (lr 0.00088), bf16 with fp32 master", "frozen_layers": f,
                   "trainable_layers": k, "batch": B, "seq_len": S, "tokens_per_step": tokens,
                   "predicted_per_step": int(len(batches[0]["masked_positions"])), "loss": round(float(loss), 5)},
        "roofline": {"bound": "mfma", "kernel": "bf16 MFMA GEMM (k_gemm_ring for forward-type and weight-gradient "
                     "products, k_gemm_mfma for data-gradient products)", "achieved": round(achieved, 1),
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                     "traffic": recorded_gemm_traffic(), "traffic_unit": "bytes per launch (L2-miss side, FETCH_SIZE + "
                     "WRITE_SIZE scaled by a 256 MiB copy)", "algorithmic_bytes_per_launch":
                     round(sum(v["bytes"] for v in gemm) / max(g_launch, 1)), "launches_per_step": round(g_launch, 1),
                     "avg_launch_us": round(g_ms * 1e3 / max(g_launch, 1), 2),
                     "gemm_ms_per_step": round(g_ms, 4), "gemm_gflop_per_step": round(g_flops / 1e9, 1),
                     "timed_with": "HIP events around every launch on the library's stream, every launch alone on the "
                     "GPU (second pass over the same steps right after the timed region); the interval also holds "
                     "the fixed-order split-k summing kernel of a product and the dispatch latency of the launch"},
        "clocks": None if (args.no_clocks or args.copy_calibration) else clocks_under_load(model, cb, f, k, False, opt),
        "kernel_classes": class_table(prof),
        "profiled_ms_per_step": round(sum(v["ms"] for v in prof.values()), 4),
        "non_gemm_counter_evidence": recorded_rowwise_traffic(),
    }

    if not args.no_compare:
        # the same kernels with all 24 layers and the embeddings trainable (the retraining step of Section 3.2)
        n_cmp = max(5, min(args.steps, 10))
        sec_full, _ = time_steps(torch, model, cb, 0, shape.n_layers, True, opt, n_cmp, 2)
        out["final_stage_vs_full"] = {"workload": "BERT-Large 24 layers, batch 64 x seq 128, LAMB",
                                      "mslt_18_frozen_6_trainable_ms": round(sec * 1e3, 4),
                                      "full_24_trainable_ms": round(sec_full * 1e3, 4),
                                      "full_tokens_per_s": round(tokens / sec_full, 1),
                                      "speedup": round(sec_full / sec, 3)}
    model.close()
    del model
    torch.cuda.empty_cache()

    if not args.no_compare:
        # BERT-Base: stage 2 (6 layers present, 3 frozen / 3 trainable) and the final stage against the full step
        sb6 = synth.bert_base_shape(6)
        bb = [synth.make_batch(sb6, B, S, seed=1 + i) for i in range(4)]
        adam = binding.adam(lr=1e-4)
        m6, W6, cb6 = build_model(binding, synth, sb6, B, S, bb)
        del W6
        n_cmp = max(5, min(args.steps, 20))
        s6, l6 = time_steps(torch, m6, cb6, 3, 3, False, adam, n_cmp, 3)
        p6 = profile_steps(m6, cb6, 3, 3, False, adam, min(n_cmp, 10))
        out["base_stage2"] = {"workload": "BERT-Base 6 layers present, bottom 3 frozen, top 3 trainable, batch 64 x seq "
                                          "128, Adam", "ms_per_step": round(s6 * 1e3, 4),
                              "tokens_per_s": round(tokens / s6, 1), "loss": round(float(l6), 5), **gemm_roofline(p6),
                              "kernel_classes": class_table(p6)}
        m6.close()
        del m6
        sb12 = synth.bert_base_shape(12)
        m12, W12, cb12 = build_model(binding, synth, sb12, B, S, bb)
        del W12
        sec_stage, _ = time_steps(torch, m12, cb12, 9, 3, False, adam, n_cmp, 3)
        p12 = profile_steps(m12, cb12, 9, 3, False, adam, min(n_cmp, 10))
        sec_full12, _ = time_steps(torch, m12, cb12, 0, 12, True, adam, n_cmp, 3)
        sec_drop, _ = time_steps(torch, m12, cb12, 9, 3, False, adam, n_cmp, 3, dropout=0.1)
        out["base_final_stage_vs_full"] = {"workload": "BERT-Base 12 layers, batch 64 x seq 128, Adam",
                                           "mslt_9_frozen_3_trainable_ms": round(sec_stage * 1e3, 4),
                                           "full_12_trainable_ms": round(sec_full12 * 1e3, 4),
                                           "mslt_tokens_per_s": round(tokens / sec_stage, 1),
                                           "full_tokens_per_s": round(tokens / sec_full12, 1),
                                           "speedup": round(sec_full12 / sec_stage, 3),
                                           "mslt_with_dropout_0.1_ms": round(sec_drop * 1e3, 4), **gemm_roofline(p12)}
        m12.close()
        del m12
        torch.cuda.empty_cache()
        out["large_schedule_sweep_32x512"] = large_schedule_sweep(torch, binding, synth, 8)

    if not args.no_cpu_baseline:
        # the oracle on a bounded sample of the headline workload: the first 16 of the 64 sequences of one batch
        # (a quarter of a step: the whole step takes it over a minute)
        from oracle import mslt_oracle as O
        threads = len(os.sched_getaffinity(0))
        try:
            from threadpoolctl import threadpool_info
            blas = [p["num_threads"] for p in threadpool_info() if p.get("user_api") == "blas"]
            if blas:
                threads = max(blas)
        except Exception:
            pass
        nb = 16
        sub = {key: (np.asarray(v)[:nb] if isinstance(v, np.ndarray) and v.ndim >= 1 and len(v) == B else v)
               for key, v in batches[0].items()}
        t0 = time.perf_counter()
        ref_loss, ref_g, _ = O.stage_step(shape, W, sub, f, k, False, full_backprop=False)
        st = O.new_opt_state(O.to_f64({n: W[n] for n in ref_g}))
        O.optimizer_update({n: W[n] for n in ref_g}, ref_g, st, kind="lamb", lr=0.00088)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(nb * S / dt, 1), "unit": "tokens/s", "cores": threads, "kind": "oracle",
                               "sample": f"one stage step + LAMB update of the headline workload on the first {nb} of the "
                                         f"{B} sequences of a batch ({nb * S} tokens; the backward stops at the lowest "
                                         "trainable layer as the method does), float64 numpy",
                               "seconds": round(dt, 2), "oracle_loss": round(float(ref_loss), 5)}
    if args.all_configs:
        out["other_configs"] = extra_workloads(torch, binding, synth, max(4, min(args.steps, 8)))
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
