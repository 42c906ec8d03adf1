#!/usr/bin/env python3
"""Benchmark of the EL-attention decode step on one MI355X.

A "step" is one pass of the whole hot path (query projection and expansion, the
attention core over H, value and output projections) over one batch of synthetic
input already resident in HBM.  The step rotates over several H buffers whose
total size exceeds the 256 MB memory-side cache, so every step streams its H from
HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME]
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
ROTATE_BYTES = 768e6           # >= 3x the 256 MB memory-side cache

ARITH = {
    "bf16": "bf16 MFMA in the attention core (EL-Q and P as high+low bf16 pairs), fp16 MFMA in the projections, fp32 accumulation and softmax",
    "f16": "fp16 MFMA (EL-Q as a high+low fp16 pair), fp32 accumulation and softmax",
    "f32": "fp32 vector FMA",
}


def kernel_source_digest() -> str:
    """sha256 over the library's kernel sources (names and contents, sorted): says which kernels a stored counter
    figure was taken on, without needing the repository's history on the machine that runs the benchmark."""
    import glob
    import hashlib
    h = hashlib.sha256()
    for path in sorted(glob.glob(os.path.join(ROOT, "paper_2105_04779_amd", "csrc", "*"))):
        h.update(os.path.basename(path).encode() + b"\0")
        with open(path, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="c3_bart_large_bf16")
    ap.add_argument("--splits", type=int, default=0, help="key-range splits (0 = automatic)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle baseline (0 = skip)")
    ap.add_argument("--same-h", action="store_true", help="reuse one H buffer every step (cache-warm; not the reported protocol)")
    ap.add_argument("--layers", type=int, default=1, help="attention layers (own weights each) that read the same H in one step")
    ap.add_argument("--check", action="store_true",
                    help="time the diagnostic input check (one read of the valid rows of H) instead of the decode step")
    ap.add_argument("--gather", action="store_true",
                    help="state maintenance instead of the decode step: re-order 512 per-beam histories of up to 1024 rows "
                         "(GPT-2-medium widths) by parent beam; one line with the bytes moved per second")
    ap.add_argument("--sweep", choices=["n", "beam"], default=None,
                    help="one line per point: input length 64..1024 at beam 4, or beam 1..8 at length 1024 (BART-large widths, B 64)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="only run a plain device copy of known size (1 GiB read + 1 GiB written per launch, 10 launches): "
                         "what FETCH_SIZE / WRITE_SIZE read for it scales the counters of the real run")
    return ap.parse_args()


def cpu_baseline(w, wl, seconds):
    """The fp64 oracle, as it stands, timed on this host on the first batch elements of the workload."""
    import numpy as np
    import oracle
    W = wl.weights(w)
    args = lambda H, Q, L: (H, L, Q, W["Wq"], W["bq"], W["Wk"], W["bk"], W["Wv"], W["bv"], W["Wo"], W["bo"])
    threads = oracle.num_threads()
    probe = min(w.B, max(1, threads))
    H, Q, L = wl.batch(w, elements=range(probe))
    t0 = time.perf_counter()
    oracle.mha_reference(*args(H, Q, L), heads=w.heads, d_k=w.d_k)
    t_probe = time.perf_counter() - t0
    total = min(w.B, max(probe, int(probe * seconds / max(t_probe, 1e-3)) // probe * probe))
    if total > probe:
        H, Q, L = wl.batch(w, elements=range(total))
        t0 = time.perf_counter()
        oracle.mha_reference(*args(H, Q, L), heads=w.heads, d_k=w.d_k)
        dt = time.perf_counter() - t0
    else:
        total, dt = probe, t_probe
    # a workload the oracle finishes in a second or two is repeated until the sample is worth ~`seconds` of CPU work
    reps = 1
    if dt < seconds / 2:
        reps = min(50, max(1, int(seconds / max(dt, 1e-3))))
        t0 = time.perf_counter()
        for _ in range(reps):
            oracle.mha_reference(*args(H, Q, L), heads=w.heads, d_k=w.d_k)
        dt = (time.perf_counter() - t0) / reps
    return {
        "value": total * w.beam / dt, "unit": "queries/s", "cores": threads, "kind": "oracle",
        "sample": f"first {total} of {w.B} batch elements of {w.name} (their real lengths, sum {int(L.sum())}), "
                  f"fp64 multi-head attention without cache, {reps} pass(es) of {dt:.2f} s",
    }


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path shards over batch elements with no "
              "exchange between GPUs); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2105_04779_amd import el_attn, traffic_model as tm, workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if a.pmc_calibration:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")   # 1 GiB
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "device copy", "bytes_read_per_launch": src.numel() * 4,
                          "bytes_written_per_launch": src.numel() * 4, "launches": 10}))
        return
    if a.check:
        print(json.dumps(measure_check(a, torch, np, el_attn, wl)), flush=True)
        return
    if a.gather:
        print(json.dumps(measure_gather(a, torch, np, el_attn, wl)), flush=True)
        return
    # ---- extra modes (rows after the contract's: sweeps of input length and beam size, several layers
    #      reading one H); each prints one line per point, without the CPU baseline ----
    if a.sweep:
        base = wl.WORKLOADS["c3_bart_large_bf16"]
        if a.sweep == "n":        # beam 4, every input of length n (section 4.1.2's first sweep)
            points = [wl.custom(f"sweep_n{n}", dtype=base.dtype, B=base.B, beam=4, heads=base.heads, d_m=base.d_m,
                                d_k=base.d_k, n=n, index=200 + k) for k, n in enumerate((64, 128, 256, 512, 1024))]
        else:                     # n = 1024, beam 1..8 (its second sweep)
            points = [wl.custom(f"sweep_beam{x}", dtype=base.dtype, B=base.B, beam=x, heads=base.heads, d_m=base.d_m,
                                d_k=base.d_k, n=1024, index=210 + k) for k, x in enumerate((1, 2, 4, 6, 8))]
        for w in points:
            print(json.dumps(measure(a, w, torch, np, el_attn, tm, wl)), flush=True)
        return
    w = wl.WORKLOADS[a.workload]
    line = measure(a, w, torch, np, el_attn, tm, wl)
    if a.cpu_seconds > 0 and a.layers == 1:
        line["cpu_baseline"] = cpu_baseline(w, wl, a.cpu_seconds)
    print(json.dumps(line), flush=True)


def measure_gather(a, torch, np, el_attn, wl):
    """Beam re-order of per-beam histories (section 3.1.1's state for self-attention): every new beam copies the
    valid rows of its parent's H.  Bytes moved = valid rows read once + written once; bound: HBM."""
    w = wl.WORKLOADS["c5_gpt2_medium_n1024_bf16"]
    B, n, d_m = w.B, w.n, w.d_m
    g = torch.Generator(device="cuda").manual_seed(wl.BASE_SEED + 300)
    src = torch.randn((B, n, d_m), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    dst = torch.empty_like(src)
    rng = np.random.default_rng(wl.BASE_SEED + 301)
    lens = rng.integers(n // 2, n, size=B, endpoint=True).astype(np.int32)
    index = (np.arange(B) // 4 * 4 + rng.integers(0, 4, size=B)).astype(np.int32)   # a parent among the 4 beams of the same sentence
    Ld, Idx = torch.from_numpy(lens).cuda(), torch.from_numpy(index).cuda()
    out_lens = torch.empty((B,), dtype=torch.int32, device="cuda")
    for _ in range(a.warmup):
        el_attn.gather_batch(src, Ld, Idx, H_dst=dst, lengths_dst=out_lens)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(a.steps):
        el_attn.gather_batch(src, Ld, Idx, H_dst=dst, lengths_dst=out_lens)
    e1.record()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / a.steps
    moved = 2 * int(lens[index].sum()) * d_m * 2
    gbs = moved / (ms * 1e-3) / 1e9
    return {"metric": "state gather, bytes read + written per second", "value": gbs, "unit": "GB/s", "n_gpus": 1,
            "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "u8", "data": "synthetic",
            "config": {"workload": "beam re-order of per-beam histories, GPT-2-medium widths", "B": B, "n": n, "d_m": d_m,
                       "sum_len": int(lens[index].sum()), "event_ms_per_step": e0.elapsed_time(e1) / a.steps},
            "roofline": {"bound": "hbm", "kernel": "k_gather_batch", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": gbs / HBM_PEAK_GBS, "traffic": None, "bytes_per_launch": moved, "avg_launch_us": ms * 1e3}}


def measure_check(a, torch, np, el_attn, wl):
    """The diagnostic input check on the per-beam histories of the self-attention workload: every valid row of H is
    read once and classified.  Bound: HBM."""
    w = wl.WORKLOADS["c5_gpt2_medium_n1024_bf16"]
    B, n, d_m = w.B, w.n, w.d_m
    g = torch.Generator(device="cuda").manual_seed(wl.BASE_SEED + 310)
    H = torch.randn((B, n, d_m), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    lens = np.random.default_rng(wl.BASE_SEED + 311).integers(n // 2, n, size=B, endpoint=True).astype(np.int32)
    Ld = torch.from_numpy(lens).cuda()
    report = torch.empty(4, dtype=torch.int64, device="cuda")
    for _ in range(a.warmup):
        el_attn.check_inputs(H, Ld, report=report)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        el_attn.check_inputs(H, Ld, report=report)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / a.steps
    read = int(lens.sum()) * d_m * 2
    assert report.cpu().tolist() == [0, 0, 0, int(lens.sum()) * d_m]
    gbs = read / (ms * 1e-3) / 1e9
    return {"metric": "input check, bytes read per second", "value": gbs, "unit": "GB/s", "n_gpus": 1,
            "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "u16", "data": "synthetic",
            "config": {"workload": "input check of per-beam histories, GPT-2-medium widths", "B": B, "n": n, "d_m": d_m,
                       "sum_len": int(lens.sum())},
            "roofline": {"bound": "hbm", "kernel": "k_check_inputs", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": gbs / HBM_PEAK_GBS, "traffic": None, "bytes_per_launch": read, "avg_launch_us": ms * 1e3}}


def measure(a, w, torch, np, el_attn, tm, wl):
    """One bench line for workload `w`: whole-step throughput, then the core kernel timed by itself."""
    from dataclasses import replace
    td = {"f16": torch.float16, "bf16": torch.bfloat16, "f32": torch.float32}[w.dtype]

    # ---- inputs, resident in HBM before anything is timed -----------------------------------
    device_weights = el_attn.device_weights
    # `--layers L`: L attention layers with their own weights read the same H in every step (what the L
    # decoder layers of one model do with one encoder output); layer 0 has the workload's own weights
    layers = []
    for k in range(a.layers):
        W = wl.weights(w if k == 0 else replace(w, index=w.index + 1000 * k))
        layers.append(el_attn.ElAttention(device_weights(W, w.dtype), heads=w.heads, d_k=w.d_k, dtype=w.dtype,
                                          max_batch=w.B, max_beam=w.beam, max_n=w.n))
    layer = layers[0]
    if a.splits:
        for ly in layers:
            ly.set_splits(a.splits)
    lens = wl.lengths(w)
    Ld = torch.from_numpy(lens).cuda()
    h_bytes = w.B * w.n * w.d_m * w.elem_bytes
    nbuf = 1 if a.same_h else max(2, int(np.ceil(ROTATE_BYTES / h_bytes)))
    g = torch.Generator(device="cuda").manual_seed(wl.BASE_SEED + w.index)
    Hs = [torch.randn((w.B, w.n, w.d_m), generator=g, device="cuda", dtype=torch.float32).to(td) for _ in range(nbuf)]
    Q = torch.randn((w.B, w.beam, w.d_m), generator=g, device="cuda", dtype=torch.float32).to(td)
    out = torch.empty((w.B, w.beam, w.d_m), device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()

    def run(steps, start=0):
        for i in range(steps):
            H = Hs[(start + i) % nbuf]
            for ly in layers:
                ly.decode_step(H, Ld, Q, out=out)

    # ---- whole-step throughput -------------------------------------------------------------
    run(a.warmup)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    run(a.steps, a.warmup)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = wall_ms / a.steps
    ev_ms_per_step = e0.elapsed_time(e1) / a.steps
    assert torch.isfinite(out).all()

    # ---- the dominant kernel (attention core) timed by itself, HIP events on its own stream ----
    # (with several layers: the last layer's, i.e. the one that finds H already touched in this step)
    core_steps = min(a.steps, 1000)
    timed = layers[-1]
    timed.core_timing(core_steps)
    run(core_steps, a.warmup + a.steps)
    torch.cuda.synchronize()
    core_ms = timed.read_core_timing(core_steps)
    timed.core_timing(0)
    core_avg_ms = float(np.mean(core_ms))

    sum_len = int(lens.sum())
    core_bytes = tm.core_algorithmic_bytes(sum_len, w.d_m, w.elem_bytes)
    step_bytes = tm.step_algorithmic_bytes(sum_len, w.B, w.beam, w.d_m, w.heads * w.d_k, w.elem_bytes, 4)
    achieved = core_bytes / (core_avg_ms * 1e-3) / 1e9
    # HBM bytes per launch of that kernel from the committed rocprofv3 counter runs (FETCH_SIZE + WRITE_SIZE,
    # each scaled by what the same counter reads for a plain copy of known size).  The counters cannot be read
    # inside this run, so the stored figure carries the digest of the kernel sources it was taken on: it is
    # reported only while those sources are unchanged, and is null otherwise (or if none is committed).
    traffic, traffic_detail = None, None
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{w.name}.json")
    if os.path.exists(tpath) and a.layers == 1:
        with open(tpath) as f:
            traffic_detail = json.load(f)
        if traffic_detail.get("kernel_source_sha256") == kernel_source_digest():
            traffic = traffic_detail["fetch_bytes"] + traffic_detail["write_bytes"]
        else:
            traffic_detail = {"stale": True, "reason": "the kernel sources changed since the committed counter run",
                              "counters_taken_on": traffic_detail.get("kernel_source_sha256")}

    L = a.layers
    line = {
        "metric": "decode-step queries/sec (B x beam)" + ("" if L == 1 else f", {L} layers on one H, a query counted once per layer"),
        "value": w.B * w.beam * L / (ms_per_step * 1e-3),
        "unit": "queries/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "arith": ARITH[w.dtype] if layer.uses_mfma else ARITH["f32"], "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "beam": w.beam, "heads": w.heads, "d_m": w.d_m, "d_k": w.d_k,
                   "n": w.n, "sum_len": sum_len, "h_buffers_rotated": nbuf, "mfma_path": layer.uses_mfma,
                   "splits": a.splits, "layers": L},
        "roofline": {"bound": "hbm", "kernel": "attention core (a3-a5)", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_detail": traffic_detail,
                     "bytes_per_launch": core_bytes, "avg_launch_us": core_avg_ms * 1e3,
                     "min_launch_us": float(np.min(core_ms)) * 1e3},
        "step": {"algorithmic_bytes": step_bytes, "event_ms_per_step": ev_ms_per_step, "ms_per_layer": ms_per_step / L,
                 "hbm_frac_whole_step": step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
                 "flops": L * tm.step_flops(sum_len, w.B, w.beam, w.heads, w.d_m, w.d_k),
                 "tflops": L * tm.step_flops(sum_len, w.B, w.beam, w.heads, w.d_m, w.d_k) / (ms_per_step * 1e-3) / 1e12},
    }
    for ly in layers:
        ly.close()
    return line


if __name__ == "__main__":
    main()
