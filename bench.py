#!/usr/bin/env python3
"""Benchmark of the SpecKV hot path on one MI355X.

A step is one `speckv_compress` call over the whole synthetic workload (all layers):
scoring pass 1, row-statistics merge, scoring pass 2, pooling, selection, compaction.
Inputs are generated on the GPU and resident in HBM before the timed region.  Prints ONE
JSON line: whole-job throughput in prompt keys scored + compacted per second
(n_in x layers x kv_heads / time), a roofline object for the dominant kernel (timed live
with HIP events recorded on the launch stream inside the timed steps) and the CPU oracle
timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c3|c2|c4]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E


def _hip_runtime() -> ctypes.CDLL:
    """The HIP runtime already mapped into this process (the one torch and libspeckv use)."""
    path = None
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64.so" in line:
                path = line.split()[-1]
                break
    if path is None:
        raise RuntimeError("HIP runtime is not loaded")
    hip = ctypes.CDLL(path)
    hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    hip.hipEventCreate.restype = ctypes.c_int
    hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    hip.hipEventElapsedTime.restype = ctypes.c_int
    hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
    hip.hipEventDestroy.restype = ctypes.c_int
    return hip


def _traffic_from_profile(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if any."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic_%s.txt" % workload)
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\s*%s\s+hbm_bytes_per_launch=([0-9.eE+]+)" % re.escape(kernel), line)
        if m:
            return float(m.group(1))
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--lse-variant", action="store_true",
                    help="also time the single-sweep variant with caller-supplied row normalisers")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (known HBM traffic) so that a rocprofv3 "
                         "--pmc run of this command can scale its FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; sharding over several GPUs is a design note "
              "only (sequence / layer / KV-head sharding needs no exchange). Use --gpus 1.",
              file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2

    import paper_2506_08373_amd as S
    S.load_library()
    torch.cuda.set_device(0)
    w = workloads.PRESETS[args.workload]()
    t0 = time.time()
    data = workloads.generate(w, device="cuda")
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    q, k, v = data["q"], data["k"], data["v"]

    p = S.SpecKVParams.for_tensors(q, k, seq_lens=w.seq_lens, n_window=w.n_window, pool_k=w.pool_k,
                                   c_max=w.c_max, sm_scale=w.sm_scale)
    KT = S.total_keep(p)
    L, H, d = w.n_layers, w.n_kv_heads, w.head_dim
    idx = torch.empty((L, H * KT), dtype=torch.int32, device="cuda")
    k_out = torch.empty((L, H * KT, d), dtype=w.torch_dtype, device="cuda")
    v_out = torch.empty_like(k_out)
    ws = torch.empty(S.workspace_bytes(p), dtype=torch.uint8, device="cuda")

    hip = _hip_runtime()
    NE = S.N_STAGE_EVENTS
    ev_sets = []
    for _ in range(args.steps):
        arr = (ctypes.c_void_p * NE)()
        for i in range(NE):
            h = ctypes.c_void_p()
            if hip.hipEventCreate(ctypes.byref(h)) != 0:
                raise RuntimeError("hipEventCreate failed")
            arr[i] = h
        ev_sets.append(arr)

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        S.speckv_compress(p, q, k, v, idx, k_out, v_out, ws)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in range(args.steps):
        S.speckv_compress_events(p, q, k, v, idx, k_out, v_out, ws, ev_sets[step])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    stage_ms = np.zeros((args.steps, NE - 1))
    for step, arr in enumerate(ev_sets):
        for i in range(NE - 1):
            ms = ctypes.c_float()
            if hip.hipEventElapsedTime(ctypes.byref(ms), arr[i], arr[i + 1]) != 0:
                raise RuntimeError("hipEventElapsedTime failed")
            stage_ms[step, i] = ms.value
    for arr in ev_sets:
        for i in range(NE):
            hip.hipEventDestroy(arr[i])
    mean_ms = stage_ms.mean(axis=0)

    # algorithmic work per launch
    qk_flops = 2.0 * w.n_rows * w.n_q_heads * w.total_tokens * d * L        # one Q.K^T over the workload
    elt = 2 if w.dtype == "bf16" else 4
    compact_bytes = 2.0 * 2.0 * H * KT * d * elt * L + 4.0 * H * KT * L      # K,V read + write, indices
    kernels = {}
    for name, ms in zip(S.STAGE_NAMES, mean_ms):
        entry = {"ms": round(float(ms), 4)}
        if name in ("score_pass1", "score_pass2"):
            entry.update(bound="mfma", achieved=round(qk_flops / (ms * 1e-3) / 1e12, 2),
                         peak=PEAK_BF16_TFLOPS, unit="TFLOP/s")
        elif name == "compact":
            entry.update(bound="hbm", achieved=round(compact_bytes / (ms * 1e-3) / 1e9, 1),
                         peak=PEAK_HBM_GBS, unit="GB/s")
        if "achieved" in entry:
            entry["frac"] = round(entry["achieved"] / entry["peak"], 4)
        kernels[name] = entry
    dominant = max(("score_pass1", "score_pass2"), key=lambda n: kernels[n]["ms"])
    roofline = {"kernel": dominant, "bound": "mfma", "achieved": kernels[dominant]["achieved"],
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": kernels[dominant]["frac"],
                "traffic": _traffic_from_profile(dominant, args.workload),
                "avg_launch_ms": kernels[dominant]["ms"]}
    k_read_gbs = (w.total_tokens * H * d * elt * L) / (kernels[dominant]["ms"] * 1e-3) / 1e9

    ms_per_step = elapsed / args.steps * 1e3
    value = w.key_units / (elapsed / args.steps)

    # Context figure (not the headline): the same step when the caller already holds the row
    # log-sum-exps (e.g. from the prefill attention kernel) and scoring needs one sweep only.
    lse_variant = None
    if args.lse_variant:
        lse_in = torch.empty((L, w.n_seqs, w.n_rows, w.n_q_heads), dtype=torch.float32, device="cuda")
        cu = w.cu_seqlens
        for layer in range(L):
            for s_ in range(w.n_seqs):
                kk = k[layer, cu[s_]:cu[s_ + 1]].float()                       # [n, Hkv, d]
                qq = q[layer, s_].float().view(w.n_rows, H, w.group, d)        # [R, Hkv, G, d]
                logits = torch.einsum("rhgd,nhd->rhgn", qq, kk) * w.sm_scale   # causal mask ignored: timing only
                lse_in[layer, s_] = torch.logsumexp(logits, dim=-1).reshape(w.n_rows, w.n_q_heads)
                del logits, kk, qq
        for _ in range(args.warmup):
            S.speckv_compress_lse(p, q, k, v, lse_in, idx, k_out, v_out, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            S.speckv_compress_lse(p, q, k, v, lse_in, idx, k_out, v_out, ws)
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        lse_variant = {"ms_per_step": round(el / args.steps * 1e3, 4),
                       "value": round(w.key_units / (el / args.steps), 1), "unit": "keys/s",
                       "note": "speckv_compress_lse: row normalisers supplied by the caller, one sweep over K"}
        del lse_in
        # restore the headline outputs for the parity check below
        S.speckv_compress(p, q, k, v, idx, k_out, v_out, ws)
        torch.cuda.synchronize()

    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import speckv_oracle as orc          # CPU baseline leg only
        try:
            from threadpoolctl import threadpool_info
            blas_threads = max([x.get("num_threads", 1) for x in threadpool_info()] or [1])
        except Exception:
            blas_threads = 1
        cores = len(os.sched_getaffinity(0))
        s = 0
        cu = w.cu_seqlens
        n0 = w.seq_lens[s]
        keep0 = w.n_keep(s)
        # bounded sample: about 10 s of oracle time (one 128K layer of the 8B shape takes ~2.5 s)
        n_sample = max(1, min(L, int(round(4 * (131072 * 8) / (n0 * H)))))
        layers = sorted(set(int(round(x)) for x in np.linspace(0, L - 1, n_sample)))
        cpu_s, rows_equal = 0.0, 0
        for layer in layers:
            qh = workloads.to_float64(q[layer, s])
            kh = workloads.to_float64(k[layer, cu[s]:cu[s + 1]])
            vh = workloads.to_float64(v[layer, cu[s]:cu[s + 1]])
            t0 = time.perf_counter()
            ref = orc.speckv_layer(qh, kh, vh, w.n_window, w.pool_k, w.c_max, w.sm_scale)
            cpu_s += time.perf_counter() - t0
            got = idx[layer, : H * keep0].reshape(H, keep0).cpu().numpy()
            rows_equal += int(sum(np.array_equal(got[g], ref["idx"][g]) for g in range(H)))
        cpu_baseline = {"value": round(len(layers) * n0 * H / cpu_s, 1), "unit": "keys/s",
                        "cores": min(cores, blas_threads), "kind": "oracle", "seconds": round(cpu_s, 2),
                        "host_cores_visible": cores,
                        "sample": "layers %s, sequence %d of %s (all %d KV heads, n_in=%d): %d/%d of a step"
                                  % (layers, s, w.name, H, n0, len(layers) * n0 * H, w.key_units)}
        parity = {"sample": "layers %s seq %d" % (layers, s), "index_rows_equal_to_oracle": rows_equal,
                  "index_rows": H * len(layers)}

    out = {
        "metric": "prompt keys scored+compacted/sec (n_in x layers x kv_heads)",
        "value": round(value, 1), "unit": "keys/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n_layers": L, "n_q_heads": w.n_q_heads, "n_kv_heads": H,
                   "head_dim": d, "n_in": list(w.seq_lens), "n_window": w.n_window,
                   "n_lookahead": w.n_lookahead, "pool_k": w.pool_k, "c_max": w.c_max,
                   "parallelism": "single GPU"},
        "roofline": roofline,
        "kernels": kernels,
        "k_read_GBps_in_dominant_kernel": round(k_read_gbs, 1),
        "single_sweep_variant": lse_variant,
        "cpu_baseline": cpu_baseline,
        "parity_check": parity,
        "input_generation_s": round(gen_s, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
