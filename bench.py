#!/usr/bin/env python3
"""Benchmark of the SpecKV hot path on one MI355X.

A step is one pass of the whole hot path over the synthetic workload: for the SpecKV
workloads (c1-c4) one `speckv_compress` call over all layers (scoring pass 1, row-statistics
merge, scoring pass 2, pooling, selection, compaction); for the prompt-token workload (c5) one
`specpc_select_tokens` call (the two scoring sweeps over all layers, the cross-layer reduction
and pooling, top-k selection, neighbour expansion and id gather).  Inputs are generated on the
GPU and resident in HBM before the timed region.  Prints ONE JSON line: whole-job throughput in
prompt keys scored + compacted per second (n_in x layers x kv_heads / time), a roofline object
for the dominant kernel (timed live with HIP events recorded on the launch stream inside the
timed steps), the single-sweep variant (row normalisers supplied by the caller) and the CPU
oracle timed on a bounded sample of the same workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload c1|c2|c3|c4|c5]
                    [--layers L] [--reduce sum|max]
"""
from __future__ import annotations

import argparse
import ctypes
import dataclasses
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

# MI355X published peaks
PEAK_MFMA_TFLOPS = {"bf16": 2500.0, "f16": 2500.0, "f32": 157.3}
PEAK_HBM_GBS = 8000.0
# Plain fp32 vector arithmetic without packed operations (this build disables them):
# 256 CUs x 64 lanes x 2.4 GHz x 2 flops per fused multiply-add.
PEAK_ALU_TFLOPS = 256 * 64 * 2.4e9 * 2 / 1e12
# vector work per score element and sweep: one fused multiply-add, one exp2, one add
ALU_FLOPS_PER_SCORE = 4.0


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


def _traffic_from_profile(stage: str, tag: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if any."""
    path = os.path.join(ROOT, "profiles", "pmc_traffic_%s.txt" % tag)
    if not os.path.exists(path):
        return None, None
    for line in open(path):
        m = re.match(r"\s*%s\s+hbm_bytes_per_launch=([0-9.eE+]+)" % re.escape(stage), line)
        if m:
            return float(m.group(1)), "profiles/pmc_traffic_%s.txt" % tag
    return None, None


def _scoring_kernel_symbol(S, p, w, stage: str) -> str:
    """Name of the unmasked scoring kernel of this stage as a rocprofv3 kernel trace shows it."""
    info = S.plan_info(p)
    dt = {"bf16": 0, "f32": 1, "f16": 2}[w.dtype]
    npass = 1 if stage == "score_pass1" else 2
    red = info["reduce_max"] if npass == 2 else info["fixed_reference_rows"]
    if info["q_stationary"] & npass:
        return "score_qs_kernel<%d, %d, %d, %d>" % (dt, w.head_dim, npass, red)
    fn = "score_kernel_rows" if (npass == 1 and info["waves"] == 8) else "score_kernel_cols"
    return "%s<%d, %d, %d, %d, %d, %d, false>" % (fn, dt, w.head_dim, info["blocks_per_wave"], info["waves"],
                                                  npass, red)


def _make_events(hip, n_sets: int, ne: int):
    sets = []
    for _ in range(n_sets):
        arr = (ctypes.c_void_p * ne)()
        for i in range(ne):
            h = ctypes.c_void_p()
            if hip.hipEventCreate(ctypes.byref(h)) != 0:
                raise RuntimeError("hipEventCreate failed")
            arr[i] = h
        sets.append(arr)
    return sets


def _stage_means(hip, ev_sets, ne: int) -> np.ndarray:
    ms_all = np.zeros((len(ev_sets), ne - 1))
    for step, arr in enumerate(ev_sets):
        for i in range(ne - 1):
            ms = ctypes.c_float()
            if hip.hipEventElapsedTime(ctypes.byref(ms), arr[i], arr[i + 1]) != 0:
                raise RuntimeError("hipEventElapsedTime failed")
            ms_all[step, i] = ms.value
    for arr in ev_sets:
        for i in range(ne):
            hip.hipEventDestroy(arr[i])
    return ms_all.mean(axis=0)


def _blas_threads() -> int:
    try:
        from threadpoolctl import threadpool_info
        return max([x.get("num_threads", 1) for x in threadpool_info()] or [1])
    except Exception:
        return 1


def _ceilings(S) -> dict:
    """Register-resident loops with the sweeps' instruction mix, timed with torch events on the
    current stream (the probe launches there), and one library GEMM for scale."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(7)
    operands = {"random": torch.randn(1 << 16, generator=gen, device="cuda").to(torch.bfloat16),
                "zeros": torch.zeros(1 << 16, dtype=torch.bfloat16, device="cuda")}
    out = torch.empty(256 * 512, dtype=torch.float32, device="cuda")
    names = {0: "mfma_only", 1: "mfma_softmax", 2: "mfma_softmax_lds512"}
    iters = 40000
    res = {}
    for data, ops in operands.items():
        for kind, name in names.items():
            S.probe_ceiling(kind, 2000, ops, out)                    # warm-up
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            flops = S.probe_ceiling(kind, iters, ops, out)
            e1.record()
            torch.cuda.synchronize()
            res["%s_%s_TFLOPs" % (name, data)] = round(flops / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    a = torch.randn(8192, 8192, generator=gen, device="cuda").to(torch.bfloat16)
    b = torch.randn(8192, 8192, generator=gen, device="cuda").to(torch.bfloat16)
    for _ in range(3):
        torch.matmul(a, b)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(20):
        torch.matmul(a, b)
    e1.record()
    torch.cuda.synchronize()
    res["library_gemm_8192_bf16_random_TFLOPs"] = round(20 * 2.0 * 8192 ** 3 / (e0.elapsed_time(e1) * 1e-3) / 1e12, 1)
    return {"ceilings": res, "peak_bf16_TFLOPs": PEAK_MFMA_TFLOPS["bf16"],
            "note": "256 workgroups x 512 threads, 8 MFMA 32x32x16 bf16 per tile; softmax = 16 x (fma, exp2, add) "
                    "per lane and tile; lds512 = B operands re-read from LDS every second tile"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--layers", type=int, default=0, help="override the workload's number of layers")
    ap.add_argument("--reduce", default="sum", choices=["sum", "max"],
                    help="reduction over the observation rows of a head (max: the listing's MaxReduce)")
    ap.add_argument("--paper-setting", action="store_true",
                    help="the hyper-parameter table's SpecKV column: max reduction, max pooling k = 7, "
                         "n_window = 32 (the lookahead rows grow to keep 128 rows), budget C_max - n_window")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-lse-variant", action="store_true",
                    help="skip the single-sweep figure (row normalisers supplied by the caller)")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of a workload, measure what this GPU sustains for the scoring sweeps' "
                         "instruction mix held in registers (MFMA alone, with softmax arithmetic, with LDS "
                         "operand reads; random and zero operands) plus a library bf16 GEMM, and print them")
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
    if args.ceilings:
        print(json.dumps(_ceilings(S)))
        return 0
    w = workloads.PRESETS[args.workload]()
    if args.layers > 0:
        w = dataclasses.replace(w, n_layers=args.layers, name="%s_%dlayers" % (w.name, args.layers))
    reduce = args.reduce
    if args.paper_setting:
        if args.workload == "c5":
            print("bench.py: --paper-setting applies to the SpecKV workloads c1-c4", file=sys.stderr)
            return 2
        rows = w.n_rows
        w = dataclasses.replace(w, n_window=32, n_lookahead=rows - 32, c_max=max(w.c_max - 32, 0),
                                name=w.name + "_paper_setting")
        reduce = "max"
    specpc = args.workload == "c5"
    tag = args.workload if (args.layers <= 0 and reduce == "sum" and not args.paper_setting) else None

    t0 = time.time()
    data = workloads.generate(w, device="cuda")
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    q, k, v = data["q"], data["k"], data["v"]
    L, H, d, G = w.n_layers, w.n_kv_heads, w.head_dim, w.group
    elt = 4 if w.dtype == "f32" else 2

    p = S.SpecKVParams.for_tensors(q, k, seq_lens=w.seq_lens, n_window=w.n_window, pool_k=w.pool_k,
                                   c_max=w.c_max, sm_scale=w.sm_scale, reduce=reduce)
    hip = _hip_runtime()
    NE = S.N_STAGE_EVENTS
    ev_sets = _make_events(hip, args.steps, NE)

    if specpc:
        top_k, nb = w.c_max, workloads.SPECPC_NEIGHBORS
        n = w.seq_lens[0]
        ids = workloads.generate_token_ids(w, device="cuda")
        idx_out = torch.empty(n, dtype=torch.int32, device="cuda")
        ids_out = torch.empty(n, dtype=torch.int32, device="cuda")
        count = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = torch.empty(S.specpc_workspace_bytes(p, top_k), dtype=torch.uint8, device="cuda")
        stage_names = S.SPECPC_STAGE_NAMES

        def plain_call():
            S.specpc_select_tokens(p, top_k, nb, q, k, ids, idx_out, ids_out, count, ws)

        def timed_call(ev):
            S.specpc_select_tokens_events(p, top_k, nb, q, k, ids, idx_out, ids_out, count, ws, ev)
    else:
        KT = S.total_keep(p)
        idx = torch.empty((L, H * KT), dtype=torch.int32, device="cuda")
        k_out = torch.empty((L, H * KT, d), dtype=w.torch_dtype, device="cuda")
        v_out = torch.empty_like(k_out)
        ws = torch.empty(max(S.workspace_bytes(p), 256), dtype=torch.uint8, device="cuda")
        stage_names = S.STAGE_NAMES

        def plain_call():
            S.speckv_compress(p, q, k, v, idx, k_out, v_out, ws)

        def timed_call(ev):
            S.speckv_compress_events(p, q, k, v, idx, k_out, v_out, ws, ev)

    if args.calibration_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        plain_call()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for step in range(args.steps):
        timed_call(ev_sets[step])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    mean_ms = _stage_means(hip, ev_sets, NE)
    # Context figure: the same K steps without the stage events (seven event records between dependent
    # kernels cost about 25 us per step: nothing on the 32-layer workload, a fifth of the tiny ones).
    t0 = time.perf_counter()
    for step in range(args.steps):
        plain_call()
    torch.cuda.synchronize()
    plain_elapsed = time.perf_counter() - t0

    # algorithmic work per launch
    n_scores = float(w.n_rows) * w.n_q_heads * w.total_tokens * L          # score elements of one sweep
    qk_flops = 2.0 * n_scores * d                                          # one Q.K^T over the workload
    k_bytes = float(w.total_tokens) * H * d * elt * L                      # K read once
    peak_mfma = PEAK_MFMA_TFLOPS[w.dtype]
    kernels = {}
    for name, ms in zip(stage_names, mean_ms):
        entry = {"ms": round(float(ms), 4)}
        if name in ("score_pass1", "score_pass2"):
            entry.update(bound="mfma", achieved=round(qk_flops / (ms * 1e-3) / 1e12, 2), peak=peak_mfma,
                         unit="TFLOP/s", kernel=_scoring_kernel_symbol(S, p, w, name),
                         k_read_GBps=round(k_bytes / (ms * 1e-3) / 1e9, 1),
                         alu_TFLOPs=round(ALU_FLOPS_PER_SCORE * n_scores / (ms * 1e-3) / 1e12, 2))
        elif name == "compact":
            KT = S.total_keep(p)
            compact_bytes = 2.0 * 2.0 * H * KT * d * elt * L + 4.0 * H * KT * L   # K,V read + write, indices
            entry.update(bound="hbm", achieved=round(compact_bytes / (ms * 1e-3) / 1e9, 1), peak=PEAK_HBM_GBS,
                         unit="GB/s", kernel="compact_kernel<true>")
        if "achieved" in entry:
            entry["frac"] = round(entry["achieved"] / entry["peak"], 4)
        kernels[name] = entry
    dominant = max(("score_pass1", "score_pass2"), key=lambda n_: kernels[n_]["ms"])
    dk = kernels[dominant]
    traffic, traffic_src = (None, None) if tag is None else _traffic_from_profile(dominant, tag)
    if d == 64 and elt == 2:
        # at d = 64 a 32x32 score block costs half the matrix time of d = 128 but the same softmax
        # arithmetic: these sweeps are bound by the vector pipe, priced in plain (unpacked) fp32
        roofline = {"kernel": dk["kernel"], "stage": dominant, "bound": "alu", "achieved": dk["alu_TFLOPs"],
                    "peak": round(PEAK_ALU_TFLOPS, 1), "unit": "TFLOP/s",
                    "frac": round(dk["alu_TFLOPs"] / PEAK_ALU_TFLOPS, 4),
                    "peak_derivation": "256 CUs x 64 lanes x 2.4 GHz x 2 flops, no packed fp32; 4 flops per "
                                       "score element and sweep (fma, exp2, add)",
                    "mfma_frac": dk["frac"], "hbm_frac_k_read": round(dk["k_read_GBps"] / PEAK_HBM_GBS, 4)}
    else:
        roofline = {"kernel": dk["kernel"], "stage": dominant, "bound": "mfma", "achieved": dk["achieved"],
                    "peak": peak_mfma, "unit": "TFLOP/s", "frac": dk["frac"]}
    roofline.update(traffic=traffic, traffic_source=traffic_src, avg_launch_ms=dk["ms"])
    if dominant == "score_pass1" and S.plan_info(p)["fixed_reference_rows"]:
        roofline["avg_launch_note"] = ("the stage between two HIP events: the sweep and the repair launch behind it "
                                       "(score_kernel_rows_repair, 1 % of the stage)")

    ms_per_step = elapsed / args.steps * 1e3
    value = w.key_units / (elapsed / args.steps)
    # the same algorithmic flops (one Q.K^T; the two sweeps execute it twice) over the whole step
    step_tflops = qk_flops / (ms_per_step * 1e-3) / 1e12
    roofline["whole_step"] = {"achieved": round(step_tflops, 2), "unit": "TFLOP/s", "frac": round(step_tflops / peak_mfma, 4),
                              "note": "algorithmic flops of one Q.K^T over the step time; each sweep executes them once"}

    # Context figure (not the headline): the same step when the caller already holds the row
    # log-sum-exps (e.g. from the prefill attention kernel) and scoring needs one sweep only.
    lse_variant = None
    if not args.no_lse_variant and not specpc:
        lse_in = torch.empty((L, w.n_seqs, w.n_rows, w.n_q_heads), dtype=torch.float32, device="cuda")
        cu = w.cu_seqlens
        for layer in range(L):
            for s_ in range(w.n_seqs):
                kk = k[layer, cu[s_]:cu[s_ + 1]].float()                       # [n, Hkv, d]
                qq = q[layer, s_].float().view(w.n_rows, H, G, d)              # [R, Hkv, G, d]
                for g in range(H):                                             # causal mask ignored: timing only
                    logits = torch.einsum("rgd,nd->rgn", qq[:, g], kk[:, g]) * w.sm_scale
                    lse_in[layer, s_, :, g * G:(g + 1) * G] = torch.logsumexp(logits, dim=-1)
                    del logits
                del kk, qq
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
        plain_call()                        # restore the headline outputs for the parity check below
        torch.cuda.synchronize()

    cpu_baseline = None
    parity = None
    if not args.no_cpu_baseline:
        from oracle import speckv_oracle as orc          # CPU baseline leg only
        cores = len(os.sched_getaffinity(0))
        threads = min(cores, _blas_threads())
        cu = w.cu_seqlens
        if specpc:
            n = w.seq_lens[0]
            qh, kh = workloads.to_float64(q[:, 0]), workloads.to_float64(k)
            ids_h = ids.cpu().numpy()
            t0 = time.perf_counter()
            ref = orc.specpc_select_tokens(qh, kh, ids_h, w.n_window, w.pool_k, top_k, nb, w.sm_scale)
            cpu_s = time.perf_counter() - t0
            c = int(count.item())
            got = idx_out[:c].cpu().numpy().astype(np.int64)
            cpu_baseline = {"value": round(w.key_units / cpu_s, 1), "unit": "keys/s", "cores": threads,
                            "kind": "oracle", "seconds": round(cpu_s, 2), "host_cores_visible": cores,
                            "sample": "the whole call: all %d layers of %s" % (L, w.name)}
            parity = {"sample": "whole call", "count": c, "count_oracle": int(ref["count"]),
                      "indices_equal_to_oracle": bool(np.array_equal(got, ref["idx"])),
                      "indices_in_common": int(np.isin(got, ref["idx"]).sum())}
        else:
            s = 0
            n0, keep0 = w.seq_lens[s], w.n_keep(s)
            # bounded sample: about 10 s of oracle time = four 128K layers of the 8B shape; the oracle's
            # cost per layer grows with n_in x query heads x rows x head_dim
            ref_cost = 131072.0 * 32 * 128 * 128
            n_sample = max(1, min(L, int(round(4 * ref_cost / (float(n0) * w.n_q_heads * w.n_rows * d)))))
            layers = sorted(set(int(round(x)) for x in np.linspace(0, L - 1, n_sample)))
            cpu_s, rows_equal = 0.0, 0
            for layer in layers:
                qh = workloads.to_float64(q[layer, s])
                kh = workloads.to_float64(k[layer, cu[s]:cu[s + 1]])
                vh = workloads.to_float64(v[layer, cu[s]:cu[s + 1]])
                t0 = time.perf_counter()
                ref = orc.speckv_layer(qh, kh, vh, w.n_window, w.pool_k, w.c_max, w.sm_scale, reduce=reduce)
                cpu_s += time.perf_counter() - t0
                got = idx[layer, : H * keep0].reshape(H, keep0).cpu().numpy()
                rows_equal += int(sum(np.array_equal(got[g], ref["idx"][g]) for g in range(H)))
            cpu_baseline = {"value": round(len(layers) * n0 * H / cpu_s, 1), "unit": "keys/s",
                            "cores": threads, "kind": "oracle", "seconds": round(cpu_s, 2),
                            "host_cores_visible": cores,
                            "sample": "layers %s, sequence %d of %s (all %d KV heads, n_in=%d): %d/%d of a step"
                                      % (layers, s, w.name, H, n0, len(layers) * n0 * H, w.key_units)}
            parity = {"sample": "layers %s seq %d" % (layers, s), "index_rows_equal_to_oracle": rows_equal,
                      "index_rows": H * len(layers)}

    config = {"workload": w.name, "call": "specpc_select_tokens" if specpc else "speckv_compress",
              "n_layers": L, "n_q_heads": w.n_q_heads, "n_kv_heads": H, "head_dim": d,
              "n_in": list(w.seq_lens), "n_window": w.n_window, "n_lookahead": w.n_lookahead,
              "pool_k": w.pool_k, "c_max": w.c_max, "reduce": reduce, "parallelism": "single GPU"}
    if specpc:
        config.update(top_k=w.c_max, n_neighbor=workloads.SPECPC_NEIGHBORS)
    out = {
        "metric": "prompt keys scored+compacted/sec (n_in x layers x kv_heads)",
        "value": round(value, 1), "unit": "keys/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": config,
        "roofline": roofline,
        "kernels": kernels,
        "without_stage_events": {"ms_per_step": round(plain_elapsed / args.steps * 1e3, 4),
                                 "value": round(w.key_units / (plain_elapsed / args.steps), 1), "unit": "keys/s"},
        "single_sweep_variant": lse_variant,
        "cpu_baseline": cpu_baseline,
        "parity_check": parity,
        "input_generation_s": round(gen_s, 1),
    }
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
