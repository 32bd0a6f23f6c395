#!/usr/bin/env python3
"""Benchmark of the fused-prefill hot path on one MI355X.

A step = one cb_fuse_prefill call: re-alignment of the cached keys of every layer,
then all L layers of selective recompute, on a synthetic request of the workload's
shape (weights, inputs and the pre-computed chunk caches are resident in HBM before
the timed region; the caches are restored from a pristine copy between steps, outside
the timed region, because the path fuses them in place).

Prints ONE JSON line: the whole-call throughput in recomputed token-layers per second
(sum over layers of the rows that went through attention + MLP, divided by the call
time = TTFT), the roofline position of the dominant kernel class (the MFMA GEMMs)
measured with HIP events inside the library, and the CPU oracle timed on a bounded
slice of the same workload."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"mfma_bf16_tflops": 2500.0, "hbm_gbs": 8000.0}

# Bytes moved between L2 and the memory fabric per GEMM launch (average over the GEMM launches of
# one step), from two rocprofv3 --pmc runs of this script (FETCH_SIZE, then WRITE_SIZE), each scaled
# by what the same counter reads for kernels of known size in the same run (FETCH_SIZE x 1.999,
# WRITE_SIZE x 1.000); summary under profiles/.  Keyed by (workload, schedule, layers, ratio):
# any other run reports null.
PMC_TRAFFIC_BYTES_PER_GEMM_LAUNCH = {("mistral7b", "gradual", 32, 0.15): 216.7e6}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="mistral7b")
    ap.add_argument("--layers", type=int, default=0, help="reduce depth (0 = the workload's own)")
    ap.add_argument("--ratio", type=float, default=None)
    ap.add_argument("--flat", action="store_true", help="flat schedule instead of gradual filtering")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--batch", type=int, default=1,
                    help="requests fused per call (cb_fuse_prefill_batched when > 1; distinct inputs per request)")
    ap.add_argument("--no-host-load", action="store_true",
                    help="skip the variant that loads the chunk caches from pinned host memory")
    ap.add_argument("--no-graph", action="store_true",
                    help="skip the variant that replays the call from a HIP graph")
    return ap.parse_args()


def attention_flops(model, sel_sets, n_ctx, n_suffix):
    """4 * Hq * dh * sum over processed rows of (position + 1), per layer."""
    import numpy as np
    suffix = np.arange(n_ctx, n_ctx + n_suffix, dtype=np.float64)
    total = 0.0
    for sel in sel_sets:
        pos = np.concatenate([sel.astype(np.float64), suffix])
        total += 4.0 * model.n_q_heads * model.head_dim * float(np.sum(pos + 1.0))
    return total


def cpu_baseline(w, keep):
    """The oracle as it stands on layers 0-1 of the workload (a full layer, then the first
    selective layer with its check), real widths, synthetic inputs from the same generator."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info
    from oracle import cacheblend_oracle as O
    from workloads import synth
    from dataclasses import replace

    m2 = replace(w.model, n_layers=2)
    rnd = O.storage_round(w.model.dtype)
    layers = [{k: synth.to_f64(v) for k, v in synth.layer_weights(m2, l, w.seed_weights).items()}
              for l in range(2)]
    x = synth.to_f64(synth.hidden_inputs(w))
    dt = synth.storage_dtype(w.model)
    kpre = [synth.to_f64(synth.random_rows(w.n_ctx, m2.kv_dim, 0.5, 77 + l, dtype=dt)).reshape(
        w.n_ctx, m2.n_kv_heads, m2.head_dim) for l in range(2)]
    vpre = [synth.to_f64(synth.random_rows(w.n_ctx, m2.kv_dim, 0.5, 87 + l, dtype=dt)).reshape(
        w.n_ctx, m2.n_kv_heads, m2.head_dim) for l in range(2)]
    keep2 = [keep[0], keep[1] if len(keep) > 1 else keep[0]]
    t0 = time.perf_counter()
    out = O.fuse_prefill(x, layers, m2, w.chunk_lens, w.n_suffix, kpre, vpre, keep2, kv_round=rnd)
    dt_s = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    rows = sum(out.rows)
    return {"value": rows / dt_s, "unit": "token-layers/s", "cores": int(threads), "kind": "oracle",
            "sample": f"layers 0-1 of the workload at real width (full layer on {out.rows[0]} rows, then "
                      f"K/V check on {out.rows[0]} rows and recompute of {out.rows[1]} rows), numpy float64, "
                      f"{dt_s:.1f} s"}


def bench_batched(a, w, keep, P, producer, synth, torch, np):
    """B requests of the workload's shape (own inputs each) fused by one cb_fuse_prefill_batched call."""
    from dataclasses import replace
    m, B = w.model, a.batch
    dev = torch.device("cuda:0")
    L, C, S, T = m.n_layers, w.n_ctx, w.n_suffix, w.n_tokens
    layers = [synth.layer_weights(m, l, w.seed_weights, device=dev) for l in range(L)]
    ctx = P.cb_create(m, T)
    xs, k_pre, v_pre = [], [[] for _ in range(L)], [[] for _ in range(L)]
    for b in range(B):
        xb = synth.hidden_inputs(replace(w, seed_inputs=w.seed_inputs + 101 * b), device=dev)
        kb, vb = producer.chunk_prefill(ctx, layers, xb[:C], w.chunk_lens, T)
        xs.append(xb)
        for l in range(L):
            k_pre[l].append(kb[l])
            v_pre[l].append(vb[l])
    x = torch.cat(xs).contiguous()
    k_pre = [torch.cat(t).contiguous() for t in k_pre]          # [B * T, Hkv, dh], slabs T rows apart
    v_pre = [torch.cat(t).contiguous() for t in v_pre]
    torch.cuda.synchronize()
    k_work = [t.clone() for t in k_pre]
    v_work = [t.clone() for t in v_pre]

    def restore():
        for dst, src in zip(k_work + v_work, k_pre + v_pre):
            dst.copy_(src)

    out = None

    def step():
        nonlocal out
        out = P.cb_fuse_prefill_batched(ctx, layers, x, [w.chunk_lens] * B, [S] * B, k_work, v_work, T, [keep] * B,
                                        workspace=None if out is None else out.workspace,
                                        weight_structs=None if out is None else out.weight_structs, out=out)

    for _ in range(max(1, a.warmup)):
        restore()
        step()
    torch.cuda.synchronize()
    wall = []
    for _ in range(a.steps):
        restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        step()
        torch.cuda.synchronize()
        wall.append((time.perf_counter() - t0) * 1e3)
    ms = float(np.mean(wall))
    P.cb_profile_enable(ctx, True)
    restore()
    step()
    torch.cuda.synchronize()
    prof = P.cb_profile_read(ctx)
    P.cb_profile_enable(ctx, False)
    g = prof["gemm"]
    achieved = g["flops"] / g["ms"] / 1e9
    token_layers = float(B * sum(k + S for k in keep))
    P.cb_destroy(ctx)
    print(json.dumps({
        "metric": "hkvd_recompute_tokens_per_s (token-layers recomputed per second over one fused prefill)",
        "value": token_layers / (ms * 1e-3), "unit": "token-layers/s", "n_gpus": 1, "steps": a.steps,
        "warmup": a.warmup, "ms_per_step": ms, "ms_per_request": ms / B, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": m.dtype, "data": "synthetic",
        "config": {"workload": w.name, "batch": B, "layers": L, "n_ctx": C, "n_suffix": S, "ratio": w.ratio,
                   "schedule": "flat" if a.flat else "gradual", "token_layers": token_layers},
        "roofline": {"kernel": "gemm_bf16_dma_kernel (all epilogues)", "bound": "mfma", "achieved": achieved,
                     "peak": PEAK["mfma_bf16_tflops"], "unit": "TFLOP/s", "frac": achieved / PEAK["mfma_bf16_tflops"],
                     "traffic": None},
        "cpu_baseline": None,
        "kernel_classes": {c: {"ms_per_step": v["ms"], "launches_per_step": v["launches"]} for c, v in prof.items()
                           if v["launches"]},
    }))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the path has no collectives); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from dataclasses import replace
    import paper_2405_16444_amd as P
    from paper_2405_16444_amd import producer
    from workloads import synth
    from workloads.configs import WORKLOADS

    w = WORKLOADS[a.workload]
    if a.layers:
        w = w.with_layers(a.layers)
    if a.ratio is not None:
        w = w.with_ratio(a.ratio)
    m = w.model
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    L, C, S, T = m.n_layers, w.n_ctx, w.n_suffix, w.n_tokens
    keep = P.cb_default_schedule(L, C, w.ratio, w.ratio_first, a.flat)

    if a.batch > 1:
        return bench_batched(a, w, keep, P, producer, synth, torch, np)

    # ---- setup (untimed): weights, inputs, pre-computed chunk caches ----
    layers = [synth.layer_weights(m, l, w.seed_weights, device=dev) for l in range(L)]
    x = synth.hidden_inputs(w, device=dev)
    ctx = P.cb_create(m, T)
    k_pre, v_pre = producer.chunk_prefill(ctx, layers, x[:C], w.chunk_lens, T)
    torch.cuda.synchronize()
    k_work = [t.clone() for t in k_pre]
    v_work = [t.clone() for t in v_pre]

    def restore():
        for dst, src in zip(k_work, k_pre):
            dst.copy_(src)
        for dst, src in zip(v_work, v_pre):
            dst.copy_(src)

    out = P.cb_fuse_prefill(ctx, layers, x, w.chunk_lens, S, k_work, v_work, keep, want_sel=True)
    torch.cuda.synchronize()
    sel_sets = [s.cpu().numpy() for s in out.sel]
    bench_out = None
    ws, structs = out.workspace, out.weight_structs

    def step():
        nonlocal bench_out
        bench_out = P.cb_fuse_prefill(ctx, layers, x, w.chunk_lens, S, k_work, v_work, keep,
                                      workspace=ws, weight_structs=structs, out=bench_out)

    for _ in range(a.warmup):
        restore()
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    gpu_ms, wall_ms = [], []
    for _ in range(a.steps):
        restore()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev0.record()
        step()
        ev1.record()
        torch.cuda.synchronize()
        wall_ms.append((time.perf_counter() - t0) * 1e3)
        gpu_ms.append(ev0.elapsed_time(ev1))
    ms_per_step = float(np.sum(wall_ms) / a.steps)          # host clock around launch + completion
    rows = [k + S for k in keep]
    token_layers = float(sum(rows))

    # ---- per-kernel-class times (HIP events around every launch, separate pass) ----
    classes, roofline = {}, None
    if not a.no_profile:
        P.cb_profile_enable(ctx, True)
        n_prof = max(1, min(3, a.steps))
        for _ in range(n_prof):
            restore()
            step()
        torch.cuda.synchronize()
        prof = P.cb_profile_read(ctx)
        P.cb_profile_enable(ctx, False)
        prof["attention"]["flops"] = attention_flops(m, sel_sets, C, S) * n_prof
        es = 2 if m.dtype == "bf16" else 4
        prof["attention"]["bytes"] = 2.0 * T * m.kv_dim * es * L * n_prof   # K and V of a layer streamed once
        for c, v in prof.items():
            if v["launches"]:
                classes[c] = {"ms_per_step": v["ms"] / n_prof, "launches_per_step": v["launches"] // n_prof,
                              "tflops": v["flops"] / v["ms"] / 1e9 if v["ms"] else 0.0,
                              "gbs": v["bytes"] / v["ms"] / 1e6 if v["ms"] else 0.0}
        g = prof["gemm"]
        achieved = g["flops"] / g["ms"] / 1e9
        roofline = {"kernel": "gemm_bf16_dma_kernel (all epilogues)", "bound": "mfma", "achieved": achieved,
                    "peak": PEAK["mfma_bf16_tflops"], "unit": "TFLOP/s", "frac": achieved / PEAK["mfma_bf16_tflops"],
                    "traffic": PMC_TRAFFIC_BYTES_PER_GEMM_LAUNCH.get(
                        (w.name, "flat" if a.flat else "gradual", L, w.ratio)),
                    "traffic_unit": "bytes per launch (L2 <-> fabric, rocprofv3 --pmc)",
                    "algorithmic_bytes_per_launch": g["bytes"] / g["launches"],
                    "avg_launch_us": g["ms"] / g["launches"] * 1e3,
                    "flops_per_launch": g["flops"] / g["launches"]}

    # ---- the same call recorded once into a HIP graph and replayed (not part of `value`: a graph
    # serves requests of one chunk structure and schedule only) ----
    graph_replay = None
    if not a.no_graph:
        graph = torch.cuda.CUDAGraph()
        restore()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            step()
        torch.cuda.synchronize()
        g_ms = []
        for i in range(2 + min(a.steps, 5)):
            restore()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            if i >= 2:
                g_ms.append((time.perf_counter() - t0) * 1e3)
        graph_replay = {"ttft_ms": float(np.mean(g_ms)), "steps": len(g_ms)}
        del graph

    # ---- first-token head on the prefill's final hidden states (not part of `value`) ----
    head = synth.head_weights(m, w.seed_weights, device=dev)
    logits, token = P.cb_first_token(ctx, bench_out.final_hidden, head["final_norm"], head["lm_head"])
    torch.cuda.synchronize()
    n_head = 20
    ev0.record()
    for _ in range(n_head):
        P.cb_first_token(ctx, bench_out.final_hidden, head["final_norm"], head["lm_head"], logits=logits, token=token)
    ev1.record()
    torch.cuda.synchronize()
    head_ms = ev0.elapsed_time(ev1) / n_head
    head_bytes = m.vocab * m.d_model * (2 if m.dtype == "bf16" else 4)
    first_token = {"ms": head_ms, "vocab": m.vocab, "gbs": head_bytes / head_ms / 1e6,
                   "frac_hbm": head_bytes / head_ms / 1e6 / PEAK["hbm_gbs"],
                   "ttft_with_first_token_ms": ms_per_step + head_ms,
                   "note": "weights stay in the memory-side cache between repeats when they fit"}

    # ---- same pass with the chunk caches in pinned host memory, loaded layer by layer on a
    # second stream while earlier layers compute (PCIe-inclusive; not part of `value`) ----
    host_load = None
    if not a.no_host_load:
        k_host = [torch.empty(t[:C].shape, dtype=t.dtype, pin_memory=True).copy_(t[:C]) for t in k_pre]
        v_host = [torch.empty(t[:C].shape, dtype=t.dtype, pin_memory=True).copy_(t[:C]) for t in v_pre]
        copy_stream = torch.cuda.Stream()
        pout = None
        hl_ms = []
        for i in range(2 + min(a.steps, 5)):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            pout = P.cb_fuse_prefill_pipelined(ctx, layers, x, w.chunk_lens, S, k_host, v_host, k_work, v_work,
                                               keep, copy_stream, workspace=ws, weight_structs=structs, out=pout)
            torch.cuda.synchronize()
            if i >= 2:
                hl_ms.append((time.perf_counter() - t0) * 1e3)
        same = bool(torch.equal(pout.final_hidden, bench_out.final_hidden))
        kv_bytes = sum(t.numel() * t.element_size() for t in k_host[1:] + v_host[1:])   # layer 0 is recomputed in full, not loaded
        host_load = {"ttft_ms": float(np.mean(hl_ms)), "kv_bytes_loaded": kv_bytes,
                     "serial_copy_ms_at_rate_seen": None, "equals_resident_result": same}
        # plain copy of the same bytes alone, for the PCIe rate of this machine
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for dst, src in zip(k_work[1:] + v_work[1:], k_host[1:] + v_host[1:]):
            dst[:C].copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        copy_ms = (time.perf_counter() - t0) * 1e3
        host_load["serial_copy_ms_at_rate_seen"] = copy_ms
        host_load["h2d_gbs"] = kv_bytes / copy_ms / 1e6
        del k_host, v_host

    cpu = None
    if not a.no_cpu_baseline:
        cpu = cpu_baseline(w, keep)

    P.cb_destroy(ctx)
    res = {
        "metric": "hkvd_recompute_tokens_per_s (token-layers recomputed per second over one fused prefill)",
        "value": token_layers / (ms_per_step * 1e-3), "unit": "token-layers/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "ttft_ms": ms_per_step, "ttft_ms_gpu_events_median": float(np.median(gpu_ms)),
        "context_tokens_per_s": C / (ms_per_step * 1e-3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": m.dtype, "data": "synthetic",
        "config": {"workload": w.name, "layers": L, "d_model": m.d_model, "heads": f"{m.n_q_heads}/{m.n_kv_heads}x{m.head_dim}",
                   "d_ff": m.d_ff, "chunks": f"{len(w.chunk_lens)}x{w.chunk_lens[0]}" if len(set(w.chunk_lens)) == 1
                   else f"{len(w.chunk_lens)} ragged", "n_ctx": C, "n_suffix": S, "ratio": w.ratio,
                   "schedule": "flat" if a.flat else "gradual", "keep_first": keep[1] if L > 1 else C,
                   "keep_last": keep[-1], "token_layers": token_layers},
        "roofline": roofline, "cpu_baseline": cpu, "kernel_classes": classes, "first_token": first_token,
        "host_load": host_load, "graph_replay": graph_replay,
    }
    print(json.dumps(res))


if __name__ == "__main__":
    main()
