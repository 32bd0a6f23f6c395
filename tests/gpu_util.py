"""Helpers of the GPU parity tests: move seeded inputs to the device, run the oracle on
the same values, compare with the max-abs-rel metric of the parity protocol."""
from __future__ import annotations

import sys
from dataclasses import replace

import numpy as np
import torch

from oracle import cacheblend_oracle as O
from workloads import synth
from workloads.configs import ModelShape, Workload

TOL = {"f32": 1e-4, "bf16": 2e-2}     # max|gpu - oracle| / max|oracle| per tensor


def announce(*what):
    """Name the case before the GPU step so a lost box still tells which one ran."""
    print("[gpu-case]", *what, flush=True)
    sys.stdout.flush()


def max_abs_rel(got, ref) -> float:
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def dev_noise_bound(k_rows, v_rows, dtype: str):
    """Largest deviation a candidate can show when its exact new K/V EQUAL its cached K/V (a token of
    the first chunk: a prefix, so its exact deviation is zero).  Two things separate the stored new row
    from its cached twin: (a) the hidden state it is projected from, which on this path matches the exact
    one only within the parity tolerance tol (relative), and the projection is linear in it; (b) the
    storage rounding of both rows, at most one unit in the last place per element, 2^-p |x| with p = 7
    for bf16 (8-bit significand, the coarsest spacing of a binade) and 23 for float.  Element-wise
    |new - cached| <= (tol + 2^-p) |x| in the norm of the row, hence
        dev <= (tol + 2^-p)^2 (|K row|^2 + |V row|^2).
    k_rows, v_rows: the candidates' cached rows [n, Hkv, dh] (the norm does not depend on the rotation)."""
    p = 7 if dtype == "bf16" else 23
    k = np.asarray(k_rows, np.float64).reshape(len(k_rows), -1)
    v = np.asarray(v_rows, np.float64).reshape(len(v_rows), -1)
    return (TOL[dtype] + 2.0 ** -p) ** 2 * ((k * k).sum(axis=1) + (v * v).sum(axis=1))


def to_np(t: torch.Tensor):
    return t.detach().to("cpu").to(torch.float64).numpy()


def dev_layers(layers, device="cuda"):
    return [{k: v.to(device).contiguous() for k, v in lw.items()} for lw in layers]


def np_layers(layers):
    return [{k: synth.to_f64(v) for k, v in lw.items()} for lw in layers]


def scaled_weights(model: ModelShape, seed: int, std: float | None):
    layers = synth.model_weights(model, seed)
    if std is not None:
        for lw in layers:
            for k in lw:
                if k.startswith("w"):
                    lw[k] = (lw[k].float() * (std / synth.WEIGHT_STD)).to(lw[k].dtype)
    return layers


def oracle_caches(w: Workload, npl, xn):
    """KV^pre from the oracle's own chunk prefill (stored rounded in bf16 workloads)."""
    rnd = O.storage_round(w.model.dtype)
    return O.chunk_prefill(xn[:w.n_ctx], w.chunk_lens, npl, w.model, rnd)


def cache_tensors(w: Workload, kpre, vpre, device="cuda"):
    """Per-layer device caches [T, Hkv, dh] with rows [0, C) = KV^pre (exact copies)."""
    dt = synth.storage_dtype(w.model)
    m = w.model
    ks, vs = [], []
    for l in range(m.n_layers):
        k = torch.zeros((w.n_tokens, m.n_kv_heads, m.head_dim), dtype=dt, device=device)
        v = torch.zeros_like(k)
        k[:w.n_ctx] = torch.from_numpy(kpre[l]).to(dt).to(device)
        v[:w.n_ctx] = torch.from_numpy(vpre[l]).to(dt).to(device)
        ks.append(k)
        vs.append(v)
    return ks, vs
