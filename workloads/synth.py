"""Seeded synthetic tensors for the workloads: the only code shared by the
CPU oracle's tests and the HIP path's tests/bench.  It draws random numbers and
rounds them to the storage type; it holds none of the method's arithmetic.

Recipe (stands in for trained weights and dataset text, which are not available):
  * every projection matrix  ~ N(0, 0.02^2), stored [out_features, in_features];
  * RMSNorm gains = 1 (an N(0, 0.02) gain would wipe out the signal);
  * layer-0 hidden states of all context and suffix tokens ~ N(0, 1);
  * bf16 workloads are rounded to bf16 once, here, so both sides see the very
    same values.
Each tensor has its own torch.Generator seeded from (seed, layer, tensor id), so
any single layer can be regenerated alone.  Values depend on the device the
generator runs on; whoever needs them elsewhere copies them.
"""
from __future__ import annotations

import torch

from .configs import ModelShape, Workload

_TENSOR_IDS = {"wq": 1, "wk": 2, "wv": 3, "wo": 4, "w_gate": 5, "w_up": 6, "w_down": 7}
WEIGHT_STD = 0.02


def storage_dtype(model: ModelShape) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16}[model.dtype]


def _normal(shape, std, seed, device, dtype):
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    t = torch.empty(shape, dtype=torch.float32, device=device)
    t.normal_(0.0, std, generator=g)
    return t.to(dtype)


def layer_weights(model: ModelShape, layer: int, seed: int, device="cpu"):
    """dict name -> tensor for one decoder layer (see module docstring)."""
    d, f = model.d_model, model.d_ff
    shapes = {
        "wq": (model.q_dim, d), "wk": (model.kv_dim, d), "wv": (model.kv_dim, d),
        "wo": (d, model.q_dim), "w_gate": (f, d), "w_up": (f, d), "w_down": (d, f),
    }
    dt = storage_dtype(model)
    out = {}
    for name, shp in shapes.items():
        s = (seed * 1_000_003 + layer * 101 + _TENSOR_IDS[name]) % (2 ** 63 - 1)
        out[name] = _normal(shp, WEIGHT_STD, s, device, dt)
    out["attn_norm"] = torch.ones(d, dtype=dt, device=device)
    out["mlp_norm"] = torch.ones(d, dtype=dt, device=device)
    return out


def quantize_int8(lw):
    """The same layer with every projection matrix stored as int8 plus one float scale per output
    feature (row): scale = max|row| / 127, q = round(w / scale).  Part of the input recipe of the 8-bit
    workloads (the paper serves its larger models 8-bit and names no scheme); what the stored pair MEANS,
    w = q * scale, is the consumer's business."""
    out = {}
    for name, t in lw.items():
        if name.startswith("w"):
            w = t.float()
            scale = (w.abs().amax(dim=1).clamp_min(1e-12) / 127.0).contiguous()
            out[name] = torch.round(w / scale[:, None]).clamp(-127, 127).to(torch.int8).contiguous()
            out[name + "_scale"] = scale
        else:
            out[name] = t
    return out


def head_weights(model: ModelShape, seed: int, device="cpu"):
    """Final norm gain (ones) and vocabulary projection [vocab, d] ~ N(0, 0.02^2)."""
    dt = storage_dtype(model)
    s = (seed * 1_000_003 + 977_777) % (2 ** 63 - 1)
    return {"final_norm": torch.ones(model.d_model, dtype=dt, device=device),
            "lm_head": _normal((model.vocab, model.d_model), WEIGHT_STD, s, device, dt)}


def model_weights(model: ModelShape, seed: int, device="cpu"):
    return [layer_weights(model, l, seed, device) for l in range(model.n_layers)]


def hidden_inputs(w: Workload, device="cpu"):
    """[T, d] layer-0 hidden states: context tokens chunk after chunk, then the suffix."""
    return _normal((w.n_tokens, w.model.d_model), 1.0, w.seed_inputs * 7919 + 13,
                   device, storage_dtype(w.model))


def random_rows(n, width, std, seed, device="cpu", dtype=torch.float32):
    """Generic seeded N(0, std^2) matrix for single-kernel tests."""
    return _normal((n, width), std, seed, device, dtype)


def to_f64(t: torch.Tensor):
    """Exact widening copy to a numpy float64 array (what the oracle consumes)."""
    return t.detach().to("cpu").to(torch.float64).numpy()
