"""Shapes of the synthetic workloads (no arithmetic of the method lives here).

The paper evaluates on retrieved-chunk RAG requests: 6 chunks of 512 tokens in
front of a short user query (Sec. 7.1), 200-400-token chunks for the
summarisation set, a "4K-long context" example (Sec. 5) and chunk-count /
chunk-length sweeps (Sec. 7.3).  The datasets and trained weights are not
available, so each workload below keeps only the *shape* of such a request:
decoder geometry, chunk lengths, suffix length, recompute ratio.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Tuple


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    rms_eps: float = 1e-5
    rope_theta: float = 1e4
    dtype: str = "bf16"  # "f32" or "bf16": storage type of weights, inputs, caches
    vocab: int = 32000   # rows of the vocabulary projection (first-token head only)
    rope_layout: str = "adjacent"   # rotary pairs (2i, 2i+1) as in the paper's Appendix A, or "half": (i, i + dh/2)
    weight_format: str = "native"   # "int8": projection matrices stored as int8 with one float scale per output feature

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def params_per_layer(self) -> int:
        d = self.d_model
        return d * (self.q_dim + 2 * self.kv_dim) + self.q_dim * d + 3 * d * self.d_ff


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    chunk_lens: Tuple[int, ...]
    n_suffix: int
    ratio: float                 # average recompute ratio r
    ratio_first: float           # r_1, the ratio of the first selection
    seed_weights: int
    seed_inputs: int
    schedule: str = "gradual"    # "gradual" | "flat"

    @property
    def n_ctx(self) -> int:
        return int(sum(self.chunk_lens))

    @property
    def n_tokens(self) -> int:
        return self.n_ctx + self.n_suffix

    def with_layers(self, n_layers: int) -> "Workload":
        """Same widths, reduced depth (used for end-to-end parity at real width)."""
        return replace(self, name=f"{self.name}-L{n_layers}",
                       model=replace(self.model, n_layers=n_layers))

    def with_ratio(self, r: float, r1: float | None = None) -> "Workload":
        return replace(self, name=f"{self.name}-r{r:g}", ratio=r,
                       ratio_first=(2 * r if r1 is None else r1))


def _ragged_lengths(n_chunks: int, lo: int, hi: int, seed: int):
    # SplitMix64 stream -> uniform integers in [lo, hi]; pure integer code so the
    # lengths are the same on every machine.
    out, state, mask = [], seed & 0xFFFFFFFFFFFFFFFF, 0xFFFFFFFFFFFFFFFF
    for _ in range(n_chunks):
        state = (state + 0x9E3779B97F4A7C15) & mask
        z = state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
        z ^= z >> 31
        out.append(lo + z % (hi - lo + 1))
    return tuple(out)


TINY = ModelShape(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64,
                  d_ff=688, rms_eps=1e-5, rope_theta=1e4, dtype="f32")
MISTRAL_7B = ModelShape(32, 4096, 32, 8, 128, 14336, 1e-5, 1e6, "bf16")
YI_34B = ModelShape(60, 7168, 56, 8, 128, 20480, 1e-5, 5e6, "bf16", 64000)
LLAMA_70B = ModelShape(80, 8192, 64, 8, 128, 28672, 1e-5, 1e4, "bf16")

WORKLOADS = {
    # cfg 1: the case the CPU oracle finishes in seconds
    "tiny": Workload("tiny", TINY, (128,) * 4, 32, 0.15, 0.30, 1001, 2001),
    # cfg 2: 6 retrieved chunks x 512 tokens + query (the paper's main request shape)
    "mistral7b": Workload("mistral7b", MISTRAL_7B, (512,) * 6, 64, 0.15, 0.30, 1002, 2002),
    # cfg 3: ratio sweep on the 34B shape
    "yi34b": Workload("yi34b", YI_34B, (512,) * 6, 64, 0.15, 0.30, 1003, 2003),
    # cfg 4: summarisation-style 10 x 400-token chunks on the 70B shape
    "llama70b": Workload("llama70b", LLAMA_70B, (400,) * 10, 64, 0.15, 0.30, 1004, 2004),
    # cfg 5a / 5b: 32K fused context, fixed and ragged chunk lengths
    "long32k": Workload("long32k", MISTRAL_7B, (1024,) * 32, 128, 0.15, 0.30, 1005, 2005),
    "long_ragged": Workload("long_ragged", MISTRAL_7B, _ragged_lengths(32, 256, 1024, 3005),
                            128, 0.15, 0.30, 1005, 2005),
}

