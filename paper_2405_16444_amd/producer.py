"""Producer of the pre-computed chunk caches KV^pre (paper Sec. 4.1): every chunk is
prefilled alone at positions 0.. .  This is the step *before* the fusing path and is
not timed; it drives the same cb_fuse_layer entry point with every row kept."""
from __future__ import annotations

from typing import Dict, Sequence

import torch

from . import binding as B


def chunk_prefill(ctx: B.Context, layers: Sequence[Dict[str, torch.Tensor]], x_ctx: torch.Tensor,
                  chunk_lens: Sequence[int], n_rows_alloc: int):
    """Returns (k_layers, v_layers): per layer a [n_rows_alloc, Hkv, dh] tensor whose
    rows [0, sum(chunk_lens)) hold the chunks' K/V as cached at positions 0.. ."""
    m = ctx.model
    dev = ctx.device
    ks = [torch.zeros((n_rows_alloc, m.n_kv_heads, m.head_dim), dtype=ctx.dtype, device=dev)
          for _ in range(m.n_layers)]
    vs = [torch.zeros_like(k) for k in ks]
    max_len = max(chunk_lens)
    ws = torch.empty(B.cb_layer_workspace_bytes(ctx, max_len), dtype=torch.uint8, device=dev)
    o = 0
    for ln in chunk_lens:
        h = x_ctx[o:o + ln].to(torch.float32).contiguous()
        pos = torch.arange(ln, dtype=torch.int32, device=dev)
        for l in range(m.n_layers):
            # the chunk's cache rows are a contiguous slice, addressed as a cache of ln tokens
            h, _, _ = B.cb_fuse_layer(ctx, l, layers[l], h, pos, 0, ks[l][o:o + ln], vs[l][o:o + ln],
                                      ln, workspace=ws)
        o += ln
    return ks, vs
