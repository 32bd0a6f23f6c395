"""The entry point that allocates nothing (cb_fuse_layer_static) against cb_fuse_layer: same
kernels on the library's built-in scratch array instead of a caller's workspace, so every output
must be bit-identical -- on two calls in a row, the second with a smaller input (the array keeps
the first call's contents)."""
import numpy as np
import pytest
import torch

from gpu_util import announce, dev_layers
from test_gpu_parity import BF16_M, F32_M, layer_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2405_16444_amd as pkg
    return pkg


def both_entries(P, model, n_tokens, n_rows, n_suffix, k_keep, seed):
    lw, h, pos, kc, vc = layer_case(model, n_tokens, n_rows, n_suffix, seed=seed)
    ctx = P.cb_create(model, n_tokens)
    dlw = dev_layers([lw])[0]
    hd, pd = h.cuda(), pos.cuda()
    n_out = k_keep + n_suffix
    # reference: the entry point with a caller-owned workspace
    k1, v1 = kc.cuda().contiguous(), vc.cuda().contiguous()
    h1, p1, d1 = P.cb_fuse_layer(ctx, 0, dlw, hd, pd, n_suffix, k1, v1, k_keep, want_dev=True)
    # the entry point under test: every output buffer comes from the caller, allocated beforehand
    k2, v2 = kc.cuda().contiguous(), vc.cuda().contiguous()
    h2 = torch.full((max(1, n_out), model.d_model), float("nan"), dtype=torch.float32, device="cuda")
    p2 = torch.full((max(1, n_out),), -1, dtype=torch.int32, device="cuda")
    d2 = torch.zeros((n_rows - n_suffix,), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    P.cb_fuse_layer_static(ctx, 0, dlw, hd, pd, n_suffix, k2, v2, k_keep, h2, p2, dev=d2)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before        # nothing came from torch's allocator either
    P.cb_destroy(ctx)
    assert torch.equal(p1, p2[:n_out])
    assert torch.equal(h1, h2[:n_out])
    assert torch.equal(k1, k2) and torch.equal(v1, v2)
    if k_keep < n_rows - n_suffix:
        assert torch.equal(d1, d2)


@pytest.mark.parametrize("name,model", [("bf16", BF16_M), ("f32", F32_M)])
def test_static_scratch_entry_equals_workspace_entry_twice_in_a_row(P, name, model):
    big = (700, 520, 40, 150) if name == "bf16" else (333, 200, 13, 60)
    small = (300, 97, 10, 31) if name == "bf16" else (120, 50, 5, 12)
    announce("no_alloc first call", name, *big)
    both_entries(P, model, *big, seed=4100)
    announce("no_alloc second call (smaller)", name, *small)
    both_entries(P, model, *small, seed=4200)


def test_static_scratch_entry_refuses_requests_beyond_its_array(P):
    announce("no_alloc size limit")
    from workloads.configs import WORKLOADS
    m = WORKLOADS["mistral7b"].model
    ctx = P.cb_create(m, 4096)
    rows = 4096
    assert P.cb_layer_workspace_bytes(ctx, rows) > P.cb_static_scratch_bytes()
    h = torch.zeros((rows, m.d_model), dtype=torch.float32, device="cuda")
    pos = torch.arange(rows, dtype=torch.int32, device="cuda")
    kc = torch.zeros((rows, m.n_kv_heads, m.head_dim), dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    lw = {"attn_norm": torch.ones(m.d_model, dtype=torch.bfloat16, device="cuda")}
    lw["mlp_norm"] = lw["attn_norm"]
    for k in ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down"):
        lw[k] = lw["attn_norm"]                      # never read: the call is refused before any launch
    h_out = torch.zeros_like(h)
    pos_out = torch.zeros_like(pos)
    with pytest.raises(P.CacheBlendError) as e:
        P.cb_fuse_layer_static(ctx, 0, lw, h, pos, 0, kc, vc, rows, h_out, pos_out)
    assert e.value.status == -3                      # CB_EWORKSPACE
    P.cb_destroy(ctx)
