"""Heads stored in the (i, i + head_dim/2) rotary order: re-alignment, the fused K/V and Q
projections (every GEMM kernel family and the K-split reduce launch rotate through their own
code path) and whole requests, against the oracle run with the same order.  Same parity
protocol as everywhere else."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import cacheblend_oracle as O
from workloads import synth
from workloads.configs import ModelShape

from gpu_util import TOL, announce, dev_layers, max_abs_rel, np_layers, to_np
from test_gpu_parity import (check_prefill_against_oracle, e2e_case, layer_case, oracle_layer, run_layer_both,
                             run_prefill)

pytestmark = pytest.mark.gpu

HALF = {
    "f32_dh64": ModelShape(2, 256, 4, 2, 64, 688, 1e-5, 1e4, "f32", rope_layout="half"),
    "f32_dh128": ModelShape(2, 256, 2, 1, 128, 688, 1e-5, 1e4, "f32", rope_layout="half"),      # head wider than the float tile
    "bf16": ModelShape(2, 512, 8, 2, 128, 1408, 1e-5, 1e6, "bf16", rope_layout="half"),
    "bf16_dh64": ModelShape(2, 256, 4, 2, 64, 688, 1e-5, 1e4, "bf16", rope_layout="half"),
    "bf16_k456": ModelShape(2, 456, 6, 2, 64, 1000, 1e-5, 1e4, "bf16", rope_layout="half"),     # d_model % 64 != 0: register-staged kernel
    "bf16_wide": ModelShape(2, 2048, 16, 4, 128, 1408, 1e-5, 1e6, "bf16", rope_layout="half"),  # few rows x long K: K-split projections
}


@pytest.fixture(scope="module")
def P():
    import paper_2405_16444_amd as pkg
    return pkg


@pytest.mark.parametrize("name", ["f32_dh64", "f32_dh128", "bf16", "bf16_dh64"])
def test_realign_half_order(P, name):
    model = replace(HALF[name], n_layers=2)
    announce("realign, half order", name)
    lens = (37, 1, 130, 64, 9)
    C = sum(lens)
    dt = synth.storage_dtype(model)
    ks = [synth.random_rows(C + 5, model.kv_dim, 1.0, 1900 + l, dtype=dt).view(C + 5, model.n_kv_heads, model.head_dim)
          for l in range(2)]
    ctx = P.cb_create(model, C + 5)
    kg = [k.cuda().contiguous() for k in ks]
    off = np.concatenate([[0], np.cumsum(lens)]).tolist()
    P.cb_realign_rope(ctx, kg, 0, 2, off)
    torch.cuda.synchronize()
    P.cb_destroy(ctx)
    rnd = O.storage_round(model.dtype)
    for l in range(2):
        ref = O.realign_keys(to_np(ks[l][:C]), lens, model, rnd)
        got = kg[l].cpu()
        assert max_abs_rel(to_np(got[:C]), ref) < TOL[model.dtype] * (0.01 if model.dtype == "f32" else 1)
        assert torch.equal(got[:lens[0]], ks[l][:lens[0]]) and torch.equal(got[C:], ks[l][C:])
        # not the adjacent-pair rotation by accident
        wrong = O.realign_keys(to_np(ks[l][:C]), lens, replace(model, rope_layout="adjacent"), rnd)
        assert max_abs_rel(to_np(got[:C]), wrong) > 0.1


@pytest.mark.parametrize("name,n_tokens,n_rows,n_suffix,k_keep", [
    ("f32_dh64", 333, 333, 13, 96),
    ("f32_dh128", 300, 120, 7, 31),
    ("bf16", 700, 700, 44, 197),          # Q projected after the selection
    ("bf16", 700, 260, 44, 200),          # nearly all kept: Q projected for every candidate together with K/V
    ("bf16_dh64", 419, 300, 9, 77),
    ("bf16_k456", 300, 150, 10, 40),
    ("bf16_wide", 400, 90, 6, 30),
    ("bf16_wide", 400, 400, 6, 394),      # no check: K/V/Q of every row in one projection
])
def test_layer_half_order(P, name, n_tokens, n_rows, n_suffix, k_keep):
    model = HALF[name]
    announce("layer, half order", name, n_tokens, n_rows, n_suffix, k_keep)
    lw, h, pos, kc, vc = layer_case(model, n_tokens, n_rows, n_suffix, seed=2500 + n_rows + k_keep,
                                    std=0.07 if model.d_model < 1024 else 0.03)
    n_cand = n_rows - n_suffix
    check = k_keep < n_cand
    h_out, pos_out, dev, kg, vg = run_layer_both(P, model, lw, h, pos, kc, vc, n_suffix, k_keep, want_dev=check)
    tol = TOL[model.dtype]
    if check:
        sel_pos = pos.numpy()[:n_cand][O.top_k_indices(dev.numpy(), k_keep)]
        assert np.array_equal(pos_out.numpy()[:k_keep], sel_pos)
    else:
        sel_pos = None
    h_ref, pos_ref, dev_ref, ko, vo = oracle_layer(model, lw, h, pos, kc, vc, n_suffix, k_keep, sel_pos)
    if check:
        assert max_abs_rel(dev.numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg), ko) < tol and max_abs_rel(to_np(vg), vo) < tol
    assert max_abs_rel(to_np(h_out), h_ref) < tol
    # the order matters: the adjacent-pair oracle on the same inputs is far away
    h_adj, _, _, k_adj, _ = oracle_layer(replace(model, rope_layout="adjacent"), lw, h, pos, kc, vc, n_suffix, k_keep,
                                         sel_pos)
    assert max_abs_rel(to_np(kg), k_adj) > 0.1


@pytest.mark.parametrize("name,lens,n_suffix,keep_frac", [
    ("f32_dh128", (60, 45, 70, 33), 7, (1.0, 0.4, 0.2)),
    ("bf16", (150, 97, 200), 21, (1.0, 0.35, 0.15)),
    ("bf16_dh64", (80, 120, 90), 10, (1.0, 0.3, 0.3)),
])
def test_prefill_half_order(P, name, lens, n_suffix, keep_frac):
    model = replace(HALF[name], n_layers=3)
    announce("prefill, half order", name, lens)
    w, layers, x, npl, xn, kpre, vpre = e2e_case(model, lens, n_suffix, seed=41)
    keep = [int(np.ceil(f * w.n_ctx)) for f in keep_frac]
    out, kg, vg = run_prefill(P, w, layers, x, kpre, vpre, keep)
    check_prefill_against_oracle(w, npl, xn, kpre, vpre, keep, out, kg, vg, TOL[model.dtype])


def test_half_order_model_equals_adjacent_model_with_renumbered_projections(P):
    """On the GPU too: renumbering the output channels of W_q and W_k inside every head and
    switching the order gives the same request result, K caches renumbered."""
    adj = ModelShape(3, 512, 8, 2, 128, 1408, 1e-5, 1e6, "bf16")
    half = replace(adj, rope_layout="half")
    announce("half order == adjacent order with renumbered projections")
    lens, S = (150, 97, 200), 21
    w, layers, x, npl, xn, kpre, vpre = e2e_case(adj, lens, S, seed=43)
    perm = torch.cat([torch.arange(0, 128, 2), torch.arange(1, 128, 2)])
    rows_q = (torch.arange(adj.n_q_heads)[:, None] * 128 + perm[None, :]).reshape(-1)
    rows_k = (torch.arange(adj.n_kv_heads)[:, None] * 128 + perm[None, :]).reshape(-1)
    layers_h = [dict(lw, wq=lw["wq"][rows_q].contiguous(), wk=lw["wk"][rows_k].contiguous()) for lw in layers]
    wh = replace(w, model=half)
    kpre_h = [k[..., perm.numpy()] for k in kpre]
    keep = [w.n_ctx, 157, 68]
    out_a, kg_a, vg_a = run_prefill(P, w, layers, x, kpre, vpre, keep)
    forced = [None] + [s.cpu().numpy() for s in out_a.sel[1:]]
    out_h, kg_h, vg_h = run_prefill(P, wh, layers_h, x, kpre_h, vpre, keep, forced=forced)
    tol = TOL["bf16"]
    for l in range(3):
        assert max_abs_rel(to_np(kg_h[l].cpu()), to_np(kg_a[l].cpu())[..., perm.numpy()]) < tol
        assert max_abs_rel(to_np(vg_h[l].cpu()), to_np(vg_a[l].cpu())) < tol
    assert max_abs_rel(to_np(out_h.final_hidden.cpu()), to_np(out_a.final_hidden.cpu())) < tol


@pytest.mark.parametrize("n_rows,k_keep", [(986, 877), (589, 461)])
def test_layer_half_order_at_real_width(P, n_rows, k_keep):
    """Mistral-7B width, row counts of the benchmark schedule: the big-tile kernels and their
    K-split reduce launches with the half order."""
    from test_gpu_fullsize import case, full_layer, run_gpu
    from workloads.configs import WORKLOADS
    w = WORKLOADS["mistral7b"]
    model = replace(w.model, n_layers=1, rope_layout="half")
    announce("layer at real width, half order", n_rows, k_keep)
    lw, nlw = full_layer("mistral7b")
    h, pos, kc, vc = case(model, w.n_tokens, n_rows, w.n_suffix, seed=9500 + n_rows)
    h_out, pos_out, dev, kg, vg = run_gpu(P, model, lw, h, pos, kc, vc, w.n_suffix, k_keep, True)
    tol = TOL["bf16"]
    n_cand = n_rows - w.n_suffix
    sel_pos = pos.numpy()[:n_cand][O.top_k_indices(dev.numpy(), k_keep)]
    assert np.array_equal(pos_out.numpy()[:k_keep], sel_pos)
    ko, vo = to_np(kc), to_np(vc)
    h_ref, _, dev_ref, _ = O.fuse_layer(nlw, model, to_np(h), pos.numpy(), w.n_suffix, ko, vo, k_keep,
                                        forced_sel=sel_pos, kv_round=O.round_bf16)
    assert max_abs_rel(dev.numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg), ko) < tol and max_abs_rel(to_np(vg), vo) < tol
    assert max_abs_rel(to_np(h_out), h_ref) < tol
