"""8-bit projection weights (Sec. 7.1 serves the two larger models with 8-bit weights; the scheme --
weight-only symmetric int8, one scale per output feature -- is this build's reading, "parity unpinned"
by the paper).  The oracle dequantises (w = q * scale) and runs its ordinary definitions; the HIP
projection kernels read the int8 weights themselves, multiply the exact integers on the matrix cores and
scale the finished sums (input widths that are multiples of 64), or fall back to expanding a matrix to
bf16 right before its projection (any other width)."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import cacheblend_oracle as O
from workloads import synth
from workloads.configs import ModelShape, Workload

from gpu_util import TOL, announce, cache_tensors, dev_layers, max_abs_rel, oracle_caches, scaled_weights, to_np
from test_gpu_parity import BF16_M, layer_case

pytestmark = pytest.mark.gpu
INT8_M = replace(BF16_M, weight_format="int8")           # d = 512, 8 / 2 heads of 128, SwiGLU 1408
# SwiGLU width 1392 is no multiple of 64: the down projection takes the expand-first fallback
INT8_M_ODD = replace(INT8_M, d_ff=1392)


@pytest.fixture(scope="module")
def P():
    import paper_2405_16444_amd as pkg
    return pkg


def np_int8_layer(lw8):
    return O.dequantize_int8({k: synth.to_f64(v) for k, v in lw8.items()})


@pytest.mark.parametrize("model8", [INT8_M, INT8_M_ODD], ids=["ff1408", "ff1392"])
@pytest.mark.parametrize("n_tokens,n_rows,n_suffix,k_keep", [(700, 700, 44, 197), (700, 260, 44, 216), (419, 150, 9, 141)])
def test_int8_layer_matches_oracle_on_dequantised_weights(P, model8, n_tokens, n_rows, n_suffix, k_keep):
    announce("int8 layer", model8.d_ff, n_tokens, n_rows, n_suffix, k_keep)
    native = replace(model8, weight_format="native")
    lw, h, pos, kc, vc = layer_case(native, n_tokens, n_rows, n_suffix, seed=7000 + n_rows)
    lw8 = synth.quantize_int8(lw)
    n_cand = n_rows - n_suffix
    check = k_keep < n_cand
    ctx = P.cb_create(model8, n_tokens)
    kg, vg = kc.cuda().contiguous(), vc.cuda().contiguous()
    h_out, pos_out, dev = P.cb_fuse_layer(ctx, 0, dev_layers([lw8])[0], h.cuda(), pos.cuda(), n_suffix, kg, vg, k_keep,
                                          want_dev=check)
    torch.cuda.synchronize()
    sel_pos = None
    if check:
        sel_pos = pos.numpy()[:n_cand][O.top_k_indices(dev.cpu().numpy(), k_keep)]
        assert np.array_equal(pos_out.cpu().numpy()[:k_keep], sel_pos)
    ko, vo = to_np(kc), to_np(vc)
    h_ref, pos_ref, dev_ref, _ = O.fuse_layer(np_int8_layer(lw8), model8, to_np(h), pos.numpy(), n_suffix, ko, vo, k_keep,
                                              forced_sel=sel_pos, kv_round=O.round_bf16)
    tol = TOL["bf16"]
    assert np.array_equal(pos_out.cpu().numpy(), pos_ref)
    if check:
        assert max_abs_rel(dev.cpu().numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg.cpu()), ko) < tol and max_abs_rel(to_np(vg.cpu()), vo) < tol
    assert max_abs_rel(to_np(h_out.cpu()), h_ref) < tol

    # against the bf16 path on the expanded weights bf16(q * scale): the same computation up to the rounding of
    # the expansion (the 8-bit path multiplies the exact integers and scales the float sums)
    lw_exp = {}
    for name, t in lw8.items():
        if name.endswith("_scale"):
            continue
        lw_exp[name] = (t.float() * lw8[name + "_scale"][:, None]).to(torch.bfloat16) if t.dtype == torch.int8 else t
    ctx2 = P.cb_create(native, n_tokens)
    kg2, vg2 = kc.cuda().contiguous(), vc.cuda().contiguous()
    forced = None if not check else torch.from_numpy(sel_pos.astype(np.int32)).cuda()
    h2, p2, d2 = P.cb_fuse_layer(ctx2, 0, dev_layers([lw_exp])[0], h.cuda(), pos.cuda(), n_suffix, kg2, vg2, k_keep,
                                 want_dev=check, forced_sel=forced)
    torch.cuda.synchronize()
    assert torch.equal(p2, pos_out)
    assert max_abs_rel(to_np(h2.cpu()), to_np(h_out.cpu())) < tol
    assert max_abs_rel(to_np(kg2.cpu()), to_np(kg.cpu())) < tol and max_abs_rel(to_np(vg2.cpu()), to_np(vg.cpu())) < tol
    P.cb_destroy(ctx)
    P.cb_destroy(ctx2)


def test_int8_prefill_end_to_end(P):
    model = replace(INT8_M, n_layers=3)
    w = Workload("int8", model, (150, 97, 200), 21, 0.15, 0.30, 9301, 9302)
    announce("int8 prefill end to end")
    layers8 = [synth.quantize_int8(lw) for lw in scaled_weights(replace(model, weight_format="native"), w.seed_weights, 0.05)]
    x = synth.hidden_inputs(w)
    npl, xn = [np_int8_layer(lw) for lw in layers8], synth.to_f64(x)
    kpre, vpre = oracle_caches(w, npl, xn)
    keep = O.default_schedule(model.n_layers, w.n_ctx, w.ratio, w.ratio_first)
    ctx = P.cb_create(model, w.n_tokens)
    kg, vg = cache_tensors(w, kpre, vpre)
    out = P.cb_fuse_prefill(ctx, dev_layers(layers8), x.cuda(), w.chunk_lens, w.n_suffix, kg, vg, keep,
                            want_sel=True, want_dev=True)
    torch.cuda.synchronize()
    P.cb_destroy(ctx)
    sel = [s.cpu().numpy().astype(np.int64) for s in out.sel]
    cand = np.arange(w.n_ctx)
    for l, k in enumerate(keep):
        if k < len(cand):
            assert np.array_equal(sel[l], cand[O.top_k_indices(out.dev[l].cpu().numpy(), k)]), f"layer {l}"
        cand = sel[l]
    ref = O.fuse_prefill(xn, npl, model, w.chunk_lens, w.n_suffix, kpre, vpre, keep, forced_sel=sel,
                         kv_round=O.round_bf16)
    for l in range(model.n_layers):
        assert max_abs_rel(to_np(kg[l].cpu()), ref.K[l]) < TOL["bf16"], f"K layer {l}"
        assert max_abs_rel(to_np(vg[l].cpu()), ref.V[l]) < TOL["bf16"], f"V layer {l}"
    e = max_abs_rel(to_np(out.final_hidden.cpu()), ref.final_hidden)
    print(f"int8 prefill: final hidden max-abs-rel {e:.2e}")
    assert e < TOL["bf16"]


def test_int8_argument_checks(P):
    announce("int8 argument checks")
    with pytest.raises(P.CacheBlendError) as e:
        P.cb_create(ModelShape(1, 256, 4, 2, 64, 688, 1e-5, 1e4, "f32", weight_format="int8"), 64)
    assert e.value.status == -4              # CB_EUNSUPPORTED: 8-bit weights go with bf16 activations only
    lw, h, pos, kc, vc = layer_case(BF16_M, 64, 32, 4, seed=7100)
    lw8 = synth.quantize_int8(lw)
    ctx = P.cb_create(INT8_M, 64)
    dl = dev_layers([lw8])[0]
    from paper_2405_16444_amd import binding as B
    import ctypes as C
    s = B._weights_struct(dl, torch.bfloat16, torch.device("cuda", torch.cuda.current_device()))
    s.wo_scale = None                        # a matrix without its scales
    hd, pd, kg, vg = h.cuda(), pos.cuda(), kc.cuda().contiguous(), vc.cuda().contiguous()
    h_out = torch.empty_like(hd)
    pos_out = torch.empty_like(pd)
    ws = torch.empty(P.cb_layer_workspace_bytes(ctx, 32), dtype=torch.uint8, device="cuda")
    st = B._lib.cb_fuse_layer(ctx._h, 0, C.byref(s), B._ptr(hd), B._ptr(pd), 32, 4, B._ptr(kg), B._ptr(vg), 64, 28,
                              None, B._ptr(h_out), B._ptr(pos_out), None, B._ptr(ws), ws.numel(), B._stream(None))
    assert st == -2                          # CB_ENULL, before any launch
    P.cb_destroy(ctx)
