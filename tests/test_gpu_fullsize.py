"""Parity at the real widths of the benchmark workloads, in the launch configurations
bench.py times (row counts of the gradual schedule, 3136 / 4064 / 32896-token caches).
Inputs are synthetic single-layer cases from the seeded generator (random cache rows, random
hidden rows): a full-width end-to-end oracle run would take minutes, a single layer takes
seconds.  Where even one layer is too much for the oracle (the dense layer 0), the cache rows
are checked in full and the layer output on sampled rows, which the oracle computes one by
one from its own K/V."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import cacheblend_oracle as O
from workloads import synth
from workloads.configs import WORKLOADS

from gpu_util import TOL, announce, dev_layers, max_abs_rel, np_layers, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2405_16444_amd as pkg
    return pkg


_layer_cache = {}


def full_layer(name):
    """One layer of the named workload's model: (torch weights on cpu, float64 copies)."""
    if name not in _layer_cache:
        _layer_cache.clear()                     # one 200-850 M parameter layer at a time
        w = WORKLOADS[name]
        lw = synth.layer_weights(w.model, 1, w.seed_weights)
        _layer_cache[name] = (lw, np_layers([lw])[0])
    return _layer_cache[name]


def case(model, n_tokens, n_rows, n_suffix, seed):
    g = torch.Generator().manual_seed(seed)
    dt = synth.storage_dtype(model)
    h = synth.random_rows(n_rows, model.d_model, 1.0, seed + 1)
    n_ctx = n_tokens - n_suffix
    ctx_rows = torch.sort(torch.randperm(n_ctx, generator=g)[:n_rows - n_suffix]).values
    pos = torch.cat([ctx_rows, torch.arange(n_ctx, n_tokens)]).to(torch.int32)
    shape = (n_tokens, model.n_kv_heads, model.head_dim)
    kc = synth.random_rows(n_tokens, model.kv_dim, 0.5, seed + 2, dtype=dt).view(shape)
    vc = synth.random_rows(n_tokens, model.kv_dim, 0.5, seed + 3, dtype=dt).view(shape)
    return h, pos, kc, vc


def run_gpu(P, model, lw, h, pos, kc, vc, n_suffix, k_keep, want_dev):
    ctx = P.cb_create(model, kc.shape[0])
    dlw = dev_layers([lw])[0]
    kg, vg = kc.cuda().contiguous(), vc.cuda().contiguous()
    h_out, pos_out, dev = P.cb_fuse_layer(ctx, 0, dlw, h.cuda(), pos.cuda(), n_suffix, kg, vg, k_keep,
                                          want_dev=want_dev)
    torch.cuda.synchronize()
    P.cb_destroy(ctx)
    del dlw
    return h_out.cpu(), pos_out.cpu(), None if dev is None else dev.cpu(), kg.cpu(), vg.cpu()


@pytest.mark.parametrize("name,n_tokens,n_rows,n_suffix,k_keep", [
    ("mistral7b", 3136, 3136, 64, 922),       # layer 1: first check on all 3072 context rows, Q projected after the selection
    ("mistral7b", 3136, 986, 64, 877),        # layer 2 of the gradual schedule: check on 922 candidates
    ("mistral7b", 3136, 359, 64, 231),        # last layer: 295 candidates -> 231
    ("mistral7b", 3136, 589, 64, 461),        # 525 rows kept (flat 15 %): the gate/up GEMM's last round of tiles is shared along K
    ("yi34b", 3136, 525, 64, 400),            # 7 query heads per kv head, d = 7168
    ("yi34b", 3136, 282, 64, 154),            # ratio 0.05: the row count at which the weights, not the matrix cores, would bind
    ("yi34b", 3136, 1050, 64, 922),           # ratio 0.30
    ("llama70b", 4064, 300, 64, 200),         # 8 query heads per kv head, d = 8192, d_ff = 28672
    ("llama70b", 4064, 4064, 64, 1200),       # the headline request's layer 1: first check on all 4000 context rows
    ("llama70b", 4064, 1264, 64, 1178),       # its layer 2: nearly every candidate survives (gradual filtering)
    ("llama70b", 4064, 728, 64, 600),         # a middle layer
    ("llama70b", 4064, 366, 64, 300),         # its last layer
    ("long32k", 32896, 700, 128, 500),        # 32 K-token cache: attention KV split + long positions
    ("long32k", 131200, 400, 128, 200),       # 128 K-token cache: 1025 key tiles, positions beyond 2^17
])
def test_selective_layer_at_real_width(P, name, n_tokens, n_rows, n_suffix, k_keep):
    w = WORKLOADS[name]
    model = replace(w.model, n_layers=1)
    announce("selective layer at real width", name, n_tokens, n_rows, n_suffix, k_keep)
    lw, nlw = full_layer(name)
    h, pos, kc, vc = case(model, n_tokens, n_rows, n_suffix, seed=7000 + n_rows)
    h_out, pos_out, dev, kg, vg = run_gpu(P, model, lw, h, pos, kc, vc, n_suffix, k_keep, True)
    tol = TOL["bf16"]
    n_cand = n_rows - n_suffix
    sel_pos = pos.numpy()[:n_cand][O.top_k_indices(dev.numpy(), k_keep)]
    assert np.array_equal(pos_out.numpy()[:k_keep], sel_pos)                 # bit-exact selection
    ko, vo = to_np(kc), to_np(vc)
    h_ref, pos_ref, dev_ref, _ = O.fuse_layer(nlw, model, to_np(h), pos.numpy(), n_suffix, ko, vo, k_keep,
                                              forced_sel=sel_pos, kv_round=O.round_bf16)
    assert max_abs_rel(dev.numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg), ko) < tol and max_abs_rel(to_np(vg), vo) < tol
    untouched = np.setdiff1d(np.arange(n_tokens), pos_ref)
    assert torch.equal(kg[untouched], kc[untouched]) and torch.equal(vg[untouched], vc[untouched])
    err = max_abs_rel(to_np(h_out), h_ref)
    print(f"{name}: h_out max-abs-rel {err:.2e}")
    assert err < tol


@pytest.mark.parametrize("name,n_tokens,n_rows,n_suffix,k_keep", [
    ("mistral7b", 3136, 589, 64, 461),        # gate/up tiles shared along K, int8 tiles of every projection
    ("yi34b", 3136, 525, 64, 400),            # d = 7168: 28 column tiles of 256, 7 query heads per kv head
    ("llama70b", 4064, 728, 64, 600),         # the 8-bit headline variant's middle layer
    ("llama70b", 4064, 300, 64, 200),         # few rows: the small row tiles with the deep int8 weight ring
])
def test_selective_layer_at_real_width_with_8bit_weights(P, name, n_tokens, n_rows, n_suffix, k_keep):
    """The projection kernels reading int8 weights themselves (Sec. 7.1's 8-bit serving), in the tile shapes
    the real widths select; the oracle runs its ordinary definitions on the dequantised weights."""
    w = WORKLOADS[name]
    model = replace(w.model, n_layers=1, weight_format="int8")
    announce("8-bit selective layer at real width", name, n_tokens, n_rows, n_suffix, k_keep)
    lw, _ = full_layer(name)
    lw8 = synth.quantize_int8(lw)
    nlw8 = O.dequantize_int8({k: synth.to_f64(v) for k, v in lw8.items()})
    h, pos, kc, vc = case(model, n_tokens, n_rows, n_suffix, seed=7300 + n_rows)
    h_out, pos_out, dev, kg, vg = run_gpu(P, model, lw8, h, pos, kc, vc, n_suffix, k_keep, True)
    tol = TOL["bf16"]
    n_cand = n_rows - n_suffix
    sel_pos = pos.numpy()[:n_cand][O.top_k_indices(dev.numpy(), k_keep)]
    assert np.array_equal(pos_out.numpy()[:k_keep], sel_pos)                 # bit-exact selection
    ko, vo = to_np(kc), to_np(vc)
    h_ref, pos_ref, dev_ref, _ = O.fuse_layer(nlw8, model, to_np(h), pos.numpy(), n_suffix, ko, vo, k_keep,
                                              forced_sel=sel_pos, kv_round=O.round_bf16)
    del nlw8
    assert max_abs_rel(dev.numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg), ko) < tol and max_abs_rel(to_np(vg), vo) < tol
    err = max_abs_rel(to_np(h_out), h_ref)
    print(f"{name} 8-bit: h_out max-abs-rel {err:.2e}")
    assert err < tol


def _bench_schedule_shapes():
    """(layer, rows in, kept) of layers 1..31 of the default benchmark request: the rows that enter
    a layer are the context rows the layer before kept, plus the 64 query rows."""
    w = WORKLOADS["mistral7b"]
    keep = O.default_schedule(w.model.n_layers, w.n_ctx, w.ratio, w.ratio_first)
    return [(l, int(keep[l - 1]) + w.n_suffix, int(keep[l])) for l in range(1, w.model.n_layers)]


@pytest.mark.parametrize("layer,n_rows,k_keep", _bench_schedule_shapes())
def test_every_layer_shape_of_the_benchmark_schedule(P, layer, n_rows, k_keep):
    """Each GEMM, top-k and attention launch shape of the request bench.py times (the tile plan
    changes with the row count from layer to layer), one layer at a time with inputs of its own
    so that no error is carried from layer to layer."""
    w = WORKLOADS["mistral7b"]
    model = replace(w.model, n_layers=1)
    announce("benchmark schedule layer", layer, n_rows, k_keep)
    lw, nlw = full_layer("mistral7b")
    h, pos, kc, vc = case(model, w.n_tokens, n_rows, w.n_suffix, seed=9000 + layer)
    h_out, pos_out, dev, kg, vg = run_gpu(P, model, lw, h, pos, kc, vc, w.n_suffix, k_keep, True)
    tol = TOL["bf16"]
    n_cand = n_rows - w.n_suffix
    sel_pos = pos.numpy()[:n_cand][O.top_k_indices(dev.numpy(), k_keep)]
    assert np.array_equal(pos_out.numpy()[:k_keep], sel_pos)
    ko, vo = to_np(kc), to_np(vc)
    h_ref, pos_ref, dev_ref, _ = O.fuse_layer(nlw, model, to_np(h), pos.numpy(), w.n_suffix, ko, vo, k_keep,
                                              forced_sel=sel_pos, kv_round=O.round_bf16)
    assert max_abs_rel(dev.numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg), ko) < tol and max_abs_rel(to_np(vg), vo) < tol
    assert max_abs_rel(to_np(h_out), h_ref) < tol


@pytest.mark.parametrize("T", [3136, 81920])
def test_dense_first_layer_at_real_width_sampled(P, T):
    """Layer 0 at the Mistral-7B width: every row, no check.  3136 rows is the benchmark request;
    81920 rows makes the SwiGLU output, the attention output and the partial sums larger than
    2^31 bytes each, so every row offset in the kernels has to be 64-bit.  K/V rows are compared
    in full; the layer output on 48 sampled rows, which the oracle computes one by one."""
    w = WORKLOADS["mistral7b"]
    model = replace(w.model, n_layers=1)
    S = w.n_suffix
    announce("dense first layer, sampled", T)
    lw, nlw = full_layer("mistral7b")
    h, pos, kc, vc = case(model, T, T, S, seed=9100)
    h_out, pos_out, _, kg, vg = run_gpu(P, model, lw, h, pos, kc, vc, S, T - S, False)
    assert np.array_equal(pos_out.numpy(), np.arange(T))
    hn = to_np(h)
    xn, k_ref, v_ref = O.project_kv(hn, np.arange(T), nlw, model)
    k_ref, v_ref = O.round_bf16(k_ref), O.round_bf16(v_ref)
    tol = TOL["bf16"]
    assert max_abs_rel(to_np(kg), k_ref) < tol and max_abs_rel(to_np(vg), v_ref) < tol
    rows = np.unique(np.concatenate([[0, 1, 63, 64, 127, 128, T - 1], np.random.default_rng(5).integers(0, T, 41)]))
    q = O.project_q(xn[rows], rows, nlw, model)
    o = O.attention(q, rows, k_ref, v_ref)
    ref = O.finish_block(hn[rows], o, nlw, model)
    err = max_abs_rel(to_np(h_out[torch.from_numpy(rows)]), ref)
    print(f"dense layer 0, {T} rows: sampled h_out max-abs-rel {err:.2e}")
    assert err < tol


def test_three_layer_prefill_at_real_width(P):
    """End to end at the Mistral-7B width with reduced depth: re-alignment, a full layer 0, the
    first check on all 3072 context rows, a second check on the survivors.  The pre-computed caches
    are seeded random rows (an input like any other); the whole parity protocol applies."""
    w = WORKLOADS["mistral7b"].with_layers(3)
    model = w.model
    announce("three-layer prefill at real width", w.n_tokens)
    layers = [synth.layer_weights(model, l, w.seed_weights) for l in range(3)]
    npl = np_layers(layers)
    x = synth.hidden_inputs(w)
    dt = synth.storage_dtype(model)
    C, T = w.n_ctx, w.n_tokens
    shape = (C, model.n_kv_heads, model.head_dim)
    kpre = [synth.random_rows(C, model.kv_dim, 0.5, 8100 + l, dtype=dt).view(shape) for l in range(3)]
    vpre = [synth.random_rows(C, model.kv_dim, 0.5, 8200 + l, dtype=dt).view(shape) for l in range(3)]
    keep = [C, 922, 877]
    ctx = P.cb_create(model, T)
    kg = [torch.zeros((T,) + shape[1:], dtype=dt, device="cuda") for _ in range(3)]
    vg = [torch.zeros_like(t) for t in kg]
    for l in range(3):
        kg[l][:C] = kpre[l].cuda()
        vg[l][:C] = vpre[l].cuda()
    out = P.cb_fuse_prefill(ctx, dev_layers(layers), x.cuda(), w.chunk_lens, w.n_suffix, kg, vg, keep,
                            want_sel=True, want_dev=True)
    torch.cuda.synchronize()
    P.cb_destroy(ctx)
    tol = TOL["bf16"]
    sel = [s.cpu().numpy().astype(np.int64) for s in out.sel]
    cand = np.arange(C)
    for l in (1, 2):
        d = out.dev[l].cpu().numpy()
        assert np.array_equal(sel[l], cand[O.top_k_indices(d, keep[l])]), f"layer {l}"      # bit-exact selection
        cand = sel[l]
    ref = O.fuse_prefill(to_np(x), npl, model, w.chunk_lens, w.n_suffix, [to_np(t) for t in kpre],
                         [to_np(t) for t in vpre], keep, forced_sel=sel, kv_round=O.round_bf16)
    for l in range(3):
        assert max_abs_rel(to_np(kg[l].cpu()), ref.K[l]) < tol and max_abs_rel(to_np(vg[l].cpu()), ref.V[l]) < tol
        if l:
            assert max_abs_rel(out.dev[l].cpu().numpy(), ref.dev[l]) < tol
    err = max_abs_rel(to_np(out.final_hidden.cpu()), ref.final_hidden)
    print(f"three layers at real width: final hidden max-abs-rel {err:.2e}")
    assert err < tol


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_layer_with_rows_wider_than_the_finish_kernel_keeps_in_registers(P, dtype):
    """d_model = 9216: the launches that finish the float outputs (sum of the K splits + residual +
    RMSNorm) hold rows of up to 8192 elements in registers and take their loop form beyond that."""
    from workloads.configs import ModelShape
    model = ModelShape(1, 9216, 8, 2, 128, 2048, 1e-5, 1e4, dtype)
    n_tokens, n_rows, n_suffix, k_keep = 300, 140, 12, 70
    announce("wide rows", dtype)
    lw = synth.layer_weights(model, 1, 4242)
    nlw = np_layers([lw])[0]
    h, pos, kc, vc = case(model, n_tokens, n_rows, n_suffix, seed=9216)
    h_out, pos_out, dev, kg, vg = run_gpu(P, model, lw, h, pos, kc, vc, n_suffix, k_keep, True)
    tol = TOL[dtype]
    sel_pos = pos.numpy()[:n_rows - n_suffix][O.top_k_indices(dev.numpy(), k_keep)]
    assert np.array_equal(pos_out.numpy()[:k_keep], sel_pos)
    ko, vo = to_np(kc), to_np(vc)
    h_ref, pos_ref, dev_ref, _ = O.fuse_layer(nlw, model, to_np(h), pos.numpy(), n_suffix, ko, vo, k_keep,
                                              forced_sel=sel_pos, kv_round=O.round_bf16 if dtype == "bf16" else O.identity)
    assert max_abs_rel(dev.numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg), ko) < tol and max_abs_rel(to_np(vg), vo) < tol
    err = max_abs_rel(to_np(h_out), h_ref)
    print(f"d_model 9216 {dtype}: h_out max-abs-rel {err:.2e}")
    assert err < tol
