"""Layer-pipelined loading (Sec. 5): the pre-computed caches start in pinned host memory and
are copied layer by layer on a second stream while earlier layers are recomputed.  The result
must be the one of the device-resident entry point bit for bit (the same kernels run on the
same values), which the other tests hold against the oracle; the tiny workload is also checked
against the oracle directly."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import cacheblend_oracle as O
from workloads import synth
from workloads.configs import WORKLOADS

from gpu_util import TOL, announce, cache_tensors, dev_layers, max_abs_rel, np_layers, oracle_caches, to_np
from test_gpu_parity import MODELS, e2e_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2405_16444_amd as pkg
    return pkg


def host_caches(w, pre):
    dt = synth.storage_dtype(w.model)
    out = []
    for a in pre:
        t = torch.empty((w.n_ctx, w.model.n_kv_heads, w.model.head_dim), dtype=dt, pin_memory=True)
        t.copy_(torch.from_numpy(a).to(dt))
        out.append(t)
    return out


def run_both(P, w, layers, x, kpre, vpre, keep):
    dl = dev_layers(layers)
    ctx = P.cb_create(w.model, w.n_tokens)
    kg, vg = cache_tensors(w, kpre, vpre)
    ref = P.cb_fuse_prefill(ctx, dl, x.cuda(), w.chunk_lens, w.n_suffix, kg, vg, keep, want_sel=True)
    torch.cuda.synchronize()
    kh, vh = host_caches(w, kpre), host_caches(w, vpre)
    dt = synth.storage_dtype(w.model)
    shape = (w.n_tokens, w.model.n_kv_heads, w.model.head_dim)
    # destination rows start as garbage: everything the result needs must come from the host copies
    kp = [torch.full(shape, 7.0, dtype=dt, device="cuda") for _ in kh]
    vp = [torch.full(shape, -3.0, dtype=dt, device="cuda") for _ in vh]
    copy_stream = torch.cuda.Stream()
    out = P.cb_fuse_prefill_pipelined(ctx, dl, x.cuda(), w.chunk_lens, w.n_suffix, kh, vh, kp, vp, keep, copy_stream)
    torch.cuda.synchronize()
    # second call on the same ctx: the copies must wait for the first call's work on the buffers
    out2 = P.cb_fuse_prefill_pipelined(ctx, dl, x.cuda(), w.chunk_lens, w.n_suffix, kh, vh, kp, vp, keep,
                                       copy_stream, workspace=out.workspace)
    torch.cuda.synchronize()
    P.cb_destroy(ctx)
    C = w.n_ctx
    for l in range(w.model.n_layers):
        # suffix rows of layers whose suffix... every layer writes its suffix rows, so whole caches compare
        assert torch.equal(kp[l], kg[l]) and torch.equal(vp[l], vg[l]), f"layer {l}"
    assert torch.equal(out.final_hidden, ref.final_hidden) and torch.equal(out2.final_hidden, ref.final_hidden)
    out.sel = ref.sel           # the pipelined entry takes no dumps; it is bitwise the resident call, whose sets these are
    return out, kp, vp


def test_pipelined_tiny_workload_matches_oracle_and_resident_path(P):
    w = WORKLOADS["tiny"]
    announce("pipelined tiny")
    layers = synth.model_weights(w.model, w.seed_weights)
    x = synth.hidden_inputs(w)
    npl, xn = np_layers(layers), synth.to_f64(x)
    kpre, vpre = oracle_caches(w, npl, xn)
    keep = O.default_schedule(w.model.n_layers, w.n_ctx, w.ratio, w.ratio_first)
    out, kp, vp = run_both(P, w, layers, x, kpre, vpre, keep)
    # the oracle is forced to the kept sets of the GPU (parity protocol), so the plain tolerance applies
    sel = [t.cpu().numpy().astype(np.int64) for t in out.sel]
    ref = O.fuse_prefill(xn, npl, w.model, w.chunk_lens, w.n_suffix, kpre, vpre, keep, forced_sel=sel)
    assert max_abs_rel(to_np(out.final_hidden.cpu()), ref.final_hidden) < TOL["f32"]
    for l in range(w.model.n_layers):
        assert max_abs_rel(to_np(kp[l].cpu()), ref.K[l]) < TOL["f32"] and max_abs_rel(to_np(vp[l].cpu()), ref.V[l]) < TOL["f32"]


@pytest.mark.parametrize("name,lens,n_suffix,keep_frac", [
    ("bf16", (150, 97, 200), 21, (1.0, 0.35, 0.15)),
    ("bf16_g7", (80, 120, 90), 10, (1.0, 0.3, 0.3)),
])
def test_pipelined_three_layers_bitwise(P, name, lens, n_suffix, keep_frac):
    model = replace(MODELS[name], n_layers=3)
    announce("pipelined three layers", name, lens)
    w, layers, x, npl, xn, kpre, vpre = e2e_case(model, lens, n_suffix, seed=41)
    keep = [int(np.ceil(f * w.n_ctx)) for f in keep_frac]
    run_both(P, w, layers, x, kpre, vpre, keep)


def test_pipelined_rejects_one_stream_for_both(P):
    w = WORKLOADS["tiny"]
    layers = dev_layers(synth.model_weights(w.model, w.seed_weights))
    x = synth.hidden_inputs(w).cuda()
    ctx = P.cb_create(w.model, w.n_tokens)
    z = [np.zeros((w.n_ctx, w.model.n_kv_heads, w.model.head_dim), np.float32)] * w.model.n_layers
    kh, vh = host_caches(w, z), host_caches(w, z)
    kg, vg = cache_tensors(w, z, z)
    keep = P.cb_default_schedule(w.model.n_layers, w.n_ctx, w.ratio, w.ratio_first)
    with pytest.raises(P.CacheBlendError):
        P.cb_fuse_prefill_pipelined(ctx, layers, x, w.chunk_lens, w.n_suffix, kh, vh, kg, vg, keep,
                                    torch.cuda.current_stream())
    P.cb_destroy(ctx)
