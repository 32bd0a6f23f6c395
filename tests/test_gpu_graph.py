"""The fused prefill recorded into a HIP graph: with caller-owned workspace and outputs the entry
point allocates nothing and only queues kernels and device-to-device copies on the stream it is
given, so a serving loop can capture it once and replay it.  Every replay (with eager work and
synchronisations in between) must reproduce the eager call bit for bit."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from gpu_util import announce, cache_tensors, dev_layers
from test_gpu_parity import MODELS, e2e_case

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2405_16444_amd as pkg
    return pkg


@pytest.mark.parametrize("name", ["bf16", "f32"])
def test_captured_prefill_replays_bitwise(P, name):
    model = replace(MODELS[name], n_layers=3)
    announce("prefill in a HIP graph", name)
    w, layers, x, npl, xn, kpre, vpre = e2e_case(model, (150, 97, 200), 21, seed=60)
    keep = [w.n_ctx, int(np.ceil(0.35 * w.n_ctx)), int(np.ceil(0.15 * w.n_ctx))]
    ctx = P.cb_create(model, w.n_tokens)
    dl = dev_layers(layers)
    xg = x.cuda()
    k_src, v_src = cache_tensors(w, kpre, vpre)
    k_work = [t.clone() for t in k_src]
    v_work = [t.clone() for t in v_src]

    # eager call: the reference, and the run that sets every kernel's launch attributes
    out = P.cb_fuse_prefill(ctx, dl, xg, w.chunk_lens, w.n_suffix, k_work, v_work, keep, want_sel=True)
    torch.cuda.synchronize()
    ref_h = out.final_hidden.clone()
    ref_k = [t.clone() for t in k_work]
    ref_sel = [s.clone() for s in out.sel]

    def restore_and_run():
        for dst, src in zip(k_work + v_work, k_src + v_src):
            dst.copy_(src)
        P.cb_fuse_prefill(ctx, dl, xg, w.chunk_lens, w.n_suffix, k_work, v_work, keep, want_sel=True,
                          workspace=out.workspace, weight_structs=out.weight_structs, out=out)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        restore_and_run()
    torch.cuda.synchronize()
    for replay in range(3):
        # eager work between the replays: spoil the outputs and the workspace
        out._final_buf.fill_(float("nan"))
        out.workspace.fill_(0xFF)
        for t in k_work:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out.final_hidden, ref_h), f"replay {replay}"
        for l in range(3):
            assert torch.equal(k_work[l], ref_k[l]) and torch.equal(out.sel[l], ref_sel[l]), f"replay {replay}"
    del graph
    P.cb_destroy(ctx)
