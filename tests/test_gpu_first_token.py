"""First-token head (final norm, vocabulary projection, greedy pick) and the loading
controller's host arithmetic, through the C ABI, against the oracle."""
from dataclasses import replace

import numpy as np
import pytest
import torch

from oracle import cacheblend_oracle as O
from workloads import synth
from workloads.configs import WORKLOADS, ModelShape

from gpu_util import TOL, announce, max_abs_rel, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2405_16444_amd as pkg
    return pkg


def run_case(P, model, n_suffix, seed, head=None):
    head = head or synth.head_weights(model, seed)
    h = synth.random_rows(n_suffix, model.d_model, 1.5, seed + 5)          # residual stream: float
    ctx = P.cb_create(model, 64)
    logits, token = P.cb_first_token(ctx, h.cuda(), head["final_norm"].cuda(), head["lm_head"].cuda())
    torch.cuda.synchronize()
    P.cb_destroy(ctx)
    ref_logits, _ = O.first_token(to_np(h), to_np(head["final_norm"]), to_np(head["lm_head"]), model.rms_eps)
    got = logits.cpu().numpy()
    err = max_abs_rel(got, ref_logits)
    # the pick is an integer decided by floats: both sides decide on the GPU's logits
    assert int(token.item()) == O.arg_max_first(got)
    return err, got, int(token.item())


@pytest.mark.parametrize("dtype,d,vocab,n_suffix", [
    ("f32", 256, 1003, 32),        # ragged vocabulary tail (not a multiple of 32 rows per workgroup)
    ("f32", 64, 7, 1),             # fewer rows than one wavefront takes
    ("bf16", 512, 4099, 3),
    ("bf16", 1024, 32, 64),
    ("bf16", 16384, 520, 2),       # the widest model the head accepts (the normalised row fills 64 KB of LDS)
    ("f32", 16384, 96, 1),
])
def test_first_token_small(P, dtype, d, vocab, n_suffix):
    model = ModelShape(1, d, 4, 2, 64, 128, 1e-5, 1e4, dtype, vocab)
    announce("first token", dtype, d, vocab, n_suffix)
    err, _, _ = run_case(P, model, n_suffix, seed=400 + vocab)
    assert err < TOL[dtype]


@pytest.mark.parametrize("name", ["mistral7b", "yi34b"])
def test_first_token_at_real_width(P, name):
    w = WORKLOADS[name]
    announce("first token at real width", name, w.model.d_model, w.model.vocab)
    err, _, _ = run_case(P, w.model, w.n_suffix, seed=w.seed_weights)
    print(f"{name}: logits max-abs-rel {err:.2e}")
    assert err < TOL["bf16"]


def test_equal_logits_go_to_the_lowest_index(P):
    model = ModelShape(1, 256, 4, 2, 64, 128, 1e-5, 1e4, "f32", 300)
    head = synth.head_weights(model, 5)
    head["lm_head"][:] = head["lm_head"][17]            # every row equal -> every logit equal
    announce("first token ties")
    _, got, tok = run_case(P, model, 4, seed=9, head=head)
    assert np.all(got == got[0]) and tok == 0
    head = synth.head_weights(model, 6)
    head["lm_head"][250] = head["lm_head"][40]          # a duplicated row can only tie with itself
    _, got, tok = run_case(P, model, 4, seed=10, head=head)
    assert got[250] == got[40] and tok != 250


def test_first_token_rejects_bad_arguments(P):
    model = ModelShape(1, 256, 4, 2, 64, 128, 1e-5, 1e4, "f32", 100)
    head = synth.head_weights(model, 1)
    ctx = P.cb_create(model, 64)
    h = torch.zeros(0, 256, device="cuda")
    with pytest.raises(P.CacheBlendError):
        P.cb_first_token(ctx, h, head["final_norm"].cuda(), head["lm_head"].cuda())
    P.cb_destroy(ctx)
    ctx = P.cb_create(model, 64)
    with pytest.raises(P.CacheBlendError):                       # vocab of 0 rows
        P.cb_first_token(ctx, torch.zeros(1, 256, device="cuda"), head["final_norm"].cuda(),
                         torch.zeros(0, 256, device="cuda"))
    P.cb_destroy(ctx)
