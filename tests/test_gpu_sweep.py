"""Seeded sweep of single-layer shapes: row counts around every tile edge of the kernels, head
groupings, widths that are and are not multiples of 64, with and without a check, against the
oracle with the usual protocol (kept set bit-exact for the GPU's deviation vector, everything
else within tolerance with the oracle forced to that set)."""
import numpy as np
import pytest
import torch

from oracle import cacheblend_oracle as O
from workloads.configs import ModelShape

from gpu_util import TOL, announce, max_abs_rel, to_np
from test_gpu_parity import layer_case, oracle_layer, run_layer_both

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    import paper_2405_16444_amd as pkg
    return pkg


def cases():
    rng = np.random.default_rng(20240527)
    geoms = [(256, 4, 2, 64, 512), (512, 8, 2, 64, 1024), (512, 4, 4, 128, 768), (896, 7, 1, 128, 1536),
             (256, 4, 1, 64, 688)]                              # last: d_ff not a multiple of 64
    rows_pool = [1, 2, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 383, 385, 511, 513, 640]
    out = []
    for i in range(36):
        d, hq, hkv, dh, f = geoms[i % len(geoms)]
        dtype = "f32" if i % 9 == 4 else "bf16"
        n_rows = int(rows_pool[int(rng.integers(len(rows_pool)))])
        n_suffix = int(min(n_rows, rng.integers(0, 40)))
        n_cand = n_rows - n_suffix
        mode = i % 3                                             # 0: no check, 1: keep most, 2: keep few
        k = n_cand if mode == 0 else int(n_cand * (0.9 if mode == 1 else 0.3))
        n_tokens = n_rows + int(rng.integers(0, 300))
        out.append((i, dtype, d, hq, hkv, dh, f, n_tokens, n_rows, n_suffix, k))
    return out


@pytest.mark.parametrize("case", cases(), ids=lambda c: f"{c[0]}-{c[1]}-d{c[2]}-h{c[3]}/{c[4]}x{c[5]}-r{c[8]}-s{c[9]}-k{c[10]}")
def test_layer_shape_sweep(P, case):
    i, dtype, d, hq, hkv, dh, f, n_tokens, n_rows, n_suffix, k = case
    model = ModelShape(1, d, hq, hkv, dh, f, 1e-5, 1e4, dtype)
    announce("sweep", case)
    lw, h, pos, kc, vc = layer_case(model, n_tokens, n_rows, n_suffix, seed=5000 + i)
    n_cand = n_rows - n_suffix
    check = k < n_cand
    h_out, pos_out, dev, kg, vg = run_layer_both(P, model, lw, h, pos, kc, vc, n_suffix, k, want_dev=check)
    tol = TOL[dtype]
    forced = None
    if check:
        sel_pos = pos.numpy()[:n_cand][O.top_k_indices(dev.numpy(), k)]
        assert np.array_equal(pos_out.numpy()[:k], sel_pos)
        forced = sel_pos
    h_ref, pos_ref, dev_ref, ko, vo = oracle_layer(model, lw, h, pos, kc, vc, n_suffix, k, forced)
    assert np.array_equal(pos_out.numpy(), pos_ref)
    if check and n_cand:
        assert max_abs_rel(dev.numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg), ko) < tol and max_abs_rel(to_np(vg), vo) < tol
    untouched = np.setdiff1d(np.arange(n_tokens), pos_ref)
    assert torch.equal(kg[untouched], kc[untouched]) and torch.equal(vg[untouched], vc[untouched])
    if h_ref.size:
        assert max_abs_rel(to_np(h_out), h_ref) < tol


@pytest.mark.parametrize("dh,hq,hkv", [(64, 4, 1), (64, 4, 4), (128, 2, 1)])
def test_rows_with_no_visible_key_in_a_later_piece_of_the_key_range(P, dh, hq, hkv):
    """Few query workgroups -> the key range is cut into pieces handled by separate workgroups.  A
    wavefront whose rows straddle a piece boundary then holds rows that see no key at all in the
    later piece; their partial result must be an exact zero weight, whatever the softmax scale."""
    model = ModelShape(1, 256, hq, hkv, dh, 704, 1e-5, 1e4, "bf16")
    announce("fully masked rows in a piece", dh, hq, hkv)
    n_tokens, n_rows, n_suffix = 702, 513, 12
    lw, h, pos, kc, vc = layer_case(model, n_tokens, n_rows, n_suffix, seed=5019)
    k = n_rows - n_suffix
    h_out, pos_out, dev, kg, vg = run_layer_both(P, model, lw, h, pos, kc, vc, n_suffix, k, want_dev=False)
    assert bool(torch.isfinite(h_out).all())
    h_ref, pos_ref, _, ko, vo = oracle_layer(model, lw, h, pos, kc, vc, n_suffix, k, None)
    assert max_abs_rel(to_np(h_out), h_ref) < TOL["bf16"]


def prefill_cases():
    rng = np.random.default_rng(77001)
    out = []
    names = ["f32", "bf16", "bf16_g7", "bf16_dh64"]
    for i in range(14):
        n_layers = int(rng.integers(2, 4))    # deeper stacks of these wide-weight test models leave the bf16 budget
        n_chunks = int(rng.integers(1, 10))
        lens = tuple(int(v) for v in rng.integers(1, 150, n_chunks))
        n_suffix = int(rng.integers(0, 34))
        fr = np.sort(rng.random(n_layers - 1))[::-1]
        if i % 4 == 1:
            fr[-1] = 0.0                                  # ends with nothing kept but the suffix
        if i % 4 == 2:
            fr[:] = fr[0]                                 # one selection, then no further check
        if i % 5 == 3:
            fr[0] = 1.0                                   # the first "check" keeps everything
        out.append((i, names[i % 4], n_layers, lens, n_suffix, tuple(float(v) for v in fr)))
    return out


@pytest.mark.parametrize("case", prefill_cases(), ids=lambda c: f"{c[0]}-{c[1]}-L{c[2]}-c{len(c[3])}-s{c[4]}")
def test_prefill_sweep(P, case):
    from dataclasses import replace
    from test_gpu_parity import MODELS, check_prefill_against_oracle, e2e_case, run_prefill
    i, name, n_layers, lens, n_suffix, fr = case
    if n_suffix == 0 and fr[-1] == 0.0:
        n_suffix = 1                                      # keep at least one row alive to the end
    model = replace(MODELS[name], n_layers=n_layers)
    announce("prefill sweep", case)
    w, layers, x, npl, xn, kpre, vpre = e2e_case(model, lens, n_suffix, seed=900 + i)
    keep = [w.n_ctx]
    for f in fr:
        keep.append(min(keep[-1], int(np.ceil(f * w.n_ctx))))
    out, kg, vg = run_prefill(P, w, layers, x, kpre, vpre, keep)
    check_prefill_against_oracle(w, npl, xn, kpre, vpre, keep, out, kg, vg, TOL[model.dtype])


def wide_cases():
    rng = np.random.default_rng(4242)
    geoms = [(1024, 8, 2, 128, 2048), (1024, 16, 2, 64, 4096), (1536, 12, 4, 128, 3072), (1024, 8, 1, 128, 2816),
             (2048, 16, 2, 128, 1024)]
    out = []
    for i in range(15):
        d, hq, hkv, dh, f = geoms[i % len(geoms)]
        n_rows = int(rng.choice([97, 200, 257, 390, 513, 700, 769, 1025, 1300]))
        n_suffix = int(rng.integers(0, 65))
        n_suffix = min(n_suffix, n_rows)
        n_cand = n_rows - n_suffix
        mode = i % 3
        k = n_cand if mode == 0 else int(n_cand * (0.93 if mode == 1 else 0.4))
        n_tokens = n_rows + int(rng.integers(0, 2500))
        out.append((i, d, hq, hkv, dh, f, n_tokens, n_rows, n_suffix, k))
    return out


@pytest.mark.parametrize("case", wide_cases(), ids=lambda c: f"{c[0]}-d{c[1]}-h{c[2]}/{c[3]}x{c[4]}-f{c[5]}-T{c[6]}-r{c[7]}-s{c[8]}-k{c[9]}")
def test_layer_sweep_wider_models(P, case):
    """Widths at which the big-tile GEMM variants, their K splits and shared tail tiles, and the
    different key-range splits of the attention kernel all come into play."""
    i, d, hq, hkv, dh, f, n_tokens, n_rows, n_suffix, k = case
    model = ModelShape(1, d, hq, hkv, dh, f, 1e-5, 1e4, "bf16")
    announce("wide sweep", case)
    lw, h, pos, kc, vc = layer_case(model, n_tokens, n_rows, n_suffix, seed=6000 + i, std=0.04)
    n_cand = n_rows - n_suffix
    check = k < n_cand
    h_out, pos_out, dev, kg, vg = run_layer_both(P, model, lw, h, pos, kc, vc, n_suffix, k, want_dev=check)
    tol = TOL["bf16"]
    forced = None
    if check:
        sel_pos = pos.numpy()[:n_cand][O.top_k_indices(dev.numpy(), k)]
        assert np.array_equal(pos_out.numpy()[:k], sel_pos)
        forced = sel_pos
    h_ref, pos_ref, dev_ref, ko, vo = oracle_layer(model, lw, h, pos, kc, vc, n_suffix, k, forced)
    assert np.array_equal(pos_out.numpy(), pos_ref)
    if check:
        assert max_abs_rel(dev.numpy(), dev_ref) < tol
    assert max_abs_rel(to_np(kg), ko) < tol and max_abs_rel(to_np(vg), vo) < tol
    untouched = np.setdiff1d(np.arange(n_tokens), pos_ref)
    assert torch.equal(kg[untouched], kc[untouched]) and torch.equal(vg[untouched], vc[untouched])
    assert max_abs_rel(to_np(h_out), h_ref) < tol
