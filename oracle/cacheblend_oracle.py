"""CPU oracle for CacheBlend's KV-cache fusing (arXiv 2405.16444).

TEST INFRASTRUCTURE ONLY.  Plain numpy in float64, no blocking, no fusion: every
function follows one passage of the paper and is meant to be checked against it
by eye.  Nothing here is shared with, imported by, or derived from the HIP
library; only tests, the smoke check and the bench's `cpu_baseline` leg may call
it.

What the paper fixes and where:
  * prefill = per-layer Q/K/V, masked softmax attention, further layers
    producing the next layer's input                              (Sec. 2)
  * pre-computed caches: each chunk prefilled alone as a prefix   (Sec. 4.1)
  * positional recovery of cached keys by one more rotation       (Sec. 4.3
    footnote, Appendix A definition of the rotary matrix)
  * selective recompute of one layer: reduce the input to the selected tokens,
    project Q/K/V for them, fill the other K/V rows from the cache, run the same
    attention, hand the selected rows to the next layer            (Sec. 4.2)
  * HKVD selection: keep the tokens with the largest KV deviation  (Sec. 4.3)
  * gradual filtering: candidates of a layer are the tokens kept on the layer
    before                                                   (Sec. 4.3, Fig. 9)
  * deviation measured between the newly computed and the loaded KV; only the
    kept tokens' KV is updated                                      (Sec. 6)

The decoder block itself (RMSNorm, GQA, SwiGLU, no biases) is the one the
workload configurations name; the paper treats it as a black box.

Readings this file takes where the paper is silent (each is also a row of the
design document): deviation = squared L2 distance over K and V of all kv heads,
K compared after the rotation; first informative selection is on layer 1
because layer-0 K/V depend on the token alone; selection happens right after the
K/V projection ("early filter"); ties go to the lower position; suffix (query)
tokens are always kept and never candidates.

Beyond the fusing path: the first-token head (final norm + vocabulary
projection + greedy pick of the last query token: what "time to first token"
ends with, Sec. 2) and the loading controller's delay estimators and choices
(Sec. 5.1 and its two footnotes).

Pinned by tests/test_oracle_*.py.  Unpinned readings: the deviation norm, the
early-filter order, the ratio schedule and the rounding of k (the paper gives
nothing to check them against) -- "parity unpinned" for those choices only.
"""
from __future__ import annotations

import math
from types import SimpleNamespace

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- #
# storage rounding
# --------------------------------------------------------------------------- #
def identity(a):
    return np.asarray(a, dtype=F64)


def round_bf16(a):
    """Round to the nearest bfloat16 (ties to even); result held in float64.

    bf16 = the upper 16 bits of an IEEE binary32, so rounding is done on the
    binary32 bit pattern (float64 -> float32 first, as a device would).
    """
    f = np.ascontiguousarray(np.asarray(a, dtype=np.float32))
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(F64).reshape(f.shape)


def dequantize_int8(lw):
    """Layer weights stored 8-bit (the paper serves its two larger models with 8-bit weights, Sec. 7.1,
    without naming a scheme; this build's reading is weight-only symmetric int8 with one scale per output
    feature -- "parity unpinned" by the paper): every matrix name that comes with a `<name>_scale` vector
    means w[o, i] = q[o, i] * scale[o].  Returns the layer with those matrices in float64; everything
    downstream is the ordinary definition of the block."""
    out = {}
    for name, v in lw.items():
        if name.endswith("_scale"):
            continue
        if name + "_scale" in lw:
            out[name] = np.asarray(v, F64) * np.asarray(lw[name + "_scale"], F64)[:, None]
        else:
            out[name] = np.asarray(v, F64)
    return out


def storage_round(dtype: str):
    return {"f32": identity, "bf16": round_bf16}[dtype]


# --------------------------------------------------------------------------- #
# decoder-block pieces
# --------------------------------------------------------------------------- #
def rms_norm(x, gain, eps):
    """x / sqrt(mean(x^2) + eps) * gain, row by row."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, F64)


def rope_frequencies(head_dim, theta):
    """theta_i = theta^(-2i/head_dim), i = 0 .. head_dim/2 - 1 (Appendix A)."""
    i = np.arange(head_dim // 2, dtype=F64)
    return theta ** (-2.0 * i / head_dim)


def rope(v, pos, theta, layout="adjacent"):
    """Apply the rotary matrix R_{Theta,pos} of Appendix A to every head.

    v [n, H, dh]; pos [n].  The matrix is block diagonal with 2x2 blocks acting
    on the adjacent pair (2i, 2i+1):
        [cos p*th_i  -sin p*th_i] [v_2i  ]
        [sin p*th_i   cos p*th_i] [v_2i+1]
    layout "half" is the same matrix with the channels of a head renumbered so
    that block i acts on the pair (i, i + dh/2) -- the order in which widely
    used checkpoints store their query/key projections.  The paper defines
    only the adjacent order; the other one is this renumbering and nothing else.
    """
    v = np.asarray(v, F64)
    n, _, dh = v.shape
    ang = np.asarray(pos, F64).reshape(n, 1, 1) * rope_frequencies(dh, theta).reshape(1, 1, -1)
    c, s = np.cos(ang), np.sin(ang)
    if layout == "adjacent":
        first, second = (slice(0, None, 2), slice(1, None, 2))
    elif layout == "half":
        first, second = (slice(0, dh // 2), slice(dh // 2, None))
    else:
        raise ValueError(f"unknown rotary layout {layout!r}")
    a, b = v[..., first], v[..., second]
    out = np.empty_like(v)
    out[..., first] = a * c - b * s
    out[..., second] = a * s + b * c
    return out


def rope_layout(m):
    """Channel order of the rotary pairs of a model description ("adjacent" unless it says otherwise)."""
    return getattr(m, "rope_layout", "adjacent")


def attention(q, q_pos, k_cache, v_cache):
    """Masked softmax attention of some query rows over a cache (Sec. 2).

    q [n, Hq, dh] with positions q_pos [n]; k_cache, v_cache [T, Hkv, dh] hold
    the key/value of position j in row j.  A query at position p sees keys
    j <= p.  Query head h reads kv head h // (Hq / Hkv).  Returns [n, Hq, dh].
    """
    q = np.asarray(q, F64)
    n, hq, dh = q.shape
    hkv = k_cache.shape[1]
    group = hq // hkv
    q_pos = np.asarray(q_pos, dtype=np.int64)
    out = np.zeros((n, hq, dh), F64)
    if n == 0:
        return out
    n_keys = int(q_pos.max()) + 1
    visible = np.arange(n_keys)[None, :] <= q_pos[:, None]          # [n, n_keys]
    for h in range(hq):
        kv = h // group
        scores = q[:, h, :] @ np.asarray(k_cache[:n_keys, kv, :], F64).T / math.sqrt(dh)
        scores = np.where(visible, scores, -np.inf)
        scores = scores - scores.max(axis=1, keepdims=True)
        p = np.exp(scores)
        p = p / p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ np.asarray(v_cache[:n_keys, kv, :], F64)
    return out


def silu(z):
    return z / (1.0 + np.exp(-z))


def finish_block(h_rows, attn_out, lw, m):
    """Everything after attention: output projection + residual, then the
    SwiGLU MLP + residual (the further per-layer networks of Sec. 2)."""
    n = h_rows.shape[0]
    h = h_rows + attn_out.reshape(n, m.n_q_heads * m.head_dim) @ lw["wo"].T
    y = rms_norm(h, lw["mlp_norm"], m.rms_eps)
    return h + (silu(y @ lw["w_gate"].T) * (y @ lw["w_up"].T)) @ lw["w_down"].T


def project_kv(h_rows, pos, lw, m):
    """K (rotated to `pos`) and V of some rows; also returns the normed input."""
    n = h_rows.shape[0]
    x = rms_norm(h_rows, lw["attn_norm"], m.rms_eps)
    k = rope((x @ lw["wk"].T).reshape(n, m.n_kv_heads, m.head_dim), pos, m.rope_theta, rope_layout(m))
    v = (x @ lw["wv"].T).reshape(n, m.n_kv_heads, m.head_dim)
    return x, k, v


def project_q(x_rows, pos, lw, m):
    n = x_rows.shape[0]
    return rope((x_rows @ lw["wq"].T).reshape(n, m.n_q_heads, m.head_dim), pos, m.rope_theta, rope_layout(m))


def as_f64_weights(lw):
    return {k: np.asarray(v, F64) for k, v in lw.items()}


# --------------------------------------------------------------------------- #
# full prefill (= full KV recompute) and the pre-computed chunk caches
# --------------------------------------------------------------------------- #
def full_prefill(x, layers, m, kv_round=identity, first_pos=0):
    """Plain causal prefill of the rows of x at positions first_pos, first_pos+1, ...

    Returns (K, V, H): per-layer caches [n, Hkv, dh] as stored (after kv_round)
    and the residual stream after the last layer [n, d].
    """
    h = np.asarray(x, F64)
    n = h.shape[0]
    pos = np.arange(first_pos, first_pos + n)
    ks, vs = [], []
    for lw in layers:
        lw = as_f64_weights(lw)
        xn, k, v = project_kv(h, pos, lw, m)
        k, v = kv_round(k), kv_round(v)
        q = project_q(xn, pos, lw, m)
        # keys are stored by row here, so query "positions" are row numbers
        o = attention(q, np.arange(n), k, v)
        h = finish_block(h, o, lw, m)
        ks.append(k)
        vs.append(v)
    return ks, vs, h


def chunk_prefill(x_ctx, chunk_lens, layers, m, kv_round=identity):
    """KV^pre: every chunk prefilled alone, as if it were a prefix (Sec. 4.1),
    i.e. at positions 0 .. len-1; per layer the chunks' caches are concatenated."""
    x_ctx = np.asarray(x_ctx, F64)
    per_layer_k = [[] for _ in layers]
    per_layer_v = [[] for _ in layers]
    o = 0
    for ln in chunk_lens:
        ks, vs, _ = full_prefill(x_ctx[o:o + ln], layers, m, kv_round)
        for l in range(len(layers)):
            per_layer_k[l].append(ks[l])
            per_layer_v[l].append(vs[l])
        o += ln
    return ([np.concatenate(a, axis=0) for a in per_layer_k],
            [np.concatenate(a, axis=0) for a in per_layer_v])


def chunk_offsets(chunk_lens):
    return np.concatenate([[0], np.cumsum(np.asarray(chunk_lens, dtype=np.int64))])


def realign_keys(k_pre, chunk_lens, m, kv_round=identity):
    """Positional recovery (Sec. 4.3 footnote): a key cached at local position t
    of chunk c already carries R(t); multiplying by R(o_c) moves it to o_c + t.
    Chunk 0 is left as it is.  V carries no position."""
    off = chunk_offsets(chunk_lens)
    out = np.array(k_pre, dtype=F64, copy=True)
    for c in range(1, len(chunk_lens)):
        a, b = off[c], off[c + 1]
        out[a:b] = kv_round(rope(out[a:b], np.full(b - a, off[c]), m.rope_theta, rope_layout(m)))
    return out


# --------------------------------------------------------------------------- #
# HKVD selection
# --------------------------------------------------------------------------- #
def kv_deviation(k_new, v_new, k_old, v_old):
    """Per-token deviation between two KV rows: sum of squared differences over
    every kv head and channel of K and of V (Sec. 4.1 defines it as a difference of the two;
    the norm is this build's reading)."""
    dk = np.asarray(k_new, F64) - np.asarray(k_old, F64)
    dv = np.asarray(v_new, F64) - np.asarray(v_old, F64)
    n = dk.shape[0]
    if n == 0:                      # no candidate left (numpy cannot infer the row length of an empty array)
        return np.zeros(0, F64)
    return (dk * dk).reshape(n, -1).sum(axis=1) + (dv * dv).reshape(n, -1).sum(axis=1)


def top_k_indices(dev, k):
    """Indices of the k largest entries, equal values resolved towards the
    smaller index, returned in ascending index order."""
    dev = np.asarray(dev)
    order = np.argsort(-dev, kind="stable")      # stable: ties keep index order
    return np.sort(order[:k]).astype(np.int64)


def default_schedule(n_layers, n_ctx, r, r1=None, kind="gradual"):
    """keep_counts[l] = number of context tokens kept on layer l.

    Layer 0 is full.  "flat": ceil(r*C) from layer 1 on (select once on the first
    informative layer, reuse everywhere -- the scheme Sec. 4.3 starts from).
    "gradual" (gradual filtering): the ratio falls from r1 on layer 1 to
    (3r - r1)/2 on the last layer along (1-t)^2, whose mean over layers is r.
    """
    if r1 is None:
        r1 = 2.0 * r
    keep = [int(n_ctx)]
    r_end = (3.0 * r - r1) / 2.0
    for l in range(1, n_layers):
        if kind == "flat":
            rl = r
        else:
            t = (l - 1) / max(1, n_layers - 2)
            rl = r_end + (r1 - r_end) * (1.0 - t) ** 2
        k = int(math.ceil(rl * n_ctx - 1e-9))
        keep.append(max(0, min(k, keep[-1])))
    return keep


# --------------------------------------------------------------------------- #
# one layer of selective recompute, and the whole fused prefill
# --------------------------------------------------------------------------- #
def fuse_layer(lw, m, h_rows, row_pos, n_suffix, k_cache, v_cache, k_keep,
               forced_sel=None, kv_round=identity):
    """Selective recompute of one layer (Sec. 4.2 workflow + Sec. 6 check step).

    h_rows [n, d]: this layer's input for the rows at ascending positions
    row_pos [n]; the last n_suffix rows are the suffix.  k_cache / v_cache
    [T, Hkv, dh] hold the re-aligned pre-computed rows and are updated in place.
    k_keep context rows survive.  forced_sel: context positions to keep instead
    of the top-k (parity protocol).
    Returns (h_next [k_keep + n_suffix, d], pos_next, dev or None, kept positions).
    """
    lw = as_f64_weights(lw)
    row_pos = np.asarray(row_pos, dtype=np.int64)
    n = h_rows.shape[0]
    n_cand = n - n_suffix
    assert 0 <= k_keep <= n_cand

    # K, V of every row that reached this layer
    xn, k_new, v_new = project_kv(np.asarray(h_rows, F64), row_pos, lw, m)
    k_new, v_new = kv_round(k_new), kv_round(v_new)

    # check step: deviation of the new KV from the loaded KV, keep the largest
    dev = None
    if k_keep < n_cand or forced_sel is not None:
        cand_pos = row_pos[:n_cand]
        dev = kv_deviation(k_new[:n_cand], v_new[:n_cand], k_cache[cand_pos], v_cache[cand_pos])
    if forced_sel is not None:
        kept_pos = np.asarray(forced_sel, dtype=np.int64)
        assert kept_pos.shape[0] == k_keep
        kept_rows = np.searchsorted(row_pos[:n_cand], kept_pos)
        assert np.array_equal(row_pos[kept_rows], kept_pos), "forced positions must be candidates"
    elif k_keep < n_cand:
        kept_rows = top_k_indices(dev, k_keep)
    else:
        kept_rows = np.arange(n_cand)
    rows = np.concatenate([kept_rows, np.arange(n_cand, n)]).astype(np.int64)
    pos_next = row_pos[rows]

    # only the kept tokens' KV is updated; everything else stays as loaded
    k_cache[pos_next] = k_new[rows]
    v_cache[pos_next] = v_new[rows]

    # attention of the kept rows over the whole (mixed) cache, rest of the block
    q = project_q(xn[rows], pos_next, lw, m)
    o = attention(q, pos_next, k_cache, v_cache)
    h_next = finish_block(np.asarray(h_rows, F64)[rows], o, lw, m)
    return h_next, pos_next, dev, pos_next[:k_keep].copy()


def fuse_prefill(x, layers, m, chunk_lens, n_suffix, k_pre, v_pre, keep_counts,
                 forced_sel=None, kv_round=identity):
    """Whole CacheBlend fusing pass.

    x [T, d] layer-0 input (context tokens then suffix); k_pre / v_pre: per layer
    [C, Hkv, dh] concatenated chunk caches, each chunk cached at positions 0.. .
    keep_counts[l]: context rows kept on layer l (keep_counts[0] == C).
    Returns a namespace: K, V (per layer [T, Hkv, dh] fused caches),
    final_hidden [n_suffix, d], dev (per layer array or None), sel (per layer
    kept context positions), rows (per layer number of rows that went through
    attention and MLP).
    """
    n_ctx = int(sum(chunk_lens))
    n_tok = n_ctx + n_suffix
    x = np.asarray(x, F64)
    assert x.shape[0] == n_tok and keep_counts[0] == n_ctx
    h, pos = x, np.arange(n_tok)
    out = SimpleNamespace(K=[], V=[], dev=[], sel=[], rows=[])
    for l, lw in enumerate(layers):
        k_cache = np.zeros((n_tok, m.n_kv_heads, m.head_dim), F64)
        v_cache = np.zeros_like(k_cache)
        k_cache[:n_ctx] = realign_keys(k_pre[l], chunk_lens, m, kv_round)
        v_cache[:n_ctx] = np.asarray(v_pre[l], F64)
        force = None if forced_sel is None else forced_sel[l]
        h, pos, dev, sel = fuse_layer(lw, m, h, pos, n_suffix, k_cache, v_cache,
                                      int(keep_counts[l]), force, kv_round)
        out.K.append(k_cache)
        out.V.append(v_cache)
        out.dev.append(dev)
        out.sel.append(sel)
        out.rows.append(len(pos))
    out.final_hidden = h[len(pos) - n_suffix:]
    return out


# --------------------------------------------------------------------------- #
# first token (Sec. 2: the prefill phase ends when the first token is generated)
# --------------------------------------------------------------------------- #
def first_token(final_hidden, norm_gain, lm_head, eps):
    """Logits of the token that follows the last query token, and the greedy pick.

    final_hidden [n_suffix, d] residual stream after the last layer; norm_gain
    [d]; lm_head [vocab, d].  Returns (logits [vocab], token) with token the
    smallest index among the largest logits.
    """
    x = rms_norm(np.asarray(final_hidden, F64)[-1], norm_gain, eps)
    logits = np.asarray(lm_head, F64) @ x
    return logits, arg_max_first(logits)


def arg_max_first(values):
    """Index of the largest entry; equal entries resolved towards the smaller index."""
    values = np.asarray(values)
    best = 0
    for i in range(1, values.shape[0]):
        if values[i] > values[best]:
            best = i
    return best


# --------------------------------------------------------------------------- #
# loading controller (Sec. 5.1)
# --------------------------------------------------------------------------- #
def recompute_delay(ratio, prefill_delay):
    """T_recompute(r, LLM, L) = r x Prefill(LLM, L)  (first footnote of Sec. 5.1);
    prefill_delay is the profiled full-prefill delay in the caller's unit."""
    return ratio * prefill_delay


def load_delay(per_token_kv_bytes, n_tokens, throughput_bytes_per_s):
    """T_load(LLM, L, device) = PerTokenKVSize(LLM) x L / Throughput(device), seconds
    (second footnote of Sec. 5.1).  per_token_kv_bytes is for whatever unit of the
    cache is loaded (one layer for the layer-by-layer pipeline)."""
    return per_token_kv_bytes * n_tokens / throughput_bytes_per_s


def pick_recompute_ratio(prefill_delay, loading_delay, min_ratio=0.15):
    """The ratio at which recompute takes as long as loading, but never below the
    minimal ratio that keeps quality (r* = 15 % in the paper) nor above 1."""
    r_equal = loading_delay / prefill_delay
    return min(1.0, max(min_ratio, r_equal))


def pick_storage_device(recompute_delay_value, load_delays, costs):
    """Index of the cheapest device whose loading delay the recompute delay hides
    (T_recompute >= T_load); ties in cost go to the lower index; -1 if none."""
    best = -1
    for i, (t, c) in enumerate(zip(load_delays, costs)):
        if t <= recompute_delay_value and (best < 0 or c < costs[best]):
            best = i
    return best


# --------------------------------------------------------------------------- #
# diagnostics (Sec. 4.1 definitions, Sec. 4.3 insight 2); analysis only
# --------------------------------------------------------------------------- #
def forward_attention_matrix(q, q_pos, k_cache):
    """A [Hq, n, n_keys]: softmax of the masked scaled scores of the query rows (the "forward
    attention matrix" of Sec. 4.1), n_keys = largest query position + 1."""
    q = np.asarray(q, F64)
    n, hq, dh = q.shape
    group = hq // k_cache.shape[1]
    q_pos = np.asarray(q_pos, dtype=np.int64)
    n_keys = int(q_pos.max()) + 1
    visible = np.arange(n_keys)[None, :] <= q_pos[:, None]
    out = np.zeros((hq, n, n_keys), F64)
    for h in range(hq):
        sc = q[:, h, :] @ np.asarray(k_cache[:n_keys, h // group, :], F64).T / math.sqrt(dh)
        sc = np.where(visible, sc, -np.inf)
        sc = np.exp(sc - sc.max(axis=1, keepdims=True))
        out[h] = sc / sc.sum(axis=1, keepdims=True)
    return out


def attention_deviation(a, a_full):
    """Delta_attn(A, A_full): the L2 norm of the difference of two forward attention matrices
    (Sec. 4.1)."""
    d = np.asarray(a, F64) - np.asarray(a_full, F64)
    return float(np.sqrt(np.sum(d * d)))


def spearman_rank_correlation(x, y):
    """Spearman's rank correlation of two score vectors (Sec. 4.3 uses it between the KV
    deviations of the same tokens on neighbouring layers): Pearson correlation of the ranks,
    equal values sharing the mean of their ranks."""
    def ranks(v):
        v = np.asarray(v, F64)
        order = np.argsort(v, kind="stable")
        r = np.empty(len(v), F64)
        i = 0
        while i < len(v):
            j = i
            while j + 1 < len(v) and v[order[j + 1]] == v[order[i]]:
                j += 1
            r[order[i:j + 1]] = 0.5 * (i + j) + 1.0
            i = j + 1
        return r
    rx, ry = ranks(x), ranks(y)
    rx, ry = rx - rx.mean(), ry - ry.mean()
    return float(np.sum(rx * ry) / math.sqrt(np.sum(rx * rx) * np.sum(ry * ry)))
