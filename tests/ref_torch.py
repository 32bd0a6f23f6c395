"""Independent re-statement of a Llama-style decoder with torch *library* ops
(F.linear, F.rms_norm, F.silu, F.scaled_dot_product_attention, complex
multiplication for the rotary embedding).  Used only to pin the oracle: it shares
no code with oracle/ and takes a different route to every quantity."""
import torch
import torch.nn.functional as F


def rope_complex(v, pos, theta):
    """Rotate adjacent pairs by multiplying (v_2i + i v_2i+1) with exp(i p th_i)."""
    n, h, dh = v.shape
    freqs = theta ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    ang = pos.to(torch.float64)[:, None] * freqs[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    vc = torch.view_as_complex(v.reshape(n, h, dh // 2, 2).contiguous())
    return torch.view_as_real(vc * rot).reshape(n, h, dh)


def rope_rotate_half(v, pos, theta):
    """The other common statement of the rotary embedding: x * cos + swap(x) * sin, with
    swap(x) = concat(-second half, first half) and the dh/2 angles repeated for both halves."""
    n, h, dh = v.shape
    freqs = theta ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    ang = pos.to(torch.float64)[:, None] * freqs[None, :]
    ang = torch.cat([ang, ang], dim=-1)[:, None, :]
    swapped = torch.cat([-v[..., dh // 2:], v[..., :dh // 2]], dim=-1)
    return v * torch.cos(ang) + swapped * torch.sin(ang)


def layer_forward(h, lw, m, pos):
    n = h.shape[0]
    x = F.rms_norm(h, (m.d_model,), lw["attn_norm"], m.rms_eps)
    q = rope_complex(F.linear(x, lw["wq"]).view(n, m.n_q_heads, m.head_dim), pos, m.rope_theta)
    k = rope_complex(F.linear(x, lw["wk"]).view(n, m.n_kv_heads, m.head_dim), pos, m.rope_theta)
    v = F.linear(x, lw["wv"]).view(n, m.n_kv_heads, m.head_dim)
    g = m.n_q_heads // m.n_kv_heads
    kk = k.repeat_interleave(g, dim=1).transpose(0, 1)
    vv = v.repeat_interleave(g, dim=1).transpose(0, 1)
    o = F.scaled_dot_product_attention(q.transpose(0, 1), kk, vv, is_causal=True)
    o = o.transpose(0, 1).reshape(n, -1)
    h = h + F.linear(o, lw["wo"])
    y = F.rms_norm(h, (m.d_model,), lw["mlp_norm"], m.rms_eps)
    h = h + F.linear(F.silu(F.linear(y, lw["w_gate"])) * F.linear(y, lw["w_up"]), lw["w_down"])
    return h, k, v


def full_prefill(x, layers, m, first_pos=0):
    h = x.to(torch.float64)
    pos = torch.arange(first_pos, first_pos + h.shape[0])
    ks, vs = [], []
    for lw in layers:
        lw = {k_: v_.to(torch.float64) for k_, v_ in lw.items()}
        h, k, v = layer_forward(h, lw, m, pos)
        ks.append(k)
        vs.append(v)
    return ks, vs, h
