"""ctypes binding of libcacheblend.so: same entry-point names as include/cacheblend.h,
argument marshalling only.  torch supplies device memory and the stream handle; every
step of the path runs in the library's HIP kernels.  There is no fallback: a missing
library is an ImportError."""
from __future__ import annotations

import ctypes as C
import os
from types import SimpleNamespace
from typing import Dict, List, Optional, Sequence

import torch  # imported before the library so both share one HIP runtime

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcacheblend.so")

CB_F32, CB_BF16 = 0, 1
PROF_CLASSES = ("gemm", "attention", "realign", "deviation", "topk", "norm", "other", "finish",
                "first_token", "phase_first_layer", "phase_selective_layers")


class CacheBlendError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {_lib.cb_strerror(status).decode()} ({status})")


class _ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ff", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32),
                ("rope_layout", C.c_int32), ("weight_format", C.c_int32)]


_ROPE_LAYOUTS = {"adjacent": 0, "half": 1}
_WEIGHT_FORMATS = {"native": 0, "int8": 1}


_WEIGHT_FIELDS = ("attn_norm", "wq", "wk", "wv", "wo", "mlp_norm", "w_gate", "w_up", "w_down")
_MATRIX_FIELDS = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")
_SCALE_FIELDS = tuple(n + "_scale" for n in _MATRIX_FIELDS)


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WEIGHT_FIELDS + _SCALE_FIELDS]


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2405_16444_amd.build` "
            "(there is no non-HIP fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t
    lib.cb_strerror.restype = C.c_char_p
    lib.cb_strerror.argtypes = [C.c_int]
    lib.cb_create.argtypes = [C.POINTER(_ModelDesc), i32, C.POINTER(vp)]
    lib.cb_destroy.argtypes = [vp]
    lib.cb_destroy.restype = None
    lib.cb_layer_workspace_bytes.argtypes = [vp, i32]
    lib.cb_layer_workspace_bytes.restype = sz
    lib.cb_prefill_workspace_bytes.argtypes = [vp, i32]
    lib.cb_prefill_workspace_bytes.restype = sz
    lib.cb_default_schedule.argtypes = [i32, i32, C.c_double, C.c_double, i32, C.POINTER(i32)]
    lib.cb_realign_rope.argtypes = [vp, C.POINTER(vp), i32, i32, C.POINTER(i32), i32, vp]
    lib.cb_fuse_layer.argtypes = [vp, i32, C.POINTER(_LayerWeights), vp, vp, i32, i32, vp, vp, i32, i32,
                                  vp, vp, vp, vp, vp, sz, vp]
    lib.cb_static_scratch_bytes.argtypes = []
    lib.cb_static_scratch_bytes.restype = sz
    lib.cb_fuse_layer_static.argtypes = [vp, i32, C.POINTER(_LayerWeights), vp, vp, i32, i32, vp, vp, i32, i32,
                                         vp, vp, vp, vp, vp]
    lib.cb_fuse_prefill.argtypes = [vp, C.POINTER(_LayerWeights), vp, C.POINTER(i32), i32, i32,
                                    C.POINTER(vp), C.POINTER(vp), C.POINTER(i32), C.POINTER(vp), vp,
                                    C.POINTER(vp), C.POINTER(vp), vp, sz, vp]
    lib.cb_fuse_prefill_pipelined.argtypes = [vp, C.POINTER(_LayerWeights), vp, C.POINTER(i32), i32, i32,
                                              C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                              C.POINTER(i32), vp, vp, sz, vp, vp]
    lib.cb_batched_workspace_bytes.argtypes = [vp, i32]
    lib.cb_batched_workspace_bytes.restype = sz
    lib.cb_fuse_prefill_batched.argtypes = [vp, C.POINTER(_LayerWeights), i32, vp, C.POINTER(i32), C.POINTER(i32),
                                            C.POINTER(i32), C.POINTER(vp), C.POINTER(vp), i32, C.POINTER(i32),
                                            vp, C.POINTER(vp), C.POINTER(vp), vp, sz, vp]
    lib.cb_first_token.argtypes = [vp, vp, i32, vp, vp, i32, vp, vp, vp]
    dbl = C.c_double
    lib.cb_recompute_delay.argtypes = [dbl, dbl]
    lib.cb_recompute_delay.restype = dbl
    lib.cb_load_delay.argtypes = [dbl, dbl, dbl]
    lib.cb_load_delay.restype = dbl
    lib.cb_pick_recompute_ratio.argtypes = [dbl, dbl, dbl]
    lib.cb_pick_recompute_ratio.restype = dbl
    lib.cb_pick_storage_device.argtypes = [dbl, C.POINTER(dbl), C.POINTER(dbl), i32]
    lib.cb_pick_storage_device.restype = i32
    lib.cb_profile_enable.argtypes = [vp, i32]
    lib.cb_profile_read.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_int64),
                                    C.POINTER(C.c_double), C.POINTER(C.c_double)]
    return lib


_lib = _load()
EXPORTS = ("cb_create", "cb_destroy", "cb_strerror", "cb_layer_workspace_bytes",
           "cb_prefill_workspace_bytes", "cb_default_schedule", "cb_realign_rope", "cb_fuse_layer",
           "cb_static_scratch_bytes", "cb_fuse_layer_static", "cb_fuse_prefill", "cb_fuse_prefill_pipelined", "cb_batched_workspace_bytes",
           "cb_fuse_prefill_batched", "cb_first_token", "cb_recompute_delay", "cb_load_delay",
           "cb_pick_recompute_ratio", "cb_pick_storage_device", "cb_profile_enable", "cb_profile_read")


def _check(status: int, where: str):
    if status != 0:
        raise CacheBlendError(status, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _dtype_code(model) -> int:
    return {"f32": CB_F32, "bf16": CB_BF16}[model.dtype]


def _torch_dtype(code: int):
    return torch.float32 if code == CB_F32 else torch.bfloat16


def _weights_struct(lw: Dict[str, torch.Tensor], dtype, device) -> _LayerWeights:
    """Pointers of one layer.  Matrices are of `dtype`, or int8 with a float `<name>_scale` vector each."""
    s = _LayerWeights()
    for name in _WEIGHT_FIELDS:
        t = lw[name]
        assert t.is_contiguous() and t.device == device, name
        if t.dtype == torch.int8:
            sc = lw[name + "_scale"]
            assert name in _MATRIX_FIELDS and sc.dtype == torch.float32 and sc.is_contiguous(), name
            assert sc.device == device and sc.numel() == t.shape[0], name
            setattr(s, name + "_scale", sc.data_ptr())
        else:
            assert t.dtype == dtype, name
        setattr(s, name, t.data_ptr())
    return s


def _i32_array(values: Sequence[int]):
    return (C.c_int32 * len(values))(*[int(v) for v in values])


def _ptr_array(tensors: Sequence[Optional[torch.Tensor]]):
    return (C.c_void_p * len(tensors))(*[None if t is None else t.data_ptr() for t in tensors])


class Context:
    """Owns a cb_ctx (rotary table on the current device)."""

    def __init__(self, model, max_tokens: int):
        self.model = model
        self.max_tokens = int(max_tokens)
        self.dtype_code = _dtype_code(model)
        self.dtype = _torch_dtype(self.dtype_code)
        desc = _ModelDesc(model.n_layers, model.d_model, model.n_q_heads, model.n_kv_heads,
                          model.head_dim, model.d_ff, model.rms_eps, model.rope_theta, self.dtype_code,
                          _ROPE_LAYOUTS[getattr(model, "rope_layout", "adjacent")],
                          _WEIGHT_FORMATS[getattr(model, "weight_format", "native")])
        self.int8_weights = getattr(model, "weight_format", "native") == "int8"
        handle = C.c_void_p()
        _check(_lib.cb_create(C.byref(desc), self.max_tokens, C.byref(handle)), "cb_create")
        self._h = handle
        self.device = torch.device("cuda", torch.cuda.current_device())

    def close(self):
        # at interpreter shutdown the module globals may already be gone; the process is ending anyway
        if getattr(self, "_h", None) and _lib is not None:
            _lib.cb_destroy(self._h)
            self._h = None

    __del__ = close


def cb_create(model, max_tokens: int) -> Context:
    return Context(model, max_tokens)


def cb_destroy(ctx: Context):
    ctx.close()


def cb_strerror(status: int) -> str:
    return _lib.cb_strerror(status).decode()


def cb_layer_workspace_bytes(ctx: Context, max_rows: int) -> int:
    return int(_lib.cb_layer_workspace_bytes(ctx._h, max_rows))


def cb_prefill_workspace_bytes(ctx: Context, n_tokens: int) -> int:
    return int(_lib.cb_prefill_workspace_bytes(ctx._h, n_tokens))


def cb_default_schedule(n_layers: int, n_ctx: int, r: float, r1: float = 0.0, flat: bool = False) -> List[int]:
    out = (C.c_int32 * n_layers)()
    _check(_lib.cb_default_schedule(n_layers, n_ctx, r, r1, int(flat), out), "cb_default_schedule")
    return list(out)


def cb_realign_rope(ctx: Context, k_cache_layers: Sequence[torch.Tensor], layer_begin: int, layer_end: int,
                    chunk_offsets: Sequence[int], stream=None):
    for t in k_cache_layers:
        assert t.dtype == ctx.dtype and t.is_contiguous()
    _check(_lib.cb_realign_rope(ctx._h, _ptr_array(k_cache_layers), layer_begin, layer_end,
                                _i32_array(chunk_offsets), len(chunk_offsets) - 1, _stream(stream)),
           "cb_realign_rope")


def cb_fuse_layer(ctx: Context, layer: int, weights: Dict[str, torch.Tensor], h_in: torch.Tensor,
                  row_pos: torch.Tensor, n_suffix: int, k_cache: torch.Tensor, v_cache: torch.Tensor,
                  k_keep: int, forced_sel: Optional[torch.Tensor] = None, want_dev: bool = False,
                  workspace: Optional[torch.Tensor] = None, stream=None):
    """Returns (h_out, pos_out, dev or None).  k_cache / v_cache are updated in place."""
    dev_ = ctx.device
    n_rows = h_in.shape[0]
    assert h_in.dtype == torch.float32 and h_in.is_contiguous() and h_in.shape[1] == ctx.model.d_model
    assert row_pos.dtype == torch.int32 and row_pos.shape == (n_rows,) and row_pos.is_contiguous()
    assert k_cache.dtype == ctx.dtype and v_cache.dtype == ctx.dtype
    assert k_cache.is_contiguous() and v_cache.is_contiguous() and k_cache.shape == v_cache.shape
    if forced_sel is not None:
        assert forced_sel.dtype == torch.int32 and forced_sel.numel() == k_keep and forced_sel.is_contiguous()
    n_out = k_keep + n_suffix
    # at least one row is allocated so that the pointers are never NULL
    h_out = torch.empty((max(1, n_out), ctx.model.d_model), dtype=torch.float32, device=dev_)
    pos_out = torch.empty((max(1, n_out),), dtype=torch.int32, device=dev_)
    dev = torch.zeros((n_rows - n_suffix,), dtype=torch.float32, device=dev_) if want_dev else None
    if workspace is None:
        workspace = torch.empty(max(1, cb_layer_workspace_bytes(ctx, max(1, n_rows))), dtype=torch.uint8,
                                device=dev_)
    w = _weights_struct(weights, ctx.dtype, dev_)
    _check(_lib.cb_fuse_layer(ctx._h, layer, C.byref(w), _ptr(h_in), _ptr(row_pos), n_rows, n_suffix,
                              _ptr(k_cache), _ptr(v_cache), k_cache.shape[0], k_keep, _ptr(forced_sel),
                              _ptr(h_out), _ptr(pos_out), _ptr(dev), _ptr(workspace), workspace.numel(),
                              _stream(stream)), "cb_fuse_layer")
    return h_out[:n_out], pos_out[:n_out], dev


def cb_static_scratch_bytes() -> int:
    return int(_lib.cb_static_scratch_bytes())


def cb_fuse_layer_static(ctx: Context, layer: int, weights: Dict[str, torch.Tensor], h_in: torch.Tensor,
                         row_pos: torch.Tensor, n_suffix: int, k_cache: torch.Tensor, v_cache: torch.Tensor,
                         k_keep: int, h_out: torch.Tensor, pos_out: torch.Tensor,
                         forced_sel: Optional[torch.Tensor] = None, dev: Optional[torch.Tensor] = None,
                         stream=None):
    """cb_fuse_layer on the library's built-in scratch array.  The caller passes every output
    (h_out float [>= k_keep + n_suffix, d], pos_out int32, dev float [n_rows - n_suffix] or None):
    nothing is allocated here or in the library."""
    n_rows = h_in.shape[0]
    n_out = k_keep + n_suffix
    assert h_in.dtype == torch.float32 and h_in.is_contiguous() and h_in.shape[1] == ctx.model.d_model
    assert row_pos.dtype == torch.int32 and row_pos.shape == (n_rows,) and row_pos.is_contiguous()
    assert k_cache.dtype == ctx.dtype and v_cache.dtype == ctx.dtype
    assert k_cache.is_contiguous() and v_cache.is_contiguous() and k_cache.shape == v_cache.shape
    assert h_out.dtype == torch.float32 and h_out.is_contiguous() and h_out.shape[0] >= n_out
    assert h_out.shape[1] == ctx.model.d_model
    assert pos_out.dtype == torch.int32 and pos_out.is_contiguous() and pos_out.numel() >= n_out
    if forced_sel is not None:
        assert forced_sel.dtype == torch.int32 and forced_sel.numel() == k_keep and forced_sel.is_contiguous()
    if dev is not None:
        assert dev.dtype == torch.float32 and dev.is_contiguous() and dev.numel() >= n_rows - n_suffix
    w = _weights_struct(weights, ctx.dtype, ctx.device)
    _check(_lib.cb_fuse_layer_static(ctx._h, layer, C.byref(w), _ptr(h_in), _ptr(row_pos), n_rows, n_suffix,
                                     _ptr(k_cache), _ptr(v_cache), k_cache.shape[0], k_keep, _ptr(forced_sel),
                                     _ptr(h_out), _ptr(pos_out), _ptr(dev), _stream(stream)),
           "cb_fuse_layer_static")
    return h_out[:n_out], pos_out[:n_out], dev


def cb_fuse_prefill(ctx: Context, layers: Sequence[Dict[str, torch.Tensor]], x: torch.Tensor,
                    chunk_lens: Sequence[int], n_suffix: int, k_cache_layers: Sequence[torch.Tensor],
                    v_cache_layers: Sequence[torch.Tensor], keep_counts: Sequence[int],
                    forced_sel: Optional[Sequence[Optional[torch.Tensor]]] = None, want_sel: bool = False,
                    want_dev: bool = False, workspace: Optional[torch.Tensor] = None, stream=None,
                    weight_structs=None, out: Optional[SimpleNamespace] = None):
    """Returns a namespace with final_hidden and (optionally) per-layer sel / dev tensors.
    The caches are fused in place.  `weight_structs` / `out` let a benchmark reuse the
    marshalled arguments and output buffers across calls."""
    dev_ = ctx.device
    L, d = ctx.model.n_layers, ctx.model.d_model
    n_ctx = int(sum(chunk_lens))
    T = n_ctx + n_suffix
    assert len(layers) == L and len(k_cache_layers) == L and len(v_cache_layers) == L and len(keep_counts) == L
    assert x.dtype == ctx.dtype and x.shape == (T, d) and x.is_contiguous()
    for t in list(k_cache_layers) + list(v_cache_layers):
        assert t.dtype == ctx.dtype and t.is_contiguous() and t.shape[0] == T
    if weight_structs is None:
        weight_structs = (_LayerWeights * L)(*[_weights_struct(lw, ctx.dtype, dev_) for lw in layers])
    if out is None:
        out = SimpleNamespace()
        out._final_buf = torch.empty((max(1, n_suffix), d), dtype=torch.float32, device=dev_)
        out.final_hidden = out._final_buf[:n_suffix]
        out.sel = out.dev = None
        if want_sel:
            out._sel_buf = [torch.empty((max(1, int(k)),), dtype=torch.int32, device=dev_) for k in keep_counts]
            out.sel = [b[:int(k)] for b, k in zip(out._sel_buf, keep_counts)]
        if want_dev:
            cand = [n_ctx] + [int(k) for k in keep_counts[:-1]]
            out._dev_buf = [torch.zeros((max(1, c),), dtype=torch.float32, device=dev_) for c in cand]
            out.dev = [b[:c] for b, c in zip(out._dev_buf, cand)]
    if workspace is None:
        workspace = torch.empty(cb_prefill_workspace_bytes(ctx, T), dtype=torch.uint8, device=dev_)
    forced_arr = None
    if forced_sel is not None:
        for l, f in enumerate(forced_sel):
            assert f is None or (f.dtype == torch.int32 and f.numel() == keep_counts[l] and f.is_contiguous())
        forced_arr = _ptr_array(forced_sel)
    sel_arr = _ptr_array(out._sel_buf) if out.sel is not None else None
    dev_arr = _ptr_array(out._dev_buf) if out.dev is not None else None
    _check(_lib.cb_fuse_prefill(ctx._h, weight_structs, _ptr(x), _i32_array(chunk_lens), len(chunk_lens),
                                n_suffix, _ptr_array(k_cache_layers), _ptr_array(v_cache_layers),
                                _i32_array(keep_counts), forced_arr, _ptr(out._final_buf), sel_arr,
                                dev_arr, _ptr(workspace), workspace.numel(), _stream(stream)),
           "cb_fuse_prefill")
    out.workspace = workspace
    out.weight_structs = weight_structs
    return out


def cb_fuse_prefill_pipelined(ctx: Context, layers: Sequence[Dict[str, torch.Tensor]], x: torch.Tensor,
                              chunk_lens: Sequence[int], n_suffix: int, k_host_layers: Sequence[torch.Tensor],
                              v_host_layers: Sequence[torch.Tensor], k_cache_layers: Sequence[torch.Tensor],
                              v_cache_layers: Sequence[torch.Tensor], keep_counts: Sequence[int], copy_stream,
                              workspace: Optional[torch.Tensor] = None, stream=None, weight_structs=None,
                              out: Optional[SimpleNamespace] = None):
    """cb_fuse_prefill with the pre-computed caches in (pinned) host tensors [n_ctx, Hkv, dh];
    copy_stream: a torch.cuda.Stream of default priority, different from `stream`."""
    dev_ = ctx.device
    L, d = ctx.model.n_layers, ctx.model.d_model
    n_ctx = int(sum(chunk_lens))
    T = n_ctx + n_suffix
    assert len(layers) == L and len(k_cache_layers) == L and len(v_cache_layers) == L and len(keep_counts) == L
    assert len(k_host_layers) == L and len(v_host_layers) == L
    assert x.dtype == ctx.dtype and x.shape == (T, d) and x.is_contiguous()
    for t in list(k_cache_layers) + list(v_cache_layers):
        assert t.dtype == ctx.dtype and t.is_contiguous() and t.shape[0] == T and t.is_cuda
    for t in list(k_host_layers) + list(v_host_layers):
        assert t.dtype == ctx.dtype and t.is_contiguous() and t.shape[0] == n_ctx and not t.is_cuda
    if weight_structs is None:
        weight_structs = (_LayerWeights * L)(*[_weights_struct(lw, ctx.dtype, dev_) for lw in layers])
    if out is None:
        out = SimpleNamespace()
        out._final_buf = torch.empty((max(1, n_suffix), d), dtype=torch.float32, device=dev_)
        out.final_hidden = out._final_buf[:n_suffix]
    if workspace is None:
        workspace = torch.empty(cb_prefill_workspace_bytes(ctx, T), dtype=torch.uint8, device=dev_)
    _check(_lib.cb_fuse_prefill_pipelined(
        ctx._h, weight_structs, _ptr(x), _i32_array(chunk_lens), len(chunk_lens), n_suffix,
        _ptr_array(k_host_layers), _ptr_array(v_host_layers), _ptr_array(k_cache_layers),
        _ptr_array(v_cache_layers), _i32_array(keep_counts), _ptr(out._final_buf), _ptr(workspace),
        workspace.numel(), _stream(stream), _stream(copy_stream)), "cb_fuse_prefill_pipelined")
    out.workspace = workspace
    out.weight_structs = weight_structs
    return out


def cb_batched_workspace_bytes(ctx: Context, total_tokens: int) -> int:
    return int(_lib.cb_batched_workspace_bytes(ctx._h, total_tokens))


def cb_fuse_prefill_batched(ctx: Context, layers: Sequence[Dict[str, torch.Tensor]], x: torch.Tensor,
                            chunk_lens: Sequence[Sequence[int]], n_suffix: Sequence[int],
                            k_cache_layers: Sequence[torch.Tensor], v_cache_layers: Sequence[torch.Tensor],
                            cache_stride: int, keep_counts: Sequence[Sequence[int]], want_sel: bool = False,
                            want_dev: bool = False, workspace: Optional[torch.Tensor] = None, stream=None,
                            weight_structs=None, out: Optional[SimpleNamespace] = None):
    """Several requests stacked in one call.  chunk_lens / n_suffix / keep_counts: one entry per
    request; caches: per layer one tensor [n_requests * cache_stride, Hkv, dh].  Returns a namespace
    with final_hidden [sum n_suffix, d], sel[b][l] and dev[l] (when asked for)."""
    dev_ = ctx.device
    B, L, d = len(chunk_lens), ctx.model.n_layers, ctx.model.d_model
    T = [int(sum(cl)) + int(s) for cl, s in zip(chunk_lens, n_suffix)]
    N, S_tot = sum(T), int(sum(n_suffix))
    assert len(n_suffix) == B and len(keep_counts) == B and all(len(k) == L for k in keep_counts)
    assert len(layers) == L and len(k_cache_layers) == L and len(v_cache_layers) == L
    assert x.dtype == ctx.dtype and x.shape == (N, d) and x.is_contiguous()
    for t in list(k_cache_layers) + list(v_cache_layers):
        assert t.dtype == ctx.dtype and t.is_contiguous() and t.shape[0] == B * cache_stride
    if weight_structs is None:
        weight_structs = (_LayerWeights * L)(*[_weights_struct(lw, ctx.dtype, dev_) for lw in layers])
    if out is None:
        out = SimpleNamespace()
        out._final_buf = torch.empty((max(1, S_tot), d), dtype=torch.float32, device=dev_)
        out.final_hidden = out._final_buf[:S_tot]
        out.sel = out.dev = None
        if want_sel:
            out._sel_buf = [torch.empty((max(1, int(k)),), dtype=torch.int32, device=dev_)
                            for kc in keep_counts for k in kc]
            out.sel = [[out._sel_buf[b * L + l][:int(keep_counts[b][l])] for l in range(L)] for b in range(B)]
        if want_dev:
            rows_in = [N] + [sum(int(keep_counts[b][l]) + int(n_suffix[b]) for b in range(B)) for l in range(L - 1)]
            out._dev_buf = [torch.zeros((max(1, r),), dtype=torch.float32, device=dev_) for r in rows_in]
            out.dev = [b_[:r] for b_, r in zip(out._dev_buf, rows_in)]
    if workspace is None:
        workspace = torch.empty(cb_batched_workspace_bytes(ctx, N), dtype=torch.uint8, device=dev_)
    flat_chunks = [int(v) for cl in chunk_lens for v in cl]
    flat_keep = [int(v) for kc in keep_counts for v in kc]
    sel_arr = _ptr_array(out._sel_buf) if out.sel is not None else None
    dev_arr = _ptr_array(out._dev_buf) if out.dev is not None else None
    _check(_lib.cb_fuse_prefill_batched(
        ctx._h, weight_structs, B, _ptr(x), _i32_array(flat_chunks), _i32_array([len(cl) for cl in chunk_lens]),
        _i32_array(n_suffix), _ptr_array(k_cache_layers), _ptr_array(v_cache_layers), cache_stride,
        _i32_array(flat_keep), _ptr(out._final_buf), sel_arr, dev_arr, _ptr(workspace), workspace.numel(),
        _stream(stream)), "cb_fuse_prefill_batched")
    out.workspace = workspace
    out.weight_structs = weight_structs
    return out


def cb_first_token(ctx: Context, final_hidden: torch.Tensor, final_norm: torch.Tensor, lm_head: torch.Tensor,
                   stream=None, logits: Optional[torch.Tensor] = None, token: Optional[torch.Tensor] = None):
    """(logits float [vocab], token int32 [1]) for the last row of final_hidden."""
    n_suffix, vocab = final_hidden.shape[0], lm_head.shape[0]
    dev = final_hidden.device
    if logits is None:
        logits = torch.empty(vocab, dtype=torch.float32, device=dev)
    if token is None:
        token = torch.empty(1, dtype=torch.int32, device=dev)
    _check(_lib.cb_first_token(ctx._h, _ptr(final_hidden), n_suffix, _ptr(final_norm), _ptr(lm_head), vocab,
                               _ptr(logits), _ptr(token), _stream(stream)), "cb_first_token")
    return logits, token


def cb_recompute_delay(ratio: float, prefill_delay: float) -> float:
    return _lib.cb_recompute_delay(ratio, prefill_delay)


def cb_load_delay(per_token_kv_bytes: float, n_tokens: float, throughput_bytes_per_s: float) -> float:
    return _lib.cb_load_delay(per_token_kv_bytes, n_tokens, throughput_bytes_per_s)


def cb_pick_recompute_ratio(prefill_delay: float, load_delay: float, min_ratio: float = 0.15) -> float:
    return _lib.cb_pick_recompute_ratio(prefill_delay, load_delay, min_ratio)


def cb_pick_storage_device(recompute_delay: float, load_delays: Sequence[float], costs: Sequence[float]) -> int:
    n = len(load_delays)
    return _lib.cb_pick_storage_device(recompute_delay, (C.c_double * n)(*load_delays), (C.c_double * n)(*costs), n)


def cb_profile_enable(ctx: Context, enable):
    """0 / False: off; 1 / True: every launch and the two phases; 2: the two phases only."""
    _check(_lib.cb_profile_enable(ctx._h, int(enable)), "cb_profile_enable")


def cb_profile_read(ctx: Context):
    """dict class -> {ms, launches, flops, bytes} accumulated since the last read."""
    n = len(PROF_CLASSES)
    ms, fl, by = (C.c_double * n)(), (C.c_double * n)(), (C.c_double * n)()
    la = (C.c_int64 * n)()
    _check(_lib.cb_profile_read(ctx._h, ms, la, fl, by), "cb_profile_read")
    return {c: {"ms": ms[i], "launches": la[i], "flops": fl[i], "bytes": by[i]}
            for i, c in enumerate(PROF_CLASSES)}
