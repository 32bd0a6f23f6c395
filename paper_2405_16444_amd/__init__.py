"""MI355X-native CacheBlend KV-cache fusor: HIP kernels behind a C ABI
(include/cacheblend.h) and a thin ctypes binding with the same entry-point names.

The binding is loaded on first use so that `python -m paper_2405_16444_amd.build`
can run before the library exists; using any entry point without the built library
raises ImportError (there is no CPU or torch fallback)."""

_BINDING_NAMES = ("Context", "CacheBlendError", "cb_create", "cb_destroy", "cb_strerror",
                  "cb_layer_workspace_bytes", "cb_prefill_workspace_bytes", "cb_default_schedule",
                  "cb_realign_rope", "cb_fuse_layer", "cb_static_scratch_bytes", "cb_fuse_layer_static", "cb_fuse_prefill", "cb_fuse_prefill_pipelined", "cb_batched_workspace_bytes",
                  "cb_fuse_prefill_batched", "cb_first_token",
                  "cb_recompute_delay", "cb_load_delay", "cb_pick_recompute_ratio",
                  "cb_pick_storage_device", "cb_profile_enable",
                  "cb_profile_read", "PROF_CLASSES", "EXPORTS")


def __getattr__(name):
    if name in _BINDING_NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
