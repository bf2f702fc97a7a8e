"""MI355X-native verify-step attention for tree / sequence speculative decoding.

The product is ``libowl.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/owl.h``); ``binding`` marshals arguments to it, ``runner`` keeps a
verify step's buffers resident on the GPU for tests and benchmarks, and
``workloads`` draws the seeded synthetic inputs.

Submodules are imported on first use, so that ``workloads`` (data only, shared
with the checker) can be used without touching the binding.
"""
import importlib

_BINDING_NAMES = (
    "OwlError", "owl_build_tree_mask", "owl_build_tree_mask_host", "owl_gather_kv",
    "owl_verify_attn", "owl_verify_attn_phases", "owl_verify_attn_plan", "owl_verify_attn_workspace_size",
)


def __getattr__(name):
    if name in ("binding", "runner", "workloads", "build"):
        return importlib.import_module("." + name, __name__)
    if name in _BINDING_NAMES:
        return getattr(importlib.import_module(".binding", __name__), name)
    raise AttributeError(name)
