"""MI355X-native verify-step attention for tree / sequence speculative decoding.

The product is ``libowl.so`` (hand-written HIP for gfx950 behind the C ABI of
``include/owl.h``); ``binding`` marshals arguments to it, ``runner`` keeps a
verify step's buffers resident on the GPU for tests and benchmarks, and
``workloads`` draws the seeded synthetic inputs.
"""
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    OwlError, owl_build_tree_mask, owl_build_tree_mask_host, owl_gather_kv, owl_stream_read_probe,
    owl_verify_attn, owl_verify_attn_phases,
    owl_verify_attn_plan, owl_verify_attn_workspace_size,
)
