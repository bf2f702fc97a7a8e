"""Thin ctypes binding of libowl.so: argument marshalling only.

Every step of the verify-attention path runs inside the library's HIP kernels;
torch is used here for nothing but device pointers and the current stream.
There is no CPU fallback: a missing library is an ImportError-like failure.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_PKG = os.path.dirname(os.path.abspath(__file__))
# OWL_LIB_PATH points the binding at another build of the same library (the host-sanitizer build
# of tests/test_sanitizers.py); there is still no fallback if the file is missing.
LIB_PATH = os.environ.get("OWL_LIB_PATH") or os.path.join(_PKG, "libowl.so")

OWL_BF16, OWL_F32, OWL_F16 = 0, 1, 2
OWL_OK = 0
OWL_ERR_INVALID_ARG, OWL_ERR_BAD_TREE, OWL_ERR_TOO_MANY_DRAFT = -1, -2, -3
OWL_ERR_UNSUPPORTED, OWL_ERR_WORKSPACE, OWL_ERR_HIP = -4, -5, -6
OWL_DEV_BAD_PARENT, OWL_DEV_BAD_PAGE, OWL_DEV_BAD_CTX_LEN, OWL_DEV_BAD_ACCEPT = 1, 2, 4, 8
OWL_DEV_BAD_NDRAFT = 16
OWL_DEV_BAD_TOKEN, OWL_DEV_BAD_ROW = 32, 64
OWL_DRAFTER_PROJ, OWL_DRAFTER_GATES, OWL_DRAFTER_ALL = 1, 2, 3
OWL_W_ROWS, OWL_W_TILED = 0, 1

OWL_FLAG_FP32_PARTIALS = 1

# entry points declared in include/owl.h (the product interface) ...
EXPORTS = (
    "owl_verify_attn_plan", "owl_verify_attn_workspace_size", "owl_verify_attn",
    "owl_verify_attn_phases",
    "owl_build_tree_mask", "owl_build_tree_mask_host", "owl_gather_kv",
    "owl_prepare_spec_tree", "owl_accept_greedy", "owl_commit_kv", "owl_verify_attn_ragged",
    "owl_drafter_cell", "owl_drafter_cell_phases", "owl_drafter_cell_workspace_size", "owl_drafter_alpha",
    "owl_drafter_tiled_weight_bytes", "owl_drafter_tile_weights",
    "owl_verify_attn_init", "owl_verify_attn_noalloc",
    "owl_status_str", "owl_version",
)
# ... and in include/owl_probe.h (measurement and self-test aids)
PROBE_EXPORTS = (
    "owl_stream_read_probe", "owl_gather_read_probe", "owl_mfma_probe", "owl_selftest_quad_max",
    "owl_debug_set_timeline", "owl_step_probe", "owl_verify_attn_split_timed", "owl_probe_event_create",
    "owl_probe_event_destroy", "owl_probe_event_elapsed_ms",
)
OWL_NOALLOC_SCRATCH_BYTES = 48 << 20


class VerifyDesc(ctypes.Structure):
    """Mirror of owl_verify_desc (include/owl.h)."""
    _fields_ = [
        ("batch", ctypes.c_int32), ("n_draft", ctypes.c_int32),
        ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32), ("page_size", ctypes.c_int32),
        ("max_pages_per_seq", ctypes.c_int32), ("max_ctx_len", ctypes.c_int32),
        ("qkv_dtype", ctypes.c_int32), ("split_tokens", ctypes.c_int32),
        ("scale", ctypes.c_float), ("out_dtype", ctypes.c_int32),
        ("kv_stride_page", ctypes.c_int64), ("kv_stride_head", ctypes.c_int64),
        ("kv_stride_token", ctypes.c_int64), ("n_pool_pages", ctypes.c_int64),
        ("flags", ctypes.c_int32), ("reserved_", ctypes.c_int32),
    ]


class Plan(ctypes.Structure):
    """Mirror of owl_plan."""
    _fields_ = [
        ("split_tokens", ctypes.c_int32), ("max_splits", ctypes.c_int32),
        ("rows_per_kv", ctypes.c_int32), ("row_tiles", ctypes.c_int32),
        ("row_groups", ctypes.c_int32), ("tiles_per_wave", ctypes.c_int32),
        ("kernel_variant", ctypes.c_int32), ("n_workgroups", ctypes.c_int32),
        ("reserved_", ctypes.c_int32),
        ("workspace_bytes", ctypes.c_size_t),
    ]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_ if not n.startswith("reserved")}


class DrafterDesc(ctypes.Structure):
    """Mirror of owl_drafter_desc."""
    _fields_ = [
        ("d_in", ctypes.c_int32), ("d", ctypes.c_int32), ("n_states", ctypes.c_int32),
        ("n_rows", ctypes.c_int32), ("vocab", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("alpha", ctypes.c_float), ("eps", ctypes.c_float),
        ("w_layout", ctypes.c_int32), ("reserved_", ctypes.c_int32),
    ]


class OwlError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {status_str(code)} ({code})")
        self.code = code


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded C-ABI library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2510_07535_amd.build` "
                "(there is no fallback path)")
        l = ctypes.CDLL(LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        l.owl_verify_attn_plan.restype = ctypes.c_int
        l.owl_verify_attn_plan.argtypes = [ctypes.POINTER(VerifyDesc), ctypes.POINTER(Plan)]
        l.owl_verify_attn_workspace_size.restype = ctypes.c_int
        l.owl_verify_attn_workspace_size.argtypes = [ctypes.POINTER(VerifyDesc),
                                                     ctypes.POINTER(ctypes.c_size_t)]
        l.owl_verify_attn.restype = ctypes.c_int
        l.owl_verify_attn.argtypes = [ctypes.POINTER(VerifyDesc), vp, vp, vp, vp, vp, vp, vp,
                                      vp, ctypes.c_size_t, vp, vp]
        l.owl_verify_attn_init.restype = ctypes.c_int
        l.owl_verify_attn_init.argtypes = [ctypes.POINTER(VerifyDesc)]
        l.owl_verify_attn_noalloc.restype = ctypes.c_int
        l.owl_verify_attn_noalloc.argtypes = [ctypes.POINTER(VerifyDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp]
        l.owl_verify_attn_ragged.restype = ctypes.c_int
        l.owl_verify_attn_ragged.argtypes = [ctypes.POINTER(VerifyDesc), vp, vp, vp, vp, vp, vp, vp, vp,
                                             vp, ctypes.c_size_t, vp, vp]
        l.owl_verify_attn_phases.restype = ctypes.c_int
        l.owl_verify_attn_phases.argtypes = [ctypes.POINTER(VerifyDesc), vp, vp, vp, vp, vp, vp, vp,
                                             vp, ctypes.c_size_t, vp, vp, i32]
        l.owl_stream_read_probe.restype = ctypes.c_int
        l.owl_stream_read_probe.argtypes = [vp, ctypes.c_size_t, vp, i32, vp]
        l.owl_mfma_probe.restype = ctypes.c_int
        l.owl_mfma_probe.argtypes = [vp, ctypes.c_size_t, i32, vp, vp, i32, vp]
        l.owl_gather_read_probe.restype = ctypes.c_int
        l.owl_gather_read_probe.argtypes = [vp, vp, i32, vp, i32, vp]
        l.owl_debug_set_timeline.restype = ctypes.c_int
        l.owl_debug_set_timeline.argtypes = [vp, i64]
        l.owl_verify_attn_split_timed.restype = ctypes.c_int
        l.owl_verify_attn_split_timed.argtypes = [ctypes.POINTER(VerifyDesc), vp, vp, vp, vp, vp, vp, vp,
                                                  vp, ctypes.c_size_t, vp, vp, vp, vp]
        l.owl_probe_event_create.restype = ctypes.c_int
        l.owl_probe_event_create.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        l.owl_probe_event_destroy.restype = ctypes.c_int
        l.owl_probe_event_destroy.argtypes = [vp]
        l.owl_probe_event_elapsed_ms.restype = ctypes.c_int
        l.owl_probe_event_elapsed_ms.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_float)]
        l.owl_step_probe.restype = ctypes.c_int
        l.owl_step_probe.argtypes = [i32, vp, i32, vp, vp, i32, vp]
        l.owl_selftest_quad_max.restype = ctypes.c_int
        l.owl_selftest_quad_max.argtypes = [vp, vp, vp]
        l.owl_build_tree_mask.restype = ctypes.c_int
        l.owl_build_tree_mask.argtypes = [vp, i32, i32, vp, vp, vp, vp]
        l.owl_build_tree_mask_host.restype = ctypes.c_int
        l.owl_build_tree_mask_host.argtypes = [vp, i32, vp, vp]
        l.owl_gather_kv.restype = ctypes.c_int
        l.owl_gather_kv.argtypes = [ctypes.POINTER(VerifyDesc), vp, vp, i32, i64, i64, vp, vp, vp]
        l.owl_drafter_cell_workspace_size.restype = ctypes.c_int
        l.owl_drafter_cell_workspace_size.argtypes = [ctypes.POINTER(DrafterDesc), ctypes.POINTER(ctypes.c_size_t)]
        l.owl_drafter_cell.restype = ctypes.c_int
        l.owl_drafter_cell.argtypes = [ctypes.POINTER(DrafterDesc)] + [vp] * 14 + [ctypes.c_size_t, vp, vp]
        l.owl_drafter_cell_phases.restype = ctypes.c_int
        l.owl_drafter_cell_phases.argtypes = [ctypes.POINTER(DrafterDesc)] + [vp] * 14 + [ctypes.c_size_t, vp, vp, i32]
        l.owl_drafter_tiled_weight_bytes.restype = ctypes.c_int
        l.owl_drafter_tiled_weight_bytes.argtypes = [ctypes.POINTER(DrafterDesc), ctypes.POINTER(ctypes.c_size_t)]
        l.owl_drafter_tile_weights.restype = ctypes.c_int
        l.owl_drafter_tile_weights.argtypes = [ctypes.POINTER(DrafterDesc), vp, vp, vp]
        l.owl_drafter_alpha.restype = ctypes.c_int
        l.owl_drafter_alpha.argtypes = [i32, i32, ctypes.POINTER(ctypes.c_float)]
        l.owl_prepare_spec_tree.restype = ctypes.c_int
        l.owl_prepare_spec_tree.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp]
        l.owl_accept_greedy.restype = ctypes.c_int
        l.owl_accept_greedy.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, vp]
        l.owl_commit_kv.restype = ctypes.c_int
        l.owl_commit_kv.argtypes = [ctypes.POINTER(VerifyDesc), vp, vp, vp, vp, vp, vp, vp, vp, vp]
        l.owl_status_str.restype = ctypes.c_char_p
        l.owl_status_str.argtypes = [ctypes.c_int]
        l.owl_version.restype = ctypes.c_char_p
        _lib = l
    return _lib


def status_str(code: int) -> str:
    return lib().owl_status_str(int(code)).decode()


def _check(code: int, what: str) -> None:
    if code != OWL_OK:
        raise OwlError(code, what)


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream() -> int:
    import torch
    return int(torch.cuda.current_stream().cuda_stream)


def make_desc(*, batch, n_draft, n_q_heads, n_kv_heads, head_dim, max_pages_per_seq, max_ctx_len,
              qkv_dtype, scale, kv_stride_page, kv_stride_head, kv_stride_token, n_pool_pages,
              page_size=16, split_tokens=0, out_dtype=OWL_F32, flags=0) -> VerifyDesc:
    return VerifyDesc(batch=batch, n_draft=n_draft, n_q_heads=n_q_heads, n_kv_heads=n_kv_heads,
                      head_dim=head_dim, page_size=page_size, max_pages_per_seq=max_pages_per_seq,
                      max_ctx_len=max_ctx_len, qkv_dtype=qkv_dtype, split_tokens=split_tokens,
                      scale=scale, out_dtype=out_dtype, kv_stride_page=kv_stride_page,
                      kv_stride_head=kv_stride_head, kv_stride_token=kv_stride_token,
                      n_pool_pages=n_pool_pages, flags=flags, reserved_=0)


def owl_verify_attn_plan(desc: VerifyDesc) -> Plan:
    plan = Plan()
    _check(lib().owl_verify_attn_plan(ctypes.byref(desc), ctypes.byref(plan)), "owl_verify_attn_plan")
    return plan


def owl_verify_attn_workspace_size(desc: VerifyDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().owl_verify_attn_workspace_size(ctypes.byref(desc), ctypes.byref(n)),
           "owl_verify_attn_workspace_size")
    return int(n.value)


def owl_verify_attn(desc: VerifyDesc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, out,
                    workspace, dev_status=None, stream: Optional[int] = None) -> None:
    """All tensor arguments are torch CUDA tensors (or None where the C ABI
    allows NULL); nothing is copied or allocated here."""
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().owl_verify_attn(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                               _ptr(page_table), _ptr(ctx_lens), _ptr(tree_parent), _ptr(out),
                               _ptr(workspace), ws_bytes, _ptr(dev_status),
                               _stream() if stream is None else stream)
    _check(rc, "owl_verify_attn")


def owl_verify_attn_init(desc: VerifyDesc) -> None:
    _check(lib().owl_verify_attn_init(ctypes.byref(desc)), "owl_verify_attn_init")


def owl_verify_attn_noalloc(desc: VerifyDesc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, out,
                            dev_status=None, stream: Optional[int] = None) -> None:
    """owl_verify_attn without a workspace argument (the library's own fixed scratch buffer)."""
    rc = lib().owl_verify_attn_noalloc(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                       _ptr(page_table), _ptr(ctx_lens), _ptr(tree_parent), _ptr(out),
                                       _ptr(dev_status), _stream() if stream is None else stream)
    _check(rc, "owl_verify_attn_noalloc")


PHASE_SPLIT, PHASE_COMBINE, PHASE_ALL = 1, 2, 3


def owl_verify_attn_phases(desc: VerifyDesc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent,
                           out, workspace, dev_status=None, stream: Optional[int] = None,
                           phases: int = PHASE_ALL) -> None:
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = lib().owl_verify_attn_phases(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                      _ptr(page_table), _ptr(ctx_lens), _ptr(tree_parent), _ptr(out),
                                      _ptr(workspace), ws_bytes, _ptr(dev_status),
                                      _stream() if stream is None else stream, phases)
    _check(rc, "owl_verify_attn_phases")


def owl_stream_read_probe(src, sink, n_workgroups: int, stream: Optional[int] = None) -> None:
    rc = lib().owl_stream_read_probe(_ptr(src), src.numel() * src.element_size(), _ptr(sink),
                                     n_workgroups, _stream() if stream is None else stream)
    _check(rc, "owl_stream_read_probe")


def owl_gather_read_probe(src, block_order, sink, n_workgroups: int, stream: Optional[int] = None) -> None:
    rc = lib().owl_gather_read_probe(_ptr(src), _ptr(block_order), int(block_order.numel()), _ptr(sink),
                                     n_workgroups, _stream() if stream is None else stream)
    _check(rc, "owl_gather_read_probe")


def owl_debug_set_timeline(buffer) -> None:
    """buffer: int64 CUDA tensor with 10 entries per split-KV workgroup (its length gives the
    number of workgroups it has room for), or None to switch the recording off."""
    n = 0 if buffer is None else int(buffer.numel()) // 10
    _check(lib().owl_debug_set_timeline(_ptr(buffer), n), "owl_debug_set_timeline")


class KernelTimer:
    """A pair of HIP events that the library attaches to the dispatch of the split-KV kernel itself."""

    def __init__(self):
        a, b = ctypes.c_void_p(), ctypes.c_void_p()
        _check(lib().owl_probe_event_create(ctypes.byref(a)), "owl_probe_event_create")
        _check(lib().owl_probe_event_create(ctypes.byref(b)), "owl_probe_event_create")
        self.start, self.stop = a, b

    def elapsed_ms(self) -> float:
        ms = ctypes.c_float(0.0)
        _check(lib().owl_probe_event_elapsed_ms(self.start, self.stop, ctypes.byref(ms)), "owl_probe_event_elapsed_ms")
        return float(ms.value)

    def __del__(self):
        try:
            lib().owl_probe_event_destroy(self.start)
            lib().owl_probe_event_destroy(self.stop)
        except Exception:
            pass


def owl_verify_attn_split_timed(desc: VerifyDesc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, out,
                                workspace, timer: KernelTimer, dev_status=None, stream: Optional[int] = None) -> None:
    rc = lib().owl_verify_attn_split_timed(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                           _ptr(page_table), _ptr(ctx_lens), _ptr(tree_parent), _ptr(out),
                                           _ptr(workspace), workspace.numel() * workspace.element_size(),
                                           _ptr(dev_status), _stream() if stream is None else stream,
                                           timer.start, timer.stop)
    _check(rc, "owl_verify_attn_split_timed")


STEP_PROBE_VARIANTS = (
    (0, "3 + 2 tiles", 5), (1, "3 + 2 tiles, barrier every 64 keys", 5), (2, "3 + 2 tiles, V by 64-bit LDS reads", 5),
    (3, "3 + 2 tiles, barrier + 64-bit V reads", 5), (4, "2 + 2 tiles", 4), (5, "2 + 2 tiles, barrier + 64-bit V reads", 4),
)


def owl_step_probe(variant: int, src, iters: int, sink, cycles, n_workgroups: int, stream: Optional[int] = None) -> None:
    rc = lib().owl_step_probe(variant, _ptr(src), iters, _ptr(sink), _ptr(cycles), n_workgroups,
                              _stream() if stream is None else stream)
    _check(rc, "owl_step_probe")


def owl_selftest_quad_max(in64, out64, stream: Optional[int] = None) -> None:
    rc = lib().owl_selftest_quad_max(_ptr(in64), _ptr(out64), _stream() if stream is None else stream)
    _check(rc, "owl_selftest_quad_max")


def owl_build_tree_mask(tree_parent, anc_mask, depth=None, dev_status=None,
                        stream: Optional[int] = None) -> None:
    B, N = tree_parent.shape
    rc = lib().owl_build_tree_mask(_ptr(tree_parent), B, N, _ptr(anc_mask), _ptr(depth),
                                   _ptr(dev_status), _stream() if stream is None else stream)
    _check(rc, "owl_build_tree_mask")


def owl_build_tree_mask_host(parent):
    """numpy int32 [N] -> (anc uint64 [N], depth int32 [N]); raises OwlError on a bad tree."""
    import numpy as np
    par = np.ascontiguousarray(parent, dtype=np.int32)
    n = int(par.shape[0])
    anc = np.zeros(max(n, 1), dtype=np.uint64)
    depth = np.zeros(max(n, 1), dtype=np.int32)
    rc = lib().owl_build_tree_mask_host(par.ctypes.data, n, anc.ctypes.data, depth.ctypes.data)
    _check(rc, "owl_build_tree_mask_host")
    return anc[:n], depth[:n]


def owl_gather_kv(desc: VerifyDesc, cache, page_table, seq: int, first_pos: int, n_tokens: int, dst,
                  dev_status=None, stream: Optional[int] = None) -> None:
    rc = lib().owl_gather_kv(ctypes.byref(desc), _ptr(cache), _ptr(page_table), seq, first_pos,
                             n_tokens, _ptr(dst), _ptr(dev_status),
                             _stream() if stream is None else stream)
    _check(rc, "owl_gather_kv")


def owl_prepare_spec_tree(tree_parent, ctx_lens, tree_parent2, anc_mask, depth=None, pos_ids=None,
                          dev_status=None, stream: Optional[int] = None) -> None:
    B, n = tree_parent.shape
    rc = lib().owl_prepare_spec_tree(_ptr(tree_parent), _ptr(ctx_lens), B, n, _ptr(tree_parent2),
                                     _ptr(anc_mask), _ptr(depth), _ptr(pos_ids), _ptr(dev_status),
                                     _stream() if stream is None else stream)
    _check(rc, "owl_prepare_spec_tree")


def owl_accept_greedy(tokens, tree_parent, target_root, target_next, n_cand: int, accepted, n_accept, bonus,
                      last, dev_status=None, stream: Optional[int] = None) -> None:
    B, N = tokens.shape
    rc = lib().owl_accept_greedy(_ptr(tokens), _ptr(tree_parent), _ptr(target_root), _ptr(target_next), B, N,
                                 n_cand, _ptr(accepted), _ptr(n_accept), _ptr(bonus), _ptr(last),
                                 _ptr(dev_status), _stream() if stream is None else stream)
    _check(rc, "owl_accept_greedy")


def owl_commit_kv(desc: VerifyDesc, k_cache, v_cache, page_table, ctx_lens, accepted, n_accept,
                  new_ctx_lens=None, dev_status=None, stream: Optional[int] = None) -> None:
    rc = lib().owl_commit_kv(ctypes.byref(desc), _ptr(k_cache), _ptr(v_cache), _ptr(page_table),
                             _ptr(ctx_lens), _ptr(accepted), _ptr(n_accept), _ptr(new_ctx_lens),
                             _ptr(dev_status), _stream() if stream is None else stream)
    _check(rc, "owl_commit_kv")


def owl_verify_attn_ragged(desc: VerifyDesc, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, n_draft_seq,
                           out, workspace, dev_status=None, stream: Optional[int] = None) -> None:
    rc = lib().owl_verify_attn_ragged(ctypes.byref(desc), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(page_table),
                                      _ptr(ctx_lens), _ptr(tree_parent), _ptr(n_draft_seq), _ptr(out),
                                      _ptr(workspace), workspace.numel() * workspace.element_size(),
                                      _ptr(dev_status), _stream() if stream is None else stream)
    _check(rc, "owl_verify_attn_ragged")


def owl_mfma_probe(src, iters: int, sink, n_workgroups: int, stream: Optional[int] = None, clock_ghz=None) -> None:
    rc = lib().owl_mfma_probe(_ptr(src), src.numel() * src.element_size(), iters, _ptr(sink), _ptr(clock_ghz),
                              n_workgroups,
                              _stream() if stream is None else stream)
    _check(rc, "owl_mfma_probe")


def owl_drafter_alpha(max_depth: int, d: int) -> float:
    a = ctypes.c_float(0.0)
    _check(lib().owl_drafter_alpha(max_depth, d, ctypes.byref(a)), "owl_drafter_alpha")
    return float(a.value)


def owl_drafter_cell_workspace_size(desc: DrafterDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().owl_drafter_cell_workspace_size(ctypes.byref(desc), ctypes.byref(n)),
           "owl_drafter_cell_workspace_size")
    return int(n.value)


def owl_drafter_cell_phases(desc: DrafterDesc, h, z, tokens, parent_row, w, emb, gamma_c, beta_c, gamma_z, beta_z,
                            h_out, h_out_f32, z_out, workspace, dev_status=None, stream: Optional[int] = None,
                            phases: int = OWL_DRAFTER_ALL) -> None:
    rc = lib().owl_drafter_cell_phases(ctypes.byref(desc), _ptr(h), _ptr(z), _ptr(tokens), _ptr(parent_row),
                                       _ptr(w), _ptr(emb), _ptr(gamma_c), _ptr(beta_c), _ptr(gamma_z),
                                       _ptr(beta_z), _ptr(h_out), _ptr(h_out_f32), _ptr(z_out), _ptr(workspace),
                                       workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                       _ptr(dev_status), _stream() if stream is None else stream, phases)
    _check(rc, "owl_drafter_cell_phases")


def owl_drafter_cell(desc: DrafterDesc, h, z, tokens, parent_row, w, emb, gamma_c, beta_c, gamma_z, beta_z,
                     h_out, h_out_f32, z_out, workspace, dev_status=None, stream: Optional[int] = None) -> None:
    rc = lib().owl_drafter_cell(ctypes.byref(desc), _ptr(h), _ptr(z), _ptr(tokens), _ptr(parent_row),
                                _ptr(w), _ptr(emb), _ptr(gamma_c), _ptr(beta_c), _ptr(gamma_z),
                                _ptr(beta_z), _ptr(h_out), _ptr(h_out_f32), _ptr(z_out), _ptr(workspace),
                                workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                _ptr(dev_status), _stream() if stream is None else stream)
    _check(rc, "owl_drafter_cell")


def owl_drafter_tiled_weight_bytes(desc: DrafterDesc) -> int:
    n = ctypes.c_size_t(0)
    _check(lib().owl_drafter_tiled_weight_bytes(ctypes.byref(desc), ctypes.byref(n)),
           "owl_drafter_tiled_weight_bytes")
    return int(n.value)


def owl_drafter_tile_weights(desc: DrafterDesc, w_rows, w_tiled, stream: Optional[int] = None) -> None:
    _check(lib().owl_drafter_tile_weights(ctypes.byref(desc), _ptr(w_rows), _ptr(w_tiled),
                                          _stream() if stream is None else stream), "owl_drafter_tile_weights")
