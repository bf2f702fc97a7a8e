"""Host-side checks that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before any launch."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2510_07535_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _good(**over):
    kw = dict(batch=1, n_draft=6, n_q_heads=32, n_kv_heads=8, head_dim=128, max_pages_per_seq=2049,
              max_ctx_len=32768, qkv_dtype=B.OWL_BF16, scale=0.0883883, kv_stride_page=8 * 16 * 128,
              kv_stride_head=16 * 128, kv_stride_token=128, n_pool_pages=2049)
    kw.update(over)
    return B.make_desc(**kw)


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    for fname, names in (("owl.h", B.EXPORTS), ("owl_probe.h", B.PROBE_EXPORTS)):
        header = open(os.path.join(ROOT, "include", fname)).read()
        declared = set(re.findall(r"\b(owl_[a-z_]+)\s*\(", header))
        assert declared == set(names), (fname, declared ^ set(names))
        for name in declared:
            assert getattr(lib, name) is not None
    assert lib.owl_version().decode().count(".") == 1


def test_struct_layout_matches_header():
    assert ctypes.sizeof(B.VerifyDesc) == 12 * 4 + 4 * 8 + 2 * 4
    assert B.VerifyDesc.out_dtype.offset == 44 and B.VerifyDesc.kv_stride_page.offset == 48
    assert B.VerifyDesc.flags.offset == 80
    assert ctypes.sizeof(B.Plan) == 10 * 4 + 8 and B.Plan.workspace_bytes.offset == 40


def test_plan_matches_shapes():
    p = B.owl_verify_attn_plan(_good())
    assert p.rows_per_kv == 24 and p.row_tiles == 2 and p.row_groups == 1 and p.tiles_per_wave == 1
    assert p.split_tokens % 64 == 0 and p.split_tokens * p.max_splits >= 32768 + 6
    assert p.workspace_bytes == B.owl_verify_attn_workspace_size(_good())
    p = B.owl_verify_attn_plan(_good(n_draft=40, n_q_heads=64, max_ctx_len=131072, max_pages_per_seq=8200))
    assert p.rows_per_kv == 320 and p.row_tiles == 20 and p.tiles_per_wave == 3
    p = B.owl_verify_attn_plan(_good(split_tokens=1000))
    assert p.split_tokens == 1024
    p = B.owl_verify_attn_plan(_good(n_draft=64, n_q_heads=64, max_ctx_len=131072, max_pages_per_seq=8200))   # 512 rows
    assert p.row_tiles == 32 and p.row_groups == 2 and p.tiles_per_wave == 2
    # few KV streams: the rows go to more, smaller groups until the launch has about a workgroup per compute unit
    p = B.owl_verify_attn_plan(_good(n_draft=64, n_q_heads=64, max_ctx_len=8192, max_pages_per_seq=520))   # 512 rows, 8K
    assert p.row_tiles == 32 and p.row_groups == 8 and p.tiles_per_wave == 1
    p = B.owl_verify_attn_plan(_good(n_draft=40, n_q_heads=8, n_kv_heads=1, max_ctx_len=131072, max_pages_per_seq=8200))
    assert p.row_tiles == 20 and p.row_groups == 2 and p.tiles_per_wave == 2 and 192 <= p.n_workgroups <= 256
    assert p.n_workgroups % 8 == 0 and p.split_tokens >= 4 * 320
    p = B.owl_verify_attn_plan(_good(n_draft=40, n_q_heads=8, n_kv_heads=1, max_ctx_len=24000, max_pages_per_seq=1510))
    assert p.row_groups == 5 and p.tiles_per_wave == 1


@pytest.mark.parametrize("over,code", [
    (dict(batch=0), B.OWL_ERR_INVALID_ARG),
    (dict(n_draft=0), B.OWL_ERR_INVALID_ARG),
    (dict(n_draft=65), B.OWL_ERR_TOO_MANY_DRAFT),
    (dict(n_q_heads=30), B.OWL_ERR_INVALID_ARG),
    (dict(head_dim=96), B.OWL_ERR_UNSUPPORTED),
    (dict(page_size=32), B.OWL_ERR_UNSUPPORTED),
    (dict(qkv_dtype=7), B.OWL_ERR_UNSUPPORTED),
    (dict(scale=0.0), B.OWL_ERR_INVALID_ARG),
    (dict(scale=float("nan")), B.OWL_ERR_INVALID_ARG),
    (dict(max_ctx_len=-1), B.OWL_ERR_INVALID_ARG),
    (dict(kv_stride_token=100), B.OWL_ERR_INVALID_ARG),
    (dict(kv_stride_head=2052), B.OWL_ERR_INVALID_ARG),
    (dict(n_pool_pages=0), B.OWL_ERR_INVALID_ARG),
    (dict(split_tokens=-5), B.OWL_ERR_INVALID_ARG),
])
def test_bad_descriptors_are_rejected(over, code):
    with pytest.raises(B.OwlError) as e:
        B.owl_verify_attn_plan(_good(**over))
    assert e.value.code == code


def test_verify_attn_rejects_before_launch():
    """Null / misaligned pointers and a short workspace come back as errors
    without touching a device (fake non-null addresses are never dereferenced
    on these paths)."""
    lib = B.lib()
    d = _good()
    need = B.owl_verify_attn_workspace_size(d)
    A = 0x10000
    args = [A, A, A, A, A, A, A, A, need, None, None]      # q k v pt ctx parent out ws bytes status stream
    def call(a):
        return lib.owl_verify_attn(ctypes.byref(d), *a)
    for null_at in (0, 1, 2, 4, 5, 6):
        a = list(args); a[null_at] = None
        assert call(a) == B.OWL_ERR_INVALID_ARG
    a = list(args); a[7] = None
    assert call(a) == B.OWL_ERR_WORKSPACE
    a = list(args); a[8] = need - 1
    assert call(a) == B.OWL_ERR_WORKSPACE
    a = list(args); a[0] = A + 2
    assert call(a) == B.OWL_ERR_INVALID_ARG
    a = list(args); a[7] = A + 16
    assert call(a) == B.OWL_ERR_INVALID_ARG
    short = _good(max_pages_per_seq=100)                    # table cannot cover max_ctx_len + N
    assert lib.owl_verify_attn(ctypes.byref(short), *args) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_verify_attn(None, *args) == B.OWL_ERR_INVALID_ARG


def test_mask_host_twin():
    anc, dep = B.owl_build_tree_mask_host(np.array([-1, 0, 0, 0, 1, 2], np.int32))
    assert list(anc) == [0b1, 0b11, 0b101, 0b1001, 0b10011, 0b100101]
    assert list(dep) == [1, 2, 2, 2, 3, 3]
    for bad in ([0], [-1, 1], [-3], [-1, 0, 3]):
        with pytest.raises(B.OwlError) as e:
            B.owl_build_tree_mask_host(np.array(bad, np.int32))
        assert e.value.code == B.OWL_ERR_BAD_TREE
    with pytest.raises(B.OwlError) as e:
        B.owl_build_tree_mask_host(np.arange(-1, 64, dtype=np.int32))
    assert e.value.code == B.OWL_ERR_TOO_MANY_DRAFT
    lib = B.lib()
    assert lib.owl_build_tree_mask(None, 1, 4, 0x1000, None, None, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_build_tree_mask(0x1000, 1, 65, 0x1000, None, None, None) == B.OWL_ERR_TOO_MANY_DRAFT
    assert lib.owl_gather_kv(ctypes.byref(_good()), None, None, 0, 0, 1, 0x1000, None, None) == B.OWL_ERR_INVALID_ARG
    assert "workspace" in B.status_str(B.OWL_ERR_WORKSPACE)


def test_step_entry_points_reject_before_launch():
    """Prepare / accept / commit: argument errors are host-side and launch nothing."""
    lib = B.lib()
    A = 0x10000
    # prepare: (parent, ctx, B, n, parent2, anc, depth, pos, status, stream)
    assert lib.owl_prepare_spec_tree(None, A, 1, 3, A, A, None, None, None, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_prepare_spec_tree(A, A, 1, 3, None, A, None, None, None, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_prepare_spec_tree(A, A, 0, 3, A, A, None, None, None, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_prepare_spec_tree(A, A, 1, 33, A, A, None, None, None, None) == B.OWL_ERR_TOO_MANY_DRAFT
    # accept: (tokens, parent, root, next, B, N, n_cand, accepted, n_accept, bonus, last, status, stream)
    ok = [A, A, A, A, 1, 8, 8, A, A, A, A, None, None]
    for null_at in (0, 1, 2, 3, 7, 8, 9, 10):
        a = list(ok); a[null_at] = None
        assert lib.owl_accept_greedy(*a) == B.OWL_ERR_INVALID_ARG
    a = list(ok); a[6] = 9
    assert lib.owl_accept_greedy(*a) == B.OWL_ERR_INVALID_ARG          # more candidates than nodes
    a = list(ok); a[5] = 65; a[6] = 65
    assert lib.owl_accept_greedy(*a) == B.OWL_ERR_TOO_MANY_DRAFT
    # commit: (desc, k, v, page_table, ctx, accepted, n_accept, new_ctx, status, stream)
    d = _good()
    assert lib.owl_commit_kv(ctypes.byref(d), None, A, A, A, A, A, None, None, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_commit_kv(ctypes.byref(d), A, A, A, A, A, A, A, None, None) == B.OWL_ERR_INVALID_ARG   # new_ctx aliases ctx
    assert lib.owl_commit_kv(ctypes.byref(d), A + 2, A, A, A, A, A, None, None, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_commit_kv(None, A, A, A, A, A, A, None, None, None) == B.OWL_ERR_INVALID_ARG
    short = _good(max_pages_per_seq=100)
    assert lib.owl_commit_kv(ctypes.byref(short), A, A, A, A, A, A, None, None, None) == B.OWL_ERR_INVALID_ARG


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; any other --gpus exits with a message and code 2, before touching a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_ragged_entry_point_rejects_null_counts():
    lib = B.lib()
    d = _good()
    need = B.owl_verify_attn_workspace_size(d)
    A = 0x10000
    assert lib.owl_verify_attn_ragged(ctypes.byref(d), A, A, A, A, A, A, None, A, A, need, None, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_verify_attn_ragged(ctypes.byref(d), A, A, A, A, A, A, A, A, None, need, None, None) == B.OWL_ERR_WORKSPACE


def test_mfma_probe_rejects_before_launch():
    lib = B.lib()
    A = 0x10000
    assert lib.owl_mfma_probe(None, 4096, 10, A, None, 4, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_mfma_probe(A, 4096, 10, None, None, 4, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_mfma_probe(A, 4100, 10, A, None, 4, None) == B.OWL_ERR_INVALID_ARG       # not a multiple of 16
    assert lib.owl_mfma_probe(A, 4096, 0, A, None, 4, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_mfma_probe(A + 4, 4096, 10, A, None, 4, None) == B.OWL_ERR_INVALID_ARG


# --------------------------------------------------------------------------- drafter cell
def _drafter(**over):
    kw = dict(d_in=12288, d=12288, n_states=10, n_rows=10, vocab=128256, dtype=B.OWL_BF16, alpha=0.002, eps=1e-5)
    kw.update(over)
    return B.DrafterDesc(**kw)


def test_drafter_struct_and_workspace():
    assert ctypes.sizeof(B.DrafterDesc) == 10 * 4
    # 4 * 12288 rows in groups of 64, 12288 / 32 k-steps, 4 KiB per (group, k-step)
    assert B.owl_drafter_tiled_weight_bytes(_drafter()) == (4 * 12288 // 64) * (12288 // 32) * 4096 == 4 * 12288 * 12288 * 2
    assert B.owl_drafter_tiled_weight_bytes(_drafter(d=48, d_in=96)) == 3 * 3 * 4096
    assert B.owl_drafter_tiled_weight_bytes(_drafter(d=16, d_in=32)) == 4096     # one padded group
    assert B.owl_drafter_cell_workspace_size(_drafter()) == (10 * 4 * 12288 + 2 * 10 * 16 * 2) * 4


@pytest.mark.parametrize("over,code", [
    (dict(d_in=0), B.OWL_ERR_INVALID_ARG),
    (dict(d_in=100), B.OWL_ERR_UNSUPPORTED),
    (dict(d=24), B.OWL_ERR_UNSUPPORTED),
    (dict(d=16400), B.OWL_ERR_UNSUPPORTED),
    (dict(n_states=65), B.OWL_ERR_TOO_MANY_DRAFT),
    (dict(n_rows=0), B.OWL_ERR_INVALID_ARG),
    (dict(dtype=B.OWL_F32), B.OWL_ERR_UNSUPPORTED),
    (dict(eps=-1.0), B.OWL_ERR_INVALID_ARG),
    (dict(alpha=float("nan")), B.OWL_ERR_INVALID_ARG),
    (dict(vocab=0), B.OWL_ERR_INVALID_ARG),
    (dict(w_layout=2), B.OWL_ERR_UNSUPPORTED),
])
def test_drafter_bad_descriptors_are_rejected(over, code):
    with pytest.raises(B.OwlError) as e:
        B.owl_drafter_cell_workspace_size(_drafter(**over))
    assert e.value.code == code


def test_drafter_cell_rejects_before_launch():
    lib = B.lib()
    d = _drafter()
    fake = 0x1000                                       # never dereferenced: every call below fails its checks

    def call(desc, h=fake, z=fake, tokens=fake, parent=fake, w=fake, emb=fake, z_out=fake, ws=fake,
             ws_bytes=1 << 30, phases=3):
        return lib.owl_drafter_cell_phases(ctypes.byref(desc), h, z, tokens, parent, w, emb, None, None, None, None,
                                           None, None, z_out, ws, ws_bytes, None, None, phases)
    assert call(d, h=None) == B.OWL_ERR_INVALID_ARG
    assert call(d, w=None) == B.OWL_ERR_INVALID_ARG
    assert call(d, z_out=None) == B.OWL_ERR_INVALID_ARG
    assert call(d, w=fake + 2) == B.OWL_ERR_INVALID_ARG
    assert call(d, z=fake + 4) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_drafter_tile_weights(ctypes.byref(d), None, fake, None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_drafter_tile_weights(ctypes.byref(d), fake, fake + 8, None) == B.OWL_ERR_INVALID_ARG
    assert call(d, phases=0) == B.OWL_ERR_INVALID_ARG
    assert call(d, phases=4) == B.OWL_ERR_INVALID_ARG
    assert call(d, ws=None) == B.OWL_ERR_WORKSPACE
    assert call(d, ws_bytes=100) == B.OWL_ERR_WORKSPACE
    assert call(_drafter(n_rows=7), parent=None) == B.OWL_ERR_INVALID_ARG   # identity needs n_rows == n_states


def test_drafter_alpha_host():
    import math
    assert B.owl_drafter_alpha(1, 8) == pytest.approx(2 * math.sqrt(2) / 8, rel=1e-6)
    with pytest.raises(B.OwlError):
        B.owl_drafter_alpha(0, 8)


def test_output_type_and_reserved_fields():
    for over, code in ((dict(out_dtype=7), B.OWL_ERR_UNSUPPORTED), (dict(flags=2), B.OWL_ERR_INVALID_ARG)):
        with pytest.raises(B.OwlError) as e:
            B.owl_verify_attn_plan(_good(**over))
        assert e.value.code == code
    for od in (B.OWL_F32, B.OWL_BF16, B.OWL_F16):
        B.owl_verify_attn_plan(_good(out_dtype=od))
    # fp32 partials on request: a larger workspace, the same plan otherwise
    assert (B.owl_verify_attn_workspace_size(_good(flags=B.OWL_FLAG_FP32_PARTIALS))
            > B.owl_verify_attn_workspace_size(_good()))


def test_init_and_noalloc_reject_before_touching_a_device():
    lib = B.lib()
    A = 0x10000
    assert lib.owl_verify_attn_init(None) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_verify_attn_init(ctypes.byref(_good(head_dim=96))) == B.OWL_ERR_UNSUPPORTED
    # the entry point without a workspace: a shape whose partials exceed the library's fixed buffer
    big = _good(batch=16, n_draft=26, max_ctx_len=65536, max_pages_per_seq=4100, n_pool_pages=16 * 4100)
    assert B.owl_verify_attn_workspace_size(big) > B.OWL_NOALLOC_SCRATCH_BYTES
    assert lib.owl_verify_attn_noalloc(ctypes.byref(big), A, A, A, A, A, A, A, None, None) == B.OWL_ERR_WORKSPACE
    assert lib.owl_verify_attn_noalloc(None, A, A, A, A, A, A, A, None, None) == B.OWL_ERR_INVALID_ARG
    header = open(os.path.join(ROOT, "include", "owl.h")).read()
    assert f"#define OWL_NOALLOC_SCRATCH_BYTES ({B.OWL_NOALLOC_SCRATCH_BYTES >> 20}u << 20)" in header


def test_timeline_switch_checks_its_arguments():
    lib = B.lib()
    assert lib.owl_debug_set_timeline(0x10000, 0) == B.OWL_ERR_INVALID_ARG
    assert lib.owl_debug_set_timeline(None, 0) == B.OWL_OK
