"""ctypes front end of the CPU fp64 oracle (``owl_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke``
and by the ``cpu_baseline`` leg of ``bench.py``.  The product package never
imports this module, and this module never imports the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "owl_oracle.c")
# OWL_ORACLE_SANITIZE=1 selects a build with AddressSanitizer and UndefinedBehaviorSanitizer (the
# process must then run with gcc's libasan preloaded; tests/test_sanitizers.py does that)
_SANITIZE = os.environ.get("OWL_ORACLE_SANITIZE", "") == "1"
_LIB = os.path.join(_HERE, "libowl_oracle_san.so" if _SANITIZE else "libowl_oracle.so")
_lib = None


class _Problem(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int32),
        ("B", ctypes.c_int32), ("N", ctypes.c_int32), ("Hq", ctypes.c_int32),
        ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32),
        ("scale", ctypes.c_double),
        ("stride_page", ctypes.c_int64), ("stride_head", ctypes.c_int64),
        ("stride_token", ctypes.c_int64),
        ("q", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
        ("page_table", ctypes.c_void_p), ("ctx_lens", ctypes.c_void_p),
        ("tree_parent", ctypes.c_void_p),
    ]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over output rows)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        extra = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                 "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        subprocess.check_call(
            ["gcc", *extra, "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.owl_oracle_verify_attn.restype = ctypes.c_int
        lib.owl_oracle_verify_attn.argtypes = [
            ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_void_p]
        lib.owl_oracle_tree_mask.restype = ctypes.c_int
        lib.owl_oracle_tree_mask.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        lib.owl_oracle_gather_kv.restype = ctypes.c_int
        lib.owl_oracle_gather_kv.argtypes = [
            ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_void_p]
        lib.owl_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().owl_oracle_num_threads())


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle returned {code}")
        self.code = code


def _problem(*, dtype, q, k_cache, v_cache, page_table, ctx_lens, tree_parent, Hq, Hkv, D,
             scale, stride_page, stride_head, stride_token, page_size=16):
    """Returns (struct, keepalive list)."""
    q = np.ascontiguousarray(q)
    k_cache = np.ascontiguousarray(k_cache)
    v_cache = np.ascontiguousarray(v_cache)
    ctx = np.ascontiguousarray(ctx_lens, dtype=np.int32)
    par = np.ascontiguousarray(tree_parent, dtype=np.int32)
    B, N = par.shape
    keep = [q, k_cache, v_cache, ctx, par]
    pt_ptr, max_pages = None, 0
    if page_table is not None:
        pt = np.ascontiguousarray(page_table, dtype=np.int32)
        keep.append(pt)
        pt_ptr, max_pages = pt.ctypes.data, pt.shape[1]
    p = _Problem(
        dtype=dtype, B=B, N=N, Hq=Hq, Hkv=Hkv, D=D, page_size=page_size, max_pages=max_pages,
        scale=float(scale), stride_page=stride_page, stride_head=stride_head,
        stride_token=stride_token, q=q.ctypes.data, k_cache=k_cache.ctypes.data,
        v_cache=v_cache.ctypes.data, page_table=pt_ptr, ctx_lens=ctx.ctypes.data,
        tree_parent=par.ctypes.data)
    return p, keep


def verify_attn(*, rows: Optional[np.ndarray] = None, chunk_tokens: int = 0, **kw) -> np.ndarray:
    """fp64 attention output: [B, N, Hq, D], or [n_rows, D] when ``rows`` (an
    int array of (b, i, h) triples) selects single output rows.  Keyword
    arguments are the fields of a verify step (see ``verify_attn_case``)."""
    lib = _load()
    p, keep = _problem(**kw)
    if rows is None:
        out = np.empty((p.B, p.N, p.Hq, p.D), dtype=np.float64)
        rc = lib.owl_oracle_verify_attn(ctypes.byref(p), None, 0, int(chunk_tokens), out.ctypes.data)
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
        out = np.empty((rows.shape[0], p.D), dtype=np.float64)
        rc = lib.owl_oracle_verify_attn(ctypes.byref(p), rows.ctypes.data, rows.shape[0],
                                        int(chunk_tokens), out.ctypes.data)
    del keep
    if rc:
        raise OracleError(rc)
    return out


def case_kwargs(case) -> dict:
    """Field mapping for any object carrying the attributes of a verify step
    (duck-typed; the oracle does not import the generator module)."""
    return dict(dtype=case.dtype, q=case.q, k_cache=case.k_pool, v_cache=case.v_pool,
                page_table=case.page_table, ctx_lens=case.ctx_lens, tree_parent=case.tree_parent,
                Hq=case.Hq, Hkv=case.Hkv, D=case.D, scale=case.scale,
                stride_page=case.stride_page, stride_head=case.stride_head,
                stride_token=case.stride_token)


def verify_attn_case(case, rows: Optional[np.ndarray] = None, chunk_tokens: int = 0) -> np.ndarray:
    return verify_attn(rows=rows, chunk_tokens=chunk_tokens, **case_kwargs(case))


def tree_mask(parent: np.ndarray):
    """(anc uint64 [N], depth int32 [N]) of one parent array."""
    lib = _load()
    par = np.ascontiguousarray(parent, dtype=np.int32)
    n = par.shape[0]
    anc = np.zeros(max(n, 1), dtype=np.uint64)
    depth = np.zeros(max(n, 1), dtype=np.int32)
    rc = lib.owl_oracle_tree_mask(par.ctypes.data, n, anc.ctypes.data, depth.ctypes.data)
    if rc:
        raise OracleError(rc)
    return anc[:n], depth[:n]


def gather_kv(case, which: str, b: int, first_pos: int, n_tokens: int) -> np.ndarray:
    """Rows first_pos.. of sequence b of the K ('k') or V ('v') cache in logical
    order, [n_tokens, Hkv, D], storage bits untouched."""
    lib = _load()
    p, keep = _problem(**case_kwargs(case))
    cache = keep[1] if which == "k" else keep[2]
    dst = np.empty((n_tokens, case.Hkv, case.D), dtype=cache.dtype)
    rc = lib.owl_oracle_gather_kv(ctypes.byref(p), cache.ctypes.data, b, first_pos, n_tokens,
                                  dst.ctypes.data)
    if rc:
        raise OracleError(rc)
    return dst


def verify_attn_ragged_case(case, n_draft_seq) -> np.ndarray:
    """A batch whose sequences carry different numbers of drafted tokens
    (Algorithm 1 of the paper mixes sequence and tree drafts): sequence b is
    verified on its own with the first n_draft_seq[b] nodes of its tree, i.e.
    the plain step with N = n_draft_seq[b]; output rows of absent nodes are
    zero.  Returns [B, N, Hq, D] (fp64)."""
    kw = case_kwargs(case)
    B, N = np.asarray(kw["tree_parent"]).shape
    out = np.zeros((B, N, kw["Hq"], kw["D"]), dtype=np.float64)
    for b in range(B):
        n = int(n_draft_seq[b])
        if not 0 <= n <= N:
            raise ValueError("n_draft_seq out of range")
        if n == 0:
            continue
        sub = dict(kw)
        sub["q"] = np.ascontiguousarray(np.asarray(kw["q"])[b:b + 1, :n])
        sub["tree_parent"] = np.ascontiguousarray(np.asarray(kw["tree_parent"])[b:b + 1, :n])
        sub["ctx_lens"] = np.asarray(kw["ctx_lens"])[b:b + 1]
        if kw["page_table"] is not None:
            sub["page_table"] = np.asarray(kw["page_table"])[b:b + 1]
        elif B != 1:
            raise ValueError("identity paging is defined for one sequence")
        out[b, :n] = verify_attn(**sub)[0]
    return out
