"""Device residency for one verify step: uploads a ``workloads.Case`` once,
owns the output / workspace / status buffers, and calls the C ABI.  Only
memory management and argument marshalling happen here."""
from __future__ import annotations

from typing import Optional

import numpy as np
import torch

from . import binding as B
from . import workloads as W


def _to_dev(a: np.ndarray, device) -> torch.Tensor:
    """Upload without reinterpreting bits (uint16 carries bf16/f16 patterns)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).to(device)
    return torch.from_numpy(a).to(device)


class VerifyStep:
    def __init__(self, case: W.Case, device: str = "cuda:0", split_tokens: int = 0,
                 max_ctx_len: Optional[int] = None, out_dtype: int = B.OWL_F32, flags: int = 0):
        self.case = case
        self.device = torch.device(device)
        self.q = _to_dev(case.q, self.device)
        self.k = _to_dev(case.k_pool, self.device)
        self.v = _to_dev(case.v_pool, self.device)
        self.page_table = None if case.page_table is None else _to_dev(case.page_table, self.device)
        self.ctx_lens = _to_dev(case.ctx_lens, self.device)
        self.tree_parent = _to_dev(np.ascontiguousarray(case.tree_parent), self.device)
        self.out = torch.empty((case.B, case.N, case.Hq, case.D), device=self.device,
                               dtype=torch.float32 if out_dtype == B.OWL_F32 else torch.int16)
        self.status = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.desc = B.make_desc(
            batch=case.B, n_draft=case.N, n_q_heads=case.Hq, n_kv_heads=case.Hkv, head_dim=case.D,
            max_pages_per_seq=case.max_pages_per_seq,
            max_ctx_len=case.max_ctx_len if max_ctx_len is None else max_ctx_len,
            qkv_dtype=case.dtype, scale=case.scale, kv_stride_page=case.stride_page,
            kv_stride_head=case.stride_head, kv_stride_token=case.stride_token,
            n_pool_pages=case.n_pool_pages, split_tokens=split_tokens, out_dtype=out_dtype, flags=flags)
        self.plan = B.owl_verify_attn_plan(self.desc)
        self.workspace = torch.empty(max(self.plan.workspace_bytes, 256), dtype=torch.uint8,
                                     device=self.device)

    def run(self, k=None, v=None, page_table=None, stream: Optional[int] = None,
            phases: int = B.PHASE_ALL) -> torch.Tensor:
        """One verify step.  ``k``/``v``/``page_table`` let a caller rotate
        through several resident copies of the cache; ``phases`` selects the
        split-KV pass and/or the combine (measurement only)."""
        args = (self.desc, self.q, self.k if k is None else k, self.v if v is None else v,
                self.page_table if page_table is None else page_table,
                self.ctx_lens, self.tree_parent, self.out, self.workspace, self.status)
        if phases == B.PHASE_ALL:
            B.owl_verify_attn(*args, stream=stream)
        else:
            B.owl_verify_attn_phases(*args, stream=stream, phases=phases)
        return self.out

    def run_split_timed(self, timer, k=None, v=None, stream: Optional[int] = None) -> None:
        """The split-KV pass alone with ``timer``'s events attached to the kernel's dispatch (measurement)."""
        B.owl_verify_attn_split_timed(self.desc, self.q, self.k if k is None else k, self.v if v is None else v,
                                      self.page_table, self.ctx_lens, self.tree_parent, self.out, self.workspace,
                                      timer, self.status, stream=stream)

    def result(self) -> np.ndarray:
        """``out`` on the host: float32, or the uint16 bit patterns of a 16-bit output type."""
        torch.cuda.synchronize(self.device)
        a = self.out.cpu().numpy()
        return a if a.dtype == np.float32 else a.view(np.uint16)

    def dev_status(self) -> int:
        torch.cuda.synchronize(self.device)
        return int(self.status.item())


class DrafterStep:
    """Device residency for one step of the drafter's cell on a ``workloads.DrafterCase``."""

    def __init__(self, case: W.DrafterCase, alpha: float, device: str = "cuda:0", tiled: bool = True):
        self.case = case
        self.device = torch.device(device)
        up = lambda a: None if a is None else _to_dev(np.ascontiguousarray(a), self.device)
        self.h, self.z, self.w, self.emb = up(case.h), up(case.z), up(case.W), up(case.E)
        self.tokens, self.parent_row = up(case.tokens), up(case.parent_row)
        self.gamma_c, self.beta_c = up(case.gamma_c), up(case.beta_c)
        self.gamma_z, self.beta_z = up(case.gamma_z), up(case.beta_z)
        self.h_out = torch.zeros((case.M, case.d), dtype=torch.int16, device=self.device)
        self.h_out_f32 = torch.zeros((case.M, case.d), dtype=torch.float32, device=self.device)
        self.z_out = torch.zeros((case.M, case.d), dtype=torch.float32, device=self.device)
        self.status = torch.zeros(1, dtype=torch.int32, device=self.device)
        self.desc = B.DrafterDesc(d_in=case.d_in, d=case.d, n_states=case.P, n_rows=case.M, vocab=case.vocab,
                                  dtype=case.dtype, alpha=alpha, eps=case.eps,
                                  w_layout=B.OWL_W_TILED if tiled else B.OWL_W_ROWS)
        if tiled:                                            # the library's own one-time re-layout of the weights
            self.w_rows = self.w
            self.w = torch.empty(B.owl_drafter_tiled_weight_bytes(self.desc), dtype=torch.uint8, device=self.device)
            B.owl_drafter_tile_weights(self.desc, self.w_rows, self.w)
        self.workspace = torch.empty(B.owl_drafter_cell_workspace_size(self.desc), dtype=torch.uint8,
                                     device=self.device)

    def run(self, w=None, stream: Optional[int] = None, phases: int = B.OWL_DRAFTER_ALL) -> None:
        """``w`` lets a caller rotate through several resident copies of the weights."""
        args = (self.desc, self.h, self.z, self.tokens, self.parent_row, self.w if w is None else w, self.emb,
                self.gamma_c, self.beta_c, self.gamma_z, self.beta_z, self.h_out, self.h_out_f32, self.z_out,
                self.workspace, self.status)
        if phases == B.OWL_DRAFTER_ALL:
            B.owl_drafter_cell(*args, stream=stream)
        else:
            B.owl_drafter_cell_phases(*args, stream=stream, phases=phases)

    def result(self):
        """(h' float32, h' in the storage type as uint16 bits, z' float32) as numpy arrays."""
        torch.cuda.synchronize(self.device)
        return (self.h_out_f32.cpu().numpy(), self.h_out.cpu().numpy().view(np.uint16), self.z_out.cpu().numpy())

    def dev_status(self) -> int:
        torch.cuda.synchronize(self.device)
        return int(self.status.item())
