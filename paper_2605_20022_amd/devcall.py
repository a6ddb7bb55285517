"""Device-side marshalling shared by the tests and the benchmark: move seeded host inputs to the
GPU, fill the C-ABI argument struct, bring results back.  No arithmetic of the method and nothing
of the oracle lives here."""
from __future__ import annotations

import numpy as np
import torch


def to_dev(x: np.ndarray, bf16: bool = False) -> torch.Tensor:
    if x.dtype == np.uint16:                         # bf16 bit patterns
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def from_dev(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float64 / int64 host array (bf16 widened exactly)."""
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy().astype(np.float64)
    if t.dtype == torch.float32:
        return t.cpu().numpy().astype(np.float64)
    return t.cpu().numpy()


class AttnCall:
    """Device-resident inputs/outputs of one fd_verify_draft_attn call."""

    def __init__(self, fd, inp: dict, *, mask_vis=None, flags=0, kv_chunk=0, sm_scale=0.0, want_lse=True,
                 max_kv_len=None, max_new_rows=None):
        self.fd = fd
        self.inp = inp
        d = {k: to_dev(inp[k]) for k in ("q", "k_new", "v_new", "k_cache", "v_cache")}
        for k in ("page_indptr", "page_indices", "kv_len", "row_indptr", "verify_len"):
            d[k] = torch.from_numpy(np.ascontiguousarray(inp[k], dtype=np.int32)).cuda()
        if d["page_indices"].numel() == 0:
            d["page_indices"] = torch.zeros(1, dtype=torch.int32, device="cuda")
        d["mask_vis"] = None if mask_vis is None else torch.from_numpy(np.asarray(mask_vis, dtype=np.int32)).cuda()
        mb = inp.get("mask_blocks")
        d["mask_blocks"] = None if mb is None else torch.from_numpy(np.asarray(mb, dtype=np.int32)).cuda()
        self.d = d
        R, Hq, D = d["q"].shape
        self.out = torch.full((R, Hq, D), float("nan"), dtype=d["q"].dtype, device="cuda")
        self.lse = torch.full((R, Hq), float("nan"), dtype=torch.float32, device="cuda") if want_lse else None
        self.status = torch.zeros(1, dtype=torch.int32, device="cuda")
        rows = np.diff(inp["row_indptr"])
        self.max_kv_len = int(inp["kv_len"].max()) if max_kv_len is None and len(inp["kv_len"]) else (max_kv_len or 0)
        self.max_new_rows = int(rows.max()) if max_new_rows is None and len(rows) else (max_new_rows or 0)
        self.args = fd.make_attn_args(
            d["q"], d["k_new"], d["v_new"], d["k_cache"], d["v_cache"], d["page_indptr"], d["page_indices"],
            d["kv_len"], d["row_indptr"], d["verify_len"], d["mask_vis"], d["mask_blocks"], out=self.out, lse=self.lse,
            max_kv_len=self.max_kv_len, max_new_rows=self.max_new_rows, sm_scale=sm_scale, flags=flags,
            kv_chunk=kv_chunk, status=self.status)
        need = fd.fd_verify_draft_attn_workspace(self.args)
        self.workspace = fd.alloc_workspace(need)
        self.args.workspace = self.workspace.data_ptr()
        self.args.workspace_bytes = self.workspace.numel()

    def run(self):
        self.fd.fd_verify_draft_attn(self.args)
        torch.cuda.synchronize()
        assert int(self.status.item()) == 0, f"device status word {int(self.status.item())}"
        return from_dev(self.out), (None if self.lse is None else from_dev(self.lse))
