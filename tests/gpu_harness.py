"""Helpers for the GPU parity tests: move seeded host inputs to the device, call the
C-ABI through the binding, bring results back, and run the oracle on the same inputs
(or on a subset of the sequences when the full problem is too large for the CPU)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import acceptance as oc
from oracle import attention as oa


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


def subset_inputs(inp: dict, ids) -> dict:
    """The same problem restricted to sequences `ids` (caches and page ids untouched)."""
    ids = list(ids)
    rows = [np.arange(inp["row_indptr"][i], inp["row_indptr"][i + 1]) for i in ids]
    keep = np.concatenate(rows) if rows else np.zeros(0, dtype=np.int64)
    sub = dict(inp)
    for k in ("q", "k_new", "v_new"):
        sub[k] = inp[k][keep]
    sub["kv_len"] = inp["kv_len"][ids]
    sub["verify_len"] = inp["verify_len"][ids]
    if inp.get("mask_blocks") is not None:
        sub["mask_blocks"] = np.asarray(inp["mask_blocks"])[ids]
    sub["row_indptr"] = np.concatenate([[0], np.cumsum([len(r) for r in rows])]).astype(np.int32)
    pages = [inp["page_indices"][inp["page_indptr"][i]:inp["page_indptr"][i + 1]] for i in ids]
    sub["page_indices"] = np.concatenate(pages).astype(np.int32) if pages else np.zeros(0, dtype=np.int32)
    sub["page_indptr"] = np.concatenate([[0], np.cumsum([len(p) for p in pages])]).astype(np.int32)
    sub["_rows"] = keep
    return sub


def oracle_attention(inp: dict, mask_vis=None, sm_scale=None):
    ps = inp["k_cache"].shape[2]
    return oa.verify_draft_attention(
        inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"], inp["page_indptr"],
        inp["page_indices"], inp["kv_len"], inp["row_indptr"], inp["verify_len"], mask_vis,
        inp.get("mask_blocks"), page_size=ps, sm_scale=sm_scale)


def assert_attn_close(got, ref, dtype: str, what=""):
    """fp32: 1e-5 absolute.  bf16: 2e-2 absolute, and additionally 2e-2 of the largest
    reference magnitude so that the check keeps its teeth when outputs are small."""
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    if dtype == "f32":
        assert err.max() <= 1e-5, f"{what}: max |diff| {err.max():.3e} > 1e-5"
    else:
        bound = min(2e-2, 2e-2 * max(np.abs(ref).max(), 1e-30))
        assert err.max() <= bound, f"{what}: max |diff| {err.max():.3e} > {bound:.3e} (max |ref| {np.abs(ref).max():.3e})"
    return float(err.max())


def run_greedy(fd, logits: np.ndarray, row_indptr, tokens, *, vocab=None, want_argmax=True):
    B = len(row_indptr) - 1
    lg = to_dev(logits)
    Rv = lg.shape[0]
    ip = torch.from_numpy(np.asarray(row_indptr, dtype=np.int32)).cuda()
    tk = torch.from_numpy(np.asarray(tokens, dtype=np.int32)).cuda() if Rv else torch.zeros(1, dtype=torch.int32, device="cuda")
    acc = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    bon = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    am = torch.full((max(Rv, 1),), -7, dtype=torch.int32, device="cuda") if want_argmax else None
    V = lg.shape[1] if vocab is None else vocab
    ws = fd.alloc_workspace(fd.fd_accept_workspace(B, Rv, V, False))
    kmax = int(np.diff(row_indptr).max()) if B else 0
    fd.fd_accept_greedy(lg, ip, tk, acc, bon, vocab=V, max_rows_per_seq=kmax, row_argmax=am, workspace=ws)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), bon.cpu().numpy(), (None if am is None else am.cpu().numpy()[:Rv])


def run_draft_select(fd, logits: np.ndarray, row_indptr, temperature, threshold, *, vocab=None, want_conf=True):
    B = len(row_indptr) - 1
    lg = to_dev(logits)
    R = lg.shape[0]
    ip = torch.from_numpy(np.asarray(row_indptr, dtype=np.int32)).cuda()
    tok = torch.full((max(R, 1),), -7, dtype=torch.int32, device="cuda")
    conf = torch.full((max(R, 1),), -7.0, dtype=torch.float32, device="cuda") if want_conf else None
    keep = torch.full((max(B, 1),), -7, dtype=torch.int32, device="cuda")[:B]
    V = lg.shape[1] if vocab is None else vocab
    ws = fd.alloc_workspace(fd.fd_draft_select_workspace(R, V))
    kmax = int(np.diff(row_indptr).max()) if B else 0
    fd.fd_draft_select(lg, ip, tok, keep, temperature=temperature, threshold=threshold, max_rows_per_seq=kmax,
                       confidence=conf, vocab=V, workspace=ws)
    torch.cuda.synchronize()
    return tok.cpu().numpy()[:R], (None if conf is None else conf.cpu().numpy()[:R]), keep.cpu().numpy()


def run_sample(fd, target, draft, row_indptr, tokens, ua, ur, temperature, *, vocab=None):
    B = len(row_indptr) - 1
    tg, dr = to_dev(target), to_dev(draft)
    Rv = tg.shape[0]
    ip = torch.from_numpy(np.asarray(row_indptr, dtype=np.int32)).cuda()
    tk = torch.from_numpy(np.asarray(tokens, dtype=np.int32)).cuda()
    uat = torch.from_numpy(np.asarray(ua, dtype=np.float32)).cuda()
    urt = torch.from_numpy(np.asarray(ur, dtype=np.float32)).cuda()
    acc = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    bon = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    V = tg.shape[1] if vocab is None else vocab
    ws = fd.alloc_workspace(fd.fd_accept_workspace(B, Rv, V, True))
    kmax = int(np.diff(row_indptr).max()) if B else 0
    fd.fd_accept_sample(tg, dr, ip, tk, uat, urt, acc, bon, temperature=temperature, vocab=V,
                        max_rows_per_seq=kmax, workspace=ws)
    torch.cuda.synchronize()
    return acc.cpu().numpy(), bon.cpu().numpy()


# A decision of the sampling rule is held to exact agreement when the oracle's margin
# exceeds these bounds; below them fp32 exponentials cannot be expected to fall on the
# same side.  fp32 expf carries ~1e-7 relative error per term, p and q each take two of
# them plus a normaliser, hence 1e-5 on the accept ratio; the inverse-CDF position is a
# sum of ~1e5 such terms with independent errors, hence 1e-7 relative to the total weight.
ACCEPT_MARGIN = 1e-5
RESAMPLE_MARGIN = 1e-7


def compare_sampling(acc, bon, o_acc, o_bon, info, row_indptr, target, draft, tokens, ua, ur, temperature):
    """Exact agreement wherever the oracle's margins are clear; for a thin margin the GPU may
    land on the adjacent outcome, which is then re-derived with the oracle by nudging the
    uniform across the boundary.  Returns the number of thin-margin sequences."""
    thin = 0
    for i in range(len(row_indptr) - 1):
        r0, r1 = int(row_indptr[i]), int(row_indptr[i + 1])
        if r1 == r0:
            assert acc[i] == 0 and bon[i] == -1
            continue
        am = info["accept_margin"][r0:r1]
        am = am[~np.isnan(am)]
        clear = (am.size == 0 or am.min() > ACCEPT_MARGIN) and info["resample_margin"][i] > RESAMPLE_MARGIN
        if clear:
            assert acc[i] == o_acc[i] and bon[i] == o_bon[i], \
                f"seq {i}: gpu ({acc[i]},{bon[i]}) oracle ({o_acc[i]},{o_bon[i]}) margins {am.min() if am.size else None} {info['resample_margin'][i]}"
        else:
            thin += 1
            if acc[i] == o_acc[i] and bon[i] == o_bon[i]:
                continue
            # valid alternative: the result of the oracle with one uniform nudged by 4 margins
            ok = False
            for arr, scale in ((ua, 4 * ACCEPT_MARGIN), (ur, 4 * RESAMPLE_MARGIN)):
                for j in range(r0, r1):
                    for sgn in (-1.0, 1.0):
                        a2 = np.array(arr, dtype=np.float64)
                        a2[j] = min(max(a2[j] * (1 + sgn * scale) + sgn * 1e-12, 0.0), np.nextafter(1.0, 0.0))
                        args = (a2, ur) if arr is ua else (ua, a2)
                        oa2, ob2, _ = oc.accept_sample(target[r0:r1], draft[r0:r1], [0, r1 - r0], tokens[r0:r1],
                                                       np.asarray(args[0])[r0:r1], np.asarray(args[1])[r0:r1], temperature)
                        ok = ok or (oa2[0] == acc[i] and ob2[0] == bon[i])
            assert ok, f"seq {i}: gpu ({acc[i]},{bon[i]}) is not an outcome adjacent to the oracle's ({o_acc[i]},{o_bon[i]})"
    return thin
