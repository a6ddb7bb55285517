"""Helpers for the GPU parity tests: move seeded host inputs to the device, call the
C-ABI through the binding, bring results back, and run the oracle on the same inputs
(or on a subset of the sequences when the full problem is too large for the CPU)."""
from __future__ import annotations

import numpy as np
import torch

from oracle import acceptance as oc
from oracle import attention as oa
from paper_2605_20022_amd.devcall import AttnCall, from_dev, to_dev  # noqa: F401  (re-exported for the tests)
from paper_2605_20022_amd.workloads import subset_inputs  # noqa: F401


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
