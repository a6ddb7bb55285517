"""GPU parity: fd_append_kv against oracle.attention.append_accepted_kv (bit-exact: it only moves
bytes), and a two-step loop - attend, accept, commit, attend again - against the oracle run on the
oracle's own committed cache."""
import numpy as np
import pytest
import torch

from oracle import attention as oa
from paper_2605_20022_amd import workloads as W
from tests.gpu_harness import AttnCall, assert_attn_close, from_dev

pytestmark = pytest.mark.gpu


def _with_room(inp, extra_tokens):
    """The same inputs with enough spare pages behind every sequence for `extra_tokens` more tokens."""
    ps = inp["k_cache"].shape[2]
    B = len(inp["kv_len"])
    lists, nxt = [], inp["k_cache"].shape[0]
    for i in range(B):
        own = list(inp["page_indices"][inp["page_indptr"][i]:inp["page_indptr"][i + 1]])
        need = (int(inp["kv_len"][i]) + extra_tokens + ps - 1) // ps
        while len(own) < need:
            own.append(nxt); nxt += 1
        lists.append(own)
    grow = nxt - inp["k_cache"].shape[0]
    out = dict(inp)
    if grow:
        rng = np.random.default_rng(3)
        for name in ("k_cache", "v_cache"):
            x = inp[name]
            draw = rng.standard_normal((grow,) + x.shape[1:]).astype(np.float32)
            filler = W.f32_to_bf16_bits(draw) if x.dtype == np.uint16 else draw
            out[name] = np.concatenate([x, filler])
    out["page_indices"] = np.concatenate(lists).astype(np.int32)
    out["page_indptr"] = np.concatenate([[0], np.cumsum([len(l) for l in lists])]).astype(np.int32)
    out["num_pages"] = nxt
    return out


@pytest.mark.parametrize("dtype,D,ps", [("bf16", 128, 16), ("f32", 64, 8), ("bf16", 64, 1)])
def test_append_matches_oracle(fd, dtype, D, ps):
    w = W.AttnWorkload("app", dtype, 7, 8, 2, D, ps, (0, 90), (1, 6), 3, 1.0, seed=81, spare_page_frac=0.2)
    inp = _with_room(W.make_attention_inputs(w), 9)
    rng = np.random.default_rng(5)
    n = np.diff(inp["row_indptr"])
    acc = np.array([rng.integers(0, k) for k in inp["verify_len"]], dtype=np.int32)       # 0 .. k_i - 1
    call = AttnCall(fd, inp)
    acc_d = torch.from_numpy(acc).cuda()
    new_len = torch.full((w.batch,), -5, dtype=torch.int32, device="cuda")
    fd.fd_append_kv(call.args, call.d["k_cache"], call.d["v_cache"], acc_d, new_len)
    torch.cuda.synchronize()
    assert int(call.status.item()) == 0
    kc, vc, ref_len = oa.append_accepted_kv(inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"],
                                            inp["page_indptr"], inp["page_indices"], inp["kv_len"],
                                            inp["row_indptr"], inp["verify_len"], acc, page_size=ps)
    as_bits = (lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)) if dtype == "bf16" else (lambda t: t.cpu().numpy())
    assert np.array_equal(as_bits(call.d["k_cache"]), kc)
    assert np.array_equal(as_bits(call.d["v_cache"]), vc)
    assert np.array_equal(new_len.cpu().numpy(), ref_len)
    # in place: the output may be the input array
    call2 = AttnCall(fd, inp)
    fd.fd_append_kv(call2.args, call2.d["k_cache"], call2.d["v_cache"], acc_d, call2.d["kv_len"])
    torch.cuda.synchronize()
    assert np.array_equal(call2.d["kv_len"].cpu().numpy(), ref_len)
    assert np.array_equal(as_bits(call2.d["k_cache"]), kc)


def test_append_reports_bad_device_data(fd):
    w = W.AttnWorkload("appbad", "bf16", 3, 8, 2, 128, 16, (10, 40), (2, 4), 2, 1.0, seed=82)
    inp = W.make_attention_inputs(w)                    # no spare room: kv 10..40 may fill its last page
    inp["kv_len"][:] = (np.diff(inp["page_indptr"]) * 16).astype(np.int32)   # every page list exactly full
    call = AttnCall(fd, inp)
    acc = torch.zeros(3, dtype=torch.int32, device="cuda")
    out_len = torch.zeros(3, dtype=torch.int32, device="cuda")
    before = call.d["k_cache"].clone()
    fd.fd_append_kv(call.args, call.d["k_cache"], call.d["v_cache"], acc, out_len)
    torch.cuda.synchronize()
    assert int(call.status.item()) & 4                   # FD_DEV_PAGE_RANGE: no page for the row
    assert torch.equal(before, call.d["k_cache"])        # nothing was written
    assert np.array_equal(out_len.cpu().numpy(), inp["kv_len"])
    call.status.zero_()
    acc[1] = int(inp["verify_len"][1])                   # one more than the verify rows: a mask row
    fd.fd_append_kv(call.args, call.d["k_cache"], call.d["v_cache"], acc, out_len)
    torch.cuda.synchronize()
    assert int(call.status.item()) & 2                   # FD_DEV_ROWS_RANGE


def test_append_never_commits_mask_rows(fd):
    """Sequences without verify rows (mask-only draft pass, Sec. 4.3) mixed with ordinary ones: the
    former keep their pages and lengths whatever accept_len holds (the acceptance calls give 0 for
    them); the others commit up to all k_i verify rows and never a mask row (Sec. 4.1: mask tokens
    stay invisible to the clean prefix)."""
    w = W.AttnWorkload("appmask", "bf16", 9, 8, 2, 128, 16, (5, 120), (0, 3), 4, 1.0, seed=84, spare_page_frac=0.2)
    inp = _with_room(W.make_attention_inputs(w), 8)
    k = inp["verify_len"]
    assert (k == 0).any() and (k > 0).any()
    acc = np.where(k > 0, k - 1, 0).astype(np.int32)     # every verify row; 0 where there is none
    call = AttnCall(fd, inp)
    new_len = torch.full((w.batch,), -5, dtype=torch.int32, device="cuda")
    fd.fd_append_kv(call.args, call.d["k_cache"], call.d["v_cache"], torch.from_numpy(acc).cuda(), new_len)
    torch.cuda.synchronize()
    assert int(call.status.item()) == 0
    kc, vc, ref_len = oa.append_accepted_kv(inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"],
                                            inp["page_indptr"], inp["page_indices"], inp["kv_len"],
                                            inp["row_indptr"], k, acc, page_size=16)
    bits = lambda t: t.view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(bits(call.d["k_cache"]), kc) and np.array_equal(bits(call.d["v_cache"]), vc)
    assert np.array_equal(new_len.cpu().numpy(), ref_len)
    assert np.array_equal(ref_len[k == 0], inp["kv_len"][k == 0])
    # an accept_len that reaches into the mask rows is clamped to the verify rows and reported
    call2 = AttnCall(fd, inp)
    bad = acc.copy(); bad[k > 0] += 2
    fd.fd_append_kv(call2.args, call2.d["k_cache"], call2.d["v_cache"], torch.from_numpy(bad).cuda(), new_len)
    torch.cuda.synchronize()
    assert int(call2.status.item()) & 2                  # FD_DEV_ROWS_RANGE
    assert np.array_equal(bits(call2.d["k_cache"]), kc) and np.array_equal(new_len.cpu().numpy(), ref_len)


def test_two_steps_of_the_loop(fd):
    """attend -> (pretend) accept -> commit -> attend again with fresh new rows: the second call's
    result must equal the oracle's on the oracle's committed cache."""
    w = W.AttnWorkload("loop", "bf16", 4, 8, 2, 128, 16, (30, 300), (4, 4), 4, 1.0, seed=83)
    inp = _with_room(W.make_attention_inputs(w), 8)
    acc = np.array([0, 3, 1, 2], dtype=np.int32)
    call = AttnCall(fd, inp)
    out1, _ = call.run()
    ref1, _ = oa.verify_draft_attention(inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"],
                                        inp["page_indptr"], inp["page_indices"], inp["kv_len"], inp["row_indptr"],
                                        inp["verify_len"], page_size=16)
    assert_attn_close(out1, ref1, "bf16", "loop step 1")
    fd.fd_append_kv(call.args, call.d["k_cache"], call.d["v_cache"], torch.from_numpy(acc).cuda(), call.d["kv_len"])
    kc, vc, len2 = oa.append_accepted_kv(inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"], inp["page_indptr"],
                                         inp["page_indices"], inp["kv_len"], inp["row_indptr"], inp["verify_len"], acc, page_size=16)
    # step 2: new rows drawn afresh, same row layout; the device call reuses the (now longer) cache
    rng = np.random.default_rng(7)
    step2 = dict(inp, k_cache=kc, v_cache=vc, kv_len=len2)
    for name in ("q", "k_new", "v_new"):
        step2[name] = W.f32_to_bf16_bits(rng.standard_normal(inp[name].shape).astype(np.float32))
        call.d[name].copy_(torch.from_numpy(step2[name].view(np.int16)).view(torch.bfloat16).cuda())
    call.args.max_kv_len = int(len2.max())
    out2, _ = call.run()
    ref2, _ = oa.verify_draft_attention(step2["q"], step2["k_new"], step2["v_new"], kc, vc, inp["page_indptr"],
                                        inp["page_indices"], len2, inp["row_indptr"], inp["verify_len"], page_size=16)
    assert_attn_close(out2, ref2, "bf16", "loop step 2")
