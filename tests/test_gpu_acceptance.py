"""GPU parity: fd_accept_greedy / fd_accept_sample (through the C ABI) against the oracle.

Greedy results are integers and must match bit for bit, ties included (lowest index).
Sampling decisions are compared exactly wherever the oracle's decision margin is above
what fp32 exponentials can resolve (gpu_harness.ACCEPT_MARGIN / RESAMPLE_MARGIN); a
thin-margin decision may land on the adjacent outcome, which is verified to be adjacent.
"""
import numpy as np
import pytest
import torch

from oracle import acceptance as oc
from paper_2605_20022_amd import workloads as W
from tests.gpu_harness import compare_sampling, run_draft_select, run_greedy, run_sample

pytestmark = pytest.mark.gpu


def _greedy_case(fd, logits, indptr, toks, **kw):
    acc, bon, am = run_greedy(fd, logits, indptr, toks, **kw)
    V = kw.get("vocab")
    ref_logits = logits if V is None else logits[:, :V]
    o_acc, o_bon, o_am = oc.accept_greedy(ref_logits, indptr, toks)
    assert np.array_equal(am, o_am), "row arg-max differs"
    assert np.array_equal(acc, o_acc) and np.array_equal(bon, o_bon)
    return o_acc, o_bon, o_am


def test_cfg1_greedy_fp32_vocab_1000(fd):
    """4 verify rows; drafts 1 and 2 equal the target arg-max, draft 3 is random."""
    _, a = W.CONFIGS["cfg1"]
    lg = W.make_logits(a, 4)["target_logits"]
    _, _, am = oc.accept_greedy(lg, [0, 4], [0, 0, 0, 0])
    rng = np.random.default_rng(a.seed)
    toks = np.array([5, am[0], am[1], (am[2] + 1 + rng.integers(0, 998)) % 1000], dtype=np.int32)
    o_acc, o_bon, _ = _greedy_case(fd, lg, [0, 4], toks)
    assert o_acc[0] == 2 and o_bon[0] == am[2]           # committed length 3


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_greedy_ties_ragged_and_edges(fd, dtype):
    rng = np.random.default_rng(3)
    for V in (1, 7, 513, 4099, 20000):
        ks = [0, 1, 3, 70, 2, 0, 5]
        indptr = np.concatenate([[0], np.cumsum(ks)]).astype(np.int32)
        Rv = int(indptr[-1])
        # coarse grid of values => many exact ties, including at the maximum; some -inf
        vals = rng.integers(-4, 5, size=(Rv, V)).astype(np.float32) * 0.5
        vals[rng.random((Rv, V)) < 0.05] = -np.inf
        vals[3] = -np.inf; vals[3, V - 1] = -1.0       # maximum in the very last slot
        vals[4] = 2.0                                   # whole row tied: index 0 wins
        logits = W.f32_to_bf16_bits(vals) if dtype == "bf16" else vals
        _, _, am = oc.accept_greedy(logits, indptr, np.zeros(Rv, dtype=np.int64))
        toks = rng.integers(0, V, size=Rv)
        agree = rng.random(Rv) < 0.8
        toks[1:][agree[:-1]] = am[:-1][agree[:-1]]
        _greedy_case(fd, logits, indptr, toks.astype(np.int32))


def test_greedy_row_stride_and_unaligned_rows(fd):
    """vocab smaller than the row pitch, and an odd pitch that breaks 16-byte row alignment."""
    rng = np.random.default_rng(8)
    vals = rng.standard_normal((6, 1003)).astype(np.float32)
    logits = W.f32_to_bf16_bits(vals)
    toks = rng.integers(0, 990, size=6).astype(np.int32)
    _greedy_case(fd, logits, [0, 2, 6], toks, vocab=990)
    _greedy_case(fd, vals, [0, 2, 6], toks, vocab=1001)


def test_cfg3_greedy_vocab_151936(fd):
    w, a = W.CONFIGS["cfg3"]
    lens = W.make_lengths(w)
    indptr = W.verify_row_indptr(lens)
    lg = W.make_logits(a, int(indptr[-1]))["target_logits"]
    _, _, am = oc.accept_greedy(lg, indptr, np.zeros(int(indptr[-1]), dtype=np.int64))
    toks = W.make_draft_tokens_agreeing(a, indptr, am)
    o_acc, _, _ = _greedy_case(fd, lg, indptr, toks)
    # the workload really exercises the tie-break and a spread of accepted lengths
    f = (lg.astype(np.uint32) << 16).view(np.float32)
    ties = int(((f == f.max(axis=1, keepdims=True)).sum(axis=1) > 1).sum())
    assert ties >= 1 and len(set(o_acc.tolist())) >= 3


def _sampling_inputs(a, indptr, T):
    Rv = int(indptr[-1])
    lg = W.make_logits(a, Rv)

    def q_row(j):
        return oc.softmax64(oc.to_f64(lg["draft_logits"][j]) / T)
    toks = W.make_draft_tokens_from_probs(a, indptr, q_row)
    return lg, toks


def _sample_case(fd, a, indptr, T):
    lg, toks = _sampling_inputs(a, indptr, T)
    acc, bon = run_sample(fd, lg["target_logits"], lg["draft_logits"], indptr, toks, lg["u_accept"], lg["u_resample"], T)
    o_acc, o_bon, info = oc.accept_sample(lg["target_logits"], lg["draft_logits"], indptr, toks,
                                          lg["u_accept"], lg["u_resample"], T)
    thin = compare_sampling(acc, bon, o_acc, o_bon, info, indptr, lg["target_logits"], lg["draft_logits"], toks,
                            lg["u_accept"], lg["u_resample"], T)
    return o_acc, thin


@pytest.mark.parametrize("dtype,V,T", [("f32", 50, 1.0), ("bf16", 1000, 0.7), ("bf16", 5003, 1.0), ("f32", 20011, 1.3)])
def test_sampling_small_vocabularies(fd, dtype, V, T):
    a = W.AcceptWorkload("s", dtype, V, "sample", 2.0, draft_noise_std=0.7, temperature=T, seed=77 + V)
    ks = [3, 0, 1, 9, 17, 2]
    indptr = np.concatenate([[0], np.cumsum(ks)]).astype(np.int32)
    o_acc, thin = _sample_case(fd, a, indptr, T)
    assert thin <= 1


def test_sampling_degenerate_distributions(fd):
    """p == q: everything is kept.  Drafter one-hot on a token the target gives zero mass: rejected at once."""
    V = 300
    rng = np.random.default_rng(2)
    x = rng.standard_normal((4, V)).astype(np.float32)
    toks = rng.integers(0, V, size=4).astype(np.int32)
    ua = np.full(4, 0.999, dtype=np.float32); ur = rng.random(4).astype(np.float32)
    acc, bon = run_sample(fd, x, x.copy(), [0, 4], toks, ua, ur, 1.0)
    o_acc, o_bon, _ = oc.accept_sample(x, x, [0, 4], toks, ua, ur, 1.0)
    assert acc[0] == 3 == o_acc[0] and bon[0] == o_bon[0]
    xt = x.copy(); xd = np.full((4, V), -np.inf, dtype=np.float32)
    xt[0, 17] = -np.inf; xd[:, 17] = 0.0
    toks2 = np.array([0, 17, 17, 17], dtype=np.int32)
    acc, bon = run_sample(fd, xt, xd, [0, 4], toks2, np.zeros(4, dtype=np.float32), ur, 1.0)
    o_acc, o_bon, _ = oc.accept_sample(xt, xd, [0, 4], toks2, np.zeros(4), ur, 1.0)
    assert acc[0] == 0 == o_acc[0] and bon[0] == o_bon[0] and bon[0] != 17


def test_cfg5_sampling_vocab_151936(fd):
    w, a = W.CONFIGS["cfg5"]
    lens = W.make_lengths(w)
    indptr = W.verify_row_indptr(lens)
    o_acc, thin = _sample_case(fd, a, indptr, a.temperature)
    assert thin <= 1
    assert o_acc.min() >= 0 and o_acc.max() <= 15


@pytest.mark.parametrize("B,V,dtype", [(4, 1048576, "bf16"), (65535, 5, "f32"), (6000, 97, "bf16")])
def test_acceptance_extreme_shapes(fd, B, V, dtype):
    """A vocabulary of 2^20 entries, the largest row count the entry points take (65535), thousands of
    ragged sequences: greedy, sampling and draft selection against the oracle."""
    rng = np.random.default_rng(B + V)
    ks = np.ones(B, dtype=np.int64) if B == 65535 else rng.integers(0, 12, size=B)
    if B == 4:
        ks = np.array([3, 0, 1, 5])
    indptr = np.concatenate([[0], np.cumsum(ks)]).astype(np.int32)
    Rv = int(indptr[-1])
    vals = (rng.standard_normal((Rv, V)) * 3).astype(np.float32)
    vals[Rv // 2, V - 1] = 50.0                          # a maximum in the very last slot
    logits = W.f32_to_bf16_bits(vals) if dtype == "bf16" else vals
    _, _, am = oc.accept_greedy(logits, indptr, np.zeros(Rv, dtype=np.int64))
    toks = rng.integers(0, V, size=Rv)
    agree = rng.random(Rv) < 0.8
    toks[1:][agree[:-1]] = am[:-1][agree[:-1]]
    _greedy_case(fd, logits, indptr, toks.astype(np.int32))
    a = W.AcceptWorkload("s", dtype, V, "sample", 2.0, draft_noise_std=0.7, temperature=0.8, seed=B)
    _, thin = _sample_case(fd, a, indptr, 0.8)
    assert thin <= max(1, Rv // 2000)
    lg = W.make_peaked_logits(V, Rv, seed=B, dtype=dtype, peak_lo=2.0, peak_hi=12.0)
    _draft_select_case(fd, lg, indptr, 1.0, 0.3)


def test_acceptance_argument_errors(fd):
    import torch
    lg = torch.zeros((2, 64), dtype=torch.float32, device="cuda")
    ip = torch.tensor([0, 2], dtype=torch.int32, device="cuda")
    tk = torch.zeros(2, dtype=torch.int32, device="cuda")
    acc = torch.zeros(1, dtype=torch.int32, device="cuda"); bon = torch.zeros(1, dtype=torch.int32, device="cuda")
    small = fd.alloc_workspace(0)[:16]
    with pytest.raises(fd.FlexDraftError) as e:
        fd.fd_accept_greedy(lg, ip, tk, acc, bon, max_rows_per_seq=2, workspace=small)
    assert e.value.code in (1, 3)
    ws = fd.alloc_workspace(fd.fd_accept_workspace(1, 2, 64, True))
    u = torch.zeros(2, dtype=torch.float32, device="cuda")
    with pytest.raises(fd.FlexDraftError) as e:
        fd.fd_accept_sample(lg, lg, ip, tk, u, u, acc, bon, temperature=0.0, max_rows_per_seq=2, workspace=ws)
    assert e.value.code == 1


def test_select_branch_matches_oracle(fd):
    """fd_select_branch against oracle.attention.select_branch on a ragged batch, including
    indices that need clamping and a sequence whose tokens do not split into its blocks."""
    from oracle import attention as oa
    rng = np.random.default_rng(9)
    B = 37
    nb = rng.integers(1, 6, size=B).astype(np.int32)
    mb = rng.integers(1, 17, size=B).astype(np.int32)
    lens = nb * mb
    lens[5] += 1 if nb[5] > 1 else 0                          # does not split evenly (when nb > 1)
    indptr = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    toks = rng.integers(0, 151936, size=int(indptr[-1])).astype(np.int32)
    acc = rng.integers(0, 8, size=B).astype(np.int32)
    fv = rng.integers(0, 4, size=B).astype(np.int32)
    stride = 16
    out = torch.full((B, stride), -7, dtype=torch.int32, device="cuda")
    blk = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    dev = lambda a: torch.from_numpy(a).cuda()
    fd.fd_select_branch(dev(toks), dev(indptr), dev(nb), dev(acc), out, first_vis=dev(fv), out_block=blk)
    torch.cuda.synchronize()
    got, gb = out.cpu().numpy(), blk.cpu().numpy()
    for i in range(B):
        if lens[i] % nb[i]:
            assert (got[i] == -1).all() and gb[i] == -1
            continue
        ref = oa.select_branch(toks[indptr[i]:indptr[i + 1]], [0, lens[i]], [nb[i]], [acc[i]], [fv[i]])
        m = lens[i] // nb[i]
        assert got[i, :m].tolist() == ref[0].tolist() and (got[i, m:] == -1).all()
        assert gb[i] == min(max(acc[i] + 1 - fv[i], 0), nb[i] - 1)
    # without first_vis the attention call's default applies: block 0 saw k - nb + 1 verify rows
    k = (nb + rng.integers(-1, 4, size=B)).clip(0).astype(np.int32)     # fewer blocks than verify rows, as many, more
    fd.fd_select_branch(dev(toks), dev(indptr), dev(nb), dev(acc), out, verify_len=dev(k), out_block=blk)
    torch.cuda.synchronize()
    got, gb = out.cpu().numpy(), blk.cpu().numpy()
    for i in range(B):
        if lens[i] % nb[i] == 0:
            ref = oa.select_branch(toks[indptr[i]:indptr[i + 1]], [0, lens[i]], [nb[i]], [acc[i]], [max(k[i] - nb[i] + 1, 0)])
            m = lens[i] // nb[i]
            assert got[i, :m].tolist() == ref[0].tolist()
            assert gb[i] == min(max(acc[i] + 1 - max(k[i] - nb[i] + 1, 0), 0), nb[i] - 1)
    with pytest.raises(fd.FlexDraftError):                 # neither first_vis nor verify_len
        fd.fd_select_branch(dev(toks), dev(indptr), dev(nb), dev(acc), out, out_block=blk)


def test_default_visibility_pairs_attention_with_branch_selection(fd):
    """Selective verification prunes the hypotheses (Sec. 4.3, Eq. 5): fewer candidate blocks than
    verify rows.  With the defaults of both calls (no mask_vis, no first_vis) block b is drafted
    seeing k - nb + 1 + b verify rows, and r accepted drafts must select the block that saw r + 1 of
    them.  Each block carries, as its 'tokens', the number of verify rows the oracle's visibility
    rule lets it see, so the selected block names the hypothesis it was drafted under."""
    from oracle import attention as oa
    B, k, nb, mb = 5, 6, 3, 2
    vis_rows = []
    for b in range(nb):
        vis = oa.visibility(0, k, nb * mb, k - nb + 1, nb)           # the attention call's default first_vis
        seen = int(vis[k + b * mb, :k].sum())                        # verify rows the block's first row sees
        vis_rows += [seen] * mb
    toks = np.tile(np.array(vis_rows, dtype=np.int32), B)
    indptr = np.arange(0, B * nb * mb + 1, nb * mb, dtype=np.int32)
    acc = np.array([3, 4, 5, 0, 5], dtype=np.int32)                  # accepted drafts; r + 1 rows are clean
    out = torch.full((B, mb), -7, dtype=torch.int32, device="cuda")
    dev = lambda a: torch.from_numpy(a).cuda()
    fd.fd_select_branch(dev(toks), dev(indptr), dev(np.full(B, nb, np.int32)), dev(acc), out,
                        verify_len=dev(np.full(B, k, np.int32)))
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for i in range(B):
        want = min(max(acc[i] + 1, k - nb + 1), k)                   # hypotheses below the pruned range clamp to block 0
        assert (got[i] == want).all(), (i, got[i], want)


# fp32 exponentials carry ~1e-6 relative error on a confidence (the exponent's argument is
# rounded at magnitude ~20) and a block multiplies up to 15 of them: a product within 1e-4 of
# the threshold may fall on either side.
DRAFT_MARGIN = 1e-4


def _draft_select_case(fd, logits, indptr, T, thr, **kw):
    tok, conf, keep = run_draft_select(fd, logits, indptr, T, thr, **kw)
    V = kw.get("vocab")
    ref = logits if V is None else logits[:, :V]
    o_tok, o_conf, o_keep, o_margin = oc.draft_select(ref, indptr, T, thr)
    assert np.array_equal(tok, o_tok), "draft token differs"
    if conf is not None:
        np.testing.assert_allclose(conf, o_conf, rtol=2e-5, atol=1e-30)
    # the kept length is an integer decided by a float comparison: exact where the oracle's
    # margin is resolvable in fp32, otherwise the neighbouring length is also a valid outcome
    firm = o_margin > DRAFT_MARGIN
    assert np.array_equal(keep[firm], o_keep[firm])
    if not firm.all():
        _, _, k_lo, _ = oc.draft_select(ref, indptr, T, thr * (1 + DRAFT_MARGIN))
        _, _, k_hi, _ = oc.draft_select(ref, indptr, T, thr * (1 - DRAFT_MARGIN))
        assert np.all((k_lo <= keep) & (keep <= k_hi))
    return o_tok, o_conf, o_keep


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_draft_select_small_and_edges(fd, dtype):
    rng = np.random.default_rng(21)
    for V in (1, 9, 700, 4099, 20000):
        ks = [0, 1, 7, 3, 0, 15, 2]
        indptr = np.concatenate([[0], np.cumsum(ks)]).astype(np.int32)
        lg = W.make_peaked_logits(V, int(indptr[-1]), seed=V, dtype=dtype, peak_lo=2.0, peak_hi=12.0)
        for T, thr in ((1.0, 0.3), (0.7, 0.05), (1.5, 0.9), (1.0, 0.0), (1.0, 1.5)):
            _, _, o_keep = _draft_select_case(fd, lg, indptr, T, thr)
            if thr == 0.0:
                assert np.array_equal(o_keep, ks)           # nothing pruned
            if thr > 1.0 and V > 1:
                assert not o_keep.any()                     # nothing survives
    # exact ties at the maximum (lowest index wins) and -inf entries
    vals = rng.integers(-3, 4, size=(12, 513)).astype(np.float32)
    vals[rng.random(vals.shape) < 0.1] = -np.inf
    vals[5] = -np.inf; vals[5, 512] = 0.5                   # one finite entry: confidence exactly 1
    logits = W.f32_to_bf16_bits(vals) if dtype == "bf16" else vals
    _draft_select_case(fd, logits, [0, 4, 4, 12], 1.0, 0.01)
    _draft_select_case(fd, logits, [0, 4, 4, 12], 1.0, 0.01, want_conf=False)


def test_draft_select_row_stride(fd):
    lg = W.make_peaked_logits(1003, 6, seed=5, dtype="f32")
    _draft_select_case(fd, lg, [0, 2, 6], 1.0, 0.2, vocab=1001)
    _draft_select_case(fd, W.f32_to_bf16_bits(lg), [0, 2, 6], 1.0, 0.2, vocab=990)


def test_draft_select_full_vocabulary(fd):
    """B = 32 blocks of 15 draft positions over the 151 936-entry vocabulary."""
    indptr = (np.arange(33) * 15).astype(np.int32)
    lg = W.make_peaked_logits(151936, 480, seed=77, dtype="bf16", peak_lo=10.0, peak_hi=20.0)
    _, o_conf, o_keep = _draft_select_case(fd, lg, indptr, 1.0, 0.3)
    assert 0 < o_keep.min() + 1 and o_keep.max() <= 15 and len(set(o_keep.tolist())) > 3
    assert o_conf.min() < 0.5 < o_conf.max()


def test_draft_select_argument_errors(fd):
    lg = torch.zeros(4, 100, device="cuda")
    ip = torch.tensor([0, 4], dtype=torch.int32, device="cuda")
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    keep = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = fd.alloc_workspace(fd.fd_draft_select_workspace(4, 100))
    kw = dict(max_rows_per_seq=4, workspace=ws)
    with pytest.raises(fd.FlexDraftError):
        fd.fd_draft_select(lg, ip, tok, keep, temperature=0.0, threshold=0.3, **kw)
    with pytest.raises(fd.FlexDraftError):
        fd.fd_draft_select(lg, ip, tok, keep, temperature=1.0, threshold=float("nan"), **kw)
    with pytest.raises(fd.FlexDraftError):
        fd.fd_draft_select(lg, ip, tok, keep, temperature=1.0, threshold=0.3, max_rows_per_seq=4,
                           workspace=ws[:16])
    fd.fd_draft_select(lg, ip, tok, keep, temperature=1.0, threshold=0.3, **kw)
    torch.cuda.synchronize()
    assert keep.item() == 0 and tok.tolist() == [0, 0, 0, 0]   # uniform rows: p = 1/100 < 0.3
