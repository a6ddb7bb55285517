"""Pins for oracle/attention.py against things other than itself (CPU only).

Every check here states the expected result independently of the oracle's own
code path: hand-derived closed forms, explicitly listed visible sets, a library
attention routine called token by token, and algebraic invariants of the mask
rules of Sec. 4.1.
"""
import os

import numpy as np
import pytest
import torch

from oracle import attention as oa

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_case(seed, B=3, Hq=4, Hkv=2, D=8, ps=4, Ls=(5, 9, 0), ks=(2, 3, 1), ms=(3, 0, 2), shuffle=True):
    rng = np.random.default_rng(seed)
    Ls, ks, ms = list(Ls)[:B], list(ks)[:B], list(ms)[:B]
    rows = [k + m for k, m in zip(ks, ms)]
    row_indptr = np.concatenate([[0], np.cumsum(rows)]).astype(np.int32)
    npages = [(L + ps - 1) // ps for L in Ls]
    page_indptr = np.concatenate([[0], np.cumsum(npages)]).astype(np.int32)
    P = int(page_indptr[-1]) + 2
    page_indices = (rng.permutation(P)[:page_indptr[-1]] if shuffle else np.arange(page_indptr[-1])).astype(np.int32)
    R = int(row_indptr[-1])
    return dict(
        q=rng.standard_normal((R, Hq, D)), k_new=rng.standard_normal((R, Hkv, D)),
        v_new=rng.standard_normal((R, Hkv, D)),
        k_cache=rng.standard_normal((P, Hkv, ps, D)), v_cache=rng.standard_normal((P, Hkv, ps, D)),
        page_indptr=page_indptr, page_indices=page_indices,
        kv_len=np.array(Ls, dtype=np.int32), row_indptr=row_indptr,
        verify_len=np.array(ks, dtype=np.int32), page_size=ps)


def _run(c, **kw):
    args = dict(c); ps = args.pop("page_size")
    args.update(kw)
    return oa.verify_draft_attention(page_size=ps, **args)


def _logical_kv(c, i):
    """Prefix K/V of sequence i gathered by hand (independent of oracle.gather_prefix)."""
    ps = c["page_size"]; L = int(c["kv_len"][i])
    pages = c["page_indices"][c["page_indptr"][i]:c["page_indptr"][i + 1]]
    K = np.stack([c["k_cache"][pages[p // ps], :, p % ps, :] for p in range(L)]) if L else np.zeros((0,) + c["k_cache"].shape[1:2] + c["k_cache"].shape[3:])
    V = np.stack([c["v_cache"][pages[p // ps], :, p % ps, :] for p in range(L)]) if L else np.zeros_like(K)
    return K, V


def test_golden_log_keys():
    """Hand-derived closed form (tests/golden/attention_log_keys.txt)."""
    expect = {}
    for line in open(os.path.join(GOLDEN, "attention_log_keys.txt")):
        if line.startswith("v="):
            parts = line.split()
            expect[int(parts[0][2:])] = [float(x) for x in parts[1:]]
    assert set(expect) == {0, 1, 2}
    j = np.arange(1, 8, dtype=np.float64)
    keys, vals = np.log(j), j * j
    ps = 2
    k_cache = np.zeros((2, 1, ps, 1)); v_cache = np.zeros((2, 1, ps, 1))
    # logical tokens 0,1 in physical page 1, token 2 in physical page 0 (slot 1 of it is stale junk)
    k_cache[1, 0, :, 0] = keys[0:2]; v_cache[1, 0, :, 0] = vals[0:2]
    k_cache[0, 0, 0, 0] = keys[2];   v_cache[0, 0, 0, 0] = vals[2]
    k_cache[0, 0, 1, 0] = 50.0;      v_cache[0, 0, 1, 0] = -1e6
    for v, exp in expect.items():
        out, lse = oa.verify_draft_attention(
            q=np.ones((4, 1, 1)), k_new=keys[3:].reshape(4, 1, 1), v_new=vals[3:].reshape(4, 1, 1),
            k_cache=k_cache, v_cache=v_cache, page_indptr=[0, 2], page_indices=[1, 0],
            kv_len=[3], row_indptr=[0, 4], verify_len=[2], mask_vis=[v], page_size=ps, sm_scale=1.0)
        np.testing.assert_allclose(out[:, 0, 0], exp, rtol=1e-13)
    # log-sum-exp of verify row 0: ln(1+2+3+4)
    assert abs(lse[0, 0] - np.log(10.0)) < 1e-13


def test_softmax_rows_sum_to_one_and_constant_values():
    c = _rand_case(1)
    out, lse, probs = _run(c, return_probs=True)
    for _, _, P in probs:
        np.testing.assert_allclose(P.sum(axis=1), 1.0, atol=1e-12)
        assert (P >= 0).all()
    c2 = dict(c)
    c2["v_new"] = np.full_like(c["v_new"], 3.25); c2["v_cache"] = np.full_like(c["v_cache"], 3.25)
    out2, _ = _run(c2)
    np.testing.assert_allclose(out2, 3.25, atol=1e-12)


@pytest.mark.parametrize("vis_mode", ["default", "partial"])
def test_zero_query_gives_mean_over_visible_set(vis_mode):
    """Q = 0 makes every visible key equally weighted, so each output is the plain
    mean of V over the visible set; the sets are listed here from the paper's rules."""
    c = _rand_case(2)
    c["q"] = np.zeros_like(c["q"])
    mv = None if vis_mode == "default" else np.array([1, 0, 1], dtype=np.int32)
    out, _ = _run(c, mask_vis=mv)
    Hq, Hkv = c["q"].shape[1], c["k_new"].shape[1]
    G = Hq // Hkv
    for i in range(3):
        r0, r1 = c["row_indptr"][i], c["row_indptr"][i + 1]
        k = int(c["verify_len"][i]); n = r1 - r0
        v = k if mv is None else int(mv[i])
        _, Vc = _logical_kv(c, i)
        for r in range(n):
            if r < k:       # prefix + verify rows 0..r
                new_ids = list(range(0, r + 1))
            else:           # prefix + first v verify rows + the whole mask block
                new_ids = list(range(0, v)) + list(range(k, n))
            count = int(c["kv_len"][i]) + len(new_ids)
            assert count == (c["kv_len"][i] + r + 1 if r < k else c["kv_len"][i] + v + (n - k))
            for h in range(Hq):
                g = h // G
                pool = np.concatenate([Vc[:, g], c["v_new"][r0:r1][new_ids, g]], axis=0)
                assert pool.shape[0] == count
                np.testing.assert_allclose(out[r0 + r, h], pool.mean(axis=0), atol=1e-12)


def _sdpa(q, K, V, scale):
    """Library attention of one query over a key set, float64, no mask."""
    qt = torch.from_numpy(q).reshape(1, 1, 1, -1)
    Kt = torch.from_numpy(np.ascontiguousarray(K)).reshape(1, 1, K.shape[0], -1)
    Vt = torch.from_numpy(np.ascontiguousarray(V)).reshape(1, 1, V.shape[0], -1)
    return torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=scale).reshape(-1).numpy()


def test_rows_equal_library_attention_token_by_token():
    """Verify rows are ordinary causal decoding (Sec. 4.1: the clean path is the
    unchanged autoregressive computation); a mask row is unmasked attention over
    prefix + visible verify rows + its block."""
    c = _rand_case(3, Ls=(6, 10, 3), ks=(3, 2, 1), ms=(2, 4, 0))
    mv = np.array([2, 2, 1], dtype=np.int32)
    out, _ = _run(c, mask_vis=mv, sm_scale=0.37)
    Hq, Hkv = c["q"].shape[1], c["k_new"].shape[1]
    G = Hq // Hkv
    for i in range(3):
        r0, r1 = c["row_indptr"][i], c["row_indptr"][i + 1]
        k = int(c["verify_len"][i]); n = r1 - r0; v = int(mv[i])
        Kc, Vc = _logical_kv(c, i)
        for r in range(n):
            ids = list(range(r + 1)) if r < k else list(range(v)) + list(range(k, n))
            for h in range(Hq):
                g = h // G
                K = np.concatenate([Kc[:, g], c["k_new"][r0:r1][ids, g]])
                V = np.concatenate([Vc[:, g], c["v_new"][r0:r1][ids, g]])
                ref = _sdpa(c["q"][r0 + r, h], K, V, 0.37)
                np.testing.assert_allclose(out[r0 + r, h], ref, atol=1e-12)


def test_default_scale_is_inverse_sqrt_head_dim():
    c = _rand_case(4)
    a, _ = _run(c)
    b, _ = _run(c, sm_scale=1.0 / np.sqrt(c["q"].shape[2]))
    assert np.array_equal(a, b)
    # and the k = 1, m = 0 case is textbook single-token decoding
    c1 = _rand_case(5, B=1, Ls=(7,), ks=(1,), ms=(0,))
    o, _ = _run(c1)
    Kc, Vc = _logical_kv(c1, 0)
    for h in range(4):
        g = h // 2
        K = np.concatenate([Kc[:, g], c1["k_new"][:1, g]]); V = np.concatenate([Vc[:, g], c1["v_new"][:1, g]])
        np.testing.assert_allclose(o[0, h], _sdpa(c1["q"][0, h], K, V, 1 / np.sqrt(8)), atol=1e-12)


def test_verify_rows_blind_to_mask_tokens():
    """Mask tokens are invisible to clean tokens: changing their Q/K/V leaves every
    verify-row output bit-identical."""
    c = _rand_case(6)
    base, _ = _run(c)
    rng = np.random.default_rng(99)
    c2 = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in c.items()}
    is_verify = np.zeros(c["q"].shape[0], dtype=bool)
    for i in range(3):
        r0 = c["row_indptr"][i]; k = c["verify_len"][i]
        is_verify[r0:r0 + k] = True
    for name in ("q", "k_new", "v_new"):
        c2[name][~is_verify] += rng.standard_normal(c2[name][~is_verify].shape) * 5
    pert, _ = _run(c2)
    assert np.array_equal(base[is_verify], pert[is_verify])
    assert not np.allclose(base[~is_verify], pert[~is_verify])


def test_sequential_mode_is_row_selection():
    """Dropping the mask block (m = 0) reproduces the verify rows of the joint call
    (Fig. 2b: the sequential mode selects rows of the parallel mask)."""
    c = _rand_case(7)
    joint, jl = _run(c)
    keep = np.concatenate([np.arange(c["row_indptr"][i], c["row_indptr"][i] + c["verify_len"][i]) for i in range(3)])
    c2 = dict(c)
    for name in ("q", "k_new", "v_new"):
        c2[name] = c[name][keep]
    c2["row_indptr"] = np.concatenate([[0], np.cumsum(c["verify_len"])]).astype(np.int32)
    seq, sl = _run(c2)
    # (matrix shapes differ between the two calls, so the library products may round differently)
    np.testing.assert_allclose(seq, joint[keep], atol=1e-13)
    np.testing.assert_allclose(sl, jl[keep], atol=1e-13)


def test_block_is_bidirectional_permutation_equivariant():
    """Permuting the mask block's rows permutes their outputs and changes nothing else."""
    c = _rand_case(8, B=1, Ls=(9,), ks=(2,), ms=(4,))
    base, _ = _run(c)
    perm = np.array([0, 1, 4, 2, 5, 3])
    c2 = dict(c)
    for name in ("q", "k_new", "v_new"):
        c2[name] = c[name][perm]
    out, _ = _run(c2)
    np.testing.assert_allclose(out, base[perm], atol=1e-13)
    # whereas verify rows are order dependent (causal): swapping them changes row 0
    perm2 = np.array([1, 0, 2, 3, 4, 5])
    c3 = dict(c)
    for name in ("q", "k_new", "v_new"):
        c3[name] = c[name][perm2]
    out3, _ = _run(c3)
    assert not np.allclose(out3[1], base[0])


def test_mask_vis_limits_which_verify_rows_the_block_sees():
    """With v < k the block must not depend on verify rows v..k-1 (Eq. 2: a branch is
    conditioned on the first r drafts only)."""
    c = _rand_case(9, B=1, Ls=(5,), ks=(3,), ms=(2,))
    mv = np.array([1], dtype=np.int32)
    base, _ = _run(c, mask_vis=mv)
    c2 = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in c.items()}
    c2["k_new"][1:3] += 3.0; c2["v_new"][1:3] -= 2.0
    out, _ = _run(c2, mask_vis=mv)
    assert np.array_equal(out[3:], base[3:])
    c2["k_new"][0] += 3.0
    out, _ = _run(c2, mask_vis=mv)
    assert not np.allclose(out[3:], base[3:])


def test_paging_and_gqa_equivalences():
    c = _rand_case(10)
    shuffled, _ = _run(c)
    # same logical cache laid out contiguously
    ps = c["page_size"]
    c2 = dict(c)
    used = int(c["page_indptr"][-1])
    c2["k_cache"] = c["k_cache"][c["page_indices"]]; c2["v_cache"] = c["v_cache"][c["page_indices"]]
    c2["page_indices"] = np.arange(used, dtype=np.int32)
    contig, _ = _run(c2)
    assert np.array_equal(shuffled, contig)
    # grouped-query attention == multi-head attention with every KV head repeated G times
    G = c["q"].shape[1] // c["k_new"].shape[1]
    c3 = dict(c)
    for name in ("k_new", "v_new"):
        c3[name] = np.repeat(c[name], G, axis=1)
    for name in ("k_cache", "v_cache"):
        c3[name] = np.repeat(c[name], G, axis=1)
    mha, _ = _run(c3)
    assert np.array_equal(shuffled, mha)
    # stale slots past kv_len and spare pages are never read
    c4 = {k: (v.copy() if isinstance(v, np.ndarray) else v) for k, v in c.items()}
    for i in range(3):
        L = int(c["kv_len"][i]); pages = c["page_indices"][c["page_indptr"][i]:c["page_indptr"][i + 1]]
        if L % ps:
            c4["k_cache"][pages[-1], :, L % ps:, :] = 1e3; c4["v_cache"][pages[-1], :, L % ps:, :] = -1e3
    spare = np.setdiff1d(np.arange(c["k_cache"].shape[0]), c["page_indices"])
    c4["k_cache"][spare] = 1e3; c4["v_cache"][spare] = 1e3
    stale, _ = _run(c4)
    assert np.array_equal(shuffled, stale)


def test_bf16_widening_is_exact():
    bits = np.array([0x3F80, 0xBF80, 0x4049, 0x0000, 0x8000, 0x7F80, 0x0001, 0x3DCD], dtype=np.uint16)
    got = oa.widen_bf16(bits)
    exp = torch.tensor(bits.astype(np.int16)).view(torch.bfloat16).double().numpy()
    assert np.array_equal(got, exp)
    assert got[0] == 1.0 and got[1] == -1.0 and got[2] == 3.140625 and np.isinf(got[5])


# ---------------------------------------------------------------------------------------
# Several mask blocks per sequence (Sec. 3, parallel speculative decoding; Sec. 4.1: blocks
# are isolated from one another)
# ---------------------------------------------------------------------------------------
def _multi_block_case(seed, k=3, nb=3, mb=2, L=6):
    c = _rand_case(seed, B=1, Ls=(L,), ks=(k,), ms=(nb * mb,))
    return c, k, nb, mb


def test_blocks_visible_sets_by_q_zero():
    """Q = 0 makes every output the arithmetic mean of V over the visible set; the sets are
    written out here row by row, independently of oracle.visibility."""
    c, k, nb, mb = _multi_block_case(3)
    c["q"][:] = 0.0
    out, _ = _run(c, mask_blocks=[nb], mask_vis=[1])
    Kc, Vc = _logical_kv(c, 0)
    L = len(Vc)
    for h in range(c["q"].shape[1]):
        g = h // 2
        vals = np.concatenate([Vc[:, g], c["v_new"][:, g]])
        for r in range(k + nb * mb):
            if r < k:
                seen = list(range(L + r + 1))
            else:
                b = (r - k) // mb
                seen = list(range(L)) + [L + t for t in range(1 + b)] + [L + k + b * mb + j for j in range(mb)]
            np.testing.assert_allclose(out[r, h], vals[seen].mean(axis=0), atol=1e-12)


def test_each_block_equals_a_single_block_call():
    """Block b of a multi-block call == the (k, mb) single-block call fed that block's rows with
    mask_vis = first_vis + b: reduces the new rule to the single-block rule pinned above."""
    c, k, nb, mb = _multi_block_case(4, k=4, nb=3, mb=3, L=9)
    out, lse = _run(c, mask_blocks=[nb], mask_vis=[2])
    for b in range(nb):
        rows = list(range(k)) + list(range(k + b * mb, k + (b + 1) * mb))
        sub = dict(c)
        for name in ("q", "k_new", "v_new"):
            sub[name] = c[name][rows]
        sub["row_indptr"] = np.array([0, len(rows)], dtype=np.int32)
        o1, l1 = _run(sub, mask_vis=[min(2 + b, k)])
        np.testing.assert_allclose(out[rows], o1, atol=1e-12)
        np.testing.assert_allclose(lse[rows], l1, atol=1e-12)


def test_blocks_are_isolated_and_invisible_to_verify_rows():
    c, k, nb, mb = _multi_block_case(5, k=3, nb=3, mb=2)
    base, _ = _run(c, mask_blocks=[nb])
    pert = {n_: c[n_].copy() for n_ in ("q", "k_new", "v_new")}
    blk1 = slice(k + mb, k + 2 * mb)
    rng = np.random.default_rng(0)
    for n_ in pert:
        pert[n_][blk1] = rng.standard_normal(pert[n_][blk1].shape)
    moved, _ = _run(dict(c, **pert), mask_blocks=[nb])
    untouched = [r for r in range(k + nb * mb) if not (k + mb <= r < k + 2 * mb)]
    assert np.array_equal(base[untouched], moved[untouched])
    assert not np.array_equal(base[blk1], moved[blk1])


def test_default_first_visibility_lets_the_last_block_see_every_verify_row():
    c, k, nb, mb = _multi_block_case(6, k=3, nb=3, mb=2)
    a, _ = _run(c, mask_blocks=[nb])
    b, _ = _run(c, mask_blocks=[nb], mask_vis=[1])
    assert np.array_equal(a, b)                      # k - nb + 1 = 1
    one, _ = _run(c)                                  # one block of nb * mb rows sees all k rows
    explicit, _ = _run(c, mask_blocks=[1], mask_vis=[k])
    assert np.array_equal(one, explicit)
    with pytest.raises(ValueError):
        _run(c, mask_blocks=[4])                      # 6 mask rows do not split into 4 blocks


def test_select_branch():
    toks = np.arange(100, 100 + 12)                   # sequence 0: 3 blocks of 2; sequence 1: 2 blocks of 3
    indptr = [0, 6, 12]
    got = oa.select_branch(toks, indptr, [3, 2], accept_len=[1, 0], first_vis=[1, 2])
    assert got[0].tolist() == [102, 103]              # r = 1 accepted -> block 1 (drafted seeing 2 rows)
    assert got[1].tolist() == [106, 107, 108]         # r = 0 but the first block already assumes 1: clamped to block 0
    got = oa.select_branch(toks, indptr, [3, 2], accept_len=[9, 2], first_vis=[1, 2])
    assert got[0].tolist() == [104, 105] and got[1].tolist() == [109, 110, 111]


def test_append_accepted_kv_then_attend_equals_attending_with_the_rows_as_new_rows():
    """After committing the anchor and r accepted drafts, a plain decode query over the longer prefix
    must see exactly what a verify row r of the original call saw: prefix + new rows 0..r (causal).
    Independent of the append code: the expected value comes from the un-appended call."""
    ps = 4
    c = _rand_case(11, B=2, Ls=(5, 10), ks=(4, 3), ms=(2, 0), ps=ps)
    # give every sequence spare pages for the rows that may be committed
    pages = []
    extra = 2
    P0 = c["k_cache"].shape[0]
    rng = np.random.default_rng(2)
    grow = rng.standard_normal((2 * extra,) + c["k_cache"].shape[1:])
    c["k_cache"] = np.concatenate([c["k_cache"], grow]); c["v_cache"] = np.concatenate([c["v_cache"], grow * 0.5])
    new_indptr = [0]
    for i in range(2):
        own = list(c["page_indices"][c["page_indptr"][i]:c["page_indptr"][i + 1]]) + [P0 + i * extra + e for e in range(extra)]
        pages += own; new_indptr.append(len(pages))
    c["page_indices"] = np.array(pages, dtype=np.int32); c["page_indptr"] = np.array(new_indptr, dtype=np.int32)
    base, _ = _run(c)
    acc = [2, 0]
    kc, vc, new_len = oa.append_accepted_kv(c["k_cache"], c["v_cache"], c["k_new"], c["v_new"], c["page_indptr"],
                                            c["page_indices"], c["kv_len"], c["row_indptr"], c["verify_len"], acc, page_size=ps)
    assert new_len.tolist() == [5 + 3, 10 + 1]
    # untouched slots keep their values
    assert (kc != c["k_cache"]).any(axis=(1, 3)).sum() == 4          # 3 + 1 (page, slot) pairs rewritten
    for i in range(2):
        r = acc[i]                                                    # last committed row
        row = int(c["row_indptr"][i]) + r
        # the last committed row queried again as the only new row over the prefix before it
        d = dict(c, k_cache=kc, v_cache=vc,
                 kv_len=np.array([new_len[i] - 1], dtype=np.int32),
                 page_indptr=np.array([0, c["page_indptr"][i + 1] - c["page_indptr"][i]], dtype=np.int32),
                 page_indices=c["page_indices"][c["page_indptr"][i]:c["page_indptr"][i + 1]],
                 row_indptr=np.array([0, 1], dtype=np.int32), verify_len=np.array([1], dtype=np.int32),
                 q=c["q"][row:row + 1], k_new=c["k_new"][row:row + 1], v_new=c["v_new"][row:row + 1])
        got, _ = _run(d)
        np.testing.assert_allclose(got[0], base[row], atol=1e-12)
    for bad in ([6, 0], [4, 0], [0, 3], [-1, 0]):                     # only verify rows (4 and 3 of them) can be committed
        with pytest.raises(ValueError):
            oa.append_accepted_kv(c["k_cache"], c["v_cache"], c["k_new"], c["v_new"], c["page_indptr"], c["page_indices"],
                                  c["kv_len"], c["row_indptr"], c["verify_len"], bad, page_size=ps)
    # the largest legal count commits every verify row and never a mask row: the cache slots that
    # changed hold exactly the verify rows' keys
    kc2, _, len2 = oa.append_accepted_kv(c["k_cache"], c["v_cache"], c["k_new"], c["v_new"], c["page_indptr"],
                                         c["page_indices"], c["kv_len"], c["row_indptr"], c["verify_len"], [3, 2], page_size=ps)
    assert len2.tolist() == [5 + 4, 10 + 3]
    assert (kc2 != c["k_cache"]).any(axis=(1, 3)).sum() == 7


def test_append_skips_sequences_without_verify_rows():
    """A mask-only draft pass (Sec. 4.3, decoupled execution) has k = 0: nothing of it may reach the
    clean cache, whatever accept_len says (the acceptance calls return 0 for such a sequence)."""
    ps = 4
    c = _rand_case(12, B=2, Ls=(6, 3), ks=(0, 2), ms=(3, 2), ps=ps)
    P0 = c["k_cache"].shape[0]
    grow = np.random.default_rng(3).standard_normal((2,) + c["k_cache"].shape[1:])
    c["k_cache"] = np.concatenate([c["k_cache"], grow]); c["v_cache"] = np.concatenate([c["v_cache"], grow])
    pages, indptr = [], [0]
    for i in range(2):
        pages += list(c["page_indices"][c["page_indptr"][i]:c["page_indptr"][i + 1]]) + [P0 + i]
        indptr.append(len(pages))
    c["page_indices"] = np.array(pages, dtype=np.int32); c["page_indptr"] = np.array(indptr, dtype=np.int32)
    kc, vc, new_len = oa.append_accepted_kv(c["k_cache"], c["v_cache"], c["k_new"], c["v_new"], c["page_indptr"],
                                            c["page_indices"], c["kv_len"], c["row_indptr"], c["verify_len"], [0, 1], page_size=ps)
    assert new_len.tolist() == [6, 3 + 2]
    pg0 = c["page_indices"][c["page_indptr"][0]:c["page_indptr"][1]]
    assert np.array_equal(kc[pg0], c["k_cache"][pg0]) and np.array_equal(vc[pg0], c["v_cache"][pg0])
    assert (kc != c["k_cache"]).any(axis=(1, 3)).sum() == 2
