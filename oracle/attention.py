"""fp64 oracle for hybrid-mask verify+draft attention.  TEST INFRASTRUCTURE ONLY.

What is computed (paper, Sec. 4.1 "Attention Tuning" and "Inference", Fig. 2b
caption): one target forward pass carries, per sequence, k verify rows (the
anchor/bonus token followed by the previous draft) and a block of m mask
tokens.  Visibility rules, in the paper's words restated:

  * verify (clean) rows are processed exactly as the autoregressive model
    would process them: each sees the cached clean prefix and the verify rows
    up to and including itself; mask tokens are invisible to them;
  * a mask token sees the clean prefix and every token of its own block, in
    both directions.  "Clean prefix" for the block includes the first
    `mask_vis` verify rows of this step (the accepted-count hypothesis the
    block is drafted under, Eq. 2); the default is all k of them.

The result is the plain masked-softmax definition
    O[r] = sum_j softmax_j(scale * q_r . k_j  restricted to visible j) * v_j
written out densely in float64, one sequence and one head at a time.  There is
no tiling, no online softmax and no splitting here on purpose.

Pins (tests/test_oracle_attention.py): softmax rows sum to one; Q = 0 gives the
arithmetic mean of V over the visible set (visible sets written out
independently in the test); a closed-form worked example with logarithmic keys;
verify rows equal token-by-token causal attention computed with a library
routine; mask rows equal unmasked attention over prefix + visible verify rows +
block; invariance of verify rows under perturbation of mask-token Q/K/V;
permutation equivariance inside the block; paging and GQA equivalences.
"""
from __future__ import annotations

import numpy as np


def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> float64, exactly (bf16 is the top half of fp32)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    f32 = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return f32.astype(np.float64)


def to_f64(x: np.ndarray) -> np.ndarray:
    """Stored values widened exactly: uint16 arrays are bf16 bit patterns."""
    if x.dtype == np.uint16:
        return widen_bf16(x)
    return np.asarray(x, dtype=np.float64)


def visibility(L: int, k: int, m: int, v: int, nb: int = 1) -> np.ndarray:
    """Boolean [k+m, L+k+m]: may new row r look at key j?

    Keys 0..L-1 are the cached prefix, key L+t is new row t (verify rows first,
    then the mask rows).  Sec. 4.1: prefix visible to everyone; verify rows
    causal among themselves and blind to mask tokens; a mask row sees the verify
    rows its block is conditioned on and its whole block, both directions.

    The m mask rows form nb blocks of m/nb rows each (Sec. 3, parallel
    speculative decoding: one candidate block per hypothetical number of
    accepted drafts; Sec. 4.1: blocks are isolated from one another).  Block b
    is drafted under the hypothesis that the first v + b verify rows are the
    clean context (never more than all k of them).
    """
    if nb < 1 or m % nb:
        raise ValueError("the mask rows must split evenly into the blocks")
    if not (0 <= v <= k):
        raise ValueError("mask_vis must lie in [0, verify_len]")
    n = k + m
    mb = m // nb
    vis = np.zeros((n, L + n), dtype=bool)
    vis[:, :L] = True                       # cached clean prefix: every row sees it
    for r in range(n):
        for t in range(n):                  # new key t sits at column L + t
            if r < k:                       # verify row: causal, never a mask key
                vis[r, L + t] = t <= r
            else:                           # mask row of block b
                b = (r - k) // mb
                lo = k + b * mb
                vis[r, L + t] = (t < min(v + b, k)) or (lo <= t < lo + mb)
    return vis


def gather_prefix(cache: np.ndarray, page_ids: np.ndarray, L: int, page_size: int) -> np.ndarray:
    """cache [P, Hkv, page_size, D] (float64) -> [L, Hkv, D], token p taken from
    physical page page_ids[p // page_size], slot p % page_size."""
    Hkv, D = cache.shape[1], cache.shape[3]
    out = np.empty((L, Hkv, D), dtype=np.float64)
    for p in range(L):
        out[p] = cache[int(page_ids[p // page_size]), :, p % page_size, :]
    return out


def masked_softmax_attention(q, keys, vals, vis, scale):
    """q [n, D], keys/vals [J, D], vis [n, J] -> (O [n, D], P [n, J], lse [n]).

    The definition: scores, -inf where invisible, subtract the row maximum,
    exponentiate, normalise, weight the values.
    """
    s = scale * (q @ keys.T)
    s = np.where(vis, s, -np.inf)
    mx = s.max(axis=1, keepdims=True)
    e = np.exp(s - mx)
    z = e.sum(axis=1, keepdims=True)
    P = e / z
    return P @ vals, P, (mx[:, 0] + np.log(z[:, 0]))


def verify_draft_attention(q, k_new, v_new, k_cache, v_cache, page_indptr, page_indices,
                           kv_len, row_indptr, verify_len, mask_vis=None, mask_blocks=None, *,
                           page_size: int, sm_scale: float | None = None,
                           return_probs: bool = False):
    """Hybrid-mask attention for a ragged batch.

    q       [R, Hq, D]        packed new rows; sequence i owns rows
                              row_indptr[i]:row_indptr[i+1], verify rows first
    k_new, v_new [R, Hkv, D]  keys/values of the new rows (never in the cache)
    k_cache, v_cache [P, Hkv, page_size, D]
    page_indices[page_indptr[i]:page_indptr[i+1]]  physical pages of sequence i
    kv_len[i]                 cached prefix tokens L_i (new rows excluded)
    verify_len[i]             k_i;  m_i = rows_i - k_i
    mask_blocks[i]            number of mask blocks nb_i (default 1)
    mask_vis[i]               verify rows block 0 sees; block b sees b more
                              (default k_i - nb_i + 1: the last block sees all)

    uint16 arrays are bf16 bit patterns.  Returns (out [R,Hq,D], lse [R,Hq]) in
    float64, plus the list of per-(sequence, head) probability matrices when
    return_probs is set.
    """
    q = to_f64(q); k_new = to_f64(k_new); v_new = to_f64(v_new)
    k_cache = to_f64(k_cache); v_cache = to_f64(v_cache)
    R, Hq, D = q.shape
    Hkv = k_new.shape[1]
    if Hq % Hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    G = Hq // Hkv
    scale = (1.0 / np.sqrt(D)) if not sm_scale else float(sm_scale)
    B = len(kv_len)
    out = np.zeros((R, Hq, D), dtype=np.float64)
    lse = np.zeros((R, Hq), dtype=np.float64)
    probs = []
    for i in range(B):
        r0, r1 = int(row_indptr[i]), int(row_indptr[i + 1])
        n = r1 - r0
        if n == 0:
            continue
        L = int(kv_len[i]); k = int(verify_len[i]); m = n - k
        if m < 0:
            raise ValueError("verify_len exceeds the sequence's row count")
        nb = 1 if mask_blocks is None else int(mask_blocks[i])
        v = max(k - nb + 1, 0) if mask_vis is None else int(mask_vis[i])
        pages = np.asarray(page_indices[int(page_indptr[i]):int(page_indptr[i + 1])])
        Kc = gather_prefix(k_cache, pages, L, page_size)
        Vc = gather_prefix(v_cache, pages, L, page_size)
        keys = np.concatenate([Kc, k_new[r0:r1]], axis=0)      # [L+n, Hkv, D]
        vals = np.concatenate([Vc, v_new[r0:r1]], axis=0)
        vis = visibility(L, k, m, v, nb)
        for h in range(Hq):
            g = h // G
            O, P, l = masked_softmax_attention(q[r0:r1, h], keys[:, g], vals[:, g], vis, scale)
            out[r0:r1, h] = O
            lse[r0:r1, h] = l
            if return_probs:
                probs.append((i, h, P))
    if return_probs:
        return out, lse, probs
    return out, lse


def select_branch(block_tokens, block_indptr, mask_blocks, accept_len, first_vis):
    """Tokens of the candidate block that matches the verified outcome (Sec. 3,
    parallel speculative decoding: once the number of accepted drafts r is known,
    the branch drafted under that hypothesis is kept).

    block_tokens[block_indptr[i]:block_indptr[i+1]] holds sequence i's nb_i blocks
    of equal length back to back; block b was drafted with first_vis[i] + b verify
    rows visible, i.e. (anchor row included) under the hypothesis of
    first_vis[i] + b - 1 accepted drafts.  Returns a list of arrays, one per
    sequence; the index is clamped to the blocks that exist.
    """
    out = []
    for i in range(len(accept_len)):
        toks = np.asarray(block_tokens[int(block_indptr[i]):int(block_indptr[i + 1])])
        nb = int(mask_blocks[i])
        if nb < 1 or len(toks) % nb:
            raise ValueError("tokens must split evenly into the blocks")
        mb = len(toks) // nb
        b = int(accept_len[i]) + 1 - int(first_vis[i])
        b = min(max(b, 0), nb - 1)
        out.append(toks[b * mb:(b + 1) * mb].copy())
    return out


def append_accepted_kv(k_cache, v_cache, k_new, v_new, page_indptr, page_indices, kv_len, row_indptr,
                       verify_len, accept_len, *, page_size: int):
    """Make the verified rows part of the clean prefix (Sec. 4.3, decoupled execution: the KV cache
    written by target verification is what the next draft step reuses).

    Sequence i commits its anchor row and its first accept_len[i] drafts, i.e. new rows
    0 .. accept_len[i] (the bonus token has no K/V yet: it is the next step's anchor).  Only verify
    rows can be committed: mask tokens must stay invisible to the clean prefix (Sec. 4.1), so a
    sequence with no verify row (a mask-only draft pass, Sec. 4.3) commits nothing and
    accept_len[i] must stay below verify_len[i].  Row j goes
    to logical position kv_len[i] + j: page page_indices[page_indptr[i] + pos // page_size], slot
    pos % page_size.  Works on copies; returns (k_cache, v_cache, new kv_len).  Arrays keep their
    dtype (bf16 bit patterns are moved as they are).
    """
    kc, vc = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    new_len = np.array(kv_len, dtype=np.int32, copy=True)
    for i in range(len(kv_len)):
        r0, n = int(row_indptr[i]), int(row_indptr[i + 1]) - int(row_indptr[i])
        k = int(verify_len[i])
        if n == 0 or k == 0:
            continue
        take = int(accept_len[i]) + 1
        if take < 1 or take > k:
            raise ValueError("only the sequence's verify rows can be committed")
        pages = np.asarray(page_indices[int(page_indptr[i]):int(page_indptr[i + 1])])
        for j in range(take):
            pos = int(kv_len[i]) + j
            if pos // page_size >= len(pages):
                raise ValueError("the page list has no room for the committed rows")
            pg = int(pages[pos // page_size])
            kc[pg, :, pos % page_size, :] = k_new[r0 + j]
            vc[pg, :, pos % page_size, :] = v_new[r0 + j]
        new_len[i] += take
    return kc, vc, new_len
