"""fp64 oracle for the lossless acceptance step.  TEST INFRASTRUCTURE ONLY.

Sec. 3 (preliminaries): the target verifies the k drafted tokens of a step with
speculative sampling -- a drafted token is kept according to the ratio between
the target distribution p and the drafter distribution q, and at the first
rejected position a token is drawn from the residual target distribution; that
token is the bonus token; with r_acc drafts kept the step commits
L_acc = r_acc + 1 tokens.

Row convention used by the whole build: sequence i feeds k_i verify rows into
the forward pass, row 0 holding the anchor (the previous step's bonus token)
and rows 1..k_i-1 the drafted tokens.  Logits row j is the model's prediction
for the token after row j, so row j judges the token fed at row j+1, and row
k_i-1 supplies the bonus token when every draft is kept.

Greedy (temperature -> 0 of the rule above): p is a point mass on the row's
arg-max, so a draft is kept iff it equals the arg-max and the bonus token is the
arg-max of the first row whose draft was not kept.  Ties go to the lowest index.

Sampling: accept iff u < min(1, p(d)/q(d)), evaluated without the division as
u*q(d) < p(d); residual = normalised max(0, p - q), drawn by inverse CDF in
ascending token order with a supplied uniform (first index whose inclusive
cumulative sum exceeds u' * total).  The uniforms are inputs, so the result is
a deterministic function of the arguments.

Pins (tests/test_oracle_acceptance.py): brute-force loops on tiny vocabularies,
by-construction accepted lengths, planted ties, the exact lossless identity
(emitted-token distribution equals p) recovered by bisection on the uniforms,
p == q accepts everything, q one-hot on a token with p = 0 is always rejected,
temperature equivalence, and the small-temperature limit meeting greedy.
"""
from __future__ import annotations

import numpy as np

from .attention import to_f64


def row_argmax(row: np.ndarray) -> int:
    """Smallest index attaining the row maximum (values compared exactly)."""
    mx = row.max()
    return int(np.flatnonzero(row == mx)[0])


def accept_greedy(target_logits, row_indptr, input_tokens):
    """target_logits [Rv, V] (uint16 = bf16 bits, else float); row_indptr [B+1]
    over verify rows; input_tokens [Rv] = token fed at each verify row.

    Returns (accept_len [B], bonus [B], row_argmax [Rv]) as int64 arrays.
    accept_len counts kept drafts r_i in [0, k_i-1]; a sequence with no rows
    gets accept_len 0 and bonus -1.
    """
    x = to_f64(target_logits)
    Rv = x.shape[0]
    amax = np.array([row_argmax(x[j]) for j in range(Rv)], dtype=np.int64)
    B = len(row_indptr) - 1
    acc = np.zeros(B, dtype=np.int64)
    bonus = np.full(B, -1, dtype=np.int64)
    for i in range(B):
        r0, r1 = int(row_indptr[i]), int(row_indptr[i + 1])
        k = r1 - r0
        if k == 0:
            continue
        r = 0
        while r < k - 1 and amax[r0 + r] == int(input_tokens[r0 + r + 1]):
            r += 1
        acc[i] = r
        bonus[i] = amax[r0 + r]
    return acc, bonus, amax


def softmax64(x: np.ndarray) -> np.ndarray:
    e = np.exp(x - x.max())
    return e / e.sum()


def inverse_cdf(w: np.ndarray, u: float):
    """First index whose inclusive cumulative weight exceeds u * sum(w), plus the
    distance of u*sum(w) to the nearer enclosing CDF edge, relative to sum(w)."""
    W = float(w.sum())
    c = np.cumsum(w)
    thr = u * W
    hits = np.flatnonzero(c > thr)
    # u < 1 and W > 0 guarantee a hit in exact arithmetic; guard the rounding corner
    idx = int(hits[0]) if hits.size else int(np.flatnonzero(w > 0)[-1])
    lo = c[idx] - w[idx]
    margin = min(thr - lo, c[idx] - thr) / W
    return idx, float(margin)


def accept_sample(target_logits, draft_logits, row_indptr, input_tokens,
                  u_accept, u_resample, temperature: float):
    """Speculative-sampling acceptance with supplied uniforms.

    target_logits, draft_logits [Rv, V]; draft row j is the distribution the
    token fed at verify row j+1 was drawn from (each sequence's last draft row
    is unused).  u_accept[j] decides row j's test, u_resample[j] draws the bonus
    token if row j is where the step stops.

    Returns (accept_len [B], bonus [B], info) where info['accept_margin'][j] is
    |u*q(d) - p(d)| / max(p(d), q(d)) for every test that was evaluated (nan
    elsewhere) and info['resample_margin'][i] the inverse-CDF margin of
    sequence i's draw.  A parity test needs the margins to know which decisions
    fp32 arithmetic can be held to.
    """
    if not temperature > 0:
        raise ValueError("temperature must be positive; use accept_greedy for T -> 0")
    xt = to_f64(target_logits) / float(temperature)
    xd = to_f64(draft_logits) / float(temperature)
    ua = np.asarray(u_accept, dtype=np.float64)
    ur = np.asarray(u_resample, dtype=np.float64)
    Rv = xt.shape[0]
    B = len(row_indptr) - 1
    acc = np.zeros(B, dtype=np.int64)
    bonus = np.full(B, -1, dtype=np.int64)
    a_margin = np.full(Rv, np.nan)
    r_margin = np.full(B, np.nan)
    for i in range(B):
        r0, r1 = int(row_indptr[i]), int(row_indptr[i + 1])
        k = r1 - r0
        if k == 0:
            continue
        stop = k - 1                       # row that emits the bonus if all kept
        rejected = False
        for j in range(k - 1):
            p = softmax64(xt[r0 + j]); q = softmax64(xd[r0 + j])
            d = int(input_tokens[r0 + j + 1])
            lhs = ua[r0 + j] * q[d]
            a_margin[r0 + j] = abs(lhs - p[d]) / max(p[d], q[d], np.finfo(float).tiny)
            if not (lhs < p[d]):
                stop = j
                rejected = True
                break
        p = softmax64(xt[r0 + stop])
        if rejected:
            w = np.maximum(0.0, p - softmax64(xd[r0 + stop]))
            if w.sum() == 0.0:             # p == q exactly: residual undefined, fall back to p
                w = p
        else:
            w = p
        idx, mg = inverse_cdf(w, float(ur[r0 + stop]))
        acc[i] = stop
        bonus[i] = idx
        r_margin[i] = mg
    return acc, bonus, {"accept_margin": a_margin, "resample_margin": r_margin}


def draft_select(draft_logits, row_indptr, temperature: float, threshold: float):
    """Draft tokens of a mask block, their confidences, and how many of them are worth verifying
    (Sec. 4.3, selective verification, Eq. 5).

    Row j of a sequence holds the drafter's logits for draft position j+1.  The drafted token is
    the row's arg-max (lowest index on ties), its confidence p_j the softmax probability of that
    token at the given temperature, and the chance that the accepted length reaches position i is
    estimated by the running product p_1 ... p_i.  Positions are kept while that product stays
    at or above `threshold`; the first one below it, and everything after it, is pruned.  Returns
    (tokens [R] int32, confidence [R] float64, keep_len [B] int32, margin [B] float64) where
    margin[i] is the smallest relative distance |product - threshold| / threshold over the
    comparisons that decided keep_len[i] (inf if the threshold is 0: nothing to decide).
    """
    x = to_f64(np.asarray(draft_logits)) / float(temperature)
    R = x.shape[0]
    tokens = np.zeros(R, dtype=np.int32)
    conf = np.zeros(R, dtype=np.float64)
    for j in range(R):
        tokens[j] = row_argmax(x[j])
        conf[j] = softmax64(x[j])[tokens[j]]
    B = len(row_indptr) - 1
    keep = np.zeros(B, dtype=np.int32)
    margin = np.full(B, np.inf)
    for i in range(B):
        prod = 1.0
        for j in range(int(row_indptr[i]), int(row_indptr[i + 1])):
            prod *= conf[j]
            if threshold > 0:
                margin[i] = min(margin[i], abs(prod - threshold) / threshold)
            if prod < threshold:
                break
            keep[i] += 1
    return tokens, conf, keep, margin
