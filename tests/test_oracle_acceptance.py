"""Pins for oracle/acceptance.py against things other than itself (CPU only).

Greedy: brute-force Python loops on tiny vocabularies, accepted lengths fixed by
construction, planted ties.  Sampling: the lossless identity of speculative
sampling (Sec. 3: the committed token is distributed exactly as the target
distribution p) recovered from the oracle's decisions by bisection on the
supplied uniforms, plus degenerate cases with known answers.
"""

import numpy as np
import pytest

from oracle import acceptance as oc


def _brute_greedy(logits, indptr, toks):
    """Plain loops, written separately from the oracle."""
    B = len(indptr) - 1
    acc, bonus = [], []
    for i in range(B):
        r0, r1 = indptr[i], indptr[i + 1]
        if r1 == r0:
            acc.append(0); bonus.append(-1); continue
        best = []
        for j in range(r0, r1):
            bi = 0
            for v in range(1, logits.shape[1]):
                if logits[j, v] > logits[j, bi]:
                    bi = v
            best.append(bi)
        r = 0
        for j in range(r1 - r0 - 1):
            if best[j] == toks[r0 + j + 1]:
                r += 1
            else:
                break
        acc.append(r); bonus.append(best[r])
    return np.array(acc), np.array(bonus)


def test_greedy_matches_brute_force_on_tiny_vocabularies():
    rng = np.random.default_rng(0)
    for trial in range(200):
        V = int(rng.integers(2, 7)); B = int(rng.integers(1, 4))
        ks = rng.integers(0, 5, size=B)
        indptr = np.concatenate([[0], np.cumsum(ks)])
        Rv = int(indptr[-1])
        # few distinct values => many ties
        logits = rng.integers(-2, 3, size=(Rv, V)).astype(np.float64)
        toks = rng.integers(0, V, size=Rv)
        a, b, _ = oc.accept_greedy(logits, indptr, toks)
        ea, eb = _brute_greedy(logits, indptr, toks)
        assert np.array_equal(a, ea) and np.array_equal(b, eb)


@pytest.mark.parametrize("r_expect", [0, 1, 2, 3, 4])
def test_greedy_accepted_length_by_construction(r_expect):
    """k = 5 verify rows: plant the arg-max of rows 0..r-1 as the next fed token, break row r."""
    rng = np.random.default_rng(r_expect)
    V, k = 50, 5
    logits = rng.standard_normal((k, V))
    winners = rng.integers(0, V, size=k)
    for j in range(k):
        logits[j, winners[j]] = 10.0 + j
    toks = np.zeros(k, dtype=np.int64); toks[0] = 7
    for j in range(k - 1):
        toks[j + 1] = winners[j] if j < r_expect else (winners[j] + 1) % V
    a, b, am = oc.accept_greedy(logits, [0, k], toks)
    assert a[0] == r_expect and b[0] == winners[r_expect]
    assert np.array_equal(am, winners)
    # committed length L_acc = r_acc + 1 (Sec. 3)
    assert a[0] + 1 == r_expect + 1


def test_greedy_ties_break_to_lowest_index_and_bf16_bits():
    logits = np.array([[0.5, 2.0, 2.0, -1.0], [3.0, 3.0, 3.0, 3.0]])
    a, b, am = oc.accept_greedy(logits, [0, 2], [0, 1])
    assert list(am) == [1, 0] and a[0] == 1 and b[0] == 0
    a, b, _ = oc.accept_greedy(logits, [0, 2], [0, 2])      # token 2 ties but is not the lowest index
    assert a[0] == 0 and b[0] == 1
    # bf16 bit patterns: 0x4000 = 2.0, 0x3F80 = 1.0, 0xC000 = -2.0, 0xFF80 = -inf
    bits = np.array([[0x3F80, 0x4000, 0xC000, 0x4000], [0xFF80, 0xC000, 0xFF80, 0xC000]], dtype=np.uint16)
    a, b, am = oc.accept_greedy(bits, [0, 2], [3, 1])
    assert list(am) == [1, 1] and a[0] == 1 and b[0] == 1
    # a single verify row is plain decoding: nothing to accept, bonus = arg-max
    a, b, _ = oc.accept_greedy(logits[:1], [0, 1], [0])
    assert a[0] == 0 and b[0] == 1


def _bisect_threshold(f, lo=0.0, hi=1.0, iters=60):
    """Largest u in [lo, hi) with f(u) True, assuming f is True then False."""
    if not f(lo):
        return lo
    if f(np.nextafter(hi, 0)):
        return hi
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        if f(mid):
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def _emitted_distribution(xt, xd, T):
    """Distribution of the first committed token for k = 2 verify rows (one draft),
    measured from the oracle's decisions only: integrate over the draft token d ~ q
    and the two uniforms by locating the decision boundaries with bisection."""
    V = xt.shape[1]
    q = np.exp(xd[0] / T - np.max(xd[0] / T)); q /= q.sum()
    indptr = [0, 2]
    emitted = np.zeros(V)
    for d in range(V):
        if q[d] == 0:
            continue
        toks = [0, d]

        def accepted(u):
            a, _, _ = oc.accept_sample(xt, xd, indptr, toks, [u, 0.0], [0.5, 0.5], T)
            return a[0] == 1
        a_prob = _bisect_threshold(accepted)
        emitted[d] += q[d] * a_prob
        if a_prob < 1.0:
            # residual draw at row 0: find the CDF breakpoints of u_resample
            u_rej = 0.5 * (a_prob + 1.0)
            cur = 0.0
            while cur < 1.0:
                _, b0, _ = oc.accept_sample(xt, xd, indptr, toks, [u_rej, 0.0], [cur, 0.5], T)
                tok = int(b0[0])

                def same(u, tok=tok):
                    _, bb, _ = oc.accept_sample(xt, xd, indptr, toks, [u_rej, 0.0], [u, 0.5], T)
                    return int(bb[0]) == tok
                nxt = _bisect_threshold(same, lo=cur, hi=1.0)
                emitted[tok] += q[d] * (1.0 - a_prob) * (nxt - cur)
                if nxt >= 1.0:
                    break
                cur = np.nextafter(nxt, 2.0) + 1e-15
    return emitted


@pytest.mark.parametrize("seed,V,T", [(0, 3, 1.0), (1, 4, 1.0), (2, 5, 0.7), (3, 4, 2.0)])
def test_sampling_is_lossless_exact_enumeration(seed, V, T):
    """Sum over drafts and uniforms of what the oracle commits equals softmax(target/T)."""
    rng = np.random.default_rng(seed)
    xt = rng.standard_normal((2, V)) * 1.5
    xd = xt + rng.standard_normal((2, V))
    p = np.exp(xt[0] / T - np.max(xt[0] / T)); p /= p.sum()
    emitted = _emitted_distribution(xt, xd, T)
    np.testing.assert_allclose(emitted.sum(), 1.0, atol=1e-9)
    np.testing.assert_allclose(emitted, p, atol=1e-9)


def test_sampling_all_accepted_bonus_comes_from_last_row_target():
    """p == q: every draft is kept whatever u is; the bonus is an inverse-CDF draw from
    the last row's target distribution with known breakpoints."""
    x = np.log(np.array([[0.1, 0.2, 0.3, 0.4], [0.25, 0.25, 0.25, 0.25], [0.4, 0.1, 0.4, 0.1]]))
    for u in (0.0, 0.3, 0.999999):
        a, b, _ = oc.accept_sample(x, x, [0, 3], [0, 3, 1], [u, u, u], [0.0, 0.0, 0.45], 1.0)
        assert a[0] == 2 and b[0] == 1          # cdf of the last row: .4 .5 .9 1.0 ; 0.45 lies in token 1's interval
    # explicit breakpoints of the last row (0.4, 0.5, 0.9, 1.0)
    for u, tok in [(0.0, 0), (0.39, 0), (0.41, 1), (0.49, 1), (0.51, 2), (0.89, 2), (0.91, 3), (0.999, 3)]:
        a, b, _ = oc.accept_sample(x, x, [0, 3], [0, 3, 1], [0.5, 0.5, 0.5], [0.0, 0.0, u], 1.0)
        assert a[0] == 2 and b[0] == tok, (u, tok, b)


def test_sampling_known_ratio_and_residual():
    """p = (.5,.3,.2), q = (.2,.5,.3).  Draft token 1: ratio .6 -> accepted iff u < .6.
    Residual max(0,p-q) = (.3,0,0) -> bonus is token 0 whatever u' is.  Draft token 0:
    ratio 2.5 -> always accepted."""
    xt = np.log(np.array([[0.5, 0.3, 0.2], [0.2, 0.2, 0.6]]))
    xd = np.log(np.array([[0.2, 0.5, 0.3], [1 / 3, 1 / 3, 1 / 3]]))
    for u, kept in [(0.0, True), (0.59, True), (0.61, False), (0.99, False)]:
        a, b, info = oc.accept_sample(xt, xd, [0, 2], [0, 1], [u, 0.0], [0.77, 0.1], 1.0)
        assert (a[0] == 1) == kept
        if not kept:
            assert b[0] == 0
        else:
            assert b[0] == 0            # last row target cdf .2 .4 1.0, u' = 0.1 -> token 0
        np.testing.assert_allclose(info["accept_margin"][0], abs(u * 0.5 - 0.3) / 0.5, atol=1e-12)
    a, _, _ = oc.accept_sample(xt, xd, [0, 2], [0, 0], [0.999999, 0.0], [0.5, 0.5], 1.0)
    assert a[0] == 1
    # residual with two surviving tokens: p = (.5,.3,.2), q = (.1,.1,.8) -> (.4,.2,0)/.6
    xd2 = np.log(np.array([[0.1, 0.1, 0.8], [1 / 3, 1 / 3, 1 / 3]]))
    for u2, tok in [(0.0, 0), (0.66, 0), (0.67, 1), (0.999, 1)]:
        a, b, _ = oc.accept_sample(xt, xd2, [0, 2], [0, 2], [0.9, 0.0], [u2, 0.5], 1.0)
        assert a[0] == 0 and b[0] == tok


def test_sampling_zero_target_probability_is_always_rejected():
    xt = np.array([[0.0, -np.inf, 0.0], [0.0, 0.0, 0.0]])
    xd = np.array([[-np.inf, 0.0, -np.inf], [0.0, 0.0, 0.0]])     # drafter one-hot on a token with p = 0
    for u in (0.0, 0.5):
        a, b, _ = oc.accept_sample(xt, xd, [0, 2], [0, 1], [u, 0.0], [0.6, 0.0], 1.0)
        assert a[0] == 0 and b[0] == 2          # residual = p = (.5, 0, .5); u' = .6 -> token 2


def test_sampling_temperature_divides_both_logit_sets():
    rng = np.random.default_rng(5)
    xt = rng.standard_normal((6, 9)); xd = xt + 0.5 * rng.standard_normal((6, 9))
    toks = rng.integers(0, 9, size=6); ua = rng.random(6); ur = rng.random(6)
    a1, b1, _ = oc.accept_sample(xt, xd, [0, 2, 6], toks, ua, ur, 0.5)
    a2, b2, _ = oc.accept_sample(xt / 0.5, xd / 0.5, [0, 2, 6], toks, ua, ur, 1.0)
    assert np.array_equal(a1, a2) and np.array_equal(b1, b2)


def test_small_temperature_limit_meets_greedy():
    """T -> 0: p collapses onto the arg-max, so sampling acceptance reproduces greedy
    acceptance when the drafter is also sharp (ties excluded)."""
    rng = np.random.default_rng(6)
    for trial in range(50):
        V, k = 12, 5
        xt = rng.permutation(V * k).reshape(k, V).astype(np.float64)     # all distinct per row
        best = xt.argmax(axis=1)
        toks = np.zeros(k, dtype=np.int64)
        xd = np.zeros((k, V))
        for j in range(k - 1):
            toks[j + 1] = best[j] if rng.random() < 0.6 else (best[j] + 1 + rng.integers(0, V - 1)) % V
            xd[j, toks[j + 1]] = 1.0                                     # drafter puts its mass on what it drafted
        ga, gb, _ = oc.accept_greedy(xt, [0, k], toks)
        sa, sb, _ = oc.accept_sample(xt, xd, [0, k], toks, rng.random(k) * 0.999, rng.random(k), 1e-3)
        assert np.array_equal(ga, sa) and np.array_equal(gb, sb)


def test_monte_carlo_first_token_distribution():
    """Draw d ~ q and fresh uniforms many times; the committed first token follows p (chi-square)."""
    rng = np.random.default_rng(7)
    V, n = 6, 20000
    xt = rng.standard_normal((2, V)); xd = xt + rng.standard_normal((2, V))
    p = np.exp(xt[0]); p /= p.sum()
    q = np.exp(xd[0]); q /= q.sum()
    counts = np.zeros(V)
    ds = rng.choice(V, size=n, p=q); ua = rng.random((n, 2)); ur = rng.random((n, 2))
    for t in range(n):
        a, b, _ = oc.accept_sample(xt, xd, [0, 2], [0, ds[t]], ua[t], ur[t], 1.0)
        counts[ds[t] if a[0] == 1 else b[0]] += 1
    chi2 = ((counts - n * p) ** 2 / (n * p)).sum()
    assert chi2 < 25.0          # 5 degrees of freedom: P(chi2 > 25) ~ 1.4e-4


def test_empty_sequences_and_margins():
    xt = np.zeros((1, 4)); xd = np.zeros((1, 4))
    a, b, info = oc.accept_sample(xt, xd, [0, 0, 1], [2], [0.5], [0.30], 1.0)
    assert list(a) == [0, 0] and list(b) == [-1, 1]
    np.testing.assert_allclose(info["resample_margin"][1], 0.05, atol=1e-12)
    a, b, _ = oc.accept_greedy(xt, [0, 0, 1], [2])
    assert list(a) == [0, 0] and list(b) == [-1, 0]


# ---------------------------------------------------------------------------------------
# Selective verification (Sec. 4.3, Eq. 5): confidence products against a threshold
# ---------------------------------------------------------------------------------------
def test_draft_select_closed_form_two_valued_rows():
    """A row that is `a` at one token and 0 elsewhere has p = e^(a/T) / (e^(a/T) + V - 1)."""
    V, T = 50, 0.7
    a = np.array([3.0, 2.0, 4.0, 0.5])
    pos = [7, 0, 49, 3]
    x = np.zeros((4, V))
    for j in range(4):
        x[j, pos[j]] = a[j]
    p = np.exp(a / T) / (np.exp(a / T) + V - 1)
    tok, conf, keep, margin = oc.draft_select(x, [0, 4], T, threshold=p[0] * p[1] * 0.999)
    assert tok.tolist() == pos
    np.testing.assert_allclose(conf, p, rtol=1e-13)
    assert keep.tolist() == [2]                       # p0 p1 >= thr > p0 p1 p2
    np.testing.assert_allclose(margin[0], 0.001 / 0.999, rtol=1e-9)     # the comparison that kept position 2
    assert oc.draft_select(x, [0, 4], T, threshold=0.0)[2].tolist() == [4]      # nothing pruned
    assert oc.draft_select(x, [0, 4], T, threshold=1.1)[2].tolist() == [0]      # everything pruned
    assert p[1] < p[0] * 0.99
    assert oc.draft_select(x, [0, 1, 1, 4], T, threshold=p[0] * 0.99)[2].tolist() == [1, 0, 0]   # ragged, one empty


def test_draft_select_brute_force_and_ties():
    rng = np.random.default_rng(12)
    V = 6
    x = rng.integers(-2, 3, size=(9, V)).astype(np.float64)          # small integers: plenty of ties
    indptr = [0, 3, 3, 7, 9]
    thr = 0.08
    tok, conf, keep, _ = oc.draft_select(x, indptr, 1.0, thr)
    for j in range(9):
        best = max(range(V), key=lambda v: (x[j, v], -v))            # highest value, lowest index
        assert tok[j] == best
        z = sum(np.exp(x[j, v]) for v in range(V))
        assert abs(conf[j] - np.exp(x[j, best]) / z) < 1e-14
    for i in range(4):
        prod, n = 1.0, 0
        for j in range(indptr[i], indptr[i + 1]):
            prod *= conf[j]
            if prod < thr:
                break
            n += 1
        assert keep[i] == n
    uniform = np.zeros((2, 10))
    t2, c2, k2, _ = oc.draft_select(uniform, [0, 2], 1.0, 0.05)
    assert t2.tolist() == [0, 0] and np.allclose(c2, 0.1) and k2.tolist() == [1]     # 0.1 >= 0.05 > 0.01
