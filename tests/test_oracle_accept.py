"""Pins for the acceptance oracle (verification phase of Sec. II-A2; rule of the speculative
sampling works cited in Sec. I): planted greedy cases, special cases, exact enumeration of the
accept/resample distribution on a tiny vocabulary, expected emitted length."""
import math

import numpy as np
import pytest

from oracle import spin_oracle as orc


def softmax(x):
    e = [math.exp(v - max(x)) for v in x]
    s = sum(e)
    return [v / s for v in e]


def make_rows(rng, draft_len, V, sigma=2.0):
    R = int(np.sum(draft_len)); B = len(draft_len)
    target = rng.normal(0, sigma, (R + B, V)).astype(np.float32)
    draft = rng.normal(0, sigma, (R, V)).astype(np.float32)
    return target, draft


def target_rows_of(draft_len):
    """[(first target row, first draft row)] per request."""
    out, r = [], 0
    for i, g in enumerate(draft_len):
        out.append((r + i, r)); r += int(g)
    return out


# ------------------------------------------------------------------ greedy
@pytest.mark.parametrize("seed", range(3))
def test_greedy_planted_prefix_lengths(seed):
    rng = np.random.default_rng(seed)
    draft_len = np.array([1, 2, 3, 4, 5, 5, 5, 5, 5, 5])
    want_n = np.array([0, 2, 1, 4, 0, 1, 2, 3, 4, 5])
    target, _ = make_rows(rng, draft_len, 50)
    tops = target.argmax(axis=1)
    toks = np.zeros(int(draft_len.sum()), dtype=np.int32)
    for i, (tb, db) in enumerate(target_rows_of(draft_len)):
        for t in range(draft_len[i]):
            good = tops[tb + t]
            toks[db + t] = good if t < want_n[i] else (good + 1) % 50
        # tokens AFTER the first mismatch that happen to match must not count
        if want_n[i] + 1 < draft_len[i]:
            toks[db + want_n[i] + 1] = tops[tb + want_n[i] + 1]
    n, nxt, margin = orc.accept_greedy(draft_len, toks, target)
    np.testing.assert_array_equal(n, want_n)
    for i, (tb, _) in enumerate(target_rows_of(draft_len)):
        assert nxt[i] == tops[tb + want_n[i]]            # correction token, or bonus row when all kept
    assert (margin > 0).all()


def test_greedy_ties_take_lowest_id():
    target = np.zeros((2, 6), dtype=np.float32)
    target[0, [2, 4]] = 1.0
    target[1, [1, 5]] = 3.0
    n, nxt, margin = orc.accept_greedy(np.array([1]), np.array([2], dtype=np.int32), target)
    assert n[0] == 1 and nxt[0] == 1 and margin[0] == 0.0
    n, nxt, _ = orc.accept_greedy(np.array([1]), np.array([4], dtype=np.int32), target)
    assert n[0] == 0 and nxt[0] == 2


# ------------------------------------------------------------------ rejection: special cases
def test_identical_models_accept_everything():
    rng = np.random.default_rng(0)
    draft_len = np.array([3, 1, 5])
    target, _ = make_rows(rng, draft_len, 40)
    keep = np.ones(len(target), dtype=bool)
    keep[[3, 5, 11]] = False                                   # bonus rows
    draft = target[keep].copy()
    toks = rng.integers(0, 40, size=9).astype(np.int32)
    u = rng.random(9); us = rng.random(3)
    n, nxt, _ = orc.accept_rejection(draft_len, toks, target, draft, u, us)
    np.testing.assert_array_equal(n, draft_len)                # u*q < p  <=>  u < 1
    for i, (tb, _) in enumerate(target_rows_of(draft_len)):    # next token = inverse CDF of the bonus row
        p = softmax(target[tb + draft_len[i]].astype(np.float64).tolist())
        acc, k = 0.0, None
        for x, px in enumerate(p):
            acc += px
            if acc > us[i]:
                k = x; break
        assert nxt[i] == k


def test_zero_uniform_accepts_wherever_target_has_mass():
    rng = np.random.default_rng(1)
    draft_len = np.array([4, 2])
    target, draft = make_rows(rng, draft_len, 30)
    toks = rng.integers(0, 30, size=6).astype(np.int32)
    n, _, _ = orc.accept_rejection(draft_len, toks, target, draft, np.zeros(6), rng.random(2))
    np.testing.assert_array_equal(n, draft_len)


def test_draft_mass_on_token_the_target_excludes():
    # q is (numerically) one-hot on token 3, p gives token 3 no mass: reject at row 0 and the
    # residual max(0, p-q) equals p, so the next token follows p.
    V = 8
    target = np.zeros((3, V), dtype=np.float32); target[:, 3] = -1e4
    draft = np.full((2, V), -1e4, dtype=np.float32); draft[:, 3] = 0.0
    p = softmax(target[0].astype(np.float64).tolist())
    for us in (0.0, 0.2, 0.5, 0.99):
        n, nxt, _ = orc.accept_rejection(np.array([2]), np.array([3, 3], dtype=np.int32), target, draft,
                                         np.array([0.5, 0.5]), np.array([us]))
        acc, k = 0.0, None
        for x, px in enumerate(p):
            acc += px
            if acc > us:
                k = x; break
        assert n[0] == 0 and nxt[0] == k and k != 3


def test_strict_inequality_at_equality():
    # p(d) = 1/4 and q(d) = 1/2 exactly (logits 0 and -inf make both softmaxes exact):
    # u = 1/2 is the boundary u*q == p -> rejected; just below -> kept
    ninf = np.float32(-np.inf)
    target = np.zeros((2, 4), dtype=np.float32)
    draft = np.array([[0, 0, ninf, ninf]], dtype=np.float32)          # q = (1/2, 1/2, 0, 0)
    args = (np.array([1]), np.array([0], dtype=np.int32), target, draft)
    n, nxt, margin = orc.accept_rejection(*args, np.array([0.5]), np.array([0.0]))
    assert n[0] == 0 and margin[0] == 0.0
    assert nxt[0] == 2                                            # residual is (0, 0, 1/4, 1/4)
    n, nxt, _ = orc.accept_rejection(*args, np.array([0.5]), np.array([0.5]))
    assert n[0] == 0 and nxt[0] == 3                              # CDF step at exactly u'Z: strict '>'
    n, _, _ = orc.accept_rejection(*args, np.array([0.4999]), np.array([0.0]))
    assert n[0] == 1


def test_later_rows_ignored_after_first_reject():
    rng = np.random.default_rng(2)
    draft_len = np.array([4])
    target, draft = make_rows(rng, draft_len, 20)
    toks = rng.integers(0, 20, size=4).astype(np.int32)
    p1 = np.array(softmax(target[1].astype(np.float64).tolist()))
    q1 = np.array(softmax(draft[1].astype(np.float64).tolist()))
    toks[1] = int(np.argmax(q1 / p1))                  # the token the draft over-weights most
    u = np.array([0.0, 0.999999, 0.0, 0.0])            # rows 2 and 3 would be kept if reached
    assert not (u[1] * q1[toks[1]] < p1[toks[1]])
    n, nxt, _ = orc.accept_rejection(draft_len, toks, target, draft, u, np.array([0.3]))
    assert n[0] == 1
    assert p1[nxt[0]] > q1[nxt[0]]                     # resampled where the residual has mass


# ------------------------------------------------------------------ rejection: distribution identity
@pytest.mark.parametrize("seed", range(4))
def test_emitted_token_distribution_equals_target(seed):
    """One draft row over a tiny vocabulary.  Enumerate every draft token x (weight q(x)) and fine
    regular grids of the two uniforms; the frequency of each emitted first token must be p.

    emitted first token = x if kept, else the resampled token.  Grid midpoints make each frequency
    exact up to one grid cell per decision boundary.
    """
    rng = np.random.default_rng(seed)
    V = int(rng.integers(3, 9))
    target = rng.normal(0, 1.5, (2, V)).astype(np.float32)
    draft = rng.normal(0, 1.5, (1, V)).astype(np.float32)
    p = np.array(softmax(target[0].astype(np.float64).tolist()))
    q = np.array(softmax(draft[0].astype(np.float64).tolist()))
    N = 400
    grid = (np.arange(N) + 0.5) / N
    emitted = np.zeros(V)
    for x in range(V):
        keep = 0
        for u in grid:
            n, _, _ = orc.accept_rejection(np.array([1]), np.array([x], dtype=np.int32), target, draft,
                                           np.array([u]), np.array([0.5]))
            keep += int(n[0])
        emitted[x] += q[x] * keep / N
        # kept fraction is min(1, p/q) to within one grid cell
        assert abs(keep / N - min(1.0, p[x] / q[x])) <= 1.0 / N + 1e-12
        if keep < N:
            # resampled token over the u' grid, at a u that rejects
            cnt = np.zeros(V)
            for us in grid:
                n, nxt, _ = orc.accept_rejection(np.array([1]), np.array([x], dtype=np.int32), target, draft,
                                                 np.array([grid[-1]]), np.array([us]))
                assert n[0] == 0
                cnt[nxt[0]] += 1
            emitted += q[x] * (1 - keep / N) * cnt / N
    assert np.abs(emitted - p).max() < 3.0 * V / N
    # and the closed form the rule is built on:  q*min(1,p/q) + (1 - sum min(p,q)) * r/Z = p
    r = np.maximum(p - q, 0)
    closed = np.minimum(p, q) + (1 - np.minimum(p, q).sum()) * r / r.sum()
    np.testing.assert_allclose(closed, p, rtol=1e-12)


def test_expected_emitted_length_iid_rows():
    """All rows share p and q: with alpha = sum_x min(p,q), E[#emitted] = (1-alpha^(g+1))/(1-alpha)."""
    rng = np.random.default_rng(5)
    V, g, B = 6, 3, 4000
    tl = rng.normal(0, 1.0, V).astype(np.float32); dl = rng.normal(0, 1.0, V).astype(np.float32)
    p = np.array(softmax(tl.astype(np.float64).tolist())); q = np.array(softmax(dl.astype(np.float64).tolist()))
    alpha = np.minimum(p, q).sum()
    draft_len = np.full(B, g)
    target = np.tile(tl, (B * (g + 1), 1)); draft = np.tile(dl, (B * g, 1))
    toks = rng.choice(V, size=B * g, p=q).astype(np.int32)
    n, nxt, _ = orc.accept_rejection(draft_len, toks, target, draft, rng.random(B * g), rng.random(B))
    want = (1 - alpha ** (g + 1)) / (1 - alpha)
    got = (n + 1).mean()
    se = (n + 1).std() / math.sqrt(B)
    assert abs(got - want) < 4 * se
    # every emitted sequence's first token follows p: chi-square over the B first tokens
    first = np.where(n > 0, toks[::g], nxt)
    obs = np.bincount(first, minlength=V)
    chi2 = ((obs - B * p) ** 2 / (B * p)).sum()
    assert chi2 < 25.0                                   # 5 dof, p ~ 1e-4


def test_margins_report_close_calls():
    target = np.zeros((2, 4), dtype=np.float32)
    draft = np.array([[0, 0, -np.inf, -np.inf]], dtype=np.float32)
    _, _, far = orc.accept_rejection(np.array([1]), np.array([0], dtype=np.int32), target, draft,
                                     np.array([0.1]), np.array([0.1]))
    assert far[0] > 0.05
