"""Pins for the decomposition oracle (Sec. V-A): exact tiling, counts, L search vs. exhaustion."""
import numpy as np
import pytest

from oracle import spin_oracle as orc


def coverage(prefix, draft, subs):
    """Per parent, a (g x p+g) count matrix of how often each visible cell is covered, and the
    number of cells covered that are NOT visible (must stay 0 only where pieces are clipped:
    a rectangle may stick out past the causal edge, that part simply holds nothing)."""
    mats = [np.zeros((int(g), int(p + g)), dtype=np.int64) for p, g in zip(prefix, draft)]
    for parent, qb, ql, kb, kl in subs:
        p = int(prefix[parent])
        assert 0 <= qb and ql >= 1 and qb + ql <= draft[parent]
        assert 0 <= kb and kl >= 1 and kb + kl <= p + draft[parent]
        for t in range(qb, qb + ql):
            hi = min(kb + kl, p + t + 1)
            if hi > kb:
                mats[parent][t, kb:hi] += 1
    return mats


def assert_exact_tiling(prefix, draft, subs):
    for i, m in enumerate(coverage(prefix, draft, subs)):
        p, g = int(prefix[i]), int(draft[i])
        for t in range(g):
            assert (m[t, : p + t + 1] == 1).all(), (i, t)
            assert (m[t, p + t + 1:] == 0).all(), (i, t)


@pytest.mark.parametrize("width", [1, 2, 4, 5, 16])
def test_q_split_tiles_exactly(width):
    rng = np.random.default_rng(width)
    prefix = rng.integers(0, 40, size=9); draft = rng.integers(1, 17, size=9)
    subs = orc.decompose_q_split(prefix, draft, width)
    assert_exact_tiling(prefix, draft, subs)
    assert len(subs) == int(np.sum(-(-draft // width)))
    # each row's keys all sit in one piece: kv_begin is 0 and the piece ends at its last row's edge
    for parent, qb, ql, kb, kl in subs:
        assert kb == 0 and kl == prefix[parent] + qb + ql
    # deterministic order
    key = [(s[0], s[1], s[3]) for s in subs.tolist()]
    assert key == sorted(key)


@pytest.mark.parametrize("length", [1, 3, 16, 32, 1000])
def test_kv_split_tiles_exactly(length):
    rng = np.random.default_rng(length)
    prefix = rng.integers(0, 70, size=8); draft = rng.integers(1, 9, size=8)
    subs = orc.decompose_kv_split(prefix, draft, length)
    assert_exact_tiling(prefix, draft, subs)
    n = prefix + draft
    assert len(subs) == int(np.sum(-(-n // length)))
    for parent, qb, ql, kb, kl in subs:
        assert qb == 0 and ql == draft[parent]          # the whole draft block rides along
        assert kb % length == 0 and kl <= length
    rows, pad = orc.kv_padding(prefix, draft, length)
    assert rows == len(subs)
    assert pad == rows * length - int(n.sum())


def test_figure_scenario_needs_fewer_pads():
    # The illustration of Sec. V-A: request A has 4 prompt + 3 candidate tokens, B and C are
    # shorter.  Their lengths are not recoverable from the text, so this is a smoke scenario:
    # with B and C of 3 prompt + 1 candidate tokens, padding to A's length costs 6 slots while
    # rows of length 4 cost 1.
    prefix = np.array([4, 3, 3]); draft = np.array([3, 1, 1])
    assert orc.kv_padding(prefix, draft, 7) == (3, 6)
    assert orc.kv_padding(prefix, draft, 4) == (4, 1)
    subs = orc.decompose_kv_split(prefix, draft, 4)
    assert subs.tolist() == [[0, 0, 3, 0, 4], [0, 0, 3, 4, 3], [1, 0, 1, 0, 4], [2, 0, 1, 0, 4]]


def exhaustive_best_length(prefix, draft, max_rows, l_min, l_max, step):
    n = [int(a + b) for a, b in zip(prefix, draft)]
    cands = []
    for L in range(l_min, l_max + 1):
        if L % step:
            continue
        rows = sum(-(-x // L) for x in n)
        pad = sum(-(-x // L) * L - x for x in n)
        if rows <= max_rows:
            cands.append((pad, -L))
    if not cands:
        return None
    return -min(cands)[1]


@pytest.mark.parametrize("seed", range(8))
def test_length_search_matches_exhaustion(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 12))
    prefix = rng.integers(0, 300, size=B); draft = rng.integers(1, 9, size=B)
    step = int(rng.choice([1, 4, 16]))
    l_min = int(rng.integers(1, 40)); l_max = int((prefix + draft).max())
    for max_rows in (B, B + 3, 3 * B):
        got = orc.search_kv_length(prefix, draft, max_rows, l_min, l_max, step)
        want = exhaustive_best_length(prefix, draft, max_rows, l_min, l_max, step)
        assert got == want


def test_length_search_not_monotone():
    # Sec. V-A notes that padding is not linear in L: a known non-monotone instance
    prefix = np.array([9, 19, 29]); draft = np.array([1, 1, 1])        # n = 10, 20, 30
    pads = [orc.kv_padding(prefix, draft, L)[1] for L in (10, 11, 15, 20, 30)]
    assert pads == [0, 6, 15, 20, 30]
    assert orc.search_kv_length(prefix, draft, 6, 1, 30, 1) == 10
    assert orc.search_kv_length(prefix, draft, 5, 1, 30, 1) == 15      # 6 rows at L=10 no longer fit
    assert orc.search_kv_length(prefix, draft, 2, 1, 30, 1) is None
