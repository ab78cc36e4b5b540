"""Pins of the oracle's tree-shaped draft mask (token trees, the related work the paper names beside
speculative decoding).  The defining property of tree attention -- every node's output equals what a
linear draft holding just its root-to-node path would give -- is checked against the dense brute force
of test_oracle_attention, which knows nothing about masks, pages or trees.
"""
import math

import numpy as np
import pytest

import spin_inputs as si
from oracle import spin_oracle as orc
from test_oracle_attention import tiny_problem, bits_to_float, run_oracle, random_rectangles


def tree_oracle(table, q, kp, vp, hq, hkv, scale, masks):
    return orc.verify_attention(table.prefix_len, table.draft_len, table.q_offset, table.pt_offset, table.page_table,
                                table.page_size, q, kp, vp, hq, hkv, scale, tree_mask=masks)


def path_to(parents, t):
    """Draft indices from the tree's first level down to t, by walking the parent pointers."""
    path = []
    while t >= 0:
        path.append(t)
        t = int(parents[t])
    return path[::-1]


def path_attention(q_row, Kp, Vp, Kd, Vd, path, scale):
    """Attention of one query over the prefix followed by the draft tokens on `path`: python loops, math.exp."""
    keys = [Kp[j] for j in range(len(Kp))] + [Kd[u] for u in path]
    vals = [Vp[j] for j in range(len(Vp))] + [Vd[u] for u in path]
    s = [scale * sum(float(a) * float(b) for a, b in zip(q_row, k)) for k in keys]
    mx = max(s)
    w = [math.exp(x - mx) for x in s]
    tot = sum(w)
    return [sum(w[j] * float(vals[j][c]) for j in range(len(keys))) / tot for c in range(len(q_row))]


@pytest.mark.parametrize("seed,shape", [(0, "random"), (1, "random"), (2, "wide"), (3, "star")])
def test_every_node_equals_linear_attention_over_its_path(seed, shape):
    prefix = np.array([5, 0, 9, 2]); draft = np.array([6, 4, 1, 9])
    table, q, kp, vp, dk, dv = tiny_problem(seed + 30, prefix, draft, n_q_heads=2, n_kv_heads=1)
    parents, masks = si.random_trees(draft, np.random.default_rng(seed), shape)
    got = tree_oracle(table, q, kp, vp, 2, 1, 0.4, masks)
    qf = bits_to_float(q)
    for i in range(len(prefix)):
        p, g, r0 = int(prefix[i]), int(draft[i]), int(table.q_offset[i])
        for t in range(g):
            path = path_to(parents[r0:r0 + g], t)
            for h in range(2):
                want = path_attention(qf[r0 + t, h], dk[i][:p, 0], dv[i][:p, 0], dk[i][p:, 0], dv[i][p:, 0], path, 0.4)
                np.testing.assert_allclose(got[r0 + t, h], want, rtol=1e-11, atol=1e-13)


def test_chain_tree_is_the_linear_draft():
    prefix = np.array([7, 0, 3]); draft = np.array([5, 3, 8])
    table, q, kp, vp, dk, dv = tiny_problem(40, prefix, draft)
    _, masks = si.random_trees(draft, None, "chain")
    np.testing.assert_array_equal(tree_oracle(table, q, kp, vp, 2, 2, 0.3, masks), run_oracle(table, q, kp, vp, 2, 2, 0.3))


def test_star_tree_rows_ignore_their_siblings():
    # all draft tokens are children of the last prefix token: changing token u's K/V moves row u only
    prefix = np.array([6]); draft = np.array([5])
    table, q, kp, vp, dk, dv = tiny_problem(41, prefix, draft)
    _, masks = si.random_trees(draft, None, "star")
    base = tree_oracle(table, q, kp, vp, 2, 2, 0.5, masks)
    pt = table.page_table
    pos = 6 + 2                                     # draft token 2
    kp2, vp2 = kp.copy(), vp.copy()
    kp2[pt[pos // 4], :, pos % 4, :] ^= 0x8000      # flip the sign of its K and V
    vp2[pt[pos // 4], :, pos % 4, :] ^= 0x8000
    moved = tree_oracle(table, q, kp2, vp2, 2, 2, 0.5, masks)
    changed = np.any(moved != base, axis=(1, 2))
    assert changed.tolist() == [False, False, True, False, False]


def test_masks_from_parents_hold_exactly_the_ancestors():
    rng = np.random.default_rng(5)
    draft = np.array([12, 1, 30])
    parents, masks = si.random_trees(draft, rng)
    r0 = 0
    for g in draft:
        for t in range(g):
            want = sum(1 << u for u in path_to(parents[r0:r0 + g], t))
            assert int(masks[r0 + t]) == want
        r0 += g


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_decomposed_tree_attention_matches_whole(seed):
    rng = np.random.default_rng(seed + 50)
    prefix = np.array([9, 0, 17]); draft = np.array([6, 5, 3])
    table, q, kp, vp, dk, dv = tiny_problem(seed + 50, prefix, draft)
    _, masks = si.random_trees(draft, rng)
    whole = tree_oracle(table, q, kp, vp, 2, 2, 0.35, masks)
    subs = np.array([(i,) + r for i in range(3) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))], dtype=np.int32)
    parts = orc.verify_attention_decomposed(table.prefix_len, table.draft_len, table.q_offset, table.pt_offset,
                                            table.page_table, table.page_size, q, kp, vp, 2, 2, 0.35, subs, tree_mask=masks)
    np.testing.assert_allclose(parts, whole, rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------------------------ greedy tree acceptance
def greedy_paths_brute_force(g, parents, tokens, rows):
    """All root-to-node paths along which every token equals the arg-max of its parent's row; the
    accepted one is maximal and, among those, the first in child order at every fork."""
    tops = [int(np.flatnonzero(r == r.max())[0]) for r in rows]           # rows[0]: root, rows[1+t]: node t
    matched = [t for t in range(g) if int(tokens[t]) == tops[int(parents[t]) + 1]]
    paths = [[]]
    for t in matched:                                                     # parents come first, so one sweep builds all
        for p in list(paths):
            if (p[-1] if p else -1) == int(parents[t]):
                paths.append(p + [t])
    maximal = [p for p in paths if not any(q[:len(p)] == p and len(q) > len(p) for q in paths)]
    best = min(maximal, key=lambda p: p)      # lists compare element by element: lowest child first, then onwards
    return best, tops[(best[-1] if best else -1) + 1]


@pytest.mark.parametrize("seed", range(6))
def test_tree_greedy_against_path_enumeration(seed):
    rng = np.random.default_rng(seed + 100)
    draft = np.array([7, 1, 12, 5]); vocab = 4                            # tiny vocabulary: many matches, many forks
    parents, _ = si.random_trees(draft, rng, "random" if seed % 2 else "wide")
    R, B = int(draft.sum()), len(draft)
    tokens = rng.integers(0, vocab, R)
    logits = rng.normal(0, 1, (R + B, vocab)).astype(np.float32)
    n_acc, path, nxt, margin = orc.accept_tree_greedy(draft, parents, tokens, logits)
    r = 0
    for i, g in enumerate(draft):
        want_path, want_next = greedy_paths_brute_force(int(g), parents[r:r + g], tokens[r:r + g], logits[r + i:r + i + g + 1])
        assert n_acc[i] == len(want_path)
        assert path[r:r + n_acc[i]].tolist() == want_path and (path[r + n_acc[i]:r + g] == -1).all()
        assert nxt[i] == want_next
        r += g
    assert n_acc.max() >= 1


def test_tree_greedy_on_a_chain_is_linear_greedy():
    rng = np.random.default_rng(7)
    draft = np.array([4, 9, 1, 6]); vocab = 50
    parents, _ = si.random_trees(draft, None, "chain")
    R, B = int(draft.sum()), len(draft)
    logits = rng.normal(0, 2, (R + B, vocab)).astype(np.float32)
    # plant accepted prefixes of lengths 2, 9 (all), 0, 3
    tokens = rng.integers(0, vocab, R)
    r = 0
    for i, (g, keep) in enumerate(zip(draft, [2, 9, 0, 3])):
        for t in range(g):
            top = int(np.argmax(logits[r + i + t]))
            tokens[r + t] = top if t < keep else (top + 1) % vocab
        r += g
    n_t, path, nxt_t, _ = orc.accept_tree_greedy(draft, parents, tokens, logits)
    n_l, nxt_l, _ = orc.accept_greedy(draft, tokens, logits)
    assert n_t.tolist() == n_l.tolist() == [2, 9, 0, 3] and nxt_t.tolist() == nxt_l.tolist()
    r = 0
    for g, n in zip(draft, n_t):
        assert path[r:r + n].tolist() == list(range(n))
        r += g


def test_tree_greedy_takes_the_lowest_numbered_of_equal_children():
    # two children of the root carry the arg-max token; only the first one's subtree may be walked
    draft = np.array([5]); parents = np.array([-1, -1, 0, 1, 1])
    logits = np.zeros((6, 3), dtype=np.float32)
    logits[0, 2] = 1.0          # root -> token 2
    logits[1, 0] = 1.0          # after node 0 -> token 0
    logits[2, 1] = 1.0          # after node 1 -> token 1 (never consulted)
    logits[3, 1] = 1.0          # after node 2 -> token 1
    tokens = np.array([2, 2, 0, 1, 1])
    n_acc, path, nxt, _ = orc.accept_tree_greedy(draft, parents, tokens, logits)
    assert n_acc[0] == 2 and path.tolist() == [0, 2, -1, -1, -1] and nxt[0] == 1


# ------------------------------------------------------------------------------ rejection sampling over trees
@pytest.mark.parametrize("seed", range(8))
def test_tree_rejection_on_a_chain_is_linear_rejection(seed):
    rng = np.random.default_rng(seed + 200)
    draft = np.array([4, 7, 1, 5]); V = int(rng.choice([3, 30, 500]))
    parents, _ = si.random_trees(draft, None, "chain")
    R, B = int(draft.sum()), len(draft)
    tl = rng.normal(0, 2, (R + B, V)).astype(np.float32)
    own = np.delete(tl, np.cumsum(draft) + np.arange(B), axis=0)          # the target row each draft token is checked against
    dl = (0.9 * own + 0.44 * rng.normal(0, 2, (R, V))).astype(np.float32)
    tok = np.array([rng.choice(V, p=orc._softmax64(dl[k])) for k in range(R)])
    ua, us = rng.random(R), rng.random(B)
    n_t, path, nxt_t, m_t = orc.accept_tree_rejection(draft, parents, tok, tl, dl, ua, us)
    n_l, nxt_l, m_l = orc.accept_rejection(draft, tok, tl, dl, ua, us)
    assert n_t.tolist() == n_l.tolist() and nxt_t.tolist() == nxt_l.tolist()
    np.testing.assert_allclose(m_t, m_l, rtol=1e-12)
    r = 0
    for g, n in zip(draft, n_t):
        assert path[r:r + n].tolist() == list(range(n)) and (path[r + n:r + g] == -1).all()
        r += g


def first_emitted_distribution(p_logits, q_logits, k):
    """Distribution of the first emitted token when the root has k children drawn i.i.d. from q, by
    treating the oracle as a black box: acceptance thresholds by bisection on each child's uniform,
    the final draw by a fine grid of u'."""
    V = len(p_logits)
    q = orc._softmax64(q_logits)
    draft = np.array([k]); parents = np.full(k, -1)
    tl = np.stack([p_logits] + [p_logits] * k).astype(np.float32)         # rows after the children are never emitted first
    dl = np.stack([q_logits] * k).astype(np.float32)
    out = np.zeros(V)
    grid = (np.arange(4000) + 0.5) / 4000
    for combo in np.ndindex(*([V] * k)):
        w = float(np.prod([q[x] for x in combo]))
        tok = np.array(combo)
        reach = 1.0                                                        # probability that children 0..c-1 were all rejected
        for c in range(k):
            ua = np.full(k, 0.999999)                                      # earlier children: rejected (p/q < 1 is needed, else unreachable)
            lo, hi = 0.0, 1.0
            for _ in range(40):                                            # largest u_c that still accepts child c
                mid = 0.5 * (lo + hi)
                ua[c] = mid
                n, path, _, _ = orc.accept_tree_rejection(draft, parents, tok, tl, dl, ua, np.array([0.5]))
                if n[0] >= 1 and path[0] == c:
                    lo = mid
                else:
                    hi = mid
            # (if an earlier child is accepted even at u = 0.999999 the later ones are unreachable: reach is then ~0)
            ua_prev = np.full(k, 0.999999)
            n, path, _, _ = orc.accept_tree_rejection(draft, parents, tok, tl, dl, ua_prev, np.array([0.5]))
            first_acc = path[0] if n[0] >= 1 else k
            if first_acc < c:
                reach = 0.0
            out[tok[c]] += w * reach * lo
            reach *= 1.0 - lo
        if reach > 0:
            ua = np.full(k, 0.999999)
            counts = np.zeros(V)
            for u in grid:
                _, _, nx, _ = orc.accept_tree_rejection(draft, parents, tok, tl, dl, ua, np.array([u]))
                counts[nx[0]] += 1
            out += w * reach * counts / len(grid)
    return out


@pytest.mark.parametrize("k", [1, 2])
def test_tree_rejection_emits_the_target_distribution(k):
    # the point of the rule: whatever the draft distribution and however many children are tried,
    # the first emitted token is distributed exactly as the target says
    rng = np.random.default_rng(300 + k)
    V = 3
    p_logits = rng.normal(0, 1.5, V)
    q_logits = rng.normal(0, 1.5, V)
    got = first_emitted_distribution(p_logits, q_logits, k)
    np.testing.assert_allclose(got, orc._softmax64(p_logits.astype(np.float32)), atol=2e-3)
    assert abs(got.sum() - 1.0) < 1e-3


def test_tree_rejection_child_outside_vocabulary_and_vanishing_residual():
    # target == draft: a child whose token id is invalid is rejected, the residual max(0, p - q) vanishes,
    # the child is ignored and the next token comes from p itself; a valid sibling after it is then accepted
    V = 6
    rng = np.random.default_rng(9)
    row = rng.normal(0, 1, V).astype(np.float32)
    draft = np.array([2]); parents = np.array([-1, -1])
    tl = np.stack([row, row, row]); dl = np.stack([row, row])
    tok = np.array([V + 3, 4])
    n, path, nxt, _ = orc.accept_tree_rejection(draft, parents, tok, tl, dl, np.array([0.0, 0.5]), np.array([0.3]))
    assert n[0] == 1 and path.tolist() == [1, -1]
    tok = np.array([V + 3, -1])
    n, path, nxt, _ = orc.accept_tree_rejection(draft, parents, tok, tl, dl, np.array([0.0, 0.5]), np.array([0.3]))
    p = orc._softmax64(row)
    assert n[0] == 0 and nxt[0] == int(np.searchsorted(np.cumsum(p), 0.3 * p.sum(), side="right"))


def test_tree_rejection_walks_into_the_accepted_subtree_only():
    # root children 0 and 1; 0 is rejected (u = 1 - eps against p/q < 1), 1 accepted (u = 0); 1's child 3 accepted, 0's child 2 never looked at
    V = 5
    rng = np.random.default_rng(10)
    draft = np.array([4]); parents = np.array([-1, -1, 0, 1])
    tl = rng.normal(0, 1, (5, V)).astype(np.float32)
    dl = rng.normal(0, 1, (4, V)).astype(np.float32)
    p0, q0 = orc._softmax64(tl[0]), orc._softmax64(dl[0])
    tok = np.array([int(np.argmin(p0 / q0)), 0, 1, 2])
    assert p0[tok[0]] / q0[tok[0]] < 1
    res = np.maximum(p0 - q0, 0)
    tok[1] = int(np.argmax(res))                                           # has residual mass, so u = 0 accepts it
    ua = np.array([1 - 1e-12, 0.0, 0.0, 0.0])
    n, path, nxt, _ = orc.accept_tree_rejection(draft, parents, tok, tl, dl, ua, np.array([0.5]))
    assert n[0] == 2 and path.tolist() == [1, 3, -1, -1]
    # the bonus draw comes from node 3's row
    p_last = orc._softmax64(tl[4])
    assert nxt[0] == int(np.searchsorted(np.cumsum(p_last), 0.5 * np.cumsum(p_last)[-1], side="right"))
