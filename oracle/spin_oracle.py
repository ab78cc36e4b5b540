"""CPU oracle for the batched verification step (TEST INFRASTRUCTURE ONLY).

A plain, slow float64 numpy implementation of what the verification step computes.
It shares no code with the HIP library and must never be imported by the product
package: only tests, the smoke check and the benchmark's cpu_baseline leg call it.

What it follows
  * verify_attention         -- the self-attention definition of Sec. II-A1, Eq. (2)
                                 (a_ij = F(Q_i,K_j)/sum_j F(Q_i,K_j), F = exp(Q K^T),
                                 O_i = sum_j a_ij V_j), restricted to the keys a draft row
                                 may see, read through a page table.
  * verify_attention_decomposed -- Sec. V-A, Eq. (13): when a request is cut into
                                 sub-requests, the softmax denominator of a row runs over
                                 all tokens of the ORIGINAL request in the batch.
  * append_kv                -- the KV cache of Sec. II-A1: the candidate tokens' K/V enter the
                                 cache at the positions after the prefix (plain scatter).
  * accept_tree_greedy / accept_tree_rejection -- verification of token trees (related work of Sec. I):
                                 greedy matching, and multi-round rejection sampling over the children.
  * decompose_*              -- Sec. V-A: request decomposition and the choice of the
                                 KV-tensor length L for a fixed width B.
  * accept_greedy / accept_rejection -- the verification phase of Sec. II-A2 (draft tokens that
                                 agree with the LLM's own output are kept); the paper does
                                 not print the rule, so these follow the speculative
                                 sampling rule of the works it cites in Sec. I.

Readings taken where the paper is silent or ambiguous:
  * Eq. (2) has no 1/sqrt(d): `scale` is a parameter (1.0 gives the literal formula).
  * Eq. (2) sums over all n tokens; autoregressive visibility is only in prose.  Here draft row
    t of request i sees keys j <= p_i + t (whole prefix, causal inside the draft block).
  * Eq. (13) redefines only a_ij; the output is read as the sum over every visible token
    of the original request, whichever sub-request holds it.

Pins (tests/test_oracle_*.py): pure-Python brute force on tiny inputs, draft length 1
against a separately written decode attention, closed forms (zero queries, constant
values, one dominant key, empty prefix), invariances (key shift, joint permutation of
prefix pairs, page relocation, NaN in unowned slots, grouped-query = repeated heads),
decomposition invariance under Eq. (13), planted greedy cases, p == q, u == 0, exact
enumeration of the accept/resample distribution on a tiny vocabulary, and the expected
emitted length for i.i.d. rows; the KV append against a cache filled position by position and
against dense brute-force attention; tree masks against plain attention over every node's
root-to-node path; the greedy tree acceptance against an enumeration of all matched paths and
against the linear acceptance on chains.  No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

NEG_INF = -np.inf


# --------------------------------------------------------------------------- helpers
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float64 exactly."""
    b = np.ascontiguousarray(bits).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def _as_f64(a: np.ndarray) -> np.ndarray:
    if a.dtype == np.uint16:
        return bf16_bits_to_f64(a)
    return np.asarray(a, dtype=np.float64)


def gather_request_kv(pool: np.ndarray, page_table: np.ndarray, page_size: int,
                      kv_head: int, lo: int, hi: int) -> np.ndarray:
    """Tokens lo..hi-1 of one request and one KV head, as float64 [hi-lo, d].

    `pool` is indexed [physical page, kv head, slot in page, dim]; token j of the request
    lives in page page_table[j // page_size], slot j % page_size.
    """
    j = np.arange(lo, hi)
    pages = page_table[j // page_size]
    slots = j % page_size
    return _as_f64(pool[pages, kv_head, slots, :])


# --------------------------------------------------------------------------- attention
def _tree_visible(masks, p, k0, k1) -> np.ndarray:
    """[rows, k1-k0] booleans: key j is a prefix key (j < p) or draft key p+u with bit u of the row's mask set."""
    keys = np.arange(k0, k1)
    out = np.ones((len(masks), k1 - k0), dtype=bool)
    for t, m in enumerate(masks):
        m = int(m)
        for c, j in enumerate(keys):
            if j >= p:
                out[t, c] = bool((m >> int(j - p)) & 1)
    return out


def verify_attention(prefix_len, draft_len, q_offset, pt_offset, page_table, page_size,
                     q, k_pool, v_pool, n_q_heads, n_kv_heads, scale,
                     requests=None, heads=None, tree_mask=None) -> np.ndarray:
    """Eq. (2) per request, per query head, per draft row, over the visible keys.

    Returns float64 [R, n_q_heads, d].  `requests` / `heads` restrict the work to a sample
    (other entries stay NaN) so that large batches can be spot-checked.

    tree_mask (uint64 [R], optional): the drafts are token trees (the related work the paper names
    next to speculative decoding); row t then sees the prefix and those draft keys p+u whose bit
    u is set in tree_mask[row] -- its ancestors and itself -- instead of every earlier draft key.
    """
    R = int(q_offset[-1])
    d = q.shape[-1]
    G = n_q_heads // n_kv_heads
    out = np.full((R, n_q_heads, d), np.nan, dtype=np.float64)
    req_iter = range(len(prefix_len)) if requests is None else requests
    head_iter = range(n_q_heads) if heads is None else heads
    for i in req_iter:
        p, g = int(prefix_len[i]), int(draft_len[i])
        n = p + g
        pt = page_table[pt_offset[i]:pt_offset[i + 1]]
        r0 = int(q_offset[i])
        for h in head_iter:
            hk = h // G
            K = gather_request_kv(k_pool, pt, page_size, hk, 0, n)       # [n, d]
            V = gather_request_kv(v_pool, pt, page_size, hk, 0, n)
            Q = _as_f64(q[r0:r0 + g, h, :])                               # [g, d]
            S = scale * (Q @ K.T)                                         # [g, n]
            visible = np.arange(n)[None, :] <= (p + np.arange(g))[:, None]
            if tree_mask is not None:
                visible = visible & _tree_visible(tree_mask[r0:r0 + g], p, 0, n)
            S = np.where(visible, S, NEG_INF)
            m = S.max(axis=1, keepdims=True)
            F = np.where(visible, np.exp(S - m), 0.0)                     # F(Q_i,K_j) up to e^-m
            a = F / F.sum(axis=1, keepdims=True)
            out[r0:r0 + g, h, :] = a @ V
    return out


def verify_attention_decomposed(prefix_len, draft_len, q_offset, pt_offset, page_table, page_size,
                                q, k_pool, v_pool, n_q_heads, n_kv_heads, scale, subs, tree_mask=None) -> np.ndarray:
    """Attention evaluated sub-request by sub-request, then joined as Eq. (13) demands.

    `subs` is an int array [n_sub, 5] of (parent, q_begin, q_len, kv_begin, kv_len): a rectangle
    of the parent's (draft row x key) score matrix.  Every rectangle yields, per row, the
    un-normalised sums  l = sum_j F(Q_i,K_j)  and  N = sum_j F(Q_i,K_j) V_j  over ITS visible
    keys (kept as (m, l e^-m, N e^-m) for range); the row's output is  sum_s N_s / sum_s l_s
    over all rectangles s of the same parent that contain the row.
    """
    R = int(q_offset[-1])
    d = q.shape[-1]
    G = n_q_heads // n_kv_heads
    num = np.zeros((R, n_q_heads, d), dtype=np.float64)
    den = np.zeros((R, n_q_heads), dtype=np.float64)
    mx = np.full((R, n_q_heads), NEG_INF, dtype=np.float64)
    for parent, qb, ql, kb, kl in np.asarray(subs, dtype=np.int64):
        p = int(prefix_len[parent])
        pt = page_table[pt_offset[parent]:pt_offset[parent + 1]]
        r0 = int(q_offset[parent]) + qb
        for h in range(n_q_heads):
            hk = h // G
            K = gather_request_kv(k_pool, pt, page_size, hk, kb, kb + kl)
            V = gather_request_kv(v_pool, pt, page_size, hk, kb, kb + kl)
            Q = _as_f64(q[r0:r0 + ql, h, :])
            S = scale * (Q @ K.T)
            visible = (kb + np.arange(kl))[None, :] <= (p + qb + np.arange(ql))[:, None]
            if tree_mask is not None:
                visible = visible & _tree_visible(tree_mask[r0:r0 + ql], p, kb, kb + kl)
            for t in range(ql):
                vis = visible[t]
                if not vis.any():
                    continue                      # an empty piece adds nothing to either sum
                s = S[t, vis]
                m_s = s.max()
                F = np.exp(s - m_s)
                l_s = F.sum()
                N_s = F @ V[vis]
                r = r0 + t
                M = max(mx[r, h], m_s)
                w_old = np.exp(mx[r, h] - M) if np.isfinite(mx[r, h]) else 0.0
                w_new = np.exp(m_s - M)
                num[r, h] = num[r, h] * w_old + N_s * w_new
                den[r, h] = den[r, h] * w_old + l_s * w_new
                mx[r, h] = M
    return num / den[:, :, None]


def append_kv(prefix_len, draft_len, q_offset, pt_offset, page_table, page_size, k_pool, v_pool, k_new, v_new):
    """The step before the attention: draft token t of request i (packed row q_offset[i]+t of k_new /
    v_new, indexed [row, kv head, dim]) is cached at position p_i + t.  Writes into the pools in place."""
    for i in range(len(prefix_len)):
        pt = page_table[pt_offset[i]:pt_offset[i + 1]]
        for t in range(int(draft_len[i])):
            pos = int(prefix_len[i]) + t
            r = int(q_offset[i]) + t
            k_pool[pt[pos // page_size], :, pos % page_size, :] = k_new[r]
            v_pool[pt[pos // page_size], :, pos % page_size, :] = v_new[r]


# --------------------------------------------------------------------------- decomposition
def decompose_q_split(prefix_len, draft_len, width: int) -> np.ndarray:
    """Cut every request's draft block into pieces of at most `width` rows.

    Piece k of request i: rows [k*width, min((k+1)*width, g_i)), keys [0, p_i + last row + 1).
    Each row's softmax is complete inside one piece.  Order: parent, then q_begin.
    """
    out = []
    for i, (p, g) in enumerate(zip(prefix_len, draft_len)):
        p, g = int(p), int(g)
        k = 0
        while k * width < g:
            qb = k * width
            ql = min(width, g - qb)
            out.append((i, qb, ql, 0, p + qb + ql))
            k += 1
    return np.asarray(out, dtype=np.int32).reshape(-1, 5)


def decompose_kv_split(prefix_len, draft_len, length: int) -> np.ndarray:
    """Sec. V-A: lay every request out in rows of a KV tensor of length L = `length`.

    Request i (n_i = p_i + g_i tokens) becomes ceil(n_i / L) sub-requests; each carries the
    whole draft block as queries (the replicated Q rows of Sec. V-A) and keys
    [k*L, min((k+1)*L, n_i)).  Order: parent, then kv_begin.
    """
    out = []
    for i, (p, g) in enumerate(zip(prefix_len, draft_len)):
        n = int(p) + int(g)
        kb = 0
        while kb < n:
            out.append((i, 0, int(g), kb, min(length, n - kb)))
            kb += length
    return np.asarray(out, dtype=np.int32).reshape(-1, 5)


def kv_padding(prefix_len, draft_len, length: int):
    """(#rows, #padding tokens) of the B x L KV tensor of Sec. V-A for a given L."""
    n = np.asarray(prefix_len, dtype=np.int64) + np.asarray(draft_len, dtype=np.int64)
    rows = (n + length - 1) // length
    return int(rows.sum()), int((rows * length - n).sum())


def search_kv_length(prefix_len, draft_len, max_rows: int, l_min: int, l_max: int, step: int):
    """Sec. V-A: with the tensor width (number of rows) capped at `max_rows`, scan every
    candidate L and keep the one with the fewest padding tokens.

    Candidates: multiples of `step` within [l_min, l_max].  Ties go to the larger L (fewer
    sub-requests, fewer replicated Q rows).  Returns L, or None if no candidate fits.
    """
    best = None
    best_pad = None
    L = ((l_min + step - 1) // step) * step
    while L <= l_max:
        rows, pad = kv_padding(prefix_len, draft_len, L)
        if rows <= max_rows and (best_pad is None or pad <= best_pad):
            best, best_pad = L, pad
        L += step
    return best


# --------------------------------------------------------------------------- acceptance
def _softmax64(row: np.ndarray) -> np.ndarray:
    x = np.asarray(row, dtype=np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def _first_argmax(row: np.ndarray) -> int:
    return int(np.argmax(row))        # numpy returns the lowest index among equal maxima


def accept_greedy(draft_len, draft_tokens, target_logits):
    """Greedy-match verification.

    Request i owns target rows base..base+g_i (base = q_offset[i] + i; the last is the bonus
    row).  n_i = number of leading draft tokens equal to the target's arg-max at their row;
    next_token = arg-max of target row n_i.  Returns (n_accepted[B], next_token[B], margin[B])
    where margin is the smallest top-1/top-2 logit gap over the rows that were consulted.
    """
    B = len(draft_len)
    n_acc = np.zeros(B, dtype=np.int32)
    nxt = np.zeros(B, dtype=np.int32)
    margin = np.full(B, np.inf)
    r = 0
    for i in range(B):
        g = int(draft_len[i])
        base = r + i
        n = 0
        while True:
            row = target_logits[base + n]
            top = _first_argmax(row)
            if len(row) > 1:                      # (a one-token vocabulary has no runner-up)
                part = np.partition(row, -2)[-2:]
                margin[i] = min(margin[i], float(part[1] - part[0]))
            if n < g and int(draft_tokens[r + n]) == top:
                n += 1
                continue
            nxt[i] = top
            break
        n_acc[i] = n
        r += g
    return n_acc, nxt, margin


def accept_tree_greedy(draft_len, parents, draft_tokens, target_logits):
    """Greedy verification of token trees (the token trees of the related work named in Sec. I).

    Draft token t of request i hangs below token parents[r+t] of the same request (-1: the last
    prefix token).  Request i owns target rows base..base+g_i, base = q_offset[i] + i: row base is the
    model's output after the prefix, row base+1+t its output after token t.  From the root, move to
    the lowest-numbered child whose token equals the arg-max of the current node's row; stop when
    no child does.  Returns (n_accepted[B], path[R] (-1 beyond each request's path), next_token[B],
    margin[B]) with margin the smallest top-1/top-2 logit gap over the rows that were consulted.
    """
    B = len(draft_len)
    R = int(np.sum(draft_len))
    n_acc = np.zeros(B, dtype=np.int32)
    nxt = np.zeros(B, dtype=np.int32)
    path = np.full(R, -1, dtype=np.int32)
    margin = np.full(B, np.inf)
    r = 0
    for i in range(B):
        g = int(draft_len[i])
        base = r + i
        cur, n = -1, 0
        while True:
            row = target_logits[base + cur + 1]
            top = _first_argmax(row)
            if len(row) > 1:
                part = np.partition(row, -2)[-2:]
                margin[i] = min(margin[i], float(part[1] - part[0]))
            step = [t for t in range(g) if int(parents[r + t]) == cur and int(draft_tokens[r + t]) == top]
            if not step:
                nxt[i] = top
                break
            cur = step[0]
            path[r + n] = cur
            n += 1
        n_acc[i] = n
        r += g
    return n_acc, path, nxt, margin


def _inverse_cdf(mass: np.ndarray, u: float):
    """Smallest k with  mass[0]+...+mass[k] > u * total ; on rounding overshoot the last k
    with positive mass.  Also returns the distance of u*total to the nearest CDF step,
    relative to total."""
    c = np.cumsum(mass)
    total = c[-1]
    thr = u * total
    k = int(np.searchsorted(c, thr, side="right"))
    if k >= len(mass):
        k = int(np.nonzero(mass > 0)[0][-1])
    near = np.abs(c - thr).min() / total if total > 0 else 0.0
    return k, float(near)


def accept_rejection(draft_len, draft_tokens, target_logits, draft_logits, u_accept, u_sample):
    """Rejection-sampling verification with caller-supplied uniforms.

    Rows as in accept_greedy; p_t = softmax(target row t), q_t = softmax(draft row t), float64.
    Draft token d_t is kept iff  u_t * q_t(d_t) < p_t(d_t)  (u < min(1, p/q) without the
    division).  n_i = first rejected row, or g_i.  If a row was rejected the next token is drawn
    from the residual  r(x) = max(0, p_n(x) - q_n(x))  by inverse CDF with u'_i; if r sums to
    zero (p == q up to rounding) from p_n.  If all were kept it is drawn from the bonus row
    p_{g_i}.  Returns (n_accepted[B], next_token[B], margin[B]); margin is the smallest relative
    distance of any decision taken to its threshold (|u q - p| / p and the CDF distance).
    """
    B = len(draft_len)
    n_acc = np.zeros(B, dtype=np.int32)
    nxt = np.zeros(B, dtype=np.int32)
    margin = np.full(B, np.inf)
    r = 0
    for i in range(B):
        g = int(draft_len[i])
        base = r + i
        n = 0
        while n < g:
            d = int(draft_tokens[r + n])
            p = _softmax64(target_logits[base + n])
            q = _softmax64(draft_logits[r + n])
            lhs = float(u_accept[r + n]) * q[d]
            rhs = p[d]
            if rhs > 0:
                margin[i] = min(margin[i], abs(lhs - rhs) / rhs)
            if lhs < rhs:
                n += 1
            else:
                break
        p = _softmax64(target_logits[base + n])
        if n < g:
            q = _softmax64(draft_logits[r + n])
            mass = np.maximum(p - q, 0.0)
            if not mass.sum() > 0:
                mass = p
        else:
            mass = p
        k, near = _inverse_cdf(mass, float(u_sample[i]))
        margin[i] = min(margin[i], near)
        n_acc[i] = n
        nxt[i] = k
        r += g
    return n_acc, nxt, margin


def accept_tree_rejection(draft_len, parents, draft_tokens, target_logits, draft_logits, u_accept, u_sample):
    """Rejection-sampling verification of token trees: at every node the children are tried one after
    the other, and every rejected child takes its draft distribution out of what is left of the
    target distribution (the multi-round speculative sampling of the token-tree systems named in
    Sec. I; for a chain it is accept_rejection).

    Rows as in accept_tree_greedy; token t was drawn from q_t = softmax(draft row t).  At the node
    reached so far let R_0 = p = softmax(its target row) and s_0 = 1.  Child c (in index order,
    token d_c) is accepted iff  u_c * q_c(d_c) * s_k < R_k(d_c)  (u < min(1, r/q) for the residual
    r = R_k / s_k, without a division); the walk then moves to c with a fresh R_0.  A rejected child
    gives  R_{k+1}(x) = max(0, R_k(x) - s_k q_c(x)),  s_{k+1} = sum_x R_{k+1}(x); if that sum is zero
    (residual and q_c equal up to rounding) the child is ignored and R_k, s_k stay.  When no child is
    accepted (or there is none) the next token is drawn from R_k by inverse CDF with u'_i.
    Returns (n_accepted[B], path[R], next_token[B], margin[B]).
    """
    B = len(draft_len)
    R_rows = int(np.sum(draft_len))
    n_acc = np.zeros(B, dtype=np.int32)
    nxt = np.zeros(B, dtype=np.int32)
    path = np.full(R_rows, -1, dtype=np.int32)
    margin = np.full(B, np.inf)
    r = 0
    for i in range(B):
        g = int(draft_len[i])
        base = r + i
        V = target_logits.shape[1]
        cur, n = -1, 0
        while True:
            Rk = _softmax64(target_logits[base + cur + 1])
            sk = 1.0
            moved = False
            for c in range(g):
                if int(parents[r + c]) != cur:
                    continue
                q = _softmax64(draft_logits[r + c])
                d = int(draft_tokens[r + c])
                if 0 <= d < V:
                    lhs = float(u_accept[r + c]) * q[d] * sk
                    rhs = Rk[d]
                    if rhs > 0:
                        margin[i] = min(margin[i], abs(lhs - rhs) / rhs)
                    if lhs < rhs:
                        cur = c
                        path[r + n] = c
                        n += 1
                        moved = True
                        break
                nxt_R = np.maximum(Rk - sk * q, 0.0)
                tot = nxt_R.sum()
                if tot > 0:
                    Rk, sk = nxt_R, tot
            if moved:
                continue
            k, near = _inverse_cdf(Rk, float(u_sample[i]))
            margin[i] = min(margin[i], near)
            nxt[i] = k
            break
        n_acc[i] = n
        r += g
    return n_acc, path, nxt, margin

