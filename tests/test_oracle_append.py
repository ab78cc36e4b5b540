"""Pins of the oracle's KV append (the cache of Sec. II-A1 receiving the candidate tokens' K/V).

The oracle's scatter is checked against things it does not compute itself: a cache that was filled
position by position from dense per-request arrays (the test's own loop), and the dense brute-force
attention of test_oracle_attention, which never sees a page.
"""
import numpy as np

from oracle import spin_oracle as orc
from test_oracle_attention import tiny_problem, brute_force, run_oracle, bits_to_float


def blank_draft_slots(table, k_pool, v_pool, fill):
    """Remove the draft tokens from a filled cache, returning their rows as packed [R][Hkv][d]."""
    R = table.n_rows
    k_new = np.zeros((R,) + k_pool.shape[1:2] + k_pool.shape[3:], dtype=k_pool.dtype)
    v_new = np.zeros_like(k_new)
    P = table.page_size
    for i in range(table.n_req):
        pages = table.page_table[table.pt_offset[i]:table.pt_offset[i + 1]]
        for t in range(int(table.draft_len[i])):
            j = int(table.prefix_len[i]) + t
            r = int(table.q_offset[i]) + t
            k_new[r] = k_pool[pages[j // P], :, j % P, :]
            v_new[r] = v_pool[pages[j // P], :, j % P, :]
            k_pool[pages[j // P], :, j % P, :] = fill
            v_pool[pages[j // P], :, j % P, :] = fill
    return k_new, v_new


def do_append(table, kp, vp, k_new, v_new):
    orc.append_kv(table.prefix_len, table.draft_len, table.q_offset, table.pt_offset, table.page_table,
                  table.page_size, kp, vp, k_new, v_new)


def test_append_restores_a_cache_filled_position_by_position():
    prefix = np.array([5, 0, 9, 3, 16]); draft = np.array([3, 2, 1, 4, 8])
    table, q, kp, vp, dk, dv = tiny_problem(11, prefix, draft, n_q_heads=4, n_kv_heads=2)
    kp0, vp0 = kp.copy(), vp.copy()
    k_new, v_new = blank_draft_slots(table, kp, vp, 0x7fc0)      # NaN pattern where the drafts were
    assert not np.array_equal(kp, kp0)
    do_append(table, kp, vp, k_new, v_new)
    assert np.array_equal(kp, kp0) and np.array_equal(vp, vp0)   # every slot, owned or not


def test_append_touches_only_the_draft_slots():
    prefix = np.array([7, 1]); draft = np.array([2, 5])
    table, q, kp, vp, dk, dv = tiny_problem(12, prefix, draft)
    before_k, before_v = kp.copy(), vp.copy()
    R = table.n_rows
    k_new = np.full((R, 2, 8), 0x1234, dtype=np.uint16)
    v_new = np.full((R, 2, 8), 0x4321, dtype=np.uint16)
    do_append(table, kp, vp, k_new, v_new)
    changed_k = np.any(kp != before_k, axis=(1, 3))              # [page][slot]
    changed_v = np.any(vp != before_v, axis=(1, 3))
    assert changed_k.sum() == R and changed_v.sum() == R
    assert (kp[changed_k.nonzero()[0], :, changed_k.nonzero()[1], :] == 0x1234).all()
    assert (vp[changed_v.nonzero()[0], :, changed_v.nonzero()[1], :] == 0x4321).all()


def test_rows_and_heads_are_not_transposed():
    # each (row, head) carries its own marker value, found again at the dense position
    prefix = np.array([3, 6, 0]); draft = np.array([4, 1, 3])
    table, q, kp, vp, dk, dv = tiny_problem(13, prefix, draft, n_q_heads=3, n_kv_heads=3)
    R = table.n_rows
    k_new = (np.arange(R)[:, None, None] * 16 + np.arange(3)[None, :, None] + np.zeros((1, 1, 8))).astype(np.uint16)
    v_new = k_new + 0x100
    do_append(table, kp, vp, k_new, v_new)
    P = table.page_size
    for i in range(3):
        pages = table.page_table[table.pt_offset[i]:table.pt_offset[i + 1]]
        for t in range(int(draft[i])):
            j = int(prefix[i]) + t
            r = int(table.q_offset[i]) + t
            for h in range(3):
                assert (kp[pages[j // P], h, j % P] == r * 16 + h).all()
                assert (vp[pages[j // P], h, j % P] == r * 16 + h + 0x100).all()


def test_append_then_attention_matches_dense_brute_force():
    prefix = np.array([5, 0, 9]); draft = np.array([3, 2, 4])
    table, q, kp, vp, dk, dv = tiny_problem(14, prefix, draft)
    k_new, v_new = blank_draft_slots(table, kp, vp, 0x7fc0)
    do_append(table, kp, vp, k_new, v_new)
    got = run_oracle(table, q, kp, vp, 2, 2, 0.4)
    want = brute_force(table, q, dk, dv, 2, 2, 0.4)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)
