"""Pins for the attention oracle (CPU only).

Each test checks oracle.spin_oracle.verify_attention against something that is not the
oracle: a pure-Python brute force, a separately written decode attention, closed forms
and invariances that follow from Eq. (2) of Sec. II-A1 and Eq. (13) of Sec. V-A.
"""
import math

import numpy as np
import pytest
import torch

import spin_inputs as si
from oracle import spin_oracle as orc


def f32_to_bf16_bits(x):
    t = torch.from_numpy(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return si.bf16_bits(t)


def bits_to_float(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def tiny_problem(seed, prefix, draft, n_q_heads=2, n_kv_heads=2, d=8, page=4, shuffle=True, sigma=1.0):
    """Dense per-request K/V/Q lists (python floats via bf16 rounding) + the same data paged."""
    rng = np.random.default_rng(seed)
    table = si.make_table(prefix, draft, page, rng if shuffle else None)
    B = len(prefix)
    k_pool = np.zeros((table.n_pages, n_kv_heads, page, d), dtype=np.uint16)
    v_pool = np.zeros_like(k_pool)
    dense_k, dense_v = [], []
    for i in range(B):
        n = int(prefix[i] + draft[i])
        kb = f32_to_bf16_bits(rng.normal(0, sigma, (n, n_kv_heads, d)))
        vb = f32_to_bf16_bits(rng.normal(0, sigma, (n, n_kv_heads, d)))
        dense_k.append(bits_to_float(kb))
        dense_v.append(bits_to_float(vb))
        pt = table.page_table[table.pt_offset[i]:table.pt_offset[i + 1]]
        for j in range(n):
            k_pool[pt[j // page], :, j % page, :] = kb[j]
            v_pool[pt[j // page], :, j % page, :] = vb[j]
    R = table.n_rows
    qb = f32_to_bf16_bits(rng.normal(0, sigma, (R, n_q_heads, d)))
    return table, qb, k_pool, v_pool, dense_k, dense_v


def run_oracle(table, q, k_pool, v_pool, hq, hkv, scale):
    return orc.verify_attention(table.prefix_len, table.draft_len, table.q_offset, table.pt_offset,
                                table.page_table, table.page_size, q, k_pool, v_pool, hq, hkv, scale)


def brute_force(table, q_bits, dense_k, dense_v, hq, hkv, scale):
    """Triple python loop over rows, keys and dims with math.exp; no numpy linear algebra."""
    qf = bits_to_float(q_bits)
    R, _, d = qf.shape
    G = hq // hkv
    out = np.zeros((R, hq, d))
    for i in range(table.n_req):
        p, g = int(table.prefix_len[i]), int(table.draft_len[i])
        for t in range(g):
            r = int(table.q_offset[i]) + t
            for h in range(hq):
                hk = h // G
                last = p + t                          # last visible key
                scores = []
                for j in range(last + 1):
                    s = 0.0
                    for c in range(d):
                        s += qf[r, h, c] * dense_k[i][j, hk, c]
                    scores.append(scale * s)
                mx = max(scores)
                w = [math.exp(s - mx) for s in scores]
                tot = sum(w)
                for c in range(d):
                    acc = 0.0
                    for j in range(last + 1):
                        acc += w[j] * dense_v[i][j, hk, c]
                    out[r, h, c] = acc / tot
    return out


@pytest.mark.parametrize("seed,scale", [(0, 0.35), (1, 1.0), (2, 0.1)])
def test_brute_force_tiny(seed, scale):
    prefix = np.array([5, 0, 9, 3]); draft = np.array([3, 2, 1, 4])
    table, q, kp, vp, dk, dv = tiny_problem(seed, prefix, draft)
    got = run_oracle(table, q, kp, vp, 2, 2, scale)
    want = brute_force(table, q, dk, dv, 2, 2, scale)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_brute_force_gqa():
    prefix = np.array([6, 2]); draft = np.array([2, 3])
    table, q, kp, vp, dk, dv = tiny_problem(3, prefix, draft, n_q_heads=4, n_kv_heads=2)
    got = run_oracle(table, q, kp, vp, 4, 2, 0.5)
    want = brute_force(table, q, dk, dv, 4, 2, 0.5)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def decode_attention_reference(q_row, K, V, scale):
    """Ordinary single-query decode attention, written with scipy-free log-sum-exp."""
    s = scale * (K @ q_row)
    lse = np.log(np.sum(np.exp(s - s.max()))) + s.max()
    return np.exp(s - lse) @ V


def test_draft_len_one_is_decode_attention():
    prefix = np.array([7, 12, 1, 30]); draft = np.ones(4, dtype=np.int64)
    table, q, kp, vp, dk, dv = tiny_problem(4, prefix, draft, d=16)
    got = run_oracle(table, q, kp, vp, 2, 2, 0.25)
    qf = bits_to_float(q)
    for i in range(4):
        for h in range(2):
            # the single draft token sees the prefix and itself: a decode step at length p+1
            want = decode_attention_reference(qf[i, h], dk[i][:, h, :], dv[i][:, h, :], 0.25)
            np.testing.assert_allclose(got[i, h], want, rtol=1e-12, atol=1e-13)


def test_zero_queries_give_running_mean_of_values():
    prefix = np.array([4, 0]); draft = np.array([3, 2])
    table, q, kp, vp, dk, dv = tiny_problem(5, prefix, draft)
    q[:] = 0
    got = run_oracle(table, q, kp, vp, 2, 2, 1.0)
    for i in range(2):
        for t in range(int(draft[i])):
            want = dv[i][: prefix[i] + t + 1].mean(axis=0)          # [hkv, d]
            np.testing.assert_allclose(got[table.q_offset[i] + t], want, rtol=1e-13, atol=1e-14)


def test_constant_values_pass_through():
    prefix = np.array([9]); draft = np.array([4])
    table, q, kp, vp, dk, dv = tiny_problem(6, prefix, draft)
    vp[:] = f32_to_bf16_bits(np.float32(0.375))
    got = run_oracle(table, q, kp, vp, 2, 2, 1.0)
    np.testing.assert_allclose(got, 0.375, rtol=1e-13)


def test_dominant_key_selects_its_value():
    prefix = np.array([10]); draft = np.array([2])
    table, q, kp, vp, dk, dv = tiny_problem(7, prefix, draft, n_q_heads=1, n_kv_heads=1, d=8)
    pt = table.page_table
    # all queries = e_0 * 8; key 6 = e_0 * 64, the rest tiny -> score 512 vs ~0
    q[:] = 0; q[:, :, 0] = f32_to_bf16_bits(np.float32(8.0))
    kp[:] = 0
    kp[pt[6 // 4], 0, 6 % 4, 0] = f32_to_bf16_bits(np.float32(64.0))
    got = run_oracle(table, q, kp, vp, 1, 1, 1.0)
    for t in range(2):
        np.testing.assert_allclose(got[t, 0], dv[0][6, 0], rtol=1e-12, atol=1e-200)


def test_empty_prefix_first_row_returns_first_value():
    prefix = np.array([0]); draft = np.array([3])
    table, q, kp, vp, dk, dv = tiny_problem(8, prefix, draft)
    got = run_oracle(table, q, kp, vp, 2, 2, 0.7)
    np.testing.assert_allclose(got[0], dv[0][0], rtol=1e-14)


def test_causal_mask_inside_draft_block():
    # A later draft key must not influence an earlier draft row: change the last draft
    # token's K and V and only the last row may move.
    prefix = np.array([5]); draft = np.array([3])
    table, q, kp, vp, dk, dv = tiny_problem(9, prefix, draft)
    base = run_oracle(table, q, kp, vp, 2, 2, 0.5)
    j = 7
    pg = table.page_table[j // 4]
    kp[pg, :, j % 4, :] = f32_to_bf16_bits(np.full((2, 8), 3.0, dtype=np.float32))
    vp[pg, :, j % 4, :] = f32_to_bf16_bits(np.full((2, 8), -5.0, dtype=np.float32))
    moved = run_oracle(table, q, kp, vp, 2, 2, 0.5)
    np.testing.assert_array_equal(moved[:2], base[:2])
    assert np.abs(moved[2] - base[2]).max() > 1e-3


def test_key_shift_invariance():
    # Adding one vector c to every key of a request adds Q_t.c to every score of row t.
    # Dyadic inputs keep the shifted keys exactly representable in bf16.
    rng = np.random.default_rng(10)
    prefix = np.array([6]); draft = np.array([3])
    table, q, kp, vp, dk, dv = tiny_problem(10, prefix, draft)
    kq = rng.integers(-4, 5, size=kp.shape).astype(np.float32) / 4
    kp[:] = f32_to_bf16_bits(kq)
    q[:] = f32_to_bf16_bits(rng.integers(-4, 5, size=q.shape).astype(np.float32) / 4)
    base = run_oracle(table, q, kp, vp, 2, 2, 0.5)
    c = rng.integers(-4, 5, size=(2, 8)).astype(np.float32) / 2
    kp2 = f32_to_bf16_bits(kq + c[None, :, None, :])
    moved = run_oracle(table, q, kp2, vp, 2, 2, 0.5)
    np.testing.assert_allclose(moved, base, rtol=1e-11, atol=1e-12)


def test_element_types_read_as_values():
    """The oracle takes bf16 as raw uint16 bit patterns and fp16 as a numpy float16 array.  Dyadic values are
    exact in both types, so the two forms of the same problem give the same answer to the last bit, and so does the
    float64 form; half-precision values that bf16 cannot hold (1 + 2^-10) are read exactly too."""
    rng = np.random.default_rng(12)
    prefix = np.array([9, 2]); draft = np.array([3, 1])
    table, q, kp, vp, dk, dv = tiny_problem(12, prefix, draft)
    qv = rng.integers(-8, 9, size=q.shape).astype(np.float32) / 8
    kv = rng.integers(-8, 9, size=kp.shape).astype(np.float32) / 8
    vv = rng.integers(-8, 9, size=vp.shape).astype(np.float32) / 8
    as_bf16 = run_oracle(table, f32_to_bf16_bits(qv), f32_to_bf16_bits(kv), f32_to_bf16_bits(vv), 2, 2, 0.5)
    as_f16 = run_oracle(table, qv.astype(np.float16), kv.astype(np.float16), vv.astype(np.float16), 2, 2, 0.5)
    as_f64 = run_oracle(table, qv.astype(np.float64), kv.astype(np.float64), vv.astype(np.float64), 2, 2, 0.5)
    np.testing.assert_array_equal(as_bf16, as_f16)
    np.testing.assert_array_equal(as_bf16, as_f64)
    fine = np.float16(1.0 + 2.0 ** -10)
    vv16 = np.full(vp.shape, fine, dtype=np.float16)
    out = run_oracle(table, qv.astype(np.float16), kv.astype(np.float16), vv16, 2, 2, 0.5)
    np.testing.assert_allclose(out[~np.isnan(out)], 1.0 + 2.0 ** -10, rtol=1e-15)


def test_joint_permutation_of_prefix_pairs():
    prefix = np.array([8]); draft = np.array([2])
    table, q, kp, vp, dk, dv = tiny_problem(11, prefix, draft, shuffle=False)
    base = run_oracle(table, q, kp, vp, 2, 2, 0.5)
    perm = np.random.default_rng(0).permutation(8)
    kp2, vp2 = kp.copy(), vp.copy()
    for dst, src in enumerate(perm):
        kp2[dst // 4, :, dst % 4] = kp[src // 4, :, src % 4]
        vp2[dst // 4, :, dst % 4] = vp[src // 4, :, src % 4]
    moved = run_oracle(table, q, kp2, vp2, 2, 2, 0.5)
    np.testing.assert_allclose(moved, base, rtol=1e-12, atol=1e-13)


def test_page_relocation_changes_nothing():
    prefix = np.array([9, 3]); draft = np.array([2, 4])
    table, q, kp, vp, dk, dv = tiny_problem(12, prefix, draft)
    base = run_oracle(table, q, kp, vp, 2, 2, 0.5)
    perm = np.random.default_rng(1).permutation(table.n_pages)     # old page -> new page
    kp2 = np.empty_like(kp); vp2 = np.empty_like(vp)
    kp2[perm] = kp; vp2[perm] = vp
    t2 = si.RequestTable(table.prefix_len, table.draft_len, table.q_offset, table.pt_offset,
                         perm[table.page_table].astype(np.int32), table.page_size, table.n_pages)
    moved = run_oracle(t2, q, kp2, vp2, 2, 2, 0.5)
    np.testing.assert_array_equal(moved, base)


def test_unowned_slots_never_read():
    cfg = si.CONFIGS["tiny"]
    b = si.make_verify_batch(cfg, 3, poison_unused=True)
    clean = si.make_verify_batch(cfg, 3, poison_unused=False)
    assert torch.isnan(b.k_pool.float()).any()
    args = lambda x: (x.table.prefix_len, x.table.draft_len, x.table.q_offset, x.table.pt_offset,
                      x.table.page_table, cfg.page_size, si.bf16_bits(x.q), si.bf16_bits(x.k_pool),
                      si.bf16_bits(x.v_pool), cfg.n_q_heads, cfg.n_kv_heads, 0.125)
    got = orc.verify_attention(*args(b))
    want = orc.verify_attention(*args(clean))
    assert np.isfinite(got).all()
    np.testing.assert_array_equal(got, want)


def test_gqa_equals_mha_with_repeated_heads():
    prefix = np.array([7, 4]); draft = np.array([3, 2])
    table, q, kp, vp, dk, dv = tiny_problem(13, prefix, draft, n_q_heads=4, n_kv_heads=2)
    got = run_oracle(table, q, kp, vp, 4, 2, 0.4)
    kp_rep = np.repeat(kp, 2, axis=1); vp_rep = np.repeat(vp, 2, axis=1)
    want = run_oracle(table, q, kp_rep, vp_rep, 4, 4, 0.4)
    np.testing.assert_array_equal(got, want)


def random_rectangles(rng, p, g):
    """A random exact tiling of the visible cells of a (g rows x p+g keys) score matrix:
    cut rows into bands, and each band's key range [0, p+last_row+1) into pieces."""
    subs = []
    qb = 0
    while qb < g:
        ql = int(rng.integers(1, g - qb + 1))
        end = p + qb + ql
        kb = 0
        while kb < end:
            kl = int(rng.integers(1, end - kb + 1))
            subs.append((qb, ql, kb, kl))
            kb += kl
        qb += ql
    return subs


@pytest.mark.parametrize("seed", range(6))
def test_decomposition_invariance_eq13(seed):
    rng = np.random.default_rng(100 + seed)
    prefix = rng.integers(0, 12, size=3); draft = rng.integers(1, 6, size=3)
    table, q, kp, vp, dk, dv = tiny_problem(seed, prefix, draft, n_q_heads=2, n_kv_heads=1)
    whole = run_oracle(table, q, kp, vp, 2, 1, 0.6)
    base_args = (table.prefix_len, table.draft_len, table.q_offset, table.pt_offset, table.page_table,
                 table.page_size, q, kp, vp, 2, 1, 0.6)
    # (a) width-w split of the draft rows, (b) length-L split of the keys, (c) random 2-D tilings
    for subs in (orc.decompose_q_split(prefix, draft, 2),
                 orc.decompose_kv_split(prefix, draft, 3),
                 orc.decompose_kv_split(prefix, draft, 4)):
        got = orc.verify_attention_decomposed(*base_args, subs)
        np.testing.assert_allclose(got, whole, rtol=1e-12, atol=1e-13)
    subs = [(i,) + r for i in range(3) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))]
    got = orc.verify_attention_decomposed(*base_args, np.array(subs))
    np.testing.assert_allclose(got, whole, rtol=1e-12, atol=1e-13)


def test_decomposed_mode_matches_brute_force_directly():
    # pins verify_attention_decomposed to the python loops, not just to verify_attention
    prefix = np.array([5, 2]); draft = np.array([4, 3])
    table, q, kp, vp, dk, dv = tiny_problem(21, prefix, draft)
    subs = orc.decompose_kv_split(prefix, draft, 4)
    got = orc.verify_attention_decomposed(table.prefix_len, table.draft_len, table.q_offset,
                                          table.pt_offset, table.page_table, table.page_size,
                                          q, kp, vp, 2, 2, 1.0, subs)
    want = brute_force(table, q, dk, dv, 2, 2, 1.0)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_wrong_denominator_is_detected():
    # Normalising each sub-request on its own (what Sec. V-A warns against) must NOT match:
    # guards against a pin that cannot tell Eq. (13) from per-piece softmax.
    prefix = np.array([6]); draft = np.array([2])
    table, q, kp, vp, dk, dv = tiny_problem(22, prefix, draft, n_q_heads=1, n_kv_heads=1)
    whole = run_oracle(table, q, kp, vp, 1, 1, 1.0)
    subs = orc.decompose_kv_split(prefix, draft, 4)
    qf = bits_to_float(q)
    wrong = np.zeros_like(whole)
    for _, qb, ql, kb, kl in subs:
        for t in range(ql):
            js = [j for j in range(kb, kb + kl) if j <= 6 + t]
            if not js:
                continue
            s = np.array([qf[t, 0] @ dk[0][j, 0] for j in js])
            a = np.exp(s - s.max()); a /= a.sum()
            wrong[t, 0] += a @ dv[0][js, 0]
    assert np.abs(wrong - whole).max() > 1e-2


def test_sampled_mode_matches_full():
    cfg = si.CONFIGS["tiny"]
    b = si.make_verify_batch(cfg, 0)
    t = b.table
    args = (t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, cfg.page_size,
            si.bf16_bits(b.q), si.bf16_bits(b.k_pool), si.bf16_bits(b.v_pool), 2, 2, 0.125)
    full = orc.verify_attention(*args)
    part = orc.verify_attention(*args, requests=[2], heads=[1])
    r0, r1 = t.q_offset[2], t.q_offset[3]
    np.testing.assert_array_equal(part[r0:r1, 1], full[r0:r1, 1])
    assert np.isnan(part[:r0]).all()
