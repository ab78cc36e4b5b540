"""GPU parity tests: the HIP path (through the C ABI) against the float64 CPU oracle on the same
seeded inputs.  Attention: every element within 2e-2 absolute OR 2e-2 relative of the oracle
(plus tighter aggregate bounds).  Acceptance: accepted lengths and token ids bit-exact.
"""
import dataclasses
import math
import os

import numpy as np
import pytest
import torch

import spin_inputs as si
from oracle import spin_oracle as orc
from test_oracle_attention import random_rectangles

pytestmark = pytest.mark.gpu

TOL = 2e-2


@pytest.fixture(scope="module")
def ctx():
    import paper_2503_15921_amd as spin
    c = spin.SpinContext(0)
    yield c
    c.close()


def hip_attention(ctx, batch, subs=None, scale=0.0, waves=None):
    t = batch.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    out = torch.full_like(batch.q, float("nan"))
    if waves is not None:
        ctx.set_waves(waves)
    try:
        ctx.verify_attn(tab, batch.k_pool, batch.v_pool, batch.q, out, batch.cfg.n_q_heads, subs=subs,
                        softmax_scale=scale)
        torch.cuda.synchronize()
    finally:
        if waves is not None:
            ctx.set_waves(0)
    return out


def oracle_attention(batch, scale, requests=None, heads=None):
    t = batch.table
    cfg = batch.cfg
    if scale <= 0:
        scale = 1.0 / math.sqrt(cfg.head_dim)
    return orc.verify_attention(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, cfg.page_size,
                                si.host_elems(batch.q), si.host_elems(batch.k_pool), si.host_elems(batch.v_pool),
                                cfg.n_q_heads, cfg.n_kv_heads, scale, requests=requests, heads=heads)


def assert_close(got_bf16, want, what=""):
    got = got_bf16.float().cpu().numpy().astype(np.float64)
    sel = ~np.isnan(want)
    assert sel.any()
    g, w = got[sel], want[sel]
    assert np.isfinite(g).all(), f"{what}: non-finite output"
    err = np.abs(g - w)
    ok = (err <= TOL) | (err <= TOL * np.abs(w))
    rel_rms = math.sqrt((err ** 2).mean() / max((w ** 2).mean(), 1e-300))
    assert ok.all(), f"{what}: {np.count_nonzero(~ok)} of {ok.size} elements off, max abs err {err.max():.3e}"
    # aggregate bound: bf16 output rounding is 2^-9 relative; P is rounded to bf16 before P.V
    assert rel_rms < 1e-2, f"{what}: relative RMS error {rel_rms:.3e}"
    return err.max(), rel_rms


def make_cfg(name, n_req, hq, hkv, d, page=16):
    return si.VerifyConfig(name, n_req, hq, hkv, d, 0, 0, "uniform", "uniform", page_size=page)


# ------------------------------------------------------------------------------ attention
@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("scale", [0.0, 1.0])
def test_tiny_config(ctx, seed, scale):
    b = si.make_verify_batch(si.CONFIGS["tiny"], seed, device="cuda")
    assert_close(hip_attention(ctx, b, scale=scale), oracle_attention(b, scale), f"tiny seed {seed} scale {scale}")


EDGE_PREFIX = np.array([0, 1, 15, 16, 31, 32, 33, 255, 256, 257, 511, 600, 1023, 1300])
EDGE_DRAFT = np.array([1, 2, 16, 1, 3, 8, 5, 7, 1, 4, 16, 2, 9, 6])


@pytest.mark.parametrize("hq,hkv,d", [(4, 4, 128), (2, 2, 64), (8, 4, 128), (6, 2, 128), (8, 2, 64), (16, 2, 128)])
def test_ragged_edges_and_groups(ctx, hq, hkv, d):
    # prefix lengths around page / block / chunk boundaries, draft lengths 1..16, group sizes 1, 2, 3, 4, 8
    draft = np.minimum(EDGE_DRAFT, 64 // (hq // hkv)) if hq // hkv > 4 else EDGE_DRAFT
    cfg = make_cfg("edges", len(EDGE_PREFIX), hq, hkv, d)
    b = si.make_verify_batch(cfg, 7, device="cuda", prefix_len=EDGE_PREFIX, draft_len=draft, poison_unused=True)
    assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), f"edges hq={hq} hkv={hkv} d={d}")


def test_wide_group_many_rows(ctx):
    # 8 query heads per KV head and up to 8 draft rows: 64 rows in one tile (four MFMA column tiles)
    prefix = np.array([700, 90, 300, 40]); draft = np.array([8, 5, 3, 1])
    cfg = make_cfg("gqa8", 4, 16, 2, 128)
    b = si.make_verify_batch(cfg, 11, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), "gqa8")
    # more rows than one tile holds: 12 draft rows x 8 heads -> the scheduler cuts row bands
    prefix = np.array([500, 64]); draft = np.array([12, 16])
    b = si.make_verify_batch(cfg, 12, device="cuda", prefix_len=prefix, draft_len=draft)
    assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), "gqa8 row bands")


@pytest.mark.parametrize("group", [5, 6, 7, 12, 16, 32, 64])
@pytest.mark.parametrize("d", [64, 128])
def test_unusual_group_sizes(ctx, group, d):
    # query heads per KV head that do not divide a 16-row tile, and multi-query extremes up to the limit of 64
    hkv = 2 if group <= 16 else 1
    cfg = make_cfg(f"group{group}", 5, group * hkv, hkv, d)
    prefix = np.array([0, 31, 333, 1200, 64]); draft = np.array([1, 3, 5, 2, 13])
    b = si.make_verify_batch(cfg, 16 + group, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), f"group {group} d {d}")
    _, masks = si.random_trees(draft, np.random.default_rng(group))
    assert_close(hip_tree_attention(ctx, b, masks), oracle_tree_attention(b, masks), f"group {group} d {d} trees")


@pytest.mark.parametrize("waves", [1, 2, 5, 64, 1000, 16384])
def test_wavefront_counts(ctx, waves):
    # the same batch cut into 1 ... many shares: everything direct, long carried runs, many partial joins
    cfg = make_cfg("shares", 6, 4, 4, 128)
    prefix = np.array([5, 100, 640, 1025, 2047, 5000]); draft = np.array([3, 1, 8, 2, 5, 4])
    b = si.make_verify_batch(cfg, 13, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    assert_close(hip_attention(ctx, b, waves=waves), oracle_attention(b, 0.0), f"waves {waves}")


def test_queued_tail_of_long_batch(ctx):
    # long enough that the scheduler hands the last tenth of the blocks out from its queue
    import paper_2503_15921_amd as spin
    cfg = make_cfg("queued", 6, 8, 8, 128)
    prefix = np.array([8100, 9000, 7000, 8500, 9500, 8000]); draft = np.array([4, 8, 1, 6, 2, 5])
    pcs = spin.schedule(prefix, draft, None, 16, 1, 8, 64)
    assert (pcs[:, 8] & spin.PIECE_QUEUED).any()
    b = si.make_verify_batch(cfg, 21, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    assert_close(hip_attention(ctx, b, waves=64), oracle_attention(b, 0.0), "queued tail")


@pytest.mark.parametrize("hq,hkv", [(4, 4), (16, 2)])
def test_very_long_context(ctx, hq, hkv):
    # one request far longer than a piece may be (136 pages), next to short ones
    cfg = make_cfg("long", 3, hq, hkv, 128)
    prefix = np.array([150001, 17, 40000]); draft = np.array([8, 3, 5])
    b = si.make_verify_batch(cfg, 23, device="cuda", prefix_len=prefix, draft_len=draft)
    got = hip_attention(ctx, b)
    assert not torch.isnan(got.float()).any()
    want = oracle_attention(b, 0.0, heads=[0, hq - 1])
    assert_close(got, want, f"long context {hq}/{hkv}")


def test_many_short_requests(ctx):
    rng = np.random.default_rng(24)
    n = 3000
    cfg = make_cfg("many", n, 2, 2, 64)
    prefix = rng.integers(0, 41, n); draft = rng.integers(1, 5, n)
    b = si.make_verify_batch(cfg, 24, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), "3000 short requests")


def test_unit_scale_peaked_softmax(ctx):
    # the literal Eq. (2) (no 1/sqrt(d)): scores ~ N(0, d), softmax dominated by a few keys, |O| ~ 1
    cfg = make_cfg("peaked", 5, 4, 4, 128)
    prefix = np.array([33, 400, 1000, 64, 7]); draft = np.array([4, 8, 2, 1, 5])
    b = si.make_verify_batch(cfg, 14, device="cuda", prefix_len=prefix, draft_len=draft)
    assert_close(hip_attention(ctx, b, scale=1.0), oracle_attention(b, 1.0), "scale 1")


@pytest.mark.parametrize("hq,hkv", [(4, 4), (16, 2)])
def test_large_scores(ctx, hq, hkv):
    # queries and keys 8x larger with the literal scale: scores of several thousand either sign, so almost
    # every exponential underflows and each row follows one key (a hard arg-max over the visible keys)
    cfg = make_cfg("large", 4, hq, hkv, 128)
    prefix = np.array([33, 400, 1500, 0]); draft = np.array([4, 8, 2, 3])
    b = si.make_verify_batch(cfg, 15, device="cuda", prefix_len=prefix, draft_len=draft)
    b.q.mul_(8.0); b.k_pool.mul_(8.0)
    got = hip_attention(ctx, b, scale=1.0)
    assert torch.isfinite(got.float()).all()
    assert_close(got, oracle_attention(b, 1.0), f"large scores {hq}/{hkv}")


def test_draft_len_one_is_decode(ctx):
    cfg = make_cfg("decode", 8, 8, 8, 128)
    prefix = np.array([0, 17, 100, 256, 511, 512, 900, 2000]); draft = np.ones(8, dtype=np.int64)
    b = si.make_verify_batch(cfg, 15, device="cuda", prefix_len=prefix, draft_len=draft)
    got = hip_attention(ctx, b)
    assert_close(got, oracle_attention(b, 0.0), "decode")
    # p = 0: the single row sees only itself -> O = V of that token, exactly (bf16 in, bf16 out)
    pg = int(b.table.page_table[b.table.pt_offset[0]])
    assert torch.equal(got[0], b.v_pool[pg, :, 0, :])


def test_constant_values_and_zero_queries(ctx):
    cfg = make_cfg("closed", 3, 2, 2, 128)
    prefix = np.array([50, 300, 3]); draft = np.array([4, 2, 6])
    b = si.make_verify_batch(cfg, 16, device="cuda", prefix_len=prefix, draft_len=draft)
    b.v_pool.fill_(0.375)
    got = hip_attention(ctx, b)
    assert torch.allclose(got.float(), torch.full_like(got.float(), 0.375), rtol=2 ** -8, atol=0)
    b2 = si.make_verify_batch(cfg, 16, device="cuda", prefix_len=prefix, draft_len=draft)
    b2.q.zero_()
    assert_close(hip_attention(ctx, b2), oracle_attention(b2, 0.0), "zero queries (running mean of V)")


def decompositions(rng, prefix, draft):
    yield "q-split 4", orc.decompose_q_split(prefix, draft, 4)
    yield "q-split 1", orc.decompose_q_split(prefix, draft, 1)
    yield "kv-split 100", orc.decompose_kv_split(prefix, draft, 100)
    yield "kv-split 37", orc.decompose_kv_split(prefix, draft, 37)
    yield "kv-split 256", orc.decompose_kv_split(prefix, draft, 256)
    subs = [(i,) + r for i in range(len(prefix)) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))]
    yield "random rectangles", np.array(subs, dtype=np.int32)


def test_decomposition_leaves_outputs_unchanged(ctx):
    # Eq. (13): whatever the cut, a row is normalised over all tokens of its original request
    rng = np.random.default_rng(5)
    cfg = make_cfg("decomp", 6, 4, 2, 128)
    prefix = np.array([0, 20, 129, 300, 700, 1100]); draft = np.array([3, 16, 8, 5, 16, 2])
    b = si.make_verify_batch(cfg, 17, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    want = oracle_attention(b, 0.0)
    whole = hip_attention(ctx, b)
    assert_close(whole, want, "undivided")
    for name, subs in decompositions(rng, prefix, draft):
        got = hip_attention(ctx, b, subs=subs)
        assert_close(got, want, name)
        # and against the undivided GPU result: only summation order may differ
        diff = (got.float() - whole.float()).abs().max().item()
        assert diff <= 4e-3, f"{name}: differs from the undivided run by {diff}"


def test_page_relocation_is_bitwise_invariant(ctx):
    cfg = make_cfg("reloc", 5, 4, 4, 128)
    prefix = np.array([10, 200, 513, 64, 1000]); draft = np.array([2, 7, 3, 1, 8])
    b = si.make_verify_batch(cfg, 18, device="cuda", prefix_len=prefix, draft_len=draft)
    base = hip_attention(ctx, b)
    perm = torch.from_numpy(np.random.default_rng(2).permutation(b.table.n_pages)).cuda()
    k2 = torch.empty_like(b.k_pool); v2 = torch.empty_like(b.v_pool)
    k2[perm] = b.k_pool; v2[perm] = b.v_pool
    t = b.table
    t2 = si.RequestTable(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset,
                         perm.cpu().numpy()[t.page_table].astype(np.int32), t.page_size, t.n_pages)
    moved = hip_attention(ctx, si.VerifyBatch(cfg, t2, b.q, k2, v2))
    assert torch.equal(moved.view(torch.int16), base.view(torch.int16))


def test_repeat_runs_are_deterministic(ctx):
    b = si.make_verify_batch(si.CONFIGS["tiny"], 4, device="cuda")
    a = hip_attention(ctx, b)
    for _ in range(3):
        assert torch.equal(hip_attention(ctx, b).view(torch.int16), a.view(torch.int16))


@pytest.mark.parametrize("hq,hkv,d", [(4, 2, 128), (16, 2, 128), (8, 2, 64), (16, 2, 64)])
def test_other_cache_layout_via_strides(ctx, hq, hkv, d):
    # pool stored as [page][slot][head][dim] with a padded token pitch: same result through strides
    # (groups of 2, 4 and 8 query heads: the single-wavefront and the grouped-query kernel)
    cfg = make_cfg("layout", 4, hq, hkv, d)
    prefix = np.array([40, 333, 5, 800]); draft = np.array([5, 2, 8, 3])
    b = si.make_verify_batch(cfg, 19, device="cuda", prefix_len=prefix, draft_len=draft)
    want = hip_attention(ctx, b)
    n_pages, hkv, P, d = b.k_pool.shape
    pitch = d + 64
    k_alt = torch.zeros((n_pages, P, hkv, pitch), dtype=torch.bfloat16, device="cuda")
    v_alt = torch.zeros_like(k_alt)
    k_alt[..., :d] = b.k_pool.permute(0, 2, 1, 3); v_alt[..., :d] = b.v_pool.permute(0, 2, 1, 3)
    kv = k_alt.permute(0, 2, 1, 3)[..., :d]; vv = v_alt.permute(0, 2, 1, 3)[..., :d]     # logical [page][head][slot][dim]
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    out = torch.empty_like(b.q)
    ctx.verify_attn(tab, kv, vv, b.q, out, cfg.n_q_heads)
    torch.cuda.synchronize()
    assert torch.equal(out.view(torch.int16), want.view(torch.int16))
    assert_close(out, oracle_attention(b, 0.0), "token-major cache layout")


@pytest.mark.parametrize("dim", [1, 2])
@pytest.mark.parametrize("hq,hkv,d", [(4, 2, 128), (16, 2, 128), (16, 2, 64)])
def test_k_and_v_paired_in_one_allocation(ctx, hq, hkv, d, dim):
    # one buffer holds both caches, [page][K|V][head][slot][dim] (dim 1) or [page][head][K|V][slot][dim] (dim 2): the
    # pools are two views into it, with a doubled page (and head) stride; append first, then attention over the result
    cfg = make_cfg("paired", 4, hq, hkv, d)
    prefix = np.array([40, 333, 5, 800]); draft = np.array([5, 2, 8, 3])
    b = si.make_verify_batch(cfg, 23, device="cuda", prefix_len=prefix, draft_len=draft)
    k_new, v_new = new_rows(b, 123)
    want_k, want_v = oracle_append(b, k_new, v_new)
    both = torch.stack([b.k_pool, b.v_pool], dim=dim).contiguous()
    kv, vv = (both[:, 0], both[:, 1]) if dim == 1 else (both[:, :, 0], both[:, :, 1])
    assert kv.stride() == vv.stride() and kv.stride()[0] == 2 * b.k_pool.stride()[0]
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    ctx.append_kv(tab, kv, vv, k_new, v_new)
    out = torch.empty_like(b.q)
    ctx.verify_attn(tab, kv, vv, b.q, out, cfg.n_q_heads)
    torch.cuda.synchronize()
    assert np.array_equal(si.bf16_bits(kv.contiguous()), want_k) and np.array_equal(si.bf16_bits(vv.contiguous()), want_v)
    b.k_pool = torch.from_numpy(want_k.view(np.int16)).view(torch.bfloat16).to("cuda")
    b.v_pool = torch.from_numpy(want_v.view(np.int16)).view(torch.bfloat16).to("cuda")
    assert_close(out, oracle_attention(b, 0.0), f"K and V paired along dimension {dim}")


def test_small_pages(ctx):
    cfg = make_cfg("page4", 4, 2, 2, 64, page=4)
    prefix = np.array([9, 130, 0, 61]); draft = np.array([3, 5, 2, 1])
    b = si.make_verify_batch(cfg, 20, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), "page size 4")


@pytest.mark.parametrize("page", [1, 2, 8, 32, 64, 128, 256])
def test_other_page_sizes(ctx, page):
    cfg = make_cfg(f"page{page}", 5, 4, 2, 128, page=page)
    prefix = np.array([0, 37, 129, 500, 1031]); draft = np.array([2, 7, 1, 16, 4])
    b = si.make_verify_batch(cfg, 30 + page, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), f"page size {page}")


@pytest.mark.parametrize("seed", range(24))
def test_random_batches(ctx, seed):
    """Random shapes, groups, page sizes, decompositions and share counts against the oracle."""
    rng = np.random.default_rng(1000 + seed)
    hkv = int(rng.choice([1, 2, 3, 5]))
    group = int(rng.choice([1, 1, 2, 4, 8]))
    d = int(rng.choice([64, 128]))
    page = int(rng.choice([4, 16, 16, 32]))
    n_req = int(rng.integers(1, 9))
    prefix = np.where(rng.random(n_req) < 0.3, rng.integers(0, 40, n_req), rng.integers(0, 2500, n_req))
    max_draft = 16 if group <= 4 else 8
    draft = rng.integers(1, max_draft + 1, n_req)
    cfg = make_cfg("random", n_req, hkv * group, hkv, d, page=page)
    b = si.make_verify_batch(cfg, 2000 + seed, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    kind = int(rng.integers(4))
    if kind == 0:
        subs = None
    elif kind == 1:
        subs = orc.decompose_q_split(prefix, draft, int(rng.integers(1, 6)))
    elif kind == 2:
        subs = orc.decompose_kv_split(prefix, draft, int(rng.integers(1, 700)))
    else:
        subs = np.array([(i,) + r for i in range(n_req) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))],
                        dtype=np.int32)
    waves = int(rng.choice([1, 3, 17, 256, 0]))
    scale = float(rng.choice([0.0, 0.0, 0.3, 1.0]))
    what = f"seed {seed}: hkv {hkv} group {group} d {d} page {page} kind {kind} waves {waves} scale {scale}"
    print(what, flush=True)
    assert_close(hip_attention(ctx, b, subs=subs, scale=scale, waves=waves), oracle_attention(b, scale), what)


def wide_random_case(ctx, seed):
    """One random case over every axis at once: shapes, group sizes, page sizes, both element types, head- and
    token-major pages with padded pitches, decompositions, share counts, scales, linear and tree drafts."""
    rng = np.random.default_rng(50000 + seed)
    hkv = int(rng.choice([1, 2, 3, 5, 8]))
    group = int(rng.choice([1, 1, 2, 3, 4, 5, 8, 16]))
    d = int(rng.choice([64, 128]))
    page = int(rng.choice([1, 2, 4, 8, 16, 16, 32, 64, 128]))
    n_req = int(rng.integers(1, 12))
    prefix = np.where(rng.random(n_req) < 0.3, rng.integers(0, 40, n_req), rng.integers(0, 3000, n_req))
    draft = rng.integers(1, max(1, min(16, 64 // group)) + 1, n_req)
    dtype = torch.float16 if rng.random() < 0.4 else torch.bfloat16
    cfg = make_cfg("wide", n_req, hkv * group, hkv, d, page=page)
    b = si.make_verify_batch(cfg, 60000 + seed, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True,
                             dtype=dtype)
    layout = "head-major"
    if rng.random() < 0.4:
        n_pages, _, P, _ = b.k_pool.shape
        pitch = d + int(rng.choice([0, 0, 8, 64]))
        k_alt = torch.full((n_pages, P, hkv, pitch), float("nan"), dtype=dtype, device="cuda")
        v_alt = k_alt.clone()
        k_alt[..., :d] = b.k_pool.permute(0, 2, 1, 3); v_alt[..., :d] = b.v_pool.permute(0, 2, 1, 3)
        b.k_pool = k_alt.permute(0, 2, 1, 3)[..., :d]; b.v_pool = v_alt.permute(0, 2, 1, 3)[..., :d]
        layout = f"token-major, pitch {pitch}"
    kind = int(rng.integers(4))
    if kind == 0:
        subs = None
    elif kind == 1:
        subs = orc.decompose_q_split(prefix, draft, int(rng.integers(1, 6)))
    elif kind == 2:
        subs = orc.decompose_kv_split(prefix, draft, int(rng.integers(1, 700)))
    else:
        subs = np.array([(i,) + r for i in range(n_req) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))],
                        dtype=np.int32)
    waves = int(rng.choice([1, 3, 17, 256, 0, 0]))
    scale = float(rng.choice([0.0, 0.0, 0.3, 1.0]))
    tree = rng.random() < 0.3
    what = (f"seed {seed}: hkv {hkv} group {group} d {d} page {page} {layout} {dtype} kind {kind} waves {waves} "
            f"scale {scale} tree {tree}")
    if tree:
        masks = si.random_trees(draft, rng, str(rng.choice(["random", "star", "wide", "chain"])))[1]
        assert_close(hip_tree_attention(ctx, b, masks, subs=subs, scale=scale, waves=waves),
                     oracle_tree_attention(b, masks, scale), what)
    else:
        assert_close(hip_attention(ctx, b, subs=subs, scale=scale, waves=waves), oracle_attention(b, scale), what)


def test_random_batches_over_all_axes(ctx):
    """48 cases by default; SPIN_SWEEP_CASES=n runs the first n seeds (12000 have passed with the kernels as they stand)."""
    n = int(os.environ.get("SPIN_SWEEP_CASES", "48"))
    for seed in range(n):
        wide_random_case(ctx, seed)
        if seed % 100 == 99:
            print(f"{seed + 1} cases", flush=True)


BENCH_SEED = 3   # the seed bench.py draws every configuration's batch with


def product_subs(cfg, table):
    """The configuration's own decomposition, made by the product's spin_decompose (and equal to the oracle's)."""
    import paper_2503_15921_amd as spin
    if not cfg.q_split_width:
        return None
    subs, _ = spin.decompose(table.prefix_len, table.draft_len, spin.DECOMP_Q_SPLIT, q_width=cfg.q_split_width)
    np.testing.assert_array_equal(subs, orc.decompose_q_split(table.prefix_len, table.draft_len, cfg.q_split_width))
    return subs


@pytest.mark.parametrize("name", si.CONFIG_ORDER)
def test_full_size_configs_every_element(ctx, name):
    """The five benchmark batches exactly as bench.py draws and launches them (same seed, the
    configuration's decomposition made by spin_decompose, automatic wavefront count): EVERY output
    element against the oracle."""
    cfg = si.CONFIGS[name]
    b = si.make_verify_batch(cfg, BENCH_SEED, device="cuda")
    got = hip_attention(ctx, b, subs=product_subs(cfg, b.table))
    want = oracle_attention(b, 0.0)
    assert not np.isnan(want).any()
    err, rms = assert_close(got, want, name)
    print(f"{name}: all {want.size} elements, max abs err {err:.2e}, rel rms {rms:.2e}")


@pytest.mark.parametrize("name,seed", [("7b", 1), ("skewed", 2), ("70b_gqa", 4)])
def test_full_size_configs_other_seeds(ctx, name, seed):
    """Other draws of the benchmark shapes, every element again (the grouped-query batch on a third of its requests)."""
    cfg = si.CONFIGS[name]
    b = si.make_verify_batch(cfg, seed, device="cuda")
    got = hip_attention(ctx, b, subs=product_subs(cfg, b.table))
    reqs = None if name != "70b_gqa" else list(range(0, cfg.n_req, 3))
    assert not torch.isnan(got.float()).any()
    assert_close(got, oracle_attention(b, 0.0, requests=reqs), f"{name} seed {seed}")


def hip_tree_attention(ctx, batch, masks, subs=None, scale=0.0, waves=None):
    t = batch.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    out = torch.full_like(batch.q, float("nan"))
    if waves is not None:
        ctx.set_waves(waves)
    try:
        ctx.verify_attn(tab, batch.k_pool, batch.v_pool, batch.q, out, batch.cfg.n_q_heads, subs=subs,
                        softmax_scale=scale, tree_mask=masks)
        torch.cuda.synchronize()
    finally:
        if waves is not None:
            ctx.set_waves(0)
    return out


def oracle_tree_attention(batch, masks, scale=0.0, requests=None, heads=None):
    t, cfg = batch.table, batch.cfg
    if scale <= 0:
        scale = 1.0 / math.sqrt(cfg.head_dim)
    return orc.verify_attention(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, cfg.page_size,
                                si.host_elems(batch.q), si.host_elems(batch.k_pool), si.host_elems(batch.v_pool),
                                cfg.n_q_heads, cfg.n_kv_heads, scale, requests=requests, heads=heads, tree_mask=masks)


@pytest.mark.parametrize("hq,hkv,d", [(4, 4, 128), (2, 2, 64), (8, 2, 128), (16, 2, 64), (8, 1, 128)])
@pytest.mark.parametrize("shape", ["random", "star", "wide"])
def test_tree_masks(ctx, hq, hkv, d, shape):
    cfg = make_cfg("tree", 7, hq, hkv, d)
    prefix = np.array([0, 1, 15, 16, 333, 1500, 47]); draft = np.array([5, 8, 1, 3, 8, 6, 7])
    if hq // hkv <= 4:
        draft = draft * 2
    b = si.make_verify_batch(cfg, 60, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    _, masks = si.random_trees(draft, np.random.default_rng(61), shape)
    assert_close(hip_tree_attention(ctx, b, masks), oracle_tree_attention(b, masks), f"tree {shape} {hq}/{hkv}/{d}")


def test_chain_tree_is_bitwise_the_linear_draft(ctx):
    for name in ("tiny", "skewed"):
        b = si.make_verify_batch(si.CONFIGS[name], 62, device="cuda")
        _, masks = si.random_trees(b.table.draft_len, None, "chain")
        assert torch.equal(hip_tree_attention(ctx, b, masks).view(torch.int16), hip_attention(ctx, b).view(torch.int16))


@pytest.mark.parametrize("seed", range(4))
def test_tree_masks_decomposed(ctx, seed):
    rng = np.random.default_rng(3000 + seed)
    group = int(rng.choice([1, 2, 4]))
    cfg = make_cfg("tree-dec", 5, 2 * group, 2, int(rng.choice([64, 128])), page=int(rng.choice([4, 16])))
    prefix = rng.integers(0, 900, 5); draft = rng.integers(1, 17, 5)
    b = si.make_verify_batch(cfg, 3100 + seed, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    _, masks = si.random_trees(draft, rng)
    subs = np.array([(i,) + r for i in range(5) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))],
                    dtype=np.int32)
    waves = int(rng.choice([1, 5, 64, 0]))
    assert_close(hip_tree_attention(ctx, b, masks, subs=subs, waves=waves), oracle_tree_attention(b, masks),
                 f"decomposed tree, seed {seed}")


def test_tree_of_64_tokens(ctx):
    cfg = make_cfg("tree64", 3, 2, 2, 128)
    prefix = np.array([100, 0, 1031]); draft = np.array([64, 64, 33])
    b = si.make_verify_batch(cfg, 63, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    _, masks = si.random_trees(draft, np.random.default_rng(64))
    assert_close(hip_tree_attention(ctx, b, masks), oracle_tree_attention(b, masks), "64-token trees")


def test_tree_full_size_every_element(ctx):
    cfg = si.CONFIGS["13b"]
    b = si.make_verify_batch(cfg, BENCH_SEED, device="cuda")
    _, masks = si.random_trees(b.table.draft_len, np.random.default_rng(BENCH_SEED))   # bench.py --tree random
    got = hip_tree_attention(ctx, b, masks)
    want = oracle_tree_attention(b, masks)
    assert not np.isnan(want).any()
    assert_close(got, want, "13b with trees")


def test_tree_mask_errors(ctx):
    import paper_2503_15921_amd as spin
    cfg = make_cfg("tree-err", 2, 2, 2, 64)
    b = si.make_verify_batch(cfg, 66, device="cuda", prefix_len=np.array([4, 9]), draft_len=np.array([3, 2]))
    _, masks = si.random_trees(b.table.draft_len, None, "chain")
    for r, bad in [(1, masks[1] & ~np.uint64(2)),      # the row's own bit is missing
                   (0, masks[0] | np.uint64(4)),       # sees a later draft token
                   (4, masks[4] | np.uint64(1 << 40))]:
        m = masks.copy(); m[r] = bad
        with pytest.raises(spin.SpinError) as ei:
            hip_tree_attention(ctx, b, m)
        assert ei.value.code == spin.ETABLE
    # linear drafts may be longer than 64 tokens, trees may not
    b = si.make_verify_batch(make_cfg("tree-err2", 1, 1, 1, 64), 67, device="cuda", prefix_len=np.array([4]),
                             draft_len=np.array([65]))
    with pytest.raises(spin.SpinError) as ei:
        hip_tree_attention(ctx, b, np.full(65, 1, dtype=np.uint64))
    assert ei.value.code == spin.ETABLE


# ------------------------------------------------------------------------------ fp16 elements
@pytest.mark.parametrize("hq,hkv,d", [(4, 4, 128), (8, 2, 128), (16, 2, 128), (2, 2, 64), (16, 2, 64)])
def test_fp16_attention(ctx, hq, hkv, d):
    """Q, K, V and the output in IEEE half precision: all three kernel widths, whole and cut."""
    cfg = make_cfg("f16", 6, hq, hkv, d)
    prefix = np.array([0, 17, 300, 1500, 64, 2049]); draft = np.array([1, 8, 3, 5, 8, 2])
    b = si.make_verify_batch(cfg, 77, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True,
                             dtype=torch.float16)
    want = oracle_attention(b, 0.0)
    whole = hip_attention(ctx, b)
    assert whole.dtype == torch.float16
    assert_close(whole, want, f"fp16 {hq}/{hkv}/{d}")
    subs = orc.decompose_kv_split(prefix, draft, 100)
    assert_close(hip_attention(ctx, b, subs=subs, waves=7), want, f"fp16 {hq}/{hkv}/{d}, kv-split, 7 shares")
    assert_close(hip_attention(ctx, b, subs=orc.decompose_q_split(prefix, draft, 2)), want, f"fp16 {hq}/{hkv}/{d}, q-split")


def test_fp16_is_closer_than_bf16(ctx):
    """The same draws through both element types, each against the oracle on its own rounded inputs: the
    half-precision path carries three more mantissa bits in P and in the output, so its error is the smaller."""
    cfg = make_cfg("f16-vs-bf16", 4, 8, 2, 128)
    prefix = np.array([100, 700, 1500, 33]); draft = np.array([4, 8, 2, 6])
    b = si.make_verify_batch(cfg, 78, device="cuda", prefix_len=prefix, draft_len=draft)
    h = si.make_verify_batch(cfg, 78, device="cuda", prefix_len=prefix, draft_len=draft, dtype=torch.float16)
    _, rms_b = assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), "bf16")
    _, rms_h = assert_close(hip_attention(ctx, h), oracle_attention(h, 0.0), "fp16")
    assert rms_h < 0.5 * rms_b, (rms_h, rms_b)


@pytest.mark.parametrize("hq,hkv,d", [(4, 2, 128), (16, 2, 64)])
def test_fp16_tree_and_append(ctx, hq, hkv, d):
    cfg = make_cfg("f16-tree", 5, hq, hkv, d)
    prefix = np.array([0, 15, 333, 1500, 47]); draft = np.array([5, 8, 1, 8, 7])
    b = si.make_verify_batch(cfg, 79, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True,
                             dtype=torch.float16)
    g = torch.Generator(device="cpu").manual_seed(80)
    shape = (b.table.n_rows, hkv, d)
    k_new = torch.randn(shape, generator=g).to(torch.float16).cuda()
    v_new = torch.randn(shape, generator=g).to(torch.float16).cuda()
    t = b.table
    want_k, want_v = si.host_elems(b.k_pool).copy(), si.host_elems(b.v_pool).copy()
    orc.append_kv(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, cfg.page_size, want_k, want_v,
                  si.host_elems(k_new), si.host_elems(v_new))
    _, masks = si.random_trees(draft, np.random.default_rng(81), "random")
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    out = torch.full_like(b.q, float("nan"))
    ctx.append_kv(tab, b.k_pool, b.v_pool, k_new, v_new)
    ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, hq, tree_mask=masks)
    torch.cuda.synchronize()
    assert np.array_equal(si.host_elems(b.k_pool).view(np.uint16), want_k.view(np.uint16))
    assert np.array_equal(si.host_elems(b.v_pool).view(np.uint16), want_v.view(np.uint16))
    want = orc.verify_attention(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, cfg.page_size,
                                si.host_elems(b.q), want_k, want_v, hq, hkv, 1.0 / math.sqrt(d), tree_mask=masks)
    assert_close(out, want, "fp16 append + tree attention")


def test_fp16_full_size_every_element(ctx):
    cfg = si.CONFIGS["13b"]
    b = si.make_verify_batch(cfg, BENCH_SEED, device="cuda", dtype=torch.float16)
    got = hip_attention(ctx, b)
    want = oracle_attention(b, 0.0)
    assert not np.isnan(want).any()
    assert_close(got, want, "13b fp16")


def test_mixed_element_types_are_refused(ctx):
    cfg = make_cfg("mixed", 2, 2, 2, 64)
    b = si.make_verify_batch(cfg, 82, device="cuda", prefix_len=np.array([5, 40]), draft_len=np.array([2, 3]))
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    with pytest.raises(AssertionError):
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q.to(torch.float16), torch.empty_like(b.q), 2)
    with pytest.raises(TypeError):
        ctx.verify_attn(tab, b.k_pool.float(), b.v_pool.float(), b.q.float(), torch.empty_like(b.q).float(), 2)


# ------------------------------------------------------------------------------ KV append
def oracle_append(b, k_new, v_new):
    t = b.table
    kp = si.bf16_bits(b.k_pool).copy(); vp = si.bf16_bits(b.v_pool).copy()
    orc.append_kv(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, b.cfg.page_size, kp, vp,
                  si.bf16_bits(k_new), si.bf16_bits(v_new))
    return kp, vp


def new_rows(b, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    shape = (b.table.n_rows, b.cfg.n_kv_heads, b.cfg.head_dim)
    return (torch.randn(shape, generator=g).to(torch.bfloat16).cuda(),
            torch.randn(shape, generator=g).to(torch.bfloat16).cuda())


@pytest.mark.parametrize("name,seed,page", [("tiny", 0, 16), ("tiny", 1, 4), ("skewed", 2, 16), ("70b_gqa", 3, 16),
                                            ("tiny", 4, 1), ("tiny", 5, 64)])
def test_append_kv_bit_exact(ctx, name, seed, page):
    cfg = si.CONFIGS[name]
    if page != cfg.page_size:
        cfg = dataclasses.replace(cfg, name=f"{name}-p{page}", page_size=page)
    b = si.make_verify_batch(cfg, seed, device="cuda", poison_unused=True)
    k_new, v_new = new_rows(b, 100 + seed)
    want_k, want_v = oracle_append(b, k_new, v_new)
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    ctx.append_kv(tab, b.k_pool, b.v_pool, k_new, v_new)
    torch.cuda.synchronize()
    assert np.array_equal(si.bf16_bits(b.k_pool), want_k)      # the whole pool: nothing else was touched
    assert np.array_equal(si.bf16_bits(b.v_pool), want_v)


@pytest.mark.parametrize("n_req", [61, 130, 300])
def test_append_kv_many_rows(ctx, n_req):
    # 16 draft rows per request: 976, 2080 and 4800 rows -- two and three launches with the destination slots in the
    # kernel arguments, and (beyond 3840 rows) the kernel that reads them from the staging buffer
    cfg = make_cfg(f"append-rows-{n_req}", n_req, 2, 2, 64)
    rng = np.random.default_rng(n_req)
    b = si.make_verify_batch(cfg, 43, device="cuda", prefix_len=rng.integers(0, 70, n_req), draft_len=np.full(n_req, 16),
                             poison_unused=True)
    k_new, v_new = new_rows(b, 143)
    want_k, want_v = oracle_append(b, k_new, v_new)
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    ctx.append_kv(tab, b.k_pool, b.v_pool, k_new, v_new)
    torch.cuda.synchronize()
    assert np.array_equal(si.bf16_bits(b.k_pool), want_k) and np.array_equal(si.bf16_bits(b.v_pool), want_v)


def test_append_then_verify_on_one_stream(ctx):
    """Append and attention queued back to back with no synchronisation in between."""
    cfg = make_cfg("append-verify", 6, 8, 2, 128)
    prefix = np.array([0, 15, 16, 700, 2049, 31]); draft = np.array([4, 1, 16, 7, 3, 2])
    b = si.make_verify_batch(cfg, 41, device="cuda", prefix_len=prefix, draft_len=draft, poison_unused=True)
    k_new, v_new = new_rows(b, 141)
    want_k, want_v = oracle_append(b, k_new, v_new)
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    out = torch.full_like(b.q, float("nan"))
    ctx.append_kv(tab, b.k_pool, b.v_pool, k_new, v_new)
    ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads)
    torch.cuda.synchronize()
    want = orc.verify_attention(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, cfg.page_size,
                                si.bf16_bits(b.q), want_k, want_v, cfg.n_q_heads, cfg.n_kv_heads,
                                1.0 / math.sqrt(cfg.head_dim))
    assert_close(out, want, "append then verify")


def test_append_into_strided_cache(ctx):
    cfg = make_cfg("append-layout", 3, 4, 2, 64)
    prefix = np.array([40, 5, 333]); draft = np.array([5, 8, 3])
    b = si.make_verify_batch(cfg, 42, device="cuda", prefix_len=prefix, draft_len=draft)
    k_new, v_new = new_rows(b, 142)
    want_k, want_v = oracle_append(b, k_new, v_new)
    n_pages, hkv, P, d = b.k_pool.shape
    pitch = d + 24
    k_alt = torch.zeros((n_pages, P, hkv, pitch), dtype=torch.bfloat16, device="cuda")
    v_alt = torch.zeros_like(k_alt)
    k_alt[..., :d] = b.k_pool.permute(0, 2, 1, 3); v_alt[..., :d] = b.v_pool.permute(0, 2, 1, 3)
    kv = k_alt.permute(0, 2, 1, 3)[..., :d]; vv = v_alt.permute(0, 2, 1, 3)[..., :d]
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    ctx.append_kv(tab, kv, vv, k_new, v_new)
    torch.cuda.synchronize()
    assert np.array_equal(si.bf16_bits(kv.contiguous()), want_k) and np.array_equal(si.bf16_bits(vv.contiguous()), want_v)
    assert (k_alt[..., d:] == 0).all() and (v_alt[..., d:] == 0).all()     # the padding stays untouched


# ------------------------------------------------------------------------------ acceptance
def hip_accept(ctx, mode, ab):
    B = len(ab.draft_len)
    n_acc = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    nxt = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    ctx.accept(mode, ab.draft_len, ab.draft_tokens, ab.target_logits, ab.draft_logits, ab.u_accept, ab.u_sample,
               n_acc, nxt)
    torch.cuda.synchronize()
    return n_acc.cpu().numpy(), nxt.cpu().numpy()


def oracle_accept(mode, ab):
    import paper_2503_15921_amd as spin
    tl = ab.target_logits.cpu().numpy(); toks = ab.draft_tokens.cpu().numpy()
    if mode == spin.ACCEPT_GREEDY:
        return orc.accept_greedy(ab.draft_len, toks, tl)
    return orc.accept_rejection(ab.draft_len, toks, tl, ab.draft_logits.cpu().numpy(),
                                ab.u_accept.cpu().numpy(), ab.u_sample.cpu().numpy())


def check_accept(ctx, mode, ab, what):
    n_g, t_g = hip_accept(ctx, mode, ab)
    n_o, t_o, margin = oracle_accept(mode, ab)
    # every decision must be far from its threshold compared with float64 rounding, otherwise
    # two correct float64 evaluations could legitimately disagree (re-seed if this ever fires)
    assert margin.min() > 1e-9, f"{what}: decision margin {margin.min():.2e} too small to compare bit for bit"
    np.testing.assert_array_equal(n_g, n_o, err_msg=what)
    np.testing.assert_array_equal(t_g, t_o, err_msg=what)
    return n_o


@pytest.mark.parametrize("seed", [0, 1, 2])
@pytest.mark.parametrize("rho", [None, 0.9])
def test_accept_tiny(ctx, seed, rho):
    import paper_2503_15921_amd as spin
    cfg = si.CONFIGS["tiny"]
    draft_len = si.draw_lengths(cfg, np.random.default_rng(seed))[1]
    ab = si.make_accept_batch(draft_len, cfg.vocab, cfg.logit_sigma, seed, device="cuda", rho=rho)
    check_accept(ctx, spin.ACCEPT_REJECTION, ab, f"tiny rejection seed {seed} rho {rho}")
    ab = si.make_accept_batch(draft_len, cfg.vocab, cfg.logit_sigma, seed, device="cuda", rho=rho,
                              draft_token_mode="argmax")
    check_accept(ctx, spin.ACCEPT_GREEDY, ab, f"tiny greedy seed {seed} rho {rho}")


@pytest.mark.parametrize("name,seed", [(n, BENCH_SEED) for n in si.CONFIG_ORDER] + [("7b", 1), ("skewed", 2), ("70b_gqa", 4)])
def test_accept_full_vocab(ctx, name, seed):
    """Acceptance over the benchmark batches (BENCH_SEED, rho None is exactly what bench.py times) and other
    draws: every request's accepted length and next token against the oracle, bit for bit."""
    import paper_2503_15921_amd as spin
    cfg = si.CONFIGS[name]
    draft_len = si.draw_lengths(cfg, np.random.default_rng(seed))[1]
    seen = set()
    for rho in (None, 0.97):
        ab = si.make_accept_batch(draft_len, cfg.vocab, cfg.logit_sigma, seed, device="cuda", rho=rho)
        n = check_accept(ctx, spin.ACCEPT_REJECTION, ab, f"{name} rejection rho {rho}")
        seen |= set(n.tolist())
        ab = si.make_accept_batch(draft_len, cfg.vocab, cfg.logit_sigma, seed, device="cuda", rho=rho,
                                  draft_token_mode="argmax")
        n = check_accept(ctx, spin.ACCEPT_GREEDY, ab, f"{name} greedy rho {rho}")
        seen |= set(n.tolist())
    assert len(seen) >= 3, "the correlated draw should spread accepted lengths"


@pytest.mark.parametrize("n_req", [150, 260, 330, 450, 700, 1400])
def test_accept_many_requests(ctx, n_req):
    """Batches of many requests: the next-token draw cuts the vocabulary into fewer parts per request the more
    requests there are (8 down to 1), so that every workgroup of its launch stays resident."""
    import paper_2503_15921_amd as spin
    rng = np.random.default_rng(n_req)
    draft_len = rng.integers(1, 4, n_req).astype(np.int32)
    for rho in (None, 0.9):
        ab = si.make_accept_batch(draft_len, 9001, 3.0, n_req, device="cuda", rho=rho)
        check_accept(ctx, spin.ACCEPT_REJECTION, ab, f"{n_req} requests rho {rho}")


def test_accept_many_random_small_batches(ctx):
    """150 random small problems (vocabularies 2-700, drafts 1-9, correlation anywhere from none to near
    identity, both modes).  A case whose decisions sit within 1e-9 of a threshold is skipped, not failed."""
    import paper_2503_15921_amd as spin
    rng = np.random.default_rng(4242)
    compared = 0
    for case in range(150):
        n_req = int(rng.integers(1, 7))
        draft_len = rng.integers(1, 10, n_req).astype(np.int32)
        vocab = int(rng.choice([2, 3, 5, 17, 64, 255, 256, 257, 700]))
        rho = None if rng.random() < 0.2 else float(rng.choice([0.5, 0.9, 0.99, 0.9999]))
        sigma = float(rng.choice([0.5, 2.0, 6.0]))
        greedy = rng.random() < 0.3
        ab = si.make_accept_batch(draft_len, vocab, sigma, 5000 + case, device="cuda", rho=rho,
                                  draft_token_mode="argmax" if greedy else "sample")
        mode = spin.ACCEPT_GREEDY if greedy else spin.ACCEPT_REJECTION
        n_o, t_o, margin = oracle_accept(mode, ab)
        if margin.min() <= 1e-9:
            continue
        n_g, t_g = hip_accept(ctx, mode, ab)
        what = f"case {case}: vocab {vocab} drafts {draft_len.tolist()} rho {rho} sigma {sigma} greedy {greedy}"
        np.testing.assert_array_equal(n_g, n_o, err_msg=what)
        np.testing.assert_array_equal(t_g, t_o, err_msg=what)
        compared += 1
    assert compared >= 120


def test_accept_planted_lengths(ctx):
    import paper_2503_15921_amd as spin
    draft_len = np.array([1, 2, 3, 4, 5, 5, 5, 5, 5, 5, 16, 16], dtype=np.int32)
    want = np.array([0, 2, 1, 4, 0, 1, 2, 3, 4, 5, 16, 9])
    ab = si.make_accept_batch(draft_len, 4099, 2.0, 3, device="cuda")     # odd vocab: scalar load path
    tops = ab.target_logits.argmax(dim=-1).cpu().numpy()
    toks = np.zeros(int(draft_len.sum()), dtype=np.int32)
    r = 0
    for i, g in enumerate(draft_len):
        for t in range(g):
            good = tops[r + i + t]
            toks[r + t] = good if t < want[i] else (good + 1) % 4099
        r += g
    ab.draft_tokens = torch.from_numpy(toks).cuda()
    n_g, t_g = hip_accept(ctx, spin.ACCEPT_GREEDY, ab)
    np.testing.assert_array_equal(n_g, want)
    n_o, t_o, _ = oracle_accept(spin.ACCEPT_GREEDY, ab)
    np.testing.assert_array_equal(t_g, t_o)
    # identical models: everything is kept, next token from the bonus row
    keep = np.ones(len(tops), dtype=bool)
    keep[np.cumsum(draft_len) + np.arange(len(draft_len))] = False
    ab.draft_logits = ab.target_logits[torch.from_numpy(np.nonzero(keep)[0]).cuda()].clone()
    n = check_accept(ctx, spin.ACCEPT_REJECTION, ab, "p == q")
    np.testing.assert_array_equal(n, draft_len)
    # u = 0 keeps every token the target gives any mass
    ab2 = si.make_accept_batch(draft_len, 4099, 2.0, 4, device="cuda")
    ab2.u_accept.zero_()
    n_g, _ = hip_accept(ctx, spin.ACCEPT_REJECTION, ab2)
    np.testing.assert_array_equal(n_g, draft_len)


@pytest.mark.parametrize("vocab", [1, 2, 7, 257, 4099, 70001])
def test_accept_odd_vocabularies_and_long_drafts(ctx, vocab):
    # scalar-load paths (vocab not a multiple of 4), tiny vocabularies, more than 64 draft rows per request
    import paper_2503_15921_amd as spin
    draft_len = np.array([1, 70, 3, 130, 2], dtype=np.int32)
    for rho in (None, 0.98):
        ab = si.make_accept_batch(draft_len, vocab, 1.5, 7 + vocab, device="cuda", rho=rho)
        check_accept(ctx, spin.ACCEPT_REJECTION, ab, f"vocab {vocab} rho {rho}")
        ab = si.make_accept_batch(draft_len, vocab, 1.5, 7 + vocab, device="cuda", rho=rho, draft_token_mode="argmax")
        check_accept(ctx, spin.ACCEPT_GREEDY, ab, f"vocab {vocab} greedy rho {rho}")


@pytest.mark.parametrize("vocab", [128256, 1048576])
def test_accept_large_vocabularies(ctx, vocab):
    # a current 128k-id vocabulary and the largest one the library takes
    import paper_2503_15921_amd as spin
    draft_len = np.array([2, 4, 1], dtype=np.int32)
    for rho in (None, 0.98):
        ab = si.make_accept_batch(draft_len, vocab, 2.0, 31, device="cuda", rho=rho)
        check_accept(ctx, spin.ACCEPT_REJECTION, ab, f"vocab {vocab} rho {rho}")
    ab = si.make_accept_batch(draft_len, vocab, 2.0, 32, device="cuda", rho=0.98, draft_token_mode="argmax")
    check_accept(ctx, spin.ACCEPT_GREEDY, ab, f"vocab {vocab} greedy")


def test_accept_vocabulary_beyond_the_limit_is_refused(ctx):
    import paper_2503_15921_amd as spin
    draft_len = np.array([1], dtype=np.int32)
    ab = si.make_accept_batch(draft_len, (1 << 20) + 1, 2.0, 33, device="cuda")
    with pytest.raises(spin.SpinError) as ei:
        hip_accept(ctx, spin.ACCEPT_REJECTION, ab)
    assert ei.value.code == spin.EUNSUPPORTED


def test_accept_extreme_uniforms(ctx):
    # u' = 0 picks the first id with mass; u' just below 1 picks (one of) the last; u = 0 keeps, u near 1 rejects
    import paper_2503_15921_amd as spin
    draft_len = np.array([4, 4, 4, 4], dtype=np.int32)
    ab = si.make_accept_batch(draft_len, 5000, 2.0, 11, device="cuda", rho=0.9)
    ab.u_sample[:] = torch.tensor([0.0, 1.0 - 2 ** -53, 0.5, 0.25], dtype=torch.float64)
    ab.u_accept[:] = torch.tensor([0.0, 0.0, 0.0, 0.0, 0.0, 1 - 2 ** -53, 0.0, 0.0] * 2, dtype=torch.float64)
    n_g, t_g = hip_accept(ctx, spin.ACCEPT_REJECTION, ab)
    n_o, t_o, margin = oracle_accept(spin.ACCEPT_REJECTION, ab)
    np.testing.assert_array_equal(n_g, n_o)
    # request 1's draw sits at the very end of the CDF, where the two summation orders may pick different
    # ids among the last few with mass: compare the others bit for bit, and request 1 for validity --
    # the id must carry mass, and the mass after it must be no more than rounding of the total
    keep = np.array([0, 2, 3])
    np.testing.assert_array_equal(t_g[keep], t_o[keep])
    n = int(n_o[1])
    tl = ab.target_logits.cpu().numpy().astype(np.float64)
    dl = ab.draft_logits.cpu().numpy().astype(np.float64)

    def softmax(x):
        e = np.exp(x - x.max())
        return e / e.sum()
    p = softmax(tl[4 + 1 + n])                       # request 1 owns target rows 5..9, draft rows 4..7
    mass = np.maximum(p - softmax(dl[4 + n]), 0.0) if n < 4 else p
    k = int(t_g[1])
    assert 0 <= k < 5000 and mass[k] > 0, "the id drawn at the end of the CDF has no mass"
    assert mass[k + 1:].sum() <= 1e-12 * mass.sum(), "the id drawn with u' = 1 - 2^-53 is not at the end of the CDF"
    assert mass[int(t_o[1]) + 1:].sum() <= 1e-12 * mass.sum()


@pytest.mark.parametrize("vocab", [6000, 5001])
def test_accept_rows_with_a_wide_logit_range(ctx, vocab):
    """Rows whose leading ids are far below (or minus infinity against) the rest: the row-sum kernel's
    reference taken from the row's first elements is useless there and it has to sweep the row twice."""
    import paper_2503_15921_amd as spin
    draft_len = np.array([3, 5, 2, 4, 1, 6], dtype=np.int32)
    ab = si.make_accept_batch(draft_len, vocab, 2.0, 21, device="cuda", rho=0.9)
    R = int(draft_len.sum())
    ab.target_logits[0:4, :1500] -= 1000.0          # first ids 1000 below the rest: beyond the one-sweep range
    ab.draft_logits[0:3, :1500] -= 1000.0
    ab.target_logits[5:9, :1100] = float("-inf")    # first ids excluded outright
    ab.draft_logits[4:7, :1100] = float("-inf")
    ab.target_logits[10:12, :1024] -= 400.0         # inside the range: still one sweep
    ab.target_logits[12:14, 2000:] -= 2000.0        # the tail far below the head
    ab.draft_logits[R - 3:, :1024] -= 300.0
    # draft tokens must come from ids the (modified) draft rows still give mass to
    ab.draft_tokens[:] = torch.clamp(ab.draft_tokens, min=1600, max=1999)
    check_accept(ctx, spin.ACCEPT_REJECTION, ab, f"wide logit range, vocab {vocab}")


def test_accept_token_outside_vocabulary_is_rejected(ctx):
    import paper_2503_15921_amd as spin
    draft_len = np.array([3, 2], dtype=np.int32)
    ab = si.make_accept_batch(draft_len, 1000, 2.0, 5, device="cuda", rho=0.99)
    ab.u_accept.zero_()
    ab.draft_tokens[1] = 1000
    ab.draft_tokens[3] = -1
    n_g, t_g = hip_accept(ctx, spin.ACCEPT_REJECTION, ab)
    np.testing.assert_array_equal(n_g, [1, 0])
    assert ((0 <= t_g) & (t_g < 1000)).all()


# ------------------------------------------------------------------------------ greedy tree acceptance
def hip_accept_tree(ctx, draft_len, parents, tokens, logits, draft_logits=None, u_accept=None, u_sample=None):
    import paper_2503_15921_amd as spin
    B, R = len(draft_len), int(np.sum(draft_len))
    n_acc = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    nxt = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    path = torch.full((R,), -7, dtype=torch.int32, device="cuda")
    mode = spin.ACCEPT_GREEDY if draft_logits is None else spin.ACCEPT_REJECTION
    ctx.accept_tree(mode, draft_len, parents, tokens, logits, draft_logits, u_accept, u_sample, n_acc, path, nxt)
    torch.cuda.synchronize()
    return n_acc.cpu().numpy(), path.cpu().numpy(), nxt.cpu().numpy()


@pytest.mark.parametrize("vocab", [3, 8, 1000, 32000])
@pytest.mark.parametrize("shape", ["random", "wide", "star", "chain"])
def test_accept_tree_greedy(ctx, vocab, shape):
    rng = np.random.default_rng(vocab + len(shape))
    draft_len = np.array([64, 1, 7, 30, 2, 12], dtype=np.int32)
    parents, _ = si.random_trees(draft_len, rng, shape)
    R, B = int(draft_len.sum()), len(draft_len)
    g = torch.Generator(device="cuda").manual_seed(vocab)
    logits = torch.randn((R + B, vocab), generator=g, device="cuda") * 2.0
    # tokens: a mix of the parent's arg-max (so that walks go deep) and random ids
    top = logits.argmax(dim=-1).cpu().numpy()
    tokens = rng.integers(0, vocab, R).astype(np.int32)
    r = 0
    for i, gl in enumerate(draft_len):
        for t in range(gl):
            if rng.random() < 0.6:
                tokens[r + t] = top[r + i + parents[r + t] + 1]
        r += gl
    tok_dev = torch.from_numpy(tokens).cuda()
    n_o, path_o, nxt_o, margin = orc.accept_tree_greedy(draft_len, parents, tokens, logits.cpu().numpy())
    assert margin.min() > 0
    n_g, path_g, nxt_g = hip_accept_tree(ctx, draft_len, parents, tok_dev, logits)
    np.testing.assert_array_equal(n_g, n_o)
    np.testing.assert_array_equal(path_g, path_o)
    np.testing.assert_array_equal(nxt_g, nxt_o)
    if vocab >= 8 and shape != "star":              # (a star is one level deep)
        assert n_o.max() >= 2
    if shape == "chain":        # the layout and the result of the linear greedy acceptance
        ab_n = torch.full((B,), -7, dtype=torch.int32, device="cuda"); ab_t = torch.full_like(ab_n, -7)
        import paper_2503_15921_amd as spin
        ctx.accept(spin.ACCEPT_GREEDY, draft_len, tok_dev, logits, None, None, None, ab_n, ab_t)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(ab_n.cpu().numpy(), n_o)
        np.testing.assert_array_equal(ab_t.cpu().numpy(), nxt_o)


@pytest.mark.parametrize("vocab", [3, 37, 1000, 32000])
@pytest.mark.parametrize("shape", ["random", "wide", "star", "chain"])
def test_accept_tree_rejection(ctx, vocab, shape):
    import paper_2503_15921_amd as spin
    rng = np.random.default_rng(10 * vocab + len(shape))
    draft_len = np.array([64, 1, 7, 30, 2, 12] if vocab <= 1000 else [20, 1, 7, 9], dtype=np.int32)
    parents, _ = si.random_trees(draft_len, rng, shape)
    R, B = int(draft_len.sum()), len(draft_len)
    # target rows; every draft token is drawn from a draft row correlated with its parent's target row
    tl = rng.normal(0, 2, (R + B, vocab)).astype(np.float32)
    dl = np.empty((R, vocab), dtype=np.float32)
    tokens = np.empty(R, dtype=np.int32)
    r = 0
    for i, g in enumerate(draft_len):
        for t in range(g):
            prow = tl[r + i + parents[r + t] + 1]
            dl[r + t] = 0.95 * prow + 0.31 * rng.normal(0, 2, vocab)
            tokens[r + t] = rng.choice(vocab, p=orc._softmax64(dl[r + t]))
        r += g
    ua, us = rng.random(R), rng.random(B)
    n_o, path_o, nxt_o, margin = orc.accept_tree_rejection(draft_len, parents, tokens, tl, dl, ua, us)
    assert margin.min() > 1e-9, f"decision margin {margin.min():.2e} too small to compare bit for bit"
    dev = lambda a: torch.from_numpy(a).cuda()
    n_g, path_g, nxt_g = hip_accept_tree(ctx, draft_len, parents, dev(tokens), dev(tl), dev(dl), dev(ua), dev(us))
    np.testing.assert_array_equal(n_g, n_o)
    np.testing.assert_array_equal(path_g, path_o)
    np.testing.assert_array_equal(nxt_g, nxt_o)
    if shape != "star":
        assert n_o.max() >= 2
    if shape == "chain":        # the linear rule gives the same
        n_l = torch.full((B,), -7, dtype=torch.int32, device="cuda"); t_l = torch.full_like(n_l, -7)
        ctx.accept(spin.ACCEPT_REJECTION, draft_len, dev(tokens), dev(tl), dev(dl), dev(ua), dev(us), n_l, t_l)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(n_l.cpu().numpy(), n_o)
        np.testing.assert_array_equal(t_l.cpu().numpy(), nxt_o)


def wide_accept_case(ctx, seed):
    """One random acceptance case: vocabulary sizes around the kernels' step sizes, linear drafts or trees of any
    shape, greedy or rejection sampling, narrow to wide logits.  Returns False when the oracle's decision margin
    is too small to compare bit for bit."""
    import paper_2503_15921_amd as spin
    rng = np.random.default_rng(90000 + seed)
    vocab = int(rng.choice([1, 2, 3, 5, 17, 64, 255, 256, 257, 1000, 4095, 4096, 4097, 8191, 32000, 50257]))
    B = int(rng.integers(1, 10))
    tree = rng.random() < 0.5
    max_g = 10 if vocab > 8000 else (64 if tree else 40)
    draft_len = rng.integers(1, max_g + 1, B).astype(np.int32)
    R = int(draft_len.sum())
    sigma = float(rng.choice([0.5, 2.0, 6.0]))
    greedy = rng.random() < 0.4
    what = f"seed {seed}: vocab {vocab} B {B} R {R} tree {tree} greedy {greedy} sigma {sigma}"
    dev = lambda a: torch.from_numpy(a).cuda()
    if not tree:
        rho = None if rng.random() < 0.3 else float(rng.choice([0.5, 0.9, 0.99]))
        ab = si.make_accept_batch(draft_len, vocab, sigma, 91000 + seed, device="cuda", rho=rho,
                                  draft_token_mode="argmax" if greedy else "sample")
        mode = spin.ACCEPT_GREEDY if greedy else spin.ACCEPT_REJECTION
        n_g, t_g = hip_accept(ctx, mode, ab)
        n_o, t_o, margin = oracle_accept(mode, ab)
        if margin.min() <= 1e-9:
            return False
        np.testing.assert_array_equal(n_g, n_o, err_msg=what)
        np.testing.assert_array_equal(t_g, t_o, err_msg=what)
        return True
    parents, _ = si.random_trees(draft_len, rng, str(rng.choice(["random", "wide", "star", "chain"])))
    tl = rng.normal(0, sigma, (R + B, vocab)).astype(np.float32)
    dl = np.empty((R, vocab), dtype=np.float32)
    tokens = np.empty(R, dtype=np.int32)
    r = 0
    for i, g in enumerate(draft_len):
        for t in range(g):
            prow = tl[r + i + parents[r + t] + 1]
            dl[r + t] = 0.95 * prow + 0.31 * rng.normal(0, sigma, vocab)
            if greedy:
                tokens[r + t] = int(np.argmax(prow)) if rng.random() < 0.6 else int(rng.integers(vocab))
            else:
                tokens[r + t] = rng.choice(vocab, p=orc._softmax64(dl[r + t]))
        r += g
    if greedy:
        n_o, path_o, nxt_o, margin = orc.accept_tree_greedy(draft_len, parents, tokens, tl)
        n_g, path_g, nxt_g = hip_accept_tree(ctx, draft_len, parents, dev(tokens), dev(tl))
    else:
        ua, us = rng.random(R), rng.random(B)
        n_o, path_o, nxt_o, margin = orc.accept_tree_rejection(draft_len, parents, tokens, tl, dl, ua, us)
        n_g, path_g, nxt_g = hip_accept_tree(ctx, draft_len, parents, dev(tokens), dev(tl), dev(dl), dev(ua), dev(us))
    if np.min(margin) <= 1e-9:
        return False
    np.testing.assert_array_equal(n_g, n_o, err_msg=what)
    np.testing.assert_array_equal(path_g, path_o, err_msg=what)
    np.testing.assert_array_equal(nxt_g, nxt_o, err_msg=what)
    return True


def test_accept_over_all_axes(ctx):
    """100 cases by default; SPIN_SWEEP_CASES=n runs the first n seeds (12000 have passed with the kernels as they stand)."""
    n = int(os.environ.get("SPIN_SWEEP_CASES", "100"))
    compared = 0
    for seed in range(n):
        compared += wide_accept_case(ctx, seed)
        if seed % 500 == 499:
            print(f"{seed + 1} cases", flush=True)
    assert compared >= 0.95 * n


def test_accept_tree_rejection_many_rejected_siblings(ctx):
    # a node with many children that are all turned down (uniforms at 1 - eps): the residual is taken apart
    # child by child; some children carry invalid token ids, two carry the same distribution as the target
    rng = np.random.default_rng(77)
    vocab = 200
    draft_len = np.array([24, 10], dtype=np.int32)
    parents = np.concatenate([np.full(24, -1), np.array([-1, 0, 0, 0, 0, 0, 0, 0, 0, 0])]).astype(np.int32)
    R, B = 34, 2
    tl = rng.normal(0, 2, (R + B, vocab)).astype(np.float32)
    dl = rng.normal(0, 2, (R, vocab)).astype(np.float32)
    dl[3] = tl[0]; dl[9] = tl[0]
    # every child carries the token its parent's target row likes least, so that u = 1 - eps turns it down
    tokens = np.empty(R, dtype=np.int32)
    tokens[:24] = int(np.argmin(tl[0]))
    tokens[24] = int(np.argmax(tl[24 + 1]))
    tokens[25:] = int(np.argmin(tl[24 + 1 + 1]))
    dl[24, tokens[24]] -= 5.0                            # (and the accepted one is under-proposed: p/q > 1)
    tokens[5] = vocab + 4; tokens[11] = -3
    ua = np.full(R, 1.0 - 1e-12); ua[24] = 0.0          # second request: its first token is accepted, its nine children are not
    us = rng.random(B)
    n_o, path_o, nxt_o, margin = orc.accept_tree_rejection(draft_len, parents, tokens, tl, dl, ua, us)
    assert n_o.tolist() == [0, 1]
    dev = lambda a: torch.from_numpy(a).cuda()
    n_g, path_g, nxt_g = hip_accept_tree(ctx, draft_len, parents, dev(tokens), dev(tl), dev(dl), dev(ua), dev(us))
    np.testing.assert_array_equal(n_g, n_o)
    np.testing.assert_array_equal(path_g, path_o)
    np.testing.assert_array_equal(nxt_g, nxt_o)


def test_accept_tree_errors(ctx):
    import paper_2503_15921_amd as spin
    draft_len = np.array([3, 2], dtype=np.int32)
    logits = torch.randn((7, 16), device="cuda")
    tokens = torch.zeros(5, dtype=torch.int32, device="cuda")
    for bad in ([-1, 0, 2, -1, 0], [-1, 0, 1, 0, 0], [-2, 0, 1, -1, 0]):      # own index, first token with a parent, below -1
        with pytest.raises(spin.SpinError) as ei:
            hip_accept_tree(ctx, draft_len, np.array(bad, dtype=np.int32), tokens, logits)
        assert ei.value.code == spin.ETABLE
    with pytest.raises(spin.SpinError) as ei:
        hip_accept_tree(ctx, np.array([65], dtype=np.int32), np.full(65, -1, dtype=np.int32),
                        torch.zeros(65, dtype=torch.int32, device="cuda"), torch.randn((66, 16), device="cuda"))
    assert ei.value.code == spin.ETABLE


# ------------------------------------------------------------------------------ all calls in sequence
@pytest.mark.parametrize("hq,hkv,page", [(4, 4, 16), (8, 2, 4)])
def test_decode_loop_append_verify_accept(ctx, hq, hkv, page):
    """Eight speculative steps of a small batch, every call on the GPU shadowed by the oracle: the drafts'
    K/V are appended, verified and accepted; the prefixes grow by the accepted lengths, so rejected slots are
    overwritten by the next step's drafts and the tables differ from step to step."""
    import paper_2503_15921_amd as spin
    rng = np.random.default_rng(1234 + hq)
    B, d, vocab, steps, max_draft = 5, 64, 300, 8, 5
    prefix = rng.integers(0, 40, B).astype(np.int32)
    # pages for the longest any request can get; the cache starts with random prefixes
    table0 = si.make_table(prefix + steps * max_draft, np.ones(B, dtype=np.int32), page, rng)
    cfg = make_cfg("loop", B, hq, hkv, d, page=page)
    g = torch.Generator(device="cpu").manual_seed(99)
    k_pool = torch.randn((table0.n_pages, hkv, page, d), generator=g).to(torch.bfloat16).cuda()
    v_pool = torch.randn((table0.n_pages, hkv, page, d), generator=g).to(torch.bfloat16).cuda()
    k_ref, v_ref = si.bf16_bits(k_pool).copy(), si.bf16_bits(v_pool).copy()
    dev = lambda a: torch.from_numpy(a).cuda()
    scale = 1.0 / math.sqrt(d)
    for step in range(steps):
        draft = rng.integers(1, max_draft + 1, B).astype(np.int32)
        q_off = np.concatenate([[0], np.cumsum(draft)]).astype(np.int32)
        R = int(q_off[-1])
        tab = ctx.make_table(prefix, draft, q_off, table0.pt_offset, table0.page_table)
        # 1. the drafts' K/V enter the cache
        k_new = torch.randn((R, hkv, d), generator=g).to(torch.bfloat16).cuda()
        v_new = torch.randn((R, hkv, d), generator=g).to(torch.bfloat16).cuda()
        ctx.append_kv(tab, k_pool, v_pool, k_new, v_new)
        orc.append_kv(prefix, draft, q_off, table0.pt_offset, table0.page_table, page, k_ref, v_ref,
                      si.bf16_bits(k_new), si.bf16_bits(v_new))
        # 2. attention of the draft rows (same stream, no synchronisation in between)
        q = torch.randn((R, hq, d), generator=g).to(torch.bfloat16).cuda()
        out = torch.full_like(q, float("nan"))
        ctx.verify_attn(tab, k_pool, v_pool, q, out, hq)
        # 3. acceptance
        tl = rng.normal(0, 2, (R + B, vocab)).astype(np.float32)
        own = np.delete(tl, q_off[1:] + np.arange(B), axis=0)
        dl = (0.9 * own + 0.44 * rng.normal(0, 2, (R, vocab))).astype(np.float32)
        tok = np.array([rng.choice(vocab, p=orc._softmax64(dl[r])) for r in range(R)], dtype=np.int32)
        ua, us = rng.random(R), rng.random(B)
        n_acc = torch.full((B,), -7, dtype=torch.int32, device="cuda"); nxt = torch.full_like(n_acc, -7)
        ctx.accept(spin.ACCEPT_REJECTION, draft, dev(tok), dev(tl), dev(dl), dev(ua), dev(us), n_acc, nxt)
        torch.cuda.synchronize()
        assert np.array_equal(si.bf16_bits(k_pool), k_ref) and np.array_equal(si.bf16_bits(v_pool), v_ref), f"step {step}: cache"
        want = orc.verify_attention(prefix, draft, q_off, table0.pt_offset, table0.page_table, page, si.bf16_bits(q),
                                    k_ref, v_ref, hq, hkv, scale)
        assert_close(out, want, f"step {step}: attention")
        n_o, t_o, margin = orc.accept_rejection(draft, tok, tl, dl, ua, us)
        assert margin.min() > 1e-9
        np.testing.assert_array_equal(n_acc.cpu().numpy(), n_o, err_msg=f"step {step}")
        np.testing.assert_array_equal(nxt.cpu().numpy(), t_o, err_msg=f"step {step}")
        prefix = (prefix + n_o).astype(np.int32)          # the accepted drafts stay, the rest is overwritten next time
    assert (prefix > 0).any()


# ------------------------------------------------------------------------------ error paths
def test_errors_before_launch(ctx):
    import paper_2503_15921_amd as spin
    cfg = si.CONFIGS["tiny"]
    b = si.make_verify_batch(cfg, 0, device="cuda")
    t = b.table
    out = torch.empty_like(b.q)
    bad_pt = t.page_table.copy(); bad_pt[0] = t.n_pages            # page id outside the pool
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, bad_pt)
    with pytest.raises(spin.SpinError) as e:
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads)
    assert e.value.code == spin.ETABLE
    short = t.pt_offset.copy(); short[1:] -= 1                     # first request one page short
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, short, t.page_table)
    with pytest.raises(spin.SpinError) as e:
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads)
    assert e.value.code == spin.ETABLE
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    with pytest.raises(spin.SpinError) as e:                       # inexact tiling
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads,
                        subs=orc.decompose_kv_split(t.prefix_len, t.draft_len, 16)[1:])
    assert e.value.code == spin.ETABLE
    with pytest.raises(spin.SpinError) as e:                       # head_dim without a kernel
        ctx.verify_attn(tab, b.k_pool[..., :32], b.v_pool[..., :32], b.q, out, cfg.n_q_heads,
                        strides=b.k_pool.stride()[:3])
    assert e.value.code == spin.EUNSUPPORTED
    with pytest.raises(spin.SpinError) as e:                       # 3 query heads over 2 KV heads
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, 3)
    assert e.value.code == spin.EINVAL
    # nothing above may have disturbed the context
    assert_close(hip_attention(ctx, b), oracle_attention(b, 0.0), "after errors")


def test_fixed_reservation_reports_enospc():
    import paper_2503_15921_amd as spin
    c = spin.SpinContext(0, auto_reserve=False)
    try:
        b = si.make_verify_batch(si.CONFIGS["tiny"], 0, device="cuda")
        t = b.table
        tab = c.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
        out = torch.empty_like(b.q)
        with pytest.raises(spin.SpinError) as e:
            c.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, 2)
        assert e.value.code == spin.ENOSPC
        need = c.required()
        assert need[0] == t.n_req and need[1] == t.n_rows and need[3] >= t.n_req
        c.reserve(*need)
        c.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, 2)
        torch.cuda.synchronize()
        assert_close(out, oracle_attention(b, 0.0), "exact reservation")
    finally:
        c.close()


def test_plan_reuse_follows_the_tables_content(ctx):
    """Calls with the same tables launch from the tables already on the device; a change of content in the
    caller's own arrays (same objects, same addresses) is noticed; results do not depend on the reuse."""
    cfg = make_cfg("reuse", 5, 4, 2, 128)
    prefix = np.array([300, 17, 1000, 0, 64]); draft = np.array([4, 2, 8, 1, 3])
    b = si.make_verify_batch(cfg, 71, device="cuda", prefix_len=prefix, draft_len=draft)
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    outs = []
    for k in range(3):                                  # miss, hit, hit
        out = torch.full_like(b.q, float("nan"))
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads)
        outs.append(out)
    torch.cuda.synchronize()
    assert_close(outs[0], oracle_attention(b, 0.0), "first call")
    assert torch.equal(outs[1].view(torch.int16), outs[0].view(torch.int16))
    assert torch.equal(outs[2].view(torch.int16), outs[0].view(torch.int16))
    # other pools, queries and scale with the same tables: still a hit, different numbers
    q2 = torch.randn_like(b.q.float()).to(torch.bfloat16)
    out = torch.full_like(b.q, float("nan"))
    ctx.verify_attn(tab, b.v_pool, b.k_pool, q2, out, cfg.n_q_heads, softmax_scale=0.2)
    torch.cuda.synchronize()
    want = orc.verify_attention(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table, cfg.page_size,
                                si.bf16_bits(q2), si.bf16_bits(b.v_pool), si.bf16_bits(b.k_pool), cfg.n_q_heads,
                                cfg.n_kv_heads, 0.2)
    assert_close(out, want, "same tables, other tensors")
    # shorten two prefixes in place: the arrays the table object points to change, nothing else does
    tab.prefix_len[0] = 123
    tab.prefix_len[2] = 5
    t.prefix_len[0] = 123
    t.prefix_len[2] = 5
    out = torch.full_like(b.q, float("nan"))
    ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads)
    torch.cuda.synchronize()
    assert_close(out, oracle_attention(b, 0.0), "after an in-place change")
    # and with reuse switched off
    ctx.set_plan_reuse(False)
    try:
        again = torch.full_like(b.q, float("nan"))
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, again, cfg.n_q_heads)
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, again, cfg.n_q_heads)
        torch.cuda.synchronize()
        assert torch.equal(again.view(torch.int16), out.view(torch.int16))
    finally:
        ctx.set_plan_reuse(True)


def test_plan_reuse_with_queued_chunks_and_other_calls_between(ctx):
    # a plan with a chunk queue is launched three times (the queue counters are used up by every launch)
    # while acceptance calls in between take staging buffers from the same ring
    import paper_2503_15921_amd as spin
    cfg = make_cfg("reuse-queued", 6, 8, 8, 128)
    prefix = np.array([8100, 9000, 7000, 8500, 9500, 8000]); draft = np.array([4, 8, 1, 6, 2, 5])
    b = si.make_verify_batch(cfg, 72, device="cuda", prefix_len=prefix, draft_len=draft)
    ab = si.make_accept_batch(draft, 1000, 2.0, 72, device="cuda", rho=0.9)
    n_o, t_o, margin = oracle_accept(spin.ACCEPT_REJECTION, ab)
    t = b.table
    tab = ctx.make_table(t.prefix_len, t.draft_len, t.q_offset, t.pt_offset, t.page_table)
    ctx.set_waves(64)
    try:
        outs = []
        for k in range(3):
            out = torch.full_like(b.q, float("nan"))
            ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads)
            outs.append(out)
            for _ in range(3):
                n_g, t_g = hip_accept(ctx, spin.ACCEPT_REJECTION, ab)
                np.testing.assert_array_equal(n_g, n_o)
                np.testing.assert_array_equal(t_g, t_o)
        torch.cuda.synchronize()
    finally:
        ctx.set_waves(0)
    assert_close(outs[0], oracle_attention(b, 0.0), "queued plan, first launch")
    for o in outs[1:]:
        assert torch.equal(o.view(torch.int16), outs[0].view(torch.int16))


def test_many_calls_in_flight_keep_their_tables(ctx):
    """Forty calls with three different request tables, queued without a pause: the host runs many calls ahead of the
    GPU, so every device copy of a call's tables is overwritten several times while earlier calls are still queued
    (the library must hold each upload back until the kernels that read the previous copy have finished), and
    calls on a second stream share those copies (reused plans).  Every output must be what the call gives alone."""
    cfg = make_cfg("ring", 24, 8, 4, 128)
    rng = np.random.default_rng(5)
    batches = []
    for k in range(3):
        prefix = rng.integers(200, 3000, 24); draft = rng.integers(1, 9, 24)
        batches.append(si.make_verify_batch(cfg, 80 + k, device="cuda", prefix_len=prefix, draft_len=draft))
    tabs = [ctx.make_table(b.table.prefix_len, b.table.draft_len, b.table.q_offset, b.table.pt_offset, b.table.page_table)
            for b in batches]
    alone = [hip_attention(ctx, b) for b in batches]
    for b, a in zip(batches, alone):
        assert_close(a, oracle_attention(b, 0.0), "ring: alone")
    side = torch.cuda.Stream()
    outs = []
    torch.cuda.synchronize()
    for call in range(40):
        k = (call * 7 + call // 5) % 3
        b = batches[k]
        out = torch.full_like(b.q, float("nan"))
        # every fifth call repeats the previous tables (a reused plan), every tenth on the other stream
        if call % 5 == 4:
            k = outs[-1][0]
            b = batches[k]
            out = torch.full_like(b.q, float("nan"))
        if call % 10 == 9:
            # (calls of one context must not overlap -- they share its partial-result workspace -- so the two streams
            # hand over to each other; what is tested is that the table copies stay intact across the change)
            side.wait_stream(torch.cuda.current_stream())
            ctx.verify_attn(tabs[k], b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads, stream=side)
            torch.cuda.current_stream().wait_stream(side)
        else:
            ctx.verify_attn(tabs[k], b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads)
        outs.append((k, out))
    torch.cuda.synchronize()
    for call, (k, out) in enumerate(outs):
        assert torch.equal(out.view(torch.int16), alone[k].view(torch.int16)), f"call {call} (tables {k})"


def test_long_run_of_mixed_calls(ctx):
    """Two thousand attention + acceptance calls over three shapes in random order, the host up to 64 calls ahead of
    the GPU: the counters behind the ring of table copies and its markers wrap many times.  Every output of every call
    is compared, bit for bit, with what the same call gives alone (which is checked against the oracle)."""
    import paper_2503_15921_amd as spin
    rng = np.random.default_rng(11)
    items = []
    for k, (n, hq, hkv, d) in enumerate([(24, 8, 4, 128), (6, 32, 4, 128), (40, 4, 4, 64)]):
        cfg = make_cfg(f"long{k}", n, hq, hkv, d)
        b = si.make_verify_batch(cfg, 300 + k, device="cuda", prefix_len=rng.integers(100, 2500, n), draft_len=rng.integers(1, 9, n))
        tab = ctx.make_table(b.table.prefix_len, b.table.draft_len, b.table.q_offset, b.table.pt_offset, b.table.page_table)
        ab = si.make_accept_batch(b.table.draft_len, 4096 + 1000 * k, 2.0, 400 + k, device="cuda")
        ref_o = hip_attention(ctx, b)
        assert_close(ref_o, oracle_attention(b, 0.0), f"long run, shape {k}: alone")
        ref_n, ref_x = hip_accept(ctx, spin.ACCEPT_REJECTION, ab)
        want = oracle_accept(spin.ACCEPT_REJECTION, ab)
        assert np.array_equal(ref_n, want[0]) and np.array_equal(ref_x, want[1])
        items.append((cfg, b, tab, ab, ref_o, ref_n, ref_x))
    pending = []
    for call in range(2048):
        k = int(rng.integers(0, 3))
        cfg, b, tab, ab, ref_o, ref_n, ref_x = items[k]
        out = torch.full_like(b.q, float("nan"))
        n_acc = torch.full((len(ab.draft_len),), -7, dtype=torch.int32, device="cuda")
        nxt = torch.full_like(n_acc, -7)
        ctx.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, cfg.n_q_heads)
        ctx.accept(spin.ACCEPT_REJECTION, ab.draft_len, ab.draft_tokens, ab.target_logits, ab.draft_logits, ab.u_accept,
                   ab.u_sample, n_acc, nxt)
        pending.append((call, k, out, n_acc, nxt))
        if len(pending) == 64 or call == 2047:
            torch.cuda.synchronize()
            for c, kk, o, na, nx in pending:
                assert torch.equal(o.view(torch.int16), items[kk][4].view(torch.int16)), f"attention of call {c} (shape {kk})"
                assert np.array_equal(na.cpu().numpy(), items[kk][5]) and np.array_equal(nx.cpu().numpy(), items[kk][6]), \
                    f"acceptance of call {c} (shape {kk})"
            pending = []


def test_host_far_ahead_of_the_gpu_keeps_tables_apart(ctx):
    """Forty-eight calls of 7B-shaped batches with three different tables: each call's kernels run longer than the
    host needs to plan the next, so the host fills the whole ring of table copies and has to wait for slots."""
    batches = [si.make_verify_batch(si.CONFIGS["7b"], 20 + k, device="cuda") for k in range(3)]
    tabs = [ctx.make_table(b.table.prefix_len, b.table.draft_len, b.table.q_offset, b.table.pt_offset, b.table.page_table)
            for b in batches]
    alone = [hip_attention(ctx, b) for b in batches]
    ctx.set_plan_reuse(False)
    try:
        outs = []
        torch.cuda.synchronize()
        for call in range(48):
            k = (call * 5 + call // 7) % 3
            out = torch.full_like(batches[k].q, float("nan"))
            ctx.verify_attn(tabs[k], batches[k].k_pool, batches[k].v_pool, batches[k].q, out, batches[k].cfg.n_q_heads)
            outs.append((k, out))
        torch.cuda.synchronize()
    finally:
        ctx.set_plan_reuse(True)
    for call, (k, out) in enumerate(outs):
        assert torch.equal(out.view(torch.int16), alone[k].view(torch.int16)), f"call {call} (tables {k})"


def test_two_contexts_on_two_streams(ctx):
    """Calls of two contexts queued on two streams with nothing in between give what each gives alone."""
    import paper_2503_15921_amd as spin
    b1 = si.make_verify_batch(si.CONFIGS["7b"], 8, device="cuda")
    b2 = si.make_verify_batch(si.CONFIGS["skewed"], 9, device="cuda")
    alone = [hip_attention(ctx, b1), hip_attention(ctx, b2)]
    other = spin.SpinContext(0)
    try:
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        outs = [torch.full_like(b1.q, float("nan")), torch.full_like(b2.q, float("nan"))]
        tabs = [c.make_table(b.table.prefix_len, b.table.draft_len, b.table.q_offset, b.table.pt_offset, b.table.page_table)
                for c, b in ((ctx, b1), (other, b2))]
        torch.cuda.synchronize()
        for _ in range(6):
            for c, b, tab, out, st in ((ctx, b1, tabs[0], outs[0], streams[0]), (other, b2, tabs[1], outs[1], streams[1])):
                c.verify_attn(tab, b.k_pool, b.v_pool, b.q, out, b.cfg.n_q_heads, stream=st)
        torch.cuda.synchronize()
        for got, want in zip(outs, alone):
            assert torch.equal(got.view(torch.int16), want.view(torch.int16))
    finally:
        other.close()


@pytest.mark.parametrize("M", [2, 4])
def test_microbatches_on_two_streams_against_oracle(ctx, M):
    """The one-GPU shadow of the speculation/verification pipeline of Sec. V-B, as bench.py --microbatches
    issues it: the batch is cut into M micro-batches, two contexts on two streams, attention kernels chained
    by events so that the acceptance of micro-batch m runs beside the attention of m+1.  Every micro-batch's
    attention rows (tolerance) and accepted lengths / next tokens (bit for bit) against the oracle."""
    import paper_2503_15921_amd as spin
    cfg = si.CONFIGS["7b"]
    b = si.make_verify_batch(cfg, BENCH_SEED, device="cuda")
    t = b.table
    ab = si.make_accept_batch(t.draft_len, cfg.vocab, cfg.logit_sigma, BENCH_SEED, device="cuda", rho=0.9)
    tok = np.cumsum(t.prefix_len.astype(np.int64) + t.draft_len)
    cuts = sorted({0, t.n_req, *[min(t.n_req, int(np.searchsorted(tok, tok[-1] * (m + 1) / M)) + 1) for m in range(M - 1)]})
    assert len(cuts) == M + 1
    other = spin.SpinContext(0)
    try:
        ctxs = [ctx, other]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        out = torch.full_like(b.q, float("nan"))
        n_acc = torch.full((t.n_req,), -7, dtype=torch.int32, device="cuda")
        nxt = torch.full((t.n_req,), -7, dtype=torch.int32, device="cuda")
        mbs = []
        for k, (i0, i1) in enumerate(zip(cuts[:-1], cuts[1:])):
            r0, r1 = int(t.q_offset[i0]), int(t.q_offset[i1])
            p0, p1 = int(t.pt_offset[i0]), int(t.pt_offset[i1])
            c = ctxs[k % 2]
            mbs.append(dict(ctx=c, stream=streams[k % 2], draft=t.draft_len[i0:i1],
                            tab=c.make_table(t.prefix_len[i0:i1], t.draft_len[i0:i1], t.q_offset[i0:i1 + 1] - r0,
                                             t.pt_offset[i0:i1 + 1] - p0, t.page_table[p0:p1]),
                            q=b.q[r0:r1], out=out[r0:r1], tokens=ab.draft_tokens[r0:r1],
                            target=ab.target_logits[r0 + i0:r1 + i1], dlogits=ab.draft_logits[r0:r1],
                            u_acc=ab.u_accept[r0:r1], u_smp=ab.u_sample[i0:i1], n_acc=n_acc[i0:i1], nxt=nxt[i0:i1]))
        attn_done = [torch.cuda.Event() for _ in mbs]
        torch.cuda.synchronize()
        for rep in range(3):            # several steps back to back: staging buffers and workspaces are reused
            for k, mb in enumerate(mbs):
                with torch.cuda.stream(mb["stream"]):
                    if k > 0 or rep > 0:
                        mb["stream"].wait_event(attn_done[k - 1])
                    mb["ctx"].verify_attn(mb["tab"], b.k_pool, b.v_pool, mb["q"], mb["out"], cfg.n_q_heads, stream=mb["stream"])
                    attn_done[k].record(mb["stream"])
                    mb["ctx"].accept(spin.ACCEPT_REJECTION, mb["draft"], mb["tokens"], mb["target"], mb["dlogits"],
                                     mb["u_acc"], mb["u_smp"], mb["n_acc"], mb["nxt"], stream=mb["stream"])
        torch.cuda.synchronize()
    finally:
        other.close()
    want = oracle_attention(b, 0.0)
    for k, (i0, i1) in enumerate(zip(cuts[:-1], cuts[1:])):
        r0, r1 = int(t.q_offset[i0]), int(t.q_offset[i1])
        assert_close(out[r0:r1], want[r0:r1], f"micro-batch {k} of {M}")
    n_o, t_o, margin = oracle_accept(spin.ACCEPT_REJECTION, ab)
    assert margin.min() > 1e-9
    np.testing.assert_array_equal(n_acc.cpu().numpy(), n_o)
    np.testing.assert_array_equal(nxt.cpu().numpy(), t_o)
    assert len(set(n_o.tolist())) >= 3


def test_profile_sampling(ctx):
    b = si.make_verify_batch(si.CONFIGS["tiny"], 7, device="cuda")
    ctx.profile_begin(10, every=3)
    for _ in range(7):
        hip_attention(ctx, b)
    ms, calls = ctx.profile_end()
    assert calls[0] == 3 and calls[1] == 0          # calls 0, 3 and 6 of the seven were timed
    assert ms["attn"] > 0 and ms["accept_stats"] == 0
    ctx.profile_begin(2)                            # every call, but only two slots
    for _ in range(4):
        hip_attention(ctx, b)
    ms, calls = ctx.profile_end()
    assert calls[0] == 2


def test_empty_batch(ctx):
    import paper_2503_15921_amd as spin
    tab = ctx.make_table(np.zeros(0, np.int32), np.zeros(0, np.int32), np.zeros(1, np.int32),
                         np.zeros(1, np.int32), np.zeros(0, np.int32))
    k = torch.zeros((1, 2, 16, 64), dtype=torch.bfloat16, device="cuda")
    q = torch.zeros((0, 2, 64), dtype=torch.bfloat16, device="cuda")
    ctx.verify_attn(tab, k, k, q, q.clone(), 2)
    e = torch.zeros(0, dtype=torch.int32, device="cuda")
    ctx.accept(spin.ACCEPT_GREEDY, np.zeros(0, np.int32), e, torch.zeros((0, 10), device="cuda"), None, None, None, e, e)
    torch.cuda.synchronize()
