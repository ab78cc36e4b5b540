"""CPU-only tests of libspin's host side: the library loads and exports what include/spin.h declares,
spin_decompose / spin_kv_padding agree with the oracle, spin_check_tiling accepts exactly the exact
tilings, the scheduler's work items tile every request once, and error codes come back as documented.
No GPU call is made here."""
import os
import re

import numpy as np
import pytest

import paper_2503_15921_amd as spin
from oracle import spin_oracle as orc
from test_oracle_decompose import assert_exact_tiling
from test_oracle_attention import random_rectangles

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "spin.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(spin_[a-z_]+)\s*\(", header))
    assert {"spin_verify_attn", "spin_decompose", "spin_accept"} <= declared
    lib = spin.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    from paper_2503_15921_amd.binding import EXPORTS
    assert declared == set(EXPORTS)


def test_stream_probe_refuses_what_would_not_fit():
    # the measuring kernels of bench.py --calib-stream check their sizes on the host before anything is launched
    import ctypes as C
    from paper_2503_15921_amd.build import PROBE_LIB
    lib = C.CDLL(PROBE_LIB)
    lib.spin_probe_read_beside_writers.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p, C.c_uint64,
                                                   C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    lib.spin_probe_read_blocks.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
    invalid = 1   # hipErrorInvalidValue
    fake = 4096   # stands for a device address; never dereferenced by a refused call
    assert lib.spin_probe_read_beside_writers(fake, fake, 1024, 1024, fake, 256 * 18 * 4096 - 1, 256, 18, 16, 0, fake, None) == invalid
    assert lib.spin_probe_read_beside_writers(fake, fake, 1024, 1024, fake, 1 << 30, 256, 18, 16, 4, fake, None) == invalid
    assert lib.spin_probe_read_beside_writers(fake, fake, 1024, 1022, fake, 1 << 30, 256, 18, 16, 0, fake, None) == invalid
    assert lib.spin_probe_read_beside_writers(None, fake, 1024, 1024, fake, 1 << 30, 256, 18, 16, 0, fake, None) == invalid
    assert lib.spin_probe_read_blocks(None, fake, 1024, 1024, 1, fake, None) != 0


def test_strerror():
    lib = spin.load_library()
    assert lib.spin_strerror(0) == b"ok"
    for code in (spin.EINVAL, spin.ETABLE, spin.ENOSPC, spin.EUNSUPPORTED, spin.EHIP):
        assert len(lib.spin_strerror(code)) > 3


@pytest.mark.parametrize("seed", range(5))
def test_decompose_matches_oracle(seed):
    rng = np.random.default_rng(seed)
    B = int(rng.integers(1, 20))
    prefix = rng.integers(0, 500, size=B); draft = rng.integers(1, 17, size=B)
    for w in (1, 3, 4, 16):
        got, _ = spin.decompose(prefix, draft, spin.DECOMP_Q_SPLIT, q_width=w)
        np.testing.assert_array_equal(got, orc.decompose_q_split(prefix, draft, w))
    for L in (1, 16, 37, 128, 4096):
        got, Lout = spin.decompose(prefix, draft, spin.DECOMP_KV_SPLIT, kv_len=L)
        np.testing.assert_array_equal(got, orc.decompose_kv_split(prefix, draft, L))
        assert Lout == L
        assert spin.kv_padding(prefix, draft, L) == orc.kv_padding(prefix, draft, L)
    got, _ = spin.decompose(prefix, draft, spin.DECOMP_NONE)
    np.testing.assert_array_equal(got, orc.decompose_kv_split(prefix, draft, 1 << 20))


@pytest.mark.parametrize("seed", range(6))
def test_kv_search_matches_oracle(seed):
    rng = np.random.default_rng(50 + seed)
    B = int(rng.integers(1, 16))
    prefix = rng.integers(0, 400, size=B); draft = rng.integers(1, 9, size=B)
    step = int(rng.choice([1, 16]))
    l_min, l_max = int(rng.integers(1, 64)), int((prefix + draft).max())
    for max_rows in (B, B + 2, 4 * B):
        want = orc.search_kv_length(prefix, draft, max_rows, l_min, l_max, step)
        if want is None:
            with pytest.raises(spin.SpinError) as e:
                spin.decompose(prefix, draft, spin.DECOMP_KV_SEARCH, max_subreq=max_rows, l_min=l_min,
                               l_max=l_max, l_step=step)
            assert e.value.code == spin.ENOSPC
        else:
            got, L = spin.decompose(prefix, draft, spin.DECOMP_KV_SEARCH, max_subreq=max_rows, l_min=l_min,
                                    l_max=l_max, l_step=step)
            assert L == want
            np.testing.assert_array_equal(got, orc.decompose_kv_split(prefix, draft, want))
            assert len(got) <= max_rows


def test_decompose_capacity_protocol():
    prefix = np.array([10, 20]); draft = np.array([8, 3])
    with pytest.raises(spin.SpinError) as e:
        spin.decompose(prefix, draft, spin.DECOMP_Q_SPLIT, q_width=2, cap=3)
    assert e.value.code == spin.ENOSPC
    got, _ = spin.decompose(prefix, draft, spin.DECOMP_Q_SPLIT, q_width=2, cap=6)
    assert len(got) == 6


def test_decompose_rejects_bad_input():
    for kwargs in (dict(policy=spin.DECOMP_Q_SPLIT, q_width=0), dict(policy=spin.DECOMP_KV_SPLIT, kv_len=0),
                   dict(policy=99), dict(policy=spin.DECOMP_KV_SEARCH, max_subreq=0, l_min=1, l_max=4)):
        with pytest.raises(spin.SpinError) as e:
            spin.decompose(np.array([4]), np.array([2]), **kwargs)
        assert e.value.code == spin.EINVAL
    with pytest.raises(spin.SpinError) as e:
        spin.decompose(np.array([4]), np.array([0]), spin.DECOMP_NONE)       # draft length < 1
    assert e.value.code == spin.EINVAL
    with pytest.raises(spin.SpinError):
        spin.decompose(np.array([-1]), np.array([1]), spin.DECOMP_NONE)


def test_check_tiling_accepts_exact_and_rejects_broken():
    rng = np.random.default_rng(3)
    prefix = rng.integers(0, 30, size=5); draft = rng.integers(1, 7, size=5)
    good = [orc.decompose_q_split(prefix, draft, 2), orc.decompose_kv_split(prefix, draft, 7),
            np.array([(i,) + r for i in range(5) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))])]
    for subs in good:
        assert_exact_tiling(prefix, draft, subs)
        assert spin.check_tiling(prefix, draft, subs) == 0
        # order must not matter
        assert spin.check_tiling(prefix, draft, subs[rng.permutation(len(subs))]) == 0
        # drop one piece -> a hole; duplicate one -> an overlap
        assert spin.check_tiling(prefix, draft, subs[1:]) == spin.ETABLE
        assert spin.check_tiling(prefix, draft, np.concatenate([subs, subs[:1]])) == spin.ETABLE
    bad = good[1].copy(); bad[0, 4] += 1000                      # sticks out of its parent
    assert spin.check_tiling(prefix, draft, bad) == spin.ETABLE
    bad = good[1].copy(); bad[0, 0] = 77                         # unknown parent
    assert spin.check_tiling(prefix, draft, bad) == spin.ETABLE
    # a piece wholly beyond the causal edge is legal and covers nothing
    p, g = 4, 3
    subs = np.array([[0, 0, 3, 0, 7], ])
    assert spin.check_tiling([p], [g], subs) == 0
    subs = np.array([[0, 0, 1, 0, 5], [0, 1, 2, 0, 7], [0, 0, 1, 5, 2]])   # last one: row 0, keys 5..6 -> invisible
    assert spin.check_tiling([p], [g], subs) == 0


def test_check_tiling_against_a_cell_bitmap():
    """Random sets of rectangles on small requests -- exact tilings with one rectangle moved, grown, shrunk or
    doubled, and rectangles drawn at random -- judged by the library and by counting how often every visible
    cell is covered."""
    rng = np.random.default_rng(17)
    n_ok = n_bad = 0
    for case in range(600):
        p, g = int(rng.integers(0, 12)), int(rng.integers(1, 7))
        if case % 3 == 0:
            rects = [tuple(int(x) for x in (rng.integers(0, g), 1, rng.integers(0, p + g), 1)) for _ in range(int(rng.integers(1, 6)))]
            rects = [(qb, int(rng.integers(1, g - qb + 1)), kb, int(rng.integers(1, p + g - kb + 1))) for qb, _, kb, _ in rects]
        else:
            rects = list(random_rectangles(rng, p, g))
            k = int(rng.integers(len(rects)))
            qb, ql, kb, kl = rects[k]
            what = int(rng.integers(5))
            if what == 0 and kb + kl < p + g:
                kl += 1
            elif what == 1 and kl > 1:
                kl -= 1
            elif what == 2 and qb + ql < g:
                ql += 1
            elif what == 3 and kb > 0:
                kb -= 1
                kl += 1
            rects[k] = (qb, ql, kb, kl)      # (what == 4 or an impossible move: left exact)
        cover = np.zeros((g, p + g), dtype=np.int64)
        for qb, ql, kb, kl in rects:
            cover[qb:qb + ql, kb:kb + kl] += 1
        exact = all((cover[t, :p + t + 1] == 1).all() for t in range(g))
        subs = np.array([(0,) + tuple(r) for r in rects], dtype=np.int32)
        assert (spin.check_tiling([p], [g], subs) == 0) == exact, (p, g, rects)
        n_ok += exact
        n_bad += not exact
    assert n_ok > 50 and n_bad > 50


def test_check_tiling_of_many_pieces_is_fast():
    # a KV-split with a short length on long requests: ~10^5 pieces per request
    import time
    prefix = np.array([200000, 150000]); draft = np.array([4, 8])
    subs = orc.decompose_kv_split(prefix, draft, 2)
    t0 = time.perf_counter()
    assert spin.check_tiling(prefix, draft, subs) == 0
    assert time.perf_counter() - t0 < 2.0


def blocks_of(piece, bk=32):
    return -(-int(piece[4]) // bk)


def check_schedule(prefix, draft, subs, page, group, n_kv, n_waves):
    """Everything a schedule must satisfy, whatever the inputs."""
    pcs = spin.schedule(prefix, draft, subs, page, group, n_kv, n_waves)
    for h in range(n_kv):
        assert_exact_tiling(prefix, draft, pcs[pcs[:, 5] == h][:, :5])
    widest = int((pcs[:, 2] * group).max())        # one launch per call, sized for the widest strip
    call_cls = 0 if widest <= 16 else 1 if widest <= 32 else 2
    bk = 128 if call_cls == 2 else 32
    for pc in pcs:
        parent, qb, ql, kb, kl, kvh, cls, wave, flags = (int(x) for x in pc)
        assert ql * group <= 64 and cls == call_cls
        assert kl >= 1 and (kb + kl - 1) // page - kb // page + 1 <= 136
        assert wave >= 0
    for cls in range(3):
        c = pcs[pcs[:, 6] == cls]
        if len(c) == 0:
            continue
        # equal shares: the wavefronts of a class differ by at most one block; queued chunks
        # (handed out at run time) come after them and hold 1..64 blocks
        per_share = np.zeros(int(c[:, 7].max()) + 1, dtype=np.int64)
        for pc in c:
            per_share[pc[7]] += blocks_of(pc, bk)
        queued = np.zeros(len(per_share), dtype=bool)
        queued[c[(c[:, 8] & spin.PIECE_QUEUED) != 0][:, 7]] = True
        static = per_share[~queued]
        assert len(static) <= n_waves and static.min() >= 1
        if static.mean() > 8.5:
            assert static.max() - static.min() <= 1
        else:      # short shares: boundaries within 4 blocks of the end of a (rectangle, head) moved there
            assert static.max() <= static.mean() + 9
        if queued.any():
            assert cls < 2                      # the grouped-query kernel gets equal shares only
            assert queued[len(static):].all() and n_waves >= 64
            assert per_share[queued].min() >= 1 and per_share[queued].max() * bk <= 1024
            assert static.min() * bk >= 5000 and 0.05 < per_share[queued].sum() / per_share.sum() < 0.15
        # a share's pieces are consecutive in the class's streaming order
        assert list(c[:, 7]) == sorted(c[:, 7])
    # flags: CARRY_IN / CARRY_OUT link neighbours of one (rectangle, head) inside one wavefront;
    # DIRECT only where one wavefront holds a whole rectangle that reaches from key 0 to its causal edge
    for k, pc in enumerate(pcs):
        parent, qb, ql, kb, kl, kvh, cls, wave, flags = (int(x) for x in pc)
        same_prev = k > 0 and tuple(pcs[k - 1][[0, 1, 2, 5, 6, 7]]) == (parent, qb, ql, kvh, cls, wave) \
            and pcs[k - 1][3] + pcs[k - 1][4] == kb
        assert bool(flags & spin.PIECE_CARRY_IN) == bool(same_prev)
        if flags & spin.PIECE_CARRY_IN:
            assert pcs[k - 1][8] & spin.PIECE_CARRY_OUT
        if flags & spin.PIECE_DIRECT:
            chain_start = k
            while pcs[chain_start][8] & spin.PIECE_CARRY_IN:
                chain_start -= 1
            assert pcs[chain_start][3] == 0 and kb + kl == prefix[parent] + qb + ql
            assert not (flags & spin.PIECE_CARRY_OUT)
    return pcs


@pytest.mark.parametrize("group,n_kv,n_waves,page,top", [(1, 4, 64, 16, 3000), (1, 2, 7, 16, 3000), (8, 2, 100, 16, 3000),
                                                         (4, 1, 3, 4, 3000), (1, 3, 1000, 1, 3000), (3, 2, 16, 16, 3000),
                                                         (1, 8, 64, 16, 30000)])
def test_scheduler_pieces_tile_every_request_and_head(group, n_kv, n_waves, page, top):
    rng = np.random.default_rng(group * 1000 + n_waves)
    prefix = rng.integers(0, top, size=7); draft = rng.integers(1, 17, size=7)
    decomps = [None, orc.decompose_q_split(prefix, draft, 4), orc.decompose_kv_split(prefix, draft, 100),
               np.array([(i,) + r for i in range(7) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))])]
    for subs in decomps:
        check_schedule(prefix, draft, subs, page, group, n_kv, n_waves)


def test_scheduler_on_many_random_small_batches():
    rng = np.random.default_rng(77)
    for case in range(120):
        n_req = int(rng.integers(1, 12))
        group = int(rng.choice([1, 1, 2, 4, 8, 16, 64]))
        n_kv = int(rng.integers(1, 5))
        page = int(rng.choice([1, 4, 16, 64]))
        n_waves = int(rng.choice([1, 2, 5, 64, 300, 1024, 16384]))
        top = int(rng.choice([8, 40, 200, 1500]))
        prefix = rng.integers(0, top + 1, size=n_req)
        draft = rng.integers(1, max(2, 64 // group) + 1 if rng.random() < 0.5 else 9, size=n_req)
        kind = int(rng.integers(3))
        subs = None if kind == 0 else orc.decompose_kv_split(prefix, draft, int(rng.integers(1, 300))) if kind == 1 else \
            np.array([(i,) + r for i in range(n_req) for r in random_rectangles(rng, int(prefix[i]), int(draft[i]))])
        try:
            check_schedule(prefix, draft, subs, page, group, n_kv, n_waves)
        except AssertionError as e:
            raise AssertionError(f"case {case}: n_req {n_req} group {group} n_kv {n_kv} page {page} waves {n_waves} "
                                 f"prefix {prefix.tolist()} draft {draft.tolist()} kind {kind}: {e}") from e


def test_scheduler_keeps_short_pairs_whole():
    # many short requests: every (request, head) fits a few blocks, so no share boundary cuts one,
    # everything is written directly and nothing is left for the join kernel
    rng = np.random.default_rng(8)
    prefix = rng.integers(0, 120, size=40); draft = rng.integers(1, 6, size=40)
    pcs = spin.schedule(prefix, draft, None, 16, 1, 2, 1024)
    ends = pcs[(pcs[:, 8] & spin.PIECE_CARRY_OUT) == 0]
    assert len(ends) == 40 * 2 and (ends[:, 8] & spin.PIECE_DIRECT).all()
    for h in range(2):
        assert_exact_tiling(prefix, draft, pcs[pcs[:, 5] == h][:, :5])
    # a long request among them is still cut
    prefix[7] = 4000
    pcs = spin.schedule(prefix, draft, None, 16, 1, 2, 1024)
    assert (pcs[pcs[:, 0] == 7][:, 8] & spin.PIECE_DIRECT).sum() == 0
    short = pcs[(pcs[:, 0] != 7) & ((pcs[:, 8] & spin.PIECE_CARRY_OUT) == 0)]
    assert (short[:, 8] & spin.PIECE_DIRECT).mean() > 0.9


def test_scheduler_queues_a_tail_for_long_single_wavefront_shares_only():
    rng = np.random.default_rng(7)
    prefix = rng.integers(3000, 9000, 24).astype(np.int32)
    draft = rng.integers(5, 9, 24).astype(np.int32)
    mha = check_schedule(prefix, draft, None, 16, 1, 8, 128)          # strips of at most 8 rows
    assert (mha[:, 8] & spin.PIECE_QUEUED).any()
    gqa = check_schedule(prefix, draft, None, 16, 8, 8, 128)          # strips of up to 64 rows
    assert (gqa[:, 6] == 2).all() and not (gqa[:, 8] & spin.PIECE_QUEUED).any()


def test_scheduler_rejoins_row_bands_sharing_a_prefix():
    # width-4 pieces of a 16-row draft block all start at key 0: they are streamed as one band, so
    # the schedule equals that of the undivided request; so does a cut along the keys
    prefix = np.array([1000, 300]); draft = np.array([16, 2])
    whole = spin.schedule(prefix, draft, None, 16, 1, 2, 8)
    split = spin.schedule(prefix, draft, orc.decompose_q_split(prefix, draft, 4), 16, 1, 2, 8)
    np.testing.assert_array_equal(whole, split)
    kv = spin.schedule(prefix, draft, orc.decompose_kv_split(prefix, draft, 100), 16, 1, 2, 8)
    np.testing.assert_array_equal(whole, kv)


def test_scheduler_single_wave_writes_everything_directly():
    prefix = np.array([100, 5000, 0]); draft = np.array([3, 8, 1])
    pcs = spin.schedule(prefix, draft, None, 16, 1, 2, 1)
    ends = pcs[(pcs[:, 8] & spin.PIECE_CARRY_OUT) == 0]
    assert len(ends) == 3 * 2 and (ends[:, 8] & spin.PIECE_DIRECT).all()
    # the long request is cut into page-id windows that carry their accumulators along
    assert (pcs[pcs[:, 0] == 1][:, 4] <= 2048).all() and (pcs[:, 8] & spin.PIECE_CARRY_IN).any()


def test_scheduler_rejects_inexact_tiling():
    prefix = np.array([40]); draft = np.array([4])
    subs = orc.decompose_kv_split(prefix, draft, 16)[:-1]
    with pytest.raises(spin.SpinError) as e:
        spin.schedule(prefix, draft, subs, 16, 1, 1, 8)
    assert e.value.code == spin.ETABLE


def test_create_without_gpu_reports_hip_error():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(spin.SpinError) as e:
        spin.SpinContext(0)
    assert e.value.code == spin.EHIP
