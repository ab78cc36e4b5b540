"""GPU test of spin_accept_noalloc, the entry point for callers that cannot allocate: its outputs against
spin_accept's (and the oracle's) bit for bit, on two calls in a row, the second with a smaller input."""
import numpy as np
import pytest
import torch

import spin_inputs as si
from oracle import spin_oracle as orc

pytestmark = pytest.mark.gpu


def run_both(ctx, spin, mode, ab):
    B = len(ab.draft_len)
    q_off = torch.from_numpy(np.concatenate([[0], np.cumsum(ab.draft_len)]).astype(np.int32)).cuda()
    outs = []
    for kind in ("ctx", "noalloc"):
        n_acc = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        nxt = torch.full((B,), -7, dtype=torch.int32, device="cuda")
        if kind == "ctx":
            ctx.accept(mode, ab.draft_len, ab.draft_tokens, ab.target_logits, ab.draft_logits, ab.u_accept, ab.u_sample,
                       n_acc, nxt)
        else:
            torch.cuda.synchronize()
            before = torch.cuda.memory_allocated()
            spin.accept_noalloc(mode, q_off, ab.draft_tokens, ab.target_logits, ab.draft_logits, ab.u_accept,
                                ab.u_sample, n_acc, nxt)
            assert torch.cuda.memory_allocated() == before
        torch.cuda.synchronize()
        outs.append((n_acc.cpu().numpy(), nxt.cpu().numpy()))
    return outs


def test_noalloc_accept_matches_spin_accept_twice_in_a_row():
    import paper_2503_15921_amd as spin
    ctx = spin.SpinContext(0)
    try:
        # first the 13B-shaped batch, then a smaller one: the second call finds the first call's statistics
        # in the shared static array and must not be disturbed by them
        for name, seed, rho in (("13b", 3, 0.95), ("7b", 5, 0.9), ("tiny", 1, None)):
            cfg = si.CONFIGS[name]
            draft_len = si.draw_lengths(cfg, np.random.default_rng(seed))[1]
            for mode, tok_mode in ((spin.ACCEPT_REJECTION, "sample"), (spin.ACCEPT_GREEDY, "argmax")):
                ab = si.make_accept_batch(draft_len, cfg.vocab, cfg.logit_sigma, seed, device="cuda", rho=rho,
                                          draft_token_mode=tok_mode)
                (n_c, t_c), (n_s, t_s) = run_both(ctx, spin, mode, ab)
                np.testing.assert_array_equal(n_s, n_c, err_msg=f"{name} mode {mode}")
                np.testing.assert_array_equal(t_s, t_c, err_msg=f"{name} mode {mode}")
                tl = ab.target_logits.cpu().numpy(); toks = ab.draft_tokens.cpu().numpy()
                if mode == spin.ACCEPT_GREEDY:
                    n_o, t_o, margin = orc.accept_greedy(ab.draft_len, toks, tl)
                else:
                    n_o, t_o, margin = orc.accept_rejection(ab.draft_len, toks, tl, ab.draft_logits.cpu().numpy(),
                                                            ab.u_accept.cpu().numpy(), ab.u_sample.cpu().numpy())
                assert margin.min() > 1e-9
                np.testing.assert_array_equal(n_s, n_o)
                np.testing.assert_array_equal(t_s, t_o)
    finally:
        ctx.close()


def test_noalloc_accept_limits_and_bad_offsets():
    import paper_2503_15921_amd as spin
    lib = spin.load_library()
    draft_len = np.array([3, 1, 2], dtype=np.int32)
    ab = si.make_accept_batch(draft_len, 100, 2.0, 0, device="cuda")
    n_acc = torch.full((3,), -7, dtype=torch.int32, device="cuda")
    nxt = torch.full((3,), -7, dtype=torch.int32, device="cuda")
    q_off = torch.tensor([0, 3, 4, 6], dtype=torch.int32, device="cuda")
    # beyond the static array: refused before anything is launched
    with pytest.raises(spin.SpinError) as ei:
        spin.accept_noalloc(spin.ACCEPT_REJECTION, q_off, ab.draft_tokens, ab.target_logits, ab.draft_logits,
                            ab.u_accept, ab.u_sample, n_acc, nxt, n_rows=20000)
    assert ei.value.code == spin.ENOSPC
    with pytest.raises(spin.SpinError) as ei:
        spin.accept_noalloc(spin.ACCEPT_REJECTION, q_off, ab.draft_tokens, ab.target_logits, ab.draft_logits,
                            ab.u_accept, ab.u_sample, n_acc, nxt, n_rows=2)
    assert ei.value.code == spin.EINVAL
    torch.cuda.synchronize()
    assert (n_acc.cpu().numpy() == -7).all()
    # offsets the host cannot see: a request whose rows fall outside the tensors reports -1, the others are served
    bad = torch.tensor([0, 3, 3, 9], dtype=torch.int32, device="cuda")
    spin.accept_noalloc(spin.ACCEPT_REJECTION, bad, ab.draft_tokens, ab.target_logits, ab.draft_logits,
                        ab.u_accept, ab.u_sample, n_acc, nxt)
    torch.cuda.synchronize()
    assert n_acc.cpu().numpy()[1] == -1 and nxt.cpu().numpy()[1] == -1
    assert n_acc.cpu().numpy()[2] == -1 and nxt.cpu().numpy()[2] == -1
    assert 0 <= n_acc.cpu().numpy()[0] <= 3
