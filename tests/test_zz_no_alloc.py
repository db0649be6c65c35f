"""hs_draft_static -- the entry point that allocates nothing (its scratch is a static device array) -- against
hs_draft on the same inputs: every output array bit for bit, on two calls in a row, the second on a smaller input
(fewer sequences, shorter histories) so that stale contents of the shared array would show; then on a context with
no workspace bound at all, and the capacity check."""
import ctypes as C

import numpy as np
import pytest
import torch

from hs_inputs import CONFIG_SHAPES, config_seed, make_weights, rope_table
from gpu_common import np_of

pytestmark = pytest.mark.gpu

OUT = ("draft_start", "match_len", "draft_len", "row_off", "tok", "pos", "parent", "anc_mask", "row2seq")


def _case(rng, vocab, B, n_cand, hist_len, W, n_ctx):
    """Sequences whose last tokens occur in their histories (so drafts exist), plus some that match nothing."""
    toks, cands = [], []
    for b in range(B):
        t = rng.integers(0, vocab, n_ctx + int(rng.integers(0, 9))).astype(np.int32)
        row = []
        for c in range(n_cand):
            h = rng.integers(0, vocab, hist_len + int(rng.integers(0, 50))).astype(np.int32)
            if (b + c) % 4 != 3:
                at = int(rng.integers(W, len(h) - 40))
                m = int(rng.integers(3, W + 1))
                h[at - m:at] = t[-m:]
            row.append(h)
        toks.append(t)
        cands.append(row)
    return toks, cands


def _run(eng, pol, static):
    from paper_2508_18588_amd import hs_draft, hs_draft_args, hs_draft_static
    for v in eng.st.values():
        v.fill_(-7)
    args = hs_draft_args(eng.n_cand, eng.hist.data_ptr(), eng.hist_off.data_ptr(), pol.c())
    (hs_draft_static if static else hs_draft)(eng.ctx, args, eng.c_seq, eng.c_step, eng.stream())
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    return {k: np_of(eng.st[k]).copy() for k in OUT}


def test_static_scratch_draft_equals_hs_draft_twice_in_a_row():
    from paper_2508_18588_amd import HS_K_MATCHLEN
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = CONFIG_SHAPES[1]
    w = make_weights(shape, config_seed(1))
    rng = np.random.default_rng(41)
    W = 16
    pol = Policy(window=W, m_min=3, k_mode=HS_K_MATCHLEN, k_max=16)
    eng = Engine(shape, w, rope_table(20000, shape.head_dim), max_batch=96, k_max=16, c_max=2, max_len=64)
    drafted = []
    # first call: 96 sequences, two candidates of ~17k tokens (five history segments each); second: 5 sequences, one
    # candidate of ~300 tokens (one segment) -- most of the array keeps the first call's winners
    for B, n_cand, hist_len in ((96, 2, 17000), (5, 1, 300)):
        toks, cands = _case(rng, shape.vocab, B, n_cand, hist_len, W, 40)
        eng.load_sequences(toks, budgets=[50] * B)
        eng.set_history(cands)
        want = _run(eng, pol, static=False)
        got = _run(eng, pol, static=True)
        for k in OUT:
            assert (got[k] == want[k]).all(), (B, k)
        assert want["row_off"][B] > B          # drafts were made
        drafted.append(int(want["row_off"][B]) - B)
    eng.close()
    print("static-scratch draft: drafted tokens per call", drafted)


def test_static_scratch_draft_needs_no_workspace_and_rejects_oversize():
    import paper_2508_18588_amd as hs
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = CONFIG_SHAPES[1]
    w = make_weights(shape, config_seed(1))
    rng = np.random.default_rng(43)
    pol = Policy(window=8, m_min=3, k_fixed=4, k_max=4)
    toks, cands = _case(rng, shape.vocab, 7, 1, 500, 8, 30)
    eng = Engine(shape, w, rope_table(1024, shape.head_dim), max_batch=8, k_max=4, c_max=1, max_len=64)
    eng.load_sequences(toks, budgets=[20] * 7)
    eng.set_history(cands)
    want = _run(eng, pol, static=False)
    # the same context with its workspace taken away: hs_draft refuses, hs_draft_static still works
    hs.hs_set_flags(eng.ctx, hs.HS_FLAG_FP32_ACTIVATIONS)        # larger layout: the bound workspace is dropped
    args = hs.hs_draft_args(eng.n_cand, eng.hist.data_ptr(), eng.hist_off.data_ptr(), pol.c())
    with pytest.raises(hs.HsError) as e:
        hs.hs_draft(eng.ctx, args, eng.c_seq, eng.c_step, eng.stream())
    assert e.value.status == hs.HS_ERR_CAPACITY
    got = _run(eng, pol, static=True)
    for k in OUT:
        assert (got[k] == want[k]).all(), k
    eng.close()
    # capacity: 1200 sequences x 2 candidates x 33 segments (max_pos 131072) = 79200 slots > 65536
    big = Engine(shape, w, rope_table(131072, shape.head_dim), max_batch=1200, k_max=1, c_max=2, max_len=32)
    toks, cands = _case(rng, shape.vocab, 1200, 2, 100, 8, 10)
    big.load_sequences(toks, budgets=[4] * 1200)
    big.set_history(cands)
    args = hs.hs_draft_args(2, big.hist.data_ptr(), big.hist_off.data_ptr(),
                            Policy(window=8, m_min=3, k_fixed=1, k_max=1).c())
    with pytest.raises(hs.HsError) as e:
        hs.hs_draft_static(big.ctx, args, big.c_seq, big.c_step, big.stream())
    assert e.value.status == hs.HS_ERR_CAPACITY and "65536" in str(e.value)
    hs.hs_draft(big.ctx, args, big.c_seq, big.c_step, big.stream())      # the workspace variant takes it
    torch.cuda.synchronize()
    big.close()
