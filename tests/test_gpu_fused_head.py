"""The path that keeps no logits: the LM head's row-maximum epilogue (every workgroup reduces its columns of a row to
one key), the argmax finished inside the acceptance kernel, and acceptance + commit as one launch -- against the path
that materialises the fp32 logits and runs argmax, acceptance and commit as separate launches.  Same accumulators on
both sides, so everything must agree bit for bit."""
import numpy as np
import pytest
import torch

from hs_inputs import CONFIG_SHAPES, ModelShape, config_seed, make_prompts, make_weights, rope_table
from gpu_common import make_histories, np_of

pytestmark = pytest.mark.gpu


def test_row_maximum_epilogue_names_the_first_maximum_of_every_row():
    """hs_debug_gemm with the row-maximum epilogue against the same projection stored as fp32: for every row the
    largest key over the column groups carries the bits of the row's largest logit and the LOWEST column holding it
    (ties planted by duplicating weight rows inside one column group and across groups)."""
    from paper_2508_18588_amd import hs_debug_rowmax_groups
    from paper_2508_18588_amd.runtime import Engine
    shape = ModelShape(n_layers=1, d_model=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ffn=1024, vocab=16448)
    w = make_weights(shape, 57)
    lm = w["lm_head"]
    lm[7] = lm[3]            # same column group
    lm[9000] = lm[3]         # another group
    lm[16447] = lm[16440]    # the ragged last group
    m_max = 1100
    eng = Engine(shape, w, rope_table(64, shape.head_dim), max_batch=64, k_max=16, c_max=1, max_len=32, max_rows=m_max)
    g = torch.Generator(device="cuda:0").manual_seed(3)
    a = torch.randn(m_max, shape.d_model, device="cuda:0", generator=g)
    # some rows point along a duplicated weight row, so that the duplicated columns hold the row's maximum
    wf = eng.w["lm_head"].view(torch.bfloat16).float()
    a[5] = wf[3] * 40
    a[40] = wf[16440] * 40
    a[700] = wf[3] * 25
    a = a.to(torch.bfloat16).view(torch.int16)
    ng = hs_debug_rowmax_groups(shape.vocab)
    for m in (1, 33, 220, 385, 1054):
        m_dev = torch.full((1,), m, dtype=torch.int32, device="cuda:0")
        logits = torch.zeros(m_max, shape.vocab, dtype=torch.float32, device="cuda:0")
        eng.gemm(0, a, eng.w["lm_head"], None, logits, m_dev, m_max, m)
        keys = torch.full((m_max, ng), -1, dtype=torch.int64, device="cuda:0")
        eng.gemm(3, a, eng.w["lm_head"], None, keys, m_dev, m_max, m)
        torch.cuda.synchronize()
        assert eng.poll_error() == 0
        k = np_of(keys).view(np.uint64)
        assert (k[m:] == np.uint64(0xFFFFFFFFFFFFFFFF)).all(), "rows beyond M were written"
        best = k[:m].max(axis=1)
        col = (np.uint64(0xFFFFFFFF) - (best & np.uint64(0xFFFFFFFF))).astype(np.int64)
        lg = np_of(logits[:m])
        assert col.tolist() == lg.argmax(axis=1).tolist(), m          # numpy's argmax is the first maximum
        u = (best >> np.uint64(32)).astype(np.uint32)
        bits = np.where(u & np.uint32(0x80000000), u & np.uint32(0x7FFFFFFF), ~u).astype(np.uint32)
        assert (bits.view(np.float32) == lg.max(axis=1)).all(), m
        if m > 40:
            assert col[5] == 3 and col[40] == 16440
    eng.close()


def _rollout(keep_logits, fused_call, shape, w, rope, prompts, cands, pol, steps):
    from paper_2508_18588_amd.runtime import Engine
    eng = Engine(shape, w, rope, max_batch=len(prompts), k_max=pol.k_max, c_max=len(cands[0]), max_len=64 + 200,
                 shuffle_pages_seed=9, keep_logits=keep_logits)
    eng.load_sequences(list(prompts), budgets=[150] * len(prompts))
    eng.set_history(cands)
    eng.prefill(list(prompts))
    trace = []
    for _ in range(steps):
        eng.draft(pol)
        eng.verify()
        if fused_call:
            eng.accept_commit(pol)
        else:
            eng.accept()
            eng.commit(pol)
        torch.cuda.synchronize()
        assert eng.poll_error() == 0
        m = int(eng.st["row_off"][len(prompts)])
        trace.append({k: np_of(eng.st[k]).copy() for k in ("row_off", "accept_len", "n_out", "out_tok", "path_row")}
                     | {"argmax": np_of(eng.st["argmax"])[:m].copy()})
    state = {k: np_of(getattr(eng, k)).copy() for k in ("seq_len", "tail", "tail_len", "k_state", "budget_left",
                                                        "tokens", "counters")}
    kv = (np_of(eng.kc).copy(), np_of(eng.vc).copy())
    eng.close()
    return trace, state, kv


@pytest.mark.parametrize("n_cand", [1, 2])
def test_no_logits_path_and_fused_accept_commit_equal_the_separate_launches(n_cand):
    """Toy configuration, chains and 2-branch trees (tree commit relocates K/V), adaptive draft length: 60 steps
    with (logits kept, three launches) and with (no logits, one launch) -- every step's argmax, acceptance, emitted
    tokens, and the final sequence state and cache are identical."""
    from paper_2508_18588_amd import HS_K_AIMD
    from paper_2508_18588_amd.runtime import Policy
    from test_gpu_decode import gpu_ar_rollout
    shape = CONFIG_SHAPES[1]          # vocabulary 4096 and d_model 256: the LM head does not split K
    w = make_weights(shape, config_seed(1))
    rope = rope_table(512, shape.head_dim)
    prompts = make_prompts(6, 64, shape.vocab, 88)
    rolls = gpu_ar_rollout(shape, w, rope, list(prompts), 150)
    pol = Policy(window=8, m_min=3, k_mode=HS_K_AIMD, k_max=8)
    c0 = make_histories(prompts, rolls, 8, 0.10, 0.02, shape.vocab, seed=5)
    c1 = make_histories(prompts, rolls, 8, 0.25, 0.0, shape.vocab, seed=6)
    cands = [[c0[b][0]] + ([c1[b][0]] if n_cand == 2 else []) for b in range(6)]
    ref = _rollout(True, False, shape, w, rope, prompts, cands, pol, 60)
    for keep, fused in ((False, True), (False, False), (True, True)):
        got = _rollout(keep, fused, shape, w, rope, prompts, cands, pol, 60)
        for s, (x, y) in enumerate(zip(ref[0], got[0])):
            for k in x:
                assert (x[k] == y[k]).all(), (keep, fused, s, k)
        for k in ref[1]:
            assert (ref[1][k] == got[1][k]).all(), (keep, fused, k)
        assert (ref[2][0] == got[2][0]).all() and (ref[2][1] == got[2][1]).all()
    assert sum(int(t["accept_len"].sum()) for t in ref[0]) > 60       # drafts were accepted


def test_rejection_sampling_without_logits_is_refused():
    from paper_2508_18588_amd import HS_ACCEPT_REJECTION, HS_ERR_INVALID_ARG, HS_FLAG_WORKSPACE_LOGITS, HsError
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = CONFIG_SHAPES[1]
    w = make_weights(shape, config_seed(1))
    prompts = make_prompts(2, 16, shape.vocab, 89)
    eng = Engine(shape, w, rope_table(128, shape.head_dim), max_batch=2, k_max=2, c_max=1, max_len=64,
                 keep_logits=False)
    eng.load_sequences(list(prompts), budgets=[8] * 2)
    eng.set_history([[np.zeros(0, np.int32)] for _ in range(2)])
    eng.prefill(list(prompts))
    pol = Policy(window=8, m_min=3, k_fixed=0, k_max=2)
    eng.draft(pol)
    eng.verify()
    with pytest.raises(HsError) as e:
        eng.accept(HS_ACCEPT_REJECTION, 1.0, 7)
    assert e.value.status == HS_ERR_INVALID_ARG and "logits" in str(e.value)
    eng.set_flags(HS_FLAG_WORKSPACE_LOGITS)      # the library keeps them in its workspace
    eng.verify()
    eng.accept_commit(pol, HS_ACCEPT_REJECTION, 1.0, 7)
    torch.cuda.synchronize()
    assert eng.poll_error() == 0 and np_of(eng.st["n_out"])[:2].tolist() == [1, 1]
    eng.close()
