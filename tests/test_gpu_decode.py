"""GPU parity of the whole decode iteration (hs_draft -> hs_verify -> hs_accept -> hs_kv_commit) against the
oracle, in lock-step: both sides hold the same committed tokens; each iteration the oracle recomputes the logits
of exactly the rows the GPU verified.  Bars: integer outputs (draft, accept length, state) bit-exact; logits
within 2e-2 absolute; emitted tokens identical wherever the oracle's top-2 logit margin exceeds that tolerance
(positions below it are counted and the oracle follows the GPU's token there so the comparison can go on)."""
import numpy as np
import pytest
import torch

import oracle
from hs_inputs import (CONFIG_SHAPES, ModelShape, make_weights, rope_table, make_prompts, config_seed, mutate,
                       history_with_context)
from gpu_common import LOGIT_TOL, OracleBatch, check_cache, make_histories, np_of, top2_margin

pytestmark = pytest.mark.gpu


def lockstep(eng, ob, cands, pol, max_steps, check_kv_layers=(), gate=None, tol=LOGIT_TOL, rel_tol=None,
             bruteforce=False):
    """Run until every budget is spent.  Returns statistics.  gate: the oracle's copy of the speculation gate's
    words (the engine holds its own); the oracle decides each step from the oracle-side totals, and a step it
    switches off must come out of the HIP path as one row per live sequence.  tol: absolute logit tolerance;
    rel_tol: if given, additionally max|dlogit| of a row <= rel_tol * max|logit| of that row.
    bruteforce: the GPU's acceptance is also compared with acceptance by definition (the oracle decodes
    autoregressively from the same state and takes the longest prefix the draft tree spells out)."""
    import dataclasses
    B = len(ob.x)
    stats = dict(steps=0, accepted=0, emitted=0, flagged=0, max_logit_err=0.0, max_rel_err=0.0, rows=0, drafted=0,
                 off_steps=0, positions=0, margin_below_tol=0)
    pol_on = pol
    pol_off = dataclasses.replace(pol, k_mode=oracle.K_FIXED, k_fixed=0)
    for _ in range(max_steps):
        if all(b <= 0 for b in ob.budget):
            break
        if gate is not None:
            live = sum(b > 0 for b in ob.budget)
            on = oracle.gate_step(gate, live, stats["drafted"], stats["accepted"])
            pol = pol_on if on else pol_off
            stats["off_steps"] += not on
        eng.step(pol_on)
        torch.cuda.synchronize()
        assert eng.poll_error() == 0
        st = {k: np_of(v) for k, v in eng.st.items()}
        lg = np_of(eng.logits)
        ro = st["row_off"]
        for b in range(B):
            info, tree = ob.draft(b, cands[b], pol)
            C = len(cands[b])
            for c in range(C):
                got = (st["draft_start"][b * C + c], st["match_len"][b * C + c], st["draft_len"][b * C + c])
                assert got == info[c], (b, c, got, info[c])
            if tree is None:
                assert ro[b + 1] == ro[b] and st["n_out"][b] == 0
                continue
            sl = slice(ro[b], ro[b + 1])
            assert st["tok"][sl].tolist() == tree["tok"].tolist()
            assert st["parent"][sl].tolist() == tree["parent"].tolist()
            want = ob.logits(b, tree)
            err = float(np.abs(lg[sl] - want).max())
            stats["max_logit_err"] = max(stats["max_logit_err"], err)
            assert err <= tol, (b, err)
            rel = float((np.abs(lg[sl] - want).max(1) / np.abs(want).max(1)).max())
            stats["max_rel_err"] = max(stats["max_rel_err"], rel)
            if rel_tol is not None:
                assert rel <= rel_tol, (b, rel)
            stats["positions"] += len(want)
            stats["margin_below_tol"] += sum(top2_margin(r) <= tol for r in want)
            # the GPU's argmax must be the argmax of its own logits (lowest id on ties)
            assert st["argmax"][sl].tolist() == [int(np.argmax(r)) for r in lg[sl]]
            # oracle decision on oracle logits vs GPU decision; the GPU's walk must also be the greedy walk of
            # its own argmax
            arg_o = [oracle.argmax(r) for r in want]
            a_o, out_o, path_o = oracle.accept_greedy(tree["tok"], tree["parent"], arg_o)
            a_g, out_g, path_g = oracle.accept_greedy(tree["tok"], tree["parent"], st["argmax"][sl])
            n = st["n_out"][b]
            assert st["accept_len"][b] == a_g and n == a_g + 1
            assert st["out_tok"][b, :n].tolist() == out_g.tolist()
            assert st["path_row"][b, :n].tolist() == path_g.tolist()
            if bruteforce:
                a_b, out_b, path_b = ob.seqs[b].accept_greedy_bruteforce(tree["tok"], tree["parent"])
                assert (a_b, out_b.tolist(), path_b.tolist()) == (a_o, out_o.tolist(), path_o.tolist())
                stats["bruteforce_checked"] = stats.get("bruteforce_checked", 0) + 1
                stats["bruteforce_equal"] = stats.get("bruteforce_equal", 0) + int(
                    (a_b, out_b.tolist(), path_b.tolist()) == (a_g, out_g.tolist(), path_g.tolist()))
            if out_g.tolist() != out_o.tolist():
                # allowed only where a visited row's top-2 margin is within the logit tolerance
                visited = set(path_o.tolist()) | set(path_g.tolist())
                assert min(top2_margin(want[r]) for r in visited) <= tol, (b, out_g, out_o)
                stats["flagged"] += 1
            ob.commit(b, tree, a_g, out_g, path_g, pol_on)   # the oracle follows the GPU's tokens
            stats["accepted"] += a_g
            stats["emitted"] += int(n)
            stats["rows"] += len(tree["tok"])
            stats["drafted"] += len(tree["tok"]) - 1
        # state after commit
        assert np_of(eng.seq_len)[:B].tolist() == [len(x) for x in ob.x]
        assert np_of(eng.budget_left)[:B].tolist() == ob.budget
        tail, tl = np_of(eng.tail), np_of(eng.tail_len)
        for b in range(B):
            m = min(len(ob.x[b]), eng.w_max)
            assert tl[b] == m and tail[b, eng.w_max - m:].tolist() == ob.x[b][-m:]
        if pol_on.k_mode == oracle.K_AIMD:
            assert np_of(eng.k_state)[:B].tolist() == ob.k_state
        if gate is not None:
            assert np_of(eng.gate).tolist() == gate.tolist()
            c = np_of(eng.counters)
            assert (int(c[1]), int(c[2])) == (stats["drafted"], stats["accepted"])
            if not on:
                assert int(ro[B]) == live and not st["draft_len"][:B * len(cands[0])].any()
        stats["steps"] += 1
    toks = np_of(eng.tokens)
    for b in range(B):
        assert toks[b, :len(ob.x[b])].tolist() == ob.x[b]
    for layer in check_kv_layers:
        check_cache(eng, ob, layer, tol=tol, rtol=2e-2 if rel_tol is None else 10 * rel_tol)
    return stats


def setup_rollout(shape, w, rope, B, prompt_len, n_new, seed):
    model = oracle.Model(shape, w, rope)
    prompts = make_prompts(B, prompt_len, shape.vocab, seed)
    rollouts = []
    for b in range(B):
        s = oracle.Seq(model, prompt_len + n_new + 8)
        s.extend(prompts[b][:-1])
        rollouts.append(oracle.ar_greedy(s, prompts[b][-1], n_new))
    return model, prompts, rollouts


def gpu_ar_rollout(shape, w, rope, toks, n_new):
    """The HIP path's own plain autoregressive greedy rollout (no drafts): the text a previous epoch would have
    produced with unchanged weights."""
    from paper_2508_18588_amd.runtime import Engine, Policy
    B = len(toks)
    pol = Policy(window=8, m_min=3, k_fixed=0, k_max=0)
    eng = Engine(shape, w, rope, max_batch=B, k_max=0, c_max=1, max_len=max(len(t) for t in toks) + n_new)
    eng.load_sequences(toks, budgets=[n_new] * B)
    eng.set_history([[np.zeros(0, np.int32)] for _ in range(B)])
    eng.prefill(toks)
    for _ in range(n_new):
        eng.step(pol)
    out = np_of(eng.tokens)
    eng.close()
    return [out[b, len(toks[b]):len(toks[b]) + n_new].copy() for b in range(B)]


@pytest.fixture(scope="module")
def config1():
    shape = CONFIG_SHAPES[1]
    seed = config_seed(1)
    w = make_weights(shape, seed)
    rope = rope_table(512, shape.head_dim)
    model, prompts, rollouts = setup_rollout(shape, w, rope, 4, 64, 256, seed)
    return shape, w, rope, model, prompts, rollouts


@pytest.mark.parametrize("reference_kernels", [True, False])
def test_config1_full_rollout_lockstep(config1, reference_kernels):
    """Configuration 1 in full: B=4, prompt 64, 256-token greedy rollout, history = the oracle's rollout with 10 %
    of positions replaced, window 8, K=4, greedy, pages of 16."""
    from paper_2508_18588_amd import HS_FLAG_REFERENCE_KERNELS
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape, w, rope, model, prompts, rollouts = config1
    pol = Policy(window=8, m_min=3, k_fixed=4, k_max=4)
    cands = make_histories(prompts, rollouts, 8, 0.10, 0.0, shape.vocab, seed=77)
    eng = Engine(shape, w, rope, max_batch=4, k_max=4, c_max=1, max_len=64 + 256, shuffle_pages_seed=5)
    if reference_kernels:
        eng.set_flags(HS_FLAG_REFERENCE_KERNELS)
    eng.load_sequences(list(prompts), budgets=[256] * 4)
    eng.set_history(cands)
    eng.prefill(list(prompts))
    ob = OracleBatch(model, list(prompts), [256] * 4, 64 + 256 + 8)
    stats = lockstep(eng, ob, cands, pol, max_steps=300, check_kv_layers=(0, 1))
    eng.close()
    print("config1", "plain" if reference_kernels else "mfma", stats)
    assert stats["emitted"] == 4 * 256
    assert stats["accepted"] > 40             # speculation really happened (until a near-tie leaves the history)
    assert stats["flagged"] <= 24
    # where nothing was flagged the output is the oracle's own autoregressive greedy rollout
    if stats["flagged"] == 0:
        for b in range(4):
            assert ob.x[b][64:] == rollouts[b]


@pytest.mark.parametrize("mode", ["matchlen", "aimd"])
def test_adaptive_draft_lengths_lockstep(config1, mode):
    """Variable K per sequence (match-length policy, and the AIMD window 2,+2,cap,reset), ragged prompts and
    budgets, one sequence finishing early."""
    from paper_2508_18588_amd import HS_K_AIMD, HS_K_MATCHLEN
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape, w, rope, model, prompts, rollouts = config1
    if mode == "matchlen":
        pol = Policy(window=16, m_min=3, k_mode=HS_K_MATCHLEN, k_max=16)
    else:
        pol = Policy(window=7, m_min=3, k_mode=HS_K_AIMD, k_max=32)
    lens = [64, 37, 50, 21]
    toks = [prompts[b][64 - lens[b]:] for b in range(4)]
    rolls = gpu_ar_rollout(shape, w, rope, toks, 120)
    cands = make_histories(toks, rolls, pol.window, 0.05, 0.03, shape.vocab, seed=78)
    budgets = [120, 60, 120, 9]
    eng = Engine(shape, w, rope, max_batch=4, k_max=pol.k_max, c_max=1, max_len=64 + 130, shuffle_pages_seed=6)
    eng.load_sequences(toks, budgets)
    eng.set_history(cands)
    eng.prefill(toks)
    ob = OracleBatch(model, toks, budgets, 64 + 140 + 40)
    stats = lockstep(eng, ob, cands, pol, max_steps=200, check_kv_layers=(1,))
    eng.close()
    print(mode, stats)
    assert stats["emitted"] == sum(budgets)
    assert stats["rows"] > 2 * stats["steps"]   # drafts longer than a token were verified
    assert stats["flagged"] <= 6


def test_speculative_equals_autoregressive_bitwise_on_gpu(config1):
    """Sec. 2.2: speculation must not change the output.  The GPU path keeps every reduction order independent of
    how many rows share a launch, so the greedy token streams with and without drafts are identical."""
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape, w, rope, model, prompts, rollouts = config1
    rolls = gpu_ar_rollout(shape, w, rope, list(prompts), 256)
    cands = make_histories(prompts, rolls, 8, 0.10, 0.02, shape.vocab, seed=79)
    outs = []
    for k in (0, 4):
        pol = Policy(window=8, m_min=3, k_fixed=k, k_max=4)
        eng = Engine(shape, w, rope, max_batch=4, k_max=4, c_max=1, max_len=64 + 256, shuffle_pages_seed=7 + k)
        eng.load_sequences(list(prompts), budgets=[256] * 4)
        eng.set_history(cands)
        eng.prefill(list(prompts))
        steps = 0
        while int(eng.budget_left.max()) > 0:
            eng.step(pol)
            steps += 1
        outs.append((np_of(eng.tokens)[:, :64 + 256].copy(), steps, np_of(eng.counters).copy()))
        eng.close()
    assert (outs[0][0] == outs[1][0]).all()
    for b in range(4):
        assert outs[0][0][b, 64:].tolist() == rolls[b].tolist()
    assert outs[0][1] == 256 and outs[1][1] < 200
    assert outs[0][2][2] == 0 and outs[1][2][2] > 300   # accepted-token counters


@pytest.mark.parametrize("k_mode", ["fixed", "aimd"])
def test_speculation_gate_lockstep(config1, k_mode):
    """Throughput-aware speculation control (Sec. 5.4, last paragraph): histories that are accurate for the first
    80 tokens and 40 % wrong afterwards, ragged budgets.  The gate's table lets speculation run at any rate once one
    sequence is left, and for up to four only from rate bucket 10 (62 %) on; it probes every 5 steps.  Every word of
    the gate, every decision and the rows of every step must equal the oracle's."""
    from paper_2508_18588_amd import HS_K_AIMD, HS_K_FIXED
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape, w, rope, model, prompts, rollouts = config1
    rng = np.random.default_rng(4242)
    cands = []
    for b in range(4):
        r = np.asarray(rollouts[b], np.int32)
        h = np.concatenate([mutate(r[:80], 0.03, 0.0, shape.vocab, rng), mutate(r[80:], 0.40, 0.0, shape.vocab, rng)])
        cands.append([history_with_context(prompts[b], h, 8)])
    pol = Policy(window=8, m_min=2, k_mode=HS_K_AIMD if k_mode == "aimd" else HS_K_FIXED, k_fixed=4, k_max=8,
                 aimd_cap=8)
    budgets = [256, 200, 150, 110]
    table = [1] * 10 + [4] * 7
    eng = Engine(shape, w, rope, max_batch=4, k_max=8, c_max=1, max_len=64 + 256, shuffle_pages_seed=11)
    eng.load_sequences(list(prompts), budgets=budgets)
    eng.set_history(cands)
    eng.prefill(list(prompts))
    eng.set_gate(table, probe_every=5)
    gate = np.zeros(32, np.int32)
    gate[4] = 5
    gate[8:25] = table
    ob = OracleBatch(model, list(prompts), budgets, 64 + 256 + 16)
    stats = lockstep(eng, ob, cands, pol, max_steps=600, gate=gate)
    eng.close()
    print("gate", k_mode, stats, gate[:8].tolist())
    assert stats["emitted"] == sum(budgets)
    assert 20 <= stats["off_steps"] <= stats["steps"] - 20      # both states were held for a while
    assert stats["accepted"] > 40


def test_tree_drafts_two_candidates_lockstep(config1):
    """Two history candidates per sequence (two prior epochs) merged into a draft tree of depth 8, verified with
    the ancestor mask, greedy acceptance, accepted nodes of the second branch relocated by the commit."""
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape, w, rope, model, prompts, rollouts = config1
    pol = Policy(window=8, m_min=3, k_fixed=8, k_max=8)
    rolls = gpu_ar_rollout(shape, w, rope, list(prompts), 128)
    h0 = make_histories(prompts, rolls, 8, 0.40, 0.0, shape.vocab, seed=80)
    h1 = make_histories(prompts, rolls, 8, 0.25, 0.0, shape.vocab, seed=81)
    cands = [[h0[b][0], h1[b][0]] for b in range(4)]
    eng = Engine(shape, w, rope, max_batch=4, k_max=8, c_max=2, max_len=64 + 128, shuffle_pages_seed=9)
    eng.load_sequences(list(prompts), budgets=[128] * 4)
    eng.set_history(cands)
    eng.prefill(list(prompts))
    ob = OracleBatch(model, list(prompts), [128] * 4, 64 + 128 + 24)
    stats = lockstep(eng, ob, cands, pol, max_steps=200, check_kv_layers=(0, 1))
    eng.close()
    print("tree", stats)
    assert stats["emitted"] == 4 * 128 and stats["flagged"] <= 6
    assert stats["rows"] > 9 * stats["steps"]   # forks occurred: more than one chain's worth of rows


def test_gqa_head_dim_128_small_model():
    """A small decoder with the large configurations' attention geometry (grouped queries 6:1... head_dim 128)."""
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = ModelShape(n_layers=2, d_model=384, n_q_heads=6, n_kv_heads=1, head_dim=128, d_ffn=640, vocab=1024)
    w = make_weights(shape, 31, norm_jitter=0.1)
    rope = rope_table(4096, shape.head_dim)
    model = oracle.Model(shape, w, rope)
    prompts = make_prompts(3, 40, shape.vocab, 32)
    rollouts = gpu_ar_rollout(shape, w, rope, list(prompts), 80)
    pol = Policy(window=8, m_min=3, k_fixed=8, k_max=8)
    cands = make_histories(prompts, rollouts, 8, 0.1, 0.0, shape.vocab, seed=82)
    eng = Engine(shape, w, rope, max_batch=3, k_max=8, c_max=1, max_len=40 + 80, shuffle_pages_seed=10)
    eng.load_sequences(list(prompts), budgets=[80] * 3)
    eng.set_history(cands)
    eng.prefill(list(prompts))
    ob = OracleBatch(model, list(prompts), [80] * 3, 40 + 80 + 16)
    stats = lockstep(eng, ob, cands, pol, max_steps=100, check_kv_layers=(1,))
    eng.close()
    print("gqa128", stats)
    assert stats["emitted"] == 240 and stats["accepted"] > 60 and stats["flagged"] <= 6


def test_batch_of_300_ragged_sequences_mixed_unit_kinds():
    """More sequences than one block of the device-side list builders handles at once (256), three KV heads (the
    wavefronts of a workgroup then straddle partitions), contexts of 2..700 tokens (1..3 partitions of 256 keys),
    finished sequences in between, and drafts of up to 12 tokens next to sequences that draft nothing: units for
    single wavefronts and units for workgroups in one launch.  The cache comes from hs_prefill (its row builder also
    walks the batch in blocks).  Three decode steps in lock-step with the oracle."""
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = ModelShape(n_layers=2, d_model=384, n_q_heads=9, n_kv_heads=3, head_dim=64, d_ffn=512, vocab=512)
    w = make_weights(shape, 51, norm_jitter=0.1)
    rope = rope_table(1024, shape.head_dim)
    model = oracle.Model(shape, w, rope)
    rng = np.random.default_rng(52)
    B = 300
    lens = rng.integers(2, 701, B)
    toks = [rng.integers(0, shape.vocab, int(n)).astype(np.int32) for n in lens]
    budgets = [0 if b % 7 == 3 else 20 for b in range(B)]
    # history: for two sequences in three the true continuation is not known (no match -> one row); for the others
    # a planted copy of the text's last tokens followed by 12 tokens makes hs_draft take a 12-token draft
    cands = []
    for b in range(B):
        if b % 3 == 0:
            cands.append([np.concatenate([toks[b][-6:], rng.integers(0, shape.vocab, 12)]).astype(np.int32)])
        else:
            cands.append([np.zeros(0, np.int32)])
    pol = Policy(window=6, m_min=3, k_fixed=12, k_max=12)
    eng = Engine(shape, w, rope, max_batch=B, k_max=12, c_max=1, max_len=int(lens.max()) + 24, shuffle_pages_seed=53)
    eng.load_sequences(toks, budgets=budgets)
    eng.set_history(cands)
    eng.prefill_chunked(64)
    ob = OracleBatch(model, toks, budgets, int(lens.max()) + 40)
    stats = lockstep(eng, ob, cands, pol, max_steps=3)
    eng.close()
    print("batch300", stats)
    live = sum(b > 0 for b in budgets)
    assert stats["steps"] == 3 and stats["emitted"] >= 3 * live
    assert stats["rows"] > 3 * live + 900          # the planted drafts were taken (12 extra rows each, first step)


@pytest.mark.gpu
@pytest.mark.parametrize("head_dim", [64, 128])
def test_workgroup_attention_units_with_one_to_four_live_row_tiles(head_dim):
    """Drafts of 4..32 tokens on 4 query heads per KV head: 20..132 query rows per KV head, i.e. streamed wavefront
    units next to workgroup units with two, three and four live row tiles and, for the longest draft, a second unit
    of one tile -- every staging split of the workgroup path (wavefronts that only stage K/V next to those that
    compute) -- over contexts of 1..11 tiles of 128 keys with ragged ends.  Two decode steps in lock-step with the
    oracle."""
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = ModelShape(n_layers=2, d_model=256, n_q_heads=8, n_kv_heads=2, head_dim=head_dim, d_ffn=384, vocab=512)
    w = make_weights(shape, 61, norm_jitter=0.1)
    rope = rope_table(2048, shape.head_dim)
    model = oracle.Model(shape, w, rope)
    rng = np.random.default_rng(62 + head_dim)
    draft_lens = [4, 8, 12, 16, 22, 27, 32, 0]
    B = 24
    lens = rng.integers(100, 1400, B)
    toks = [rng.integers(0, shape.vocab, int(n)).astype(np.int32) for n in lens]
    budgets = [40] * B
    cands = []
    for b in range(B):
        k = draft_lens[b % len(draft_lens)]
        if k:   # a copy of the text's last tokens followed by k tokens: hs_draft takes exactly k (the history ends)
            cands.append([np.concatenate([toks[b][-6:], rng.integers(0, shape.vocab, k)]).astype(np.int32)])
        else:
            cands.append([np.zeros(0, np.int32)])
    pol = Policy(window=6, m_min=3, k_fixed=32, k_max=32)
    eng = Engine(shape, w, rope, max_batch=B, k_max=32, c_max=1, max_len=int(lens.max()) + 80, shuffle_pages_seed=63)
    eng.load_sequences(toks, budgets=budgets)
    eng.set_history(cands)
    eng.prefill_chunked(128)
    ob = OracleBatch(model, toks, budgets, int(lens.max()) + 120)
    stats = lockstep(eng, ob, cands, pol, max_steps=2)
    eng.close()
    print("live-tiles", head_dim, stats)
    assert stats["steps"] == 2
    assert stats["rows"] >= B + 3 * sum(draft_lens)      # every planted draft was taken in the first step


def test_split_and_serial_gemm_execution_agree_bitwise():
    """The narrow projections cut K into a fixed number of chunks; with few rows each chunk runs in its own
    workgroup and an ordered reduce adds them, with many rows one workgroup folds the chunks itself.  Both must
    give the same bits (the row hint is a launch-shape hint only), and both must match the oracle."""
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = ModelShape(n_layers=2, d_model=1024, n_q_heads=8, n_kv_heads=2, head_dim=128, d_ffn=2048, vocab=2048)
    w = make_weights(shape, 41)
    rope = rope_table(1024, shape.head_dim)
    model = oracle.Model(shape, w, rope)
    prompts = make_prompts(4, 33, shape.vocab, 42)
    rollouts = gpu_ar_rollout(shape, w, rope, list(prompts), 40)
    pol = Policy(window=8, m_min=3, k_fixed=6, k_max=6)
    cands = make_histories(prompts, rollouts, 8, 0.1, 0.0, shape.vocab, seed=83)
    results = []
    for hint in (1, 100000):
        eng = Engine(shape, w, rope, max_batch=4, k_max=6, c_max=1, max_len=33 + 40, shuffle_pages_seed=11)
        eng.set_rows_hint(hint)
        eng.load_sequences(list(prompts), budgets=[40] * 4)
        eng.set_history(cands)
        eng.prefill(list(prompts))
        if hint == 1:
            ob = OracleBatch(model, list(prompts), [40] * 4, 33 + 40 + 16)
            stats = lockstep(eng, ob, cands, pol, max_steps=60, check_kv_layers=(0, 1))
            print("split-gemm", stats)
            assert stats["emitted"] == 160 and stats["accepted"] > 40
        else:
            while int(eng.budget_left.max()) > 0:
                eng.step(pol)
        torch.cuda.synchronize()
        results.append((np_of(eng.tokens).copy(), np_of(eng.logits).copy(), np_of(eng.kc).copy(), np_of(eng.vc).copy()))
        eng.close()
    for a, b in zip(*results):
        assert (a == b).all()


def test_whole_step_replayed_from_a_hip_graph_equals_eager_steps(config1):
    """One decode iteration (draft, verify, accept + commit) recorded into a HIP graph: the row count lives on the
    device, so the same graph serves every step.  40 replays, each followed by a synchronisation and eager reads,
    against an engine that runs the same steps eagerly: rows, argmax, acceptance and emitted tokens of every step, and
    the final sequence state and cache, are identical."""
    from paper_2508_18588_amd import HS_K_AIMD
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape, w, rope, model, prompts, rollouts = config1
    pol = Policy(window=8, m_min=3, k_mode=HS_K_AIMD, k_max=8)
    cands = make_histories(prompts, rollouts, 8, 0.10, 0.02, shape.vocab, seed=91)
    engs = []
    for _ in range(2):
        eng = Engine(shape, w, rope, max_batch=4, k_max=8, c_max=1, max_len=64 + 256, shuffle_pages_seed=8,
                     keep_logits=False)
        eng.load_sequences(list(prompts), budgets=[200] * 4)
        eng.set_history(cands)
        eng.prefill(list(prompts))
        eng.set_rows_hint(12)
        for _ in range(3):
            eng.step(pol)
        engs.append(eng)
    eager, replayed = engs
    graph = replayed.capture_step(pol)
    keys = ("row_off", "tok", "parent", "argmax", "accept_len", "n_out", "out_tok", "path_row")
    emitted = 0
    for s in range(40):
        eager.step(pol)
        graph.replay()
        torch.cuda.synchronize()
        assert replayed.poll_error() == 0
        m = int(eager.st["row_off"][4])
        for k in keys:
            a, b = np_of(eager.st[k]), np_of(replayed.st[k])
            if k in ("tok", "parent", "argmax"):
                a, b = a[:m], b[:m]
            assert (a == b).all(), (s, k)
        emitted += int(np_of(eager.st["n_out"]).sum())
    for k in ("seq_len", "tail", "tail_len", "k_state", "budget_left", "tokens", "counters"):
        assert (np_of(getattr(eager, k)) == np_of(getattr(replayed, k))).all(), k
    assert (np_of(eager.kc) == np_of(replayed.kc)).all() and (np_of(eager.vc) == np_of(replayed.vc)).all()
    assert emitted > 4 * 40        # drafts were accepted along the way
    for e in engs:
        e.close()
