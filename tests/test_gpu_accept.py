"""GPU parity of hs_accept in rejection-sampling mode (and greedy mode on given logits) against the oracle.

The acceptance rule is speculative sampling with a point-mass draft (Sec. 2.2 of the paper: the verified tokens
that are valid are kept and the output distribution is preserved).  Both sides get the SAME fp32 logits, the same
seed, sequence ids and positions, so every decision (accepted path, emitted tokens) must be identical; the only
admissible differences are decisions whose uniform lies within rounding distance of its threshold, which the
oracle reports as a margin.  The Philox stream is thereby checked bit for bit as well: one wrong uniform changes
a decision somewhere in thousands of draws."""
import numpy as np
import pytest
import torch

import oracle
from hs_inputs import CONFIG_SHAPES, make_weights, rope_table, make_prompts, config_seed
from gpu_common import LOGIT_TOL, OracleBatch, make_histories, np_of

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def toy():
    shape = CONFIG_SHAPES[1]
    return shape, make_weights(shape, seed=1), rope_table(4096, shape.head_dim)


def random_trees(rng, B, k_max, vocab, two):
    trees = []
    for b in range(B):
        k0 = int(rng.integers(0, k_max + 1))
        c0 = rng.integers(0, vocab, k0)
        chains = [c0]
        if two:
            k1 = int(rng.integers(0, k_max + 1))
            share = int(rng.integers(0, min(k0, k1) + 1))
            chains.append(np.concatenate([c0[:share], rng.integers(0, vocab, k1 - share)]))
        L = int(rng.integers(0, 3000))
        trees.append(oracle.build_tree(chains, int(rng.integers(0, vocab)), L))
    return trees


@pytest.mark.parametrize("two,temperature", [(False, 1.0), (True, 1.0), (True, 0.6)])
def test_rejection_accept_matches_oracle_on_given_logits(toy, two, temperature):
    from paper_2508_18588_amd import HS_ACCEPT_GREEDY, HS_ACCEPT_REJECTION
    from paper_2508_18588_amd.runtime import Engine
    shape, w, rope = toy
    V, B, k_max = shape.vocab, 48, 8
    temperature = float(np.float32(temperature))   # the C ABI carries the temperature as fp32
    rng = np.random.default_rng(5 + int(two) + int(temperature * 10))
    eng = Engine(shape, w, rope, max_batch=B, k_max=k_max, c_max=2, max_len=3200)
    eng.load_sequences([np.array([1], np.int32)] * B, budgets=[100] * B,
                       seq_ids=rng.integers(0, 2 ** 62, B).astype(np.int64))
    seq_ids = np_of(eng.seq_id)[:B].astype(np.uint64)
    n_acc, n_flag, n_dec = 0, 0, 0
    for trial in range(6):
        trees = random_trees(rng, B, k_max, V, two)
        m = eng.set_rows([dict(tok=t["tok"], parent=t["parent"], pos=t["pos"]) for t in trees])
        # peaked synthetic logits: every node's children get a boost so that about half of the drafts are accepted
        lg = rng.normal(0.0, 2.0, size=(m, V)).astype(np.float32)
        r = 0
        for t in trees:
            n = len(t["tok"])
            for i in range(1, n):
                lg[r + t["parent"][i], t["tok"][i]] += rng.choice([0.0, 6.0, 9.0, 12.0])
            r += n
        eng.logits[:m].copy_(torch.from_numpy(lg))
        seed = int(rng.integers(0, 2 ** 63))
        eng.accept(HS_ACCEPT_REJECTION, temperature, seed)
        torch.cuda.synchronize()
        st = {k: np_of(v) for k, v in eng.st.items()}
        r = 0
        for b, t in enumerate(trees):
            n = len(t["tok"])
            a, out, path, margin = oracle.accept_stochastic(t["tok"], t["parent"], t["pos"],
                                                            lg[r:r + n].astype(np.float64), temperature, seed,
                                                            int(seq_ids[b]))
            got = (int(st["accept_len"][b]), st["out_tok"][b, :st["n_out"][b]].tolist(),
                   st["path_row"][b, :st["n_out"][b]].tolist())
            n_dec += 1
            if got != (a, out.tolist(), path.tolist()):
                assert margin < 1e-9, (trial, b, got, (a, out.tolist(), path.tolist()), margin)
                n_flag += 1
            assert st["n_out"][b] == st["accept_len"][b] + 1
            n_acc += a
            r += n
        # greedy mode on the same logits: walk of the per-row argmax (argmax supplied as hs_verify would)
        arg = lg[:m].argmax(1).astype(np.int32)
        eng.st["argmax"][:m].copy_(torch.from_numpy(arg))
        eng.accept(HS_ACCEPT_GREEDY)
        torch.cuda.synchronize()
        st = {k: np_of(v) for k, v in eng.st.items()}
        r = 0
        for b, t in enumerate(trees):
            n = len(t["tok"])
            a, out, path = oracle.accept_greedy(t["tok"], t["parent"], arg[r:r + n])
            assert st["accept_len"][b] == a and st["out_tok"][b, :a + 1].tolist() == out.tolist()
            assert st["path_row"][b, :a + 1].tolist() == path.tolist()
            r += n
    eng.close()
    print("rejection accept: decisions", n_dec, "accepted tokens", n_acc, "flagged", n_flag)
    assert n_acc > 50 and n_flag <= 2


def test_finished_and_empty_sequences(toy):
    """Sequences without rows (budget spent) must report n_out = 0 in both modes."""
    from paper_2508_18588_amd import HS_ACCEPT_GREEDY, HS_ACCEPT_REJECTION
    from paper_2508_18588_amd.runtime import Engine
    shape, w, rope = toy
    eng = Engine(shape, w, rope, max_batch=3, k_max=2, c_max=1, max_len=64)
    eng.load_sequences([np.array([1, 2], np.int32)] * 3, budgets=[5, 0, 5])
    t = oracle.build_tree([[7, 8]], 2, 1)
    eng.set_rows([dict(tok=t["tok"], parent=t["parent"], pos=t["pos"]), None,
                  dict(tok=t["tok"][:1], parent=t["parent"][:1], pos=t["pos"][:1])])
    eng.logits.zero_()
    eng.logits[0, 7] = 50.0   # certain accept of the first draft token
    eng.logits[1, 3] = 50.0   # then certain rejection of 8: token 3 has all the mass
    eng.logits[3, 9] = 50.0
    for mode in (HS_ACCEPT_REJECTION, HS_ACCEPT_GREEDY):
        eng.st["argmax"][:4].copy_(torch.tensor([7, 3, 0, 9], dtype=torch.int32))
        eng.accept(mode, 1.0, 123)
        torch.cuda.synchronize()
        assert np_of(eng.st["n_out"]).tolist() == [2, 0, 1]
        assert np_of(eng.st["out_tok"])[0, :2].tolist() == [7, 3]
        assert np_of(eng.st["out_tok"])[2, 0] == 9
    eng.close()


@pytest.mark.parametrize("precise", [False, True])
def test_tree_rejection_sampling_end_to_end(toy, precise):
    """Two history candidates per sequence, tree-mask verify, rejection sampling at a low temperature (so that
    drafts are accepted with a useful probability), tree commit -- in lock-step with the oracle: logits within the
    tolerance every step.  Default path: the GPU's decisions equal the oracle's rule applied to the GPU's own logits.
    fp32-activation mode: the logits agree to 1e-4 relative, and the GPU's decisions equal the oracle's rule applied
    to the ORACLE's own logits -- the whole stochastic step end to end against an independent computation (a decision
    may differ only where the oracle reports a uniform within 1e-4 of its threshold)."""
    from paper_2508_18588_amd import HS_ACCEPT_REJECTION
    from paper_2508_18588_amd.runtime import Engine, Policy
    from test_gpu_decode import gpu_ar_rollout, check_cache
    shape = CONFIG_SHAPES[1]
    seed = config_seed(5)
    w = make_weights(shape, seed)
    rope = rope_table(512, shape.head_dim)
    model = oracle.Model(shape, w, rope)
    prompts = make_prompts(4, 48, shape.vocab, seed)
    rolls = gpu_ar_rollout(shape, w, rope, list(prompts), 96)
    h0 = make_histories(prompts, rolls, 8, 0.40, 0.0, shape.vocab, seed=90)
    h1 = make_histories(prompts, rolls, 8, 0.60, 0.0, shape.vocab, seed=91)
    cands = [[h0[b][0], h1[b][0]] for b in range(4)]
    pol = Policy(window=8, m_min=3, k_fixed=8, k_max=8)
    T, pseed = float(np.float32(0.02)), 0xABCDEF12345
    eng = Engine(shape, w, rope, max_batch=4, k_max=8, c_max=2, max_len=48 + 96, shuffle_pages_seed=12,
                 precise=precise)
    sids = [11, 2 ** 40 + 5, 7, 2 ** 62 + 1]
    eng.load_sequences(list(prompts), budgets=[96] * 4, seq_ids=sids)
    eng.set_history(cands)
    eng.prefill(list(prompts))
    ob = OracleBatch(model, list(prompts), [96] * 4, 48 + 96 + 24)
    accepted = steps = flagged = 0
    while any(b > 0 for b in ob.budget) and steps < 200:
        eng.draft(pol)
        eng.verify()
        eng.accept(HS_ACCEPT_REJECTION, T, pseed)
        torch.cuda.synchronize()
        st = {k: np_of(v) for k, v in eng.st.items()}
        lg = np_of(eng.logits)
        eng.commit(pol)
        ro = st["row_off"]
        for b in range(4):
            info, tree = ob.draft(b, cands[b], pol)
            if tree is None:
                assert st["n_out"][b] == 0
                continue
            sl = slice(ro[b], ro[b + 1])
            assert st["tok"][sl].tolist() == tree["tok"].tolist()
            assert st["pos"][sl].tolist() == tree["pos"].tolist()
            want = ob.logits(b, tree)
            assert np.abs(lg[sl] - want).max() <= LOGIT_TOL
            if precise:
                assert (np.abs(lg[sl] - want).max(1) <= 1e-4 * np.abs(want).max(1)).all()
            a, out, path, margin = oracle.accept_stochastic(tree["tok"], tree["parent"], tree["pos"],
                                                            want if precise else lg[sl].astype(np.float64), T, pseed,
                                                            sids[b])
            n = st["n_out"][b]
            got = (int(st["accept_len"][b]), st["out_tok"][b, :n].tolist(), st["path_row"][b, :n].tolist())
            near = 1e-4 if precise else 1e-9
            flagged += got != (a, out.tolist(), path.tolist())
            assert got == (a, out.tolist(), path.tolist()) or margin < near, (b, got, a, out, path, margin)
            ob.commit(b, tree, got[0], np.array(got[1]), np.array(got[2]), pol)
            accepted += got[0]
        steps += 1
    torch.cuda.synchronize()
    assert np_of(eng.seq_len)[:4].tolist() == [len(x) for x in ob.x]
    toks = np_of(eng.tokens)
    for b in range(4):
        assert toks[b, :len(ob.x[b])].tolist() == ob.x[b]
    for layer in (0, 1):
        check_cache(eng, ob, layer)
    eng.close()
    print("tree rejection e2e: precise", precise, "steps", steps, "accepted", accepted, "near-threshold", flagged)
    assert flagged <= 2
    assert accepted > 5   # sampling soon leaves the greedy history; the draft path was still exercised


def test_philox_words_equal_the_oracles_on_a_million_counters():
    """The generator itself, GPU against the oracle, bit for bit: all four output words of 2^20 counters -- the
    counter layouts hs_accept uses (position, draw kind 0..7, 64-bit sequence ids) and fully random 128-bit counters
    -- under three keys."""
    import oracle
    from paper_2508_18588_amd import hs_debug_philox
    rng = np.random.default_rng(31)
    n = 1 << 20
    ctr = rng.integers(0, 2 ** 32, (n, 4), dtype=np.uint64).astype(np.uint32)
    half = n // 2
    ctr[:half, 0] = rng.integers(0, 40000, half)      # positions
    ctr[:half, 1] = rng.integers(0, 8, half)          # draw kinds
    ctr[0] = 0
    ctr[1] = 0xFFFFFFFF
    d_ctr = torch.from_numpy(ctr.view(np.int32)).cuda()
    d_out = torch.empty_like(d_ctr)
    for seed in (0, 0xC0FFEE05 * 0x9E3779B1 & (2 ** 63 - 1), 2 ** 64 - 1):
        hs_debug_philox(d_ctr.data_ptr(), seed, d_out.data_ptr(), n, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        got = d_out.cpu().numpy().view(np.uint32)
        want = oracle.philox_batch(ctr, [seed & 0xFFFFFFFF, seed >> 32])
        assert (got == want).all(), seed
