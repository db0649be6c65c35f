"""Pins for the oracle's acceptance rules and its counter-based generator.

Greedy: Sec. 2.2 says verification keeps the valid draft tokens and preserves
the output, so the emitted tokens must equal plain autoregressive greedy
decoding -- checked by brute force over every draft of a tiny vocabulary and
end to end on a small decoder.  Stochastic: the output distribution must equal
softmax(logits / T) whatever the draft is -- checked by chi-square on small
vocabularies, by the closed form of the expected accepted length, and by the
T -> 0 limit.  Philox: published known-answer vectors.
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from hs_inputs import ModelShape, make_weights, rope_table, mutate, history_with_context


# ---------------------------------------------------------------- greedy

def fake_logits(context, V):
    """Table-driven stand-in for a model: logits depend on the last two tokens."""
    a = context[-1] if len(context) >= 1 else 0
    b = context[-2] if len(context) >= 2 else 0
    rng = np.random.default_rng(1000 + 37 * a + b)
    return rng.permutation(V).astype(np.float64)  # distinct values: no ties


def test_greedy_accept_equals_lcp_with_autoregressive_decode():
    V, K = 3, 4
    for prefix in ([0], [1, 2], [2, 2, 1]):
        # plain autoregressive greedy continuation
        ctx, g = list(prefix), []
        for _ in range(K + 1):
            g.append(int(np.argmax(fake_logits(ctx, V))))
            ctx.append(g[-1])
        for draft in itertools.product(range(V), repeat=K):
            lcp = 0
            while lcp < K and draft[lcp] == g[lcp]:
                lcp += 1
            tok = [prefix[-1]] + list(draft)
            parent = list(range(-1, K))
            arg = [int(np.argmax(fake_logits(list(prefix) + list(draft[:r]), V))) for r in range(K + 1)]
            a, out, path = oracle.accept_greedy(tok, parent, arg)
            assert a == lcp
            assert out.tolist() == g[:lcp + 1]
            assert path.tolist() == list(range(lcp + 1))


def test_greedy_accept_on_trees():
    V = 3
    prefix = [1, 0]
    ctx, g = list(prefix), []
    for _ in range(4):
        g.append(int(np.argmax(fake_logits(ctx, V))))
        ctx.append(g[-1])
    for c0 in itertools.product(range(V), repeat=3):
        for c1 in itertools.product(range(V), repeat=3):
            t = oracle.build_tree([list(c0), list(c1)], prefix[-1], 1)
            # path tokens of every node
            paths = []
            for r in range(len(t["tok"])):
                p, c = [], r
                while c > 0:
                    p.append(int(t["tok"][c]))
                    c = int(t["parent"][c])
                paths.append(p[::-1])
            arg = [int(np.argmax(fake_logits(prefix + p, V))) for p in paths]
            a, out, path = oracle.accept_greedy(t["tok"], t["parent"], arg)
            want = max(sum(1 for _ in itertools.takewhile(lambda ab: ab[0] == ab[1], zip(c, g))) for c in (c0, c1))
            assert a == want and out.tolist() == g[:want + 1]
            assert paths[int(path[-1])] == g[:want]


SHAPE = ModelShape(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=64)


def oracle_spec_rollout(model, prompt, hist, n_new, W, m_min, k_mode, k_fixed, k_max, cap):
    """Speculative greedy rollout made only of oracle pieces; returns (tokens, steps, accepted)."""
    seq = oracle.Seq(model, cap)
    x = list(prompt)
    seq.extend(x[:-1])
    k_state, steps, accepted = 2, 0, 0
    while len(x) - len(prompt) < n_new:
        budget = n_new - (len(x) - len(prompt))
        p, m = oracle.suffix_match(hist, x, W, m_min)
        K = oracle.draft_len(oracle.k_policy(k_mode, k_fixed, k_state, m, k_max), len(hist), p, budget)
        tree = oracle.build_tree([hist[p:p + K]] if K else [[]], x[-1], len(x) - 1)
        lg = seq.tree_logits(tree["tok"], tree["parent"])
        arg = [oracle.argmax(r) for r in lg]
        a, out, path = oracle.accept_greedy(tree["tok"], tree["parent"], arg)
        k_state = oracle.aimd(k_state, K > 0, a == K)
        seq.extend([x[-1]] + out[:a].tolist())
        x.extend(out.tolist())
        steps += 1
        accepted += a
    return x[len(prompt):], steps, accepted


def test_bruteforce_greedy_accept_is_autoregressive_decode_plus_longest_prefix():
    """orc_accept_greedy_bruteforce on the real decoder: its emitted tokens are the plain autoregressive greedy
    continuation (oracle.ar_greedy, a separate loop), its accepted length the longest prefix of that continuation
    that the draft tree spells out (computed here from the token lists) -- and the one-pass rule (each node's argmax
    compared with its children) gives the same answer.  Chains and 2-branch trees, drafts built to agree with the
    continuation for 0..K tokens."""
    w = make_weights(SHAPE, seed=6, std=0.3)
    model = oracle.Model(SHAPE, w, rope_table(64, SHAPE.head_dim))
    rng = np.random.default_rng(3)
    prompt = rng.integers(0, SHAPE.vocab, 9).astype(np.int32)
    seq = oracle.Seq(model, 40)
    seq.extend(prompt[:-1])
    g = oracle.ar_greedy(seq, prompt[-1], 7)
    seq.truncate(len(prompt) - 1)
    other = lambda t: (t + 1) % SHAPE.vocab
    for agree0 in range(0, 6):
        for agree1 in range(0, 6):
            c0 = [g[i] if i < agree0 else other(g[i]) for i in range(5)]
            c1 = [g[i] if i < agree1 else other(other(g[i])) for i in range(5)]
            for chains in ([c0], [c0, c1]):
                t = oracle.build_tree(chains, int(prompt[-1]), len(prompt) - 1)
                a, out, path = seq.accept_greedy_bruteforce(t["tok"], t["parent"])
                assert len(seq) == len(prompt) - 1
                want = min(5, max(agree0, agree1 if len(chains) == 2 else 0))
                assert a == want and out.tolist() == g[:want + 1]
                lg = seq.tree_logits(t["tok"], t["parent"], plain=True)
                a1, out1, path1 = oracle.accept_greedy(t["tok"], t["parent"], [oracle.argmax(r) for r in lg])
                assert (a1, out1.tolist(), path1.tolist()) == (a, out.tolist(), path.tolist())


@pytest.mark.parametrize("k_mode", [oracle.K_FIXED, oracle.K_MATCHLEN, oracle.K_AIMD])
def test_speculative_greedy_equals_autoregressive_greedy(k_mode):
    w = make_weights(SHAPE, seed=5, std=0.3)
    rope = rope_table(256, SHAPE.head_dim)
    model = oracle.Model(SHAPE, w, rope)
    rng = np.random.default_rng(9)
    prompt = rng.integers(0, SHAPE.vocab, 12).astype(np.int32)
    n_new = 60
    seq = oracle.Seq(model, 128)
    seq.extend(prompt[:-1])
    ar = oracle.ar_greedy(seq, prompt[-1], n_new)
    hist = history_with_context(prompt, mutate(np.array(ar, np.int32), 0.1, 0.05, SHAPE.vocab, rng), 8)
    got, steps, accepted = oracle_spec_rollout(model, prompt, hist, n_new, 8, 3, k_mode, 4, 16, 128)
    assert got == ar
    assert accepted > 0 and steps < n_new  # the draft path was really exercised


# ------------------------------------------------------------ stochastic

def test_philox_known_answers(golden_dir):
    n = 0
    for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]
        n += 1
    assert n == 3


def test_philox_batch_is_the_generator_per_counter_and_a_bijection(golden_dir):
    """The bulk form equals the single-counter form (which carries the published known answers), and -- a keyed
    bijection of the counter space -- maps 2^16 distinct counters to 2^16 distinct outputs."""
    kat = [[int(t, 16) for t in line.split()] for line in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
           if line.strip() and not line.startswith("#")]
    for v in kat:
        assert oracle.philox_batch(np.array([v[0:4]], np.uint32), v[4:6])[0].tolist() == v[6:10]
    rng = np.random.default_rng(5)
    ctr = rng.integers(0, 2 ** 32, (2000, 4), dtype=np.uint64).astype(np.uint32)
    key = [0xDEADBEEF, 0x12345678]
    out = oracle.philox_batch(ctr, key)
    for i in range(0, 2000, 97):
        assert out[i].tolist() == oracle.philox4x32_10(ctr[i].tolist(), key)
    grid = np.zeros((1 << 16, 4), np.uint32)
    grid[:, 0] = np.arange(1 << 16) & 0xFF
    grid[:, 1] = np.arange(1 << 16) >> 8
    o = oracle.philox_batch(grid, key)
    assert len({tuple(r) for r in o.tolist()}) == 1 << 16


def test_uniform_layout_and_range():
    # top 24 bits of output word 0 with counter (position, kind, seq_id lo, hi) and key = seed
    seed, sid, pos, kind = 0x0123456789ABCDEF, 0xFEDCBA9876543210, 4242, 7
    w0 = oracle.philox4x32_10([pos, kind, sid & 0xFFFFFFFF, sid >> 32], [seed & 0xFFFFFFFF, seed >> 32])[0]
    assert oracle.uniform(seed, sid, pos, kind) == (w0 >> 8) / 2.0 ** 24
    u = np.array([oracle.uniform(1, 2, p, 0) for p in range(20000)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.005
    assert len(set(u.tolist())) > 19900  # distinct counters -> distinct draws (up to 24-bit collisions)


def chi2_ok(counts, probs, n):
    exp = probs * n
    keep = exp > 5
    chi2 = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    dof = keep.sum() - 1
    return chi2 < dof + 6 * np.sqrt(2 * dof) + 6  # ~6 sigma


def softmax(x, T=1.0):
    e = np.exp((x - x.max()) / T)
    return e / e.sum()


@pytest.mark.parametrize("chains", [[[2, 5, 1]], [[2, 5, 1], [2, 0, 3]], [[2, 5], [4, 1]]])
def test_stochastic_output_distribution_is_the_models(chains):
    V, T, N = 6, 0.8, 120000
    rng = np.random.default_rng(3)
    tree = oracle.build_tree(chains, 0, 10)
    n = len(tree["tok"])
    logits = rng.normal(size=(n, V)) * 1.5
    first = np.zeros(V)
    second_after = {}  # node accepted first -> counts of the second emitted token
    acc_hist = np.zeros(8)
    for s in range(N):
        a, out, path, _ = oracle.accept_stochastic(tree["tok"], tree["parent"], tree["pos"], logits, T, 77, s)
        first[out[0]] += 1
        acc_hist[a] += 1
        if a >= 1:
            second_after.setdefault(int(path[1]), np.zeros(V))[out[1]] += 1
    # the first emitted token follows softmax(root logits / T) regardless of the draft
    assert chi2_ok(first, softmax(logits[0], T), N)
    # given the first draft token was accepted, the next emitted token follows that node's distribution
    for node, cnt in second_after.items():
        assert chi2_ok(cnt, softmax(logits[node], T), cnt.sum())
    # a draft token is accepted exactly as often as the model would have produced it
    for c in range(1, n):
        if tree["parent"][c] == 0:
            p = softmax(logits[0], T)[tree["tok"][c]]
            got = sum(cnt.sum() for node, cnt in second_after.items() if node == c) / N
            assert abs(got - p) < 6 * np.sqrt(p * (1 - p) / N) + 1e-4


def test_expected_accept_length_closed_form():
    V, T, N = 5, 1.0, 100000
    rng = np.random.default_rng(4)
    chain = [1, 3, 0, 2]
    tree = oracle.build_tree([chain], 4, 0)
    logits = rng.normal(size=(5, V)) * 2
    total = sum(oracle.accept_stochastic(tree["tok"], tree["parent"], tree["pos"], logits, T, 5, s)[0]
                for s in range(N))
    ps = [softmax(logits[j], T)[chain[j]] for j in range(4)]
    want = sum(np.prod(ps[:j + 1]) for j in range(4))
    var_bound = 4.0
    assert abs(total / N - want) < 6 * np.sqrt(var_bound / N)


def test_low_temperature_limit_is_greedy():
    V = 7
    rng = np.random.default_rng(6)
    for trial in range(200):
        c0 = rng.integers(0, V, 3).tolist()
        c1 = rng.integers(0, V, 3).tolist()
        tree = oracle.build_tree([c0, c1], 0, 5)
        logits = rng.permutation(V * len(tree["tok"])).reshape(len(tree["tok"]), V).astype(np.float64)
        arg = [int(np.argmax(r)) for r in logits]
        g = oracle.accept_greedy(tree["tok"], tree["parent"], arg)
        s = oracle.accept_stochastic(tree["tok"], tree["parent"], tree["pos"], logits, 1e-3, 1, trial)
        assert s[0] == g[0] and s[1].tolist() == g[1].tolist() and s[2].tolist() == g[2].tolist()


def test_inverse_cdf_order_and_residual():
    # one draft child carrying token 1; probabilities 0.1, 0.6, 0.3.  If the child is rejected the final draw
    # comes from (0.25, 0, 0.75) by cumulative order of token id.
    logits = np.log(np.array([[0.1, 0.6, 0.3], [1 / 3, 1 / 3, 1 / 3]]))
    tok, par, pos = [9, 1], [-1, 0], [20, 21]
    seen = {0: 0, 2: 0}
    for s in range(4000):
        u_acc = oracle.uniform(3, s, 21, 0)
        a, out, path, _ = oracle.accept_stochastic(tok, par, pos, logits, 1.0, 3, s)
        assert (a >= 1) == (u_acc < 0.6)
        if a == 0:
            u_fin = oracle.uniform(3, s, 21, 7)
            assert out[0] == (0 if u_fin * 0.4 <= 0.1 else 2)
            seen[int(out[0])] += 1
    assert seen[0] > 0 and seen[2] > 0
