"""Pins for the oracle's draft step (suffix match, K policy, AIMD window, tree merge).

Each check compares the oracle with something that is not the oracle: a brute
force written here from the definition, the second formulation the paper
gives (pattern length backing off 7 -> 3, Sec. 5.4), closed-form special
cases, or the window trace Sec. 5.4 fixes.
"""
import itertools
import os

import numpy as np

import oracle
from hs_inputs import mutate, history_with_context


def brute_match(hist, x, w, m_min):
    """All (p, m) by direct comparison; pick max m, then min p."""
    best = (-1, 0)
    for p in range(1, len(hist)):
        m = 0
        for j in range(1, min(w, p, len(x)) + 1):
            if hist[p - j] == x[len(x) - j]:
                m = j
            else:
                break
        if m >= m_min and m > best[1]:
            best = (p, m)
    return best


def test_match_brute_force_tiny_alphabets():
    rng = np.random.default_rng(1)
    for trial in range(1500):
        V = int(rng.integers(2, 5))
        lh = int(rng.integers(0, 48))
        n = int(rng.integers(0, 24))
        w = int(rng.integers(1, 10))
        m_min = int(rng.integers(1, w + 1))
        hist = rng.integers(0, V, lh).astype(np.int32)
        x = rng.integers(0, V, n).astype(np.int32)
        assert oracle.suffix_match(hist, x, w, m_min) == brute_match(hist, x, w, m_min), (trial, hist, x, w, m_min)


def test_backoff_formulation_equals_longest_capped_match():
    # Sec. 5.4: start with the longest pattern, shorten until one occurs == longest match capped at W.
    rng = np.random.default_rng(2)
    for _ in range(1500):
        V = int(rng.integers(2, 6))
        hist = rng.integers(0, V, int(rng.integers(0, 64))).astype(np.int32)
        x = rng.integers(0, V, int(rng.integers(0, 20))).astype(np.int32)
        assert oracle.suffix_match(hist, x, 7, 3) == oracle.suffix_match(hist, x, 7, 3, backoff=True)


def test_match_special_cases():
    rng = np.random.default_rng(3)
    V = 150000
    r = rng.integers(0, V, 400).astype(np.int32)
    # history identical to the current text: after n tokens the match ends at p = n with m = W
    for n in (8, 50, 399):
        assert oracle.suffix_match(r, r[:n], 8, 3) == (n, 8)
    # fewer tokens than the minimum -> nothing
    assert oracle.suffix_match(r, r[:2], 8, 3) == (-1, 0)
    # fresh random tokens over a large vocabulary -> nothing
    assert oracle.suffix_match(r, rng.integers(0, V, 100).astype(np.int32), 8, 3) == (-1, 0)
    # a match that ends exactly at the history's end leaves no token to draft -> not eligible
    assert oracle.suffix_match(r[:100], r[:100], 8, 3) == (-1, 0)
    # planted unique 5-gram
    x = np.concatenate([rng.integers(0, V, 30), r[200:205]]).astype(np.int32)
    assert oracle.suffix_match(r, x, 8, 3) == (205, 5)
    # leftmost among equal-length matches
    pat = np.array([7, 8, 9], np.int32)
    hist = np.concatenate([[1, 2], pat, [3, 4], pat, [5, 6]]).astype(np.int32)
    assert oracle.suffix_match(hist, pat, 8, 3) == (5, 3)
    # ... but a longer match further right wins
    hist2 = np.concatenate([[1, 2], pat, [3, 4, 11], pat, [5, 6]]).astype(np.int32)
    assert oracle.suffix_match(hist2, np.array([11, 7, 8, 9], np.int32), 8, 3) == (11, 4)


def test_match_at_response_start_uses_prompt_context():
    rng = np.random.default_rng(4)
    prompt = rng.integers(0, 1000, 64).astype(np.int32)
    resp = rng.integers(0, 1000, 128).astype(np.int32)
    W = 8
    hist = history_with_context(prompt, resp, W)
    # no response token yet: the prompt's last W-1 tokens anchor the draft on the first response token
    p, m = oracle.suffix_match(hist, prompt, W, 3)
    assert (p, m) == (W - 1, W - 1)
    assert hist[p] == resp[0]


def test_trace_sim_against_brute_force():
    # Sec. 5.1 routine, restated here: key of 3 replayed tokens; longest identical following run counts.
    def sim(cur, hist, key=3):
        acc, i = 0, 0
        while i < len(cur):
            best = 0
            if i >= key:
                for p in range(key, len(hist)):
                    if list(hist[p - key:p]) == list(cur[i - key:i]):
                        run = 0
                        while p + run < len(hist) and i + run < len(cur) and hist[p + run] == cur[i + run]:
                            run += 1
                        best = max(best, run)
            if best:
                acc += best
                i += best
            else:
                i += 1
        return acc

    rng = np.random.default_rng(5)
    for _ in range(40):
        V = int(rng.integers(3, 50))
        cur = rng.integers(0, V, int(rng.integers(1, 80))).astype(np.int32)
        hist = mutate(cur, 0.2, 0.05, V, rng)
        assert oracle.trace_sim(cur, hist, 3) == sim(cur, hist)
    # identical history: everything after the first key tokens is accepted
    cur = np.arange(100, dtype=np.int32)
    assert oracle.trace_sim(cur, cur, 3) == 97


def test_run_length_shape_of_mutated_history():
    # Sec. 5.4 / Fig. "hit lengths": short identical runs dominate by count, long ones by total length.
    rng = np.random.default_rng(6)
    r = rng.integers(0, 150000, 20000).astype(np.int32)
    h = mutate(r, 0.2, 0.0, 150000, rng)
    same = (r == h).astype(np.int8)
    runs = [len(list(g)) for k, g in itertools.groupby(same) if k == 1]
    runs = np.array(runs)
    assert (runs <= 2).sum() > (runs >= 8).sum()          # short runs: more of them
    assert runs[runs >= 3].sum() > runs[runs <= 2].sum()  # long runs: more tokens in them


def test_k_policy_and_truncation():
    K_FIXED, K_MATCHLEN, K_AIMD = oracle.K_FIXED, oracle.K_MATCHLEN, oracle.K_AIMD
    assert oracle.k_policy(K_FIXED, 4, 0, 5, 32) == 4
    assert oracle.k_policy(K_FIXED, 4, 0, 0, 32) == 0          # no match -> no draft
    assert [oracle.k_policy(K_MATCHLEN, 0, 0, m, 16) for m in (3, 7, 16, 20)] == [3, 7, 16, 16]
    assert oracle.k_policy(K_AIMD, 0, 6, 3, 32) == 6
    assert oracle.k_policy(K_AIMD, 0, 40, 3, 32) == 32
    assert oracle.draft_len(8, 100, 95, 1000) == 5             # history end
    assert oracle.draft_len(8, 100, 10, 4) == 3                # budget: one token always comes from the model
    assert oracle.draft_len(8, 100, 10, 1) == 0
    assert oracle.draft_len(8, 100, -1, 1000) == 0


def test_aimd_trace(golden_dir):
    want = [int(t) for line in open(os.path.join(golden_dir, "aimd_window_trace.txt"))
            if not line.startswith("#") for t in line.split()]
    k, got = 2, [2]
    for step in range(18):
        full = step < 17
        k = oracle.aimd(k, True, full)
        got.append(k)
    assert got == want
    assert oracle.aimd(10, False, False) == 10  # no draft made: window unchanged


def test_tree_merge():
    # two chains sharing a 2-token prefix
    t = oracle.build_tree([[5, 6, 7, 8], [5, 6, 9, 10, 11]], root_tok=1, l_cached=100)
    assert t["tok"].tolist() == [1, 5, 6, 7, 8, 9, 10, 11]
    assert t["parent"].tolist() == [-1, 0, 1, 2, 3, 2, 5, 6]
    assert t["pos"].tolist() == [100, 101, 102, 103, 104, 103, 104, 105]
    # ancestor masks from the parent chain, computed independently
    for r in range(8):
        m, c = 0, r
        while c >= 0:
            m |= 1 << c
            c = t["parent"][c]
        assert int(t["anc_mask"][r]) == m
    # identical chains collapse, a prefix chain adds nothing, disjoint chains fork at the root
    assert oracle.build_tree([[5, 6], [5, 6]], 1, 0)["tok"].tolist() == [1, 5, 6]
    assert oracle.build_tree([[5, 6, 7], [5, 6]], 1, 0)["tok"].tolist() == [1, 5, 6, 7]
    assert oracle.build_tree([[5], [6]], 1, 0)["parent"].tolist() == [-1, 0, 0]
    assert oracle.build_tree([[], [6, 7]], 1, 3)["pos"].tolist() == [3, 4, 5]
    # chain = degenerate tree
    c = oracle.build_tree([[4, 4, 4]], 9, 10)
    assert c["parent"].tolist() == [-1, 0, 1, 2] and [int(x) for x in c["anc_mask"]] == [1, 3, 7, 15]
