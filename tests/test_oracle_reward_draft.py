"""Pins of the oracle's reward-aware draft over all responses of a prompt (Sec. 5.3 of the paper: one suffix tree
per prompt over the responses of its last rollout, a priority on every node = the sum of the rewards of the branch
below it, the highest-priority branch is followed).

The oracle states the rule on the flat responses (occurrences vote for their next token with their response's
reward).  It is pinned here against a literal construction of the paper's tree -- a trie of all suffixes whose
nodes carry the summed priorities -- walked the way the paper describes, against hand cases, and against the
single-response draft it must reduce to."""
import numpy as np
import pytest

import oracle


class Node:
    __slots__ = ("children", "prio", "count")

    def __init__(self):
        self.children, self.prio, self.count = {}, 0, 0


def build_suffix_trie(hists, rewards, depth):
    """Every suffix of every response (cut at `depth` tokens) is a root-to-leaf path; a leaf's priority is its
    response's reward and every node's priority the sum over the leaves below it (accumulated on the way down)."""
    root = Node()
    for h, r in zip(hists, rewards):
        for s in range(len(h)):
            node = root
            for t in h[s:s + depth]:
                node = node.children.setdefault(int(t), Node())
                node.prio += int(r)
                node.count += 1
    return root


def trie_draft(root, x, w, m_min, k):
    """Pattern length w shrinking to m_min until the pattern's node exists and has a continuation; then follow the
    child with the highest priority (more suffixes, then the smaller token id, on ties) for up to k tokens."""
    for m in range(min(w, len(x)), m_min - 1, -1):
        if m < 1:
            break
        node = root
        for t in x[len(x) - m:]:
            node = node.children.get(int(t))
            if node is None:
                break
        if node is None or not node.children:
            continue
        out = []
        while len(out) < k and node.children:
            tok, node = max(node.children.items(), key=lambda kv: (kv[1].prio, kv[1].count, -kv[0]))
            out.append(tok)
        return m, out
    return 0, []


@pytest.mark.parametrize("vocab,G,maxlen", [(2, 3, 14), (3, 4, 20), (4, 2, 24), (3, 1, 18), (6, 5, 30)])
def test_flat_vote_equals_walk_of_the_priority_tree(vocab, G, maxlen):
    rng = np.random.default_rng(100 + vocab * 10 + G)
    for trial in range(300):
        hists = [rng.integers(0, vocab, int(rng.integers(1, maxlen + 1))).astype(np.int32) for _ in range(G)]
        rewards = rng.integers(0, 3, G).astype(np.int32)
        x = rng.integers(0, vocab, int(rng.integers(1, 12))).astype(np.int32)
        w, m_min, k = int(rng.integers(2, 8)), int(rng.integers(1, 3)), int(rng.integers(1, 7))
        m_min = min(m_min, w)
        got = oracle.reward_draft(hists, rewards, x, w, m_min, k, occ_max=4096)
        m, toks = trie_draft(build_suffix_trie(hists, rewards, w + k), x, w, m_min, k)
        assert (got["m"], got["tok"].tolist()) == (m, toks), (trial, hists, rewards, x, w, m_min, k)
        if toks:
            h = hists[got["g"]]
            p = got["p"]
            assert h[p:p + len(toks)].tolist() == toks            # the draft is the text after a surviving occurrence
            assert h[p - m:p].tolist() == x[len(x) - m:].tolist()  # which follows the matched pattern


def test_reward_then_frequency_then_token_id_decide_a_branch():
    a, b, c, d, e, q, xx, y, z = range(1, 10)
    hists = [[a, b, c, d, e], [a, b, c, xx, z], [q, a, b, c, xx, y]]
    x = [7, a, b, c]
    r = oracle.reward_draft(hists, [1, 0, 0], x, 3, 3, 2)
    assert r["m"] == 3 and r["n_occ"] == 3 and r["tok"].tolist() == [d, e] and (r["g"], r["p"]) == (0, 3)
    r = oracle.reward_draft(hists, [0, 0, 0], x, 3, 3, 2)      # no reward anywhere: the more frequent continuation
    assert r["tok"].tolist() == [xx, y] and (r["g"], r["p"]) == (2, 4)   # then y < z by token id
    r = oracle.reward_draft(hists, [1, 2, 0], x, 3, 3, 2)      # sums: d = 1, xx = 2
    assert r["tok"].tolist() == [xx, z] and (r["g"], r["p"]) == (1, 3)
    r = oracle.reward_draft(hists, [1, 1, 0], x, 3, 3, 2)      # sums equal (1 vs 1): two votes beat one
    assert r["tok"].tolist() == [xx, z]


def test_walk_ends_where_the_history_ends_and_respects_the_cap():
    hists = [[5, 6, 7, 8], [5, 6, 7, 8, 9]]
    r = oracle.reward_draft(hists, [1, 1], [5, 6, 7], 3, 3, 8)
    assert r["tok"].tolist() == [8, 9]                          # the second response carries on one token further
    r = oracle.reward_draft(hists, [1, 1], [5, 6, 7], 3, 3, 8, occ_max=1)
    assert r["n_occ"] == 1 and r["tok"].tolist() == [8]         # only the first occurrence is kept
    assert oracle.reward_draft(hists, [1, 1], [1, 2, 3], 3, 3, 4)["tok"].size == 0
    # a pattern found only at the very end of a response has no continuation there: the shorter pattern is used
    r = oracle.reward_draft([[1, 2, 3], [9, 2, 3, 4]], [1, 1], [1, 2, 3], 3, 2, 4)
    assert r["m"] == 2 and r["tok"].tolist() == [4]


def test_single_response_with_one_occurrence_reduces_to_the_suffix_match_draft():
    rng = np.random.default_rng(7)
    for _ in range(100):
        V = 50000
        h = rng.integers(0, V, 400).astype(np.int32)
        s = int(rng.integers(10, 380))
        x = np.concatenate([rng.integers(0, V, 5), h[s - 6:s]]).astype(np.int32)
        p, m = oracle.suffix_match(h, x, 8, 3)
        r = oracle.reward_draft([h], [3], x, 8, 3, 6)
        assert (r["g"], r["p"], r["m"]) == (0, p, m) and r["tok"].tolist() == h[p:p + 6].tolist()
