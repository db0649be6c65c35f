"""Pins for the oracle's target-model forward pass (Sec. 2.2: one forward pass yields the logits).

The oracle pushes one token at a time through scalar loops with an explicit
K/V cache.  It is pinned against (i) the same decoder written as whole-sequence
matrix algebra with PyTorch CPU library routines in float64 (matmul, softmax,
a causal mask) -- a structurally different program; (ii) closed forms for
special weights; (iii) properties any correct implementation has (relative-
position property of the rotary embedding, prefix invariance, GQA head
sharing).
"""
import numpy as np
import pytest
import torch

import oracle
from hs_inputs import ModelShape, make_weights, rope_table, bf16_to_f32

SHAPE = ModelShape(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=50)


def torch_decoder_logits(shape, w, rope, tokens):
    """Whole-sequence causal decoder, float64 library ops.  Returns [T, V]."""
    f = lambda a: torch.from_numpy(bf16_to_f32(a).astype(np.float64))
    T = len(tokens)
    hq, hkv, h = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    x = f(w["embed"])[torch.tensor(tokens, dtype=torch.long)]
    cos = torch.from_numpy(rope[:T, :, 0].astype(np.float64))
    sin = torch.from_numpy(rope[:T, :, 1].astype(np.float64))

    def norm(x, g):
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + shape.rms_eps) * torch.from_numpy(g.astype(np.float64))

    def rot(t):  # [T, H, h]
        a, b = t[..., :h // 2], t[..., h // 2:]
        c, s = cos[:, None, :], sin[:, None, :]
        return torch.cat([a * c - b * s, b * c + a * s], -1)

    mask = torch.full((T, T), float("-inf"), dtype=torch.float64).triu(1)
    for l in range(len(w["wqkv"])):
        qkv = norm(x, w["norm1"][l]) @ f(w["wqkv"][l]).T
        q = rot(qkv[:, :hq * h].reshape(T, hq, h))
        k = rot(qkv[:, hq * h:(hq + hkv) * h].reshape(T, hkv, h))
        v = qkv[:, (hq + hkv) * h:].reshape(T, hkv, h)
        k = k.repeat_interleave(hq // hkv, dim=1)
        v = v.repeat_interleave(hq // hkv, dim=1)
        s = torch.einsum("thd,shd->hts", q, k) / np.sqrt(h) + mask
        o = torch.einsum("hts,shd->thd", torch.softmax(s, -1), v).reshape(T, hq * h)
        x = x + o @ f(w["wo"][l]).T
        n2 = norm(x, w["norm2"][l])
        x = x + (torch.nn.functional.silu(n2 @ f(w["wgate"][l]).T) * (n2 @ f(w["wup"][l]).T)) @ f(w["wdown"][l]).T
    return (norm(x, w["norm_f"]) @ f(w["lm_head"]).T).numpy()


@pytest.fixture(scope="module")
def small():
    w = make_weights(SHAPE, seed=11, norm_jitter=0.1, std=0.2)  # large std: attention and FFN terms matter
    rope = rope_table(64, SHAPE.head_dim)
    return w, rope, oracle.Model(SHAPE, w, rope)


def test_forward_matches_library_decoder(small):
    w, rope, model = small
    rng = np.random.default_rng(0)
    tokens = rng.integers(0, SHAPE.vocab, 23).tolist()
    seq = oracle.Seq(model, 64)
    got = np.stack([seq.push(t) for t in tokens])
    want = torch_decoder_logits(SHAPE, w, rope, tokens)
    assert np.abs(want).max() > 0.5  # non-trivial logits
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-10)


def test_each_term_is_live(small):
    # zeroing any one weight group must change the logits: guards against a silently dropped term
    w, rope, model = small
    tokens = [3, 9, 27, 31, 4]
    base = oracle.Seq(model, 16).extend(tokens)
    for name in ("wqkv", "wo", "wgate", "wup", "wdown"):
        w2 = dict(w)
        w2[name] = [np.zeros_like(a) for a in w[name]]
        other = oracle.Seq(oracle.Model(SHAPE, w2, rope), 16).extend(tokens)
        assert np.abs(other - base).max() > 1e-3, name


def test_closed_form_without_mixing(small):
    # with Wo = Wdown = 0 the residual stream is the embedding: logits = Wlm . RMSNorm(E[tok])
    w, rope, _ = small
    w2 = dict(w)
    w2["wo"] = [np.zeros_like(a) for a in w["wo"]]
    w2["wdown"] = [np.zeros_like(a) for a in w["wdown"]]
    model = oracle.Model(SHAPE, w2, rope)
    seq = oracle.Seq(model, 8)
    seq.push(5, want_logits=False)
    got = seq.push(17)
    e = bf16_to_f32(w["embed"][17]).astype(np.float64)
    n = e / np.sqrt((e * e).mean() + SHAPE.rms_eps) * w["norm_f"].astype(np.float64)
    want = bf16_to_f32(w["lm_head"]).astype(np.float64) @ n
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-13)


def test_first_position_attention_is_value(small):
    # one key: softmax is 1, so attention returns V itself (and position 0 has cos=1, sin=0: no rotation)
    w, rope, model = small
    seq = oracle.Seq(model, 4)
    seq.push(7, want_logits=False)
    e = bf16_to_f32(w["embed"][7]).astype(np.float64)
    n1 = e / np.sqrt((e * e).mean() + SHAPE.rms_eps) * w["norm1"][0].astype(np.float64)
    qkv = bf16_to_f32(w["wqkv"][0]).astype(np.float64) @ n1
    hq, hkv, h = SHAPE.n_q_heads, SHAPE.n_kv_heads, SHAPE.head_dim
    k, v = seq.kv(0, 0)
    np.testing.assert_allclose(k, qkv[hq * h:(hq + hkv) * h], rtol=1e-12)
    np.testing.assert_allclose(v, qkv[(hq + hkv) * h:], rtol=1e-12)


def test_attention_row_is_softmax_average():
    rng = np.random.default_rng(1)
    q, k, v = rng.normal(size=8), rng.normal(size=(13, 8)), rng.normal(size=(13, 8))
    s = torch.softmax(torch.from_numpy(k @ q * 0.3), 0).numpy()
    np.testing.assert_allclose(oracle.attention_row(q, k, v, 0.3), s @ v, rtol=1e-12)
    # uniform keys -> plain mean of the values
    np.testing.assert_allclose(oracle.attention_row(q, np.ones((5, 8)), v[:5], 1.0), v[:5].mean(0), rtol=1e-12)


def test_rope_relative_position_property(small):
    # cached K at position p is R(p) k: inner products between two rotated copies of the same vectors depend
    # only on the position difference.  Feed the same token at every position of a 1-layer model and compare
    # K[p].K[p+3] across p (layer 0's K depends only on the token, not on context).
    w, rope, model = small
    seq = oracle.Seq(model, 40)
    for _ in range(30):
        seq.push(12, want_logits=False)
    ks = np.stack([seq.kv(0, p)[0] for p in range(30)])
    h = SHAPE.head_dim
    k0 = ks[:, :h]
    d = [k0[p] @ k0[p + 3] for p in range(20)]
    np.testing.assert_allclose(d, d[0], rtol=1e-6)       # table is fp32: tolerance of its rounding
    np.testing.assert_allclose([np.linalg.norm(x) for x in k0], np.linalg.norm(k0[0]), rtol=1e-6)  # rotations
    assert abs(k0[0] @ k0[3] - k0[0] @ k0[0]) > 1e-6     # ... and it does rotate


def test_prefix_invariance_and_truncate(small):
    # logits at a position depend only on the tokens up to it; truncating and re-pushing reproduces them
    _, _, model = small
    a = [1, 2, 3, 4, 5, 6, 7]
    s1 = oracle.Seq(model, 16)
    l1 = [s1.push(t) for t in a]
    s2 = oracle.Seq(model, 16)
    l2 = [s2.push(t) for t in a[:4] + [40, 41]]
    for i in range(4):
        np.testing.assert_array_equal(l1[i], l2[i])
    s2.truncate(4)
    np.testing.assert_array_equal(s2.push(a[4]), l1[4])


def test_tree_logits_equal_plain_sequences(small):
    _, _, model = small
    prefix = [4, 8, 15, 16, 23]
    tree = oracle.build_tree([[42, 7, 9], [42, 11, 3]], root_tok=prefix[-1], l_cached=len(prefix) - 1)
    seq = oracle.Seq(model, 32)
    seq.extend(prefix[:-1])
    lg = seq.tree_logits(tree["tok"], tree["parent"], plain=True)
    assert len(seq) == len(prefix) - 1
    paths = {0: [], 1: [42], 2: [42, 7], 3: [42, 7, 9], 4: [42, 11], 5: [42, 11, 3]}
    for r, extra in paths.items():
        want = oracle.Seq(model, 32).extend(prefix + extra)
        np.testing.assert_array_equal(lg[r], want)
    # the shared-prefix walk (used where long chains are followed) gives the same bits, on this tree, on a chain
    # and on a tree whose second branch forks at the root
    np.testing.assert_array_equal(seq.tree_logits(tree["tok"], tree["parent"]), lg)
    assert len(seq) == len(prefix) - 1
    for chains in ([[5, 6, 7, 8, 9, 10]], [[1, 2, 3], [4, 5, 6]], [[]]):
        t = oracle.build_tree(chains, root_tok=prefix[-1], l_cached=len(prefix) - 1)
        np.testing.assert_array_equal(seq.tree_logits(t["tok"], t["parent"]),
                                      seq.tree_logits(t["tok"], t["parent"], plain=True))


def test_loaded_cache_reproduces_computed_cache(small):
    _, _, model = small
    a = [9, 8, 7, 6, 5, 4]
    s1 = oracle.Seq(model, 16)
    for t in a[:4]:
        s1.push(t, want_logits=False)
    k = np.stack([[s1.kv(l, p)[0] for p in range(4)] for l in range(SHAPE.n_layers)])
    v = np.stack([[s1.kv(l, p)[1] for p in range(4)] for l in range(SHAPE.n_layers)])
    s2 = oracle.Seq(model, 16)
    s2.load_kv(k, v)
    assert len(s2) == 4
    np.testing.assert_array_equal(s2.push(a[4]), s1.push(a[4]))
    np.testing.assert_array_equal(s2.push(a[5]), s1.push(a[5]))


def test_argmax_lowest_id_on_ties():
    assert oracle.argmax(np.array([1.0, 3.0, 3.0, 2.0])) == 1
    assert oracle.argmax(np.array([5.0])) == 0


def test_residual_trace_is_the_truncated_models_hidden_state(small):
    """The inspection hook returns the residual stream after the embedding and after every layer: row 0 is the
    token's embedding, and row l is exactly what a decoder made of the first l layers feeds its final norm -- so the
    logits of that shorter model (computed by a separate oracle instance) are lm_head . RMSNorm(row l)."""
    w, rope, model = small
    toks = [3, 17, 42, 8, 29]
    s = oracle.Seq(model, 16)
    s.extend(toks[:-1])
    logits, h = s.push_traced(toks[-1])
    f = lambda a: bf16_to_f32(a).astype(np.float64)
    np.testing.assert_array_equal(h[0], f(w["embed"])[toks[-1]])

    def head(x):
        n = x / np.sqrt((x * x).mean() + SHAPE.rms_eps) * w["norm_f"].astype(np.float64)
        return f(w["lm_head"]) @ n

    np.testing.assert_allclose(head(h[-1]), logits, rtol=1e-12, atol=1e-12)
    assert np.abs(h[1] - h[0]).max() > 1e-3 and np.abs(h[2] - h[1]).max() > 1e-3
    for l in (1,):
        wl = {k: (v[:l] if isinstance(v, list) else v) for k, v in w.items()}
        short = oracle.Seq(oracle.Model(SHAPE, wl, rope), 16)
        short.extend(toks[:-1])
        np.testing.assert_allclose(head(h[l]), short.push(toks[-1]), rtol=1e-12, atol=1e-12)
    # the hook is off again: a later push leaves the buffer alone
    before = h.copy()
    s.push(5)
    np.testing.assert_array_equal(h, before)
