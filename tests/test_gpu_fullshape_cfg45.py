"""Parity at the real shapes and launch configurations of benchmark configurations 4 and 5, where the oracle cannot
run the whole model over the whole batch: two layers of the shape, the full batch, and sampled outputs recomputed
by the oracle one by one (attention rows from the GPU's own queries and cache, LM-head logits as fp64 dot products),
plus the integer parts in full (draft trees, acceptance, commit).

Configuration 4: 7B shape, 256 sequences with lognormal response lengths (median 4000, sigma 0.8, clipped to
[512, 32768]) after a 512-token prompt, adaptive draft length up to 32 (33 query positions per sequence: seven
row tiles per KV head), greedy acceptance, AIMD window update.
Configuration 5: 14B shape, 64 sequences at context 8192, two history candidates per sequence forming a 2-branch
draft tree of depth 8 (tree-mask attention), rejection sampling at temperature 1 with Philox uniforms, tree commit.

Inputs are synthetic and seeded; the K/V of the context is random with the scale a prefill would write."""
import numpy as np
import pytest
import torch

import oracle
from hs_inputs import CONFIG_SHAPES, config_seed, lengths_lognormal
from hs_inputs.device import fill_kv_random, make_weights_device, rope_device
from gpu_common import check_last_layer_projections, np_of

pytestmark = pytest.mark.gpu


def bf16_bits_to_f64(t):
    return (np_of(t).view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def seq_kv(eng, layer, b, j, n_slots):
    """K and V of KV head j of sequence b, slots [0, n_slots), as fp64 [n_slots, h] arrays read from the cache."""
    shape = eng.shape
    hkv, h = shape.n_kv_heads, shape.head_dim
    kc = eng.kc.view(eng.n_layers, eng.n_blocks, hkv, 16, h)
    vc = eng.vc.view(eng.n_layers, eng.n_blocks, hkv, h, 16)
    bt = np_of(eng.block_table)
    pages = torch.from_numpy(bt[b, :(n_slots + 15) // 16].astype(np.int64)).cuda()
    kk = bf16_bits_to_f64(kc[layer, pages, j].reshape(-1, h))[:n_slots]
    vv = bf16_bits_to_f64(vc[layer, pages, j].permute(0, 2, 1).reshape(-1, h))[:n_slots]
    return kk, vv


def check_attention_rows(eng, m, ctx, ro, parents, seqs, rng, atol=6e-3):
    """Sampled (row, query head) of the last layer: softmax over the cached prefix and the node's ancestors-or-self."""
    shape = eng.shape
    hq, hkv, h = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    G = hq // hkv
    q = bf16_bits_to_f64(eng.debug_tensor(1).view(torch.int16)[:m * hq * h]).reshape(m, hq, h)
    att = bf16_bits_to_f64(eng.debug_tensor(2).view(torch.int16)[:m * hq * h]).reshape(m, hq, h)
    worst = 0.0
    for b in seqs:
        Lb, n = int(ctx[b]), int(ro[b + 1] - ro[b])
        par = parents[b]
        for node in sorted({0, n // 2, n - 1}):
            head = int(rng.integers(0, hq))
            kk, vv = seq_kv(eng, eng.n_layers - 1, b, head // G, Lb + n)
            vis = list(range(Lb))
            chain, i = [], node
            while i >= 0:
                chain.append(Lb + i)
                i = int(par[i])
            vis += sorted(chain)
            want = oracle.attention_row(q[ro[b] + node, head], kk[vis], vv[vis], 1.0 / np.sqrt(h))
            got = att[ro[b] + node, head]
            worst = max(worst, float(np.abs(got - want).max()))
            np.testing.assert_allclose(got, want, atol=atol, rtol=2e-2)
    return worst


def check_lm_head(eng, m, rng, n_rows=24, n_cols=64):
    shape = eng.shape
    d, V = shape.d_model, shape.vocab
    xn = bf16_bits_to_f64(eng.debug_tensor(0).view(torch.int16)[:m * d]).reshape(m, d)
    rs = rng.integers(0, m, n_rows)
    cs = rng.integers(0, V, n_cols)
    wsub = bf16_bits_to_f64(eng.w["lm_head"][torch.from_numpy(cs).cuda()].view(torch.int16))
    got = np_of(eng.logits[torch.from_numpy(rs).cuda()][:, torch.from_numpy(cs).cuda()])
    np.testing.assert_allclose(got, xn[rs] @ wsub.T, atol=2e-4, rtol=1e-4)


def test_config4_launch_sampled_parity_and_greedy_commit():
    from paper_2508_18588_amd import HS_ACCEPT_GREEDY, HS_K_AIMD
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = CONFIG_SHAPES[4]
    seed = config_seed(4)
    L, B, k_max, window = 2, 256, 32, 256
    rng = np.random.default_rng(seed)
    resp = lengths_lognormal(B, 4000.0, 0.8, 512, 32768, seed)
    ctx = (512 + resp - window).astype(np.int64)          # snapshot one window before the end of each response
    w = make_weights_device(shape, seed, L)
    rope = rope_device(int(ctx.max()) + 64, shape.head_dim)
    eng = Engine(shape, w, rope, max_batch=B, k_max=k_max, c_max=1, max_len=int(ctx.max()) + 64,
                 seq_caps=[int(c) + 64 for c in ctx], shuffle_pages_seed=seed & 0xFFFF, keep_logits=True)
    fill_kv_random(eng.kc, eng.vc, seed + 1, 0.02 * float(np.sqrt(shape.d_model)))
    toks = [rng.integers(0, shape.vocab, int(c) + 1).astype(np.int32) for c in ctx]
    k_init = [int(2 + 2 * (b % 16)) for b in range(B)]     # AIMD windows 2, 4, .., 32
    eng.load_sequences(toks, budgets=[window] * B)
    eng.k_state[:B].copy_(torch.tensor(k_init, dtype=torch.int32))
    rows, parents = [], []
    for b in range(B):
        k = b % (k_max + 1)                                # every draft length 0..32 occurs
        n = 1 + k
        rows.append(dict(tok=np.concatenate([[toks[b][-1]], rng.integers(0, shape.vocab, k)]).astype(np.int32),
                         parent=np.arange(-1, n - 1), pos=np.arange(int(ctx[b]), int(ctx[b]) + n)))
        parents.append(rows[-1]["parent"])
    m = eng.set_rows(rows)
    cap = eng.capture_last_layer()
    eng.set_rows_hint(m)
    eng.verify()
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    ro = np_of(eng.st["row_off"])
    # every projection of the last layer at this launch (4352 rows: twelve 384-row passes) against its definition
    print("config 4 last-layer projections, worst abs error:",
          check_last_layer_projections(eng, cap, m, [0, 383, 384, 2175, 2176, m - 2, m - 1]
                                       + rng.integers(0, m, 10).tolist(), rng))
    # sequences: 33 nodes (seven row tiles per KV head), the longest and the shortest context, a few in between
    picks = [32, 65, 98, int(np.argmax(ctx)), int(np.argmin(ctx)), 0, 3, 140, 255]
    worst = check_attention_rows(eng, m, ctx, ro, parents, picks, rng)
    check_lm_head(eng, m, rng)
    arg = np_of(eng.st["argmax"])[:m]
    for r in rng.integers(0, m, 16):
        assert arg[r] == int(np_of(eng.logits[int(r)]).argmax())
    # ---- greedy accept and commit (AIMD): force acceptance of 0..K draft tokens by editing the argmax rows
    want_a = []
    for b in range(B):
        k = b % (k_max + 1)
        a = int(rng.integers(0, k + 1))
        want_a.append(a)
        for i in range(a):
            arg[ro[b] + i] = rows[b]["tok"][i + 1]
        if a < k and arg[ro[b] + a] == rows[b]["tok"][a + 1]:
            arg[ro[b] + a] = (arg[ro[b] + a] + 1) % shape.vocab
    eng.st["argmax"][:m].copy_(torch.from_numpy(arg))
    pol = Policy(window=8, m_min=3, k_mode=HS_K_AIMD, k_max=k_max)
    eng.accept(HS_ACCEPT_GREEDY)
    eng.commit(pol)
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    st = {k: np_of(v) for k, v in eng.st.items()}
    sl, ks, tail = np_of(eng.seq_len), np_of(eng.k_state), np_of(eng.tail)
    for b in range(B):
        k = b % (k_max + 1)
        a, out, path = oracle.accept_greedy(rows[b]["tok"], rows[b]["parent"], arg[ro[b]:ro[b + 1]])
        assert a == want_a[b] and st["accept_len"][b] == a and st["n_out"][b] == a + 1
        assert st["out_tok"][b, :a + 1].tolist() == out.tolist()
        assert sl[b] == int(ctx[b]) + 1 + a + 1
        assert ks[b] == oracle.aimd(k_init[b], k > 0, k > 0 and a == k, pol.aimd_inc, pol.aimd_cap, pol.aimd_reset)
        keep = min(a + 1, eng.w_max)
        assert tail[b, -keep:].tolist() == out.tolist()[-keep:]
    eng.close()
    print("config 4 launch: rows", m, "attention max abs err", worst)


def test_config5_launch_tree_draft_verify_rejection_commit():
    from paper_2508_18588_amd import HS_ACCEPT_GREEDY, HS_ACCEPT_REJECTION
    from paper_2508_18588_amd.runtime import Engine, Policy
    shape = CONFIG_SHAPES[5]
    seed = config_seed(5)
    L, B, k_max, W, Lc = 2, 64, 8, 8, 8192
    rng = np.random.default_rng(seed)
    w = make_weights_device(shape, seed, L)
    rope = rope_device(Lc + 64, shape.head_dim)
    eng = Engine(shape, w, rope, max_batch=B, k_max=k_max, c_max=2, max_len=Lc + 64, shuffle_pages_seed=seed & 0xFFFF,
                 keep_logits=True)
    fill_kv_random(eng.kc, eng.vc, seed + 1, 0.02 * float(np.sqrt(shape.d_model)))
    toks = [rng.integers(0, shape.vocab, Lc + 1).astype(np.int32) for _ in range(B)]
    sids = rng.integers(0, 2 ** 62, B).astype(np.int64)
    eng.load_sequences(toks, budgets=[64] * B, seq_ids=sids)
    # two previous-epoch texts per sequence: both continue the sequence's last tokens; the second one shares the
    # first (b mod 9) continuation tokens with the first and then goes its own way
    cands = []
    for b in range(B):
        c0 = rng.integers(0, shape.vocab, 24).astype(np.int32)
        c1 = c0.copy()
        share = b % 9
        c1[share:] = rng.integers(0, shape.vocab, 24 - share)
        if share < 24 and c1[share] == c0[share]:
            c1[share] = (c1[share] + 1) % shape.vocab
        fill = lambda: rng.integers(0, shape.vocab, 300).astype(np.int32)
        cands.append([np.concatenate([fill(), toks[b][-W:], c0]), np.concatenate([fill(), toks[b][-W:], c1])])
    eng.set_history(cands)
    pol = Policy(window=W, m_min=3, k_fixed=k_max, k_max=k_max)
    eng.draft(pol)
    torch.cuda.synchronize()
    st = {k: np_of(v) for k, v in eng.st.items()}
    ro = st["row_off"]
    trees = []
    for b in range(B):
        chains = []
        for c in range(2):
            p, mlen = oracle.suffix_match(cands[b][c], toks[b], W, 3)
            k = oracle.draft_len(oracle.k_policy(pol.k_mode, pol.k_fixed, 2, mlen, pol.k_max), len(cands[b][c]), p, 64)
            assert (st["draft_start"][2 * b + c], st["match_len"][2 * b + c], st["draft_len"][2 * b + c]) == (p, mlen, k)
            chains.append(cands[b][c][p:p + k])
        t = oracle.build_tree(chains, int(toks[b][-1]), Lc)
        sl = slice(ro[b], ro[b + 1])
        assert st["tok"][sl].tolist() == t["tok"].tolist() and st["parent"][sl].tolist() == t["parent"].tolist()
        assert st["pos"][sl].tolist() == t["pos"].tolist()
        assert len(t["tok"]) == 1 + 8 + (8 - b % 9 if b % 9 < 8 else 0)
        trees.append(t)
    m = int(ro[B])
    cap = eng.capture_last_layer()
    eng.set_rows_hint(m)
    eng.verify()
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    # every projection of the last layer at the 14B shape (N, K = 7168 x 5120, 5120 x 5120, 2 x 13824 x 5120,
    # 5120 x 13824) against its definition
    print("config 5 last-layer projections, worst abs error:",
          check_last_layer_projections(eng, cap, m, [0, 383, 384, 767, 768, m - 1] + rng.integers(0, m, 10).tolist(),
                                       rng))
    ctx = np.full(B, Lc, np.int64)
    worst = check_attention_rows(eng, m, ctx, ro, [t["parent"] for t in trees], [0, 1, 4, 8, 9, 31, 63], rng)
    check_lm_head(eng, m, rng)
    # ---- rejection sampling at temperature 1 on the model's own (flat) logits, then on logits with the drafted
    # tokens boosted so that paths are accepted; both against the oracle's rule on the same fp32 logits
    T = 1.0
    n_acc = n_flag = 0
    for trial, boost in enumerate((0.0, 14.0)):
        if boost:
            r = 0
            for t in trees:
                for i in range(1, len(t["tok"])):
                    eng.logits[r + int(t["parent"][i]), int(t["tok"][i])] += boost * float(rng.uniform(0.7, 1.2))
                r += len(t["tok"])
        pseed = int(rng.integers(0, 2 ** 63))
        eng.accept(HS_ACCEPT_REJECTION, T, pseed)
        torch.cuda.synchronize()
        sa = {k: np_of(v) for k, v in eng.st.items()}
        for b in range(0, B, 3 if not boost else 2):        # the fp64 oracle walks 152064-wide rows: a sample of them
            t = trees[b]
            lg = np_of(eng.logits[ro[b]:ro[b + 1]]).astype(np.float64)
            a, out, path, margin = oracle.accept_stochastic(t["tok"], t["parent"], t["pos"], lg, T, pseed, int(sids[b]))
            got = (int(sa["accept_len"][b]), sa["out_tok"][b, :sa["n_out"][b]].tolist(),
                   sa["path_row"][b, :sa["n_out"][b]].tolist())
            if got != (a, out.tolist(), path.tolist()):
                assert margin < 1e-7, (trial, b, got, (a, out.tolist(), path.tolist()), margin)
                n_flag += 1
            n_acc += a
    assert n_acc > 20 and n_flag <= 2
    # ---- tree commit: greedy walk forced down the second branch where there is one; the accepted nodes' K/V must
    # land on consecutive slots after the root
    arg = np_of(eng.st["argmax"])[:m].copy()
    paths = []
    for b in range(B):
        t = trees[b]
        n = len(t["tok"])
        leaf = n - 1                                        # last node: deepest node of the second branch (or of the chain)
        chain, i = [], leaf
        while i >= 0:
            chain.append(i)
            i = int(t["parent"][i])
        chain = chain[::-1]
        for u, v in zip(chain[:-1], chain[1:]):
            arg[ro[b] + u] = t["tok"][v]
        paths.append(chain)
    eng.st["argmax"][:m].copy_(torch.from_numpy(arg))
    before = {b: [seq_kv(eng, L - 1, b, j, Lc + len(trees[b]["tok"])) for j in (0, shape.n_kv_heads - 1)] for b in (1, 4, 9, 31)}
    eng.accept(HS_ACCEPT_GREEDY)
    eng.commit(pol)
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    sc = {k: np_of(v) for k, v in eng.st.items()}
    sl = np_of(eng.seq_len)
    for b in range(B):
        a, out, path = oracle.accept_greedy(trees[b]["tok"], trees[b]["parent"], arg[ro[b]:ro[b + 1]])
        assert path.tolist() == paths[b] and sc["accept_len"][b] == a == len(paths[b]) - 1
        assert sc["path_row"][b, :a + 1].tolist() == paths[b] and sl[b] == Lc + 1 + a + 1
    for b, kvs in before.items():
        for (kk0, vv0), j in zip(kvs, (0, shape.n_kv_heads - 1)):
            kk1, vv1 = seq_kv(eng, L - 1, b, j, Lc + len(paths[b]))
            for i, node in enumerate(paths[b]):
                assert np.array_equal(kk1[Lc + i], kk0[Lc + node]) and np.array_equal(vv1[Lc + i], vv0[Lc + node])
            assert np.array_equal(kk1[:Lc], kk0[:Lc])
    eng.close()
    print("config 5 launch: rows", m, "attention max abs err", worst, "accepted", n_acc, "flagged", n_flag)
