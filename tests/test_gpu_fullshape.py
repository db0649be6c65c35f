"""Parity at the benchmark's real shape (configuration 3: 7B-shaped decoder) where the oracle cannot run the whole
model over the whole batch: (i) a two-layer slice of the 7B shape in lock-step with the oracle, logits within the
tolerance derived from the bf16 arithmetic; (ii) the full batch (128 sequences, contexts 2k..16k, the launch
configuration bench.py times) with sampled outputs of the two dominant kernels recomputed by the oracle: attention
rows from the GPU's own queries and cache, LM-head logits as fp64 dot products."""
import numpy as np
import pytest
import torch

import oracle
from hs_inputs import CONFIG_SHAPES, config_seed, lengths_uniform, make_prompts
from hs_inputs.device import fill_kv_random, make_weights_device, rope_device, weights_to_host
from gpu_common import OracleBatch, derived_logit_tol, make_histories, np_of

pytestmark = pytest.mark.gpu


def bf16_bits_to_f64(t):
    return (np_of(t).view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_7b_shape_two_layers_lockstep():
    from paper_2508_18588_amd.runtime import Engine, Policy
    from test_gpu_decode import gpu_ar_rollout, lockstep
    import gpu_common
    shape = CONFIG_SHAPES[3]
    L = 2
    w = make_weights_device(shape, config_seed(3), L)
    rope = rope_device(256, shape.head_dim)
    model = oracle.Model(shape, weights_to_host(w), np_of(rope))
    prompts = make_prompts(2, 16, shape.vocab, 301)
    rolls = gpu_ar_rollout(shape, w, rope, list(prompts), 12)
    pol = Policy(window=8, m_min=3, k_fixed=5, k_max=5)
    cands = make_histories(prompts, rolls, 8, 0.15, 0.0, shape.vocab, seed=302)
    eng = Engine(shape, w, rope, max_batch=2, k_max=5, c_max=1, max_len=16 + 12, shuffle_pages_seed=13)
    eng.load_sequences(list(prompts), budgets=[12] * 2)
    eng.set_history(cands)
    eng.prefill(list(prompts))
    ob = OracleBatch(model, list(prompts), [12] * 2, 16 + 12 + 8)
    tol = derived_logit_tol(shape, L)
    old = gpu_common.LOGIT_TOL
    import test_gpu_decode
    test_gpu_decode.LOGIT_TOL = tol          # lockstep() and check_cache() read the module-level tolerance
    gpu_common.LOGIT_TOL = tol
    try:
        stats = lockstep(eng, ob, cands, pol, max_steps=20, check_kv_layers=(1,))
    finally:
        test_gpu_decode.LOGIT_TOL = old
        gpu_common.LOGIT_TOL = old
    eng.close()
    print("7B-shape 2 layers:", stats, "tolerance", tol)
    assert stats["emitted"] == 24 and stats["max_logit_err"] <= tol


def test_full_batch_sampled_kernel_parity():
    from paper_2508_18588_amd.runtime import Engine
    shape = CONFIG_SHAPES[3]
    seed = config_seed(3)
    L, B, k_max = 2, 128, 16
    rng = np.random.default_rng(seed)
    ctx = lengths_uniform(B, 2048, 16384, seed)
    w = make_weights_device(shape, seed, L)
    rope = rope_device(int(ctx.max()) + 64, shape.head_dim)
    eng = Engine(shape, w, rope, max_batch=B, k_max=k_max, c_max=1, max_len=int(ctx.max()) + 32,
                 seq_caps=[int(c) + 32 for c in ctx], shuffle_pages_seed=77, keep_logits=True)
    fill_kv_random(eng.kc, eng.vc, seed + 1, 0.02 * float(np.sqrt(shape.d_model)))
    toks = [rng.integers(0, shape.vocab, int(c) + 1).astype(np.int32) for c in ctx]
    eng.load_sequences(toks, budgets=[64] * B)
    # hand-made chains: every draft length from 0 to 16 occurs (one row tile, several row tiles)
    rows = []
    for b in range(B):
        k = b % (k_max + 1)
        n = 1 + k
        rows.append(dict(tok=np.concatenate([[toks[b][-1]], rng.integers(0, shape.vocab, k)]).astype(np.int32),
                         parent=np.arange(-1, n - 1), pos=np.arange(int(ctx[b]), int(ctx[b]) + n)))
    m = eng.set_rows(rows)
    eng.verify()
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    ro = np_of(eng.st["row_off"])
    hq, hkv, h, V, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.vocab, shape.d_model
    G = hq // hkv
    # ---- attention of the last layer: sampled (row, query head) recomputed from the GPU's queries and cache
    q = bf16_bits_to_f64(eng.debug_tensor(1).view(torch.int16)[:m * hq * h]).reshape(m, hq, h)
    att = bf16_bits_to_f64(eng.debug_tensor(2).view(torch.int16)[:m * hq * h]).reshape(m, hq, h)
    kc = eng.kc.view(L, eng.n_blocks, hkv, 16, h)
    vc = eng.vc.view(L, eng.n_blocks, hkv, h, 16)
    bt = np_of(eng.block_table)
    worst = 0.0
    for b in (0, 3, 16, 33, 50, 84, 101, 127):        # draft lengths 0, 3, 16, 16, 16, 16, 16, 8 ...
        Lb, n = int(ctx[b]), ro[b + 1] - ro[b]
        pages = torch.from_numpy(bt[b, :(Lb + n + 15) // 16].astype(np.int64)).cuda()
        for node in sorted({0, n // 2, n - 1}):
            head = int(rng.integers(0, hq))
            j = head // G
            kk = bf16_bits_to_f64(kc[L - 1, pages, j].reshape(-1, h))[:Lb + node + 1]
            vv = bf16_bits_to_f64(vc[L - 1, pages, j].permute(0, 2, 1).reshape(-1, h))[:Lb + node + 1]
            want = oracle.attention_row(q[ro[b] + node, head], kk, vv, 1.0 / np.sqrt(h))
            got = att[ro[b] + node, head]
            worst = max(worst, float(np.abs(got - want).max()))
            np.testing.assert_allclose(got, want, atol=6e-3, rtol=2e-2)
    # ---- LM head: sampled logits as fp64 dot products of the GPU's final hidden state
    xn = bf16_bits_to_f64(eng.debug_tensor(0).view(torch.int16)[:m * d]).reshape(m, d)
    lg = np_of(eng.logits[:m])
    lm = eng.w["lm_head"]
    rs = rng.integers(0, m, 24)
    cs = rng.integers(0, V, 64)
    wsub = bf16_bits_to_f64(lm[torch.from_numpy(cs).cuda()].view(torch.int16))
    want = xn[rs] @ wsub.T
    np.testing.assert_allclose(lg[np.ix_(rs, cs)], want, atol=2e-4, rtol=1e-4)
    # argmax of every row is the first maximum of its logits
    assert np_of(eng.st["argmax"])[:m].tolist() == lg.argmax(1).tolist()
    eng.close()
    print("full batch: rows", m, "attention max abs err", worst)
