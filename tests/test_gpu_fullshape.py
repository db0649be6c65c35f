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
from gpu_common import OracleBatch, check_last_layer_projections, derived_logit_tol, make_histories, np_of

pytestmark = pytest.mark.gpu


def bf16_bits_to_f64(t):
    return (np_of(t).view(np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def test_7b_shape_two_layers_lockstep():
    from paper_2508_18588_amd.runtime import Engine, Policy
    from test_gpu_decode import gpu_ar_rollout, lockstep
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
    stats = lockstep(eng, ob, cands, pol, max_steps=20, check_kv_layers=(1,), tol=tol)
    eng.close()
    print("7B-shape 2 layers:", stats, "tolerance", tol)
    assert stats["emitted"] == 24 and stats["max_logit_err"] <= tol


def _full_batch_sampled_kernel_parity(cfg, B, ctx, k_max, picks, proj_rows):
    from paper_2508_18588_amd.runtime import Engine
    shape = CONFIG_SHAPES[cfg]
    seed = config_seed(cfg)
    L = 2
    rng = np.random.default_rng(seed)
    w = make_weights_device(shape, seed, L)
    rope = rope_device(int(ctx.max()) + 64, shape.head_dim)
    eng = Engine(shape, w, rope, max_batch=B, k_max=k_max, c_max=1, max_len=int(ctx.max()) + 32,
                 seq_caps=[int(c) + 32 for c in ctx], shuffle_pages_seed=77, keep_logits=True)
    fill_kv_random(eng.kc, eng.vc, seed + 1, 0.02 * float(np.sqrt(shape.d_model)))
    toks = [rng.integers(0, shape.vocab, int(c) + 1).astype(np.int32) for c in ctx]
    eng.load_sequences(toks, budgets=[64] * B)
    # hand-made chains: every draft length from 0 to k_max occurs (one row tile, several row tiles)
    rows = []
    for b in range(B):
        k = b % (k_max + 1)
        n = 1 + k
        rows.append(dict(tok=np.concatenate([[toks[b][-1]], rng.integers(0, shape.vocab, k)]).astype(np.int32),
                         parent=np.arange(-1, n - 1), pos=np.arange(int(ctx[b]), int(ctx[b]) + n)))
    m = eng.set_rows(rows)
    cap = eng.capture_last_layer()
    eng.set_rows_hint(m)
    eng.verify()
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    ro = np_of(eng.st["row_off"])
    # ---- every projection of the last layer at this launch against fp64 dot products of its own inputs
    worst_proj = check_last_layer_projections(eng, cap, m, [r for r in proj_rows if r < m] + [m - 1]
                                              + rng.integers(0, m, 8).tolist(), rng)
    print(f"config {cfg}: last-layer projections, worst abs error:", worst_proj)
    hq, hkv, h, V, d = shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.vocab, shape.d_model
    G = hq // hkv
    # ---- attention of the last layer: sampled (row, query head) recomputed from the GPU's queries and cache
    q = bf16_bits_to_f64(eng.debug_tensor(1).view(torch.int16)[:m * hq * h]).reshape(m, hq, h)
    att = bf16_bits_to_f64(eng.debug_tensor(2).view(torch.int16)[:m * hq * h]).reshape(m, hq, h)
    kc = eng.kc.view(L, eng.n_blocks, hkv, 16, h)
    vc = eng.vc.view(L, eng.n_blocks, hkv, h, 16)
    bt = np_of(eng.block_table)
    worst = 0.0
    for b in picks:
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
    cs = np.concatenate([rng.integers(0, V, 64), [0, V - 1]])
    wsub = bf16_bits_to_f64(lm[torch.from_numpy(cs).cuda()].view(torch.int16))
    want = xn[rs] @ wsub.T
    np.testing.assert_allclose(lg[np.ix_(rs, cs)], want, atol=2e-4, rtol=1e-4)
    # argmax of every row is the first maximum of its logits
    arg = np_of(eng.st["argmax"])[:m].copy()
    assert arg.tolist() == lg.argmax(1).tolist()
    # the same launch without a logits array: the LM head's row-maximum epilogue + the reduction inside the acceptance
    # kernel must name the same token for every row
    eng.logits = None
    eng._structs()
    eng.c_step.rows_hint = m
    eng.st["argmax"].fill_(-1)
    eng.verify()
    eng.accept()
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    assert (np_of(eng.st["argmax"])[:m] == arg).all()
    eng.close()
    print(f"config {cfg} full batch: rows", m, "attention max abs err", worst)


def test_full_batch_sampled_kernel_parity():
    """Configuration 3's launch: 128 sequences, contexts 2k..16k, draft lengths 0..16 (1152 rows: three 384-row
    passes of the GEMM, 64-row QKV/O groups, the 9-chunk down projection)."""
    ctx = lengths_uniform(128, 2048, 16384, config_seed(3))
    _full_batch_sampled_kernel_parity(3, 128, ctx, 16, (0, 3, 16, 33, 50, 84, 101, 127),
                                      [0, 31, 32, 255, 256, 383, 384, 385, 767, 768])


def test_config2_full_batch_sampled_kernel_parity():
    """Configuration 2's launch: 1.5B shape (d 1536, 12 query heads on 2 KV heads = 6 per KV head, FFN 8960,
    vocabulary 151936), 64 sequences at context 512 + 2048, draft lengths 0..8 (320 rows)."""
    ctx = np.full(64, 2560, np.int32)
    _full_batch_sampled_kernel_parity(2, 64, ctx, 8, (0, 8, 17, 35, 44, 63), [0, 31, 32, 255, 256, 257])


def test_config2_shape_lockstep_subset():
    """Configuration 2 in lock-step with the oracle on a subset: its shape and policy (K = 8 fixed, window 8, history
    mutated 20 % iid + 5 % spans), 2 sequences with a 48-token prompt and 36 response tokens each, and 3 of the 28
    layers -- the LM head over 151936 tokens dominates the oracle's time per row, so depth is what is cut; full depth
    at this shape is covered per kernel by the sampled test above.  Tolerance: the measured per-layer error curve of
    the bf16 path (see test_gpu_precise.py) with its 1.5 margin."""
    from paper_2508_18588_amd.runtime import Engine, Policy
    from test_gpu_decode import gpu_ar_rollout, lockstep
    shape = CONFIG_SHAPES[2]
    L, B, P, T = 3, 2, 48, 36
    w = make_weights_device(shape, config_seed(2), L)
    rope = rope_device(256, shape.head_dim)
    model = oracle.Model(shape, weights_to_host(w), np_of(rope))
    prompts = make_prompts(B, P, shape.vocab, 201)
    rolls = gpu_ar_rollout(shape, w, rope, list(prompts), T)
    pol = Policy(window=8, m_min=3, k_fixed=8, k_max=8)
    cands = make_histories(prompts, rolls, 8, 0.20, 0.05, shape.vocab, seed=202)
    eng = Engine(shape, w, rope, max_batch=B, k_max=8, c_max=1, max_len=P + T, shuffle_pages_seed=21)
    eng.load_sequences(list(prompts), budgets=[T] * B)
    eng.set_history(cands)
    eng.prefill(list(prompts))
    ob = OracleBatch(model, list(prompts), [T] * B, P + T + 16)
    tol = derived_logit_tol(shape, L)
    stats = lockstep(eng, ob, cands, pol, max_steps=T, check_kv_layers=(L - 1,), tol=tol)
    eng.close()
    print("config-2 shape, 3 layers:", stats, "tolerance", tol)
    assert stats["emitted"] == B * T and stats["max_logit_err"] <= tol
    assert stats["rows"] > 2 * stats["steps"] * B      # drafts were verified
