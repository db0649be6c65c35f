"""Shared pieces of the GPU parity tests: oracle-side state that advances in lock-step with the HIP path."""
import numpy as np

import oracle
from hs_inputs import history_with_context, mutate

LOGIT_TOL = 2e-2  # absolute, bf16 path (the tolerance the benchmark spec fixes)


def np_of(t):
    return t.detach().cpu().numpy()


class OracleBatch:
    """Per-sequence oracle state: committed tokens and a K/V cache holding all but the newest token."""

    def __init__(self, model, token_lists, budgets, cap):
        self.model = model
        self.x = [list(map(int, t)) for t in token_lists]
        self.budget = list(budgets)
        self.seqs = []
        for t in self.x:
            s = oracle.Seq(model, cap)
            s.extend(t[:-1])
            self.seqs.append(s)
        self.k_state = [2] * len(self.x)

    def draft(self, b, cands, pol):
        """Oracle draft for sequence b -> (per-candidate (p, m, K), tree dict or None if finished)."""
        if self.budget[b] <= 0:
            return [(-1, 0, 0)] * len(cands), None
        x = np.asarray(self.x[b], np.int32)
        info, chains = [], []
        for h in cands:
            p, m = oracle.suffix_match(h, x, pol.window, pol.m_min)
            k = oracle.draft_len(oracle.k_policy(pol.k_mode, pol.k_fixed, self.k_state[b], m, pol.k_max), len(h), p,
                                 self.budget[b])
            info.append((p, m, k))
            chains.append(np.asarray(h[p:p + k], np.int32) if k > 0 else np.zeros(0, np.int32))
        tree = oracle.build_tree(chains, x[-1], len(x) - 1)
        return info, tree

    def logits(self, b, tree):
        return self.seqs[b].tree_logits(tree["tok"], tree["parent"])

    def commit(self, b, tree, a, out, path, pol):
        """Advance by the emitted tokens `out` (a accepted + 1)."""
        n_nodes = len(tree["tok"])
        if pol.k_mode == oracle.K_AIMD:
            last = int(path[a])
            leaf = not any(int(tree["parent"][i]) == last for i in range(1, n_nodes))
            self.k_state[b] = oracle.aimd(self.k_state[b], n_nodes > 1, leaf and a > 0, pol.aimd_inc, pol.aimd_cap,
                                          pol.aimd_reset)
        self.seqs[b].extend([self.x[b][-1]] + [int(t) for t in out[:a]])
        self.x[b].extend(int(t) for t in out)
        self.budget[b] -= len(out)


def check_cache(eng, ob, layer, every=None, tol=LOGIT_TOL, rtol=2e-2):
    """Cache contents at [0, L) must equal the K/V the oracle computed for the committed tokens (K and V have the
    logits' scale 0.02 sqrt(d_model), so the logit tolerance applies).  The cache holds bf16 bits, or floats when the
    engine runs in the fp32-activation mode."""
    shape = eng.shape
    hkv, h = shape.n_kv_heads, shape.head_dim
    if getattr(eng, "precise", False):
        kc = np_of(eng.kc).reshape(eng.n_layers, eng.n_blocks, hkv, 16, h)
        vc = np_of(eng.vc).reshape(eng.n_layers, eng.n_blocks, hkv, h, 16)
        f = lambda a: a.astype(np.float64)
    else:
        kc = np_of(eng.kc).view(np.uint16).reshape(eng.n_layers, eng.n_blocks, hkv, 16, h)
        vc = np_of(eng.vc).view(np.uint16).reshape(eng.n_layers, eng.n_blocks, hkv, h, 16)
        f = lambda bits: (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    bt = np_of(eng.block_table)
    for b, s in enumerate(ob.seqs):
        for pos in range(0, len(s), every or max(1, len(s) // 40)):
            k, v = s.kv(layer, pos)
            page, ip = bt[b, pos // 16], pos % 16
            gk = f(kc[layer, page, :, ip, :]).reshape(-1)
            gv = f(vc[layer, page, :, :, ip]).reshape(-1)
            np.testing.assert_allclose(gk, k, atol=tol, rtol=rtol)
            np.testing.assert_allclose(gv, v, atol=tol, rtol=rtol)


def top2_margin(row):
    part = np.partition(row, -2)
    return float(part[-1] - part[-2])


def make_histories(prompts, rollouts, window, p_iid, p_span, vocab, seed):
    rng = np.random.default_rng(seed)
    return [[history_with_context(prompts[b], mutate(np.asarray(rollouts[b], np.int32), p_iid, p_span, vocab, rng),
                                  window)] for b in range(len(prompts))]


def derived_logit_tol(shape, n_layers):
    """Absolute logit tolerance of the default (bf16-activation) path at a given depth and width: its MEASURED error
    curve with a margin of 1.5.

    Every rounding of a GEMM input to bf16 adds a relative error of rms eps = 2^-9/sqrt(3).  Measured against the
    oracle's residual stream at the 7B shape (test_gpu_precise.py), the relative rms error after l layers is
    4.5 eps sqrt(l) (5.1e-3 sqrt(l), flat from l = 2 to 8 and continued to l = 28 by the benchmark's sample), and the
    final norm adds one more eps.  Logits have standard deviation sigma = 0.02 sqrt(d_model) (random-init weights);
    the maximum over ~10^6 logit errors is ~5.2 rms.  For the 2-layer d=256 toy configuration this gives the 2e-2 of
    the benchmark spec; the fp32-activation mode meets 2e-2 (and 1e-4 relative) at every depth."""
    sigma = 0.02 * np.sqrt(shape.d_model)
    eps = 2.0 ** -9 / np.sqrt(3.0)
    return float(5.2 * sigma * (4.5 * eps * np.sqrt(n_layers) + eps) * 1.5)
