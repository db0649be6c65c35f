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


# ---------------------------------------------------------------- last-layer projections of a real forward pass

def _rows_f64(t, idx):
    """Rows `idx` of a device matrix holding bf16 values (torch.bfloat16 or int16 bit patterns) or floats -> fp64."""
    import torch
    sub = t[torch.as_tensor(np.asarray(idx, np.int64), device=t.device)]
    if sub.dtype == torch.int16:
        sub = sub.view(torch.bfloat16)
    return sub.double().cpu().numpy()


def check_last_layer_projections(eng, cap, m, rows, rng, n_cols=24):
    """Every projection of the last layer against its definition, C = A . W^T as fp64 dot products of the path's own
    inputs of that projection (snapshots of hs_debug_capture + hs_debug_buffer), at sampled rows and columns of the
    launch that just ran: QKV (through the rotation, against the query buffer and the cache rows the step wrote),
    O and down (as the change of the fp32 residual stream), gate/up with SwiGLU (against the activation buffer).
    Tolerances: fp32 accumulation over K (2e-5 of the output scale), plus one bf16 rounding where the output is
    stored as bf16, plus the fp32 rounding of the residual add.  Returns the worst errors per projection."""
    import torch
    shape, L = eng.shape, eng.n_layers
    d, F, hq, hkv, h = shape.d_model, shape.d_ffn, shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    qh, half = hq * h, h // 2
    rows = np.asarray(sorted(set(int(r) for r in rows if 0 <= r < m)), np.int64)
    assert not eng.precise, "written for the bf16 layout of the snapshots"
    view = lambda t, dt, cols: t.view(dt)[:m * cols].view(m, cols)
    xn1 = _rows_f64(view(cap[0], torch.int16, d), rows)
    x1 = _rows_f64(view(cap[1], torch.float32, d), rows)
    xn2 = _rows_f64(view(cap[2], torch.int16, d), rows)
    x2 = _rows_f64(view(cap[3], torch.float32, d), rows)
    xf = _rows_f64(view(eng.debug_tensor(4), torch.float32, d), rows)
    q = _rows_f64(view(eng.debug_tensor(1), torch.int16, qh), rows)
    att = _rows_f64(view(eng.debug_tensor(2), torch.int16, qh), rows)
    act = _rows_f64(view(eng.debug_tensor(5), torch.int16, F), rows)
    W = eng.w
    l = L - 1
    pos = np_of(eng.st["pos"])[rows]
    r2s = np_of(eng.st["row2seq"])[rows]
    ro = np_of(eng.st["row_off"])
    rope = np_of(eng.rope).astype(np.float64)
    worst = {}
    bf = 2.0 ** -8

    def edge_cols(n, groups):
        c = set(int(x) for x in rng.integers(0, n, n_cols))
        for g in groups:
            c.update(x for x in (g - 1, g, n - g, n - g - 1) if 0 <= x < n)
        c.update((0, n - 1))
        return np.asarray(sorted(c), np.int64)

    # ---- QKV: rotated queries (buffer 1) and the K / V rows written into the cache at slot L_b + node
    heads = sorted(set(int(x) for x in rng.integers(0, hq, 4)) | {0, hq - 1})
    js = sorted(set(int(x) for x in rng.integers(0, half, 6)) | {0, half - 1})
    wq = W["wqkv"][l]
    err = 0.0
    for hd_ in heads:
        lo = np.asarray([hd_ * h + j for j in js], np.int64)
        a = xn1 @ _rows_f64(wq, lo).T
        b = xn1 @ _rows_f64(wq, lo + half).T
        c, s = rope[pos][:, js, 0], rope[pos][:, js, 1]
        for want, got in ((a * c - b * s, q[:, lo]), (b * c + a * s, q[:, lo + half])):
            tol = bf * np.abs(want) + 2e-5 * (np.abs(want).max() + 1.0)
            assert (np.abs(got - want) <= tol).all(), ("q", hd_)
            err = max(err, float(np.abs(got - want).max()))
    kc = eng.kc.view(L, eng.n_blocks, hkv, 16, h)
    vc = eng.vc.view(L, eng.n_blocks, hkv, h, 16)
    bt = np_of(eng.block_table)
    slots = np_of(eng.seq_len)[r2s] - 1 + (rows - ro[r2s])          # seq_len is still the pre-commit length
    pages = torch.as_tensor(bt[r2s, slots // 16].astype(np.int64), device="cuda:0")
    ip = torch.as_tensor((slots % 16).astype(np.int64), device="cuda:0")
    for jj in sorted({0, hkv - 1}):
        ar = torch.arange(len(rows), device="cuda:0")
        kgot = kc[l][pages, jj][ar, ip].view(torch.bfloat16).double().cpu().numpy()        # [rows, h]
        vgot = vc[l][pages, jj][ar, :, ip].view(torch.bfloat16).double().cpu().numpy()
        lo = np.asarray([qh + jj * h + j for j in js], np.int64)
        a = xn1 @ _rows_f64(wq, lo).T
        b = xn1 @ _rows_f64(wq, lo + half).T
        c, s = rope[pos][:, js, 0], rope[pos][:, js, 1]
        jn = np.asarray(js)
        for want, got in ((a * c - b * s, kgot[:, jn]), (b * c + a * s, kgot[:, jn + half])):
            tol = bf * np.abs(want) + 2e-5 * (np.abs(want).max() + 1.0)
            assert (np.abs(got - want) <= tol).all(), ("k", jj)
            err = max(err, float(np.abs(got - want).max()))
        vo = np.asarray([qh + hkv * h + jj * h + j for j in js + [j + half for j in js]], np.int64)
        want = xn1 @ _rows_f64(wq, vo).T
        got = vgot[:, np.concatenate([jn, jn + half])]
        tol = bf * np.abs(want) + 2e-5 * (np.abs(want).max() + 1.0)
        assert (np.abs(got - want) <= tol).all(), ("v", jj)
        err = max(err, float(np.abs(got - want).max()))
    worst["qkv"] = err
    # ---- O projection: residual after it minus residual before it
    cols = edge_cols(d, (64, 128, 160))
    want = att @ _rows_f64(W["wo"][l], cols).T
    got = x2[:, cols] - x1[:, cols]
    tol = 2e-5 * (np.abs(want).max() + 1.0) + 4e-7 * np.abs(x2[:, cols])
    assert (np.abs(got - want) <= tol).all(), "o"
    worst["o"] = float(np.abs(got - want).max())
    # ---- gate/up + SwiGLU: the bf16 activation
    cols = edge_cols(F, (16, 64, 80, 160))
    g_ = xn2 @ _rows_f64(W["wgate"][l], cols).T
    u_ = xn2 @ _rows_f64(W["wup"][l], cols).T
    want = g_ / (1.0 + np.exp(-g_)) * u_
    got = act[:, cols]
    # one bf16 rounding of the result; the hardware reciprocal and exponential of the epilogue add a few fp32 ulps
    tol = 1.5 * bf * np.abs(want) + 4e-5 * (np.abs(want).max() + 1.0)
    assert (np.abs(got - want) <= tol).all(), "gate_up"
    worst["gate_up"] = float(np.abs(got - want).max())
    # ---- down projection: final residual minus residual before it
    cols = edge_cols(d, (64, 128, 160))
    want = act @ _rows_f64(W["wdown"][l], cols).T
    got = xf[:, cols] - x2[:, cols]
    tol = 2e-5 * (np.abs(want).max() + 1.0) + 4e-7 * np.abs(xf[:, cols])
    assert (np.abs(got - want) <= tol).all(), "down"
    worst["down"] = float(np.abs(got - want).max())
    return worst
