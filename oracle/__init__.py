"""ctypes front-end of the CPU oracle (`hs_oracle.c`).

TEST INFRASTRUCTURE ONLY: imported by `tests/`, by `__graft_entry__.smoke()`
and by the `cpu_baseline` leg of `bench.py`.  The product package never
imports this module and this module never imports the product package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hs_oracle.c")
_LIB = os.path.join(_HERE, "libhs_oracle.so")

K_FIXED, K_MATCHLEN, K_AIMD = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (OpenMP over independent output rows only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
                               _SRC, "-o", _LIB, "-lm"])
    return _LIB


class _Model(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("max_pos", C.c_int32),
        ("rms_eps", C.c_double),
        ("embed", C.c_void_p), ("lm_head", C.c_void_p), ("norm_f", C.c_void_p),
        ("wqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)), ("wgate", C.POINTER(C.c_void_p)),
        ("wup", C.POINTER(C.c_void_p)), ("wdown", C.POINTER(C.c_void_p)),
        ("norm1", C.POINTER(C.c_void_p)), ("norm2", C.POINTER(C.c_void_p)),
        ("rope", C.c_void_p),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i32p, u64p, f64p = C.POINTER(C.c_int32), C.POINTER(C.c_uint64), C.POINTER(C.c_double)
        intp = C.POINTER(C.c_int)
        L.orc_suffix_match.argtypes = [i32p, C.c_int, i32p, C.c_int, C.c_int, C.c_int, intp, intp]
        L.orc_suffix_match_backoff.argtypes = L.orc_suffix_match.argtypes
        L.orc_trace_sim.argtypes = [i32p, C.c_int, i32p, C.c_int, C.c_int]
        L.orc_reward_draft.argtypes = [C.c_int, i32p, i32p, i32p, i32p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                       i32p, intp, intp, intp, intp]
        L.orc_k_policy.argtypes = [C.c_int] * 5
        L.orc_gate_step.argtypes = [i32p, C.c_int, C.c_uint32, C.c_uint32]
        L.orc_gate_table.argtypes = [C.POINTER(C.c_float), i32p, C.c_int, C.c_double, C.c_int, i32p]
        L.orc_gate_table.restype = None
        L.orc_plan_allocation.argtypes = [f64p, C.c_int, C.c_int, C.c_int, C.c_int, C.c_double, i32p, f64p]
        L.orc_draft_len.argtypes = [C.c_int] * 4
        L.orc_aimd.argtypes = [C.c_int] * 6
        L.orc_build_tree.argtypes = [C.c_int, C.POINTER(i32p), intp, C.c_int32, C.c_int, i32p, i32p, i32p, u64p,
                                     C.c_int]
        L.orc_bf16.argtypes = [C.c_uint16]
        L.orc_bf16.restype = C.c_double
        L.orc_attention_row.argtypes = [f64p, f64p, f64p, C.c_int, C.c_int, C.c_int, C.c_double, f64p]
        L.orc_attention_row.restype = None
        L.orc_seq_new.argtypes = [C.POINTER(_Model), C.c_int]
        L.orc_seq_new.restype = C.c_void_p
        L.orc_seq_free.argtypes = [C.c_void_p]
        L.orc_seq_free.restype = None
        L.orc_seq_len.argtypes = [C.c_void_p]
        L.orc_seq_truncate.argtypes = [C.c_void_p, C.c_int]
        L.orc_seq_kv.argtypes = [C.c_void_p, C.c_int, C.c_int, f64p, f64p]
        L.orc_seq_load_kv.argtypes = [C.c_void_p, C.c_int, f64p, f64p]
        L.orc_seq_push.argtypes = [C.c_void_p, C.c_int32, f64p]
        L.orc_seq_set_trace.argtypes = [C.c_void_p, f64p]
        L.orc_seq_set_trace.restype = None
        L.orc_argmax.argtypes = [f64p, C.c_int]
        L.orc_tree_logits.argtypes = [C.c_void_p, C.c_int, i32p, i32p, f64p]
        L.orc_tree_logits_shared.argtypes = [C.c_void_p, C.c_int, i32p, i32p, f64p]
        L.orc_accept_greedy_bruteforce.argtypes = [C.c_void_p, C.c_int, i32p, i32p, i32p, i32p]
        L.orc_accept_greedy.argtypes = [C.c_int, i32p, i32p, i32p, i32p, i32p]
        L.orc_philox4x32_10.argtypes = [C.POINTER(C.c_uint32)] * 3
        L.orc_philox4x32_10.restype = None
        L.orc_philox_batch.argtypes = [C.c_int, C.POINTER(C.c_uint32), C.POINTER(C.c_uint32), C.POINTER(C.c_uint32)]
        L.orc_philox_batch.restype = None
        L.orc_uniform.argtypes = [C.c_uint64, C.c_uint64, C.c_uint32, C.c_uint32]
        L.orc_uniform.restype = C.c_double
        L.orc_accept_stochastic.argtypes = [C.c_int, C.c_int, i32p, i32p, i32p, f64p, C.c_double, C.c_uint64,
                                            C.c_uint64, i32p, i32p, f64p]
        _lib = L
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(C.POINTER(C.c_double))


# ------------------------------------------------------------------ draft

def suffix_match(hist, x, w: int, m_min: int, backoff: bool = False):
    """(p, m): draft start position in `hist` and matched length; (-1, 0) if none."""
    h, hp = _i32(hist)
    xx, xp = _i32(x)
    p, m = C.c_int(), C.c_int()
    fn = lib().orc_suffix_match_backoff if backoff else lib().orc_suffix_match
    fn(hp, len(h), xp, len(xx), w, m_min, C.byref(p), C.byref(m))
    return p.value, m.value


def reward_draft(hists, rewards, x, w: int, m_min: int, k: int, occ_max: int = 1024):
    """Reward-priority draft over all responses of one prompt.  Returns dict(tok, m, n_occ, g, p)."""
    arrs = [np.ascontiguousarray(h, dtype=np.int32) for h in hists]
    off = np.zeros(len(arrs) + 1, np.int32)
    off[1:] = np.cumsum([len(a) for a in arrs])
    flat, fp = _i32(np.concatenate(arrs) if off[-1] else np.zeros(1, np.int32))
    o, o_p = _i32(off)
    r, rp = _i32(rewards)
    xx, xp = _i32(x)
    out = np.zeros(max(k, 1), np.int32)
    m, no, g, p = C.c_int(), C.c_int(), C.c_int(), C.c_int()
    n = lib().orc_reward_draft(len(arrs), fp, o_p, rp, xp, len(xx), w, m_min, k, occ_max,
                               out.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(m), C.byref(no), C.byref(g),
                               C.byref(p))
    return dict(tok=out[:n].copy(), m=m.value, n_occ=no.value, g=g.value, p=p.value)


def trace_sim(cur, hist, key: int = 3) -> int:
    c, cp = _i32(cur)
    h, hp = _i32(hist)
    return lib().orc_trace_sim(cp, len(c), hp, len(h), key)


def gate_step(gate: np.ndarray, live: int, drafted_total: int, accepted_total: int) -> int:
    """Advance the speculation gate (int32[32], updated in place) by one step; returns 1 if speculation runs."""
    assert gate.dtype == np.int32 and gate.flags.c_contiguous and gate.size >= 25
    return lib().orc_gate_step(gate.ctypes.data_as(C.POINTER(C.c_int32)), live, drafted_total & 0xFFFFFFFF,
                               accepted_total & 0xFFFFFFFF)


def gate_table(ms, rows, k_bar: float, b_max: int) -> np.ndarray:
    m = np.ascontiguousarray(ms, dtype=np.float32)
    r, rp = _i32(rows)
    out = np.zeros(17, np.int32)
    lib().orc_gate_table(m.ctypes.data_as(C.POINTER(C.c_float)), rp, len(m), float(k_bar), b_max,
                         out.ctypes.data_as(C.POINTER(C.c_int32)))
    return out


def plan_allocation(tau, min_wks: int, max_wks: int, wks: int, t_train: float):
    """Tier-2 planning problem (Sec. 6.2): tau[i][k - min_wks] = time of ranking group i on k workers.  Returns
    (plan int32[N], d) with d the exact smallest feasible gradient, or None if the cluster cannot meet any gradient
    in the search interval."""
    t = np.ascontiguousarray(tau, dtype=np.float64)
    n, k = t.shape
    assert k == max_wks - min_wks + 1
    plan = np.zeros(n, np.int32)
    d = np.zeros(1, np.float64)
    ok = lib().orc_plan_allocation(t.ctypes.data_as(C.POINTER(C.c_double)), n, min_wks, max_wks, wks, float(t_train),
                                   plan.ctypes.data_as(C.POINTER(C.c_int32)),
                                   d.ctypes.data_as(C.POINTER(C.c_double)))
    return (plan, float(d[0])) if ok else None


def k_policy(mode, k_fixed, k_state, match_len, k_max) -> int:
    return lib().orc_k_policy(mode, k_fixed, k_state, match_len, k_max)


def draft_len(k_pol, lh, p, budget_left) -> int:
    return lib().orc_draft_len(k_pol, lh, p, budget_left)


def aimd(k, drafted, full, inc=2, cap=32, reset=2) -> int:
    return lib().orc_aimd(k, int(bool(drafted)), int(bool(full)), inc, cap, reset)


def build_tree(chains, root_tok: int, l_cached: int, max_nodes: int = 64):
    """Merge draft chains (list of int arrays, candidate order) into a tree.
    Returns dict(tok, pos, parent, anc_mask) of length n_nodes."""
    n_c = len(chains)
    arrs = [np.ascontiguousarray(c, dtype=np.int32) for c in chains]
    ptrs = (C.POINTER(C.c_int32) * max(n_c, 1))(*[a.ctypes.data_as(C.POINTER(C.c_int32)) for a in arrs])
    lens = (C.c_int * max(n_c, 1))(*[len(a) for a in arrs])
    tok = np.zeros(max_nodes, np.int32)
    pos = np.zeros(max_nodes, np.int32)
    par = np.zeros(max_nodes, np.int32)
    anc = np.zeros(max_nodes, np.uint64)
    n = lib().orc_build_tree(n_c, ptrs, lens, int(root_tok), int(l_cached),
                             tok.ctypes.data_as(C.POINTER(C.c_int32)), pos.ctypes.data_as(C.POINTER(C.c_int32)),
                             par.ctypes.data_as(C.POINTER(C.c_int32)), anc.ctypes.data_as(C.POINTER(C.c_uint64)),
                             max_nodes)
    if n < 0:
        raise ValueError("tree exceeds max_nodes")
    return {"tok": tok[:n].copy(), "pos": pos[:n].copy(), "parent": par[:n].copy(), "anc_mask": anc[:n].copy()}


# ------------------------------------------------------------------ model

class Model:
    """Holds the weight arrays (numpy, from hs_inputs.make_weights) and the C descriptor."""

    def __init__(self, shape, weights: dict, rope: np.ndarray):
        self.shape = shape
        self._keep = []
        n_layers = len(weights["wqkv"])
        m = _Model()
        m.n_layers, m.d_model, m.n_q_heads, m.n_kv_heads = n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads
        m.head_dim, m.d_ffn, m.vocab, m.max_pos = shape.head_dim, shape.d_ffn, shape.vocab, rope.shape[0]
        m.rms_eps = shape.rms_eps

        def one(a, dt):
            a = np.ascontiguousarray(a, dtype=dt)
            self._keep.append(a)
            return a.ctypes.data

        def many(lst, dt):
            arr = (C.c_void_p * n_layers)(*[one(a, dt) for a in lst])
            self._keep.append(arr)
            return C.cast(arr, C.POINTER(C.c_void_p))

        m.embed, m.lm_head = one(weights["embed"], np.uint16), one(weights["lm_head"], np.uint16)
        m.norm_f = one(weights["norm_f"], np.float32)
        m.wqkv, m.wo = many(weights["wqkv"], np.uint16), many(weights["wo"], np.uint16)
        m.wgate, m.wup, m.wdown = (many(weights["wgate"], np.uint16), many(weights["wup"], np.uint16),
                                   many(weights["wdown"], np.uint16))
        m.norm1, m.norm2 = many(weights["norm1"], np.float32), many(weights["norm2"], np.float32)
        assert rope.shape[1] == shape.head_dim // 2
        m.rope = one(rope, np.float32)
        self.c = m
        self.n_layers = n_layers
        self.vocab = shape.vocab


class Seq:
    """One sequence with a contiguous fp64 K/V cache."""

    def __init__(self, model: Model, cap: int):
        self.model = model
        self.h = lib().orc_seq_new(C.byref(model.c), cap)
        if not self.h:
            raise MemoryError("orc_seq_new")

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_seq_free(self.h)
            self.h = None

    def __len__(self):
        return lib().orc_seq_len(self.h)

    def truncate(self, n: int):
        if lib().orc_seq_truncate(self.h, n) != 0:
            raise ValueError("truncate")

    def push(self, token: int, want_logits: bool = True):
        if want_logits:
            out = np.empty(self.model.vocab, np.float64)
            rc = lib().orc_seq_push(self.h, int(token), out.ctypes.data_as(C.POINTER(C.c_double)))
        else:
            out, rc = None, lib().orc_seq_push(self.h, int(token), None)
        if rc != 0:
            raise ValueError("orc_seq_push failed (capacity / token range)")
        return out

    def push_traced(self, token: int):
        """Push one token; returns (logits, h) with h[(n_layers+1), d_model] the residual stream of that token after
        the embedding (row 0) and after every layer."""
        h = np.empty((self.model.n_layers + 1, self.model.shape.d_model), np.float64)
        lib().orc_seq_set_trace(self.h, h.ctypes.data_as(C.POINTER(C.c_double)))
        try:
            out = self.push(token)
        finally:
            lib().orc_seq_set_trace(self.h, None)
        return out, h

    def extend(self, tokens):
        """Push tokens, return the logits after the last one (None if empty)."""
        out = None
        tokens = list(tokens)
        for i, t in enumerate(tokens):
            out = self.push(t, want_logits=(i == len(tokens) - 1))
        return out

    def kv(self, layer: int, pos: int):
        w = self.model.shape.n_kv_heads * self.model.shape.head_dim
        k, v = np.empty(w), np.empty(w)
        if lib().orc_seq_kv(self.h, layer, pos, k.ctypes.data_as(C.POINTER(C.c_double)),
                            v.ctypes.data_as(C.POINTER(C.c_double))) != 0:
            raise IndexError("kv")
        return k, v

    def load_kv(self, k, v):
        """Install a given cache: k, v are [n_layers, n, n_kv_heads*head_dim]; afterwards len(self) == n."""
        k = np.ascontiguousarray(k, np.float64)
        v = np.ascontiguousarray(v, np.float64)
        assert k.shape == v.shape and k.shape[0] == self.model.n_layers
        f64p = C.POINTER(C.c_double)
        if lib().orc_seq_load_kv(self.h, k.shape[1], k.ctypes.data_as(f64p), v.ctypes.data_as(f64p)) != 0:
            raise IndexError("load_kv")

    def tree_logits(self, tok, parent, plain: bool = False) -> np.ndarray:
        """Logits of every tree node.  plain=True: the definition (every node's whole path pushed from the cached
        prefix); default: the shared-prefix walk, pinned equal to it bit for bit and n/2 times cheaper on a chain."""
        t, tp = _i32(tok)
        p, pp = _i32(parent)
        out = np.empty((len(t), self.model.vocab), np.float64)
        fn = lib().orc_tree_logits if plain else lib().orc_tree_logits_shared
        if fn(self.h, len(t), tp, pp, out.ctypes.data_as(C.POINTER(C.c_double))) != 0:
            raise ValueError("orc_tree_logits")
        return out

    def accept_greedy_bruteforce(self, tok, parent):
        """Greedy acceptance by definition: plain autoregressive decoding from this cache, then the longest prefix of
        it that the tree spells out.  Returns (a, emitted tokens, path)."""
        t, tp = _i32(tok)
        p, pp = _i32(parent)
        n = len(t)
        out = np.zeros(n + 1, np.int32)
        path = np.zeros(n + 1, np.int32)
        a = lib().orc_accept_greedy_bruteforce(self.h, n, tp, pp, out.ctypes.data_as(C.POINTER(C.c_int32)),
                                               path.ctypes.data_as(C.POINTER(C.c_int32)))
        if a < 0:
            raise ValueError("orc_accept_greedy_bruteforce")
        return a, out[:a + 1].copy(), path[:a + 1].copy()


def threads() -> int:
    return lib().orc_threads()


def argmax(x) -> int:
    a, ap = _f64(x)
    return lib().orc_argmax(ap, len(a))


def attention_row(q, k, v, scale: float) -> np.ndarray:
    """q [h], k/v [n, h] -> [h]."""
    qq, qp = _f64(q)
    kk, kp = _f64(k)
    vv, vp = _f64(v)
    n, h = kk.shape
    out = np.empty(h, np.float64)
    lib().orc_attention_row(qp, kp, vp, n, h, h, scale, out.ctypes.data_as(C.POINTER(C.c_double)))
    return out


def ar_greedy(seq: Seq, last_token: int, n_new: int) -> list:
    """Plain autoregressive greedy decode: `last_token` is the newest committed
    token (its K/V not yet cached); returns the next n_new tokens."""
    out = []
    t = int(last_token)
    for _ in range(n_new):
        t = argmax(seq.push(t))
        out.append(t)
    return out


# ------------------------------------------------------------------ accept

def accept_greedy(tok, parent, arg):
    t, tp = _i32(tok)
    p, pp = _i32(parent)
    a, ap = _i32(arg)
    n = len(t)
    out = np.zeros(n + 1, np.int32)
    path = np.zeros(n + 1, np.int32)
    acc = lib().orc_accept_greedy(n, tp, pp, ap, out.ctypes.data_as(C.POINTER(C.c_int32)),
                                  path.ctypes.data_as(C.POINTER(C.c_int32)))
    return acc, out[:acc + 1].copy(), path[:acc + 1].copy()


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    o = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, o)
    return [int(x) for x in o]


def philox_batch(ctr: np.ndarray, key) -> np.ndarray:
    """ctr uint32 [n, 4] -> uint32 [n, 4]: the generator applied to every counter."""
    c = np.ascontiguousarray(ctr, dtype=np.uint32)
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    out = np.empty_like(c)
    u32p = C.POINTER(C.c_uint32)
    lib().orc_philox_batch(len(c), c.ctypes.data_as(u32p), k, out.ctypes.data_as(u32p))
    return out


def uniform(seed: int, seq_id: int, position: int, draw_kind: int) -> float:
    return lib().orc_uniform(seed, seq_id, position, draw_kind)


def accept_stochastic(tok, parent, pos, logits, temperature: float, seed: int, seq_id: int):
    t, tp = _i32(tok)
    p, pp = _i32(parent)
    ps, psp = _i32(pos)
    lg, lgp = _f64(logits)
    n, V = lg.shape
    out = np.zeros(n + 1, np.int32)
    path = np.zeros(n + 1, np.int32)
    margin = C.c_double()
    acc = lib().orc_accept_stochastic(n, V, tp, pp, psp, lgp, float(temperature), seed, seq_id,
                                      out.ctypes.data_as(C.POINTER(C.c_int32)),
                                      path.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(margin))
    return acc, out[:acc + 1].copy(), path[:acc + 1].copy(), margin.value
