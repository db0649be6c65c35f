"""Device-memory plumbing around the C ABI: allocates the caller-owned tensors (weights, paged KV cache,
sequence state, per-step arrays, workspace) with PyTorch, fills the ctypes structs with their addresses, and
enqueues the four calls on the current HIP stream.  No step of the decoding path is computed here.
"""
from __future__ import annotations

import ctypes as C
from dataclasses import dataclass

import numpy as np
import torch

from . import (HS_FLAG_WORKSPACE_LOGITS, hs_accept_commit, HS_FLAG_FP32_ACTIVATIONS, hs_debug_capture, hs_debug_capture_bytes, HS_ACCEPT_GREEDY, HS_GATE_TABLE, HS_GATE_WORDS, HS_K_FIXED, hs_gate_table_build, hs_accept, hs_accept_args, hs_bind_workspace, hs_create, hs_debug_buffer, hs_debug_gemm,
               hs_destroy, hs_draft, hs_draft_args, hs_draft_group, hs_group_draft_args, hs_get_profile, hs_kv_cache, hs_kv_commit, hs_limits,
               hs_model_desc, hs_policy, hs_poll_error, hs_prefill, hs_prefill_args, hs_seq_state, hs_set_flags, hs_set_profile, hs_step,
               hs_verify, hs_weights, hs_workspace_bytes)


@dataclass
class Policy:
    window: int = 8
    m_min: int = 3
    k_mode: int = HS_K_FIXED
    k_fixed: int = 4
    k_max: int = 4
    aimd_init: int = 2
    aimd_inc: int = 2
    aimd_cap: int = 32
    aimd_reset: int = 2

    def c(self) -> hs_policy:
        return hs_policy(self.window, self.m_min, self.k_mode, self.k_fixed, self.k_max, self.aimd_inc,
                         self.aimd_cap, self.aimd_reset)


def _dev(a, dtype=None):
    if isinstance(a, torch.Tensor):
        return a.cuda().contiguous()
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    t = torch.from_numpy(a).cuda()
    return t if dtype is None else t.to(dtype)


class Engine:
    """Owns every device tensor of one in-flight batch and the library context built on them."""

    def __init__(self, shape, weights: dict, rope, max_batch: int, k_max: int, c_max: int, max_len: int,
                 w_max: int = 32, seq_caps=None, shuffle_pages_seed: int | None = None, n_layers: int | None = None,
                 keep_logits: bool = True, g_max: int = 0, max_rows: int | None = None, precise: bool = False,
                 workspace_logits: bool = False):
        """keep_logits: give every step a [max_rows, vocab] fp32 logits tensor (hs_step.logits); without it (and
        without workspace_logits, which keeps them inside the library's workspace) no logits array exists and the
        argmax comes out of the LM head's epilogue.  precise: run in the library's fp32-activation mode (plain
        kernels, float KV cache)."""
        self.shape = shape
        self.dev = torch.device("cuda:0")
        L = len(weights["wqkv"]) if n_layers is None else n_layers
        self.n_layers = L
        self.max_batch, self.k_max, self.c_max, self.w_max = max_batch, k_max, c_max, w_max
        nodes = 1 + c_max * k_max
        # rows of one call: a verify step needs max_batch * nodes; a larger value lets hs_prefill take bigger bites
        self.max_rows = max(max_batch * nodes, max_rows or 0)
        # ---- weights
        self.w = {k: ([_dev(x) for x in v] if isinstance(v, list) else _dev(v)) for k, v in weights.items()}
        self.rope = _dev(rope)
        self.max_pos = int(self.rope.shape[0])
        # ---- pages: sequence b may hold up to seq_caps[b] tokens (plus the draft nodes of one step)
        caps = [max_len] * max_batch if seq_caps is None else list(seq_caps)
        need = [(c + nodes + 15) // 16 for c in caps]
        self.max_blocks = max(need)
        self.n_blocks = int(sum(need))
        ids = np.arange(self.n_blocks, dtype=np.int32)
        if shuffle_pages_seed is not None:
            np.random.default_rng(shuffle_pages_seed).shuffle(ids)
        bt = np.full((max_batch, self.max_blocks), -1, np.int32)
        o = 0
        for b, n in enumerate(need):
            bt[b, :n] = ids[o:o + n]
            o += n
        self.block_table = _dev(bt)
        kv_elems = L * self.n_blocks * shape.n_kv_heads * 16 * shape.head_dim
        self.precise = precise
        kv_dtype = torch.float32 if precise else torch.int16
        self.kc = torch.zeros(kv_elems, dtype=kv_dtype, device=self.dev)
        self.vc = torch.zeros(kv_elems, dtype=kv_dtype, device=self.dev)
        # ---- context
        desc = hs_model_desc(L, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                             shape.vocab, 16, shape.rms_eps)
        self._keep = []

        def parr(lst):
            arr = (C.c_void_p * L)(*[t.data_ptr() for t in lst[:L]])
            self._keep.append(arr)
            return C.cast(arr, C.POINTER(C.c_void_p))

        w = self.w
        hw = hs_weights(w["embed"].data_ptr(), w["lm_head"].data_ptr(), w["norm_f"].data_ptr(), parr(w["wqkv"]),
                        parr(w["wo"]), parr(w["wgate"]), parr(w["wup"]), parr(w["wdown"]), parr(w["norm1"]),
                        parr(w["norm2"]), self.rope.data_ptr())
        self.g_max = g_max
        lim = hs_limits(max_batch, k_max, c_max, self.max_rows, self.max_blocks, self.max_pos, w_max, g_max)
        self.ctx = hs_create(desc, hw, lim)
        self.flags = (HS_FLAG_FP32_ACTIVATIONS if precise else 0) | (HS_FLAG_WORKSPACE_LOGITS if workspace_logits else 0)
        if self.flags:
            hs_set_flags(self.ctx, self.flags)   # before the workspace is sized
        self.workspace = None
        self._bind_workspace()
        # ---- sequence state and step arrays
        i32 = dict(dtype=torch.int32, device=self.dev)
        B, M = max_batch, self.max_rows
        self.seq_len = torch.zeros(B, **i32)
        self.tail = torch.zeros(B, w_max, **i32)
        self.tail_len = torch.zeros(B, **i32)
        self.k_state = torch.zeros(B, **i32)
        self.budget_left = torch.zeros(B, **i32)
        self.seq_id = torch.zeros(B, dtype=torch.int64, device=self.dev)
        self.tokens_stride = max(caps) + nodes
        self.tokens = torch.zeros(B, self.tokens_stride, **i32)
        self.counters = torch.zeros(4, dtype=torch.int64, device=self.dev)
        self.gate = None
        self.st = {n: torch.zeros(B * c_max, **i32) for n in ("draft_start", "match_len", "draft_len")}
        self.st["draft_src"] = torch.zeros(B, **i32)
        self.st.update({n: torch.zeros(M, **i32) for n in ("tok", "pos", "parent", "row2seq", "argmax")})
        self.st["row_off"] = torch.zeros(B + 1, **i32)
        self.st["anc_mask"] = torch.zeros(M, dtype=torch.int64, device=self.dev)
        self.st.update({n: torch.zeros(B, **i32) for n in ("accept_len", "n_out")})
        self.st.update({n: torch.zeros(B, k_max + 1, **i32) for n in ("out_tok", "path_row")})
        self.logits = torch.zeros(M, shape.vocab, dtype=torch.float32, device=self.dev) if keep_logits else None
        self.batch = 0
        self.hist = None
        self.hist_off = None
        self.n_cand = 1
        self._structs()

    def _bind_workspace(self):
        """(Re)allocate the workspace if the current flags need more than is bound."""
        nbytes = hs_workspace_bytes(self.ctx)
        if self.workspace is None or self.workspace.numel() < nbytes + 256:
            self.workspace = torch.zeros(nbytes + 256, dtype=torch.uint8, device=self.dev)
            self._ws_ptr = (self.workspace.data_ptr() + 255) // 256 * 256
        hs_bind_workspace(self.ctx, self._ws_ptr, nbytes)

    def _structs(self):
        s = self.st
        self.c_cache = hs_kv_cache(self.kc.data_ptr(), self.vc.data_ptr(), self.n_blocks)
        self.c_seq = hs_seq_state(self.batch, self.seq_len.data_ptr(), self.block_table.data_ptr(),
                                  self.tail.data_ptr(), self.tail_len.data_ptr(), self.k_state.data_ptr(),
                                  self.budget_left.data_ptr(), self.seq_id.data_ptr(), self.tokens.data_ptr(),
                                  self.tokens_stride, self.counters.data_ptr(),
                                  self.gate.data_ptr() if self.gate is not None else None)
        self.c_step = hs_step(s["draft_start"].data_ptr(), s["match_len"].data_ptr(), s["draft_len"].data_ptr(),
                              s["row_off"].data_ptr(), s["tok"].data_ptr(), s["pos"].data_ptr(),
                              s["parent"].data_ptr(), s["anc_mask"].data_ptr(), s["row2seq"].data_ptr(),
                              self.logits.data_ptr() if self.logits is not None else None, s["argmax"].data_ptr(),
                              s["accept_len"].data_ptr(), s["n_out"].data_ptr(), s["out_tok"].data_ptr(),
                              s["path_row"].data_ptr(), getattr(self, "rows_hint", 0), s["draft_src"].data_ptr())

    def close(self):
        if self.ctx:
            torch.cuda.synchronize()
            hs_destroy(self.ctx)
            self.ctx = None

    def stream(self):
        return torch.cuda.current_stream().cuda_stream

    # ---------------------------------------------------------------- state loading (inputs only)

    def load_sequences(self, token_lists, budgets, seq_ids=None, k_init: int = 2):
        """Set the committed tokens of each sequence (no K/V is computed here)."""
        B = len(token_lists)
        assert 1 <= B <= self.max_batch
        self.batch = B
        tok = np.zeros((self.max_batch, self.tokens_stride), np.int32)
        tail = np.zeros((self.max_batch, self.w_max), np.int32)
        tl = np.zeros(self.max_batch, np.int32)
        sl = np.zeros(self.max_batch, np.int32)
        for b, t in enumerate(token_lists):
            t = np.asarray(t, np.int32)
            n = len(t)
            tok[b, :n] = t
            m = min(n, self.w_max)
            tail[b, self.w_max - m:] = t[n - m:]
            tl[b], sl[b] = m, n
        self.tokens.copy_(torch.from_numpy(tok))
        self.tail.copy_(torch.from_numpy(tail))
        self.tail_len.copy_(torch.from_numpy(tl))
        self.seq_len.copy_(torch.from_numpy(sl))
        self._lens = sl.astype(np.int64)
        bl = np.zeros(self.max_batch, np.int32)
        bl[:B] = budgets
        self.budget_left.copy_(torch.from_numpy(bl))
        sid = np.arange(self.max_batch, dtype=np.int64) if seq_ids is None else np.asarray(seq_ids, np.int64)
        self.seq_id[:len(sid)].copy_(torch.from_numpy(sid))
        self.k_state.fill_(k_init)
        self.counters.zero_()
        self._structs()

    def set_history(self, cands):
        """cands[b][c] = int array: candidate c of sequence b (already carrying its prompt context)."""
        self.n_cand = len(cands[0])
        flat, off = [], [0]
        for row in cands:
            assert len(row) == self.n_cand
            for h in row:
                flat.append(np.asarray(h, np.int32))
                off.append(off[-1] + len(h))
        self.hist = _dev(np.concatenate(flat) if off[-1] else np.zeros(1, np.int32))
        self.hist_off = _dev(np.asarray(off, np.int32))

    # ---------------------------------------------------------------- the four calls

    def draft(self, policy: Policy):
        args = hs_draft_args(self.n_cand, self.hist.data_ptr(), self.hist_off.data_ptr(), policy.c())
        hs_draft(self.ctx, args, self.c_seq, self.c_step, self.stream())

    def set_group_history(self, groups, rewards):
        """groups[b][g] = int array: response g of sequence b's prompt in its last rollout (already carrying its
        prompt context); rewards[b][g] = the reward it earned (non-negative int)."""
        self.n_resp = len(groups[0])
        flat, off, rew = [], [0], []
        for row, rr in zip(groups, rewards):
            assert len(row) == self.n_resp == len(rr)
            for h, r in zip(row, rr):
                flat.append(np.asarray(h, np.int32))
                off.append(off[-1] + len(h))
                rew.append(int(r))
        self.ghist = _dev(np.concatenate(flat) if off[-1] else np.zeros(1, np.int32))
        self.ghist_off = _dev(np.asarray(off, np.int32))
        self.greward = _dev(np.asarray(rew, np.int32))

    def draft_group(self, policy: Policy):
        args = hs_group_draft_args(self.n_resp, self.ghist.data_ptr(), self.ghist_off.data_ptr(),
                                   self.greward.data_ptr(), policy.c())
        hs_draft_group(self.ctx, args, self.c_seq, self.c_step, self.stream())

    def step_group(self, policy: Policy, mode: int = HS_ACCEPT_GREEDY, temperature: float = 1.0, seed: int = 0):
        self.draft_group(policy)
        self.verify()
        self.accept_commit(policy, mode, temperature, seed)

    def set_rows_hint(self, rows: int):
        """Tell the library how many rows to expect (a launch-shape hint; results do not depend on it)."""
        self.rows_hint = int(rows)
        self.c_step.rows_hint = self.rows_hint

    def verify(self):
        hs_verify(self.ctx, self.c_cache, self.c_seq, self.c_step, self.stream())

    def accept(self, mode: int = HS_ACCEPT_GREEDY, temperature: float = 1.0, seed: int = 0):
        hs_accept(self.ctx, hs_accept_args(mode, temperature, seed), self.c_seq, self.c_step, self.stream())

    def commit(self, policy: Policy):
        hs_kv_commit(self.ctx, self.c_cache, self.c_seq, self.c_step, policy.c(), self.stream())

    def accept_commit(self, policy: Policy, mode: int = HS_ACCEPT_GREEDY, temperature: float = 1.0, seed: int = 0):
        hs_accept_commit(self.ctx, hs_accept_args(mode, temperature, seed), self.c_cache, self.c_seq, self.c_step,
                         policy.c(), self.stream())

    def step(self, policy: Policy, mode: int = HS_ACCEPT_GREEDY, temperature: float = 1.0, seed: int = 0):
        self.draft(policy)
        self.verify()
        self.accept_commit(policy, mode, temperature, seed)

    def capture_step(self, policy: Policy, mode: int = HS_ACCEPT_GREEDY, temperature: float = 1.0, seed: int = 0):
        """Record one whole decode iteration (draft, verify, accept + commit) into a HIP graph and return it; every
        `graph.replay()` then runs one iteration.  Possible because nothing in an iteration depends on host values
        that change from step to step: the row count and every offset live on the device, launch shapes follow the
        row hint that was set when the graph was recorded.  Run a few eager steps with the same hint first (kernel
        attributes are set on a kernel's first launch), and keep profiling off."""
        g = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            self.draft(policy)
            self.verify()
            self.accept_commit(policy, mode, temperature, seed)
        return g

    def set_gate(self, table, probe_every: int = 0):
        """Switch on throughput-aware speculation control with this 17-entry table (None: off).  The monitor starts
        empty and picks the counters up where they stand."""
        if table is None:
            self.gate = None
        else:
            assert len(table) == 17
            g = np.zeros(HS_GATE_WORDS, np.int32)
            g[4] = probe_every
            c = self.counters.cpu().numpy().astype(np.uint64)
            g[5], g[6] = np.uint32(c[1] & 0xFFFFFFFF).astype(np.int32), np.uint32(c[2] & 0xFFFFFFFF).astype(np.int32)
            g[HS_GATE_TABLE:HS_GATE_TABLE + 17] = table
            self.gate = _dev(g)
        self._structs()

    @staticmethod
    def gate_table(ms, rows, k_bar: float, b_max: int):
        return hs_gate_table_build(ms, rows, k_bar, b_max)

    def poll_error(self) -> int:
        return hs_poll_error(self.ctx, self.stream())

    def set_flags(self, flags: int):
        """Replace the context's flags (a larger workspace is bound if the new layout needs one)."""
        torch.cuda.synchronize()
        self.flags = flags
        hs_set_flags(self.ctx, flags)
        self._bind_workspace()

    def set_profile(self, level: int):
        """0 off, 1 events around the attention kernel and the whole call, 2 around every launch of hs_verify."""
        hs_set_profile(self.ctx, int(level))

    def get_profile(self):
        return hs_get_profile(self.ctx)

    def gemm(self, epi: int, a, w, w2, c, m_dev, m_max: int, rows_hint: int = 0):
        """One projection through hs_debug_gemm: a [m_max, k] bf16 bits, w (and w2) [n, k] bf16 bits, c [m_max, n]
        (f32 for epi 0/1, bf16 bits for epi 2), m_dev an int32 device tensor holding the live row count."""
        n, k = int(w.shape[0]), int(w.shape[1])
        hs_debug_gemm(self.ctx, epi, a.data_ptr(), w.data_ptr(), 0 if w2 is None else w2.data_ptr(), c.data_ptr(),
                      m_dev.data_ptr(), m_max, n, k, rows_hint, self.stream())

    # ---------------------------------------------------------------- hand-made rows (prefill, tests)

    def set_rows(self, per_seq):
        """Install explicit node arrays instead of calling hs_draft: per_seq[b] = dict(tok, parent, pos) or None.
        Used to push prompt chunks through hs_verify and by kernel tests."""
        B = self.batch
        ro = np.zeros(self.max_batch + 1, np.int32)
        tok = np.zeros(self.max_rows, np.int32)
        pos = np.zeros(self.max_rows, np.int32)
        par = np.zeros(self.max_rows, np.int32)
        r2s = np.zeros(self.max_rows, np.int32)
        anc = np.zeros(self.max_rows, np.uint64)
        r = 0
        for b in range(B):
            ro[b] = r
            d = per_seq[b]
            if d is None:
                continue
            n = len(d["tok"])
            for i in range(n):
                p = int(d["parent"][i])
                anc[r + i] = (np.uint64(1) << np.uint64(i)) | (anc[r + p] if p >= 0 else np.uint64(0))
            tok[r:r + n], pos[r:r + n], par[r:r + n], r2s[r:r + n] = d["tok"], d["pos"], d["parent"], b
            r += n
        ro[B:] = r
        s = self.st
        s["row_off"].copy_(torch.from_numpy(ro[:self.max_batch + 1]))
        s["tok"].copy_(torch.from_numpy(tok))
        s["pos"].copy_(torch.from_numpy(pos))
        s["parent"].copy_(torch.from_numpy(par))
        s["row2seq"].copy_(torch.from_numpy(r2s))
        s["anc_mask"].copy_(torch.from_numpy(anc.view(np.int64)))
        return r

    def prefill(self, token_lists):
        """Write the K/V of every token but the last of each sequence by pushing chunks of up to
        1 + c_max*k_max tokens through hs_verify as teacher-forced chains."""
        chunk = 1 + self.c_max * self.k_max
        todo = [len(t) - 1 for t in token_lists]
        done = [0] * len(token_lists)
        saved = self.seq_len.clone()
        while any(d < t for d, t in zip(done, todo)):
            rows, sl = [], saved.cpu().numpy().copy()
            for b, t in enumerate(token_lists):
                n = min(chunk, todo[b] - done[b])
                if n <= 0:
                    rows.append(None)
                    continue
                c0 = done[b]
                rows.append(dict(tok=np.asarray(t[c0:c0 + n], np.int32), parent=np.arange(-1, n - 1),
                                 pos=np.arange(c0, c0 + n)))
                sl[b] = c0 + 1
                done[b] += n
            self.seq_len.copy_(torch.from_numpy(sl))
            self.set_rows(rows)
            self.verify()
        self.seq_len.copy_(saved)
        torch.cuda.synchronize()

    def prefill_chunked(self, chunk: int = 512, kv_done=None):
        """Recompute the cache of every loaded sequence's committed text (all tokens but the newest) with hs_prefill,
        `chunk` tokens per sequence and call; kv_done = positions already cached (default none).  Returns the number
        of calls.  The lengths are host knowledge (load_sequences), so no device value is read back."""
        B = self.batch
        todo = np.maximum(self._lens[:B] - 1 - (np.zeros(B, np.int64) if kv_done is None else np.asarray(kv_done)), 0)
        self.kv_done = torch.zeros(self.max_batch, dtype=torch.int32, device=self.dev)
        if kv_done is not None:
            self.kv_done[:B].copy_(torch.as_tensor(np.asarray(kv_done, np.int32)))
        calls = 0
        while todo.sum() > 0:
            # the library serves sequences in index order until max_rows rows are laid out: mirror that here
            left = self.max_rows
            for b in range(B):
                n = int(min(chunk, todo[b], left))
                todo[b] -= n
                left -= n
            args = hs_prefill_args(int(chunk), int(self.max_rows - left), self.kv_done.data_ptr())
            hs_prefill(self.ctx, self.c_cache, self.c_seq, self.c_step, args, self.stream())
            calls += 1
        return calls

    def capture_last_layer(self):
        """Switch on hs_debug_capture; returns the four snapshot slots as flat uint8 views (see the header)."""
        n = hs_debug_capture_bytes(self.ctx)
        self._capture = torch.zeros(n, dtype=torch.uint8, device=self.dev)
        hs_debug_capture(self.ctx, self._capture.data_ptr(), n)
        return [self._capture[i * (n // 4):(i + 1) * (n // 4)] for i in range(4)]

    def debug_tensor(self, which: int):
        """0 final hidden (bf16 bits), 1 queries, 2 attention output, 3 workspace logits, 4 residual stream (f32),
        5 feed-forward activation -- as flat uint8 torch views."""
        ptr, n = hs_debug_buffer(self.ctx, which)
        off = ptr - self.workspace.data_ptr()
        return self.workspace[off:off + n]
