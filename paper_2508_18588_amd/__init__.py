"""Python binding of libhistospec (history-drafted speculative decoding on MI355X).

Argument marshalling only: every step of the path (draft, verify, accept, KV
commit) runs in the HIP kernels behind the C ABI declared in
`include/histospec.h`.  PyTorch is used by callers for device memory and
streams; nothing here computes on tensors.  If the shared library has not been
built the import of the binding fails loudly -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_CSRC = os.path.join(_HERE, "csrc")
LIB_PATH = os.path.join(_HERE, "libhistospec.so")

HS_OK, HS_ERR_INVALID_ARG, HS_ERR_CAPACITY, HS_ERR_UNSUPPORTED, HS_ERR_HIP = 0, -1, -2, -3, -4
HS_DEV_BLOCK_TABLE_OVERFLOW, HS_DEV_POSITION_OVERFLOW, HS_DEV_ROW_OVERFLOW = 1, 2, 4
HS_K_FIXED, HS_K_MATCHLEN, HS_K_AIMD = 0, 1, 2
HS_ACCEPT_GREEDY, HS_ACCEPT_REJECTION = 0, 1
HS_FLAG_REFERENCE_KERNELS, HS_FLAG_FP32_ACTIVATIONS, HS_FLAG_WORKSPACE_LOGITS = 1, 2, 4
HS_GATE_WORDS, HS_GATE_TABLE = 32, 8

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(os.path.join(_CSRC, f) for f in os.listdir(_CSRC) if f.endswith(".hip"))


def build(force: bool = True) -> str:
    """Compile every HIP source for gfx950 into libhistospec.so (in-tree)."""
    srcs = sources()
    deps = srcs + [os.path.join(_CSRC, "hs_internal.h"), os.path.join(_CSRC, "hs_gemm_common.h"), os.path.join(_ROOT, "include", "histospec.h")]
    if not force and os.path.exists(LIB_PATH) and all(os.path.getmtime(LIB_PATH) >= os.path.getmtime(d) for d in deps):
        return LIB_PATH
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    inc = ["-I" + os.path.join(_ROOT, "include"), "-I" + _CSRC]
    # one object per source, compiled side by side, then one link
    import tempfile
    from concurrent.futures import ThreadPoolExecutor
    with tempfile.TemporaryDirectory(prefix="hs_build_") as tmp:
        objs = [os.path.join(tmp, os.path.basename(s_)[:-4] + ".o") for s_ in srcs]
        flags = [f for f in HIPCC_FLAGS if f != "-shared"]

        def one(pair):
            subprocess.check_call([hipcc] + flags + inc + ["-c", pair[0], "-o", pair[1]],
                                  stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)

        with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
            list(ex.map(one, zip(srcs, objs)))
        subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB_PATH],
                              stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    return LIB_PATH


class hs_model_desc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn",
                                         "vocab", "kv_block")] + [("rms_eps", C.c_float)]


class hs_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("lm_head", C.c_void_p), ("norm_f", C.c_void_p),
                ("wqkv", C.POINTER(C.c_void_p)), ("wo", C.POINTER(C.c_void_p)), ("wgate", C.POINTER(C.c_void_p)),
                ("wup", C.POINTER(C.c_void_p)), ("wdown", C.POINTER(C.c_void_p)),
                ("norm1", C.POINTER(C.c_void_p)), ("norm2", C.POINTER(C.c_void_p)), ("rope_cs", C.c_void_p)]


class hs_limits(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("max_batch", "k_max", "c_max", "max_rows", "max_blocks_per_seq", "max_pos",
                                         "w_max", "g_max")]


class hs_kv_cache(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("n_blocks", C.c_int32)]


class hs_seq_state(C.Structure):
    _fields_ = [("batch", C.c_int32), ("seq_len", C.c_void_p), ("block_table", C.c_void_p), ("tail", C.c_void_p),
                ("tail_len", C.c_void_p), ("k_state", C.c_void_p), ("budget_left", C.c_void_p),
                ("seq_id", C.c_void_p), ("tokens", C.c_void_p), ("tokens_stride", C.c_int32),
                ("counters", C.c_void_p), ("gate", C.c_void_p)]


class hs_policy(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("window", "m_min", "k_mode", "k_fixed", "k_max", "aimd_inc", "aimd_cap",
                                         "aimd_reset")]


class hs_draft_args(C.Structure):
    _fields_ = [("n_cand", C.c_int32), ("hist", C.c_void_p), ("hist_off", C.c_void_p), ("policy", hs_policy)]


class hs_group_draft_args(C.Structure):
    _fields_ = [("n_resp", C.c_int32), ("hist", C.c_void_p), ("hist_off", C.c_void_p), ("reward", C.c_void_p),
                ("policy", hs_policy)]


class hs_step(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("draft_start", "match_len", "draft_len", "row_off", "tok", "pos", "parent",
                                          "anc_mask", "row2seq", "logits", "argmax", "accept_len", "n_out",
                                          "out_tok", "path_row")] + [("rows_hint", C.c_int32), ("draft_src", C.c_void_p)]


class hs_accept_args(C.Structure):
    _fields_ = [("mode", C.c_int32), ("temperature", C.c_float), ("seed", C.c_uint64)]


class hs_prefill_args(C.Structure):
    _fields_ = [("chunk", C.c_int32), ("rows_hint", C.c_int32), ("kv_done", C.c_void_p)]


HS_PREFILL_CHUNK_MAX = 1024


EXPORTS = ("hs_create", "hs_destroy", "hs_last_error", "hs_set_flags", "hs_workspace_bytes", "hs_bind_workspace",
           "hs_draft", "hs_draft_group", "hs_verify", "hs_accept", "hs_kv_commit", "hs_poll_error", "hs_debug_buffer",
           "hs_set_profile", "hs_get_profile", "hs_debug_gemm", "hs_gate_table_build", "hs_prefill", "hs_plan_allocation",
           "hs_debug_capture", "hs_debug_capture_bytes", "hs_debug_philox", "hs_draft_static", "hs_accept_commit", "hs_debug_rowmax_groups")

_lib = None


def lib():
    """The loaded C-ABI library.  Raises if it has not been built: there is no other implementation."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run __graft_entry__.build() (hipcc, gfx950) first; "
                               "the HIP library is the only implementation of this path")
        # The library must bind to the HIP runtime PyTorch has loaded: stream handles and device pointers passed
        # across the C ABI belong to that runtime.  Importing torch first makes its libamdhip64 the one in use.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        vp = C.c_void_p
        L.hs_create.argtypes = [C.POINTER(hs_model_desc), C.POINTER(hs_weights), C.POINTER(hs_limits), C.POINTER(vp)]
        L.hs_destroy.argtypes = [vp]
        L.hs_destroy.restype = None
        L.hs_last_error.argtypes = [vp]
        L.hs_last_error.restype = C.c_char_p
        L.hs_set_flags.argtypes = [vp, C.c_uint32]
        L.hs_workspace_bytes.argtypes = [vp]
        L.hs_workspace_bytes.restype = C.c_size_t
        L.hs_bind_workspace.argtypes = [vp, vp, C.c_size_t]
        L.hs_draft.argtypes = [vp, C.POINTER(hs_draft_args), C.POINTER(hs_seq_state), C.POINTER(hs_step), vp]
        L.hs_draft_static.argtypes = [vp, C.POINTER(hs_draft_args), C.POINTER(hs_seq_state), C.POINTER(hs_step), vp]
        L.hs_draft_group.argtypes = [vp, C.POINTER(hs_group_draft_args), C.POINTER(hs_seq_state), C.POINTER(hs_step),
                                     vp]
        L.hs_verify.argtypes = [vp, C.POINTER(hs_kv_cache), C.POINTER(hs_seq_state), C.POINTER(hs_step), vp]
        L.hs_prefill.argtypes = [vp, C.POINTER(hs_kv_cache), C.POINTER(hs_seq_state), C.POINTER(hs_step),
                                 C.POINTER(hs_prefill_args), vp]
        L.hs_accept.argtypes = [vp, C.POINTER(hs_accept_args), C.POINTER(hs_seq_state), C.POINTER(hs_step), vp]
        L.hs_kv_commit.argtypes = [vp, C.POINTER(hs_kv_cache), C.POINTER(hs_seq_state), C.POINTER(hs_step),
                                   C.POINTER(hs_policy), vp]
        L.hs_debug_rowmax_groups.argtypes = [C.c_int32]
        L.hs_accept_commit.argtypes = [vp, C.POINTER(hs_accept_args), C.POINTER(hs_kv_cache), C.POINTER(hs_seq_state),
                                       C.POINTER(hs_step), C.POINTER(hs_policy), vp]
        L.hs_poll_error.argtypes = [vp, vp, C.POINTER(C.c_uint32)]
        L.hs_debug_buffer.argtypes = [vp, C.c_int32, C.POINTER(vp), C.POINTER(C.c_size_t)]
        L.hs_debug_capture_bytes.argtypes = [vp]
        L.hs_debug_capture_bytes.restype = C.c_size_t
        L.hs_debug_capture.argtypes = [vp, vp, C.c_size_t]
        L.hs_debug_philox.argtypes = [vp, C.c_uint64, vp, C.c_int32, vp]
        L.hs_set_profile.argtypes = [vp, C.c_int32]
        L.hs_get_profile.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_int32)]
        L.hs_gate_table_build.argtypes = [C.POINTER(C.c_float), C.POINTER(C.c_int32), C.c_int32, C.c_float, C.c_int32,
                                          C.POINTER(C.c_int32)]
        L.hs_plan_allocation.argtypes = [C.POINTER(C.c_double), C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double,
                                         C.c_double, C.POINTER(C.c_int32), C.POINTER(C.c_double)]
        L.hs_debug_gemm.argtypes = [vp, C.c_int32, vp, vp, vp, vp, vp, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp]
        _lib = L
    return _lib


class HsError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"histospec status {status}: {message}")
        self.status = status


def _check(ctx, status: int):
    if status != HS_OK:
        msg = lib().hs_last_error(ctx).decode() if ctx else ""
        raise HsError(status, msg)


# Same names as the C entry points; each takes the ctypes structs above.

def hs_create(desc: hs_model_desc, weights: hs_weights, limits: hs_limits):
    ctx = C.c_void_p()
    st = lib().hs_create(C.byref(desc), C.byref(weights), C.byref(limits), C.byref(ctx))
    if st != HS_OK:
        raise HsError(st, "hs_create rejected the model shape, weights or limits")
    return ctx


def hs_destroy(ctx):
    lib().hs_destroy(ctx)


def hs_set_flags(ctx, flags: int):
    _check(ctx, lib().hs_set_flags(ctx, flags))


def hs_workspace_bytes(ctx) -> int:
    return lib().hs_workspace_bytes(ctx)


def hs_bind_workspace(ctx, dev_ptr: int, nbytes: int):
    _check(ctx, lib().hs_bind_workspace(ctx, dev_ptr, nbytes))


def hs_draft(ctx, args: hs_draft_args, seq: hs_seq_state, step: hs_step, stream=None):
    _check(ctx, lib().hs_draft(ctx, C.byref(args), C.byref(seq), C.byref(step), stream))


def hs_draft_static(ctx, args: hs_draft_args, seq: hs_seq_state, step: hs_step, stream=None):
    _check(ctx, lib().hs_draft_static(ctx, C.byref(args), C.byref(seq), C.byref(step), stream))


def hs_draft_group(ctx, args: hs_group_draft_args, seq: hs_seq_state, step: hs_step, stream=None):
    _check(ctx, lib().hs_draft_group(ctx, C.byref(args), C.byref(seq), C.byref(step), stream))


def hs_verify(ctx, cache: hs_kv_cache, seq: hs_seq_state, step: hs_step, stream=None):
    _check(ctx, lib().hs_verify(ctx, C.byref(cache), C.byref(seq), C.byref(step), stream))


def hs_prefill(ctx, cache: hs_kv_cache, seq: hs_seq_state, step: hs_step, args: hs_prefill_args, stream=None):
    _check(ctx, lib().hs_prefill(ctx, C.byref(cache), C.byref(seq), C.byref(step), C.byref(args), stream))


def hs_accept(ctx, args: hs_accept_args, seq: hs_seq_state, step: hs_step, stream=None):
    _check(ctx, lib().hs_accept(ctx, C.byref(args), C.byref(seq), C.byref(step), stream))


def hs_kv_commit(ctx, cache: hs_kv_cache, seq: hs_seq_state, step: hs_step, policy: hs_policy, stream=None):
    _check(ctx, lib().hs_kv_commit(ctx, C.byref(cache), C.byref(seq), C.byref(step), C.byref(policy), stream))


def hs_accept_commit(ctx, args: hs_accept_args, cache: hs_kv_cache, seq: hs_seq_state, step: hs_step,
                     policy: hs_policy, stream=None):
    _check(ctx, lib().hs_accept_commit(ctx, C.byref(args), C.byref(cache), C.byref(seq), C.byref(step),
                                       C.byref(policy), stream))


def hs_poll_error(ctx, stream=None) -> int:
    bits = C.c_uint32()
    _check(ctx, lib().hs_poll_error(ctx, stream, C.byref(bits)))
    return bits.value


def hs_debug_buffer(ctx, which: int):
    p, n = C.c_void_p(), C.c_size_t()
    _check(ctx, lib().hs_debug_buffer(ctx, which, C.byref(p), C.byref(n)))
    return p.value, n.value


def hs_debug_capture_bytes(ctx) -> int:
    return lib().hs_debug_capture_bytes(ctx)


def hs_debug_capture(ctx, dev_ptr, nbytes: int):
    _check(ctx, lib().hs_debug_capture(ctx, dev_ptr, nbytes))


def hs_debug_philox(ctr_dev: int, seed: int, out_dev: int, n: int, stream=None):
    st = lib().hs_debug_philox(ctr_dev, seed, out_dev, n, stream)
    if st != HS_OK:
        raise HsError(st, "hs_debug_philox")


def hs_set_profile(ctx, level: int):
    _check(ctx, lib().hs_set_profile(ctx, int(level)))


def hs_debug_gemm(ctx, epi: int, a: int, w: int, w2: int, c: int, m_dev: int, m_max: int, n: int, k: int,
                  rows_hint: int, stream):
    _check(ctx, lib().hs_debug_gemm(ctx, epi, a, w, w2 or None, c, m_dev, m_max, n, k, rows_hint, stream))


def hs_debug_rowmax_groups(n: int) -> int:
    return lib().hs_debug_rowmax_groups(n)


def hs_gate_table_build(ms, rows, k_bar: float, b_max: int):
    """Table of the speculation gate (17 ints) from a profiled step time; host arithmetic in the library."""
    n = len(ms)
    m = (C.c_float * n)(*[float(x) for x in ms])
    r = (C.c_int32 * n)(*[int(x) for x in rows])
    out = (C.c_int32 * 17)()
    st = lib().hs_gate_table_build(m, r, n, float(k_bar), int(b_max), out)
    if st != HS_OK:
        raise HsError(st, "hs_gate_table_build rejected the profile")
    return list(out)


def hs_plan_allocation(tau, min_wks: int, max_wks: int, wks: int, t_train: float, precision: float = 1.0):
    """Tier-2 planner: tau[i][k - min_wks] = time of ranking group i on k workers -> (plan, d); raises HsError
    (HS_ERR_CAPACITY) if the cluster cannot meet any gradient of the search interval.  Host arithmetic only."""
    n = len(tau)
    vals = [float(x) for row in tau for x in row]
    flat = (C.c_double * max(1, len(vals)))(*vals)
    plan = (C.c_int32 * max(1, n))()
    d = C.c_double()
    st = lib().hs_plan_allocation(flat, n, min_wks, max_wks, wks, float(t_train), float(precision), plan, C.byref(d))
    if st != HS_OK:
        raise HsError(st, "hs_plan_allocation: no feasible plan" if st == HS_ERR_CAPACITY else "hs_plan_allocation")
    return list(plan), d.value


def hs_get_profile(ctx):
    ms = (C.c_float * 5)()
    n = (C.c_int32 * 5)()
    _check(ctx, lib().hs_get_profile(ctx, ms, n))
    return list(ms), list(n)
