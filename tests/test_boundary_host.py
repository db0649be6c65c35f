"""Host-only checks of the C-ABI boundary: the library loads, exports every function the header declares, and
rejects bad arguments with a status code before anything is launched (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

import paper_2508_18588_amd as hs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(hs.LIB_PATH):
        hs.build()
    return hs.lib()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "histospec.h")).read()
    declared = set(re.findall(r"^\s*(?:hs_status|void|size_t|int32_t|const char\*)\s+(hs_[a-z_]+)\(", header, re.M))
    assert declared == set(hs.EXPORTS), declared ^ set(hs.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_sizes_match_the_header_layout():
    assert C.sizeof(hs.hs_model_desc) == 36
    assert C.sizeof(hs.hs_limits) == 32
    assert C.sizeof(hs.hs_policy) == 32
    assert C.sizeof(hs.hs_weights) == 11 * 8
    assert C.sizeof(hs.hs_step) == 17 * 8
    assert C.sizeof(hs.hs_group_draft_args) == 8 + 3 * 8 + 32
    assert C.sizeof(hs.hs_accept_args) == 16
    assert C.sizeof(hs.hs_prefill_args) == 16
    assert C.sizeof(hs.hs_kv_cache) == 24


def _good():
    desc = hs.hs_model_desc(2, 256, 4, 4, 64, 1024, 4096, 16, 1e-6)
    L = 2
    fake = 0x1000  # never dereferenced on the host
    arr = (C.c_void_p * L)(fake, fake)
    p = C.cast(arr, C.POINTER(C.c_void_p))
    w = hs.hs_weights(fake, fake, fake, p, p, p, p, p, p, p, fake)
    lim = hs.hs_limits(4, 4, 1, 20, 32, 512, 8)
    return desc, w, lim, arr


def test_create_validates_shape_and_limits(lib):
    desc, w, lim, keep = _good()
    ctx = hs.hs_create(desc, w, lim)
    assert hs.hs_workspace_bytes(ctx) > 0
    hs.hs_destroy(ctx)

    def status(d=None, ww=None, ll=None):
        out = C.c_void_p()
        return lib.hs_create(C.byref(d or desc), C.byref(ww or w), C.byref(ll or lim), C.byref(out))

    bad = hs.hs_model_desc(2, 256, 4, 4, 96, 1024, 4096, 16, 1e-6)       # head_dim 96
    assert status(d=bad) == hs.HS_ERR_UNSUPPORTED
    bad = hs.hs_model_desc(2, 256, 4, 4, 64, 1024, 4096, 32, 1e-6)       # page size 32
    assert status(d=bad) == hs.HS_ERR_UNSUPPORTED
    bad = hs.hs_model_desc(2, 256, 4, 3, 64, 1024, 4096, 16, 1e-6)       # heads not divisible
    assert status(d=bad) == hs.HS_ERR_UNSUPPORTED
    bad = hs.hs_model_desc(0, 256, 4, 4, 64, 1024, 4096, 16, 1e-6)
    assert status(d=bad) == hs.HS_ERR_INVALID_ARG
    bad = hs.hs_model_desc(2, 16448, 4, 4, 64, 1024, 4096, 16, 1e-6)     # d_model beyond the row kernels' 16384
    assert status(d=bad) == hs.HS_ERR_UNSUPPORTED
    w3 = hs.hs_weights(0x1000, 0x1000, 0x1004, w.wqkv, w.wo, w.wgate, w.wup, w.wdown, w.norm1, w.norm2, 0x1000)
    assert status(ww=w3) == hs.HS_ERR_INVALID_ARG                         # norm weights not 16-byte aligned
    assert status(ll=hs.hs_limits(4, 33, 1, 200, 32, 512, 8)) == hs.HS_ERR_INVALID_ARG      # k_max > 32
    assert status(ll=hs.hs_limits(4, 32, 2, 400, 32, 512, 8)) == hs.HS_ERR_UNSUPPORTED      # 65 nodes
    assert status(ll=hs.hs_limits(4, 4, 1, 19, 32, 512, 8)) == hs.HS_ERR_CAPACITY           # too few rows
    w2 = hs.hs_weights(None, 0x1000, 0x1000, w.wqkv, w.wo, w.wgate, w.wup, w.wdown, w.norm1, w.norm2, 0x1000)
    assert status(ww=w2) == hs.HS_ERR_INVALID_ARG
    assert lib.hs_create(None, None, None, None) == hs.HS_ERR_INVALID_ARG


def test_calls_reject_bad_arguments_without_launching(lib):
    desc, w, lim, keep = _good()
    ctx = hs.hs_create(desc, w, lim)
    seq, step, cache = hs.hs_seq_state(), hs.hs_step(), hs.hs_kv_cache()
    # no workspace bound yet
    with pytest.raises(hs.HsError) as e:
        hs.hs_verify(ctx, cache, seq, step)
    assert e.value.status == hs.HS_ERR_CAPACITY and "workspace" in str(e.value)
    with pytest.raises(hs.HsError) as e:
        hs.hs_bind_workspace(ctx, 0x1001, 1 << 40)   # misaligned
    assert e.value.status == hs.HS_ERR_INVALID_ARG
    with pytest.raises(hs.HsError) as e:
        hs.hs_bind_workspace(ctx, 0x1000, 16)        # too small
    assert e.value.status == hs.HS_ERR_CAPACITY
    hs.hs_bind_workspace(ctx, 0x100000, 1 << 40)     # address only recorded, never touched by these checks
    pol = hs.hs_policy(8, 3, hs.HS_K_FIXED, 4, 4, 2, 32, 2)
    args = hs.hs_draft_args(1, 0x1000, 0x1000, pol)
    for call in (lambda: hs.hs_draft(ctx, args, seq, step), lambda: hs.hs_verify(ctx, cache, seq, step),
                 lambda: hs.hs_accept(ctx, hs.hs_accept_args(0, 1.0, 0), seq, step),
                 lambda: hs.hs_kv_commit(ctx, cache, seq, step, pol)):
        with pytest.raises(hs.HsError) as e:
            call()
        assert e.value.status == hs.HS_ERR_INVALID_ARG   # null state / step arrays
    full = hs.hs_seq_state(5, *([0x1000] * 7), None, 0, None)   # batch 5 > max_batch 4
    with pytest.raises(hs.HsError):
        hs.hs_draft(ctx, args, full, step)
    ok_seq = hs.hs_seq_state(4, *([0x1000] * 7), None, 0, None)
    ok_step = hs.hs_step(*([0x1000] * 15), 0)
    for bad_pol in (hs.hs_policy(9, 3, 0, 4, 4, 2, 32, 2),     # window > w_max
                    hs.hs_policy(8, 9, 0, 4, 4, 2, 32, 2),     # m_min > window
                    hs.hs_policy(8, 3, 7, 4, 4, 2, 32, 2),     # unknown k_mode
                    hs.hs_policy(8, 3, 0, 4, 5, 2, 32, 2)):    # k_max beyond the limit
        with pytest.raises(hs.HsError) as e:
            hs.hs_draft(ctx, hs.hs_draft_args(1, 0x1000, 0x1000, bad_pol), ok_seq, ok_step)
        assert e.value.status == hs.HS_ERR_INVALID_ARG
    with pytest.raises(hs.HsError) as e:
        hs.hs_draft(ctx, hs.hs_draft_args(2, 0x1000, 0x1000, pol), ok_seq, ok_step)   # n_cand > c_max
    assert e.value.status == hs.HS_ERR_CAPACITY
    with pytest.raises(hs.HsError):
        hs.hs_accept(ctx, hs.hs_accept_args(hs.HS_ACCEPT_REJECTION, 0.0, 0), ok_seq, ok_step)  # temperature 0
    with pytest.raises(hs.HsError):
        hs.hs_accept(ctx, hs.hs_accept_args(5, 1.0, 0), ok_seq, ok_step)
    with pytest.raises(hs.HsError):
        hs.hs_set_flags(ctx, 0x80)
    hs.hs_destroy(ctx)


def test_flags_change_the_workspace_layout_and_new_entry_points_check_their_arguments(lib):
    """Host-side behaviour of what sits around the four calls: the fp32-activation and workspace-logits flags change
    hs_workspace_bytes and drop a binding that no longer fits; rejection sampling without logits is refused before
    anything is launched; hs_accept_commit, hs_draft_static, hs_debug_capture and hs_debug_philox validate their
    arguments; the LM head's row-maximum epilogue reports its number of column groups."""
    desc, w, lim, keep = _good()
    ctx = hs.hs_create(desc, w, lim)
    base = hs.hs_workspace_bytes(ctx)
    hs.hs_bind_workspace(ctx, 0x100000, base)
    hs.hs_set_flags(ctx, hs.HS_FLAG_WORKSPACE_LOGITS)
    with_logits = hs.hs_workspace_bytes(ctx)
    assert with_logits >= base + lim.max_rows * desc.vocab * 4                   # an [rows][vocab] fp32 array appears
    seq, step, cache = hs.hs_seq_state(), hs.hs_step(), hs.hs_kv_cache()
    with pytest.raises(hs.HsError) as e:                                          # the old binding was dropped
        hs.hs_verify(ctx, cache, seq, step)
    assert e.value.status == hs.HS_ERR_CAPACITY and "workspace" in str(e.value)
    hs.hs_set_flags(ctx, hs.HS_FLAG_FP32_ACTIVATIONS)                             # plain kernels keep logits too
    assert hs.hs_workspace_bytes(ctx) > with_logits                               # and activations take 4 bytes
    hs.hs_set_flags(ctx, 0)
    assert hs.hs_workspace_bytes(ctx) == base
    hs.hs_bind_workspace(ctx, 0x100000, 1 << 40)
    pol = hs.hs_policy(8, 3, hs.HS_K_FIXED, 4, 4, 2, 32, 2)
    ok_seq = hs.hs_seq_state(4, *([0x1000] * 7), None, 0, None)
    ok_step = hs.hs_step(*([0x1000] * 9), None, *([0x1000] * 5), 0)              # no logits destination
    with pytest.raises(hs.HsError) as e:
        hs.hs_accept(ctx, hs.hs_accept_args(hs.HS_ACCEPT_REJECTION, 1.0, 0), ok_seq, ok_step)
    assert e.value.status == hs.HS_ERR_INVALID_ARG and "logits" in str(e.value)
    with pytest.raises(hs.HsError) as e:
        hs.hs_accept_commit(ctx, hs.hs_accept_args(hs.HS_ACCEPT_REJECTION, 1.0, 0), hs.hs_kv_cache(0x1000, 0x1000, 8),
                            ok_seq, ok_step, pol)
    assert "logits" in str(e.value)
    for call in (lambda: hs.hs_accept_commit(ctx, hs.hs_accept_args(0, 1.0, 0), cache, ok_seq, ok_step, pol),    # null cache
                 lambda: hs.hs_accept_commit(ctx, hs.hs_accept_args(7, 1.0, 0), hs.hs_kv_cache(0x1000, 0x1000, 8),
                                             ok_seq, ok_step, pol),                                              # mode
                 lambda: hs.hs_draft_static(ctx, hs.hs_draft_args(1, 0x1008, 0x1000, pol), ok_seq, ok_step),      # alignment
                 lambda: hs.hs_draft_static(ctx, hs.hs_draft_args(1, None, 0x1000, pol), ok_seq, ok_step)):
        with pytest.raises(hs.HsError) as e:
            call()
        assert e.value.status == hs.HS_ERR_INVALID_ARG
    with pytest.raises(hs.HsError) as e:
        hs.hs_debug_capture(ctx, 0x1000, 16)
    assert e.value.status == hs.HS_ERR_CAPACITY
    assert hs.hs_debug_capture_bytes(ctx) == 4 * lim.max_rows * desc.d_model * 4
    hs.hs_debug_capture(ctx, None, 0)                                             # off again
    with pytest.raises(hs.HsError):
        hs.hs_debug_philox(None, 1, 0x1000, 4)
    assert hs.hs_debug_rowmax_groups(152064) == 951 and hs.hs_debug_rowmax_groups(0) == 0
    hs.hs_destroy(ctx)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(hs, "_lib", None)
    monkeypatch.setattr(hs, "LIB_PATH", "/nonexistent/libhistospec.so")
    with pytest.raises(RuntimeError, match="only implementation"):
        hs.lib()


def test_gate_table_host_helper_equals_the_oracle():
    """hs_gate_table_build is host arithmetic (no device work): the table from a profiled step time must be the
    oracle's for the same points, on an affine profile, one with a plateau and a measured-looking one; bad
    profiles are rejected."""
    import numpy as np
    import oracle
    cases = [
        (np.array([1, 64, 512, 4096, 40000], np.int32), lambda r: 18.0 + 0.011 * r, 8.0, 4096),
        (np.array([1, 300, 3000], np.int32), lambda r: np.where(r <= 300, 10.0, 10.0 + (r - 300) / 30.0), 4.0, 1000),
        (np.array([128, 256, 640, 1152, 2176], np.int32), lambda r: 18.4 + 0.0001 * r + 2e-6 * r * r, 3.5, 512),
        (np.array([8, 4096], np.int32), lambda r: 1.0 + 0.5 * r, 2.25, 64),
    ]
    for rows, f, k_bar, b_max in cases:
        ms = f(rows.astype(np.float64)).astype(np.float32)
        got = hs.hs_gate_table_build(ms, rows, k_bar, b_max)
        assert got == oracle.gate_table(ms, rows, k_bar, b_max).tolist(), (rows, got)
    with pytest.raises(hs.HsError):
        hs.hs_gate_table_build([1.0], [4], 2.0, 8)
    with pytest.raises(hs.HsError):
        hs.hs_gate_table_build([1.0, 2.0, 3.0], [4, 4, 9], 2.0, 8)


def test_planner_host_function_against_the_oracles_optimum():
    """hs_plan_allocation bisects (the paper's method); the oracle enumerates the exact optimum (the definition).
    On random instances the library's gradient lies within `precision` above the optimum, its plan fits the worker
    budget, and every group is on the fewest workers that meet its deadline t0 + i d at the library's d; infeasible
    instances report HS_ERR_CAPACITY on both sides, bad arguments HS_ERR_INVALID_ARG."""
    import numpy as np
    import oracle
    rng = np.random.default_rng(17)
    n_none = 0
    for trial in range(200):
        n, width, min_wks = int(rng.integers(1, 17)), int(rng.integers(1, 9)), int(rng.integers(1, 4))
        max_wks = min_wks + width - 1
        lens = np.sort(rng.uniform(200, 16000, n)) * np.where(np.arange(n) == n - 1, rng.uniform(1, 4), 1.0)
        tau = lens[:, None] * (0.2 + 0.8 / np.arange(min_wks, max_wks + 1)[None, :])
        wks = int(rng.integers(n * min_wks, n * max_wks + 2))
        t_train = float(rng.choice([0.0, rng.uniform(0, tau[0, 0] * 1.5)]))
        p = float(rng.choice([1.0, 25.0, 0.05]))
        want = oracle.plan_allocation(tau, min_wks, max_wks, wks, t_train)
        if want is None:
            n_none += 1
            with pytest.raises(hs.HsError) as e:
                hs.hs_plan_allocation(tau, min_wks, max_wks, wks, t_train, p)
            assert e.value.status == hs.HS_ERR_CAPACITY
            continue
        plan, d = hs.hs_plan_allocation(tau, min_wks, max_wks, wks, t_train, p)
        d_opt = want[1]
        assert d_opt - 1e-9 * (1 + d_opt) <= d <= d_opt + p + 1e-9, (trial, d, d_opt, p)
        assert sum(plan) <= wks and min(plan) >= min_wks and max(plan) <= max_wks
        t0 = max(tau[0, -1], t_train)
        for i in range(n):
            assert tau[i, plan[i] - min_wks] <= t0 + i * d
            assert plan[i] == min_wks or tau[i, plan[i] - 1 - min_wks] > t0 + i * d
        # a larger gradient never needs more workers than the optimum's plan
        assert sum(plan) <= int(want[0].sum())
    assert 5 < n_none < 150
    for bad in ((0, 2, 4, 1.0), (3, 2, 4, 1.0), (1, 2, 0, 1.0), (1, 2, 4, 0.0)):
        with pytest.raises(hs.HsError) as e:
            hs.hs_plan_allocation([[3.0, 2.0][:max(0, bad[1] - bad[0] + 1)] or [1.0]], bad[0], bad[1], bad[2], 0.0, bad[3])
        assert e.value.status == hs.HS_ERR_INVALID_ARG
