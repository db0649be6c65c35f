#!/usr/bin/env python3
"""Benchmark of the history-drafted speculative decoding hot path on one MI355X.

A "step" is one pass of the whole path -- hs_draft, hs_verify, hs_accept, hs_kv_commit -- over the whole
in-flight batch.  The default workload is benchmark configuration 3 (7B-shaped decoder, batch 128, contexts
uniform 2k..16k, 70 % history similarity, draft length set by the match length, greedy acceptance); all inputs
are synthetic and seeded (weights N(0, 0.02) in bf16, random context K/V of the scale a prefill writes, previous-epoch
text = the path's own greedy continuation mutated token by token and by span edits) and resident in HBM before the
timed region starts.
`--config 2`, `--config 4 --reuse R` and `--config 5` run the other benchmark configurations (5 repeats its first
speculative step, see its workload string).

Prints ONE JSON line: accepted tokens/s over the timed steps, the roofline of the dominant kernel (verify
attention, HBM-bound) measured with HIP events on the launching stream, and the CPU oracle timed on a bounded
sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# HBM bytes per launch of the attention kernel at config 3, from the two rocprofv3 --pmc runs (FETCH_SIZE x 2.0,
# WRITE_SIZE x 1.0, factors read off 1 GiB copies in the same runs) summarised under profiles/: counters cannot be
# read inside a timed run, so the figure is carried here and re-measured whenever the kernel changes.
ATTN_TRAFFIC_BYTES_PER_LAUNCH = 2.327e9
HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0


def log(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def workload_params(config: int, reuse: float = 0.5):
    from paper_2508_18588_amd import HS_ACCEPT_REJECTION, HS_K_AIMD, HS_K_FIXED, HS_K_MATCHLEN
    if config == 3:
        return dict(name="config3: 7B shape (28L d3584 28q/4kv x128 ffn18944 V152064), B=128, context U[2048,16384], "
                         "history = GPU greedy 256-token window mutated 26.3% iid + 5% spans (70% copied), "
                         "K = match length 1..16 (window 16, min 3), greedy, KV page 16",
                    batch=128, ctx=("uniform", 2048, 16384), window_tokens=256, p_iid=[0.263], p_span=0.05,
                    policy=dict(window=16, m_min=3, k_mode=HS_K_MATCHLEN, k_max=16), k_max=16)
    if config == 2:
        return dict(name="config2: 1.5B shape (28L d1536 12q/2kv x128 ffn8960 V151936), B=64, prompt 512 + response "
                         "offset 2048, history = GPU greedy 256-token window mutated 20% iid + 5% spans, K=8 fixed, "
                         "greedy, KV page 16",
                    batch=64, ctx=("fixed", 512 + 2048), window_tokens=256, p_iid=[0.20], p_span=0.05,
                    policy=dict(window=8, m_min=3, k_mode=HS_K_FIXED, k_fixed=8, k_max=8), k_max=8)
    if config == 4:
        return dict(name="config4: 7B shape, B=256, prompt 512 + response lognormal(median 4000, sigma 0.8) clipped to "
                         f"[512, 32768], snapshot 256 tokens before each response's end, history reuse {reuse:.0%} "
                         f"(window mutated {1 - reuse:.0%} iid, no spans), K adaptive 2..32 (+2 on full accept, back "
                         "to 2 on a reject; window 16, min 3), greedy, KV page 16",
                    batch=256, ctx=("lognormal", 4000.0, 0.8, 512, 32768, 512), window_tokens=256,
                    p_iid=[1.0 - reuse], p_span=0.0,
                    policy=dict(window=16, m_min=3, k_mode=HS_K_AIMD, k_max=32), k_max=32)
    if config == 5:
        return dict(name="config5: 14B shape (48L d5120 40q/8kv x128 ffn13824 V152064), B=64, context 8192, two "
                         "histories per sequence (the sampled 64-token continuation mutated 40% and 60% iid) -> "
                         "2-branch draft tree of depth 8, tree-mask verify, rejection sampling at temperature 1 "
                         "(Philox), tree commit, KV page 16; EVERY TIMED STEP IS THE FIRST SPECULATIVE STEP AFTER "
                         "THE SNAPSHOT (sequence state restored by five small device copies inside the timed "
                         "region): a sampled token never re-enters a history of other samples, so drafting would "
                         "stop after one step, and on random-init (flat) logits the acceptance probability of a "
                         "draft token is about 1/V, so accepted tokens/s is about 0 by construction",
                    batch=64, ctx=("fixed", 8192), window_tokens=64, p_iid=[0.4, 0.6], p_span=0.0,
                    policy=dict(window=8, m_min=3, k_mode=HS_K_FIXED, k_fixed=8, k_max=8), k_max=8,
                    mode=HS_ACCEPT_REJECTION, temperature=1.0, snapshot=True)
    raise SystemExit(f"bench.py: no benchmark workload for config {config} (2, 3, 4 and 5 are available)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--reuse", type=float, default=0.5,
                    help="config 4 only: fraction of the previous epoch's tokens copied unmutated (0, 0.5, 0.9)")
    ap.add_argument("--layers", type=int, default=0, help="debug: fewer layers (result is then NOT the benchmark)")
    ap.add_argument("--window", type=int, default=0,
                    help="debug: tokens of previous-epoch text generated at set-up (default: the workload's 256)")
    ap.add_argument("--print-rows", action="store_true", help="diagnostic: log the row count of every timed step")
    ap.add_argument("--reuse-all", action="store_true",
                    help="debug: history = the rollout itself (every draft accepted, rows per step at their maximum)")
    ap.add_argument("--graph", action="store_true",
                    help="after the timed (eager) steps, record one whole step into a HIP graph and time the same number "
                         "of replays: reported as config.graph_replay (the headline value stays the eager region)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket kernels with events (roofline null)")
    ap.add_argument("--gemm-probe", default="",
                    help="instead of the benchmark: one layer's four projections and the LM head of the configuration's "
                         "shape, each launched alone at these row counts (comma separated), timed with events; "
                         "prints one JSON line (the command rocprofv3 counter runs of the GEMM kernel are made with)")
    ap.add_argument("--draft-probe", action="store_true",
                    help="instead of the benchmark: the draft scan on a scaled input (128 sequences x 16 responses x "
                         "32768 tokens = 268 MB of history through hs_draft_group), timed with events")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="after the timed steps run three 1 GiB device-to-device copies: a kernel of known traffic "
                         "that scales the FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch

    import paper_2508_18588_amd as hs
    from paper_2508_18588_amd.runtime import Engine, Policy
    from hs_inputs import CONFIG_SHAPES, config_seed, mutate, lengths_lognormal, lengths_uniform
    from hs_inputs.device import make_weights_device, fill_kv_random, rope_device, weights_to_host

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU")
    hs.lib()
    if args.gemm_probe:
        return gemm_probe_main(args, [int(r) for r in args.gemm_probe.split(",")])
    if args.draft_probe:
        return draft_probe_main(args)
    cfg = args.config
    wp = workload_params(cfg, args.reuse)
    shape = CONFIG_SHAPES[cfg]
    seed = config_seed(cfg)
    n_layers = args.layers or shape.n_layers
    B, T = wp["batch"], (args.window or wp["window_tokens"])
    pol = Policy(**wp["policy"])
    W = pol.window
    n_cand = len(wp["p_iid"])
    mode, temperature = wp.get("mode", hs.HS_ACCEPT_GREEDY), wp.get("temperature", 1.0)
    philox_seed = seed * 0x9E3779B1 & (2 ** 63 - 1)
    if args.reuse_all:
        wp["p_iid"], wp["p_span"] = [0.0] * n_cand, 0.0
    if wp["ctx"][0] == "uniform":
        ctx = lengths_uniform(B, wp["ctx"][1], wp["ctx"][2], seed)
    elif wp["ctx"][0] == "lognormal":
        _, median, sigma, lo, hi, prompt = wp["ctx"]
        ctx = (prompt + lengths_lognormal(B, median, sigma, lo, hi, seed) - T).astype(np.int32)
    else:
        ctx = np.full(B, wp["ctx"][1], np.int32)
    rng = np.random.default_rng(seed)

    t0 = time.time()
    w = make_weights_device(shape, seed, n_layers)
    max_len = int(ctx.max()) + 1 + T
    rope = rope_device(max_len + 64, shape.head_dim)
    eng = Engine(shape, w, rope, max_batch=B, k_max=wp["k_max"], c_max=n_cand, max_len=max_len,
                 seq_caps=[int(c) + 1 + T for c in ctx], shuffle_pages_seed=seed & 0xFFFF, keep_logits=False,
                 workspace_logits=(mode == hs.HS_ACCEPT_REJECTION))   # rejection sampling reads the logits
    # context: L_b cached positions (synthetic K/V of the scale a real prefill writes) + one committed root token
    kv_std = 0.02 * float(np.sqrt(shape.d_model))
    fill_kv_random(eng.kc, eng.vc, seed + 1, kv_std)
    toks = [rng.integers(0, shape.vocab, int(c) + 1).astype(np.int32) for c in ctx]
    torch.cuda.synchronize()
    log(f"setup: weights+cache in {time.time() - t0:.1f}s; KV resident {eng.kc.numel() * 4 / 1e9:.1f} GB, "
        f"weights {shape.dense_params * n_layers / shape.n_layers * 2 / 1e9:.1f} GB")

    # ---- previous-epoch text: the path's own greedy continuation (K=0), then mutated
    ar_pol = Policy(window=W, m_min=pol.m_min, k_fixed=0, k_max=wp["k_max"])
    eng.load_sequences(toks, budgets=[T] * B)
    eng.set_history([[np.zeros(0, np.int32)] for _ in range(B)])
    eng.set_rows_hint(B)   # launch-shape hint only: one row per sequence without drafts
    for _ in range(3):
        eng.step(ar_pol, mode, temperature, philox_seed)
    torch.cuda.synchronize()
    t1 = time.time()
    for _ in range(T - 3):
        eng.step(ar_pol, mode, temperature, philox_seed)
    torch.cuda.synchronize()
    ar_ms = (time.time() - t1) / (T - 3) * 1e3
    out = eng.tokens.cpu().numpy()
    rolls = [out[b, len(toks[b]):len(toks[b]) + T].copy() for b in range(B)]
    log(f"autoregressive rollout (K=0): {ar_ms:.2f} ms/step, {B / ar_ms * 1e3:.0f} tokens/s")
    hists = []
    for b in range(B):
        filler = rng.integers(0, shape.vocab, max(0, len(toks[b]) - (W - 1))).astype(np.int32)
        hists.append([np.concatenate([filler, toks[b][-(W - 1):], mutate(rolls[b], p, wp["p_span"], shape.vocab, rng)])
                      for p in wp["p_iid"]])
    eng.load_sequences(toks, budgets=[T] * B)
    eng.set_history(hists)
    # configuration 5 times the same step again and again: the state every step starts from
    state = [eng.seq_len, eng.tail, eng.tail_len, eng.k_state, eng.budget_left]
    snap = [t.clone() for t in state] if wp.get("snapshot") else None

    step_events = []   # (before hs_draft, after hs_draft, after hs_kv_commit) of every timed step

    def one_step(timed=False):
        if snap is not None:
            for t, s0 in zip(state, snap):
                t.copy_(s0)
        if not timed:
            eng.step(pol, mode, temperature, philox_seed)
            return
        # HIP events on the stream the four calls are enqueued on (torch's current stream)
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
        ev[0].record()
        eng.draft(pol)
        ev[1].record()
        eng.verify()
        eng.accept_commit(pol, mode, temperature, philox_seed)
        ev[2].record()
        step_events.append(ev)

    # ---- warm-up, then the timed region
    first = None
    warm_rows = []
    want_sample = not args.no_cpu_baseline and n_cand == 1 and mode == hs.HS_ACCEPT_GREEDY
    for i in range(args.warmup):
        if i == 0 and want_sample:   # the oracle-checked step keeps its logits (the timed steps keep none)
            eng.set_flags(eng.flags | hs.HS_FLAG_WORKSPACE_LOGITS)
        one_step()
        warm_rows.append(int(eng.st["row_off"][B].item()))
        if i == 0:
            torch.cuda.synchronize()
            first = {k: v.cpu().numpy().copy() for k, v in eng.st.items()}
            # logits of the sequence the oracle will re-compute (shortest context among those that drafted)
            ro = first["row_off"]
            cand = [b for b in range(B) if ro[b + 1] - ro[b] > 1]
            if cand and want_sample:
                bs = min(cand, key=lambda i: len(toks[i]))
                lg = eng.debug_tensor(3).view(torch.float32).view(-1, shape.vocab)
                first["sample_seq"] = bs
                first["sample_logits"] = lg[ro[bs]:ro[bs + 1]].cpu().numpy().copy()
            if want_sample:
                eng.set_flags(eng.flags & ~hs.HS_FLAG_WORKSPACE_LOGITS)
    torch.cuda.synchronize()
    if args.warmup > 0:
        # launch-shape hint: mean rows of the warm-up steps after the first (in which every sequence drafts a full
        # window because all of them start in sync with their history)
        tail = (warm_rows[1:] or warm_rows) if snap is None else warm_rows
        eng.set_rows_hint(-(-sum(tail) // len(tail)))
        log(f"rows hint for the timed steps: {eng.c_step.rows_hint}")
    c0 = eng.counters.cpu().numpy().copy()
    len0 = eng.seq_len.cpu().numpy()[:B].astype(np.int64).copy()
    if not args.no_profile:
        eng.set_profile(1)      # events around the attention kernel of every fourth layer only (and the whole call)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    step_rows = []
    for _ in range(args.steps):
        one_step(timed=True)
        if args.print_rows:     # diagnostic: synchronises every step, the timing of such a run means nothing
            step_rows.append(int(eng.st["row_off"][B].item()))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t2
    ev_all = sorted(e[0].elapsed_time(e[2]) for e in step_events)
    ev_vac = sorted(e[1].elapsed_time(e[2]) for e in step_events)
    ev_draft = sorted(e[0].elapsed_time(e[1]) for e in step_events)
    med = lambda v: (v[(len(v) - 1) // 2] + v[len(v) // 2]) / 2
    if step_rows:
        log(f"rows per timed step: {step_rows}")
    prof = None if args.no_profile else eng.get_profile()
    eng.set_profile(0)
    c1 = eng.counters.cpu().numpy().copy()
    len1 = eng.seq_len.cpu().numpy()[:B].astype(np.int64).copy()
    assert eng.poll_error() == 0, "device error word set"
    # per-class kernel times come from a few further steps with every launch bracketed (not part of the timed region)
    prof_all, prof_all_steps, rows_all = None, min(5, args.steps), 0
    if not args.no_profile:
        ca = eng.counters.cpu().numpy().copy()
        eng.set_profile(2)
        for _ in range(prof_all_steps):
            one_step()
        prof_all = eng.get_profile()
        eng.set_profile(0)
        cb = (eng.counters.cpu().numpy() - ca).tolist()
        rows_all = (cb[0] + cb[1]) / prof_all_steps
    graph_extra = {}
    if args.graph and snap is None:
        # the same steps again, replayed from a graph of one step (state simply continues: same workload statistics)
        cg0 = eng.counters.cpu().numpy().copy()
        g = eng.capture_step(pol, mode, temperature, philox_seed)
        g.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        g_el = time.perf_counter() - tg
        cg1 = (eng.counters.cpu().numpy() - cg0).tolist()
        graph_extra = {"graph_replay": {"ms_per_step": round(g_el / args.steps * 1e3, 3),
                                        "accepted_tokens_per_s": round(cg1[2] * args.steps / (args.steps + 1) / g_el, 1),
                                        "rows_per_step": round((cg1[0] + cg1[1]) / (args.steps + 1), 1),
                                        "note": "one whole step (all four calls) recorded into a HIP graph and replayed; "
                                                "not the headline value"}}
        assert eng.poll_error() == 0
    seq_steps, drafted, accepted, emitted = (c1 - c0).tolist()
    ms_per_step = elapsed / args.steps * 1e3
    rows_per_step = (drafted + seq_steps) / args.steps

    # ---- roofline of the dominant kernel: verify attention, one launch per layer and step.
    # Algorithmic bytes per launch: every cached K and V element of every sequence once (positions [0, L_b + nodes)),
    # the bf16 queries in and the bf16 attention output out.
    roofline = None
    kv_tok_bytes = 2 * shape.n_kv_heads * shape.head_dim * 2          # K+V bytes per token and layer
    mean_keys = float((len0 + len1).sum()) / 2 - B + rows_per_step     # sum_b (L_b + nodes_b), mid-region
    att_bytes = mean_keys * kv_tok_bytes + rows_per_step * shape.n_q_heads * shape.head_dim * 2 * 2
    # flops of the same launch: 4 h per (query row, head, visible key); with many rows per sequence the launch is no
    # longer bound by HBM alone (flop per KV byte = query heads per KV head x nodes)
    att_flops = 4.0 * shape.head_dim * shape.n_q_heads * float(((len0 + len1) / 2.0 - 1.0).sum()) * rows_per_step / B
    extras = {}
    if prof is not None:
        ms, n = prof
        att_ms = ms[0] / max(1, n[0])
        achieved = att_bytes / (att_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "attn_verify_mfma", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": ATTN_TRAFFIC_BYTES_PER_LAUNCH if cfg == 3 else None,
                    "algorithmic_bytes_per_launch": int(att_bytes),
                    "avg_launch_ms": round(att_ms, 4), "launches": n[0],
                    "launches_note": "the attention launch of every fourth layer of every timed step, bracketed by "
                                     "HIP events on the launching stream (all layers do the same work)",
                    "flops_per_launch": int(att_flops),
                    "flop_per_byte": round(att_flops / att_bytes, 1),
                    "frac_of_bf16_mfma_peak": round(att_flops / (att_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)}
        msa, _ = prof_all
        gemm_flops = 2.0 * rows_all * (shape.dense_params - shape.d_model * shape.vocab) * n_layers / shape.n_layers
        gemm_ms = msa[1] / prof_all_steps
        lm_flops = 2.0 * rows_all * shape.d_model * shape.vocab
        lm_ms = msa[2] / prof_all_steps
        layer_w_bytes = 2.0 * (shape.dense_params - shape.d_model * shape.vocab) * n_layers / shape.n_layers
        extras = {"verify_ms_per_step": round(ms[4] / args.steps, 3),
                  "class_profile": {"steps": prof_all_steps, "rows_per_step": round(rows_all, 1),
                                    "note": "further steps after the timed region, every launch bracketed by events",
                                    "ms_per_step": {"attention": round(msa[0] / prof_all_steps, 3),
                                                    "proj_gemm": round(gemm_ms, 3), "lm_head": round(lm_ms, 3),
                                                    "other": round(msa[3] / prof_all_steps, 3)},
                                    "gemm_tflops": round(gemm_flops / (gemm_ms * 1e-3) / 1e12, 1),
                                    "gemm_frac_of_bf16_mfma_peak": round(gemm_flops / (gemm_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                                    "gemm_weight_stream_gbs": round(layer_w_bytes / (gemm_ms * 1e-3) / 1e9, 1),
                                    "lm_head_tflops": round(lm_flops / (lm_ms * 1e-3) / 1e12, 1)}}

    # ---- the projections at the configuration's maximum row count (every sequence drafting k_max tokens): the regime
    # in which they are bound by the matrix cores rather than by streaming weights.  One layer's four projections and
    # the LM head, each launched alone through hs_debug_gemm on random activations, timed with events on the stream.
    if prof is not None and n_layers == shape.n_layers:
        extras["gemm_at_max_rows"] = gemm_probe(eng, shape, B * (n_cand * wp["k_max"] + 1))

    # ---- CPU oracle on a bounded sample: one sequence, its first speculative step at full model size
    cpu = None
    if not args.no_cpu_baseline and n_cand == 1 and mode == hs.HS_ACCEPT_GREEDY:
        cpu = cpu_baseline(eng, shape, w, rope, toks, hists, pol, first, B, n_layers, weights_to_host)

    result = {
        "metric": "accepted tokens/sec on 1 MI355X (verify step)", "value": round(accepted / elapsed, 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wp["name"] + ("" if n_layers == shape.n_layers else f" [DEBUG: {n_layers} layers]")
                   + ("" if T == wp["window_tokens"] else f" [DEBUG: window {T}]")
                   + (" [DEBUG: history == rollout]" if args.reuse_all else ""),
                   "rows_per_step": round(rows_per_step, 1),
                   "committed_tokens_per_s": round(emitted / elapsed, 1),
                   "accepted_per_seq_step": round(accepted / max(1, seq_steps), 3),
                   "acceptance_rate": round(accepted / max(1, drafted), 3),
                   "autoregressive_tokens_per_s": round(B / ar_ms * 1e3, 1),
                   "speedup_vs_autoregressive": round((emitted / elapsed) / (B / ar_ms * 1e3), 3),
                   # Sec. 5.4 (throughput-aware control): drafting pays while the acceptance rate stays above this
                   "break_even_acceptance_rate": round(max(0.0, ms_per_step / ar_ms - 1.0) * seq_steps
                                                       / max(1, drafted), 3),
                   "kv_resident_gb": round(float(len0.sum()) * kv_tok_bytes * n_layers / 1e9, 1),
                   # HIP events per step: all four calls / verify + accept + commit / the draft call alone
                   "median_ms_per_step": round(med(ev_all), 3),
                   "median_verify_accept_commit_ms": round(med(ev_vac), 3),
                   "median_draft_us": round(med(ev_draft) * 1e3, 1),
                   "accepted_tokens_per_s_at_median_step": round(accepted / args.steps / (med(ev_all) * 1e-3), 1),
                   **graph_extra, **extras},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    if args.calibrate_copy:
        calibration_copy(torch)
    eng.close()
    print(json.dumps(result), flush=True)


def gemm_probe_main(args, rows_list):
    """One layer of the configuration's shape; every projection alone at each row count."""
    import torch

    from paper_2508_18588_amd.runtime import Engine
    from hs_inputs import CONFIG_SHAPES, config_seed
    from hs_inputs.device import make_weights_device, rope_device
    shape = CONFIG_SHAPES[args.config]
    w = make_weights_device(shape, config_seed(args.config), 1)
    m_max = max(rows_list)
    eng = Engine(shape, w, rope_device(64, shape.head_dim), max_batch=max(1, (m_max + 16) // 17), k_max=16, c_max=1,
                 max_len=32, max_rows=m_max, keep_logits=False)
    out = {"probe": "gemm", "config": args.config, "per_rows": [gemm_probe(eng, shape, r, reps=args.steps) for r in rows_list]}
    if args.calibrate_copy:
        calibration_copy(torch)
    eng.close()
    print(json.dumps(out), flush=True)


def draft_probe_main(args):
    """The draft scan in its bandwidth regime: 128 sequences, 16 previous-epoch responses of 32768 tokens each
    (4 bytes per token: 268 MB of history read once per call)."""
    import numpy as np
    import torch

    from paper_2508_18588_amd.runtime import Engine, Policy
    from hs_inputs import CONFIG_SHAPES, config_seed, make_weights, rope_table
    shape = CONFIG_SHAPES[1]                     # the draft does not touch the model: the toy shape keeps set-up short
    B, G, LH, W = 128, 16, 32768, 16
    rng = np.random.default_rng(config_seed(3))
    eng = Engine(shape, make_weights(shape, 1), rope_table(LH + 64, shape.head_dim), max_batch=B, k_max=16, c_max=1,
                 max_len=64, g_max=G, keep_logits=False)
    toks = [rng.integers(0, 152064, 40).astype(np.int32) for _ in range(B)]
    groups = []
    for b in range(B):
        row = []
        for g in range(G):
            hst = rng.integers(0, 152064, LH).astype(np.int32)
            at = int(rng.integers(W, LH - 64))
            hst[at - 8:at] = toks[b][-8:]        # every response contains the sequence's last 8 tokens once
            row.append(hst)
        groups.append(row)
    eng.load_sequences(toks, budgets=[64] * B)
    eng.set_group_history(groups, [[1] * G for _ in range(B)])
    pol = Policy(window=W, m_min=3, k_fixed=8, k_max=16)
    for _ in range(3):
        eng.draft_group(pol)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        eng.draft_group(pol)
    e1.record()
    torch.cuda.synchronize()
    assert eng.poll_error() == 0
    ms = e0.elapsed_time(e1) / args.steps
    nbytes = B * G * LH * 4
    drafted = int(eng.st["row_off"][B].item()) - B
    print(json.dumps({"probe": "draft", "history_bytes": nbytes, "ms_per_call": round(ms, 4),
                      "call_gbs": round(nbytes / (ms * 1e-3) / 1e9, 1),
                      "call_frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                      "drafted_tokens": drafted,
                      "note": "whole hs_draft_group call (scan + reward walk + row build); the scan kernel alone is in "
                              "the rocprofv3 kernel trace of this command"}), flush=True)
    eng.close()


def calibration_copy(torch):
    src = torch.ones(1 << 28, dtype=torch.int32, device="cuda:0")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    log(f"calibration copy: 3 x 1 GiB read + 1 GiB written in {(time.perf_counter() - t3) * 1e3:.2f} ms "
        f"({3 * 2 * 2 ** 30 / (time.perf_counter() - t3) / 1e9:.0f} GB/s read+write)")


def gemm_probe(eng, shape, rows, reps=5):
    import torch
    dev = eng.dev
    g = torch.Generator(device=dev).manual_seed(7)
    d, F, V = shape.d_model, shape.d_ffn, shape.vocab
    qh = shape.n_q_heads * shape.head_dim
    rows = min(rows, eng.max_rows)
    m_dev = torch.full((1,), rows, dtype=torch.int32, device=dev)
    a_d = torch.randn(eng.max_rows, d, device=dev, generator=g).to(torch.bfloat16).view(torch.int16)
    a_f = torch.randn(eng.max_rows, F, device=dev, generator=g).to(torch.bfloat16).view(torch.int16)
    a_q = a_d[:, :qh].contiguous()
    W = eng.w
    cases = [("qkv", 0, a_d, W["wqkv"][0], None), ("o", 1, a_q, W["wo"][0], None),
             ("gate_up", 2, a_d, W["wgate"][0], W["wup"][0]), ("down", 1, a_f, W["wdown"][0], None),
             ("lm_head", 0, a_d, W["lm_head"], None)]
    out = {"rows": rows}
    layer_flops = layer_ms = 0.0
    for name, epi, a, w, w2 in cases:
        n, k = int(w.shape[0]), int(w.shape[1])
        c = torch.zeros(eng.max_rows, n, dtype=torch.int16 if epi == 2 else torch.float32, device=dev)
        for _ in range(2):
            eng.gemm(epi, a, w, w2, c, m_dev, eng.max_rows, rows)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            eng.gemm(epi, a, w, w2, c, m_dev, eng.max_rows, rows)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        flops = 2.0 * rows * n * k * (2 if w2 is not None else 1)
        out[name + "_tflops"] = round(flops / (ms * 1e-3) / 1e12, 1)
        out[name + "_us"] = round(ms * 1e3, 1)
        out[name + "_weight_gbs"] = round(n * k * 2 * (2 if w2 is not None else 1) / (ms * 1e-3) / 1e9, 1)
        if name != "lm_head":
            layer_flops += flops
            layer_ms += ms
        del c
    out["layer_tflops"] = round(layer_flops / (layer_ms * 1e-3) / 1e12, 1)
    out["layer_frac_of_bf16_mfma_peak"] = round(out["layer_tflops"] / MFMA_BF16_PEAK_TFLOPS, 4)
    out["lm_head_frac_of_bf16_mfma_peak"] = round(out["lm_head_tflops"] / MFMA_BF16_PEAK_TFLOPS, 4)
    out["note"] = ("each projection launched alone (split-K ones include their ordered reduce), activations random; "
                   "the timed steps above run at rows_per_step, where the projections stream weights")
    return out


def cpu_baseline(eng, shape, w, rope, toks, hists, pol, first, B, n_layers, weights_to_host):
    """Time the oracle on the first speculative step of one sequence (the shortest context that drafted), and compare
    the path's results for that sequence with it: logits, emitted tokens, and the residual stream after 1, 2, 4, ...
    layers (the path re-run on that one sequence with the first l layers of the same weights)."""
    import numpy as np
    import torch

    import oracle
    from paper_2508_18588_amd.runtime import Engine
    if first is None:
        return None
    if "sample_seq" not in first:
        return None
    b = first["sample_seq"]
    L = len(toks[b]) - 1
    t0 = time.time()
    wh = weights_to_host(w)
    model = oracle.Model(shape, wh, rope.cpu().numpy())
    hkv, h = shape.n_kv_heads, shape.head_dim
    pages = eng.block_table[b, :(L + 15) // 16].long()
    kc = eng.kc.view(n_layers, eng.n_blocks, hkv, 16, h)[:, pages].view(torch.bfloat16)
    vc = eng.vc.view(n_layers, eng.n_blocks, hkv, h, 16)[:, pages].view(torch.bfloat16)
    k_ctx = kc.permute(0, 1, 3, 2, 4).reshape(n_layers, -1, hkv * h)[:, :L]       # [layers, L, hkv*h] bf16
    v_ctx = vc.permute(0, 1, 4, 2, 3).reshape(n_layers, -1, hkv * h)[:, :L]
    seq = oracle.Seq(model, L + 64)
    seq.load_kv(k_ctx.double().cpu().numpy(), v_ctx.double().cpu().numpy())
    log(f"cpu_baseline: sequence {b} (context {L}), host copy of weights and its K/V in {time.time() - t0:.1f}s")
    x = toks[b]
    t1 = time.time()
    p, m = oracle.suffix_match(hists[b][0], x, pol.window, pol.m_min)
    kk = oracle.draft_len(oracle.k_policy(pol.k_mode, pol.k_fixed, 2, m, pol.k_max), len(hists[b][0]), p, 256)
    tree = oracle.build_tree([hists[b][0][p:p + kk]], x[-1], L)
    # one candidate: the tree is a chain, whose nodes' logits are those of its tokens pushed one after the other
    # (tree_logits does exactly that on a chain); pushed here one by one to keep each token's residual stream
    lg, hid = [], []
    for t in tree["tok"]:
        l_, h_ = seq.push_traced(int(t))
        lg.append(l_)
        hid.append(h_)
    seq.truncate(L)
    lg, hid = np.stack(lg), np.stack(hid)                                          # [rows, V], [rows, layers+1, d]
    a, out, path = oracle.accept_greedy(tree["tok"], tree["parent"], [oracle.argmax(r) for r in lg])
    dt = time.time() - t1
    gpu_out = first["out_tok"][b, :first["n_out"][b]].tolist()
    # parity of this sample: logits, tokens (equal unless a visited row's top-2 margin in the oracle's logits is
    # within the logit error: a near-tie decided by rounding)
    derr = np.abs(first["sample_logits"] - lg)
    err = float(derr.max())
    same = out.tolist() == gpu_out
    margins = np.sort(lg, axis=1)
    margins = margins[:, -1] - margins[:, -2]
    margin = None
    if not same:
        n = min(len(gpu_out), len(out))
        j = next((i for i in range(n) if gpu_out[i] != int(out[i])), n - 1)
        margin = float(margins[int(path[j])])
    log(f"cpu_baseline: {len(tree['tok'])} rows in {dt:.1f}s; oracle emitted {out.tolist()}, GPU emitted {gpu_out}")
    # ---- error against depth: the same rows through the first l layers only
    depth = {}
    rows = [dict(tok=tree["tok"], parent=tree["parent"], pos=tree["pos"])]
    for l in [d_ for d_ in (1, 2, 4, 8, 16, n_layers) if d_ <= n_layers]:
        rep = Engine(shape, w, rope, max_batch=1, k_max=len(tree["tok"]) - 1 or 1, c_max=1, max_len=L + 40,
                     n_layers=l, keep_logits=False)
        rep.load_sequences([x], budgets=[64])
        pos = torch.arange(L, device=rep.dev)
        pg, sl = rep.block_table[0, (pos // 16).long()].long(), (pos % 16).long()
        rk = rep.kc.view(l, rep.n_blocks, hkv, 16, h)
        rv = rep.vc.view(l, rep.n_blocks, hkv, h, 16)
        for li in range(l):
            rk[li, pg, :, sl, :] = k_ctx[li].view(L, hkv, h).view(torch.int16)
            rv[li, pg, :, :, sl] = v_ctx[li].view(L, hkv, h).view(torch.int16)
        mrows = rep.set_rows(rows)
        rep.verify()
        torch.cuda.synchronize()
        xr = rep.debug_tensor(4).view(torch.float32)[:mrows * shape.d_model].view(mrows, -1).double().cpu().numpy()
        rep.close()
        want = hid[:, l]
        depth[str(l)] = round(float(np.sqrt(((xr - want) ** 2).mean() / (want ** 2).mean())), 5)
    return {"value": round(a / dt, 4), "unit": "tokens/s", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"1 of {B} sequences (context {L} tokens), 1 speculative step of {len(tree['tok'])} rows "
                      f"through all {n_layers} layers; accepted {a}, committed {a + 1} tokens in {dt:.1f} s",
            "committed_tokens_per_s": round((a + 1) / dt, 4),
            "parity_sample": {"max_abs_logit_err_vs_gpu": round(err, 5),
                              "rms_logit_err_vs_gpu": round(float(np.sqrt((derr ** 2).mean())), 5),
                              "logit_std": round(float(lg.std()), 3),
                              "rows_with_top2_margin_below_max_err": int((margins <= err).sum()),
                              "rows": int(len(margins)),
                              "same_tokens_as_gpu": same,
                              "oracle_top2_margin_at_first_difference": margin,
                              "residual_rel_rms_err_after_layers": depth}}


if __name__ == "__main__":
    main()
