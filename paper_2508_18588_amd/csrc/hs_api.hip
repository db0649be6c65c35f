// C-ABI entry points: argument validation, workspace layout, and the launch sequence of one decode iteration.
#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <new>

#include "hs_internal.h"

namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

hs_status fail(hs_ctx* ctx, hs_status code, const char* msg) {
    if (ctx) ctx->err = msg;
    return code;
}

hs_status fail_hip(hs_ctx* ctx, const char* where, hipError_t e) {
    ctx->err = std::string(where) + ": kernel launch failed: " + hipGetErrorString(e);
    return HS_ERR_HIP;
}

void layout_workspace(hs_ctx* ctx) {
    const hs_model_desc& d = ctx->desc;
    const hs_limits& l = ctx->lim;
    hs_workspace_layout& w = ctx->lay;
    const size_t M = (size_t)l.max_rows;
    const size_t qh = (size_t)d.n_q_heads * d.head_dim;
    const size_t nqkv = (size_t)(d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    const size_t ab = hs_fp32_activations(ctx) ? 4 : 2;   // bytes per activation element
    w.err = take(256);
    w.x = take(M * d.d_model * 4);
    w.xn = take(M * d.d_model * ab);
    w.qkv = take(M * nqkv * 4);
    w.q = take(M * qh * ab);
    w.attn = take(M * qh * ab);
    w.act = take(M * (size_t)d.d_ffn * ab);
    w.part_o = take(M * d.n_q_heads * (size_t)ctx->max_parts * d.head_dim * 2);   // fp16
    w.part_ml = take(M * d.n_q_heads * (size_t)ctx->max_parts * 2 * 4);
    w.logits_bytes = hs_logits_in_workspace(ctx) ? M * (size_t)d.vocab * 4 : 0;
    w.logits = take(w.logits_bytes);
    w.rowmax = take(M * (size_t)hs_gemm_rowmax_groups(d.vocab) * 8);
    w.draft_best = take((size_t)l.max_batch * std::max(l.c_max, l.g_max) * ctx->max_segs * 8);
    // (the LM head splits K only when the vocabulary is small; it then writes partial sums like the others)
    const int lm_chunks = hs_gemm_chunks(d.vocab, d.d_model);
    size_t part_cols = std::max({(size_t)hs_gemm_chunks((int)nqkv, d.d_model) * nqkv,
                                 (size_t)hs_gemm_chunks(d.d_model, (int)qh) * d.d_model,
                                 (size_t)hs_gemm_chunks(d.d_model, d.d_ffn) * d.d_model,
                                 lm_chunks > 1 ? (size_t)lm_chunks * d.vocab : (size_t)0});
    w.gemm_part_bytes = M * part_cols * 4;
    w.gemm_part = take(w.gemm_part_bytes);
    w.pf_len = take((size_t)l.max_batch * 4);
    w.att_work = take((size_t)(2 + d.n_layers) * 4);
    w.att_list = take(2 * hs_attention_max_units(ctx) * 32);
    w.total = off;
}

struct Prof {
    hs_ctx* ctx;
    hipStream_t st;
    bool open = false;
    // level 1 brackets the whole call and the attention kernel of every fourth layer only (`sampled`): an event
    // record costs about 5 microseconds of stream time on either side of a launch, which a timed run should not pay
    // around all ~9 launches of each layer
    void begin(int cls, bool sampled = true) {
        open = false;
        if (!ctx->profile || (ctx->profile == 1 && ((cls != 0 && cls != 4) || !sampled))) return;
        open = true;
        if (ctx->ev_used + 2 > (int)ctx->ev.size()) {
            hipEvent_t a, b;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { ctx->profile = 0; return; }
            ctx->ev.push_back(a);
            ctx->ev.push_back(b);
            ctx->ev_class.push_back(cls);
        }
        ctx->ev_class[ctx->ev_used / 2] = cls;
        (void)hipEventRecord(ctx->ev[ctx->ev_used], st);
    }
    void end() {
        if (!ctx->profile || !open) return;
        open = false;
        (void)hipEventRecord(ctx->ev[ctx->ev_used + 1], st);
        ctx->ev_used += 2;
    }
};

// one snapshot of hs_debug_capture: [max_rows][d_model] elements of 4 bytes (bf16 snapshots use the first half)
size_t capture_slot_bytes(const hs_ctx* ctx) { return (size_t)ctx->lim.max_rows * ctx->desc.d_model * 4; }

bool step_ok(const hs_step* s) {
    return s && s->draft_start && s->match_len && s->draft_len && s->row_off && s->tok && s->pos && s->parent &&
           s->anc_mask && s->row2seq && s->argmax && s->accept_len && s->n_out && s->out_tok && s->path_row;
}

bool seq_ok(const hs_ctx* ctx, const hs_seq_state* s) {
    return s && s->batch >= 1 && s->batch <= ctx->lim.max_batch && s->seq_len && s->block_table && s->tail &&
           s->tail_len && s->k_state && s->budget_left && s->seq_id && (!s->tokens || s->tokens_stride > 0) &&
           (!s->gate || s->counters);
}

bool policy_ok(const hs_ctx* ctx, const hs_policy* p) {
    return p && p->window >= 1 && p->window <= ctx->lim.w_max && p->m_min >= 1 && p->m_min <= p->window &&
           p->k_mode >= HS_K_FIXED && p->k_mode <= HS_K_AIMD && p->k_max >= 0 && p->k_max <= ctx->lim.k_max &&
           p->k_fixed >= 0 && p->aimd_inc >= 0 && p->aimd_cap >= 0 && p->aimd_reset >= 0;
}

bool cache_ok(const hs_kv_cache* c) { return c && c->k && c->v && c->n_blocks >= 1; }

}  // namespace

extern "C" {

hs_status hs_create(const hs_model_desc* desc, const hs_weights* w, const hs_limits* lim, hs_ctx** out) {
    if (!desc || !w || !lim || !out) return HS_ERR_INVALID_ARG;
    *out = nullptr;
    const hs_model_desc& d = *desc;
    if (d.n_layers < 1 || d.d_model < 1 || d.n_q_heads < 1 || d.n_kv_heads < 1 || d.d_ffn < 1 || d.vocab < 1 ||
        !(d.rms_eps > 0.f))
        return HS_ERR_INVALID_ARG;
    if (d.kv_block != 16 || (d.head_dim != 64 && d.head_dim != 128) || d.n_q_heads % d.n_kv_heads != 0 ||
        d.n_q_heads / d.n_kv_heads > 8 || d.d_model % 64 != 0 || d.d_model > 16384 || d.d_ffn % 64 != 0 ||
        (d.n_q_heads * d.head_dim) % 64 != 0)
        return HS_ERR_UNSUPPORTED;
    const hs_limits& l = *lim;
    if (l.max_batch < 1 || l.k_max < 0 || l.k_max > 32 || l.c_max < 1 || l.c_max > 2 || l.max_blocks_per_seq < 1 ||
        l.max_pos < 1 || l.w_max < 1 || l.w_max > 32 || l.max_rows < 1 || l.g_max < 0 || l.g_max > 32)
        return HS_ERR_INVALID_ARG;
    const int nodes = 1 + l.c_max * l.k_max;
    if (nodes > HS_MAX_NODES || (d.n_q_heads / d.n_kv_heads) * nodes > 256) return HS_ERR_UNSUPPORTED;
    if ((long long)l.max_rows < (long long)l.max_batch * nodes) return HS_ERR_CAPACITY;
    {
        // the GEMM kernels address an operand with 32-bit byte offsets from its base
        const long long qh = (long long)d.n_q_heads * d.head_dim;
        const long long nqkv = (long long)(d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
        const long long widest = std::max<long long>({d.d_model, d.d_ffn, qh});
        const long long biggest = std::max<long long>({(long long)d.vocab * d.d_model, nqkv * d.d_model,
                                                       (long long)d.d_ffn * d.d_model, d.d_model * qh,
                                                       (long long)l.max_rows * widest});
        if (biggest * 2 >= (1ll << 32)) return HS_ERR_UNSUPPORTED;
    }
    if (!w->embed || !w->lm_head || !w->norm_f || !w->rope_cs || !w->wqkv || !w->wo || !w->wgate || !w->wup ||
        !w->wdown || !w->norm1 || !w->norm2)
        return HS_ERR_INVALID_ARG;
    for (int i = 0; i < d.n_layers; i++)
        if (!w->wqkv[i] || !w->wo[i] || !w->wgate[i] || !w->wup[i] || !w->wdown[i] || !w->norm1[i] || !w->norm2[i])
            return HS_ERR_INVALID_ARG;
    // the norm weights are read with 16-byte loads
    if (((uintptr_t)w->norm_f & 15u) != 0) return HS_ERR_INVALID_ARG;
    for (int i = 0; i < d.n_layers; i++)
        if ((((uintptr_t)w->norm1[i] | (uintptr_t)w->norm2[i]) & 15u) != 0) return HS_ERR_INVALID_ARG;
    hs_ctx* ctx = new (std::nothrow) hs_ctx();
    if (!ctx) return HS_ERR_CAPACITY;
    ctx->desc = d;
    ctx->lim = l;
    ctx->embed = (const bf16_t*)w->embed;
    ctx->lm_head = (const bf16_t*)w->lm_head;
    ctx->norm_f = w->norm_f;
    ctx->rope_cs = w->rope_cs;
    for (int i = 0; i < d.n_layers; i++) {
        ctx->wqkv.push_back((const bf16_t*)w->wqkv[i]);
        ctx->wo.push_back((const bf16_t*)w->wo[i]);
        ctx->wgate.push_back((const bf16_t*)w->wgate[i]);
        ctx->wup.push_back((const bf16_t*)w->wup[i]);
        ctx->wdown.push_back((const bf16_t*)w->wdown[i]);
        ctx->norm1.push_back(w->norm1[i]);
        ctx->norm2.push_back(w->norm2[i]);
    }
    // Split-KV partition length (a multiple of 32 keys, at most 64 pages): a function of the context's limits only,
    // so results are identical across calls.  The longest of 1024 / 512 / 256 keys that still cuts a full batch at
    // maximum length into a few thousand partitions per layer: longer partitions mean fewer partial results for the
    // merge kernel to re-read, shorter ones keep a small batch spread over the whole chip.
    {
        const long long keys = (long long)l.max_blocks_per_seq * 16;
        ctx->att_part = 256;
        for (int part : {1024, 512}) {
            if ((long long)l.max_batch * d.n_kv_heads * ((keys + part - 1) / part) >= 4096) {
                ctx->att_part = part;
                break;
            }
        }
    }
    const long long max_keys = (long long)l.max_blocks_per_seq * 16;
    ctx->max_parts = (int)((max_keys + ctx->att_part - 1) / ctx->att_part);
    ctx->max_segs = (l.max_pos + 32 + HS_DRAFT_SEG - 1) / HS_DRAFT_SEG;
    {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            ctx->n_cu = n;
        (void)hipGetLastError();
    }
    layout_workspace(ctx);
    *out = ctx;
    return HS_OK;
}

void hs_destroy(hs_ctx* ctx) {
    if (!ctx) return;
    for (hipEvent_t e : ctx->ev) (void)hipEventDestroy(e);
    delete ctx;
}

const char* hs_last_error(const hs_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

hs_status hs_set_flags(hs_ctx* ctx, uint32_t flags) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (flags & ~(uint32_t)(HS_FLAG_REFERENCE_KERNELS | HS_FLAG_FP32_ACTIVATIONS | HS_FLAG_WORKSPACE_LOGITS))
        return fail(ctx, HS_ERR_INVALID_ARG, "unknown flag");
    const bool relayout = flags != ctx->flags;   // activation width, and whether the logits live in the workspace
    ctx->flags = flags;
    if (relayout) {
        layout_workspace(ctx);
        if (ctx->ws && ctx->ws_bytes < ctx->lay.total) {   // the bound workspace no longer fits: calls fail until re-bound
            ctx->ws = nullptr;
            ctx->ws_bytes = 0;
        }
    }
    return HS_OK;
}

size_t hs_workspace_bytes(const hs_ctx* ctx) { return ctx ? ctx->lay.total : 0; }

hs_status hs_bind_workspace(hs_ctx* ctx, void* dev_ptr, size_t bytes) {
    if (!ctx || !dev_ptr) return HS_ERR_INVALID_ARG;
    if (((uintptr_t)dev_ptr & 255u) != 0) return fail(ctx, HS_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (bytes < ctx->lay.total) return fail(ctx, HS_ERR_CAPACITY, "workspace smaller than hs_workspace_bytes");
    ctx->ws = (char*)dev_ptr;
    ctx->ws_bytes = bytes;
    return HS_OK;
}

hs_status hs_draft(hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step, hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!ctx->ws) return fail(ctx, HS_ERR_CAPACITY, "no workspace bound");
    if (!args || !args->hist || !args->hist_off) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft: null history");
    if (((uintptr_t)args->hist & 15u) != 0) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft: hist must be 16-byte aligned");
    if (args->n_cand < 1 || args->n_cand > ctx->lim.c_max) return fail(ctx, HS_ERR_CAPACITY, "hs_draft: n_cand");
    if (!policy_ok(ctx, &args->policy)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft: policy out of range");
    if (!seq_ok(ctx, seq)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft: sequence state");
    if (!step_ok(step)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft: step arrays");
    (void)hipGetLastError();  // drop stale errors of earlier, unrelated runtime calls
    hs_launch_draft(ctx, args, seq, step, (hipStream_t)stream);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail_hip(ctx, "hs_draft", e);
    return HS_OK;
}

hs_status hs_draft_static(hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step,
                          hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!args || !args->hist || !args->hist_off) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_static: null history");
    if (((uintptr_t)args->hist & 15u) != 0)
        return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_static: hist must be 16-byte aligned");
    if (args->n_cand < 1 || args->n_cand > ctx->lim.c_max) return fail(ctx, HS_ERR_CAPACITY, "hs_draft_static: n_cand");
    if (!policy_ok(ctx, &args->policy)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_static: policy out of range");
    if (!seq_ok(ctx, seq)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_static: sequence state");
    if (!step_ok(step)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_static: step arrays");
    if ((long long)seq->batch * args->n_cand * ctx->max_segs > HS_DRAFT_STATIC_ENTRIES)
        return fail(ctx, HS_ERR_CAPACITY,
                    "hs_draft_static: batch * n_cand * history segments exceeds the static scratch (65536 slots); "
                    "use hs_draft with a workspace");
    (void)hipGetLastError();
    hipError_t why = hipSuccess;
    if (!hs_launch_draft_static(ctx, args, seq, step, (hipStream_t)stream, &why)) {
        ctx->err = std::string("hs_draft_static: address of the static scratch array: ") + hipGetErrorString(why);
        return HS_ERR_HIP;
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail_hip(ctx, "hs_draft_static", e);
    return HS_OK;
}

hs_status hs_draft_group(hs_ctx* ctx, const hs_group_draft_args* args, const hs_seq_state* seq, hs_step* step,
                         hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!ctx->ws) return fail(ctx, HS_ERR_CAPACITY, "no workspace bound");
    if (!args || !args->hist || !args->hist_off || !args->reward)
        return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_group: null history or rewards");
    if (((uintptr_t)args->hist & 15u) != 0)
        return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_group: hist must be 16-byte aligned");
    if (args->n_resp < 1 || args->n_resp > ctx->lim.g_max) return fail(ctx, HS_ERR_CAPACITY, "hs_draft_group: n_resp");
    if (!policy_ok(ctx, &args->policy)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_group: policy out of range");
    if (!seq_ok(ctx, seq)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_group: sequence state");
    if (!step_ok(step) || !step->draft_src) return fail(ctx, HS_ERR_INVALID_ARG, "hs_draft_group: step arrays");
    (void)hipGetLastError();
    hs_launch_draft_group(ctx, args, seq, step, (hipStream_t)stream);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail_hip(ctx, "hs_draft_group", e);
    return HS_OK;
}

hs_status hs_verify(hs_ctx* ctx, const hs_kv_cache* cache, const hs_seq_state* seq, hs_step* step, hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!ctx->ws) return fail(ctx, HS_ERR_CAPACITY, "no workspace bound");
    if (!cache_ok(cache)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_verify: cache");
    if (!seq_ok(ctx, seq)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_verify: sequence state");
    if (!step_ok(step)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_verify: step arrays");
    hipStream_t st = (hipStream_t)stream;
    const hs_model_desc& d = ctx->desc;
    const int m_max = ctx->lim.max_rows;
    const int32_t* m_dev = step->row_off + seq->batch;
    float* x = (float*)(ctx->ws + ctx->lay.x);
    void* xn = ctx->ws + ctx->lay.xn;      // activations: bf16, or float in the fp32-activation mode
    float* qkv = (float*)(ctx->ws + ctx->lay.qkv);
    void* q = ctx->ws + ctx->lay.q;
    void* attn = ctx->ws + ctx->lay.attn;
    void* act = ctx->ws + ctx->lay.act;
    const bool head_fused = hs_head_fused(ctx, step);
    float* logits = step->logits ? step->logits : (float*)(ctx->ws + ctx->lay.logits);
    const int qh = d.n_q_heads * d.head_dim;
    const int nqkv = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    // Few rows expected: run the narrow projections split over K (same arithmetic, more workgroups).
    const int hint = step->rows_hint > 0 ? step->rows_hint : m_max;
    const size_t cap_slot = capture_slot_bytes(ctx), cap_xn = hs_fp32_activations(ctx) ? cap_slot : cap_slot / 2;

    (void)hipGetLastError();
    Prof whole{ctx, st}, pr{ctx, st};
    whole.begin(4);
    int whole_slot = ctx->ev_used;
    if (ctx->profile) ctx->ev_used += 2;  // the whole-call pair is closed at the end

    pr.begin(3);
    hs_launch_embed(ctx, step, seq->batch, x, st);
    hs_launch_attention_worklist(ctx, seq, step, st);
    pr.end();
    // A projection run in the split execution leaves its chunk partials for the next kernel in line (RMSNorm for
    // the residual projections, rotary/KV write for QKV), which adds them up in chunk order: one launch fewer per
    // projection.  `pend` carries the number of chunks from the projection to that kernel.
    int pend = 0;
    for (int l = 0; l < d.n_layers; l++) {
        pr.begin(3);
        hs_launch_rmsnorm(ctx, x, ctx->norm1[l], xn, m_dev, pend, st);
        pr.end();
        if (ctx->capture && l + 1 == d.n_layers) {
            (void)hipMemcpyAsync(ctx->capture, xn, cap_xn, hipMemcpyDeviceToDevice, st);
            (void)hipMemcpyAsync(ctx->capture + cap_slot, x, cap_slot, hipMemcpyDeviceToDevice, st);
        }
        pr.begin(1);
        hs_launch_gemm(ctx, HS_EPI_STORE_F32, xn, ctx->wqkv[l], nullptr, qkv, m_dev, m_max, nqkv, d.d_model, hint, st,
                       &pend);
        pr.end();
        pr.begin(3);
        hs_launch_rope_kv(ctx, l, cache, seq, step, qkv, q, pend, st);
        pr.end();
        pr.begin(0, l % 4 == 0);
        hs_launch_attention(ctx, l, cache, seq, step, q, attn, st);
        pr.end();
        pr.begin(3);
        hs_launch_attention_merge(ctx, seq, step, attn, st);
        pr.end();
        pr.begin(1);
        hs_launch_gemm(ctx, HS_EPI_ADD_F32, attn, ctx->wo[l], nullptr, x, m_dev, m_max, d.d_model, qh, hint, st, &pend);
        pr.end();
        pr.begin(3);
        hs_launch_rmsnorm(ctx, x, ctx->norm2[l], xn, m_dev, pend, st);
        pr.end();
        if (ctx->capture && l + 1 == d.n_layers) {
            (void)hipMemcpyAsync(ctx->capture + 2 * cap_slot, xn, cap_xn, hipMemcpyDeviceToDevice, st);
            (void)hipMemcpyAsync(ctx->capture + 3 * cap_slot, x, cap_slot, hipMemcpyDeviceToDevice, st);
        }
        pr.begin(1);
        hs_launch_gemm(ctx, HS_EPI_SWIGLU_BF16, xn, ctx->wgate[l], ctx->wup[l], act, m_dev, m_max, d.d_ffn, d.d_model, hint, st);
        pr.end();
        pr.begin(1);
        hs_launch_gemm(ctx, HS_EPI_ADD_F32, act, ctx->wdown[l], nullptr, x, m_dev, m_max, d.d_model, d.d_ffn, hint, st,
                       &pend);
        pr.end();
    }
    pr.begin(3);
    hs_launch_rmsnorm(ctx, x, ctx->norm_f, xn, m_dev, pend, st);
    pr.end();
    if (head_fused) {
        // no [rows][vocab] array: the LM head leaves one (largest value, column) key per row and column group,
        // hs_accept / hs_accept_commit take the maximum over a row's keys
        pr.begin(2);
        hs_launch_gemm(ctx, HS_EPI_ROWMAX, xn, ctx->lm_head, nullptr, ctx->ws + ctx->lay.rowmax, m_dev, m_max, d.vocab,
                       d.d_model, hint, st);
        pr.end();
    } else {
        pr.begin(2);
        hs_launch_gemm(ctx, HS_EPI_STORE_F32, xn, ctx->lm_head, nullptr, logits, m_dev, m_max, d.vocab, d.d_model, hint,
                       st);
        pr.end();
        pr.begin(3);
        hs_launch_argmax(ctx, logits, step->argmax, m_dev, st);
        pr.end();
    }
    if (ctx->profile) {
        (void)hipEventRecord(ctx->ev[whole_slot + 1], st);
        ctx->ev_last = whole_slot + 1;
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail_hip(ctx, "hs_verify", e);
    return HS_OK;
}

hs_status hs_prefill(hs_ctx* ctx, const hs_kv_cache* cache, const hs_seq_state* seq, hs_step* step,
                     const hs_prefill_args* args, hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!ctx->ws) return fail(ctx, HS_ERR_CAPACITY, "no workspace bound");
    if (!cache_ok(cache)) return fail(ctx, HS_ERR_INVALID_ARG, "hs_prefill: cache");
    if (!seq_ok(ctx, seq) || !seq->tokens) return fail(ctx, HS_ERR_INVALID_ARG, "hs_prefill: sequence state / token log");
    if (!step || !step->row_off || !step->tok || !step->pos || !step->parent || !step->row2seq)
        return fail(ctx, HS_ERR_INVALID_ARG, "hs_prefill: step arrays");
    if (!args || !args->kv_done || args->chunk < 1 || args->chunk > HS_PREFILL_CHUNK_MAX)
        return fail(ctx, HS_ERR_INVALID_ARG, "hs_prefill: arguments");
    if (hs_plain_kernels(ctx)) return fail(ctx, HS_ERR_UNSUPPORTED, "hs_prefill: no plain-kernel mode");
    hipStream_t st = (hipStream_t)stream;
    const hs_model_desc& d = ctx->desc;
    const int m_max = ctx->lim.max_rows;
    const int32_t* m_dev = step->row_off + seq->batch;
    float* x = (float*)(ctx->ws + ctx->lay.x);
    bf16_t* xn = (bf16_t*)(ctx->ws + ctx->lay.xn);
    float* qkv = (float*)(ctx->ws + ctx->lay.qkv);
    bf16_t* q = (bf16_t*)(ctx->ws + ctx->lay.q);
    bf16_t* attn = (bf16_t*)(ctx->ws + ctx->lay.attn);
    bf16_t* act = (bf16_t*)(ctx->ws + ctx->lay.act);
    int32_t* len_plus1 = (int32_t*)(ctx->ws + ctx->lay.pf_len);
    const int qh = d.n_q_heads * d.head_dim;
    const int nqkv = (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    const int hint = args->rows_hint > 0 ? args->rows_hint : m_max;
    // the row kernels place a row at slot (sequence length - 1 + its index): here that is kv_done + i
    hs_seq_state pf = *seq;
    pf.seq_len = len_plus1;

    (void)hipGetLastError();
    hs_launch_prefill_rows(ctx, seq, args->kv_done, args->chunk, step, len_plus1, st);
    hs_launch_embed(ctx, step, seq->batch, x, st);
    int pend = 0;
    for (int l = 0; l < d.n_layers; l++) {
        hs_launch_rmsnorm(ctx, x, ctx->norm1[l], xn, m_dev, pend, st);
        hs_launch_gemm(ctx, HS_EPI_STORE_F32, xn, ctx->wqkv[l], nullptr, qkv, m_dev, m_max, nqkv, d.d_model, hint, st,
                       &pend);
        hs_launch_rope_kv(ctx, l, cache, &pf, step, qkv, q, pend, st);
        pend = 0;
        if (l + 1 == d.n_layers) break;   // the last layer's K/V are written: nothing downstream is needed
        hs_launch_attention_prefill(ctx, l, cache, &pf, len_plus1, step, q, attn, args->chunk, st);
        hs_launch_gemm(ctx, HS_EPI_ADD_F32, attn, ctx->wo[l], nullptr, x, m_dev, m_max, d.d_model, qh, hint, st, &pend);
        hs_launch_rmsnorm(ctx, x, ctx->norm2[l], xn, m_dev, pend, st);
        hs_launch_gemm(ctx, HS_EPI_SWIGLU_BF16, xn, ctx->wgate[l], ctx->wup[l], act, m_dev, m_max, d.d_ffn, d.d_model, hint, st);
        hs_launch_gemm(ctx, HS_EPI_ADD_F32, act, ctx->wdown[l], nullptr, x, m_dev, m_max, d.d_model, d.d_ffn, hint, st,
                       &pend);
    }
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail_hip(ctx, "hs_prefill", e);
    return HS_OK;
}

}  // extern "C"

namespace {

// Shared by hs_accept, hs_kv_commit and hs_accept_commit: args == nullptr skips acceptance, policy == nullptr the commit.
hs_status accept_commit(hs_ctx* ctx, const char* who, const hs_accept_args* args, const hs_kv_cache* cache,
                        const hs_seq_state* seq, const hs_step* step, const hs_policy* policy, hs_stream stream) {
    const float* logits = nullptr;
    const unsigned long long* keys = nullptr;
    if (args) {
        if (!ctx->ws) return fail(ctx, HS_ERR_CAPACITY, "no workspace bound");
        if (args->mode != HS_ACCEPT_GREEDY && args->mode != HS_ACCEPT_REJECTION)
            return fail(ctx, HS_ERR_INVALID_ARG, "acceptance mode");
        if (args->mode == HS_ACCEPT_REJECTION && !(args->temperature > 0.f))
            return fail(ctx, HS_ERR_INVALID_ARG, "temperature must be positive");
        if (hs_head_fused(ctx, step)) {
            if (args->mode == HS_ACCEPT_REJECTION)
                return fail(ctx, HS_ERR_INVALID_ARG,
                            "rejection sampling needs the logits: pass hs_step.logits or set HS_FLAG_WORKSPACE_LOGITS");
            keys = (const unsigned long long*)(ctx->ws + ctx->lay.rowmax);
        } else {
            logits = step->logits ? step->logits : (const float*)(ctx->ws + ctx->lay.logits);
        }
    }
    if (policy) {
        if (!cache_ok(cache)) return fail(ctx, HS_ERR_INVALID_ARG, "cache");
        if (!policy_ok(ctx, policy)) return fail(ctx, HS_ERR_INVALID_ARG, "policy out of range");
    }
    if (!seq_ok(ctx, seq)) return fail(ctx, HS_ERR_INVALID_ARG, "sequence state");
    if (!step_ok(step)) return fail(ctx, HS_ERR_INVALID_ARG, "step arrays");
    (void)hipGetLastError();
    hs_launch_accept_commit(ctx, args, cache, seq, step, logits, keys, hs_gemm_rowmax_groups(ctx->desc.vocab), policy,
                            (hipStream_t)stream);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail_hip(ctx, who, e);
    return HS_OK;
}

}  // namespace

extern "C" {

hs_status hs_accept(hs_ctx* ctx, const hs_accept_args* args, const hs_seq_state* seq, hs_step* step, hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!args) return fail(ctx, HS_ERR_INVALID_ARG, "hs_accept: arguments");
    return accept_commit(ctx, "hs_accept", args, nullptr, seq, step, nullptr, stream);
}

hs_status hs_kv_commit(hs_ctx* ctx, const hs_kv_cache* cache, hs_seq_state* seq, const hs_step* step,
                       const hs_policy* policy, hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!policy) return fail(ctx, HS_ERR_INVALID_ARG, "hs_kv_commit: policy");
    return accept_commit(ctx, "hs_kv_commit", nullptr, cache, seq, step, policy, stream);
}

hs_status hs_accept_commit(hs_ctx* ctx, const hs_accept_args* args, const hs_kv_cache* cache, hs_seq_state* seq,
                           hs_step* step, const hs_policy* policy, hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!args || !policy) return fail(ctx, HS_ERR_INVALID_ARG, "hs_accept_commit: arguments");
    return accept_commit(ctx, "hs_accept_commit", args, cache, seq, step, policy, stream);
}

hs_status hs_poll_error(hs_ctx* ctx, hs_stream stream, uint32_t* error_bits) {
    if (!ctx || !error_bits) return HS_ERR_INVALID_ARG;
    // the error word: in the workspace, or -- no workspace bound, only hs_draft_static can have run -- in its array
    char* word = ctx->ws ? ctx->ws + ctx->lay.err : nullptr;
    if (!word) {
        hipError_t why = hipSuccess;
        word = reinterpret_cast<char*>(hs_draft_static_error_word(&why));
        if (!word) return fail(ctx, HS_ERR_CAPACITY, "no workspace bound");
    }
    hipStream_t st = (hipStream_t)stream;
    uint32_t v = 0;
    if (hipMemcpyAsync(&v, word, 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess)
        return fail(ctx, HS_ERR_HIP, "hs_poll_error: copy failed");
    if (v != 0) {
        uint32_t zero = 0;
        if (hipMemcpyAsync(word, &zero, 4, hipMemcpyHostToDevice, st) != hipSuccess ||
            hipStreamSynchronize(st) != hipSuccess)
            return fail(ctx, HS_ERR_HIP, "hs_poll_error: clear failed");
    }
    *error_bits = v;
    return HS_OK;
}

hs_status hs_debug_buffer(const hs_ctx* ctx, int32_t which, void** dev_ptr, size_t* bytes) {
    if (!ctx || !dev_ptr || !bytes || !ctx->ws) return HS_ERR_INVALID_ARG;
    const hs_model_desc& d = ctx->desc;
    const size_t M = (size_t)ctx->lim.max_rows, qh = (size_t)d.n_q_heads * d.head_dim;
    const size_t ab = hs_fp32_activations(ctx) ? 4 : 2;
    switch (which) {
        case 0: *dev_ptr = ctx->ws + ctx->lay.xn; *bytes = M * d.d_model * ab; break;
        case 1: *dev_ptr = ctx->ws + ctx->lay.q; *bytes = M * qh * ab; break;
        case 2: *dev_ptr = ctx->ws + ctx->lay.attn; *bytes = M * qh * ab; break;
        case 3:
            if (ctx->lay.logits_bytes == 0) return HS_ERR_INVALID_ARG;   // no logits kept: see HS_FLAG_WORKSPACE_LOGITS
            *dev_ptr = ctx->ws + ctx->lay.logits; *bytes = ctx->lay.logits_bytes; break;
        case 4: *dev_ptr = ctx->ws + ctx->lay.x; *bytes = M * d.d_model * 4; break;
        case 5: *dev_ptr = ctx->ws + ctx->lay.act; *bytes = M * (size_t)d.d_ffn * ab; break;
        default: return HS_ERR_INVALID_ARG;
    }
    return HS_OK;
}

size_t hs_debug_capture_bytes(const hs_ctx* ctx) { return ctx ? 4 * capture_slot_bytes(ctx) : 0; }

hs_status hs_debug_capture(hs_ctx* ctx, void* dev_ptr, size_t bytes) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (dev_ptr && bytes < 4 * capture_slot_bytes(ctx))
        return fail(ctx, HS_ERR_CAPACITY, "hs_debug_capture: buffer smaller than hs_debug_capture_bytes");
    ctx->capture = (char*)dev_ptr;
    return HS_OK;
}

hs_status hs_gate_table_build(const float* ms, const int32_t* rows, int32_t n_points, float k_bar, int32_t b_max,
                              int32_t* table17) {
    if (!ms || !rows || !table17 || n_points < 2 || !(k_bar >= 0.f) || b_max < 0) return HS_ERR_INVALID_ARG;
    for (int i = 1; i < n_points; i++)
        if (rows[i] <= rows[i - 1]) return HS_ERR_INVALID_ARG;
    // step time at m rows: the segment of the profile that contains m, the outer segments continued beyond the ends
    auto t = [&](double m) {
        int seg = n_points - 2;
        for (int i = 0; i + 1 < n_points - 1; i++)
            if (m <= rows[i + 1]) { seg = i; break; }
        const double rise = (double)ms[seg + 1] - (double)ms[seg], run = (double)rows[seg + 1] - (double)rows[seg];
        return (double)ms[seg] + rise * (m - (double)rows[seg]) / run;
    };
    for (int i = 0; i <= 16; i++) {
        const double gain = 1.0 + (double)k_bar * i / 16.0;
        int best = 0;
        for (int b = 1; b <= b_max; b++)
            if (gain * t(b) >= t(b * (1.0 + (double)k_bar))) best = b;
        table17[i] = best;
    }
    return HS_OK;
}

hs_status hs_plan_allocation(const double* tau, int32_t n_groups, int32_t min_wks, int32_t max_wks, int32_t wks,
                             double t_train, double precision, int32_t* plan, double* d_out) {
    if (!tau || !plan || !d_out || n_groups < 1 || min_wks < 1 || max_wks < min_wks || wks < 1 || !(precision > 0.0))
        return HS_ERR_INVALID_ARG;
    const int width = max_wks - min_wks + 1;
    const double t0 = std::max(tau[width - 1], t_train);
    std::vector<int32_t> trial((size_t)n_groups);
    // workers needed at gradient d (the fewest per group that meet t0 + i d), -1 if a group cannot meet its target
    auto workers_at = [&](double d) -> long {
        long total = 0;
        for (int i = 0; i < n_groups; i++) {
            const double* row = tau + (size_t)i * width;
            const double target = t0 + i * d;
            int k = 0;
            while (k < width && !(row[k] <= target)) k++;
            if (k == width) return -1;
            trial[i] = min_wks + k;
            total += trial[i];
        }
        return total;
    };
    double lo = 0.0;
    double hi = n_groups > 1 ? (tau[(size_t)(n_groups - 1) * width] - t0) / (n_groups - 1) : 0.0;
    if (hi < 0.0) hi = 0.0;
    long need = workers_at(hi);
    if (need < 0 || need > wks) return HS_ERR_CAPACITY;
    std::copy(trial.begin(), trial.end(), plan);
    while (hi - lo > precision) {
        const double mid = (hi + lo) / 2;
        need = workers_at(mid);
        if (need < 0 || need > wks) {
            lo = mid;
        } else {
            std::copy(trial.begin(), trial.end(), plan);
            hi = mid;
        }
    }
    *d_out = hi;
    return HS_OK;
}

hs_status hs_debug_gemm(hs_ctx* ctx, int32_t epi, const void* a, const void* w, const void* w2, void* c,
                        const int32_t* m_dev, int32_t m_max, int32_t n, int32_t k, int32_t rows_hint,
                        hs_stream stream) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    if (!ctx->ws) return fail(ctx, HS_ERR_CAPACITY, "no workspace bound");
    if (epi < HS_EPI_STORE_F32 || epi > HS_EPI_ROWMAX || !a || !w || !c || !m_dev ||
        (epi == HS_EPI_SWIGLU_BF16 && !w2))
        return fail(ctx, HS_ERR_INVALID_ARG, "hs_debug_gemm: arguments");
    const hs_model_desc& d = ctx->desc;
    const long long qh = (long long)d.n_q_heads * d.head_dim;
    const long long nqkv = (long long)(d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    const long long n_lim = std::max<long long>({d.vocab, d.d_ffn, nqkv, d.d_model});
    const long long k_lim = std::max<long long>({d.d_model, d.d_ffn, qh});
    if (m_max < 1 || m_max > ctx->lim.max_rows || n < 1 || n > n_lim || k < 64 || k > k_lim || k % 64 != 0)
        return fail(ctx, HS_ERR_INVALID_ARG, "hs_debug_gemm: shape outside the context's model");
    // the split execution writes chunks * m_max * n floats of partial sums
    const int chunks = (epi == HS_EPI_SWIGLU_BF16 || epi == HS_EPI_ROWMAX) ? 1 : hs_gemm_chunks(n, k);
    if (chunks > 1 && (size_t)chunks * m_max * n * 4 > ctx->lay.gemm_part_bytes)
        return fail(ctx, HS_ERR_CAPACITY, "hs_debug_gemm: partial-sum scratch too small for this shape");
    (void)hipGetLastError();
    hs_launch_gemm(ctx, epi, (const bf16_t*)a, (const bf16_t*)w, (const bf16_t*)w2, c, m_dev, m_max, n, k,
                   rows_hint > 0 ? rows_hint : m_max, (hipStream_t)stream);
    if (hipError_t e = hipGetLastError(); e != hipSuccess) return fail_hip(ctx, "hs_debug_gemm", e);
    return HS_OK;
}

int32_t hs_debug_rowmax_groups(int32_t n) { return n > 0 ? hs_gemm_rowmax_groups(n) : 0; }

hs_status hs_set_profile(hs_ctx* ctx, int32_t enabled) {
    if (!ctx) return HS_ERR_INVALID_ARG;
    ctx->profile = enabled <= 0 ? 0 : (enabled == 1 ? 1 : 2);
    ctx->ev_used = 0;
    return HS_OK;
}

hs_status hs_get_profile(hs_ctx* ctx, float ms[5], int32_t launches[5]) {
    if (!ctx || !ms || !launches) return HS_ERR_INVALID_ARG;
    for (int i = 0; i < 5; i++) { ms[i] = 0.f; launches[i] = 0; }
    if (!ctx->profile || ctx->ev_used < 2) return fail(ctx, HS_ERR_INVALID_ARG, "no profiled hs_verify to report");
    if (hipEventSynchronize(ctx->ev[ctx->ev_last]) != hipSuccess)
        return fail(ctx, HS_ERR_HIP, "hs_get_profile: sync failed");
    for (int p = 0; p < ctx->ev_used / 2; p++) {
        float t = 0.f;
        if (hipEventElapsedTime(&t, ctx->ev[2 * p], ctx->ev[2 * p + 1]) != hipSuccess)
            return fail(ctx, HS_ERR_HIP, "hs_get_profile: elapsed time failed");
        int c = ctx->ev_class[p];
        ms[c] += t;
        launches[c] += 1;
    }
    ctx->ev_used = 0;
    return HS_OK;
}

}  // extern "C"
