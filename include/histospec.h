/*
 * histospec.h -- C ABI of the history-drafted speculative decoding hot path for AMD MI355X (gfx950).
 *
 * One decode iteration of the HistoSpec rollout engine ("History Rhymes", arXiv 2508.18588, Sec. 5.2-5.4 and
 * Sec. 2.2) is four calls enqueued on one HIP stream, with no host synchronisation in between:
 *
 *     hs_draft      every in-flight response matches its last generated tokens against its previous-epoch
 *                   response and takes the following tokens as draft              (Sec. 5.2, Sec. 5.4)
 *     hs_verify     the target decoder computes the logits of all draft positions in one forward pass over
 *                   the paged KV cache                                            (Sec. 2.2, Sec. 5.2)
 *     hs_accept     the valid draft tokens are kept (greedy comparison or rejection sampling), plus one token
 *                   from the model itself                                         (Sec. 2.2)
 *     hs_kv_commit  sequence length, KV cache, pattern tail and speculation window move forward by what was
 *                   accepted                                                      (Sec. 5.4 window rule)
 *
 * Conventions
 *   - Every pointer marked DEVICE is device memory allocated by the caller (e.g. through PyTorch) that outlives
 *     the call; the library allocates no device memory, creates no stream and never synchronises one (except
 *     hs_poll_error).  HOST pointers are read during the call only.
 *   - All calls return an hs_status.  Errors the host can see (NULL pointers, sizes beyond hs_limits, missing
 *     workspace) are returned immediately and nothing is launched.  Conditions only the device can see (a
 *     sequence that outgrows its block table) set a sticky device error word, skip the offending sequence's
 *     writes, and are reported by hs_poll_error.
 *   - hs_stream is a hipStream_t passed as an opaque pointer (NULL = the null stream).
 *   - Token ids, positions and indices are int32.  bf16 means the upper 16 bits of an IEEE fp32.
 *
 * Sequence model.  Sequence b has n_b = seq_len[b] committed tokens (prompt + response so far).  The KV cache
 * holds positions 0 .. n_b-2; the newest committed token (the "root", position L_b = n_b-1) gets its K/V from
 * the next hs_verify.  A sequence with budget_left[b] <= 0 is finished and contributes no rows.
 *
 * Rows.  hs_draft flattens the batch into M = sum_b n_nodes_b rows; row_off[b] .. row_off[b+1] are sequence b's
 * draft-tree nodes: node 0 is the root, nodes 1.. are draft tokens in creation order (candidate 0's chain, then
 * for each later candidate the part after its shared prefix).  M is known on the device only (row_off[batch]).
 */
#ifndef HISTOSPEC_H
#define HISTOSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hs_ctx hs_ctx;
typedef void* hs_stream;

typedef enum hs_status {
    HS_OK = 0,
    HS_ERR_INVALID_ARG = -1, /* NULL / out-of-range argument */
    HS_ERR_CAPACITY = -2,    /* exceeds hs_limits or the bound workspace */
    HS_ERR_UNSUPPORTED = -3, /* model shape or option this build has no kernel for */
    HS_ERR_HIP = -4          /* a HIP runtime call failed; see hs_last_error */
} hs_status;

/* Device error word bits (hs_poll_error). */
enum { HS_DEV_BLOCK_TABLE_OVERFLOW = 1, HS_DEV_POSITION_OVERFLOW = 2, HS_DEV_ROW_OVERFLOW = 4 };

enum { HS_K_FIXED = 0, HS_K_MATCHLEN = 1, HS_K_AIMD = 2 }; /* hs_policy.k_mode */
enum { HS_ACCEPT_GREEDY = 0, HS_ACCEPT_REJECTION = 1 };    /* hs_accept_args.mode */
/* hs_set_flags.  HS_FLAG_REFERENCE_KERNELS: hs_verify runs plain (slow) GEMM and attention kernels on the same bf16
 * activation buffers and cache.  HS_FLAG_FP32_ACTIVATIONS: the precise mode -- the plain kernels, with every
 * activation kept in fp32 between operations (normed input, queries, attention output, feed-forward activation),
 * sums carried in fp64, and the KV cache holding fp32 values: hs_kv_cache.k / .v then point at float arrays of the
 * same index layout (twice the bytes), for hs_verify and hs_kv_commit alike.  Only the bf16 weights are rounded, as in
 * the definition of the model, so logits agree with an fp64 evaluation to fp32 rounding (about 1e-5 of a row's
 * largest logit at 28 layers).  Slow; meant for checking the fast path's rounding, not for serving.
 * HS_FLAG_WORKSPACE_LOGITS: hs_verify keeps the fp32 logits of all rows in the workspace when hs_step.logits is
 * NULL (rejection sampling needs them; so does hs_debug_buffer 3).  Without the flag and without hs_step.logits no
 * [rows][vocab] array exists at all: the LM head reduces every row to its largest logit per column group in its
 * epilogue, and hs_accept / hs_accept_commit finish the argmax (greedy acceptance only; hs_step.argmax is then
 * written by them, not by hs_verify).  With the plain kernels, or a vocabulary so small that the LM head splits its
 * reduction, the logits are always kept. */
enum { HS_FLAG_REFERENCE_KERNELS = 1, HS_FLAG_FP32_ACTIVATIONS = 2, HS_FLAG_WORKSPACE_LOGITS = 4 };

/* Pre-norm decoder: RMSNorm, rotary embedding (pairs i, i + head_dim/2), grouped-query attention with scale
 * 1/sqrt(head_dim), SwiGLU feed-forward, untied LM head, no biases. */
typedef struct hs_model_desc {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t kv_block; /* tokens per KV page; must be 16 */
    float rms_eps;
} hs_model_desc;

/* Weights.  Matrices are bf16, row-major [out_features, in_features].  The per-layer members are HOST arrays
 * of n_layers DEVICE pointers (copied by hs_create). */
typedef struct hs_weights {
    const void* embed;          /* DEVICE bf16 [vocab, d_model] */
    const void* lm_head;        /* DEVICE bf16 [vocab, d_model] */
    const float* norm_f;        /* DEVICE f32 [d_model], 16-byte aligned (so are norm1[i], norm2[i]) */
    const void* const* wqkv;    /* bf16 [(n_q_heads + 2 n_kv_heads) head_dim, d_model]: q rows, then k, then v */
    const void* const* wo;      /* bf16 [d_model, n_q_heads head_dim] */
    const void* const* wgate;   /* bf16 [d_ffn, d_model] */
    const void* const* wup;     /* bf16 [d_ffn, d_model] */
    const void* const* wdown;   /* bf16 [d_model, d_ffn] */
    const float* const* norm1;  /* f32 [d_model], attention pre-norm */
    const float* const* norm2;  /* f32 [d_model], feed-forward pre-norm */
    const float* rope_cs;       /* DEVICE f32 [max_pos, head_dim/2, 2] = (cos, sin) of position * inv_freq */
} hs_weights;

typedef struct hs_limits {
    int32_t max_batch;          /* sequences in flight */
    int32_t k_max;              /* longest draft chain, 0..32 */
    int32_t c_max;              /* history candidates per sequence, 1 or 2; 1 + c_max*k_max <= 64 nodes, and
                                   (n_q_heads / n_kv_heads) * (1 + c_max*k_max) <= 256 query rows per KV head */
    int32_t max_rows;           /* capacity of the per-row arrays, >= max_batch * (1 + c_max * k_max) */
    int32_t max_blocks_per_seq; /* row length of block_table */
    int32_t max_pos;            /* rows of rope_cs; no position may reach it.  A history candidate is scanned
                                   up to max_pos + 32 tokens */
    int32_t w_max;              /* row length of the pattern tail, 1..32 */
    int32_t g_max;              /* responses per sequence hs_draft_group may be given, 0 (entry point unused)..32 */
} hs_limits;

/* Paged KV cache (DEVICE, bf16, zero-initialised by the caller).
 *   k: [n_layers][n_blocks][n_kv_heads][kv_block][head_dim]
 *   v: [n_layers][n_blocks][n_kv_heads][head_dim][kv_block]   (token index fastest)
 * Position t of sequence b lives in page block_table[b][t / kv_block], slot t % kv_block. */
typedef struct hs_kv_cache {
    void* k;
    void* v;
    int32_t n_blocks;
} hs_kv_cache;

/* Per-sequence state, DEVICE arrays of max_batch entries (caller-owned, updated by hs_kv_commit). */
typedef struct hs_seq_state {
    int32_t batch;            /* HOST: sequences in this batch, <= max_batch */
    int32_t* seq_len;         /* n_b */
    const int32_t* block_table; /* [batch][max_blocks_per_seq], filled by the caller for the sequence's maximum length */
    int32_t* tail;            /* [batch][w_max]: last committed tokens, right-aligned */
    int32_t* tail_len;        /* valid entries at the right end of tail[b] */
    int32_t* k_state;         /* speculation window (HS_K_AIMD) */
    int32_t* budget_left;     /* response tokens the sequence may still emit */
    const uint64_t* seq_id;   /* random-stream identity of the sequence */
    int32_t* tokens;          /* optional [batch][tokens_stride]: committed tokens are also appended here at n_b */
    int32_t tokens_stride;
    uint64_t* counters;       /* optional [4]: sequence-steps, drafted, accepted, emitted tokens (accumulated) */
    int32_t* gate;            /* optional [HS_GATE_WORDS], needs counters: throughput-aware speculation control (see
                                 hs_gate_table_build); zero-initialised by the caller except [4] and the table */
} hs_seq_state;

/* Throughput-aware speculation control (Sec. 5.4, last paragraph: the acceptance rate is monitored, pre-profiling
 * gives the largest batch at which speculation still raises throughput at each rate, above it speculation is
 * switched off).  With hs_seq_state.gate set, hs_draft / hs_draft_group decide once per step for the whole batch:
 *   monitor   D, A <- X - (X >> 3) + (tokens drafted / accepted by the previous step), from `counters`;
 *   bucket    16 A / D rounded down, capped at 16; 16 when D == 0;
 *   decision  speculate iff (sequences with budget left) <= table[bucket], or speculation has been off for
 *             probe_every steps in a row (probe_every = 0: never probe).  Off: every sequence gets a one-row step.
 * Words: [0] D, [1] A, [2] steps since speculation last ran, [3] last decision, [4] probe_every (caller-set),
 * [5] / [6] drafted / accepted totals seen (mod 2^32), [7] decisions made, [8..24] table (caller-set). */
enum { HS_GATE_WORDS = 32, HS_GATE_TABLE = 8 };

/* Draft policy (Sec. 5.4).  Pattern = the last `window` committed tokens; a match must cover at least m_min
 * of them.  HS_K_FIXED drafts k_fixed tokens, HS_K_MATCHLEN as many as matched (clamped to 1..k_max),
 * HS_K_AIMD k_state[b] tokens; all are cut by the history's end and by budget_left - 1.  hs_kv_commit applies
 * the window rule: +aimd_inc up to aimd_cap when every drafted token on the path was accepted, aimd_reset on
 * a rejection, unchanged when nothing was drafted. */
typedef struct hs_policy {
    int32_t window, m_min;
    int32_t k_mode, k_fixed, k_max;
    int32_t aimd_inc, aimd_cap, aimd_reset;
} hs_policy;

/* History of the previous epoch.  Candidate c of sequence b is hist[hist_off[b*n_cand+c] .. hist_off[b*n_cand+c+1]).
 * The caller prepends the last window-1 prompt tokens to each response so the response start is matchable. */
typedef struct hs_draft_args {
    int32_t n_cand;           /* 1..c_max */
    const int32_t* hist;      /* DEVICE, 16-byte aligned (the candidates inside it may start anywhere) */
    const int32_t* hist_off;  /* DEVICE [batch*n_cand + 1] */
    hs_policy policy;
} hs_draft_args;

/* Arguments of hs_draft_group: the n_resp responses the prompt of sequence b got in its last rollout are
 * hist[hist_off[b*n_resp + g] .. hist_off[b*n_resp + g + 1]), g = 0..n_resp-1 (each carrying the last window-1 prompt
 * tokens in front, as for hs_draft), reward[b*n_resp + g] in 0..2^20 the reward that response earned. */
typedef struct hs_group_draft_args {
    int32_t n_resp;           /* 1..g_max */
    const int32_t* hist;      /* DEVICE, 16-byte aligned */
    const int32_t* hist_off;  /* DEVICE [batch*n_resp + 1] */
    const int32_t* reward;    /* DEVICE [batch*n_resp] */
    hs_policy policy;
} hs_group_draft_args;

/* One iteration's arrays (DEVICE, caller-owned).  Sizes: per-candidate arrays batch*c_max, per-row arrays
 * max_rows, per-sequence arrays max_batch. */
typedef struct hs_step {
    int32_t* draft_start;  /* [batch*n_cand] index in the candidate's history of the first draft token, -1 = no match */
    int32_t* match_len;    /* [batch*n_cand] matched pattern length (0 = none) */
    int32_t* draft_len;    /* [batch*n_cand] draft tokens taken from that candidate */
    int32_t* row_off;      /* [batch+1] */
    int32_t* tok;          /* [M] token of each node */
    int32_t* pos;          /* [M] absolute position (rotary position) = L_b + depth */
    int32_t* parent;       /* [M] parent node index within the sequence, -1 for the root */
    uint64_t* anc_mask;    /* [M] bit i: node i of the same sequence is this node or an ancestor */
    int32_t* row2seq;      /* [M] */
    float* logits;         /* optional [max_rows][vocab]; NULL: no logits are kept unless HS_FLAG_WORKSPACE_LOGITS */
    int32_t* argmax;       /* [M] lowest index of the largest logit (written by hs_verify, or by hs_accept when no
                              logits are kept) */
    int32_t* accept_len;   /* [batch] accepted draft tokens a_b */
    int32_t* n_out;        /* [batch] emitted tokens (a_b + 1; 0 for a finished sequence) */
    int32_t* out_tok;      /* [batch][k_max+1] emitted tokens */
    int32_t* path_row;     /* [batch][k_max+1] node index of the root and of each accepted node */
    int32_t rows_hint;     /* HOST: rows M the caller expects this step (e.g. last step's row_off[batch]), 0 =
                              unknown.  Only steers how kernels are launched; results do not depend on it. */
    int32_t* draft_src;    /* [batch] hs_draft_group only (may be NULL otherwise): the response the draft was read
                              from, -1 = no match.  hs_draft_group uses entry b (not b*n_cand) of draft_start,
                              match_len and draft_len. */
} hs_step;

typedef struct hs_accept_args {
    int32_t mode;
    float temperature;  /* HS_ACCEPT_REJECTION only, > 0 */
    uint64_t seed;      /* Philox key */
} hs_accept_args;

/* Validates the shape and copies the descriptors.  Supported: head_dim 64 or 128, kv_block 16, n_q_heads a
 * multiple of n_kv_heads with at most 8 query heads per KV head, d_model / d_ffn / n_q_heads*head_dim multiples
 * of 64, d_model at most 16384.  The norm weight vectors must be 16-byte aligned (HS_ERR_INVALID_ARG otherwise).
 * The length of the attention's split-KV partitions (256, 512 or 1024 keys) is chosen here from the limits
 * alone -- results of contexts created with different limits can differ in the last bits. */
hs_status hs_create(const hs_model_desc* desc, const hs_weights* weights, const hs_limits* limits, hs_ctx** out);
void hs_destroy(hs_ctx* ctx);
const char* hs_last_error(const hs_ctx* ctx);
/* Changing the flags can change hs_workspace_bytes; a bound workspace that is too small for the new layout is
 * unbound (bind a larger one before the next call).  hs_prefill supports neither of the plain-kernel flags. */
hs_status hs_set_flags(hs_ctx* ctx, uint32_t flags);

/* Scratch the kernels need (activations, split-KV partials, logits).  The caller allocates at least
 * hs_workspace_bytes(ctx) DEVICE bytes, 256-byte aligned, zero-filled, and binds them before the first step. */
size_t hs_workspace_bytes(const hs_ctx* ctx);
hs_status hs_bind_workspace(hs_ctx* ctx, void* dev_ptr, size_t bytes);

/* Longest-suffix-match draft (Sec. 5.2; pattern backoff of Sec. 5.4 == longest match capped at `window`,
 * at least m_min; leftmost on ties).  Writes draft_start/match_len/draft_len, builds the node arrays and
 * row_off.  Reads seq.tail/tail_len/seq_len/k_state/budget_left. */
hs_status hs_draft(hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step, hs_stream stream);

/* hs_draft for callers that cannot allocate device memory or have none to spare for this call (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, same results bit for bit, but the
 * kernels' scratch -- one 8-byte winner per (sequence, candidate, 4096-token history segment) -- lives in a static
 * device array inside the library (65536 slots = 512 KiB, held by every GPU the library runs on until the process
 * ends) instead of the bound workspace; no workspace needs to be bound, and nothing is allocated or freed.
 * HS_ERR_CAPACITY if batch * n_cand * ceil((max_pos + 32) / 4096) exceeds 65536.  The device error word is the
 * workspace's if one is bound, else a word inside the static array (hs_poll_error reads whichever applies).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams) race;
 * calls on one stream, or ordered by events, are safe.  The array's address is looked up per device on the first
 * call made with that device current. */
hs_status hs_draft_static(hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step,
                          hs_stream stream);

/* Reward-aware draft from ALL responses of the prompt's last rollout (Sec. 5.3: the responses are indexed together,
 * every branch carries the summed rewards of the responses below it, and where the continuations of the matched
 * pattern differ the branch with the highest priority is followed).  Stated on the flat responses:
 *   1. m* = longest common suffix (capped at `window`, at least m_min) between the committed tokens and any place
 *      p in [1, len-1] of any response;
 *   2. the occurrences of that pattern, in (response, position) order, at most 1024 of them;
 *   3. draft token by draft token, every live occurrence votes for its next token with its response's reward; the
 *      largest reward sum wins, then the larger number of votes, then the smaller token id; occurrences that voted
 *      otherwise or ran out of text drop out; the walk ends after the policy's K tokens (cut by k_max and the
 *      response budget - 1) or when no live occurrence has a token left.
 * The result is a chain: draft_src[b] / draft_start[b] name the first surviving occurrence (the draft is the text
 * after it), match_len[b] = m*, draft_len[b] the tokens drafted; node arrays and row_off as for hs_draft. */
hs_status hs_draft_group(hs_ctx* ctx, const hs_group_draft_args* args, const hs_seq_state* seq, hs_step* step,
                         hs_stream stream);

/* One target-model forward pass over all M rows (Sec. 2.2).  Writes every row's K/V into the cache at slot
 * L_b + node index, attends over positions [0, L_b) plus the node's ancestors-or-self, and writes
 * (Numerical range: the attention runs split over key partitions whose partial outputs -- each a convex combination
 * of cached V rows -- are held in fp16 before they are merged in fp32.  Results are therefore as described only
 * while |V| < 65504 for every cached value, and V components below 6e-5 in magnitude lose bits (below 6e-8 they
 * vanish) in that intermediate; activations of a normalised decoder are far inside this range.)
 * the logits (to step.logits; or to the workspace if that is NULL and HS_FLAG_WORKSPACE_LOGITS is set) and
 * step.argmax -- or, with neither, only per-row maxima from which hs_accept derives step.argmax (see hs_set_flags). */
hs_status hs_verify(hs_ctx* ctx, const hs_kv_cache* cache, const hs_seq_state* seq, hs_step* step, hs_stream stream);

/* Chunked prefill: recomputes the KV cache of text that already exists -- the prompt, or the prompt plus the tokens a
 * migrated / deferred rollout had generated before it was moved (Sec. 6.3: such rollouts keep their tokens and
 * continue after the cache has been recomputed rather than transferred).  One call pushes, for every sequence, its
 * next min(chunk, seq_len[b] - 1 - kv_done[b]) tokens from the token log seq.tokens (positions kv_done[b]...)
 * through the decoder: token i attends to positions [0, kv_done[b] + i], its K/V go to slot kv_done[b] + i of every
 * layer, and kv_done[b] advances.  (The newest token, position seq_len - 1, is the root of the next hs_verify and is
 * never prefilled.)  Sequences are served in index order until max_rows rows are laid out; one that does not fit
 * entirely gets the rows that are left, later ones none: call again until kv_done[b] == seq_len[b] - 1 for all b
 * (ceil(total tokens / max_rows) calls at least; the host knows the lengths).  No logits are computed.
 * Overwrites step.row_off / tok / pos / parent / row2seq (the other step arrays are not touched).  The result at a
 * position does not depend on how the text is cut into chunks or calls. */
enum { HS_PREFILL_CHUNK_MAX = 1024 };
typedef struct hs_prefill_args {
    int32_t chunk;      /* HOST: at most this many tokens per sequence and call, 1..HS_PREFILL_CHUNK_MAX */
    int32_t rows_hint;  /* HOST: rows expected in this call (launch shapes only), 0 = unknown */
    int32_t* kv_done;   /* DEVICE [batch] in/out: positions of sequence b already in the cache */
} hs_prefill_args;
hs_status hs_prefill(hs_ctx* ctx, const hs_kv_cache* cache, const hs_seq_state* seq, hs_step* step,
                     const hs_prefill_args* args, hs_stream stream);

/* Acceptance (Sec. 2.2).  Greedy: follow children whose token equals the parent's argmax.  Rejection: accept
 * child j at a node with probability p(tok), p = softmax(logits/temperature) with earlier rejected tokens
 * removed; finish with one inverse-CDF sample (token-id order).  Uniforms: Philox-4x32-10, key = seed, counter
 * = (position of the token being decided, j or 7 for the final sample, seq_id lo, seq_id hi), word 0 >> 8. */
hs_status hs_accept(hs_ctx* ctx, const hs_accept_args* args, const hs_seq_state* seq, hs_step* step, hs_stream stream);

/* Moves accepted nodes' K/V to consecutive slots L_b+1.. (a no-op for a chain), then seq_len += n_out,
 * budget_left -= n_out, tail/tokens/k_state/counters updated. */
hs_status hs_kv_commit(hs_ctx* ctx, const hs_kv_cache* cache, hs_seq_state* seq, const hs_step* step,
                       const hs_policy* policy, hs_stream stream);

/* hs_accept followed by hs_kv_commit as ONE kernel launch (one workgroup per sequence: argmax of its rows where the
 * LM head left only row maxima, acceptance walk or rejection sampling, K/V relocation, state update): same arguments,
 * same results bit for bit as the two calls in a row. */
hs_status hs_accept_commit(hs_ctx* ctx, const hs_accept_args* args, const hs_kv_cache* cache, hs_seq_state* seq,
                           hs_step* step, const hs_policy* policy, hs_stream stream);

/* Synchronises `stream`, returns and clears the sticky device error word. */
hs_status hs_poll_error(hs_ctx* ctx, hs_stream stream, uint32_t* error_bits);

/* Debug view of workspace buffers, valid after hs_verify: 0 final hidden state bf16 [max_rows][d_model]
 * (after the last RMSNorm), 1 last layer's queries bf16 [max_rows][n_q_heads*head_dim] (after rotation),
 * 2 last layer's attention output bf16 (same shape), 3 logits f32 [max_rows][vocab], 4 residual stream after the
 * last layer f32 [max_rows][d_model], 5 last layer's feed-forward activation silu(gate)*up bf16 [max_rows][d_ffn].
 * With HS_FLAG_FP32_ACTIVATIONS buffers 0, 1, 2 and 5 hold floats. */
hs_status hs_debug_buffer(const hs_ctx* ctx, int32_t which, void** dev_ptr, size_t* bytes);

/* Snapshots of what the LAST layer's projections read, for checking each projection of a real forward pass against
 * its definition.  With a DEVICE buffer of hs_debug_capture_bytes(ctx) bytes set (NULL switches it off), every
 * hs_verify copies into four consecutive slots of max_rows * d_model * 4 bytes each:
 *   0 the normed input of the QKV projection (bf16, or float in the fp32-activation mode: the slot's first bytes),
 *   1 the residual stream at that point, f32 (the output of every earlier projection summed in),
 *   2 the normed input of the gate/up projection, 3 the residual stream at that point, f32.
 * Together with hs_debug_buffer 1, 2, 4, 5 and the cache rows written by the step this pins: QKV (slot 0 -> queries
 * and K/V), O (attention output -> slot 3 minus slot 1), gate/up (slot 2 -> activation) and down (activation ->
 * residual after the layer minus slot 3).  The copies are device-to-device on the call's stream. */
size_t hs_debug_capture_bytes(const hs_ctx* ctx);
hs_status hs_debug_capture(hs_ctx* ctx, void* dev_ptr, size_t bytes);

/* HOST helper: the table of the speculation gate from a profiled step time.  ms[i] = duration of one decode step
 * (all four calls) at rows[i] rows, rows ascending, n_points >= 2 (straight lines between neighbours, the outer
 * lines continued beyond the ends).  table17[i] = the largest batch b <= b_max at which drafting k_bar tokens per
 * sequence with acceptance rate i/16 emits at least as many tokens per second as not drafting:
 * (1 + k_bar i/16) t(b) >= t(b (1 + k_bar)); 0 if there is none.  No device work. */
hs_status hs_gate_table_build(const float* ms, const int32_t* rows, int32_t n_points, float k_bar, int32_t b_max,
                              int32_t* table17);

/* HOST: Tier-2 planner of the hybrid rollout pipeline (Sec. 6.2, figure "Tier-2 scheduling algorithm"): how many
 * rollout workers each ranking group gets so that the groups' finish times rise linearly, t(i) = t0 + i d, with the
 * smallest gradient d the cluster can afford.  n_groups ranking groups in ascending order of representative length;
 * tau[i * K + (k - min_wks)], K = max_wks - min_wks + 1, = pre-profiled time of group i on k data-parallel workers
 * (the caller evaluates its profile tau(l, dp), speculation included, at the groups' lengths).  t0 =
 * max(tau(group 0, max_wks), t_train); d is bisected in [0, (tau(last group, min_wks) - t0) / (n_groups - 1)] down
 * to `precision`; for a given d a group takes the fewest workers that meet its target time.  Writes plan[n_groups]
 * and *d_out (the gradient the plan was computed for).  HS_ERR_CAPACITY: even the upper end of the interval needs
 * more than `wks` workers (plan untouched).  No device work; one GPU machine never runs it for more than one worker --
 * it pairs with the sequence-sharded layout described for several GPUs. */
hs_status hs_plan_allocation(const double* tau, int32_t n_groups, int32_t min_wks, int32_t max_wks, int32_t wks,
                             double t_train, double precision, int32_t* plan, double* d_out);

/* The random generator of hs_accept on its own (Philox-4x32-10, Salmon et al., SC'11; key = (seed lo, seed hi)):
 * out[i][0..3] = the four output words of counter ctr[i][0..3], i < n.  ctr and out are DEVICE arrays of 4 n words.
 * hs_accept uses word 0 of counter (position, draw kind, seq_id lo, seq_id hi): u = (word >> 8) / 2^24. */
hs_status hs_debug_philox(const uint32_t* ctr, uint64_t seed, uint32_t* out, int32_t n, hs_stream stream);

/* One projection on its own, through the same launcher hs_verify uses (unit-level parity tests and timing):
 * C[m, n] (+)= A[m, k] . W[n, k]^T with bf16 operands, K-contiguous, fp32 accumulation in the shape's fixed K
 * order.  epi 0: C f32 = product; 1: C f32 += product; 2: SwiGLU, C bf16 [m][n] = silu(A.W^T) * (A.W2^T); 3: the
 * row-maximum epilogue of the LM head: nothing of the product is stored, C is uint64 [m_max][g], g =
 * hs_debug_rowmax_groups(n) column groups, each entry (order-preserving bits of the group's largest value of that
 * row) << 32 | (0xFFFFFFFF - its column), lowest column on ties -- the maximum over a row's entries names its argmax.
 * All pointers are device memory owned by the caller; m_dev points at the int32 row count (<= m_max, the leading
 * dimension of the partial-sum scratch, itself <= the context's max_rows); n, k must not exceed the widest
 * projection of the context's model (the split execution borrows the context's workspace) and k % 64 == 0.
 * rows_hint steers launch shapes only.  Enqueues on `stream`; HS_ERR_INVALID_ARG on bad arguments. */
int32_t hs_debug_rowmax_groups(int32_t n);
hs_status hs_debug_gemm(hs_ctx* ctx, int32_t epi, const void* a, const void* w, const void* w2, void* c,
                        const int32_t* m_dev, int32_t m_max, int32_t n, int32_t k, int32_t rows_hint,
                        hs_stream stream);

/* Kernel timing with HIP events on the call's stream.  hs_set_profile(ctx, level): 0 off; 1 brackets the attention
 * kernel of every fourth layer (0, 4, 8, ...: all layers do the same work) and the whole hs_verify call (cheap enough
 * for a timed run); 2 brackets every kernel launch of hs_verify (each pair of events costs about ten microseconds of
 * stream time: use it on steps that are not themselves being timed).  hs_get_profile waits for the last profiled call and returns, summed over all hs_verify
 * calls since the previous hs_get_profile / hs_set_profile, total milliseconds and launch counts per class (classes
 * that the level does not bracket report zero):
 * 0 attention kernel, 1 projection GEMMs (QKV, O, gate/up, down), 2 LM-head GEMM, 3 everything else (norms,
 * rotary/KV write, split-KV merge, argmax), 4 whole calls.  Events are host objects; no device memory is used. */
hs_status hs_set_profile(hs_ctx* ctx, int32_t enabled);
hs_status hs_get_profile(hs_ctx* ctx, float ms[5], int32_t launches[5]);

#ifdef __cplusplus
}
#endif
#endif /* HISTOSPEC_H */
