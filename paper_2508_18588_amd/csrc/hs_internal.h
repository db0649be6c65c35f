// Internal declarations shared by the HIP translation units of libhistospec.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "histospec.h"

typedef uint16_t bf16_t;  // storage type: upper half of an fp32

// Keys per split-KV partition of the verify attention when nothing else is known (hs_create picks 256, 512 or 1024
// from the context's limits).  Partitions are keyed to absolute position, so a row's reduction order does not
// depend on how many draft rows share its sequence.
constexpr int HS_ATT_PART_DEFAULT = 512;
// History segment scanned by one workgroup of the draft kernel.
constexpr int HS_DRAFT_SEG = 4096;
constexpr int HS_MAX_NODES = 64;  // ancestor masks are 64-bit

struct hs_workspace_layout {
    size_t x, xn, qkv, q, attn, act, part_o, part_ml, logits, logits_bytes, rowmax, draft_best, gemm_part, gemm_part_bytes, err, pf_len, att_work, att_list, total;
};

struct hs_ctx {
    hs_model_desc desc;
    hs_limits lim;
    const bf16_t *embed, *lm_head;
    const float *norm_f, *rope_cs;
    std::vector<const bf16_t*> wqkv, wo, wgate, wup, wdown;
    std::vector<const float*> norm1, norm2;
    uint32_t flags = 0;
    char* capture = nullptr;  // hs_debug_capture: snapshots of the last layer's projection inputs
    char* ws = nullptr;
    size_t ws_bytes = 0;
    hs_workspace_layout lay;
    int att_part = HS_ATT_PART_DEFAULT;
    int max_parts = 0;
    int max_segs = 0;
    int n_cu = 256;  // compute units of the device the context was created on
    std::string err;
    // profiling
    int profile = 0;
    std::vector<hipEvent_t> ev;  // pairs
    std::vector<int> ev_class;
    int ev_used = 0;
    int ev_last = 0;
};

static inline __host__ __device__ float bf16_to_f32(bf16_t b) {
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)b << 16;
    return c.f;
}

// Round to nearest even (inputs here are never NaN).
static inline __host__ __device__ bf16_t f32_to_bf16(float f) {
    union { uint32_t u; float f; } c;
    c.f = f;
    uint32_t u = c.u;
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

// hs_set_flags: plain kernels (either flag), and with them activations and KV cache in fp32.
static inline bool hs_fp32_activations(const hs_ctx* ctx) { return (ctx->flags & HS_FLAG_FP32_ACTIVATIONS) != 0; }
static inline bool hs_plain_kernels(const hs_ctx* ctx) {
    return (ctx->flags & (HS_FLAG_REFERENCE_KERNELS | HS_FLAG_FP32_ACTIVATIONS)) != 0;
}
int hs_gemm_chunks(int n, int k);
// Must the logits exist as an [rows][vocab] array?  Yes if the caller asks for them (a destination in the step, or
// HS_FLAG_WORKSPACE_LOGITS), with the plain kernels, and when the LM head splits K (a small vocabulary).  Otherwise the
// LM head reduces every row to its argmax in its epilogue and hs_accept finishes the reduction.
static inline bool hs_logits_in_workspace(const hs_ctx* ctx) {
    return (ctx->flags & HS_FLAG_WORKSPACE_LOGITS) != 0 || hs_plain_kernels(ctx) ||
           hs_gemm_chunks(ctx->desc.vocab, ctx->desc.d_model) > 1;
}
static inline bool hs_head_fused(const hs_ctx* ctx, const hs_step* step) {
    return !step->logits && !hs_logits_in_workspace(ctx);
}

// Grid of a row-strided kernel (workgroup i takes rows i, i + grid, ...) whose workgroups have `threads` threads and
// of which `per_row` work on one row: what the device holds at once (2048 threads per compute unit), at most one
// set per row.  The row count itself is only known on the device.
static inline int hs_row_grid(const hs_ctx* ctx, int threads, int per_row = 1) {
    const int resident = ctx->n_cu * (2048 / threads) / per_row;
    return resident < 1 ? 1 : (resident < ctx->lim.max_rows ? resident : ctx->lim.max_rows);
}

// ---- launchers (each enqueues on `st`; shapes have been validated by the caller) ----

// GEMM family: C[M,N] (+)= A[M,K] . W[N,K]^T, A and W bf16, fp32 accumulation in a fixed k order.
// Activation buffers (a, and c of the SwiGLU epilogue) are bf16, or float in the fp32-activation mode.
// m_dev points at the row count M on the device; the grid covers m_max rows and tiles beyond M exit.
// HS_EPI_ROWMAX (LM head only, unsplit K): nothing of the product is stored; every workgroup reduces its columns of
// each row to one 64-bit key, (order-preserving bits of the largest value) << 32 | ~column, smallest column on ties,
// written to c as unsigned long long [m_max][hs_gemm_rowmax_groups(n)] -- the maximum over a row's keys is its argmax.
enum { HS_EPI_STORE_F32 = 0, HS_EPI_ADD_F32 = 1, HS_EPI_SWIGLU_BF16 = 2, HS_EPI_ROWMAX = 3 };
// rows_hint (host-side estimate of the live row count) selects the tile height and the split execution
// (one workgroup per K chunk + an ordered reduce); results are identical whatever it is.
// pending: if not null and the split execution was chosen, the ordered reduce is NOT launched: *pending receives the
// number of chunk partials left in the workspace ([chunk][m_max][n] floats at lay.gemm_part) for the next kernel in
// line to add up in chunk order and apply the epilogue (store / add to c); otherwise *pending = 0.
void hs_launch_gemm(const hs_ctx* ctx, int epi, const void* a, const bf16_t* w, const bf16_t* w2, void* c,
                    const int32_t* m_dev, int m_max, int n, int k, int rows_hint, hipStream_t st,
                    int* pending = nullptr);
int hs_gemm_rowmax_groups(int n);   // column groups (= keys per row) of an HS_EPI_ROWMAX launch over n columns

void hs_launch_embed(const hs_ctx* ctx, const hs_step* step, int batch, float* x, hipStream_t st);
// RMSNorm of the residual stream; with pending_chunks > 0 it first adds the pending chunk partials of the
// preceding projection (in chunk order) to x.
void hs_launch_rmsnorm(const hs_ctx* ctx, float* x, const float* w, void* out, const int32_t* m_dev,
                       int pending_chunks, hipStream_t st);
// Rotary embedding + KV write; with pending_chunks > 0 the QKV values are the chunk-ordered sums of the pending
// partials instead of qkv.
void hs_launch_rope_kv(const hs_ctx* ctx, int layer, const hs_kv_cache* cache, const hs_seq_state* seq,
                       const hs_step* step, const float* qkv, void* q, int pending_chunks, hipStream_t st);
void hs_launch_attention(const hs_ctx* ctx, int layer, const hs_kv_cache* cache, const hs_seq_state* seq,
                         const hs_step* step, const void* q, void* out, hipStream_t st);
// Chunked prefill: row arrays of one call (rows of sequence b = its next tokens from the token log) and the causal
// attention over [0, kv_done + i] for token i of the chunk.  len_plus1[b] = cached positions + 1.
void hs_launch_prefill_rows(const hs_ctx* ctx, const hs_seq_state* seq, int32_t* kv_done, int chunk, hs_step* step,
                            int32_t* len_plus1, hipStream_t st);
void hs_launch_attention_prefill(const hs_ctx* ctx, int layer, const hs_kv_cache* cache, const hs_seq_state* seq,
                                 const int32_t* len_plus1, const hs_step* step, const bf16_t* q, bf16_t* out, int chunk,
                                 hipStream_t st);
// Unit lists of the verify attention (one per hs_verify call, before the first layer) and their capacity.
void hs_launch_attention_worklist(const hs_ctx* ctx, const hs_seq_state* seq, const hs_step* step, hipStream_t st);
size_t hs_attention_max_units(const hs_ctx* ctx);
void hs_launch_attention_merge(const hs_ctx* ctx, const hs_seq_state* seq, const hs_step* step, void* out,
                               hipStream_t st);
void hs_launch_argmax(const hs_ctx* ctx, const float* logits, int32_t* argmax, const int32_t* m_dev,
                      hipStream_t st);
void hs_launch_draft(const hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step,
                     hipStream_t st);
// hs_draft_static: segment winners in a static device array of HS_DRAFT_STATIC_ENTRIES slots.  Returns false (with the
// HIP error) if the array's address on the current device cannot be had.  hs_draft_static_error_word: the error word
// kept inside that array (used when no workspace is bound).
constexpr int HS_DRAFT_STATIC_ENTRIES = 1 << 16;
bool hs_launch_draft_static(const hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step,
                            hipStream_t st, hipError_t* why);
uint32_t* hs_draft_static_error_word(hipError_t* why);
void hs_launch_draft_group(const hs_ctx* ctx, const hs_group_draft_args* args, const hs_seq_state* seq,
                           hs_step* step, hipStream_t st);
// Acceptance and/or commit of one step in one launch.  args == nullptr: no acceptance; policy == nullptr: no commit.
// keys != nullptr: the rows' argmax is first reduced from the LM head's row-maximum keys (n_keys per row).
void hs_launch_accept_commit(const hs_ctx* ctx, const hs_accept_args* args, const hs_kv_cache* cache,
                             const hs_seq_state* seq, const hs_step* step, const float* logits,
                             const unsigned long long* keys, int n_keys, const hs_policy* policy, hipStream_t st);
