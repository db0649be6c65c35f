// Row-wise kernels of the verify forward pass: embedding gather, RMSNorm, rotary embedding + KV-cache write,
// and the per-row argmax over the vocabulary.  All are bandwidth-trivial next to attention and the GEMMs; each
// row is processed independently with a reduction order that depends only on the row's own length.
// The row count lives on the device, so a launch cannot size its grid to it: the grid is what the chip holds at
// once (hs_row_grid) and a workgroup takes rows blockIdx.x, blockIdx.x + gridDim.x, ...  A grid of max_rows
// workgroups, most of which only find that their row does not exist, costs several rounds of workgroup launches
// (a few microseconds) in each of the ~150 row-kernel launches of a step.
#include "hs_internal.h"

namespace {

constexpr int NORM_THREADS = 1024;  // one workgroup of 16 wavefronts per row: few rows, many loads in flight each

__device__ __forceinline__ void put(bf16_t* p, float v) { *p = f32_to_bf16(v); }
__device__ __forceinline__ void put(float* p, float v) { *p = v; }

__device__ inline float block_sum(float v, float* red) {
    // fixed tree: xor-shuffle inside each wavefront, then the wavefront sums left to right
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = red[0];
    for (int w = 1; w < NORM_THREADS / 64; w++) s += red[w];
    return s;
}

__global__ __launch_bounds__(256) void embed_kernel(const bf16_t* __restrict__ embed, const int32_t* __restrict__ tok,
                                                     const int32_t* __restrict__ m_dev, float* __restrict__ x, int d,
                                                     int vocab) {
    const int m = *m_dev;
    for (int row = blockIdx.x; row < m; row += gridDim.x) {
        int t = tok[row];
        if (t < 0 || t >= vocab) t = 0;
        const bf16_t* e = embed + (size_t)t * d;
        for (int i = threadIdx.x; i < d; i += 256) x[(size_t)row * d + i] = bf16_to_f32(e[i]);
    }
}

// One workgroup per row.  With chunks > 0 the row of the residual stream first receives the pending partial sums of
// the preceding projection: t = p0 + p1 + ... in chunk order, x += t -- the arithmetic of the stand-alone ordered
// reduce, so that the split execution gives the same bits whichever kernel finishes it.
// OutT = bf16_t (rounded activations) or float (fp32-activation mode).
// The kernel is a chain of memory round trips, not a stream: a thread keeps its (up to NORM_ITEMS x 4) elements in
// registers from the first load to the normalised store, and the norm weights are fetched with them.
constexpr int NORM_ITEMS = 4;  // d_model <= 4 * NORM_THREADS * NORM_ITEMS = 16384 (checked by hs_create)

__device__ __forceinline__ void put4(bf16_t* p, float4 v) {
    uint2 o;
    o.x = (uint32_t)f32_to_bf16(v.x) | ((uint32_t)f32_to_bf16(v.y) << 16);
    o.y = (uint32_t)f32_to_bf16(v.z) | ((uint32_t)f32_to_bf16(v.w) << 16);
    *reinterpret_cast<uint2*>(p) = o;
}
__device__ __forceinline__ void put4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }

template <typename OutT>
__global__ __launch_bounds__(NORM_THREADS) void rmsnorm_kernel(float* __restrict__ x, const float* __restrict__ w,
                                                       OutT* __restrict__ out, const int32_t* __restrict__ m_dev,
                                                       int d, float eps,
                                                       const float* __restrict__ part, int chunks,
                                                       size_t chunk_stride) {
    __shared__ float red[NORM_THREADS / 64];
    const int m = *m_dev;
    for (int row = blockIdx.x; row < m; row += gridDim.x) {
        float* xr = x + (size_t)row * d;
        const float* pr = part + (size_t)row * d;
        float4 v[NORM_ITEMS], g[NORM_ITEMS];
#pragma unroll
        for (int it = 0; it < NORM_ITEMS; it++) {
            const int i = (threadIdx.x + it * NORM_THREADS) * 4;
            if (i >= d) continue;
            v[it] = *reinterpret_cast<const float4*>(xr + i);
            g[it] = *reinterpret_cast<const float4*>(w + i);
            if (chunks > 0) {
                // several partials of an element in flight at once
                float4 t = *reinterpret_cast<const float4*>(pr + i);
#pragma unroll 8
                for (int c = 1; c < chunks; c++) {
                    const float4 q = *reinterpret_cast<const float4*>(pr + c * chunk_stride + i);
                    t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w;
                }
                v[it].x += t.x; v[it].y += t.y; v[it].z += t.z; v[it].w += t.w;
            }
        }
        // the sum of squares: same element-to-thread assignment and order with and without pending partials -- the
        // norm must not depend on which execution the preceding projection used
        float ss = 0.f;
#pragma unroll
        for (int it = 0; it < NORM_ITEMS; it++) {
            const int i = (threadIdx.x + it * NORM_THREADS) * 4;
            if (i >= d) continue;
            if (chunks > 0) *reinterpret_cast<float4*>(xr + i) = v[it];
            ss += v[it].x * v[it].x;
            ss += v[it].y * v[it].y;
            ss += v[it].z * v[it].z;
            ss += v[it].w * v[it].w;
        }
        ss = block_sum(ss, red);
        const float r = rsqrtf(ss / (float)d + eps);
#pragma unroll
        for (int it = 0; it < NORM_ITEMS; it++) {
            const int i = (threadIdx.x + it * NORM_THREADS) * 4;
            if (i >= d) continue;
            float4 o;
            o.x = v[it].x * r * g[it].x; o.y = v[it].y * r * g[it].y;
            o.z = v[it].z * r * g[it].z; o.w = v[it].w * r * g[it].w;
            put4(out + (size_t)row * d + i, o);
        }
    }
}

// One workgroup per row.  Rotates q and k heads at the row's position (pairs i, i + h/2), writes q as bf16,
// K into its page row-major and V into its page with the token index fastest.
// T = bf16_t, or float in the fp32-activation mode (queries and cache entries then keep every bit).
template <typename T>
__global__ __launch_bounds__(NORM_THREADS) void rope_kv_kernel(const float* __restrict__ qkv, const float* __restrict__ rope_cs,
                                                       const int32_t* __restrict__ pos, const int32_t* __restrict__ row2seq,
                                                       const int32_t* __restrict__ row_off,
                                                       const int32_t* __restrict__ seq_len,
                                                       const int32_t* __restrict__ block_table, int max_blocks,
                                                       int batch, T* __restrict__ q_out, T* __restrict__ kc,
                                                       T* __restrict__ vc, size_t layer_off, int hq, int hkv,
                                                       int h, int max_pos, int n_blocks,
                                                       const float* __restrict__ part, int chunks,
                                                       size_t chunk_stride) {
    extern __shared__ float row_buf[];
    const int m = row_off[batch];
    // (the conditions that skip a row are the same for all threads of the workgroup)
    for (int row = blockIdx.x; row < m; row += gridDim.x) {
        // The row's QKV vector: the projection's output, or the chunk-ordered sum of its pending partials, which is
        // first gathered into LDS with 16-byte loads (several partials of an element in flight at once).  The
        // gather comes first: it depends on nothing but the row, so its loads are on their way while the chain
        // row -> sequence -> slot -> page below is followed.
        const int nqkv = (hq + 2 * hkv) * h;
        if (chunks > 0) {
            if (row != (int)blockIdx.x) __syncthreads();  // row_buf of the previous row has been read
            const float* pr = part + (size_t)row * nqkv;
            for (int i = threadIdx.x * 4; i < nqkv; i += 4 * NORM_THREADS) {
                float4 t = *reinterpret_cast<const float4*>(pr + i);
#pragma unroll 8
                for (int c = 1; c < chunks; c++) {
                    const float4 q4 = *reinterpret_cast<const float4*>(pr + c * chunk_stride + i);
                    t.x += q4.x; t.y += q4.y; t.z += q4.z; t.w += q4.w;
                }
                *reinterpret_cast<float4*>(row_buf + i) = t;
            }
        }
        int b = row2seq[row];
        int node = row - row_off[b];
        int p = pos[row];
        int slot = seq_len[b] - 1 + node;
        int page = (slot >= 0 && (slot >> 4) < max_blocks) ? block_table[(size_t)b * max_blocks + (slot >> 4)] : -1;
        if (chunks > 0) __syncthreads();
        // (a position flagged by the draft step, a slot beyond the block table, a missing page: nothing is written)
        if (p < 0 || p >= max_pos || page < 0 || page >= n_blocks) continue;
        int in_page = slot & 15;
        int half = h >> 1;
        const float* cs = rope_cs + (size_t)p * half * 2;
        const float* src = qkv + (size_t)row * nqkv;
        auto val = [&](int e) -> float { return chunks > 0 ? row_buf[e] : src[e]; };
        // q heads
        for (int i = threadIdx.x; i < hq * half; i += NORM_THREADS) {
            int head = i / half, j = i % half;
            float c = cs[2 * j], s = cs[2 * j + 1];
            float a = val(head * h + j), bb = val(head * h + j + half);
            T* dst = q_out + (size_t)row * hq * h + head * h;
            put(dst + j, a * c - bb * s);
            put(dst + j + half, bb * c + a * s);
        }
        // k heads -> cache [page][kv head][16][h]
        const int koff = hq * h;
        for (int i = threadIdx.x; i < hkv * half; i += NORM_THREADS) {
            int head = i / half, j = i % half;
            float c = cs[2 * j], s = cs[2 * j + 1];
            float a = val(koff + head * h + j), bb = val(koff + head * h + j + half);
            T* dst = kc + layer_off + (((size_t)page * hkv + head) * 16 + in_page) * h;
            put(dst + j, a * c - bb * s);
            put(dst + j + half, bb * c + a * s);
        }
        // v heads -> cache [page][kv head][h][16]
        const int voff = koff + hkv * h;
        for (int i = threadIdx.x; i < hkv * h; i += NORM_THREADS) {
            int head = i / h, j = i % h;
            put(vc + layer_off + (((size_t)page * hkv + head) * h + j) * 16 + in_page, val(voff + head * h + j));
        }
    }
}

// One workgroup of 16 wavefronts per row; 16-byte loads where the row is aligned.  Ties resolve to the lowest id
// at every level, so the result is the first maximum whatever the reduction shape.
__global__ __launch_bounds__(1024) void argmax_kernel(const float* __restrict__ logits, int32_t* __restrict__ out,
                                                       const int32_t* __restrict__ m_dev, int vocab) {
    __shared__ float sv[16];
    __shared__ int si[16];
    const int m = *m_dev;
    for (int row = blockIdx.x; row < m; row += gridDim.x) {
        if (row != (int)blockIdx.x) __syncthreads();  // the previous row's candidates have been read
        const float* l = logits + (size_t)row * vocab;
        float bv = -INFINITY;
        int bi = 0x7fffffff;
        auto take = [&](float v, int i) { if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; } };
        if ((vocab & 3) == 0) {
            const float4* l4 = reinterpret_cast<const float4*>(l);
            for (int i = threadIdx.x; i < vocab / 4; i += 1024) {
                float4 v = l4[i];
                take(v.x, 4 * i); take(v.y, 4 * i + 1); take(v.z, 4 * i + 2); take(v.w, 4 * i + 3);
            }
        } else {
            for (int i = threadIdx.x; i < vocab; i += 1024) take(l[i], i);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            float ov = __shfl_xor(bv, o);
            int oi = __shfl_xor(bi, o);
            take(ov, oi);
        }
        if ((threadIdx.x & 63) == 0) { sv[threadIdx.x >> 6] = bv; si[threadIdx.x >> 6] = bi; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int w = 1; w < 16; w++) take(sv[w], si[w]);
            out[row] = bi;
        }
    }
}

// Rows of one prefill call: sequence b contributes its next n_b = min(chunk, seq_len - 1 - kv_done) tokens (taken
// from its token log), sequences served in index order until max_rows rows are laid out.  One workgroup.
// len_plus1[b] = kv_done[b] + 1 before the call (the later kernels' "sequence length": cached positions + 1);
// kv_done advances by n_b.
__global__ __launch_bounds__(256) void prefill_rows_kernel(
    const int32_t* __restrict__ seq_len, int32_t* __restrict__ kv_done, const int32_t* __restrict__ tokens,
    int tokens_stride, int batch, int chunk, int max_rows, int max_pos, const int32_t* __restrict__ block_table,
    int max_blocks, int32_t* __restrict__ row_off,
    int32_t* __restrict__ tok, int32_t* __restrict__ pos, int32_t* __restrict__ parent, int32_t* __restrict__ row2seq,
    int32_t* __restrict__ len_plus1, uint32_t* __restrict__ err) {
    __shared__ int sw[4];
    __shared__ int carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int b0 = 0; b0 < batch; b0 += 256) {
        const int b = b0 + threadIdx.x;
        int want = 0, done = 0;
        if (b < batch) {
            done = max(kv_done[b], 0);
            want = max(0, min(chunk, seq_len[b] - 1 - done));
            if (done + want > max_pos) {        // rotary table too short: nothing of this sequence is laid out
                atomicOr(err, (uint32_t)HS_DEV_POSITION_OVERFLOW);
                want = 0;
            } else if (want > 0 && (done + want > max_blocks * 16 ||
                                    block_table[(size_t)b * max_blocks + ((done + want - 1) >> 4)] < 0)) {
                // the sequence outgrows its block table (or the pages the caller gave it): likewise
                atomicOr(err, (uint32_t)HS_DEV_BLOCK_TABLE_OVERFLOW);
                want = 0;
            }
        }
        int incl = want;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            int t = __shfl_up(incl, o);
            if (lane >= o) incl += t;
        }
        if (lane == 63) sw[wave] = incl;
        __syncthreads();
        int before = carry_s;
        for (int w2 = 0; w2 < wave; w2++) before += sw[w2];
        const int start = before + incl - want;
        if (b < batch) {
            const int s0 = min(start, max_rows);
            const int n = max(0, min(want, max_rows - s0));
            row_off[b] = s0;
            len_plus1[b] = done + 1;
            kv_done[b] = done + n;
        }
        __syncthreads();
        if (threadIdx.x == 255) carry_s = before + incl;
        __syncthreads();
    }
    if (threadIdx.x == 0) row_off[batch] = min(carry_s, max_rows);
    __syncthreads();   // this workgroup's row_off / len_plus1 writes are visible to all its threads
    for (int b = 0; b < batch; b++) {
        const int s0 = row_off[b], n = row_off[b + 1] - s0, done = len_plus1[b] - 1;
        for (int i = threadIdx.x; i < n; i += 256) {
            tok[s0 + i] = tokens[(size_t)b * tokens_stride + done + i];
            pos[s0 + i] = done + i;
            parent[s0 + i] = i - 1;
            row2seq[s0 + i] = b;
        }
    }
}

}  // namespace

void hs_launch_prefill_rows(const hs_ctx* ctx, const hs_seq_state* seq, int32_t* kv_done, int chunk, hs_step* step,
                            int32_t* len_plus1, hipStream_t st) {
    hipLaunchKernelGGL(prefill_rows_kernel, dim3(1), dim3(256), 0, st, seq->seq_len, kv_done, seq->tokens,
                       seq->tokens_stride, seq->batch, chunk, ctx->lim.max_rows, ctx->lim.max_pos, seq->block_table,
                       ctx->lim.max_blocks_per_seq, step->row_off,
                       step->tok, step->pos, step->parent, step->row2seq, len_plus1,
                       reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.err));
}

void hs_launch_embed(const hs_ctx* ctx, const hs_step* step, int batch, float* x, hipStream_t st) {
    hipLaunchKernelGGL(embed_kernel, dim3(hs_row_grid(ctx, 256)), dim3(256), 0, st, ctx->embed, step->tok,
                       step->row_off + batch, x, ctx->desc.d_model, ctx->desc.vocab);
}

void hs_launch_rmsnorm(const hs_ctx* ctx, float* x, const float* w, void* out, const int32_t* m_dev,
                       int pending_chunks, hipStream_t st) {
    const float* part = reinterpret_cast<const float*>(ctx->ws + ctx->lay.gemm_part);
    const size_t stride = (size_t)ctx->lim.max_rows * ctx->desc.d_model;
    if (hs_fp32_activations(ctx))
        hipLaunchKernelGGL(rmsnorm_kernel<float>, dim3(hs_row_grid(ctx, NORM_THREADS)), dim3(NORM_THREADS), 0, st, x, w, (float*)out,
                           m_dev, ctx->desc.d_model, ctx->desc.rms_eps, part, pending_chunks, stride);
    else
        hipLaunchKernelGGL(rmsnorm_kernel<bf16_t>, dim3(hs_row_grid(ctx, NORM_THREADS)), dim3(NORM_THREADS), 0, st, x, w,
                           (bf16_t*)out, m_dev, ctx->desc.d_model, ctx->desc.rms_eps, part, pending_chunks, stride);
}

void hs_launch_rope_kv(const hs_ctx* ctx, int layer, const hs_kv_cache* cache, const hs_seq_state* seq,
                       const hs_step* step, const float* qkv, void* q, int pending_chunks, hipStream_t st) {
    const hs_model_desc& d = ctx->desc;
    size_t layer_off = (size_t)layer * cache->n_blocks * d.n_kv_heads * 16 * d.head_dim;
    const float* part = reinterpret_cast<const float*>(ctx->ws + ctx->lay.gemm_part);
    const size_t nqkv = (size_t)(d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim;
    const size_t lds = pending_chunks > 0 ? nqkv * 4 : 0;
#define HS_ROPE_ARGS(T)                                                                                          \
    qkv, ctx->rope_cs, step->pos, step->row2seq, step->row_off, seq->seq_len, seq->block_table,                  \
        ctx->lim.max_blocks_per_seq, seq->batch, (T*)q, (T*)cache->k, (T*)cache->v, layer_off, d.n_q_heads,      \
        d.n_kv_heads, d.head_dim, ctx->lim.max_pos, cache->n_blocks, part, pending_chunks,                       \
        (size_t)ctx->lim.max_rows * nqkv
    if (hs_fp32_activations(ctx))
        hipLaunchKernelGGL(rope_kv_kernel<float>, dim3(hs_row_grid(ctx, NORM_THREADS)), dim3(NORM_THREADS), lds, st,
                           HS_ROPE_ARGS(float));
    else
        hipLaunchKernelGGL(rope_kv_kernel<bf16_t>, dim3(hs_row_grid(ctx, NORM_THREADS)), dim3(NORM_THREADS), lds, st,
                           HS_ROPE_ARGS(bf16_t));
#undef HS_ROPE_ARGS
}

void hs_launch_argmax(const hs_ctx* ctx, const float* logits, int32_t* argmax, const int32_t* m_dev,
                      hipStream_t st) {
    hipLaunchKernelGGL(argmax_kernel, dim3(hs_row_grid(ctx, 1024)), dim3(1024), 0, st, logits, argmax, m_dev,
                       ctx->desc.vocab);
}
