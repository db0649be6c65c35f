// Ragged multi-query paged attention for the verify step.
//
// For sequence b with L cached positions and nn draft-tree nodes, every node's query (all G query heads that
// share one KV head) attends to cache positions [0, L) and to the slots L + i of the nodes i that are its
// ancestors or itself.  The KV cache is read once per (sequence, KV head) and step, shared by all G * nn query
// rows -- which is why verifying a whole draft costs about one KV traversal (Sec. 2.2 of the paper).
//
// Work decomposition: one workgroup per (partition of `part_keys` absolute positions, KV head, sequence).  K and
// V pages are staged through LDS in tiles of 32 keys (two 16-token pages); the next tile is prefetched into
// registers while the matrix cores work on the current one.  Query rows are split over the 4 wavefronts in tiles
// of 32.  Scores are computed transposed, S^T = K . Q^T (v_mfma_f32_32x32x16_bf16, A = K tile from LDS, B = Q^T
// held in registers), so that each lane owns one query row: the online-softmax statistics are per-lane scalars,
// and the exponentiated scores are already in the register layout the second product O^T = V^T . P^T needs as
// its B operand.  V is stored in the cache with the token index fastest so V^T tiles are plain 8-byte LDS reads.
//
// Partitions are keyed to absolute positions and merged in index order, masked keys contribute exact zeros, so a
// row's result is bit-identical whether it is verified next to other draft rows or decoded alone.
#include "hs_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

template <int HD, int RTW>
__global__ __launch_bounds__(256) void attn_verify_mfma(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc, size_t layer_off,
    const int32_t* __restrict__ seq_len, const int32_t* __restrict__ block_table, int max_blocks, int n_blocks,
    const int32_t* __restrict__ row_off, const uint64_t* __restrict__ anc_mask, float* __restrict__ part_o,
    float* __restrict__ part_ml, int max_parts, int part_keys, int hq, int hkv, float scale_log2) {
    constexpr int KS = HD + 8;        // sK row stride (bf16)
    constexpr int VS = 20;            // sV row stride (bf16): 16 tokens + pad, 40 bytes
    constexpr int NCK = HD / 64;      // 16-byte K chunks per thread and tile
    constexpr int NCV = HD / 64;      // 16-byte V chunks per thread and tile
    constexpr int NKS = HD / 16;      // k-steps of the score product
    constexpr int NDT = HD / 32;      // 32-wide tiles of the head dimension
    __shared__ __attribute__((aligned(16))) bf16_t sK[32 * KS];
    __shared__ __attribute__((aligned(16))) bf16_t sV[2 * HD * VS];

    const int part = blockIdx.x, j = blockIdx.y, b = blockIdx.z;
    const int r0 = row_off[b];
    const int nn = row_off[b + 1] - r0;
    if (nn <= 0) return;
    const int L = seq_len[b] - 1;
    const int total = L + nn;
    const int k_begin = part * part_keys;
    if (k_begin >= total) return;
    const int k_end = min(total, k_begin + part_keys);
    const int G = hq / hkv;
    const int R = nn * G;
    const int nrt = (R + 31) >> 5;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int32_t* bt = block_table + (size_t)b * max_blocks;

    // ---- per-row-tile state
    bf16x8 qf[RTW][NKS];
    f32x16 o[RTW][NDT];
    float m_run[RTW], l_run[RTW];
    uint64_t anc[RTW];
    bool rt_on[RTW];
#pragma unroll
    for (int t = 0; t < RTW; t++) {
        int rt = wave + 4 * t;
        rt_on[t] = rt < nrt;
        int rho = rt * 32 + l32;
        bool ok = rt_on[t] && rho < R;
        int node = ok ? rho / G : 0;
        int g = ok ? rho - node * G : 0;
        anc[t] = ok ? anc_mask[r0 + node] : 0ull;
        const bf16_t* qp = q + ((size_t)(r0 + node) * hq + j * G + g) * HD;
#pragma unroll
        for (int ks = 0; ks < NKS; ks++) {
            if (ok) {
                qf[t][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16 + half * 8);
            } else {
#pragma unroll
                for (int e = 0; e < 8; e++) qf[t][ks][e] = (__bf16)0.f;
            }
        }
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
#pragma unroll
            for (int e = 0; e < 16; e++) o[t][dt][e] = 0.f;
        m_run[t] = -INFINITY;
        l_run[t] = 0.f;
    }

    // ---- global -> register prefetch of one 32-key tile
    uint4 rk[NCK], rv[NCV];
    auto fetch = [&](int kbase) {
        // two pages of this tile
        int pg[2];
#pragma unroll
        for (int kk = 0; kk < 2; kk++) {
            int p0 = kbase + 16 * kk;
            int pidx = p0 >> 4;
            int page = (p0 < total && pidx < max_blocks) ? bt[pidx] : -1;
            pg[kk] = (page >= 0 && page < n_blocks) ? page : -1;
        }
#pragma unroll
        for (int i = 0; i < NCK; i++) {
            int c = tid + 256 * i;
            int key = c / (HD / 8), c16 = c % (HD / 8);
            int page = pg[key >> 4];
            rk[i] = make_uint4(0, 0, 0, 0);
            if (page >= 0)
                rk[i] = *reinterpret_cast<const uint4*>(kc + layer_off + (((size_t)page * hkv + j) * 16 + (key & 15)) * HD + c16 * 8);
        }
#pragma unroll
        for (int i = 0; i < NCV; i++) {
            int c = tid + 256 * i;
            int kk = c / (HD * 2), rem = c % (HD * 2);
            int page = pg[kk];
            rv[i] = make_uint4(0, 0, 0, 0);
            if (page >= 0)
                rv[i] = *reinterpret_cast<const uint4*>(vc + layer_off + ((size_t)page * hkv + j) * HD * 16 + rem * 8);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int i = 0; i < NCK; i++) {
            int c = tid + 256 * i;
            int key = c / (HD / 8), c16 = c % (HD / 8);
            *reinterpret_cast<uint4*>(&sK[key * KS + c16 * 8]) = rk[i];
        }
#pragma unroll
        for (int i = 0; i < NCV; i++) {
            int c = tid + 256 * i;
            int kk = c / (HD * 2), rem = c % (HD * 2);
            int dim = rem >> 1, hf = rem & 1;
            uint2* dst = reinterpret_cast<uint2*>(&sV[(kk * HD + dim) * VS + hf * 8]);
            dst[0] = make_uint2(rv[i].x, rv[i].y);
            dst[1] = make_uint2(rv[i].z, rv[i].w);
        }
    };

    fetch(k_begin);
    for (int kbase = k_begin; kbase < k_end; kbase += 32) {
        __syncthreads();  // previous tile fully consumed
        stage();
        __syncthreads();
        if (kbase + 32 < k_end) fetch(kbase + 32);

        const bool need_mask = kbase + 32 > L;
#pragma unroll
        for (int t = 0; t < RTW; t++) {
            if (!rt_on[t]) continue;
            f32x16 s;
#pragma unroll
            for (int e = 0; e < 16; e++) s[e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ks++) {
                bf16x8 ka = *reinterpret_cast<const bf16x8*>(&sK[l32 * KS + ks * 16 + half * 8]);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[t][ks], s, 0, 0, 0);
            }
            // element e: key kbase + 8*(e/4) + 4*half + e%4, query row = this lane's
            float tmax = -INFINITY;
#pragma unroll
            for (int e = 0; e < 16; e++) {
                float v = s[e] * scale_log2;
                if (need_mask) {
                    int kp = kbase + 8 * (e >> 2) + 4 * half + (e & 3);
                    bool vis = kp < L || (kp < total && ((anc[t] >> (kp - L)) & 1ull));
                    v = vis ? v : -INFINITY;
                }
                s[e] = v;
                tmax = fmaxf(tmax, v);
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            float m_new = fmaxf(m_run[t], tmax);
            float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
            float alpha = fast_exp2(m_run[t] - m_safe);
            float psum = 0.f;
            bf16x8 pb[2];
#pragma unroll
            for (int e = 0; e < 16; e++) {
                float p = fast_exp2(s[e] - m_safe);
                psum += p;
                pb[e >> 3][e & 7] = (__bf16)p;
            }
            psum += __shfl_xor(psum, 32);
            l_run[t] = l_run[t] * alpha + psum;
            m_run[t] = m_new;
#pragma unroll
            for (int dt = 0; dt < NDT; dt++)
#pragma unroll
                for (int e = 0; e < 16; e++) o[t][dt][e] *= alpha;
#pragma unroll
            for (int kk = 0; kk < 2; kk++)
#pragma unroll
                for (int dt = 0; dt < NDT; dt++) {
                    const bf16_t* vrow = &sV[(kk * HD + dt * 32 + l32) * VS];
                    uint2 lo = *reinterpret_cast<const uint2*>(vrow + 4 * half);
                    uint2 hi = *reinterpret_cast<const uint2*>(vrow + 8 + 4 * half);
                    union { uint4 u; bf16x8 v; } va;
                    va.u = make_uint4(lo.x, lo.y, hi.x, hi.y);
                    o[t][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.v, pb[kk], o[t][dt], 0, 0, 0);
                }
        }
    }

    // ---- partial results: unnormalised O, running max (log2 domain) and sum
#pragma unroll
    for (int t = 0; t < RTW; t++) {
        int rt = wave + 4 * t;
        int rho = rt * 32 + l32;
        if (!rt_on[t] || rho >= R) continue;
        int node = rho / G, g = rho - node * G;
        size_t prow = ((size_t)(r0 + node) * hq + j * G + g) * max_parts + part;
        float* po = part_o + prow * HD;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
#pragma unroll
            for (int g4 = 0; g4 < 4; g4++) {
                float4 v = make_float4(o[t][dt][4 * g4], o[t][dt][4 * g4 + 1], o[t][dt][4 * g4 + 2], o[t][dt][4 * g4 + 3]);
                *reinterpret_cast<float4*>(po + dt * 32 + 8 * g4 + 4 * half) = v;
            }
        if (half == 0) {
            part_ml[prow * 2] = m_run[t];
            part_ml[prow * 2 + 1] = l_run[t];
        }
    }
}

// Combine the partitions of one (row, query head) in partition order.
template <int HD>
__global__ __launch_bounds__(64) void attn_merge(const float* __restrict__ part_o, const float* __restrict__ part_ml,
                                                  const int32_t* __restrict__ row2seq, const int32_t* __restrict__ row_off,
                                                  const int32_t* __restrict__ seq_len, int batch, int max_parts,
                                                  int part_keys, int hq, bf16_t* __restrict__ out) {
    int row = blockIdx.x, head = blockIdx.y;
    if (row >= row_off[batch]) return;
    int b = row2seq[row];
    int total = seq_len[b] - 1 + (row_off[b + 1] - row_off[b]);
    int nparts = min(max_parts, (total + part_keys - 1) / part_keys);
    size_t prow = ((size_t)row * hq + head) * max_parts;
    float mg = -INFINITY;
    for (int p = 0; p < nparts; p++) mg = fmaxf(mg, part_ml[(prow + p) * 2]);
    float den = 0.f;
    for (int p = 0; p < nparts; p++) den += fast_exp2(part_ml[(prow + p) * 2] - mg) * part_ml[(prow + p) * 2 + 1];
    for (int d = threadIdx.x; d < HD; d += 64) {
        float acc = 0.f;
        for (int p = 0; p < nparts; p++)
            acc += fast_exp2(part_ml[(prow + p) * 2] - mg) * part_o[(prow + p) * HD + d];
        out[((size_t)row * hq + head) * HD + d] = f32_to_bf16(acc / den);
    }
}

// Plain kernel for debugging: one wavefront per (row, query head), keys visited one by one.
__global__ __launch_bounds__(64) void attn_verify_plain(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc, size_t layer_off,
    const int32_t* __restrict__ seq_len, const int32_t* __restrict__ block_table, int max_blocks, int n_blocks,
    const int32_t* __restrict__ row_off, const int32_t* __restrict__ row2seq, const uint64_t* __restrict__ anc_mask,
    int batch, int hq, int hkv, int hd, float scale, bf16_t* __restrict__ out) {
    int row = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
    if (row >= row_off[batch]) return;
    int b = row2seq[row];
    int L = seq_len[b] - 1, nn = row_off[b + 1] - row_off[b];
    int total = L + nn, j = head / (hq / hkv);
    uint64_t anc = anc_mask[row];
    const bf16_t* qp = q + ((size_t)row * hq + head) * hd;
    float q0 = lane < hd ? bf16_to_f32(qp[lane]) : 0.f;
    float q1 = lane + 64 < hd ? bf16_to_f32(qp[lane + 64]) : 0.f;
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    for (int kp = 0; kp < total; kp++) {
        bool vis = kp < L || ((anc >> (kp - L)) & 1ull);
        if (!vis) continue;
        if ((kp >> 4) >= max_blocks) break;
        int page = block_table[(size_t)b * max_blocks + (kp >> 4)];
        if (page < 0 || page >= n_blocks) break;
        int ip = kp & 15;
        const bf16_t* kr = kc + layer_off + (((size_t)page * hkv + j) * 16 + ip) * hd;
        float dot = 0.f;
        if (lane < hd) dot += q0 * bf16_to_f32(kr[lane]);
        if (lane + 64 < hd) dot += q1 * bf16_to_f32(kr[lane + 64]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) dot += __shfl_xor(dot, o);
        float s = dot * scale;
        float mn = fmaxf(m, s);
        float a = __expf(m - mn), p = __expf(s - mn);
        l = l * a + p;
        const bf16_t* vr = vc + layer_off + ((size_t)page * hkv + j) * hd * 16 + ip;
        float v0 = lane < hd ? bf16_to_f32(vr[(size_t)lane * 16]) : 0.f;
        float v1 = lane + 64 < hd ? bf16_to_f32(vr[(size_t)(lane + 64) * 16]) : 0.f;
        o0 = o0 * a + p * v0;
        o1 = o1 * a + p * v1;
        m = mn;
    }
    bf16_t* op = out + ((size_t)row * hq + head) * hd;
    if (lane < hd) op[lane] = f32_to_bf16(o0 / l);
    if (lane + 64 < hd) op[lane + 64] = f32_to_bf16(o1 / l);
}

template <int HD, int RTW>
void launch_mfma(const hs_ctx* ctx, size_t layer_off, const hs_kv_cache* cache, const hs_seq_state* seq,
                 const hs_step* step, const bf16_t* q, bf16_t* out, hipStream_t st) {
    const hs_model_desc& d = ctx->desc;
    float* part_o = reinterpret_cast<float*>(ctx->ws + ctx->lay.part_o);
    float* part_ml = reinterpret_cast<float*>(ctx->ws + ctx->lay.part_ml);
    float scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
    dim3 grid(ctx->max_parts, d.n_kv_heads, seq->batch);
    hipLaunchKernelGGL((attn_verify_mfma<HD, RTW>), grid, dim3(256), 0, st, q, (const bf16_t*)cache->k,
                       (const bf16_t*)cache->v, layer_off, seq->seq_len, seq->block_table,
                       ctx->lim.max_blocks_per_seq, cache->n_blocks, step->row_off, step->anc_mask, part_o, part_ml,
                       ctx->max_parts, ctx->att_part, d.n_q_heads, d.n_kv_heads, scale_log2);
}

}  // namespace

void hs_launch_attention(const hs_ctx* ctx, int layer, const hs_kv_cache* cache, const hs_seq_state* seq,
                         const hs_step* step, const bf16_t* q, bf16_t* out, hipStream_t st) {
    const hs_model_desc& d = ctx->desc;
    size_t layer_off = (size_t)layer * cache->n_blocks * d.n_kv_heads * 16 * d.head_dim;
    if (ctx->flags & HS_FLAG_REFERENCE_KERNELS) {
        hipLaunchKernelGGL(attn_verify_plain, dim3(ctx->lim.max_rows, d.n_q_heads), dim3(64), 0, st, q,
                           (const bf16_t*)cache->k, (const bf16_t*)cache->v, layer_off, seq->seq_len,
                           seq->block_table, ctx->lim.max_blocks_per_seq, cache->n_blocks, step->row_off,
                           step->row2seq, step->anc_mask, seq->batch, d.n_q_heads, d.n_kv_heads, d.head_dim,
                           1.f / sqrtf((float)d.head_dim), out);
        return;
    }
    int G = d.n_q_heads / d.n_kv_heads;
    int r_max = G * (1 + ctx->lim.c_max * ctx->lim.k_max);
    bool two = r_max > 128;
    if (d.head_dim == 128) {
        if (two) launch_mfma<128, 2>(ctx, layer_off, cache, seq, step, q, out, st);
        else launch_mfma<128, 1>(ctx, layer_off, cache, seq, step, q, out, st);
    } else {
        if (two) launch_mfma<64, 2>(ctx, layer_off, cache, seq, step, q, out, st);
        else launch_mfma<64, 1>(ctx, layer_off, cache, seq, step, q, out, st);
    }
}

void hs_launch_attention_merge(const hs_ctx* ctx, const hs_seq_state* seq, const hs_step* step, bf16_t* out,
                               hipStream_t st) {
    if (ctx->flags & HS_FLAG_REFERENCE_KERNELS) return;  // the plain kernel writes the final output itself
    const hs_model_desc& d = ctx->desc;
    float* part_o = reinterpret_cast<float*>(ctx->ws + ctx->lay.part_o);
    float* part_ml = reinterpret_cast<float*>(ctx->ws + ctx->lay.part_ml);
    dim3 grid(ctx->lim.max_rows, d.n_q_heads);
    if (d.head_dim == 128)
        hipLaunchKernelGGL((attn_merge<128>), grid, dim3(64), 0, st, part_o, part_ml, step->row2seq, step->row_off,
                           seq->seq_len, seq->batch, ctx->max_parts, ctx->att_part, d.n_q_heads, out);
    else
        hipLaunchKernelGGL((attn_merge<64>), grid, dim3(64), 0, st, part_o, part_ml, step->row2seq, step->row_off,
                           seq->seq_len, seq->batch, ctx->max_parts, ctx->att_part, d.n_q_heads, out);
}
