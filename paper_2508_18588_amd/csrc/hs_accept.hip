// Acceptance and KV commit (Sec. 2.2 of the paper: the verified draft tokens that are valid are kept, and the
// output distribution is preserved; Sec. 5.4: the per-response speculation window update).
//
// Greedy acceptance walks the draft tree from the root, following the child whose token equals the parent row's
// argmax.  Rejection acceptance is speculative sampling with a point-mass draft distribution: child j of a node
// is accepted with probability p(tok_j) under softmax(logits / T) with the tokens of earlier rejected siblings
// removed; the walk ends with one inverse-CDF sample in token-id order.  Uniforms come from Philox-4x32-10
// (Salmon et al., SC'11) keyed by the seed, with counter (position, draw kind, sequence id): the stream does not
// depend on the batch slot or on how many steps it took to reach the position.
#include "hs_internal.h"

namespace {

__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0, uint32_t k1,
                                     uint32_t out[4]) {
#pragma unroll
    for (int r = 0; r < 10; r++) {
        uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

__device__ inline double uniform01(uint64_t seed, uint64_t seq_id, uint32_t position, uint32_t kind) {
    uint32_t o[4];
    philox4x32_10(position, kind, (uint32_t)seq_id, (uint32_t)(seq_id >> 32), (uint32_t)seed, (uint32_t)(seed >> 32), o);
    return (double)(o[0] >> 8) * (1.0 / 16777216.0);
}

// Greedy walk of one sequence's tree (one thread): follow the child whose token is the current node's argmax.
__device__ inline void accept_greedy_walk(int b, int r0, int nn, const int32_t* __restrict__ tok,
                                          const int32_t* __restrict__ parent, const int32_t* __restrict__ argmax,
                                          int k_stride, int32_t* __restrict__ accept_len, int32_t* __restrict__ n_out,
                                          int32_t* __restrict__ out_tok, int32_t* __restrict__ path_row) {
    int cur = 0, a = 0;
    path_row[(size_t)b * k_stride] = 0;
    for (;;) {
        int g = argmax[r0 + cur];
        out_tok[(size_t)b * k_stride + a] = g;
        int next = -1;
        for (int i = 1; i < nn; i++)
            if (parent[r0 + i] == cur && tok[r0 + i] == g) { next = i; break; }
        if (next < 0 || a + 1 >= k_stride) break;
        cur = next;
        a++;
        path_row[(size_t)b * k_stride + a] = cur;
    }
    accept_len[b] = a;
    n_out[b] = a + 1;
}

__device__ inline double block_sum_f64(double v, double* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        int lo = __shfl_xor(__double2loint(v), o), hi = __shfl_xor(__double2hiint(v), o);
        v += __hiloint2double(hi, lo);
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

__device__ inline float block_max_f32(float v, float* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
}

// Rejection sampling of one sequence by its workgroup (nn > 0).  Probabilities are evaluated in fp64 from the fp32
// logits.
__device__ inline void accept_rejection_seq(
    int b, int r0, int nn, int vocab, const int32_t* __restrict__ tok,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ pos, const float* __restrict__ logits,
    const uint64_t* __restrict__ seq_id, double inv_temp, uint64_t seed, int k_stride,
    int32_t* __restrict__ accept_len, int32_t* __restrict__ n_out, int32_t* __restrict__ out_tok,
    int32_t* __restrict__ path_row) {
    __shared__ float redf[4];
    __shared__ double redd[4];
    __shared__ double chunk_sum[256];
    __shared__ int s_next, s_nrej, s_rej[8], s_chunk, s_pick;
    __shared__ double s_before, s_target;
    const int tid = threadIdx.x;
    const uint64_t sid = seq_id[b];
    int cur = 0, a = 0;
    if (tid == 0) path_row[(size_t)b * k_stride] = 0;
    for (;;) {
        const float* lg = logits + (size_t)(r0 + cur) * vocab;
        float mx = -INFINITY;
        for (int i = tid; i < vocab; i += 256) mx = fmaxf(mx, lg[i]);
        mx = block_max_f32(mx, redf);
        double z = 0.0;
        for (int i = tid; i < vocab; i += 256) z += exp(((double)lg[i] - (double)mx) * inv_temp);
        z = block_sum_f64(z, redd);
        const uint32_t position = (uint32_t)(pos[r0 + cur] + 1);
        if (tid == 0) {
            int next = -1, tried = 0, nrej = 0;
            double zr = z;
            for (int i = 1; i < nn && next < 0; i++) {
                if (parent[r0 + i] != cur) continue;
                int t = tok[r0 + i];
                double w = exp(((double)lg[t] - (double)mx) * inv_temp);
                for (int r = 0; r < nrej; r++) if (s_rej[r] == t) w = 0.0;
                double u = uniform01(seed, sid, position, (uint32_t)tried);
                if (u < w / zr) next = i;
                else if (nrej < 8) { s_rej[nrej++] = t; zr -= w; }
                tried++;
            }
            s_next = next;
            s_nrej = nrej;
        }
        __syncthreads();
        const int next = s_next;
        if (next >= 0 && a + 1 < k_stride) {
            if (tid == 0) {
                out_tok[(size_t)b * k_stride + a] = tok[r0 + next];
                path_row[(size_t)b * k_stride + a + 1] = next;
            }
            cur = next;
            a++;
            __syncthreads();
            continue;
        }
        // final sample from the remaining distribution: contiguous chunk per thread, chunk sums, then the
        // owning thread walks its chunk in token-id order
        const int nrej = s_nrej;
        const int per = (vocab + 255) / 256;
        const int lo = tid * per, hi = min(vocab, lo + per);
        double cs = 0.0;
        for (int i = lo; i < hi; i++) {
            double w = exp(((double)lg[i] - (double)mx) * inv_temp);
            for (int r = 0; r < nrej; r++) if (s_rej[r] == i) w = 0.0;
            cs += w;
        }
        chunk_sum[tid] = cs;
        __syncthreads();
        if (tid == 0) {
            double zt = 0.0;
            for (int c = 0; c < 256; c++) zt += chunk_sum[c];
            double u = uniform01(seed, sid, position, 7u);
            double target = u * zt, cum = 0.0;
            int chunk = -1;
            for (int c = 0; c < 256; c++) {
                if (chunk_sum[c] > 0.0 && cum + chunk_sum[c] >= target) { chunk = c; break; }
                cum += chunk_sum[c];
            }
            s_chunk = chunk; s_before = cum; s_target = target; s_pick = -1;
        }
        __syncthreads();
        if (s_chunk >= 0 && tid == s_chunk) {
            double cum = s_before;
            int pick = -1, last_nz = -1;
            for (int i = lo; i < hi; i++) {
                double w = exp(((double)lg[i] - (double)mx) * inv_temp);
                for (int r = 0; r < nrej; r++) if (s_rej[r] == i) w = 0.0;
                if (w > 0.0) last_nz = i;
                cum += w;
                if (w > 0.0 && cum >= s_target) { pick = i; break; }
            }
            s_pick = pick >= 0 ? pick : last_nz;
        }
        __syncthreads();
        if (tid == 0) {
            int pick = s_pick;
            if (pick < 0) {  // rounding left the target beyond every chunk: last token with weight
                for (int i = vocab - 1; i >= 0; i--) {
                    bool rej = false;
                    for (int r = 0; r < nrej; r++) if (s_rej[r] == i) rej = true;
                    if (!rej) { pick = i; break; }
                }
            }
            out_tok[(size_t)b * k_stride + a] = pick;
            accept_len[b] = a;
            n_out[b] = a + 1;
        }
        break;
    }
}

// Commit of one sequence by its workgroup: relocate accepted tree nodes' K/V to consecutive slots, then advance the
// state.  CT = cache element type (bf16 bits, or float in the fp32-activation mode).
template <typename CT>
__device__ inline void commit_seq(
    int b, int n_layers, int hkv, int hd, int n_blocks, CT* __restrict__ kc, CT* __restrict__ vc,
    const int32_t* __restrict__ block_table, int max_blocks, int32_t* __restrict__ seq_len,
    int32_t* __restrict__ tail, int32_t* __restrict__ tail_len, int w_max, int32_t* __restrict__ k_state,
    int32_t* __restrict__ budget_left, int32_t* __restrict__ tokens, int tokens_stride,
    unsigned long long* __restrict__ counters, const int32_t* __restrict__ row_off,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ accept_len, const int32_t* __restrict__ n_out,
    const int32_t* __restrict__ out_tok, const int32_t* __restrict__ path_row, int k_stride, const hs_policy& pol) {
    const int tid = threadIdx.x;
    const int r0 = row_off[b], nn = row_off[b + 1] - r0;
    const int no = n_out[b];
    if (nn <= 0 || no <= 0) return;
    const int a = accept_len[b];
    const int n_old = seq_len[b];
    const int L = n_old - 1;
    const int32_t* bt = block_table + (size_t)b * max_blocks;
    // accepted node path_row[j] (j = 1..a) must end up in slot L + j
    const size_t per_layer = (size_t)n_blocks * hkv * 16 * hd;
    for (int jn = 1; jn <= a; jn++) {
        int node = path_row[(size_t)b * k_stride + jn];
        if (node == jn) continue;
        int s_slot = L + node, d_slot = L + jn;
        int sp = bt[s_slot >> 4], dp = bt[d_slot >> 4];
        if (sp < 0 || sp >= n_blocks || dp < 0 || dp >= n_blocks) continue;
        int si = s_slot & 15, di = d_slot & 15;
        int per = hkv * hd;
        for (int e = tid; e < n_layers * per; e += 256) {
            int layer = e / per, r = e % per, head = r / hd, d = r % hd;
            size_t lo = (size_t)layer * per_layer;
            kc[lo + (((size_t)dp * hkv + head) * 16 + di) * hd + d] = kc[lo + (((size_t)sp * hkv + head) * 16 + si) * hd + d];
            vc[lo + (((size_t)dp * hkv + head) * hd + d) * 16 + di] = vc[lo + (((size_t)sp * hkv + head) * hd + d) * 16 + si];
        }
    }
    __syncthreads();
    if (tid != 0) return;
    // window rule: every drafted token on the path accepted <=> the last accepted node is a leaf
    if (pol.k_mode == HS_K_AIMD && nn > 1) {
        int last = path_row[(size_t)b * k_stride + a];
        bool leaf = true;
        for (int i = 1; i < nn; i++) if (parent[r0 + i] == last) { leaf = false; break; }
        int k = k_state[b];
        if (leaf && a > 0) k = min(k + pol.aimd_inc, pol.aimd_cap);
        else k = pol.aimd_reset;
        k_state[b] = k;
    }
    // pattern tail: the last w_max tokens of (old valid tail ++ emitted tokens)
    int tl = tail_len[b];
    int32_t* tb = tail + (size_t)b * w_max;
    int new_len = min(w_max, tl + no);
    int32_t tmp[32];
    for (int i = 0; i < new_len; i++) {
        int ci = tl + no - new_len + i;  // index in the concatenation
        tmp[i] = ci < tl ? tb[w_max - tl + ci] : out_tok[(size_t)b * k_stride + ci - tl];
    }
    for (int i = 0; i < new_len; i++) tb[w_max - new_len + i] = tmp[i];
    tail_len[b] = new_len;
    if (tokens) {
        for (int i = 0; i < no; i++)
            if (n_old + i < tokens_stride) tokens[(size_t)b * tokens_stride + n_old + i] = out_tok[(size_t)b * k_stride + i];
    }
    seq_len[b] = n_old + no;
    budget_left[b] -= no;
    if (counters) {
        atomicAdd(&counters[1], (unsigned long long)(nn - 1));
        atomicAdd(&counters[2], (unsigned long long)a);
        atomicAdd(&counters[3], (unsigned long long)no);
        atomicAdd(&counters[0], 1ull);
    }
}

// Acceptance and commit of one step in ONE launch, one workgroup per sequence (either half can be switched off: the
// two entry points that run them separately use the same kernel).
//   1. With `keys` (the LM head ran with its row-maximum epilogue and no logits exist): every row's argmax = the
//      largest of its n_keys per-column-group keys, one wavefront per row; written to argmax[].
//   2. Acceptance: greedy walk (thread 0) or rejection sampling (the workgroup).
//   3. Commit.
struct accept_commit_args {
    int batch, vocab, k_stride, mode, do_accept, do_commit;
    const int32_t *row_off, *tok, *parent, *pos;
    const float* logits;
    const unsigned long long* keys;
    int n_keys;
    int32_t* argmax;
    const uint64_t* seq_id;
    double inv_temp;
    uint64_t seed;
    int32_t *accept_len, *n_out, *out_tok, *path_row;
    // commit
    int n_layers, hkv, hd, n_blocks, max_blocks, w_max, tokens_stride;
    void *kc, *vc;
    const int32_t* block_table;
    int32_t *seq_len, *tail, *tail_len, *k_state, *budget_left, *tokens;
    unsigned long long* counters;
    hs_policy pol;
};

template <typename CT>
__global__ __launch_bounds__(256) void accept_commit_kernel(accept_commit_args p) {
    const int b = blockIdx.x, tid = threadIdx.x;
    const int r0 = p.row_off[b], nn = p.row_off[b + 1] - r0;
    if (p.do_accept) {
        if (nn <= 0) {
            if (tid == 0) { p.accept_len[b] = 0; p.n_out[b] = 0; }
        } else {
            if (p.keys) {
                const int lane = tid & 63, wave = tid >> 6;
                for (int r = wave; r < nn; r += 4) {
                    const unsigned long long* kr = p.keys + (size_t)(r0 + r) * p.n_keys;
                    unsigned long long best = 0ull;
                    for (int g = lane; g < p.n_keys; g += 64) {
                        const unsigned long long k = kr[g];
                        if (k > best) best = k;
                    }
#pragma unroll
                    for (int o = 32; o > 0; o >>= 1) {
                        const unsigned lo = __shfl_xor((unsigned)best, o), hi = __shfl_xor((unsigned)(best >> 32), o);
                        const unsigned long long other = ((unsigned long long)hi << 32) | lo;
                        if (other > best) best = other;
                    }
                    if (lane == 0) p.argmax[r0 + r] = (int32_t)(0xFFFFFFFFu - (unsigned)best);
                }
                __syncthreads();   // the walk reads argmax[] written by the other wavefronts
            }
            if (p.mode == HS_ACCEPT_GREEDY) {
                if (tid == 0)
                    accept_greedy_walk(b, r0, nn, p.tok, p.parent, p.argmax, p.k_stride, p.accept_len, p.n_out,
                                       p.out_tok, p.path_row);
            } else {
                accept_rejection_seq(b, r0, nn, p.vocab, p.tok, p.parent, p.pos, p.logits, p.seq_id, p.inv_temp,
                                     p.seed, p.k_stride, p.accept_len, p.n_out, p.out_tok, p.path_row);
            }
        }
        __syncthreads();           // the commit reads what thread 0 wrote
    }
    if (p.do_commit)
        commit_seq<CT>(b, p.n_layers, p.hkv, p.hd, p.n_blocks, (CT*)p.kc, (CT*)p.vc, p.block_table, p.max_blocks,
                       p.seq_len, p.tail, p.tail_len, p.w_max, p.k_state, p.budget_left, p.tokens, p.tokens_stride,
                       p.counters, p.row_off, p.parent, p.accept_len, p.n_out, p.out_tok, p.path_row, p.k_stride,
                       p.pol);
}

// The generator on its own: counter i -> its four output words (for bit-exact comparison with another
// implementation on many counters).
__global__ __launch_bounds__(256) void philox_debug_kernel(const uint32_t* __restrict__ ctr, uint32_t k0, uint32_t k1,
                                                            uint32_t* __restrict__ out, int n) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    uint32_t o[4];
    philox4x32_10(ctr[4 * i], ctr[4 * i + 1], ctr[4 * i + 2], ctr[4 * i + 3], k0, k1, o);
    out[4 * i] = o[0]; out[4 * i + 1] = o[1]; out[4 * i + 2] = o[2]; out[4 * i + 3] = o[3];
}

}  // namespace

extern "C" hs_status hs_debug_philox(const uint32_t* ctr, uint64_t seed, uint32_t* out, int32_t n, hs_stream stream) {
    if (!ctr || !out || n < 0) return HS_ERR_INVALID_ARG;
    if (n == 0) return HS_OK;
    (void)hipGetLastError();
    hipLaunchKernelGGL(philox_debug_kernel, dim3((n + 255) / 256), dim3(256), 0, (hipStream_t)stream, ctr,
                       (uint32_t)seed, (uint32_t)(seed >> 32), out, n);
    return hipGetLastError() == hipSuccess ? HS_OK : HS_ERR_HIP;
}

void hs_launch_accept_commit(const hs_ctx* ctx, const hs_accept_args* args, const hs_kv_cache* cache,
                             const hs_seq_state* seq, const hs_step* step, const float* logits,
                             const unsigned long long* keys, int n_keys, const hs_policy* policy, hipStream_t st) {
    const hs_model_desc& d = ctx->desc;
    accept_commit_args p = {};
    p.batch = seq->batch;
    p.vocab = d.vocab;
    p.k_stride = ctx->lim.k_max + 1;
    p.do_accept = args != nullptr;
    p.do_commit = policy != nullptr;
    p.row_off = step->row_off; p.tok = step->tok; p.parent = step->parent; p.pos = step->pos;
    p.logits = logits;
    p.keys = keys;
    p.n_keys = n_keys;
    p.argmax = step->argmax;
    p.seq_id = seq->seq_id;
    if (args) {
        p.mode = args->mode;
        p.inv_temp = args->mode == HS_ACCEPT_REJECTION ? 1.0 / (double)args->temperature : 1.0;
        p.seed = args->seed;
    }
    p.accept_len = step->accept_len; p.n_out = step->n_out; p.out_tok = step->out_tok; p.path_row = step->path_row;
    if (policy) {
        p.n_layers = d.n_layers; p.hkv = d.n_kv_heads; p.hd = d.head_dim;
        p.n_blocks = cache->n_blocks; p.max_blocks = ctx->lim.max_blocks_per_seq;
        p.w_max = ctx->lim.w_max; p.tokens_stride = seq->tokens_stride;
        p.kc = cache->k; p.vc = cache->v;
        p.block_table = seq->block_table;
        p.seq_len = seq->seq_len; p.tail = seq->tail; p.tail_len = seq->tail_len; p.k_state = seq->k_state;
        p.budget_left = seq->budget_left; p.tokens = seq->tokens;
        p.counters = (unsigned long long*)seq->counters;
        p.pol = *policy;
    }
    if (hs_fp32_activations(ctx))
        hipLaunchKernelGGL(accept_commit_kernel<float>, dim3(seq->batch), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(accept_commit_kernel<bf16_t>, dim3(seq->batch), dim3(256), 0, st, p);
}
