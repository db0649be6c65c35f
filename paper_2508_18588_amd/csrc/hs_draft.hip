// History-drafted speculation, draft side (Sec. 5.2 and 5.4 of the paper): every in-flight response looks for
// the longest suffix of its committed tokens (at most `window`, at least `m_min` tokens) inside its previous-epoch
// response and takes the tokens that follow as its draft.
//
// Kernel 1 (scan): one workgroup per (history segment, candidate).  The segment plus a `window`-token halo is
// staged in LDS with coalesced loads; every thread then tests end positions p against the pattern held in
// registers/LDS, and the best (match length, leftmost p) is reduced with wavefront shuffles as one packed 64-bit
// key.  Kernel 2 (build): one thread per sequence reduces the segment winners, applies the draft-length policy,
// merges the candidates' chains into a token tree, and a workgroup-wide prefix sum over node counts yields the
// ragged row offsets the verify step consumes.
#include <mutex>

#include "hs_internal.h"

namespace {

__device__ inline unsigned long long shfl_xor_u64(unsigned long long v, int o) {
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = __shfl_xor(lo, o);
    hi = __shfl_xor(hi, o);
    return ((unsigned long long)hi << 32) | lo;
}

// key = (match length << 32) | ~p : larger is better, ties -> smaller p
__global__ __launch_bounds__(256) void draft_scan_kernel(const int32_t* __restrict__ hist,
                                                          const int32_t* __restrict__ hist_off, int n_cand,
                                                          const int32_t* __restrict__ tail,
                                                          const int32_t* __restrict__ tail_len,
                                                          const int32_t* __restrict__ budget_left, int w_max,
                                                          int window, int m_min, int max_segs,
                                                          unsigned long long* __restrict__ best) {
    __shared__ __attribute__((aligned(16))) int32_t sh[HS_DRAFT_SEG + 32 + 8];
    __shared__ int32_t pat[32];
    __shared__ unsigned long long red[4];
    const int seg = blockIdx.x, bc = blockIdx.y, b = bc / n_cand;
    const int tid = threadIdx.x;
    unsigned long long* dst = best + (size_t)bc * max_segs + seg;
    const int off = hist_off[bc];
    const int lh = hist_off[bc + 1] - off;
    const int p_lo = seg * HS_DRAFT_SEG + 1;                   // end positions handled here: [p_lo, p_hi]
    const int p_hi = min((seg + 1) * HS_DRAFT_SEG, lh - 1);
    int n_pat = min(min(tail_len[b], window), w_max);
    if (budget_left[b] <= 0 || p_lo > p_hi || n_pat < m_min || n_pat <= 0) {
        if (tid == 0) *dst = 0ull;
        return;
    }
    // pattern, newest token first: pat[i] = i-th token from the end
    if (tid < n_pat) pat[tid] = tail[(size_t)b * w_max + (w_max - 1 - tid)];
    // tokens hist[base .. p_hi) are needed: base = p_lo - window (clamped).  They are staged with 16-byte loads
    // from the 16-byte boundary at or below the first token: LDS entry `shift` + i holds hist[off + base + i].
    // (Tokens in front of that boundary belong to this or the previous history: in bounds, never compared.  A
    // vector that would reach past this history's end is loaded token by token.)
    const int base = max(0, p_lo - window);
    const int count = p_hi - base;
    const int g0 = off + base, a0 = g0 & ~3, shift = g0 - a0, g_end = off + lh;
    const int4* src4 = reinterpret_cast<const int4*>(hist + a0);
    for (int v = tid; 4 * v < shift + count; v += 256) {
        if (a0 + 4 * v + 4 <= g_end) {
            *reinterpret_cast<int4*>(&sh[4 * v]) = src4[v];
        } else {
            for (int e = 0; e < 4; e++)
                if (a0 + 4 * v + e < g_end) sh[4 * v + e] = hist[a0 + 4 * v + e];
        }
    }
    __syncthreads();
    unsigned long long k = 0ull;
    const int32_t* shb = sh + shift - base;          // shb[i] = hist[off + i]
    for (int p = p_lo + tid; p <= p_hi; p += 256) {
        int lim = min(n_pat, p);
        int m = 0;
        while (m < lim && shb[p - 1 - m] == pat[m]) m++;
        if (m >= m_min) {
            unsigned long long cand = ((unsigned long long)m << 32) | (0xFFFFFFFFu - (unsigned)p);
            if (cand > k) k = cand;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned long long other = shfl_xor_u64(k, o);
        if (other > k) k = other;
    }
    if ((tid & 63) == 0) red[tid >> 6] = k;
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; w++) if (red[w] > k) k = red[w];
        *dst = k;
    }
}

__device__ inline int block_excl_scan_256(int v, int* total, int* sw) {
    // wavefront inclusive scan by shuffles, then the 4 wavefront totals
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        int t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    __syncthreads();
    if (lane == 63) sw[wave] = inc;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; w++) before += sw[w];
    *total = sw[0] + sw[1] + sw[2] + sw[3];
    return before + inc - v;
}

__global__ __launch_bounds__(256) void draft_build_kernel(
    const int32_t* __restrict__ hist, const int32_t* __restrict__ hist_off, int n_cand, int batch,
    const unsigned long long* __restrict__ best, int max_segs, const int32_t* __restrict__ seq_len,
    const int32_t* __restrict__ tail, int w_max, const int32_t* __restrict__ k_state,
    const int32_t* __restrict__ budget_left, hs_policy pol, int max_blocks, int max_pos, int max_rows,
    int32_t* __restrict__ draft_start, int32_t* __restrict__ match_len, int32_t* __restrict__ draft_len,
    int32_t* __restrict__ row_off, int32_t* __restrict__ tok, int32_t* __restrict__ pos,
    int32_t* __restrict__ parent, uint64_t* __restrict__ anc_mask, int32_t* __restrict__ row2seq,
    uint32_t* __restrict__ err, int group_n, const int32_t* __restrict__ draft_src, int32_t* __restrict__ gate,
    const unsigned long long* __restrict__ counters) {
    // group_n > 0: the draft of sequence b was chosen by the group walk (response draft_src[b] of its group_n
    // responses, start draft_start[b], length draft_len[b]); this kernel then only lays out the rows (n_cand == 1)
    __shared__ int sw[4];
    __shared__ int carry_s;
    __shared__ int live_s, spec_on_s;
    if (threadIdx.x == 0) { carry_s = 0; live_s = 0; spec_on_s = 1; }
    __syncthreads();
    if (gate) {
        // Throughput-aware speculation control (Sec. 5.4, last paragraph): one decision per step for the whole batch.
        // The monitor takes the previous step's drafted / accepted tokens from the counters hs_kv_commit keeps.
        int live = 0;
        for (int b = threadIdx.x; b < batch; b += 256) live += budget_left[b] > 0;
        if (live) atomicAdd(&live_s, live);
        __syncthreads();
        if (threadIdx.x == 0) {
            const uint32_t dt = (uint32_t)counters[1], at = (uint32_t)counters[2];
            const uint32_t d = dt - (uint32_t)gate[5], a = at - (uint32_t)gate[6];
            gate[5] = (int32_t)dt;
            gate[6] = (int32_t)at;
            gate[0] = gate[0] - (gate[0] >> 3) + (int32_t)d;
            gate[1] = gate[1] - (gate[1] >> 3) + (int32_t)a;
            const int steps_off = (gate[7] > 0 && gate[3] == 0) ? gate[2] + 1 : 0;
            int bucket = 16;
            if (gate[0] > 0) {
                const long long q = (long long)gate[1] * 16 / gate[0];
                bucket = q > 16 ? 16 : (int)q;
            }
            const int on = live_s <= gate[HS_GATE_TABLE + bucket] || (gate[4] > 0 && steps_off >= gate[4]);
            gate[2] = steps_off;
            gate[3] = on;
            gate[7] += 1;
            spec_on_s = on;
        }
        __syncthreads();
    }
    const bool spec_on = spec_on_s != 0;
    for (int b0 = 0; b0 < batch; b0 += 256) {
        const int b = b0 + threadIdx.x;
        int nn = 0, L = 0;
        int pstart[2] = {-1, -1}, klen[2] = {0, 0}, hoff[2] = {0, 0};
        int shared = 0;
        if (b < batch && budget_left[b] > 0) {
            L = seq_len[b] - 1;
            if (group_n > 0) {
                const int g = draft_src[b];
                pstart[0] = draft_start[b];
                klen[0] = (g >= 0 && spec_on) ? draft_len[b] : 0;
                hoff[0] = g >= 0 ? hist_off[b * group_n + g] + pstart[0] : 0;
            }
            for (int c = 0; c < n_cand && group_n == 0; c++) {
                const int bc = b * n_cand + c;
                const int off = hist_off[bc], lh = hist_off[bc + 1] - off;
                unsigned long long k = 0ull;
                const int nseg = (lh - 1 + HS_DRAFT_SEG - 1) / HS_DRAFT_SEG;
                for (int s = 0; s < nseg && s < max_segs; s++) {
                    unsigned long long v = best[(size_t)bc * max_segs + s];
                    if (v > k) k = v;
                }
                int m = (int)(k >> 32);
                int p = m > 0 ? (int)(0xFFFFFFFFu - (unsigned)(k & 0xFFFFFFFFull)) : -1;
                int kk = 0;
                if (m > 0) {
                    if (pol.k_mode == HS_K_FIXED) kk = pol.k_fixed;
                    else if (pol.k_mode == HS_K_MATCHLEN) kk = m < 1 ? 1 : m;
                    else kk = k_state[b];
                    kk = min(kk, pol.k_max);
                    kk = min(kk, lh - p);
                    kk = min(kk, budget_left[b] - 1);
                    kk = max(kk, 0);
                    if (!spec_on) kk = 0;
                }
                pstart[c] = p; klen[c] = kk; hoff[c] = off + (p < 0 ? 0 : p);
                draft_start[bc] = p;
                match_len[bc] = m;
            }
            if (n_cand == 2) {
                int lim = min(klen[0], klen[1]);
                while (shared < lim && hist[hoff[0] + shared] == hist[hoff[1] + shared]) shared++;
            }
            nn = 1 + klen[0] + (n_cand == 2 ? klen[1] - shared : 0);
            // capacity: every node needs a cache slot L + i and a rotary position below max_pos
            int cap_tokens = max_blocks * 16;
            if (L < 0 || L + 1 > cap_tokens || L + 1 > max_pos) {
                atomicOr(err, L + 1 > max_pos ? HS_DEV_POSITION_OVERFLOW : HS_DEV_BLOCK_TABLE_OVERFLOW);
                nn = 0; klen[0] = klen[1] = 0; shared = 0;
            } else if (L + nn > cap_tokens || L + 1 + max(klen[0], klen[1]) > max_pos) {
                atomicOr(err, L + nn > cap_tokens ? HS_DEV_BLOCK_TABLE_OVERFLOW : HS_DEV_POSITION_OVERFLOW);
                nn = 1; klen[0] = klen[1] = 0; shared = 0;
            }
            for (int c = 0; c < n_cand; c++) draft_len[b * n_cand + c] = klen[c];
        } else if (b < batch) {
            for (int c = 0; c < n_cand; c++) {
                draft_start[b * n_cand + c] = -1;
                match_len[b * n_cand + c] = 0;
                draft_len[b * n_cand + c] = 0;
            }
        }
        int total;
        int excl = block_excl_scan_256(nn, &total, sw);
        int carry = carry_s;
        int r0 = carry + excl;
        if (b < batch) {
            if (r0 + nn > max_rows) { atomicOr(err, HS_DEV_ROW_OVERFLOW); nn = 0; }
            row_off[b] = r0;
            if (nn > 0) {
                tok[r0] = tail[(size_t)b * w_max + (w_max - 1)];
                pos[r0] = L; parent[r0] = -1; anc_mask[r0] = 1ull; row2seq[r0] = b;
                // candidate 0: nodes 1..k0, a chain
                for (int i = 1; i <= klen[0]; i++) {
                    tok[r0 + i] = hist[hoff[0] + i - 1];
                    pos[r0 + i] = L + i; parent[r0 + i] = i - 1;
                    anc_mask[r0 + i] = (2ull << i) - 1ull; row2seq[r0 + i] = b;
                }
                // candidate 1: nodes after the shared prefix, hanging off node `shared`
                if (n_cand == 2) {
                    uint64_t m = (2ull << shared) - 1ull;
                    int par = shared;
                    for (int i = shared + 1; i <= klen[1]; i++) {
                        int node = klen[0] + (i - shared);
                        m |= 1ull << node;
                        tok[r0 + node] = hist[hoff[1] + i - 1];
                        pos[r0 + node] = L + i; parent[r0 + node] = par;
                        anc_mask[r0 + node] = m; row2seq[r0 + node] = b;
                        par = node;
                    }
                }
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) carry_s = carry + total;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        int total = carry_s;
        if (total > max_rows) {
            // Only with limits that hs_create does not admit (max_rows < max_batch * nodes): the first sequence that
            // does not fit and every one after it get no rows, consistently for the kernels that read row_off.
            int cut = -1;
            for (int b = 0; b < batch; b++) {
                const int end = b + 1 < batch ? row_off[b + 1] : total;
                if (cut < 0 && end > max_rows) cut = row_off[b];
                if (cut >= 0 && b + 1 < batch) row_off[b + 1] = cut;
            }
            total = cut;
        }
        row_off[batch] = total;
    }
}


// ---- reward-aware draft over all responses of the prompt's last rollout (Sec. 5.3) ----
//
// The paper keeps one suffix tree per prompt over the responses of its last rollout, with a priority on every node
// (the summed rewards of the responses whose text runs through it), and follows the highest-priority child where
// the continuations of the matched pattern branch.  On the GPU the tree is never built: the scan kernel above finds
// the longest match in every response segment; this kernel, one workgroup per sequence, collects the occurrences of
// that longest pattern in (response, position) order and lets them vote, draft token by draft token, for their
// next token with their response's reward (ties: more votes, then the smaller token id).  Occurrences that voted
// for another token, or ran out of text, drop out.  The draft is the text after the first surviving occurrence.
constexpr int HS_OCC_MAX = 1024;  // occurrences kept per sequence (in order); part of the rule, see the header

__device__ inline unsigned long long block_max_u64(unsigned long long v, unsigned long long* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        unsigned long long other = shfl_xor_u64(v, o);
        if (other > v) v = other;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    unsigned long long r = red[0];
    for (int w = 1; w < 4; w++) if (red[w] > r) r = red[w];
    return r;
}

__global__ __launch_bounds__(256) void draft_group_walk_kernel(
    const int32_t* __restrict__ hist, const int32_t* __restrict__ hist_off, const int32_t* __restrict__ reward,
    int n_resp, const unsigned long long* __restrict__ best, int max_segs, const int32_t* __restrict__ tail,
    const int32_t* __restrict__ tail_len, int w_max, const int32_t* __restrict__ k_state,
    const int32_t* __restrict__ budget_left, hs_policy pol, int32_t* __restrict__ draft_start,
    int32_t* __restrict__ match_len, int32_t* __restrict__ draft_len, int32_t* __restrict__ draft_src) {
    __shared__ int32_t pat[32];
    __shared__ int32_t occ_off[HS_OCC_MAX];   // offset in `hist` of the token that follows the occurrence
    __shared__ int32_t occ_end[HS_OCC_MAX];   // end offset of its response
    __shared__ int32_t occ_rew[HS_OCC_MAX];
    __shared__ int32_t occ_tok[HS_OCC_MAX];   // this step's vote; -2 = live but out of text, -1 = dropped out
    __shared__ unsigned long long red[4];
    __shared__ int sw[4];
    __shared__ int n_occ_s;
    const int b = blockIdx.x, tid = threadIdx.x;
    auto none = [&]() {
        if (tid == 0) { draft_start[b] = -1; match_len[b] = 0; draft_len[b] = 0; draft_src[b] = -1; }
    };
    const int n_pat = min(min(tail_len[b], pol.window), w_max);
    if (budget_left[b] <= 0 || n_pat < pol.m_min || n_pat <= 0) { none(); return; }
    if (tid < n_pat) pat[tid] = tail[(size_t)b * w_max + (w_max - 1 - tid)];
    if (tid == 0) n_occ_s = 0;
    // longest match over all segments of all responses
    unsigned long long k = 0ull;
    for (int i = tid; i < n_resp * max_segs; i += 256) {
        const int g = i / max_segs, sgm = i % max_segs;
        const int lh = hist_off[b * n_resp + g + 1] - hist_off[b * n_resp + g];
        if (sgm * HS_DRAFT_SEG + 1 <= lh - 1) {
            unsigned long long v = best[(size_t)(b * n_resp + g) * max_segs + sgm] >> 32;
            if (v > k) k = v;
        }
    }
    const int m_star = (int)block_max_u64(k, red);   // (contains the barriers that publish pat and n_occ_s)
    if (m_star < pol.m_min || m_star <= 0) { none(); return; }
    // occurrences, in (response, position) order: only segments whose best match reaches m_star hold any
    for (int g = 0; g < n_resp; g++) {
        const int off = hist_off[b * n_resp + g], lh = hist_off[b * n_resp + g + 1] - off;
        const int rew = reward[b * n_resp + g];
        for (int sgm = 0; sgm < max_segs && sgm * HS_DRAFT_SEG + 1 <= lh - 1; sgm++) {
            if ((int)(best[(size_t)(b * n_resp + g) * max_segs + sgm] >> 32) < m_star) continue;   // uniform
            const int p_hi = min((sgm + 1) * HS_DRAFT_SEG, lh - 1);
            for (int p0 = sgm * HS_DRAFT_SEG + 1; p0 <= p_hi; p0 += 256) {
                const int p = p0 + tid;
                int hit = 0;
                if (p <= p_hi && p >= m_star) {
                    int m = 0;
                    while (m < m_star && hist[off + p - 1 - m] == pat[m]) m++;
                    hit = m == m_star;
                }
                int total;
                const int before = block_excl_scan_256(hit, &total, sw);
                const int base = n_occ_s;
                if (hit && base + before < HS_OCC_MAX) {
                    occ_off[base + before] = off + p;
                    occ_end[base + before] = off + lh;
                    occ_rew[base + before] = rew;
                }
                __syncthreads();
                if (tid == 0) n_occ_s = min(HS_OCC_MAX, base + total);
                __syncthreads();
                if (n_occ_s >= HS_OCC_MAX) break;
            }
            if (n_occ_s >= HS_OCC_MAX) break;
        }
        if (n_occ_s >= HS_OCC_MAX) break;
    }
    const int n_occ = n_occ_s;
    // draft length the policy asks for
    int kk = pol.k_mode == HS_K_FIXED ? pol.k_fixed : (pol.k_mode == HS_K_MATCHLEN ? m_star : k_state[b]);
    kk = max(0, min(min(kk, pol.k_max), budget_left[b] - 1));
    // the walk
    for (int i = tid; i < n_occ; i += 256) occ_tok[i] = 0;   // live
    __syncthreads();
    int len = 0;
    for (int j = 0; j < kk; j++) {
        for (int i = tid; i < n_occ; i += 256)
            if (occ_tok[i] != -1) occ_tok[i] = (occ_off[i] + j < occ_end[i]) ? hist[occ_off[i] + j] : -2;
        __syncthreads();
        // every live occurrence prices its own token: (reward sum, votes) packed, larger is better
        unsigned long long key = 0ull;
        for (int i = tid; i < n_occ; i += 256) {
            const int t = occ_tok[i];
            if (t < 0) continue;
            unsigned long long sum = 0ull;
            unsigned votes = 0u;
            for (int q = 0; q < n_occ; q++)
                if (occ_tok[q] == t) { sum += (unsigned long long)occ_rew[q]; votes++; }
            const unsigned long long v = ((sum << 11) | votes) + 1ull;   // + 1: a live vote always beats "none"
            if (v > key) key = v;
        }
        const unsigned long long top = block_max_u64(key, red);
        if (top == 0ull) break;   // nobody has a token left: the live occurrences stay live (marked -2)
        // among the tokens with the top price, the smallest id
        unsigned long long cand = 0ull;
        for (int i = tid; i < n_occ; i += 256) {
            const int t = occ_tok[i];
            if (t < 0) continue;
            unsigned long long sum = 0ull;
            unsigned votes = 0u;
            for (int q = 0; q < n_occ; q++)
                if (occ_tok[q] == t) { sum += (unsigned long long)occ_rew[q]; votes++; }
            if (((sum << 11) | votes) + 1ull == top) {
                const unsigned long long v = 0xFFFFFFFFull - (unsigned)t;
                if (v > cand) cand = v;
            }
        }
        const int chosen = (int)(0xFFFFFFFFull - block_max_u64(cand, red));
        for (int i = tid; i < n_occ; i += 256)
            if (occ_tok[i] != chosen) occ_tok[i] = -1;
        len++;
        __syncthreads();
    }
    // first surviving occurrence (every occurrence is live if nothing was drafted; one that only ran out of text
    // at the step that ended the walk is still live)
    unsigned long long firstk = 0ull;
    for (int i = tid; i < n_occ; i += 256)
        if (len == 0 || occ_tok[i] != -1) { firstk = 0xFFFFFFFFull - (unsigned)i; break; }
    const unsigned long long fk = block_max_u64(firstk, red);
    if (fk == 0ull || n_occ <= 0) { none(); return; }   // cannot happen: the chosen token came from a live occurrence
    const int first = (int)(0xFFFFFFFFull - fk);
    if (tid == 0) {
        // its response: the one that ends where the occurrence's response ends
        int g = 0;
        while (g + 1 < n_resp && hist_off[b * n_resp + g + 1] != occ_end[first]) g++;
        draft_src[b] = g;
        draft_start[b] = occ_off[first] - hist_off[b * n_resp + g];
        match_len[b] = m_star;
        draft_len[b] = len;
    }
}

}  // namespace

namespace {

void launch_draft(const hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step,
                  unsigned long long* best, uint32_t* err, hipStream_t st) {
    const hs_policy& p = args->policy;
    dim3 grid(ctx->max_segs, seq->batch * args->n_cand);
    hipLaunchKernelGGL(draft_scan_kernel, grid, dim3(256), 0, st, args->hist, args->hist_off, args->n_cand,
                       seq->tail, seq->tail_len, seq->budget_left, ctx->lim.w_max, p.window, p.m_min,
                       ctx->max_segs, best);
    hipLaunchKernelGGL(draft_build_kernel, dim3(1), dim3(256), 0, st, args->hist, args->hist_off, args->n_cand,
                       seq->batch, best, ctx->max_segs, seq->seq_len, seq->tail, ctx->lim.w_max, seq->k_state,
                       seq->budget_left, p, ctx->lim.max_blocks_per_seq, ctx->lim.max_pos, ctx->lim.max_rows,
                       step->draft_start, step->match_len, step->draft_len, step->row_off, step->tok, step->pos,
                       step->parent, step->anc_mask, step->row2seq, err, 0, nullptr, seq->gate,
                       (const unsigned long long*)seq->counters);
}

}  // namespace

void hs_launch_draft(const hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step,
                     hipStream_t st) {
    launch_draft(ctx, args, seq, step, reinterpret_cast<unsigned long long*>(ctx->ws + ctx->lay.draft_best),
                 reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.err), st);
}

// ---- hs_draft for callers that cannot allocate: the segment winners (and, with no workspace bound, the error word)
// live in a static device array instead of the caller's workspace.
namespace {

// [0, HS_DRAFT_STATIC_ENTRIES): segment winners, 8 bytes each; then one 8-byte slot whose first word is the error word.
static __device__ __align__(256) unsigned long long scratch[HS_DRAFT_STATIC_ENTRIES + 1];

constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
unsigned long long* scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each device (each has its own copy)

// The address of this device's copy of the array, looked up once per device with that device current.
unsigned long long* scratch_on_current_device(hipError_t* why) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= MAX_DEVICES) { *why = e != hipSuccess ? e : hipErrorInvalidDevice; return nullptr; }
    std::lock_guard<std::mutex> lock(scratch_mutex);
    if (!scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { *why = e != hipSuccess ? e : hipErrorInvalidSymbol; return nullptr; }
        scratch_ptr[dev] = static_cast<unsigned long long*>(p);
    }
    return scratch_ptr[dev];
}

}  // namespace

uint32_t* hs_draft_static_error_word(hipError_t* why) {
    unsigned long long* base = scratch_on_current_device(why);
    return base ? reinterpret_cast<uint32_t*>(base + HS_DRAFT_STATIC_ENTRIES) : nullptr;
}

bool hs_launch_draft_static(const hs_ctx* ctx, const hs_draft_args* args, const hs_seq_state* seq, hs_step* step,
                            hipStream_t st, hipError_t* why) {
    unsigned long long* base = scratch_on_current_device(why);
    if (!base) return false;
    uint32_t* err = ctx->ws ? reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.err)
                            : reinterpret_cast<uint32_t*>(base + HS_DRAFT_STATIC_ENTRIES);
    // every winner slot the build kernel reads is written by the scan kernel of the same call: nothing to clear
    launch_draft(ctx, args, seq, step, base, err, st);
    return true;
}

void hs_launch_draft_group(const hs_ctx* ctx, const hs_group_draft_args* args, const hs_seq_state* seq,
                           hs_step* step, hipStream_t st) {
    unsigned long long* best = reinterpret_cast<unsigned long long*>(ctx->ws + ctx->lay.draft_best);
    uint32_t* err = reinterpret_cast<uint32_t*>(ctx->ws + ctx->lay.err);
    const hs_policy& p = args->policy;
    dim3 grid(ctx->max_segs, seq->batch * args->n_resp);
    hipLaunchKernelGGL(draft_scan_kernel, grid, dim3(256), 0, st, args->hist, args->hist_off, args->n_resp,
                       seq->tail, seq->tail_len, seq->budget_left, ctx->lim.w_max, p.window, p.m_min,
                       ctx->max_segs, best);
    hipLaunchKernelGGL(draft_group_walk_kernel, dim3(seq->batch), dim3(256), 0, st, args->hist, args->hist_off,
                       args->reward, args->n_resp, best, ctx->max_segs, seq->tail, seq->tail_len, ctx->lim.w_max,
                       seq->k_state, seq->budget_left, p, step->draft_start, step->match_len, step->draft_len,
                       step->draft_src);
    hipLaunchKernelGGL(draft_build_kernel, dim3(1), dim3(256), 0, st, args->hist, args->hist_off, 1, seq->batch,
                       best, ctx->max_segs, seq->seq_len, seq->tail, ctx->lim.w_max, seq->k_state, seq->budget_left,
                       p, ctx->lim.max_blocks_per_seq, ctx->lim.max_pos, ctx->lim.max_rows, step->draft_start,
                       step->match_len, step->draft_len, step->row_off, step->tok, step->pos, step->parent,
                       step->anc_mask, step->row2seq, err, args->n_resp, step->draft_src, seq->gate,
                       (const unsigned long long*)seq->counters);
}
