/*
 * CPU oracle for history-drafted speculative decoding (HistoSpec hot path).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, written-from-the-
 * definition version of what the GPU library computes.  It shares no code,
 * header, table or helper with the HIP path and must never be called by it.
 * Only the test-suite, the smoke check and the benchmark's cpu_baseline leg
 * load it.
 *
 * Arithmetic: every floating-point quantity is fp64.  Weights arrive as bf16
 * bit patterns (uint16) and are widened exactly; the RoPE table arrives as
 * fp32 values and is widened exactly.  No blocking, fusion or reordering is
 * applied beyond what each definition states; OpenMP only splits independent
 * output rows of a matrix-vector product.
 *
 * What each function follows (paper = "History Rhymes", arXiv 2508.18588):
 *   orc_suffix_match*      Sec. 5.2 (last generated tokens searched in the
 *                          historical response, following tokens are the
 *                          draft) and Sec. 5.4 (pattern length 7 shrinking
 *                          to 3 when nothing matches).
 *   orc_reward_draft       Sec. 5.3: all responses of the prompt's last rollout
 *                          are indexed together; where the continuations of
 *                          the matched pattern branch, the branch with the
 *                          largest sum of rewards is followed.
 *   orc_trace_sim          Sec. 5.1 token-similarity study (3-token key).
 *   orc_k_policy, orc_aimd Sec. 5.4 (window starts at 2, +2 when every draft
 *                          token is accepted, cap 32, back to 2 on a reject).
 *   orc_gate_step,
 *   orc_gate_table         Sec. 5.4, last paragraph: the acceptance rate is
 *                          monitored and speculation is switched off while the
 *                          batch is larger than the largest batch at which it
 *                          still pays at that rate (a pre-profiled table).
 *   orc_plan_allocation    Sec. 6.2, the Tier-2 planning problem: workers per
 *                          ranking group such that the groups' finish times
 *                          rise linearly with the smallest gradient the cluster
 *                          can afford -- the exact optimum (the paper bisects
 *                          towards it).
 *   orc_seq_*              Sec. 2.2: the target model's forward pass (a
 *                          standard pre-norm decoder; shape from the
 *                          benchmark configurations).
 *   orc_accept_greedy,
 *   orc_accept_stochastic  Sec. 2.2: verification accepts the valid draft
 *                          tokens and preserves the output distribution; the
 *                          rule is standard speculative sampling with a
 *                          point-mass draft distribution.
 *   orc_philox4x32_10      Salmon et al., "Parallel random numbers: as easy
 *                          as 1, 2, 3" (SC'11), Philox-4x32 with 10 rounds.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------- Tier-2 planner (HistoPipe) */

/*
 * Sec. 6.2 states the planning problem: the ranking groups (ascending representative length, group i profiled as
 * tau[i * K + (k - min_wks)] = its time on k data-parallel workers, K = max_wks - min_wks + 1) shall finish on a
 * straight line, group i no later than t0 + i d, with t0 = max(time of group 0 on max_wks workers, training time),
 * every group on the fewest workers that meet its deadline, all groups together within the worker budget -- and the
 * gradient d as small as the budget allows.  The paper reaches that d by bisection down to a precision; the oracle
 * is the definition itself: the exact smallest feasible d.
 *
 * For a given d the workers a group needs can only change where its deadline crosses one of its profiled times, i.e.
 * at d = (tau(i, k) - t0) / i, and raising d never raises any group's need.  So the smallest feasible gradient is 0
 * or one of these finitely many values: they are listed, sorted, and tried in ascending order.
 *
 * need_at: workers needed at gradient d (filling alloc), -1 if some group misses its deadline on any worker count.
 */
static long need_at(const double* tau, int n_groups, int min_wks, int max_wks, double t0, double d, int32_t* alloc) {
    int K = max_wks - min_wks + 1;
    long total = 0;
    for (int i = 0; i < n_groups; i++) {
        int fewest = 0;
        while (fewest < K && tau[(size_t)i * K + fewest] > t0 + i * d) fewest++;
        if (fewest == K) return -1;
        alloc[i] = min_wks + fewest;
        total += alloc[i];
    }
    return total;
}

static int cmp_double(const void* a, const void* b) {
    double x = *(const double*)a, y = *(const double*)b;
    return (x > y) - (x < y);
}

/*
 * Gradients are looked for in [0, d_top], d_top = (time of the last group on min_wks workers - t0) / (N - 1), the
 * interval the paper searches (reading: a negative d_top counts as 0; one group has no gradient, d = 0).  Returns 0
 * if even d_top is not affordable with `wks` workers, else 1 with plan[N] and *d_out = the smallest feasible gradient.
 */
int orc_plan_allocation(const double* tau, int n_groups, int min_wks, int max_wks, int wks, double t_train,
                        int32_t* plan, double* d_out) {
    int K = max_wks - min_wks + 1;
    double t0 = tau[K - 1] > t_train ? tau[K - 1] : t_train;
    double d_top = n_groups > 1 ? (tau[(size_t)(n_groups - 1) * K] - t0) / (n_groups - 1) : 0.0;
    if (d_top < 0.0) d_top = 0.0;
    long need = need_at(tau, n_groups, min_wks, max_wks, t0, d_top, plan);
    if (need < 0 || need > wks) return 0;
    /* candidates: 0, and every crossing point inside the interval (with its upper neighbour in floating point, since
     * t0 + i * ((tau - t0) / i) can fall one rounding short of tau) */
    size_t cap = 2 * (size_t)n_groups * K + 2, n = 0;
    double* cand = (double*)malloc(sizeof(double) * cap);
    int32_t* trial = (int32_t*)malloc(sizeof(int32_t) * (size_t)n_groups);
    cand[n++] = 0.0;
    for (int i = 1; i < n_groups; i++)
        for (int k = 0; k < K; k++) {
            double c = (tau[(size_t)i * K + k] - t0) / i;
            if (c > 0.0 && c < d_top) { cand[n++] = c; cand[n++] = nextafter(c, INFINITY); }
        }
    qsort(cand, n, sizeof(double), cmp_double);
    *d_out = d_top;
    for (size_t j = 0; j < n; j++) {
        need = need_at(tau, n_groups, min_wks, max_wks, t0, cand[j], trial);
        if (need >= 0 && need <= wks) {
            memcpy(plan, trial, sizeof(int32_t) * (size_t)n_groups);
            *d_out = cand[j];
            break;
        }
    }
    free(cand); free(trial);
    return 1;
}

/* ------------------------------------------------- speculation on / off */

/*
 * Throughput-aware speculation control (Sec. 5.4, last paragraph).  The paper:
 * acceptance rates are monitored; pre-profiling gives, per acceptance rate, the
 * largest batch at which speculation still raises throughput; above it
 * speculation is switched off.  The rest is this build's reading, in integers
 * so that both sides agree exactly:
 *   - monitor: decayed sums D (drafted) and A (accepted) over the steps so
 *     far, each step X <- X - (X >> 3) + x (a memory of about eight steps);
 *   - rate bucket = 16 A / D rounded down, 0..16 (16 when nothing was drafted
 *     lately: no evidence against speculating);
 *   - speculation runs this step iff live <= table[bucket], or it has been
 *     off for probe_every steps in a row (one probing step refreshes the
 *     monitor; probe_every = 0: never probe).
 * gate: [0] D, [1] A, [2] steps since speculation last ran, [3] last decision,
 * [4] probe_every, [5] / [6] drafted / accepted totals seen so far (mod 2^32),
 * [7] decisions made, [8..24] table.  Returns the decision (1 = speculate).
 */
int orc_gate_step(int32_t* gate, int live, uint32_t drafted_total, uint32_t accepted_total) {
    uint32_t d = drafted_total - (uint32_t)gate[5], a = accepted_total - (uint32_t)gate[6];
    gate[5] = (int32_t)drafted_total;
    gate[6] = (int32_t)accepted_total;
    gate[0] = gate[0] - (gate[0] >> 3) + (int32_t)d;
    gate[1] = gate[1] - (gate[1] >> 3) + (int32_t)a;
    int steps_off = (gate[7] > 0 && gate[3] == 0) ? gate[2] + 1 : 0;
    int bucket = 16;
    if (gate[0] > 0) {
        long long q = (long long)gate[1] * 16 / gate[0];
        bucket = q > 16 ? 16 : (int)q;
    }
    int on = live <= gate[8 + bucket] || (gate[4] > 0 && steps_off >= gate[4]);
    gate[2] = steps_off;
    gate[3] = on;
    gate[7] += 1;
    return on;
}

/* Step time at `rows` rows from profiled points (rows ascending): straight lines between neighbours, the outer
 * lines continued beyond the ends. */
static double profile_ms(const float* ms, const int32_t* rows, int n, double m) {
    int i = 0;
    while (i + 2 < n && m > rows[i + 1]) i++;
    double x0 = rows[i], x1 = rows[i + 1];
    return ms[i] + (ms[i + 1] - ms[i]) * (m - x0) / (x1 - x0);
}

/*
 * The pre-profiled table: for acceptance rate i/16 the largest batch b <= b_max
 * at which a step with drafts of k_bar tokens per sequence emits at least as
 * many tokens per second as a step without: (1 + rate k_bar) / t(b (1 + k_bar))
 * >= 1 / t(b); 0 if there is none.  t = the verify step time as a function of
 * the row count, from n >= 2 profiled points.
 */
void orc_gate_table(const float* ms, const int32_t* rows, int n, double k_bar, int b_max, int32_t* table) {
    for (int i = 0; i <= 16; i++) {
        double rate = i / 16.0;
        table[i] = 0;
        for (int b = 1; b <= b_max; b++) {
            double t0 = profile_ms(ms, rows, n, b), t1 = profile_ms(ms, rows, n, b * (1.0 + k_bar));
            if ((1.0 + rate * k_bar) * t0 >= t1) table[i] = b;
        }
    }
}

/* ------------------------------------------------------------------ draft */

/* Longest common suffix between hist[..p) and x[..n), capped at w. */
static int common_suffix(const int32_t* hist, int p, const int32_t* x, int n, int w) {
    int m = 0;
    while (m < w && m < p && m < n && hist[p - 1 - m] == x[n - 1 - m]) m++;
    return m;
}

/*
 * Plain definition of the draft position.  Over every end position p in
 * [1, lh-1] (at least one history token must follow p), m(p) is the length
 * of the longest common suffix of hist[..p) and x[..n), capped at w.  The
 * chosen p maximises m(p) subject to m(p) >= m_min; among equal m the
 * smallest p wins.  Returns 1 and sets *p_out, *m_out if a match exists, else
 * returns 0 with *p_out = -1 and *m_out = 0.
 */
int orc_suffix_match(const int32_t* hist, int lh, const int32_t* x, int n, int w, int m_min,
                     int* p_out, int* m_out) {
    int best_p = -1, best_m = 0;
    for (int p = 1; p <= lh - 1; p++) {
        int m = common_suffix(hist, p, x, n, w);
        if (m >= m_min && m > best_m) { best_m = m; best_p = p; }
    }
    *p_out = best_p;
    *m_out = best_m;
    return best_p >= 0;
}

/*
 * The same choice stated the way Sec. 5.4 words it: try a pattern of the w
 * last tokens; if it occurs nowhere, shorten it by one, down to m_min.  The
 * first (leftmost) occurrence of the longest pattern that occurs is taken.
 */
int orc_suffix_match_backoff(const int32_t* hist, int lh, const int32_t* x, int n, int w, int m_min,
                             int* p_out, int* m_out) {
    for (int len = (w < n ? w : n); len >= m_min && len >= 1; len--) {
        for (int p = len; p <= lh - 1; p++) {
            int ok = 1;
            for (int j = 0; j < len; j++)
                if (hist[p - len + j] != x[n - len + j]) { ok = 0; break; }
            if (ok) { *p_out = p; *m_out = len; return 1; }
        }
    }
    *p_out = -1;
    *m_out = 0;
    return 0;
}

/*
 * Reward-aware draft from ALL responses of the prompt's last rollout (Sec. 5.3).
 * The paper indexes the responses in one suffix tree per prompt: a node stands
 * for a token sequence, the leaves below it are the places where that sequence
 * occurs, a leaf's priority is the reward of the response it lies in, a node's
 * priority the sum over its leaves; where the continuations of the matched
 * pattern differ, the child with the highest priority is followed.  Written out
 * on the flat responses, without a tree:
 *
 *   1. m* = the longest common suffix (capped at w, at least m_min) between x
 *      and any place in any response that still has a token after it: end
 *      positions p in [1, len_g - 1] of response g.
 *   2. The occurrences are all (g, p) whose common suffix reaches m*, taken in
 *      the order of g, then p; at most occ_max of them are kept (a limit of the
 *      implementation, part of the definition so that both sides agree).
 *   3. Draft token j = 1, 2, ...: every live occurrence that has a token at
 *      p + j - 1 votes for that token with its response's reward.  The token
 *      with the largest reward sum is taken; equal sums: the one with more
 *      votes; still equal: the smaller token id.  Occurrences that voted
 *      otherwise, or ran out of tokens, drop out.  The walk ends after k tokens
 *      or when no live occurrence has a token left.
 *
 * hist = the G responses back to back, off[g] .. off[g+1] the extent of response
 * g; reward[g] >= 0.  Writes the draft tokens to out_tok (room for k), *m_out =
 * m* (0 if nothing matches), *n_occ = occurrences kept, *g_out / *p_out = the
 * first occurrence (in the order above) that is still live at the end: the
 * draft equals the tokens after it.  Returns the draft length.
 */
int orc_reward_draft(int G, const int32_t* hist, const int32_t* off, const int32_t* reward, const int32_t* x, int n,
                     int w, int m_min, int k, int occ_max, int32_t* out_tok, int* m_out, int* n_occ, int* g_out,
                     int* p_out) {
    *m_out = 0; *n_occ = 0; *g_out = -1; *p_out = -1;
    int m_star = 0;
    for (int g = 0; g < G; g++) {
        const int32_t* h = hist + off[g];
        int lh = off[g + 1] - off[g];
        for (int p = 1; p <= lh - 1; p++) {
            int m = common_suffix(h, p, x, n, w);
            if (m >= m_min && m > m_star) m_star = m;
        }
    }
    if (m_star == 0 || occ_max < 1) return 0;
    int* og = (int*)malloc(sizeof(int) * (size_t)occ_max);
    int* op = (int*)malloc(sizeof(int) * (size_t)occ_max);
    char* live = (char*)malloc((size_t)occ_max);
    int no = 0;
    for (int g = 0; g < G && no < occ_max; g++) {
        const int32_t* h = hist + off[g];
        int lh = off[g + 1] - off[g];
        for (int p = 1; p <= lh - 1 && no < occ_max; p++)
            if (common_suffix(h, p, x, n, w) >= m_star) { og[no] = g; op[no] = p; live[no] = 1; no++; }
    }
    int len = 0;
    for (int j = 0; j < k; j++) {
        /* the vote: for each candidate token (taken from the live occurrences), its reward sum and vote count */
        int have = 0, best_tok = 0, best_votes = 0;
        long long best_sum = 0;
        for (int i = 0; i < no; i++) {
            if (!live[i]) continue;
            int lh = off[og[i] + 1] - off[og[i]];
            if (op[i] + j >= lh) continue;
            int t = hist[off[og[i]] + op[i] + j];
            long long sum = 0;
            int votes = 0;
            for (int q = 0; q < no; q++) {
                if (!live[q]) continue;
                int lq = off[og[q] + 1] - off[og[q]];
                if (op[q] + j >= lq) continue;
                if (hist[off[og[q]] + op[q] + j] == t) { sum += reward[og[q]]; votes++; }
            }
            if (!have || sum > best_sum || (sum == best_sum && votes > best_votes) ||
                (sum == best_sum && votes == best_votes && t < best_tok)) {
                have = 1; best_tok = t; best_sum = sum; best_votes = votes;
            }
        }
        if (!have) break;
        for (int i = 0; i < no; i++) {
            if (!live[i]) continue;
            int lh = off[og[i] + 1] - off[og[i]];
            if (op[i] + j >= lh || hist[off[og[i]] + op[i] + j] != best_tok) live[i] = 0;
        }
        out_tok[len++] = best_tok;
    }
    *m_out = m_star;
    *n_occ = no;
    for (int i = 0; i < no; i++)
        if (live[i]) { *g_out = og[i]; *p_out = op[i]; break; }
    if (len == 0 && no > 0) { *g_out = og[0]; *p_out = op[0]; }
    free(og); free(op); free(live);
    return len;
}

/*
 * Offline similarity routine of Sec. 5.1: replay `cur` from its start; with
 * the last `key` replayed tokens as pattern, look for an exact occurrence in
 * `hist`; on a hit count the run of tokens that follow identically in both
 * (those are "accepted"), otherwise advance by one generated token.  Returns
 * the number of accepted tokens.  The leftmost occurrence with the longest
 * following run is not specified by the paper; this takes the occurrence
 * whose following run is longest (best case), first such on ties.
 */
int orc_trace_sim(const int32_t* cur, int n, const int32_t* hist, int lh, int key) {
    int accepted = 0;
    int i = 0; /* number of tokens replayed so far */
    while (i < n) {
        int best_run = 0;
        if (i >= key) {
            for (int p = key; p <= lh - 1; p++) {
                int ok = 1;
                for (int j = 0; j < key; j++)
                    if (hist[p - key + j] != cur[i - key + j]) { ok = 0; break; }
                if (!ok) continue;
                int run = 0;
                while (p + run < lh && i + run < n && hist[p + run] == cur[i + run]) run++;
                if (run > best_run) best_run = run;
            }
        }
        if (best_run > 0) { accepted += best_run; i += best_run; }
        else i += 1;
    }
    return accepted;
}

/* --------------------------------------------------------------- K policy */

enum { ORC_K_FIXED = 0, ORC_K_MATCHLEN = 1, ORC_K_AIMD = 2 };

/* Requested draft length before truncation (0 when there was no match). */
int orc_k_policy(int mode, int k_fixed, int k_state, int match_len, int k_max) {
    if (match_len <= 0) return 0;
    int k;
    if (mode == ORC_K_FIXED) k = k_fixed;
    else if (mode == ORC_K_MATCHLEN) k = match_len < 1 ? 1 : match_len;
    else k = k_state;
    if (k > k_max) k = k_max;
    if (k < 0) k = 0;
    return k;
}

/* Truncate by what the history still holds after p and by the response budget
 * (one emitted token always comes from the model itself). */
int orc_draft_len(int k_policy, int lh, int p, int budget_left) {
    if (p < 0) return 0;
    int k = k_policy;
    if (k > lh - p) k = lh - p;
    if (k > budget_left - 1) k = budget_left - 1;
    if (k < 0) k = 0;
    return k;
}

/* Window update of Sec. 5.4.  `drafted` = were there draft tokens at all,
 * `full` = every token on the verified path down to a leaf was accepted. */
int orc_aimd(int k, int drafted, int full, int inc, int cap, int reset) {
    if (!drafted) return k;
    if (full) { k += inc; if (k > cap) k = cap; return k; }
    return reset;
}

/* ------------------------------------------------------------- draft tree */

/*
 * Merge C draft chains into a token tree.  Node 0 is the root (the last
 * committed token, position l_cached).  Chains are inserted in candidate
 * order; a chain follows existing nodes while its tokens agree with them and
 * opens new nodes from its first differing token on.  Nodes are numbered in
 * creation order.  anc_mask bit i of node r is set iff node i lies on the
 * path root..r (r included).  Returns the node count.
 */
int orc_build_tree(int n_cand, const int32_t* const* chains, const int* chain_len, int32_t root_tok,
                   int l_cached, int32_t* tok, int32_t* pos, int32_t* parent, uint64_t* anc_mask,
                   int max_nodes) {
    int n = 0;
    tok[0] = root_tok; pos[0] = l_cached; parent[0] = -1; anc_mask[0] = 1ull; n = 1;
    for (int c = 0; c < n_cand; c++) {
        int cur = 0;
        for (int j = 0; j < chain_len[c]; j++) {
            int32_t t = chains[c][j];
            int found = -1;
            for (int i = 1; i < n; i++)
                if (parent[i] == cur && tok[i] == t) { found = i; break; }
            if (found < 0) {
                if (n >= max_nodes) return -1;
                tok[n] = t; pos[n] = pos[cur] + 1; parent[n] = cur;
                anc_mask[n] = anc_mask[cur] | (1ull << n);
                found = n++;
            }
            cur = found;
        }
    }
    return n;
}

/* ------------------------------------------------------------------ model */

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, max_pos;
    double rms_eps;
    const uint16_t* embed;          /* [vocab, d] bf16 bits */
    const uint16_t* lm_head;        /* [vocab, d] */
    const float* norm_f;            /* [d] */
    const uint16_t* const* wqkv;    /* per layer [(hq+2hkv)*h, d] */
    const uint16_t* const* wo;      /* per layer [d, hq*h] */
    const uint16_t* const* wgate;   /* per layer [f, d] */
    const uint16_t* const* wup;     /* per layer [f, d] */
    const uint16_t* const* wdown;   /* per layer [d, f] */
    const float* const* norm1;      /* per layer [d] */
    const float* const* norm2;      /* per layer [d] */
    const float* rope;              /* [max_pos, h/2, 2] (cos, sin) */
} orc_model;

typedef struct {
    const orc_model* m;
    int len, cap;
    int32_t* tokens;  /* tokens whose K/V are cached */
    double* k;        /* [layer][cap][hkv*h] */
    double* v;
    double* trace;    /* optional, caller-owned [(n_layers+1)][d_model]: residual stream of the last pushed token */
} orc_seq;

double orc_bf16(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* y[n_out] = W[n_out, n_in] . x[n_in], W in bf16 bits. */
static void matvec(const uint16_t* w, int n_out, int n_in, const double* x, double* y) {
#pragma omp parallel for schedule(static)
    for (int o = 0; o < n_out; o++) {
        const uint16_t* row = w + (size_t)o * n_in;
        double acc = 0.0;
        for (int i = 0; i < n_in; i++) acc += orc_bf16(row[i]) * x[i];
        y[o] = acc;
    }
}

static void rmsnorm(const double* x, const float* w, int d, double eps, double* y) {
    double ss = 0.0;
    for (int i = 0; i < d; i++) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; i++) y[i] = x[i] * r * (double)w[i];
}

/* Rotate-half pairing: element i is paired with i + h/2. */
static void rope_apply(double* vec, int h, const float* cs /* [h/2][2] */) {
    int half = h / 2;
    for (int i = 0; i < half; i++) {
        double c = (double)cs[2 * i], s = (double)cs[2 * i + 1];
        double a = vec[i], b = vec[i + half];
        vec[i] = a * c - b * s;
        vec[i + half] = b * c + a * s;
    }
}

/*
 * Softmax attention of one query over n keys: out = sum_j softmax_j(q.k_j *
 * scale) v_j.  k and v are [n][stride] with the head's h values at the front
 * of each row.
 */
void orc_attention_row(const double* q, const double* k, const double* v, int n, int stride, int h,
                       double scale, double* out) {
    double* s = (double*)malloc(sizeof(double) * (size_t)n);
    double mx = -INFINITY;
    for (int j = 0; j < n; j++) {
        double acc = 0.0;
        for (int i = 0; i < h; i++) acc += q[i] * k[(size_t)j * stride + i];
        s[j] = acc * scale;
        if (s[j] > mx) mx = s[j];
    }
    double z = 0.0;
    for (int j = 0; j < n; j++) { s[j] = exp(s[j] - mx); z += s[j]; }
    for (int i = 0; i < h; i++) {
        double acc = 0.0;
        for (int j = 0; j < n; j++) acc += s[j] * v[(size_t)j * stride + i];
        out[i] = acc / z;
    }
    free(s);
}

orc_seq* orc_seq_new(const orc_model* m, int cap) {
    orc_seq* s = (orc_seq*)calloc(1, sizeof(orc_seq));
    size_t kvw = (size_t)m->n_kv_heads * m->head_dim;
    s->m = m; s->cap = cap; s->len = 0;
    s->tokens = (int32_t*)calloc((size_t)cap, sizeof(int32_t));
    s->k = (double*)calloc((size_t)m->n_layers * cap * kvw, sizeof(double));
    s->v = (double*)calloc((size_t)m->n_layers * cap * kvw, sizeof(double));
    if (!s->tokens || !s->k || !s->v) { free(s->tokens); free(s->k); free(s->v); free(s); return NULL; }
    return s;
}

void orc_seq_free(orc_seq* s) {
    if (!s) return;
    free(s->tokens); free(s->k); free(s->v); free(s);
}

int orc_seq_len(const orc_seq* s) { return s->len; }

/* Forget every position >= len (used to re-evaluate another draft branch). */
int orc_seq_truncate(orc_seq* s, int len) {
    if (len < 0 || len > s->len) return -1;
    s->len = len;
    return 0;
}

/* Copy out the cached K and V of one layer/position ([hkv*h] each). */
int orc_seq_kv(const orc_seq* s, int layer, int pos, double* k_out, double* v_out) {
    const orc_model* m = s->m;
    size_t kvw = (size_t)m->n_kv_heads * m->head_dim;
    if (layer < 0 || layer >= m->n_layers || pos < 0 || pos >= s->len) return -1;
    memcpy(k_out, s->k + ((size_t)layer * s->cap + pos) * kvw, kvw * sizeof(double));
    memcpy(v_out, s->v + ((size_t)layer * s->cap + pos) * kvw, kvw * sizeof(double));
    return 0;
}

/* Install an externally supplied cache: k_in, v_in are [n_layers][n][n_kv_heads*head_dim]; afterwards positions
 * [0, n) count as cached. */
int orc_seq_load_kv(orc_seq* s, int n, const double* k_in, const double* v_in) {
    const orc_model* m = s->m;
    size_t kvw = (size_t)m->n_kv_heads * m->head_dim;
    if (n < 0 || n > s->cap) return -1;
    for (int l = 0; l < m->n_layers; l++) {
        memcpy(s->k + (size_t)l * s->cap * kvw, k_in + (size_t)l * n * kvw, (size_t)n * kvw * sizeof(double));
        memcpy(s->v + (size_t)l * s->cap * kvw, v_in + (size_t)l * n * kvw, (size_t)n * kvw * sizeof(double));
    }
    s->len = n;
    return 0;
}

/* Inspection hook: with a buffer of (n_layers + 1) * d_model doubles set (NULL = off), every orc_seq_push also copies
 * out the residual stream h of its token: row 0 after the embedding, row l + 1 after layer l.  No arithmetic. */
void orc_seq_set_trace(orc_seq* s, double* buf) { s->trace = buf; }

/*
 * Feed one token at position s->len: standard pre-norm decoder,
 *   h0 = E[token]
 *   per layer: n1 = RMSNorm(h); q,k,v = Wqkv n1; RoPE(q), RoPE(k) at pos;
 *              h += Wo Attn(q, K[0..pos], V[0..pos])       (causal, GQA, scale 1/sqrt(head_dim))
 *              n2 = RMSNorm(h); h += Wdown (silu(Wgate n2) * Wup n2)
 *   logits = Wlm RMSNorm(h).
 * Appends K/V to the cache.  `logits` (length vocab) may be NULL, in which
 * case the LM head is skipped.  Returns 0, or -1 when out of capacity.
 */
int orc_seq_push(orc_seq* s, int32_t token, double* logits) {
    const orc_model* m = s->m;
    int d = m->d_model, hq = m->n_q_heads, hkv = m->n_kv_heads, h = m->head_dim, f = m->d_ffn;
    int g = hq / hkv, pos = s->len;
    size_t kvw = (size_t)hkv * h;
    if (pos >= s->cap || pos >= m->max_pos || token < 0 || token >= m->vocab) return -1;
    int nqkv = (hq + 2 * hkv) * h;
    double* x = (double*)malloc(sizeof(double) * d);
    double* nx = (double*)malloc(sizeof(double) * d);
    double* qkv = (double*)malloc(sizeof(double) * nqkv);
    double* att = (double*)malloc(sizeof(double) * hq * h);
    double* proj = (double*)malloc(sizeof(double) * d);
    double* gate = (double*)malloc(sizeof(double) * f);
    double* up = (double*)malloc(sizeof(double) * f);
    const float* cs = m->rope + (size_t)pos * (h / 2) * 2;
    double scale = 1.0 / sqrt((double)h);

    for (int i = 0; i < d; i++) x[i] = orc_bf16(m->embed[(size_t)token * d + i]);
    if (s->trace) memcpy(s->trace, x, sizeof(double) * d);
    for (int l = 0; l < m->n_layers; l++) {
        rmsnorm(x, m->norm1[l], d, m->rms_eps, nx);
        matvec(m->wqkv[l], nqkv, d, nx, qkv);
        double* q = qkv;
        double* kk = qkv + (size_t)hq * h;
        double* vv = kk + kvw;
        for (int i = 0; i < hq; i++) rope_apply(q + (size_t)i * h, h, cs);
        for (int i = 0; i < hkv; i++) rope_apply(kk + (size_t)i * h, h, cs);
        double* kc = s->k + (size_t)l * s->cap * kvw;
        double* vc = s->v + (size_t)l * s->cap * kvw;
        memcpy(kc + (size_t)pos * kvw, kk, kvw * sizeof(double));
        memcpy(vc + (size_t)pos * kvw, vv, kvw * sizeof(double));
        for (int i = 0; i < hq; i++) {
            int j = i / g;
            orc_attention_row(q + (size_t)i * h, kc + (size_t)j * h, vc + (size_t)j * h, pos + 1,
                              (int)kvw, h, scale, att + (size_t)i * h);
        }
        matvec(m->wo[l], d, hq * h, att, proj);
        for (int i = 0; i < d; i++) x[i] += proj[i];
        rmsnorm(x, m->norm2[l], d, m->rms_eps, nx);
        matvec(m->wgate[l], f, d, nx, gate);
        matvec(m->wup[l], f, d, nx, up);
        for (int i = 0; i < f; i++) gate[i] = gate[i] / (1.0 + exp(-gate[i])) * up[i];
        matvec(m->wdown[l], d, f, gate, proj);
        for (int i = 0; i < d; i++) x[i] += proj[i];
        if (s->trace) memcpy(s->trace + (size_t)(l + 1) * d, x, sizeof(double) * d);
    }
    if (logits) {
        rmsnorm(x, m->norm_f, d, m->rms_eps, nx);
        matvec(m->lm_head, m->vocab, d, nx, logits);
    }
    s->tokens[pos] = token;
    s->len = pos + 1;
    free(x); free(nx); free(qkv); free(att); free(proj); free(gate); free(up);
    return 0;
}

/* Lowest index among the largest values. */
int orc_argmax(const double* x, int n) {
    int best = 0;
    for (int i = 1; i < n; i++) if (x[i] > x[best]) best = i;
    return best;
}

/*
 * Logits of every node of a draft tree, by the definition: node r's logits are those of the plain causal model fed
 * the cached prefix followed by the tokens on the path root..r.  For every node the cache is cut back to the
 * l_cached positions before the root and the whole path is pushed, token by token.  On return the cache is back at
 * l_cached.  logits is [n_nodes][vocab].
 */
int orc_tree_logits(orc_seq* s, int n_nodes, const int32_t* tok, const int32_t* parent, double* logits) {
    int base = s->len;
    int V = s->m->vocab;
    for (int r = 0; r < n_nodes; r++) {
        int path[80], np_ = 0;
        for (int c = r; c >= 0; c = parent[c]) { if (np_ >= 80) return -1; path[np_++] = c; }   /* leaf first */
        if (orc_seq_truncate(s, base) != 0) return -1;
        for (int j = np_ - 1; j >= 0; j--)
            if (orc_seq_push(s, tok[path[j]], j == 0 ? logits + (size_t)r * V : NULL) != 0) return -1;
    }
    return orc_seq_truncate(s, base);
}

/*
 * The same logits with less work, for harnesses that time or follow long chains (pinned against orc_tree_logits, to
 * which it is equal bit for bit: a position's K/V depend only on the tokens before it).  Nodes are visited in index
 * order; the K/V of the part of the path that the previously visited node shares stay in the cache, the rest is cut
 * away and the remaining path tokens are pushed.
 */
int orc_tree_logits_shared(orc_seq* s, int n_nodes, const int32_t* tok, const int32_t* parent, double* logits) {
    int base = s->len;
    int V = s->m->vocab;
    int cur[80], ncur = 0; /* nodes whose K/V sit in the cache above base, root first */
    for (int r = 0; r < n_nodes; r++) {
        int path[80], np_ = 0;
        for (int c = r; c >= 0; c = parent[c]) { if (np_ >= 80) return -1; path[np_++] = c; }
        int common = 0;
        while (common < ncur && common < np_ && cur[common] == path[np_ - 1 - common]) common++;
        if (common == np_) return -1;   /* node r itself already cached: nodes are distinct, cannot happen */
        if (orc_seq_truncate(s, base + common) != 0) return -1;
        ncur = common;
        for (int j = common; j < np_; j++) {
            int node = path[np_ - 1 - j];
            double* out = (j == np_ - 1) ? logits + (size_t)r * V : NULL;
            if (orc_seq_push(s, tok[node], out) != 0) return -1;
            cur[ncur++] = node;
        }
    }
    return orc_seq_truncate(s, base);
}

/* Threads the matrix-vector products use. */
#ifdef _OPENMP
#include <omp.h>
int orc_threads(void) { return omp_get_max_threads(); }
#else
int orc_threads(void) { return 1; }
#endif

/* ----------------------------------------------------------------- accept */

/*
 * Greedy acceptance given each node's greedy choice (arg[r] = argmax of node
 * r's logits, lowest id on ties).  Walk from the root: the model's choice g
 * at the current node is emitted; if a child carries exactly g the walk moves
 * there (the draft token is accepted), otherwise it stops.  Returns the
 * number of accepted draft tokens a; out_tok[0..a] are the a+1 emitted
 * tokens, path[0..a] the nodes visited (root first).
 */
int orc_accept_greedy(int n_nodes, const int32_t* tok, const int32_t* parent, const int32_t* arg,
                      int32_t* out_tok, int32_t* path) {
    int cur = 0, a = 0;
    path[0] = 0;
    for (;;) {
        int32_t g = arg[cur];
        out_tok[a] = g;
        int next = -1;
        for (int i = 1; i < n_nodes; i++)
            if (parent[i] == cur && tok[i] == g) { next = i; break; }
        if (next < 0) break;
        cur = next;
        a++;
        path[a] = cur;
    }
    return a;
}

/*
 * Greedy acceptance by its definition (Sec. 2.2: speculation keeps exactly the tokens plain decoding would have
 * produced).  From the cached prefix and the root token, decode autoregressively, one argmax token at a time, for as
 * many steps as the tree is deep plus one: g[0], g[1], ...  The accepted path is the deepest chain of nodes root ->
 * c1 -> c2 ... with tok[c_j] == g[j-1] for every j (at most one child of a node can carry a given token; were there
 * two, the first in node order counts); the emitted tokens are g[0..a].  The cache is back at its length on return.
 * Returns a, or -1 on error.
 */
int orc_accept_greedy_bruteforce(orc_seq* s, int n_nodes, const int32_t* tok, const int32_t* parent,
                                 int32_t* out_tok, int32_t* path) {
    int base = s->len, V = s->m->vocab;
    int depth_max = 0;
    for (int r = 0; r < n_nodes; r++) {
        int dpt = 0;
        for (int c = r; parent[c] >= 0; c = parent[c]) dpt++;
        if (dpt > depth_max) depth_max = dpt;
    }
    double* lg = (double*)malloc(sizeof(double) * (size_t)V);
    int32_t* g = (int32_t*)malloc(sizeof(int32_t) * (size_t)(depth_max + 1));
    int32_t t = tok[0];
    for (int i = 0; i <= depth_max; i++) {          /* plain autoregressive greedy decoding */
        if (orc_seq_push(s, t, lg) != 0) { free(lg); free(g); return -1; }
        g[i] = t = orc_argmax(lg, V);
    }
    int cur = 0, a = 0;
    path[0] = 0;
    for (;;) {                                       /* longest prefix of g that the tree spells out */
        int next = -1;
        for (int i = 1; i < n_nodes && next < 0; i++)
            if (parent[i] == cur && tok[i] == g[a]) next = i;
        if (next < 0) break;
        cur = next;
        path[++a] = cur;
    }
    for (int i = 0; i <= a; i++) out_tok[i] = g[i];
    free(lg); free(g);
    return orc_seq_truncate(s, base) == 0 ? a : -1;
}

/* Philox-4x32, 10 rounds (Salmon et al., SC'11). */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; r++) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The generator on n counters: out[i] = orc_philox4x32_10(ctr[i], key).  A plain loop, for bulk comparison. */
void orc_philox_batch(int n, const uint32_t* ctr, const uint32_t key[2], uint32_t* out) {
    for (int i = 0; i < n; i++) orc_philox4x32_10(ctr + 4 * (size_t)i, key, out + 4 * (size_t)i);
}

/*
 * The uniform in [0,1) that decides the token at absolute position `position`
 * of sequence `seq_id`: key = seed, counter = (position, draw_kind, seq_id);
 * the first output word's top 24 bits.  draw_kind j < 7 is the acceptance
 * test of the j-th child tried at a node, 7 is the final sample.
 */
double orc_uniform(uint64_t seed, uint64_t seq_id, uint32_t position, uint32_t draw_kind) {
    uint32_t ctr[4] = {position, draw_kind, (uint32_t)seq_id, (uint32_t)(seq_id >> 32)};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return (double)(out[0] >> 8) * (1.0 / 16777216.0);
}

/*
 * Rejection-sampling acceptance along a draft tree (speculative sampling
 * with a deterministic draft, so the draft distribution is a point mass and
 * the acceptance probability of a draft token is its target probability).
 * At the current node: p = softmax(logits / temperature).  Children are
 * tried in node order; child j is accepted iff u_j < p(tok_j); on a rejection
 * p(tok_j) is set to zero and p is renormalised.  When a child is accepted
 * the walk moves there.  When none is (or the node is a leaf) one token is
 * drawn from the remaining p by inverse CDF in increasing token id (first id
 * whose cumulative weight reaches u * total) and the walk ends.
 * logits is [n_nodes][vocab]; pos[r] is node r's absolute position, so the
 * token it decides sits at pos[r] + 1.  Returns a; out_tok[0..a], path[0..a]
 * as for the greedy rule.  margin_out (may be NULL) receives the smallest
 * distance between a uniform and the threshold it was compared with, as a
 * probability, so callers can flag decisions too close to call.
 */
int orc_accept_stochastic(int n_nodes, int vocab, const int32_t* tok, const int32_t* parent,
                          const int32_t* pos, const double* logits, double temperature, uint64_t seed,
                          uint64_t seq_id, int32_t* out_tok, int32_t* path, double* margin_out) {
    double* w = (double*)malloc(sizeof(double) * (size_t)vocab);
    int cur = 0, a = 0;
    double margin = 1.0;
    path[0] = 0;
    for (;;) {
        const double* lg = logits + (size_t)cur * vocab;
        double mx = -INFINITY;
        for (int i = 0; i < vocab; i++) if (lg[i] > mx) mx = lg[i];
        for (int i = 0; i < vocab; i++) w[i] = exp((lg[i] - mx) / temperature);
        uint32_t position = (uint32_t)(pos[cur] + 1);
        int next = -1, tried = 0;
        for (int i = 1; i < n_nodes && next < 0; i++) {
            if (parent[i] != cur) continue;
            double z = 0.0;
            for (int t = 0; t < vocab; t++) z += w[t];
            double p = w[tok[i]] / z;
            double u = orc_uniform(seed, seq_id, position, (uint32_t)tried);
            if (fabs(u - p) < margin) margin = fabs(u - p);
            if (u < p) next = i;
            else w[tok[i]] = 0.0;
            tried++;
        }
        if (next >= 0) {
            out_tok[a] = tok[next];
            cur = next;
            a++;
            path[a] = cur;
            continue;
        }
        double z = 0.0;
        for (int t = 0; t < vocab; t++) z += w[t];
        double u = orc_uniform(seed, seq_id, position, 7u);
        double target = u * z, cum = 0.0;
        int pick = -1, last_nz = 0;
        for (int t = 0; t < vocab; t++) {
            if (w[t] > 0.0) last_nz = t;
            cum += w[t];
            if (w[t] > 0.0 && cum >= target) {
                pick = t;
                double lo = (cum - w[t]) / z, hi = cum / z;
                double dm = fmin(fabs(u - lo), fabs(hi - u));
                if (dm < margin) margin = dm;
                break;
            }
        }
        if (pick < 0) pick = last_nz;
        out_tok[a] = pick;
        break;
    }
    if (margin_out) *margin_out = margin;
    free(w);
    return a;
}
