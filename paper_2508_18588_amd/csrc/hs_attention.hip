// Ragged multi-query paged attention for the verify step.
//
// For sequence b with L cached positions and nn draft-tree nodes, every node's query (all G query heads that
// share one KV head) attends to cache positions [0, L) and to the slots L + i of the nodes i that are its
// ancestors or itself.  The KV cache is read once per (sequence, KV head) and step, shared by all G * nn query
// rows -- which is why verifying a whole draft costs about one KV traversal (Sec. 2.2 of the paper).
//
// Work decomposition.  Keys are cut into partitions of `part_keys` absolute positions; every (partition, KV head,
// sequence) yields one partial result (unnormalised O, running max, running sum) per query row, and a second
// kernel merges a row's partitions in index order.  Inside a partition, keys are visited in 32-key sub-tiles (two
// 16-token pages), each through the same routine: scores transposed, S^T = K . Q^T (v_mfma_f32_32x32x16_bf16,
// A = K tile from LDS, B = Q^T held in registers), so that each lane owns one query row -- the online-softmax
// statistics are per-lane scalars and the exponentiated scores are already in the register layout the second
// product O^T = V^T . P^T needs as its B operand.  V is stored in the cache with the token index fastest so V^T
// tiles are plain 8-byte LDS reads.
//
// Two ways to run a unit (= one partition of one (sequence, KV head)), chosen per sequence by its number of query
// rows R = G * nn:
//   R <= 32 (one-token decoding and short drafts): one WAVEFRONT per unit.  A wavefront streams its units one after
//     the other through a private LDS slice and never synchronises with the others.  With a single 32-row tile the
//     softmax arithmetic of a partition is one instruction stream; giving every wavefront its own stream keeps all
//     four SIMDs of a compute unit busy and the KV stream bandwidth-bound.
//   R > 32: one WORKGROUP per unit; K/V tiles of 128 keys are staged once and shared, the (up to four) 32-row tiles
//     are dealt to the 4 wavefronts.  A sequence with more than 128 query rows per KV head is cut into units of
//     four row tiles, each of which walks the partition's keys on its own: holding two row tiles per wavefront
//     instead would cost every workgroup unit of the launch half the resident workgroups (registers), which was
//     measured to be far dearer than reading the K/V of the few very long drafts twice.  In a unit with two or three
//     live row tiles the wavefronts without a tile only stage K/V (most of each tile); the computing ones keep one
//     page per tile.
// Both run the identical per-row arithmetic on the identical partitions: masked keys contribute exact zeros and
// partitions merge in index order, so a row's result is bit-identical whether it is verified next to other draft
// rows or decoded alone.
//
// Launch.  The units of a step are listed on the device once per verify call (attn_worklist_kernel) and a
// persistent grid -- exactly the workgroups that are resident at once -- works the lists off: wavefront units by a
// static deal, workgroup units through a counter (see attn_verify_mfma).  K and V are read with non-temporal loads.
// A second entry, attn_prefill_mfma, runs the same sub-tile routine causally over a chunk of consecutive tokens.
#include "hs_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

namespace {

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// One 32-key sub-tile for one 32-row query tile: S^T = K.Q^T, online softmax per lane, O^T += V^T.P^T.
// sK points at the sub-tile's 32 key rows, sV at its two 16-token pages.  Every query row's arithmetic is
// independent of which other rows are in flight.
// CHAIN (prefill): the rows are consecutive tokens; L is then a position below which every row of the tile sees every
// key and `total` the lane's own bound (keys < total are visible), no ancestor mask.
template <int HD, bool CHAIN = false>
__device__ inline void attn_subtile(const bf16_t* sK, const bf16_t* sV, const bf16x8 (&qf)[HD / 16],
                                    f32x16 (&o)[HD / 32], float& m_run, float& l_run, uint64_t anc, int kbase, int L,
                                    int total, float scale_log2, int half, int l32) {
    constexpr int KS = HD + 8, VS = 20, NKS = HD / 16, NDT = HD / 32;
    f32x16 s;
#pragma unroll
    for (int e = 0; e < 16; e++) s[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < NKS; ks++) {
        bf16x8 ka = *reinterpret_cast<const bf16x8*>(&sK[l32 * KS + ks * 16 + half * 8]);
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[ks], s, 0, 0, 0);
    }
    // element e: key kbase + 8*(e/4) + 4*half + e%4, query row = this lane's.  Only tiles that reach past the
    // cached prefix need the tree mask.
    if (kbase + 32 > L) {
#pragma unroll
        for (int e = 0; e < 16; e++) {
            int kp = kbase + 8 * (e >> 2) + 4 * half + (e & 3);
            bool vis = kp < L || (kp < total && (CHAIN || ((anc >> (kp - L)) & 1ull)));
            s[e] = vis ? s[e] : -INFINITY;
        }
    }
    float tmax = s[0];
#pragma unroll
    for (int e = 1; e < 16; e++) tmax = fmaxf(tmax, s[e]);
    // lanes l and l+32 hold the two halves of a query row: v_permlane32_swap puts the upper half of its first
    // operand and the lower half of its second in each other's place, so the two results are, in some order, a
    // lane's own value and its partner's -- enough for a maximum and for a sum, with no trip through the LDS
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(tmax), __float_as_uint(tmax), false, false);
        tmax = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1])) * scale_log2;   // scale > 0: commutes with max
    }
    float m_new = fmaxf(m_run, tmax);
    float m_safe = (m_new == -INFINITY) ? 0.f : m_new;
    float alpha = fast_exp2(m_run - m_safe);
    float psum = 0.f;
    bf16x8 pb[2];
#pragma unroll
    for (int e = 0; e < 16; e++) {
        float p = fast_exp2(__builtin_fmaf(s[e], scale_log2, -m_safe));
        psum += p;
        pb[e >> 3][e & 7] = (__bf16)p;
    }
    {
        const auto sw = __builtin_amdgcn_permlane32_swap(__float_as_uint(psum), __float_as_uint(psum), false, false);
        psum = __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
    }
    l_run = l_run * alpha + psum;
    m_run = m_new;
    // the running maximum rarely moves after the first tiles: multiplying by exactly 1 is skipped
    if (__any(alpha != 1.f)) {
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
#pragma unroll
            for (int e = 0; e < 16; e++) o[dt][e] *= alpha;
    }
#pragma unroll
    for (int kk = 0; kk < 2; kk++)
#pragma unroll
        for (int dt = 0; dt < NDT; dt++) {
            const bf16_t* vrow = &sV[(kk * HD + dt * 32 + l32) * VS];
            u32x2 lo = *reinterpret_cast<const u32x2*>(vrow + 4 * half);
            u32x2 hi = *reinterpret_cast<const u32x2*>(vrow + 8 + 4 * half);
            union { u32x4 u; bf16x8 v; } va;
            va.u = u32x4{lo.x, lo.y, hi.x, hi.y};
            o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va.v, pb[kk], o[dt], 0, 0, 0);
        }
}

// Page holding position p0, as a wavefront-uniform value.  Positions at or beyond `total` (nothing written yet) and
// malformed table entries resolve to the sequence's first page: its keys are masked and its finite values are
// multiplied by exact zeros, so every load can be unconditional.
__device__ inline int safe_page(const int32_t* bt, int p0, int total, int max_blocks, int n_blocks) {
    int pidx = p0 >> 4;
    int page = (p0 < total && pidx < max_blocks) ? bt[pidx] : bt[0];
    page = (page >= 0 && page < n_blocks) ? page : 0;
    return __builtin_amdgcn_readfirstlane(page);
}

// Per-lane variant: the page of position p0 (which differs from lane to lane), same fall-backs.
__device__ inline int safe_page_lane(const int32_t* bt, int p0, int total, int max_blocks, int n_blocks) {
    int pidx = p0 >> 4;
    int page = (p0 < total && pidx < max_blocks) ? bt[pidx] : bt[0];
    return (page >= 0 && page < n_blocks) ? page : 0;
}

// Query fragments (B operand of S^T) and ancestor mask of the lane's row; rows beyond R read as zero.
template <int HD>
__device__ inline void load_query_tile(const bf16_t* q, const uint64_t* anc_mask, int r0, int rt, int R, int G,
                                       int hq, int j, int half, int l32, bf16x8 (&qf)[HD / 16], uint64_t& anc) {
    int rho = rt * 32 + l32;
    bool ok = rho < R;
    int node = ok ? rho / G : 0;
    int g = ok ? rho - node * G : 0;
    anc = (ok && anc_mask) ? anc_mask[r0 + node] : 0ull;
    const bf16_t* qp = q + ((size_t)(r0 + node) * hq + j * G + g) * HD;
#pragma unroll
    for (int ks = 0; ks < HD / 16; ks++) {
        if (ok) {
            qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16 + half * 8);
        } else {
#pragma unroll
            for (int e = 0; e < 8; e++) qf[ks][e] = (__bf16)0.f;
        }
    }
}

// Partial result of one partition for the lane's row: running max (log2 domain) and sum in fp32, and the partition's
// own normalised output O / l in fp16 -- a convex combination of V rows, so within fp16's range whenever V is, and
// rounded 8 times finer than the bf16 result of the merge.  Half the bytes of an fp32 partial: the partial results
// are the one write stream of the launch, and writes in the middle of the K/V read stream are dear.
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));

template <int HD>
__device__ inline void store_partial(const f32x16 (&o)[HD / 32], float m_run, float l_run, _Float16* part_o,
                                     float* part_ml, int r0, int rt, int R, int G, int hq, int j, int max_parts,
                                     int part, int half, int l32) {
    int rho = rt * 32 + l32;
    if (rho >= R) return;
    int node = rho / G, g = rho - node * G;
    size_t prow = ((size_t)(r0 + node) * hq + j * G + g) * max_parts + part;
    _Float16* po = part_o + prow * HD;
    const float inv = l_run > 0.f ? 1.f / l_run : 0.f;   // a partition in which the row sees no key: all zero
#pragma unroll
    for (int dt = 0; dt < HD / 32; dt++)
#pragma unroll
        for (int g4 = 0; g4 < 4; g4++) {
            f16x4 v = {(_Float16)(o[dt][4 * g4] * inv), (_Float16)(o[dt][4 * g4 + 1] * inv),
                       (_Float16)(o[dt][4 * g4 + 2] * inv), (_Float16)(o[dt][4 * g4 + 3] * inv)};
            *reinterpret_cast<f16x4*>(po + dt * 32 + 8 * g4 + 4 * half) = v;
        }
    if (half == 0) {
        part_ml[prow * 2] = m_run;
        part_ml[prow * 2 + 1] = l_run;
    }
}

// Everything a unit of work needs besides its own (sequence, KV head, partition).
struct AttnArgs {
    const bf16_t* q;
    const bf16_t* kc;     // already offset to the layer
    const bf16_t* vc;
    const int32_t* seq_len;
    const int32_t* block_table;
    const int32_t* row_off;
    const uint64_t* anc_mask;
    _Float16* part_o;
    float* part_ml;
    int max_blocks, n_blocks, max_parts, part_keys, hq, hkv;
    float scale_log2;
};

// A unit of work: one partition of one (sequence, KV head), with the sequence's row range and cached length, as the
// list kernel wrote it (two int4 per unit).
struct AttnUnit { int b, j, part, r0, nn, L, rt0; };   // rt0: first 32-row tile this unit covers (workgroup units)

__device__ inline AttnUnit attn_unit_from(const int4& p, const int4& q) {
    AttnUnit u;
    u.b = __builtin_amdgcn_readfirstlane(p.x);
    u.j = __builtin_amdgcn_readfirstlane(p.y);
    u.part = __builtin_amdgcn_readfirstlane(p.z);
    u.r0 = __builtin_amdgcn_readfirstlane(p.w);
    u.nn = __builtin_amdgcn_readfirstlane(q.x);
    u.L = __builtin_amdgcn_readfirstlane(q.y);
    u.rt0 = __builtin_amdgcn_readfirstlane(q.z);
    return u;
}

// Units with at most 32 query rows, taken by ONE WAVEFRONT each: the wavefront walks its units (first, first + stride,
// ...) as one uninterrupted stream of 32-key sub-tiles through a private LDS slice, always with the next sub-tile's
// K/V in flight in registers -- also across a unit boundary: the next unit's list entry is read during the current
// unit's first sub-tile, its page numbers during the second, its first sub-tile during the current unit's last.
// There is no workgroup synchronisation (a wavefront's LDS operations execute in order) and no atomic: a load or an
// atomic that returns late holds back every later load of its wavefront.
template <int HD>
__device__ inline void attn_wave_stream(const AttnArgs& a, const int4* __restrict__ list, int n_units, int first,
                                        int stride, bf16_t* sKw, bf16_t* sVw, int lane) {
    constexpr int KS = HD + 8, VS = 20, NKS = HD / 16, NDT = HD / 32;
    if (first >= n_units) return;
    const int half = lane >> 5, l32 = lane & 31;
    const int G = a.hq / a.hkv;
    const size_t page_stride = (size_t)a.hkv * 16 * HD;

    AttnUnit cu = attn_unit_from(list[2 * first], list[2 * first + 1]);
    int total = cu.L + cu.nn;
    int k_begin = cu.part * a.part_keys;
    int k_end = min(total, k_begin + a.part_keys);
    const bf16_t* kbase_ptr = a.kc + (size_t)cu.j * 16 * HD;   // + page * page_stride
    const bf16_t* vbase_ptr = a.vc + (size_t)cu.j * HD * 16;
    // the unit's page numbers, fetched once: lane l holds the page of positions k_begin + 16 l .. + 15 (a partition
    // has at most 64 pages), handed out by readlane -- no table look-up sits between two sub-tiles
    int my_page = safe_page_lane(a.block_table + (size_t)cu.b * a.max_blocks, k_begin + 16 * lane, total, a.max_blocks,
                                 a.n_blocks);

    int it_n = first + stride;
    bool have_n = it_n < n_units;
    int4 en0 = list[2 * (have_n ? it_n : first)], en1 = list[2 * (have_n ? it_n : first) + 1];
    bool n_ready = false;
    AttnUnit nu = cu;
    int total_n = total, k_begin_n = k_begin, k_end_n = k_end, my_page_n = my_page;
    const bf16_t *kbase_n = kbase_ptr, *vbase_n = vbase_ptr;

    bf16x8 qf[NKS];
    uint64_t anc;
    f32x16 o[NDT];
    float m_run = -INFINITY, l_run = 0.f;
    load_query_tile<HD>(a.q, a.anc_mask, cu.r0, 0, cu.nn * G, G, a.hq, cu.j, half, l32, qf, anc);
#pragma unroll
    for (int dt = 0; dt < NDT; dt++)
#pragma unroll
        for (int e = 0; e < 16; e++) o[dt][e] = 0.f;

    // one 32-key sub-tile = two pages; a page's K block and V^T block are each 16*HD contiguous elements, copied as
    // NCP 16-byte chunks per lane (chunk c = lane + 64*ii covers elements [8c, 8c+8)).  The loads are non-temporal:
    // K/V is read once per launch, and kept out of the caches it leaves the queries and the partial results (which
    // the merge kernel reads right after) there -- 10 % of the launch
    constexpr int NCP = HD / 32;
    u32x4 rk[2 * NCP], rv[2 * NCP];
#define HS_W_FETCH(PAGES, KPTR, VPTR, PAGE0)                                                                      \
    {                                                                                                             \
        _Pragma("unroll") for (int pp = 0; pp < 2; pp++) {                                                        \
            const size_t pofs = (size_t)__builtin_amdgcn_readlane(PAGES, (PAGE0) + pp) * page_stride;             \
            const bf16_t* kp_ = (KPTR) + pofs + lane * 8;                                                         \
            const bf16_t* vp_ = (VPTR) + pofs + lane * 8;                                                         \
            _Pragma("unroll") for (int ii = 0; ii < NCP; ii++) {                                                  \
                rk[pp * NCP + ii] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kp_ + ii * 512));                           \
                rv[pp * NCP + ii] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vp_ + ii * 512));                           \
            }                                                                                                     \
        }                                                                                                         \
    }
    HS_W_FETCH(my_page, kbase_ptr, vbase_ptr, 0)
    int kb = k_begin;
    for (;;) {
#pragma unroll
        for (int pp = 0; pp < 2; pp++)
#pragma unroll
            for (int ii = 0; ii < NCP; ii++) {
                int c = lane + 64 * ii;
                int key = pp * 16 + c / (HD / 8), c16 = c % (HD / 8);
                *reinterpret_cast<u32x4*>(&sKw[key * KS + c16 * 8]) = rk[pp * NCP + ii];
                int dim = c >> 1, hf = c & 1;
                u32x2* dst = reinterpret_cast<u32x2*>(&sVw[(pp * HD + dim) * VS + hf * 8]);
                dst[0] = u32x2{rv[pp * NCP + ii].x, rv[pp * NCP + ii].y};
                dst[1] = u32x2{rv[pp * NCP + ii].z, rv[pp * NCP + ii].w};
            }
        const bool last = kb + 32 >= k_end;
        if (have_n && !n_ready && (kb > k_begin || last)) {
            nu = attn_unit_from(en0, en1);
            total_n = nu.L + nu.nn;
            k_begin_n = nu.part * a.part_keys;
            k_end_n = min(total_n, k_begin_n + a.part_keys);
            kbase_n = a.kc + (size_t)nu.j * 16 * HD;
            vbase_n = a.vc + (size_t)nu.j * HD * 16;
            my_page_n = safe_page_lane(a.block_table + (size_t)nu.b * a.max_blocks, k_begin_n + 16 * lane, total_n,
                                       a.max_blocks, a.n_blocks);
            n_ready = true;
        }
        if (!last) HS_W_FETCH(my_page, kbase_ptr, vbase_ptr, (kb + 32 - k_begin) >> 4)
        else if (have_n) HS_W_FETCH(my_page_n, kbase_n, vbase_n, 0)
        attn_subtile<HD>(sKw, sVw, qf, o, m_run, l_run, anc, kb, cu.L, total, a.scale_log2, half, l32);
        kb += 32;
        if (last) {
            store_partial<HD>(o, m_run, l_run, a.part_o, a.part_ml, cu.r0, 0, cu.nn * G, G, a.hq, cu.j, a.max_parts, cu.part,
                              half, l32);
            if (!have_n) break;
            cu = nu;
            total = total_n; k_begin = k_begin_n; k_end = k_end_n; my_page = my_page_n;
            kbase_ptr = kbase_n; vbase_ptr = vbase_n;
            kb = k_begin;
            it_n += stride;
            have_n = it_n < n_units;
            n_ready = false;
            en0 = list[2 * (have_n ? it_n : first)];
            en1 = list[2 * (have_n ? it_n : first) + 1];
            load_query_tile<HD>(a.q, a.anc_mask, cu.r0, 0, cu.nn * G, G, a.hq, cu.j, half, l32, qf, anc);
#pragma unroll
            for (int dt = 0; dt < NDT; dt++)
#pragma unroll
                for (int e = 0; e < 16; e++) o[dt][e] = 0.f;
            m_run = -INFINITY;
            l_run = 0.f;
        }
    }
#undef HS_W_FETCH
}

// One partition of one (sequence, KV head) by the WORKGROUP (R > 32): 128-key tiles shared by the four wavefronts, the
// unit's 32-row tiles (un.rt0 .. un.rt0 + 3) dealt to them round-robin, one tile of register prefetch.  (RTW row
// tiles per wavefront; the launcher instantiates RTW = 1.)
template <int HD, int RTW, int NLIVE>
__device__ inline void attn_unit_wg_n(const AttnArgs& a, const AttnUnit& un, bf16_t* sK, bf16_t* sV, int tid) {
    constexpr int KS = HD + 8, VS = 20, NKS = HD / 16, NDT = HD / 32;
    // keys per shared tile: with one row tile per wavefront there are registers for a 128-key tile in flight (twice
    // the bytes on their way per workgroup), with two only for 64
    constexpr int TILE = RTW == 1 ? 128 : 64;
    constexpr int NCK = TILE * HD / 2048;   // 16-byte K chunks per thread and tile
    const int lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int b = un.b, j = un.j, part = un.part, r0 = un.r0, nn = un.nn, L = un.L;
    const int total = L + nn;
    const int G = a.hq / a.hkv;
    const int R = nn * G;
    const int nrt = (R + 31) >> 5;
    const int k_begin = part * a.part_keys;
    if (nn <= 0 || k_begin >= total) return;     // uniform over the workgroup
    const int k_end = min(total, k_begin + a.part_keys);
    const int32_t* bt = a.block_table + (size_t)b * a.max_blocks;
    const bf16_t* kbase_ptr = a.kc + (size_t)j * 16 * HD;
    const bf16_t* vbase_ptr = a.vc + (size_t)j * HD * 16;
    const size_t page_stride = (size_t)a.hkv * 16 * HD;
    // row tiles start at a unit-dependent wavefront so that two-tile sequences do not all use the same SIMDs
    const int slot = (wave - (part + j + b)) & 3;

    bf16x8 qf[RTW][NKS];
    f32x16 o[RTW][NDT];
    float m_run[RTW], l_run[RTW];
    uint64_t anc[RTW];
    bool rt_on[RTW];
#pragma unroll
    for (int t = 0; t < RTW; t++) {
        int rt = un.rt0 + slot + 4 * t;
        rt_on[t] = rt < nrt;
        load_query_tile<HD>(a.q, a.anc_mask, r0, rt_on[t] ? rt : 0, rt_on[t] ? R : 0, G, a.hq, j, half, l32, qf[t], anc[t]);
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
#pragma unroll
            for (int e = 0; e < 16; e++) o[t][dt][e] = 0.f;
        m_run[t] = -INFINITY;
        l_run[t] = 0.f;
    }

    // Staging.  A tile of TILE keys = TILE/16 pages, each 2*HD 16-byte chunks of K and as many of V^T.  A wavefront
    // stages a run of whole pages.  With four live row tiles (NLIVE = 4) every wavefront stages a quarter of the
    // tile; in a unit with fewer (a sequence of 33..96 query rows per KV head, or the last tile group of a longer
    // one) the wavefronts without a row tile do nothing but stage, and take most of the pages off the ones that
    // compute: loads, address arithmetic and LDS writes leave the instruction streams that carry the softmax and
    // the MFMAs.  The two kinds of wavefront run separate loops (so that the staging registers of the one and the
    // accumulators of the other do not add up) with the same two barriers per tile.
    //   pages per tile = TILE/16 = 8:   4 live tiles (or 1): 2 pages each;  3: 1 each + 5;  2: 1 each + 3 + 3
    // NLIVE = 4: every wavefront stages a quarter; NLIVE = 2: two or three live tiles (n_live), one routine for both.
    constexpr int NPG = TILE / 16;
    constexpr int PC = NLIVE == 4 ? NPG / 4 : NPG / 8;                            // pages of a computing wavefront
    constexpr int PI = NLIVE == 4 ? 1 : NPG - 3 * PC;                             // most pages of a staging-only one
    constexpr int CPP = 2 * HD / 64;                                              // 64-lane chunk rows per page
    const int n_live = NLIVE == 4 ? 4 : min(4, nrt - un.rt0);
    const int npi = __builtin_amdgcn_readfirstlane(NLIVE == 4 ? 0 : (NPG - n_live * PC) / (4 - n_live));
    const bool computes = slot < n_live;
    const int page0 = __builtin_amdgcn_readfirstlane(computes ? slot * PC : n_live * PC + (slot - n_live) * npi);
    // lane p: the page of the partition's keys 16 p .. 16 p + 15 (a partition has at most 64 pages); one vector
    // load per unit instead of a scalar load per page and tile
    const int my_page = safe_page_lane(bt, k_begin + 16 * lane, total, a.max_blocks, a.n_blocks);
    // lane parts of the addresses: chunk row r of a page holds chunks 64 r .. 64 r + 63
    const int lane_g = lane * 8;                                              // elements, global side
    const int lane_k = (lane / (HD / 8)) * KS + (lane % (HD / 8)) * 8;        // sK: 64 / (HD/8) keys per chunk row
    const int lane_v = (lane >> 1) * VS + (lane & 1) * 8;                     // sV: 32 dims per chunk row
#define HS_G_FETCH(KB, NP, NPRT)   /* NP: compile-time bound, NPRT: the wavefront's pages (>= 3 when guarded) */  \
    {                                                                                                             \
        _Pragma("unroll") for (int pg = 0; pg < NP; pg++) {                                                       \
            if (pg >= 3 && pg >= (NPRT)) break;                                                                   \
            const size_t pofs = (size_t)__builtin_amdgcn_readlane(my_page, (((KB) - k_begin) >> 4) + page0 + pg) * page_stride; \
            _Pragma("unroll") for (int r = 0; r < CPP; r++) {                                                     \
                rk[pg * CPP + r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(kbase_ptr + pofs + r * 512 + lane_g)); \
                rv[pg * CPP + r] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(vbase_ptr + pofs + r * 512 + lane_g)); \
            }                                                                                                     \
        }                                                                                                         \
    }
#define HS_G_STAGE(NP, NPRT)                                                                                      \
    {                                                                                                             \
        bf16_t* pk = sK + page0 * 16 * KS + lane_k;                                                               \
        bf16_t* pv = sV + page0 * HD * VS + lane_v;                                                               \
        _Pragma("unroll") for (int pg = 0; pg < NP; pg++)                                                         \
            _Pragma("unroll") for (int r = 0; r < CPP; r++) {                                                     \
                if (pg >= 3 && pg >= (NPRT)) break;                                                     \
                *reinterpret_cast<u32x4*>(pk + (pg * 16 + r * (512 / HD)) * KS) = rk[pg * CPP + r];               \
                u32x2* dst = reinterpret_cast<u32x2*>(pv + (pg * HD + r * 32) * VS);                              \
                dst[0] = u32x2{rv[pg * CPP + r].x, rv[pg * CPP + r].y};                                           \
                dst[1] = u32x2{rv[pg * CPP + r].z, rv[pg * CPP + r].w};                                           \
            }                                                                                                     \
    }
    if (!computes) {
        // staging only: no row tile, nothing to store at the end
        u32x4 rk[PI * CPP], rv[PI * CPP];
        HS_G_FETCH(k_begin, PI, npi)
        for (int kbase = k_begin; kbase < k_end; kbase += TILE) {
            __syncthreads();  // previous tile (or previous unit) fully consumed
            HS_G_STAGE(PI, npi)
            __syncthreads();
            if (kbase + TILE < k_end) HS_G_FETCH(kbase + TILE, PI, npi)
        }
        return;
    }
    u32x4 rk[PC * CPP], rv[PC * CPP];
    HS_G_FETCH(k_begin, PC, PC)
    for (int kbase = k_begin; kbase < k_end; kbase += TILE) {
        __syncthreads();  // previous tile (or previous unit) fully consumed
        HS_G_STAGE(PC, PC)
        __syncthreads();
        if (kbase + TILE < k_end) HS_G_FETCH(kbase + TILE, PC, PC)
#pragma unroll
        for (int sub = 0; sub < TILE / 32; sub++) {
            const int kb = kbase + 32 * sub;
            if (kb >= k_end) break;
#pragma unroll
            for (int t = 0; t < RTW; t++) {
                if (!rt_on[t]) continue;
                attn_subtile<HD>(sK + sub * 32 * KS, sV + sub * 2 * HD * VS, qf[t], o[t], m_run[t], l_run[t], anc[t],
                                 kb, L, total, a.scale_log2, half, l32);
            }
        }
    }
#undef HS_G_STAGE
#undef HS_G_FETCH
#pragma unroll
    for (int t = 0; t < RTW; t++) {
        if (!rt_on[t]) continue;
        store_partial<HD>(o[t], m_run[t], l_run[t], a.part_o, a.part_ml, r0, un.rt0 + slot + 4 * t, R, G, a.hq, j,
                          a.max_parts, part, half, l32);
    }
}

// The unit's number of live row tiles (1..4; a group of four tiles per unit) selects the staging split.
template <int HD, int RTW>
__device__ inline void attn_unit_wg(const AttnArgs& a, const AttnUnit& un, bf16_t* sK, bf16_t* sV, int tid) {
    const int nrt = (un.nn * (a.hq / a.hkv) + 31) >> 5;
    const int n_live = RTW == 1 ? min(4, nrt - un.rt0) : 4;
    if (n_live == 3 || n_live == 2) attn_unit_wg_n<HD, RTW, 2>(a, un, sK, sV, tid);
    else attn_unit_wg_n<HD, RTW, 4>(a, un, sK, sV, tid);   // also a single live tile: everyone stages a quarter
}

// The units of one step, built once per hs_verify call (the same for every layer): a unit = one partition of one
// (sequence, KV head), in (sequence, partition, head) order.  List A: units of sequences with more than 32 query rows
// per KV head (taken by whole workgroups), list B: the others (taken by single wavefronts).  An entry is two int4:
// (sequence, head, partition, first row) (rows, cached length, first row tile, 0).  work[0] = |A|, work[1] = |B|, work[2 + l] = the
// counter through which layer l's launch hands out list A (zeroed here).
__global__ __launch_bounds__(256) void attn_worklist_kernel(const int32_t* __restrict__ seq_len,
                                                             const int32_t* __restrict__ row_off, int batch,
                                                             int part_keys, int G, int hkv, int max_parts, int n_layers,
                                                             int32_t* __restrict__ work, int4* __restrict__ list_a,
                                                             int4* __restrict__ list_b) {
    __shared__ int s_nu[256], s_off[256], s_r0[256], s_nn[256], s_len[256], s_grp[256];
    __shared__ int sw_a[4], sw_b[4];
    __shared__ int carry_a, carry_b;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = tid; i < n_layers; i += 256) work[2 + i] = 0;
    if (tid == 0) { carry_a = 0; carry_b = 0; }
    __syncthreads();
    for (int b0 = 0; b0 < batch; b0 += 256) {
        const int b = b0 + tid;
        int nu = 0, r0 = 0, nn = 0, L = 0, ngrp = 1;
        bool is_a = false;
        if (b < batch) {
            r0 = row_off[b];
            nn = row_off[b + 1] - r0;
            L = seq_len[b] - 1;
            if (nn > 0 && L >= 0) {
                const int nparts = min(max_parts, (L + nn + part_keys - 1) / part_keys);
                is_a = nn * G > 32;
                // a workgroup covers four 32-row tiles: a sequence with more query rows per KV head than that gets
                // one unit per group of four tiles (each walks the partition's keys on its own)
                if (is_a) ngrp = (nn * G + 127) / 128;
                nu = nparts * hkv * ngrp;
            }
        }
        int ia = is_a ? nu : 0, ib = is_a ? 0 : nu;
        const int va = ia, vb = ib;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            int ta = __shfl_up(ia, o), tb = __shfl_up(ib, o);
            if (lane >= o) { ia += ta; ib += tb; }
        }
        if (lane == 63) { sw_a[wave] = ia; sw_b[wave] = ib; }
        __syncthreads();
        int ba = carry_a, bb = carry_b;
        for (int w2 = 0; w2 < wave; w2++) { ba += sw_a[w2]; bb += sw_b[w2]; }
        // the sign of s_nu tells the list: positive = B, negative = A
        s_nu[tid] = is_a ? -nu : nu;
        s_off[tid] = is_a ? ba + ia - va : bb + ib - vb;
        s_r0[tid] = r0;
        s_nn[tid] = nn;
        s_len[tid] = L;
        s_grp[tid] = ngrp;
        __syncthreads();
        if (tid == 255) { carry_a = ba + ia; carry_b = bb + ib; }
        const int nb = min(256, batch - b0);
        for (int i = wave; i < nb; i += 4) {     // a wavefront per sequence: a sequence has a few dozen units
            const int n = s_nu[i];
            int4* dst = (n < 0 ? list_a : list_b) + 2 * (size_t)s_off[i];
            const int cnt = n < 0 ? -n : n, grp = s_grp[i];
            for (int u = lane; u < cnt; u += 64) {
                // v = (partition, head); the tile groups of one (partition, head) are neighbours (grp is 1 or 2: at
                // most 256 query rows per KV head)
                const int v = grp == 1 ? u : (grp == 2 ? (u >> 1) : u / grp);
                dst[2 * u] = make_int4(b0 + i, v % hkv, v / hkv, s_r0[i]);
                dst[2 * u + 1] = make_int4(s_nn[i], s_len[i], 4 * (u - v * grp), 0);
            }
        }
        __syncthreads();
    }
    if (tid == 0) { work[0] = carry_a; work[1] = carry_b; }
}

// Persistent launch: exactly as many workgroups as the chip holds at once.  First every wavefront streams its share
// of the wavefront units (wavefront w of workgroup g: units 4 g + w, 4 g + w + 4 gridDim.x, ... -- dealt out
// statically, so that nothing but K/V tiles is ever waited for); then the workgroups take the workgroup units one by
// one through a counter (`take`, zeroed by the list kernel).  These are short -- four wavefronts share one partition
// -- and fill the ragged end of the first phase: a workgroup that had less to stream takes more of them.  The claim
// for the next unit is issued before the current one is computed.  No workgroup is launched for work that does not
// exist, and which workgroup computes a unit has no influence on the unit's result.
template <int HD, int RTW>
__global__ __launch_bounds__(256, (RTW == 1 ? 2 : 1)) void attn_verify_mfma(AttnArgs a, const int32_t* __restrict__ work,
                                                                            int32_t* __restrict__ take,
                                                                            const int4* __restrict__ list_a,
                                                                            const int4* __restrict__ list_b) {
    constexpr int KS = HD + 8;        // sK row stride (bf16)
    constexpr int VS = 20;            // sV row stride (bf16): 16 tokens + pad, 40 bytes
    // 128 keys of K and 8 pages of V^T: four private 32-key slices (wavefront units) or tiles of 64 keys shared by
    // the workgroup (workgroup units)
    __shared__ __attribute__((aligned(16))) bf16_t sK[128 * KS];
    __shared__ __attribute__((aligned(16))) bf16_t sV[8 * HD * VS];
    __shared__ int s_item[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_a = work[0], n_b = work[1];
    attn_wave_stream<HD>(a, list_b, n_b, blockIdx.x * 4 + wave, gridDim.x * 4, sK + wave * 32 * KS,
                         sV + wave * 2 * HD * VS, lane);
    if (n_a == 0) return;
    if (tid == 0) s_item[0] = atomicAdd(take, 1);
    __syncthreads();   // also: every private slice is consumed before shared tiles are written
    int it = s_item[0], slot = 0;
    while (it < n_a) {
        if (tid == 0) s_item[slot ^ 1] = atomicAdd(take, 1);
        const AttnUnit un = attn_unit_from(list_a[2 * it], list_a[2 * it + 1]);
        attn_unit_wg<HD, RTW>(a, un, sK, sV, tid);
        __syncthreads();
        slot ^= 1;
        it = s_item[slot];
    }
}

// Prefill of a chunk of consecutive tokens per sequence (KV recomputation of a resumed rollout): token i of the chunk
// attends to positions [0, L + i].  One workgroup per (block of 256 query rows, KV head, sequence) walks the keys
// from position 0 in 64-key tiles -- a row's arithmetic depends on absolute key positions only, not on how the text
// was cut into chunks -- and writes the normalised output itself: with hundreds of rows per sequence there is
// enough parallelism without cutting the key axis.  Row tiles of 32 rows (rows of one token's G query heads are
// adjacent) are dealt to the four wavefronts, two each; a row tile skips the key tiles that lie wholly behind it.
template <int HD>
__global__ __launch_bounds__(256, 1) void attn_prefill_mfma(
    const bf16_t* __restrict__ q, const bf16_t* __restrict__ kc, const bf16_t* __restrict__ vc, size_t layer_off,
    const int32_t* __restrict__ len_plus1, const int32_t* __restrict__ block_table, int max_blocks, int n_blocks,
    const int32_t* __restrict__ row_off, bf16_t* __restrict__ out, int hq, int hkv, float scale_log2) {
    constexpr int KS = HD + 8, VS = 20, NKS = HD / 16, NDT = HD / 32, RTW = 2, TILE = 64, NCK = HD / 32;
    __shared__ __attribute__((aligned(16))) bf16_t sK[TILE * KS];
    __shared__ __attribute__((aligned(16))) bf16_t sV[4 * HD * VS];

    const int j = blockIdx.y, b = blockIdx.z;
    const int r0 = row_off[b];
    const int nn = row_off[b + 1] - r0;
    if (nn <= 0) return;
    const int L = len_plus1[b] - 1;
    const int total = L + nn;
    const int G = hq / hkv;
    const int R = nn * G;
    const int row_base = blockIdx.x * (128 * RTW);
    if (row_base >= R) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int half = lane >> 5, l32 = lane & 31;
    const int32_t* bt = block_table + (size_t)b * max_blocks;
    const bf16_t* kbase_ptr = kc + layer_off + (size_t)j * 16 * HD;
    const bf16_t* vbase_ptr = vc + layer_off + (size_t)j * HD * 16;
    const size_t page_stride = (size_t)hkv * 16 * HD;
    // keys this block needs: up to the position of its last row's token
    const int last_node = min(nn - 1, (min(R, row_base + 128 * RTW) - 1) / G);
    const int k_end = L + last_node + 1;

    bf16x8 qf[RTW][NKS];
    f32x16 o[RTW][NDT];
    float m_run[RTW], l_run[RTW];
    int lim_lane[RTW], lim_min[RTW], lim_max[RTW];
    bool rt_on[RTW];
#pragma unroll
    for (int t = 0; t < RTW; t++) {
        const int rt = blockIdx.x * (4 * RTW) + wave + 4 * t;
        rt_on[t] = rt * 32 < R;
        uint64_t unused;
        load_query_tile<HD>(q, nullptr, r0, rt_on[t] ? rt : 0, rt_on[t] ? R : 0, G, hq, j, half, l32, qf[t], unused);
        const int rho = rt * 32 + l32;
        lim_lane[t] = (rt_on[t] && rho < R) ? L + rho / G + 1 : 0;
        lim_min[t] = L + (rt * 32) / G + 1;
        lim_max[t] = L + min(nn - 1, (rt * 32 + 31) / G) + 1;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
#pragma unroll
            for (int e = 0; e < 16; e++) o[t][dt][e] = 0.f;
        m_run[t] = -INFINITY;
        l_run[t] = 0.f;
    }

    u32x4 rk[NCK], rv[NCK];
    const int wave_c0 = tid & ~63;
#define HS_P_FETCH(KB)                                                                                            \
    {                                                                                                             \
        _Pragma("unroll") for (int i = 0; i < NCK; i++) {                                                         \
            const int kk = (wave_c0 + 256 * i) / (2 * HD);                                                        \
            const int within = (tid + 256 * i) % (2 * HD);                                                        \
            const size_t pofs = (size_t)safe_page(bt, (KB) + 16 * kk, total, max_blocks, n_blocks) * page_stride; \
            rk[i] = *reinterpret_cast<const u32x4*>(kbase_ptr + pofs + within * 8);                               \
            rv[i] = *reinterpret_cast<const u32x4*>(vbase_ptr + pofs + within * 8);                               \
        }                                                                                                         \
    }
    HS_P_FETCH(0)
    for (int kbase = 0; kbase < k_end; kbase += TILE) {
        __syncthreads();  // previous tile fully consumed
#pragma unroll
        for (int i = 0; i < NCK; i++) {
            const int kk = (wave_c0 + 256 * i) / (2 * HD);
            const int within = (tid + 256 * i) % (2 * HD);
            int key = kk * 16 + within / (HD / 8), c16 = within % (HD / 8);
            *reinterpret_cast<u32x4*>(&sK[key * KS + c16 * 8]) = rk[i];
            int dim = within >> 1, hf = within & 1;
            u32x2* dst = reinterpret_cast<u32x2*>(&sV[(kk * HD + dim) * VS + hf * 8]);
            dst[0] = u32x2{rv[i].x, rv[i].y};
            dst[1] = u32x2{rv[i].z, rv[i].w};
        }
        __syncthreads();
        if (kbase + TILE < k_end) HS_P_FETCH(kbase + TILE)
#pragma unroll
        for (int sub = 0; sub < 2; sub++) {
            const int kb = kbase + 32 * sub;
#pragma unroll
            for (int t = 0; t < RTW; t++) {
                if (!rt_on[t] || kb >= lim_max[t]) continue;   // wavefront-uniform: nothing of this sub-tile is visible
                attn_subtile<HD, true>(sK + sub * 32 * KS, sV + sub * 2 * HD * VS, qf[t], o[t], m_run[t], l_run[t], 0ull,
                                       kb, lim_min[t], lim_lane[t], scale_log2, half, l32);
            }
        }
    }
#undef HS_P_FETCH
#pragma unroll
    for (int t = 0; t < RTW; t++) {
        const int rho = (blockIdx.x * (4 * RTW) + wave + 4 * t) * 32 + l32;
        if (!rt_on[t] || rho >= R) continue;
        const int node = rho / G, g = rho - node * G;
        const float inv = 1.f / l_run[t];     // a row always sees its own key: the sum is positive
        bf16_t* po = out + ((size_t)(r0 + node) * hq + j * G + g) * HD;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
#pragma unroll
            for (int g4 = 0; g4 < 4; g4++) {
                u32x2 w;
                w.x = (uint32_t)f32_to_bf16(o[t][dt][4 * g4] * inv) | ((uint32_t)f32_to_bf16(o[t][dt][4 * g4 + 1] * inv) << 16);
                w.y = (uint32_t)f32_to_bf16(o[t][dt][4 * g4 + 2] * inv) | ((uint32_t)f32_to_bf16(o[t][dt][4 * g4 + 3] * inv) << 16);
                *reinterpret_cast<u32x2*>(po + dt * 32 + 8 * g4 + 4 * half) = w;
            }
    }
}

// Combine the partitions of one (row, query head) in partition order: one wavefront per (row, head), four per
// workgroup; rows are strided over the grid's x dimension (the row count is only known on the device).  Lane p
// holds partition p's (max, sum); weights are broadcast from there.
template <int HD>
__global__ __launch_bounds__(256) void attn_merge(const _Float16* __restrict__ part_o, const float* __restrict__ part_ml,
                                                   const int32_t* __restrict__ row2seq, const int32_t* __restrict__ row_off,
                                                   const int32_t* __restrict__ seq_len, int batch, int max_parts,
                                                   int part_keys, int hq, bf16_t* __restrict__ out) {
    const int head = blockIdx.y * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (head >= hq) return;
    const int m = row_off[batch];
    for (int row = blockIdx.x; row < m; row += gridDim.x) {
        const int b = row2seq[row];
        const int total = seq_len[b] - 1 + (row_off[b + 1] - row_off[b]);
        const int nparts = min(max_parts, (total + part_keys - 1) / part_keys);
        const size_t prow = ((size_t)row * hq + head) * max_parts;
        float mg = -INFINITY;
        for (int p0 = 0; p0 < nparts; p0 += 64) {
            float mp = (p0 + lane < nparts) ? part_ml[(prow + p0 + lane) * 2] : -INFINITY;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) mp = fmaxf(mp, __shfl_xor(mp, o));
            mg = fmaxf(mg, mp);
        }
        float den = 0.f, acc[HD / 64];
#pragma unroll
        for (int i = 0; i < HD / 64; i++) acc[i] = 0.f;
        for (int p0 = 0; p0 < nparts; p0 += 64) {
            float wl = 0.f, ll = 0.f;
            if (p0 + lane < nparts) {
                wl = fast_exp2(part_ml[(prow + p0 + lane) * 2] - mg);
                ll = part_ml[(prow + p0 + lane) * 2 + 1];
            }
            const int n = min(64, nparts - p0);
            // partition order; the values of eight partitions are fetched before the first is added, so that the loop
            // waits for memory once per eight partitions instead of once per partition
            for (int pb = 0; pb < n; pb += 8) {
                _Float16 v[8][HD / 64];
#pragma unroll
                for (int q = 0; q < 8; q++) {
                    const _Float16* po = part_o + (prow + p0 + min(pb + q, n - 1)) * HD;
#pragma unroll
                    for (int i = 0; i < HD / 64; i++) v[q][i] = po[lane + 64 * i];
                }
#pragma unroll
                for (int q = 0; q < 8; q++) {
                    if (pb + q < n) {
                        // the partition's weight in the whole: exp2(m_p - m) l_p; its output is stored normalised
                        const float w = __shfl(wl, pb + q) * __shfl(ll, pb + q);
                        den += w;
#pragma unroll
                        for (int i = 0; i < HD / 64; i++) acc[i] += w * (float)v[q][i];
                    }
                }
            }
        }
#pragma unroll
        for (int i = 0; i < HD / 64; i++) out[((size_t)row * hq + head) * HD + lane + 64 * i] = f32_to_bf16(acc[i] / den);
    }
}

// Plain kernel for debugging and for the fp32-activation mode: one wavefront per (row, query head), keys visited one
// by one.  T = bf16_t (queries, cache and output are bf16; fp32 arithmetic) or float (nothing rounded below fp32, the
// running sum and output carried in fp64, library exponential).
__device__ __forceinline__ float plain_ld(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ float plain_ld(const float* p) { return *p; }
__device__ __forceinline__ void plain_st(bf16_t* p, double v) { *p = f32_to_bf16((float)v); }
__device__ __forceinline__ void plain_st(float* p, double v) { *p = (float)v; }

template <typename T, typename ACC>
__global__ __launch_bounds__(64) void attn_verify_plain(
    const T* __restrict__ q, const T* __restrict__ kc, const T* __restrict__ vc, size_t layer_off,
    const int32_t* __restrict__ seq_len, const int32_t* __restrict__ block_table, int max_blocks, int n_blocks,
    const int32_t* __restrict__ row_off, const int32_t* __restrict__ row2seq, const uint64_t* __restrict__ anc_mask,
    int batch, int hq, int hkv, int hd, float scale, T* __restrict__ out) {
    constexpr bool PRECISE = sizeof(ACC) == 8;
    int row = blockIdx.x, head = blockIdx.y, lane = threadIdx.x;
    if (row >= row_off[batch]) return;
    int b = row2seq[row];
    int L = seq_len[b] - 1, nn = row_off[b + 1] - row_off[b];
    int total = L + nn, j = head / (hq / hkv);
    uint64_t anc = anc_mask[row];
    const T* qp = q + ((size_t)row * hq + head) * hd;
    float q0 = lane < hd ? plain_ld(qp + lane) : 0.f;
    float q1 = lane + 64 < hd ? plain_ld(qp + lane + 64) : 0.f;
    ACC m = -INFINITY, l = 0, o0 = 0, o1 = 0;
    for (int kp = 0; kp < total; kp++) {
        bool vis = kp < L || ((anc >> (kp - L)) & 1ull);
        if (!vis) continue;
        if ((kp >> 4) >= max_blocks) break;
        int page = block_table[(size_t)b * max_blocks + (kp >> 4)];
        if (page < 0 || page >= n_blocks) break;
        int ip = kp & 15;
        const T* kr = kc + layer_off + (((size_t)page * hkv + j) * 16 + ip) * hd;
        ACC dot = 0;
        if (lane < hd) dot += (ACC)q0 * (ACC)plain_ld(kr + lane);
        if (lane + 64 < hd) dot += (ACC)q1 * (ACC)plain_ld(kr + lane + 64);
        if (PRECISE) {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) {
                const double dd = (double)dot;
                const int lo = __shfl_xor(__double2loint(dd), o), hi = __shfl_xor(__double2hiint(dd), o);
                dot += (ACC)__hiloint2double(hi, lo);
            }
        } else {
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) dot += (ACC)__shfl_xor((float)dot, o);
        }
        ACC s = dot * (ACC)scale;
        ACC mn = s > m ? s : m;
        ACC a, p;
        if (PRECISE) { a = (ACC)exp((double)(m - mn)); p = (ACC)exp((double)(s - mn)); }
        else { a = (ACC)__expf((float)(m - mn)); p = (ACC)__expf((float)(s - mn)); }
        l = l * a + p;
        const T* vr = vc + layer_off + ((size_t)page * hkv + j) * hd * 16 + ip;
        float v0 = lane < hd ? plain_ld(vr + (size_t)lane * 16) : 0.f;
        float v1 = lane + 64 < hd ? plain_ld(vr + (size_t)(lane + 64) * 16) : 0.f;
        o0 = o0 * a + p * (ACC)v0;
        o1 = o1 * a + p * (ACC)v1;
        m = mn;
    }
    T* op = out + ((size_t)row * hq + head) * hd;
    if (lane < hd) plain_st(op + lane, (double)(o0 / l));
    if (lane + 64 < hd) plain_st(op + lane + 64, (double)(o1 / l));
}

template <int HD, int RTW>
void launch_mfma(const hs_ctx* ctx, int layer, size_t layer_off, const hs_kv_cache* cache, const hs_seq_state* seq,
                 const hs_step* step, const bf16_t* q, hipStream_t st) {
    const hs_model_desc& d = ctx->desc;
    AttnArgs a;
    a.q = q;
    a.kc = (const bf16_t*)cache->k + layer_off;
    a.vc = (const bf16_t*)cache->v + layer_off;
    a.seq_len = seq->seq_len;
    a.block_table = seq->block_table;
    a.row_off = step->row_off;
    a.anc_mask = step->anc_mask;
    a.part_o = reinterpret_cast<_Float16*>(ctx->ws + ctx->lay.part_o);
    a.part_ml = reinterpret_cast<float*>(ctx->ws + ctx->lay.part_ml);
    a.max_blocks = ctx->lim.max_blocks_per_seq;
    a.n_blocks = cache->n_blocks;
    a.max_parts = ctx->max_parts;
    a.part_keys = ctx->att_part;
    a.hq = d.n_q_heads;
    a.hkv = d.n_kv_heads;
    a.scale_log2 = 1.4426950408889634f / sqrtf((float)HD);
    int32_t* work = reinterpret_cast<int32_t*>(ctx->ws + ctx->lay.att_work);
    const int4* list_a = reinterpret_cast<const int4*>(ctx->ws + ctx->lay.att_list);
    const int4* list_b = list_a + 2 * hs_attention_max_units(ctx);
    // the wavefront units are dealt out statically: the grid is what is resident at once, no more
    static int per_cu = 0;
    if (per_cu == 0) {
        int n = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, (const void*)attn_verify_mfma<HD, RTW>, 256, 0) != hipSuccess ||
            n < 1)
            n = 1;
        per_cu = n;
    }
    dim3 grid(ctx->n_cu * per_cu);
    hipLaunchKernelGGL((attn_verify_mfma<HD, RTW>), grid, dim3(256), 0, st, a, work, work + 2 + layer, list_a, list_b);
}

}  // namespace

void hs_launch_attention(const hs_ctx* ctx, int layer, const hs_kv_cache* cache, const hs_seq_state* seq,
                         const hs_step* step, const void* q_any, void* out, hipStream_t st) {
    const hs_model_desc& d = ctx->desc;
    size_t layer_off = (size_t)layer * cache->n_blocks * d.n_kv_heads * 16 * d.head_dim;
    if (hs_plain_kernels(ctx)) {
        const dim3 grid(ctx->lim.max_rows, d.n_q_heads);
        const float scale = 1.f / sqrtf((float)d.head_dim);
        if (hs_fp32_activations(ctx))
            hipLaunchKernelGGL((attn_verify_plain<float, double>), grid, dim3(64), 0, st, (const float*)q_any,
                               (const float*)cache->k, (const float*)cache->v, layer_off, seq->seq_len,
                               seq->block_table, ctx->lim.max_blocks_per_seq, cache->n_blocks, step->row_off,
                               step->row2seq, step->anc_mask, seq->batch, d.n_q_heads, d.n_kv_heads, d.head_dim,
                               scale, (float*)out);
        else
            hipLaunchKernelGGL((attn_verify_plain<bf16_t, float>), grid, dim3(64), 0, st, (const bf16_t*)q_any,
                               (const bf16_t*)cache->k, (const bf16_t*)cache->v, layer_off, seq->seq_len,
                               seq->block_table, ctx->lim.max_blocks_per_seq, cache->n_blocks, step->row_off,
                               step->row2seq, step->anc_mask, seq->batch, d.n_q_heads, d.n_kv_heads, d.head_dim,
                               scale, (bf16_t*)out);
        return;
    }
    const bf16_t* q = (const bf16_t*)q_any;
    // one row tile per wavefront, two workgroups per compute unit, whatever the longest draft: a sequence with more
    // than 128 query rows per KV head comes as several units (see attn_worklist_kernel)
    if (d.head_dim == 128) launch_mfma<128, 1>(ctx, layer, layer_off, cache, seq, step, q, st);
    else launch_mfma<64, 1>(ctx, layer, layer_off, cache, seq, step, q, st);
}

size_t hs_attention_max_units(const hs_ctx* ctx) {
    // a sequence's (partition, KV head) pairs, times the groups of four row tiles its query rows can fill
    const int r_max = (ctx->desc.n_q_heads / ctx->desc.n_kv_heads) * (1 + ctx->lim.c_max * ctx->lim.k_max);
    return (size_t)ctx->lim.max_batch * ctx->max_parts * ctx->desc.n_kv_heads * ((r_max + 127) / 128);
}

void hs_launch_attention_worklist(const hs_ctx* ctx, const hs_seq_state* seq, const hs_step* step, hipStream_t st) {
    if (hs_plain_kernels(ctx)) return;
    const hs_model_desc& d = ctx->desc;
    int32_t* work = reinterpret_cast<int32_t*>(ctx->ws + ctx->lay.att_work);
    int4* list_a = reinterpret_cast<int4*>(ctx->ws + ctx->lay.att_list);
    int4* list_b = list_a + 2 * hs_attention_max_units(ctx);
    hipLaunchKernelGGL(attn_worklist_kernel, dim3(1), dim3(256), 0, st, seq->seq_len, step->row_off, seq->batch,
                       ctx->att_part, d.n_q_heads / d.n_kv_heads, d.n_kv_heads, ctx->max_parts, d.n_layers, work, list_a,
                       list_b);
}

void hs_launch_attention_prefill(const hs_ctx* ctx, int layer, const hs_kv_cache* cache, const hs_seq_state* seq,
                                 const int32_t* len_plus1, const hs_step* step, const bf16_t* q, bf16_t* out, int chunk,
                                 hipStream_t st) {
    const hs_model_desc& d = ctx->desc;
    const size_t layer_off = (size_t)layer * cache->n_blocks * d.n_kv_heads * 16 * d.head_dim;
    const int G = d.n_q_heads / d.n_kv_heads;
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)d.head_dim);
    dim3 grid((chunk * G + 255) / 256, d.n_kv_heads, seq->batch);
    if (d.head_dim == 128)
        hipLaunchKernelGGL((attn_prefill_mfma<128>), grid, dim3(256), 0, st, q, (const bf16_t*)cache->k,
                           (const bf16_t*)cache->v, layer_off, len_plus1, seq->block_table,
                           ctx->lim.max_blocks_per_seq, cache->n_blocks, step->row_off, out, d.n_q_heads, d.n_kv_heads,
                           scale_log2);
    else
        hipLaunchKernelGGL((attn_prefill_mfma<64>), grid, dim3(256), 0, st, q, (const bf16_t*)cache->k,
                           (const bf16_t*)cache->v, layer_off, len_plus1, seq->block_table,
                           ctx->lim.max_blocks_per_seq, cache->n_blocks, step->row_off, out, d.n_q_heads, d.n_kv_heads,
                           scale_log2);
}

void hs_launch_attention_merge(const hs_ctx* ctx, const hs_seq_state* seq, const hs_step* step, void* out_any,
                               hipStream_t st) {
    if (hs_plain_kernels(ctx)) return;  // the plain kernel writes the final output itself
    bf16_t* out = (bf16_t*)out_any;
    const hs_model_desc& d = ctx->desc;
    const _Float16* part_o = reinterpret_cast<const _Float16*>(ctx->ws + ctx->lay.part_o);
    float* part_ml = reinterpret_cast<float*>(ctx->ws + ctx->lay.part_ml);
    dim3 grid(hs_row_grid(ctx, 256, (d.n_q_heads + 3) / 4), (d.n_q_heads + 3) / 4);
    if (d.head_dim == 128)
        hipLaunchKernelGGL((attn_merge<128>), grid, dim3(256), 0, st, part_o, part_ml, step->row2seq, step->row_off,
                           seq->seq_len, seq->batch, ctx->max_parts, ctx->att_part, d.n_q_heads, out);
    else
        hipLaunchKernelGGL((attn_merge<64>), grid, dim3(256), 0, st, part_o, part_ml, step->row2seq, step->row_off,
                           seq->seq_len, seq->batch, ctx->max_parts, ctx->att_part, d.n_q_heads, out);
}
