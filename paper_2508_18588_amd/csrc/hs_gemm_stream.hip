// The bf16 MFMA GEMM of the projections:  C[M,N] (+)= A[M,K] . W[N,K]^T,  built for the row counts of a verify
// step (a few hundred draft-tree rows) and run in row passes for more (prefill, wide drafts).
//
// At a verify step's row count a projection is bound by streaming its weights from HBM exactly once, with the
// matrix cores needed at roughly half their rate just to keep up (220 rows: 220 flop per weight byte).  The kernel
// is laid out around the weight stream:
//   * One workgroup per (group of NU 32-row weight units, K chunk, row pass); unit and chunk counts are chosen by
//     the host so that one round of workgroups covers the 256 compute units.  A workgroup holds all rows of its
//     pass (up to 128*MT) against its weight slab, so with one pass every weight byte is fetched once.
//   * Row tile t (32 rows) belongs to wavefront t % 4.  A wavefront multiplies only the row tiles that exist
//     (M is read on the device) against all NU weight units; its accumulators stay in registers for the whole chunk.
//   * Tiles (64 deep in K) travel from global memory straight into LDS (global_load_lds_dwordx4) through an
//     SA-stage activation ring and an SW-stage weight ring.
//   * One instruction stream per SIMD: a wavefront issues one instruction at a time, so a fragment read that waits
//     its turn at the LDS, or scalar bookkeeping between two MFMAs, keeps the next MFMA from issuing.  The loop is
//     therefore software-pipelined over k-steps of 16 -- the fragments of step s+2 are read while step s is
//     multiplied, across tile boundaries -- the reads and loads are placed one by one behind single MFMAs, and
//     the steady state of the loop carries no modulo arithmetic and as few guards as possible.  The tile hand-over
//     (wait for the loads of the next tile, workgroup barrier, issue of new loads) sits in the middle of a tile,
//     after the last fragment read of the current one has been issued.
// SwiGLU pairs the gate and up rows of 16 output columns in one 32-row weight unit, so that both pre-activations of
// a column meet in one MFMA tile (lanes c and c+16).
#include "hs_gemm_common.h"

using namespace hs_gemm_detail;

namespace {

constexpr int TILE_BYTES = 32 * ROW_BYTES;  // a 32-row tile of either operand, 64 deep: 4 KB

// A pointer known to be the same in every lane, moved to scalar registers.
__device__ __forceinline__ const unsigned char* uniform_ptr(const unsigned char* p) {
    const unsigned long long v = (unsigned long long)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (const unsigned char*)(((unsigned long long)hi << 32) | lo);
}

// s_waitcnt vmcnt(n) for a wavefront-uniform run-time n (the instruction takes an immediate).
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {
    switch (n) {
#define HS_CASE(i) case i: HS_WAIT_VMCNT(i); break;
        HS_CASE(0) HS_CASE(1) HS_CASE(2) HS_CASE(3) HS_CASE(4) HS_CASE(5) HS_CASE(6) HS_CASE(7) HS_CASE(8)
        HS_CASE(9) HS_CASE(10) HS_CASE(11) HS_CASE(12) HS_CASE(13) HS_CASE(14) HS_CASE(15) HS_CASE(16)
        HS_CASE(17) HS_CASE(18) HS_CASE(19) HS_CASE(20) HS_CASE(21) HS_CASE(22) HS_CASE(23) HS_CASE(24)
        HS_CASE(25) HS_CASE(26) HS_CASE(27) HS_CASE(28) HS_CASE(29) HS_CASE(30) HS_CASE(31) HS_CASE(32)
#undef HS_CASE
        default: HS_WAIT_VMCNT(32); break;  // stricter than asked for is always correct
    }
}

struct stream_args {
    const unsigned char* A;
    const unsigned char* wb[2];  // weight matrices (gate, up) or (W, W)
    void* Cout;
    float* part;
    int M, m_max, N, K, n0, m0, kt0, kt1, chunk, group, n_groups;
    int w_once;  // the launch reads every weight byte once (one row pass): non-temporal weight loads
    int w_pre;   // the weight-only part of the prologue has been issued already (by the kernel, before M was known)
};

// The 1 KB blocks of weight tile kt that wavefront `wave` fetches: block wave + 4j = quarter `wave` of unit j, into
// stage kt % SW of the weight ring.  (A SwiGLU unit holds 16 gate rows then the 16 up rows of the same columns, so a
// wavefront's blocks are all gate rows -- wavefronts 0, 1 -- or all up rows -- 2, 3.)
template <int NU, int MT, int SA, int SW>
__device__ __forceinline__ void issue_weight_tile(const stream_args& p, const unsigned char* w_mine, unsigned smem_off,
                                                  const unsigned (&w_off)[NU], int wave, int kt) {
    constexpr int W_RING = SA * 4 * MT * TILE_BYTES, W_STAGE = NU * TILE_BYTES;
    const unsigned dst = smem_off + W_RING + (kt % SW) * W_STAGE + wave * 1024;
    const unsigned char* base = w_mine + (size_t)kt * ROW_BYTES;
#pragma unroll
    for (int j = 0; j < NU; j++) {
        if (p.w_once) load_to_lds_16_stream(base, w_off[j], dst + j * 4096);
        else load_to_lds_16(base, w_off[j], dst + j * 4096);
    }
}

// One K chunk of one row pass for a wavefront that owns NMI live row tiles (0 = loads and barriers only).
template <int EPI, bool PARTIAL, int NU, int MT, int SA, int SW, int NMI>
__device__ __forceinline__ void stream_chunk(const stream_args& p, unsigned char* smem, unsigned smem_off,
                                             const unsigned (&w_off)[NU], int wave, int lane) {
    static_assert(SA >= 2 && SA <= SW, "the hand-over bookkeeping assumes the activation ring is the shorter one");
    constexpr int A_STAGE = 4 * MT * TILE_BYTES, W_STAGE = NU * TILE_BYTES, W_RING = SA * A_STAGE;
    constexpr int NLW = NU;  // 1 KB load instructions per weight tile and wavefront
    constexpr int NM = NMI > 0 ? NMI : 1;
    const int lrow = lane >> 3, lpos = lane & 7;
    const int l32 = lane & 31, g = lane >> 5, fl = swz(l32);
    const int frag_row = l32 * ROW_BYTES;
    const unsigned a_chunk = (unsigned)((lpos ^ swz(8 * wave + lrow)) << 4);
    const int a_row = p.m0 + 8 * wave + lrow;
    const unsigned row_pitch = (unsigned)p.K * 2u;
    // 8-row blocks of the activation tile this wavefront fetches: block wave + 4j covers rows 32j + 8*wave .. +7
    // of the pass; blocks past the last row are not fetched.
    int n_a = 0;
#pragma unroll
    for (int j = 0; j < 4 * MT; j++)
        if (p.m0 + 8 * wave + 32 * j < p.M) n_a = j + 1;
    n_a = __builtin_amdgcn_readfirstlane(n_a);

    auto issue_a = [&](int kt) {
        const unsigned dst = smem_off + (kt % SA) * A_STAGE + wave * 1024;
        const unsigned char* base = p.A + (size_t)kt * ROW_BYTES;
#pragma unroll
        for (int j = 0; j < 4 * MT; j++) {
            if (j < n_a) {
                const unsigned off = (unsigned)min(a_row + 32 * j, p.M - 1) * row_pitch + a_chunk;
                load_to_lds_16(base, off, dst + j * 4096);
            }
        }
    };
    const unsigned char* w_mine = uniform_ptr((EPI == HS_EPI_SWIGLU_BF16 && wave >= 2) ? p.wb[1] : p.wb[0]);
    auto issue_w = [&](int kt) { issue_weight_tile<NU, MT, SA, SW>(p, w_mine, smem_off, w_off, wave, kt); };
    // Hand-over number h (h < kt0 before the loop, then in the middle of tile h): first the activation tile h+SA,
    // then the weight tile h+SW.  The issue order fixes the wait counts below.
    auto issue_for = [&](int h) {
        if (h + SA >= p.kt0 && h + SA < p.kt1) issue_a(h + SA);
        if (h + SW >= p.kt0 && h + SW < p.kt1) issue_w(h + SW);
    };
    // Loads complete in issue order.  Tile t is awaited in the middle of tile t-1, when the hand-overs up to t-2
    // have been made.  Its activation part was issued at hand-over t-SA, its weight part at t-SW (earlier or the
    // same).  What may still be outstanding is everything issued after the activation part of tile t: the weight
    // tile of hand-over t-SA (unless that is tile t itself), and both tiles of the later hand-overs t-SA+1 .. t-2.
    auto wait_tile = [&](int t) {
        int cnt = 0;
        if (SW > SA && t - SA + SW < p.kt1) cnt += NLW;
#pragma unroll
        for (int hh = 1; hh <= SA - 2; hh++) {
            if (t + hh < p.kt1) cnt += n_a;
            if (t - SA + hh + SW < p.kt1) cnt += NLW;
        }
        wait_vmcnt_dyn(cnt);
    };

    f32x16 acc[NM][NU];
#pragma unroll
    for (int i = 0; i < NM; i++)
#pragma unroll
        for (int j = 0; j < NU; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    // prologue: the hand-overs a longer-running loop would have made before tile kt0; of the last one only the
    // activation part (a multiplying wavefront issues its weight part during the first half of tile kt0, see below)
    // (its first SW - SA hand-overs carry weight tiles only: the kernel issues those itself before it knows M)
#pragma unroll
    for (int h = -SW; h < -1; h++)
        if (h >= -SA || !p.w_pre) issue_for(p.kt0 + h);
    wait_tile(p.kt0);
    __builtin_amdgcn_s_barrier();
    if (NMI == 0) issue_for(p.kt0 - 1);
    else if (p.kt0 - 1 + SA < p.kt1) issue_a(p.kt0 - 1 + SA);

    // Ring positions, kept incrementally: a wavefront issues one instruction at a time and nothing else while it does,
    // so every scalar instruction between two MFMAs (a modulo, a guard, an address) is time the matrix pipe may
    // idle -- with more than about four of them per MFMA it does.
    int a_cur = (int)((unsigned)p.kt0 % SA) * A_STAGE;                   // stage of tile kt ...
    int a_nxt = a_cur + A_STAGE == SA * A_STAGE ? 0 : a_cur + A_STAGE;   // ... and of tile kt+1
    int w_cur = (int)((unsigned)p.kt0 % SW) * W_STAGE;
    int w_nxt = w_cur + W_STAGE == SW * W_STAGE ? 0 : w_cur + W_STAGE;
    int w_prv = w_cur == 0 ? (SW - 1) * W_STAGE : w_cur - W_STAGE;       // stage of tile kt-1 = of tile kt-1+SW
    const unsigned char* a_src = p.A + (size_t)(p.kt0 + SA) * ROW_BYTES;          // activation tile of hand-over kt
    const unsigned char* w_src = w_mine + (size_t)(p.kt0 - 1 + SW) * ROW_BYTES;   // weight tile of hand-over kt-1
    unsigned a_off[4 * MT];
#pragma unroll
    for (int l = 0; l < 4 * MT; l++) a_off[l] = (unsigned)min(a_row + 32 * l, p.M - 1) * row_pitch + a_chunk;

    bf16x8 fa[BK / 16][NM], fb[BK / 16][NU];
    // fragments of k-step KS of the tile whose stages start at A_ / W_: lane l reads tile row l%32, k-chunk
    // 2*KS + l/32, at its swizzled position
#define HS_FRAGS(A_, W_, KS)                                                                                     \
    if (NMI > 0) {                                                                                               \
        const unsigned char* sta_ = smem + (A_) + wave * TILE_BYTES + frag_row;                                  \
        const unsigned char* stw_ = smem + W_RING + (W_) + frag_row;                                             \
        const int pos_ = ((2 * (KS) + g) ^ fl) << 4;                                                             \
        _Pragma("unroll") for (int ni = 0; ni < NU; ni++)                                                        \
            fb[KS][ni] = *reinterpret_cast<const bf16x8*>(stw_ + ni * TILE_BYTES + pos_);                        \
        _Pragma("unroll") for (int mi = 0; mi < NMI; mi++)                                                       \
            fa[KS][mi] = *reinterpret_cast<const bf16x8*>(sta_ + mi * 4 * TILE_BYTES + pos_);                    \
    }
#define HS_MFMAS(KS)                                                                                             \
    _Pragma("unroll") for (int mi = 0; mi < NMI; mi++)                                                           \
        _Pragma("unroll") for (int ni = 0; ni < NU; ni++)                                                        \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[KS][mi], fb[KS][ni], acc[mi][ni], 0, 0, 0);
    // one MFMA, one fragment read, ... while there are reads; then the remaining MFMAs
#define HS_INTERLEAVE()                                                                                          \
    _Pragma("unroll") for (int i = 0; i < NMI + NU; i++) {                                                       \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                                       \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                                       \
    }                                                                                                            \
    __builtin_amdgcn_sched_group_barrier(0x008, NMI * NU - (NMI + NU) > 0 ? NMI * NU - (NMI + NU) : 0, 0);
    // Half a tile in a pinned order: k-steps KS0 and KS0+1 are multiplied; behind each MFMA come its share of the
    // fragment reads of k-steps (KS0+2)%4 and (KS0+3)%4 from the stages A_ / W_, and its share of the NLD loads
    // that LOAD(l) issues -- one after the other, because a wavefront that issues a dozen loads back to back
    // stalls on the address path while its matrix pipe runs dry.
#define HS_HALF(KS0, A_, W_, NLD, LOAD)                                                                          \
    {                                                                                                            \
        const unsigned char* sta_ = smem + (A_) + wave * TILE_BYTES + frag_row;                                  \
        const unsigned char* stw_ = smem + W_RING + (W_) + frag_row;                                             \
        constexpr int NMF = 2 * NM * NU;                                                                         \
        _Pragma("unroll") for (int q = 0; q < NMF; q++) {                                                        \
            const int ks = (KS0) + q / (NM * NU), kr = (ks + 2) % 4, mi = (q % (NM * NU)) / NU, ni = q % NU;     \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][mi], fb[ks][ni], acc[mi][ni], 0, 0, 0); \
            const int pos_ = ((2 * kr + g) ^ fl) << 4;                                                           \
            _Pragma("unroll") for (int r = (q % (NM * NU)) * (NU + NM) / (NM * NU);                              \
                                   r < (q % (NM * NU) + 1) * (NU + NM) / (NM * NU); r++) {                       \
                if (r < NU) fb[kr][r] = *reinterpret_cast<const bf16x8*>(stw_ + r * TILE_BYTES + pos_);          \
                else fa[kr][r - NU] = *reinterpret_cast<const bf16x8*>(sta_ + (r - NU) * 4 * TILE_BYTES + pos_); \
            }                                                                                                    \
            _Pragma("unroll") for (int l = q * (NLD) / NMF; l < (q + 1) * (NLD) / NMF; l++) { LOAD(l) }          \
            __builtin_amdgcn_sched_barrier(0);                                                                   \
        }                                                                                                        \
    }
    // the loads of a tile go out in two parts: the activation blocks of hand-over kt in the second half of tile kt,
    // the weight blocks of the same hand-over in the first half of tile kt+1 (same order as issue_for: the wait
    // counts do not change), so that they reach the address path evenly
#define HS_LOAD_A(l)                                                                                             \
    if ((l) < na_eff) load_to_lds_16(a_src, a_off[l], a_dst + (l) * 4096);
#define HS_LOAD_W_ONCE(l)                                                                                        \
    if (w_on) load_to_lds_16_stream(w_src, w_off[l], w_dst + (l) * 4096);
#define HS_LOAD_W_KEEP(l)                                                                                        \
    if (w_on) load_to_lds_16(w_src, w_off[l], w_dst + (l) * 4096);

    HS_FRAGS(a_cur, w_cur, 0)
    HS_FRAGS(a_cur, w_cur, 1)
    int kt = p.kt0;
    // One tile of the k-loop.  A compare and a branch in front of a load cost the matrix pipe about 17 clocks, so
    // the steady state (kt + SW < kt1: every load of both parts exists, the wait count is a constant) comes in two
    // forms: G = 0 for a wavefront whose activation slots are all live (no guard at all), G = 2 with one guard per
    // activation slot (issuing the dead slots anyway, re-reading row M-1, costs more than the guards).  G = 1: the
    // last SW-1 tiles before the final one, with every load guarded.
    // First half of tile kt: k-steps 0 and 1, the fragments of k-steps 2 and 3 of the same tile, and the weight
    // blocks of hand-over kt-1 (tile kt-1+SW, into the stage that tile kt-1 left), in two bursts.
    // Hand-over: every fragment read of tile kt has been issued; once they have returned (lgkmcnt) and all
    // wavefronts have met, the slots of tile kt are free to be refilled.  Tile kt+1 must have landed: each
    // wavefront waits for its own part before the barrier (a bare barrier: a fenced one would wait for the
    // tiles in flight as well).
    // Second half of tile kt: k-steps 2 and 3, the first two fragment sets of tile kt+1, and the activation
    // blocks of this hand-over (tile kt+SA, into the stage of tile kt).
#define HS_W_BURST(L0, L1)                                                                                       \
    if (w_on) {                                                                                                  \
        if (p.w_once) {                                                                                          \
            _Pragma("unroll") for (int l = (L0); l < (L1); l++)                                                  \
                load_to_lds_16_stream(w_src, w_off[l], w_dst + l * 4096);                                        \
        } else {                                                                                                 \
            _Pragma("unroll") for (int l = (L0); l < (L1); l++) load_to_lds_16(w_src, w_off[l], w_dst + l * 4096); \
        }                                                                                                        \
    }
#define HS_TILE(G)                                                                                               \
    {                                                                                                            \
        __builtin_amdgcn_sched_barrier(0);                                                                       \
        if (NMI > 0) {                                                                                           \
            const bool w_on = (G) == 1 ? kt - 1 + SW < p.kt1 : true;                                             \
            const unsigned w_dst = smem_off + W_RING + w_prv + wave * 1024;                                      \
            HS_FRAGS(a_cur, w_cur, 2)                                                                            \
            HS_MFMAS(0)                                                                                          \
            HS_INTERLEAVE()                                                                                      \
            __builtin_amdgcn_sched_barrier(0);                                                                   \
            HS_W_BURST(0, NLW / 2)                                                                               \
            __builtin_amdgcn_sched_barrier(0);                                                                   \
            HS_FRAGS(a_cur, w_cur, 3)                                                                            \
            HS_MFMAS(1)                                                                                          \
            HS_INTERLEAVE()                                                                                      \
            __builtin_amdgcn_sched_barrier(0);                                                                   \
            HS_W_BURST(NLW / 2, NLW)                                                                             \
            __builtin_amdgcn_sched_barrier(0);                                                                   \
        }                                                                                                        \
        if ((G) == 1) wait_tile(kt + 1);                                                                         \
        else HS_WAIT_VMCNT(SW > SA ? NLW : 0);                                                                   \
        __builtin_amdgcn_s_waitcnt((63 & 15) | ((63 >> 4) << 14) | (7 << 4) | (0 << 8)); /* lgkmcnt(0) */        \
        __builtin_amdgcn_s_barrier();                                                                            \
        if (NMI == 0) {                                                                                          \
            issue_for(kt);                                                                                       \
        } else {                                                                                                 \
            int na_eff = (G) == 0 ? 4 * MT : (G) == 2 ? n_a : (kt + SA < p.kt1 ? n_a : 0);                       \
            if (G) asm volatile("" : "+s"(na_eff)); /* one scalar compare per slot, not a mask expression */     \
            const unsigned a_dst = smem_off + a_cur + wave * 1024;                                               \
            HS_HALF(2, a_nxt, w_nxt, 4 * MT, HS_LOAD_A)                                                          \
        }                                                                                                        \
        a_cur = a_nxt;                                                                                           \
        a_nxt = a_nxt + A_STAGE == SA * A_STAGE ? 0 : a_nxt + A_STAGE;                                           \
        w_prv = w_cur;                                                                                           \
        w_cur = w_nxt;                                                                                           \
        w_nxt = w_nxt + W_STAGE == SW * W_STAGE ? 0 : w_nxt + W_STAGE;                                           \
        a_src += ROW_BYTES;                                                                                      \
        w_src += ROW_BYTES;                                                                                      \
    }
    static_assert(SA == 2, "the constant wait count of the steady state is written for a two-stage activation ring");
    if (n_a == 4 * MT) {
        for (; kt + SW < p.kt1; kt++) HS_TILE(0)
    } else {
        for (; kt + SW < p.kt1; kt++) HS_TILE(2)
    }
    for (; kt + 1 < p.kt1; kt++) HS_TILE(1)
    // last tile of the chunk: nothing follows it
    __builtin_amdgcn_sched_barrier(0);
    HS_FRAGS(a_cur, w_cur, 2)
    HS_MFMAS(0)
    HS_INTERLEAVE()
    __builtin_amdgcn_sched_barrier(0);
    HS_FRAGS(a_cur, w_cur, 3)
    HS_MFMAS(1)
    HS_INTERLEAVE()
    __builtin_amdgcn_sched_barrier(0);
    HS_MFMAS(2)
    HS_MFMAS(3)
#undef HS_FRAGS
#undef HS_MFMAS
#undef HS_INTERLEAVE
#undef HS_HALF
#undef HS_TILE
#undef HS_W_BURST
#undef HS_LOAD_A
#undef HS_LOAD_W_ONCE
#undef HS_LOAD_W_KEEP

    // Epilogue.  Accumulator element e of a 32x32 tile: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
    if (NMI > 0) {
        const int lr = 4 * (lane >> 5), lc = lane & 31;
#pragma unroll
        for (int mi = 0; mi < NMI; mi++) {
            const int row0 = p.m0 + 32 * (wave + 4 * mi) + lr;
            if (EPI == HS_EPI_SWIGLU_BF16) {
                // Lanes c (gate) and c+16 (up) hold the two pre-activations of output column c.  Elements are taken
                // in pairs: the gate lanes finish the row of element e and the up lanes the row of element e+1, so
                // every lane computes an output.  One v_permlane16_swap does the exchange: it swaps the odd
                // 16-lane rows of its first operand (element e: the up values) with the even rows of its second
                // (element e+1: the gate values), after which the first holds every lane's gate and the second
                // every lane's up.  (32-bit element offsets: the host checks that the output stays below 4 GiB.)
                bf16_t* C = reinterpret_cast<bf16_t*>(p.Cout);
                const bool up_lane = (lc & 16) != 0;
                const int rbase = row0 + (up_lane ? 1 : 0);
#pragma unroll
                for (int ni = 0; ni < NU; ni++) {
                    const int col = p.n0 + 16 * ni + (lc & 15);
#pragma unroll
                    for (int e = 0; e < 16; e += 2) {
                        const auto sw = __builtin_amdgcn_permlane16_swap(__float_as_uint(acc[mi][ni][e]),
                                                                         __float_as_uint(acc[mi][ni][e + 1]), false, false);
                        const float gate = __uint_as_float(sw[0]), up = __uint_as_float(sw[1]);
                        const int row = rbase + 8 * (e >> 2) + (e & 3);
                        if (col < p.N && row < p.M) {
                            const float s = gate * __builtin_amdgcn_rcpf(1.f + __expf(-gate));
                            C[(unsigned)row * (unsigned)p.N + (unsigned)col] = f32_to_bf16(s * up);
                        }
                    }
                }
            } else if (EPI == HS_EPI_ROWMAX) {
                // Each row's largest value among this workgroup's columns, as a key that orders by value and then by
                // lower column: first over the lane's NU columns, then over the 32 lanes that hold the row.
                unsigned long long* keys = reinterpret_cast<unsigned long long*>(p.Cout);
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    unsigned long long key = 0ull;
#pragma unroll
                    for (int ni = 0; ni < NU; ni++) {
                        const int col = p.n0 + 32 * ni + lc;
                        unsigned u = __float_as_uint(acc[mi][ni][e]);
                        u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
                        const unsigned long long k2 = ((unsigned long long)u << 32) | (0xFFFFFFFFu - (unsigned)col);
                        if (col < p.N && k2 > key) key = k2;
                    }
#pragma unroll
                    for (int o = 16; o > 0; o >>= 1) {
                        const unsigned lo = __shfl_xor((unsigned)key, o), hi = __shfl_xor((unsigned)(key >> 32), o);
                        const unsigned long long other = ((unsigned long long)hi << 32) | lo;
                        if (other > key) key = other;
                    }
                    const int row = row0 + 8 * (e >> 2) + (e & 3);
                    if (lc == 0 && row < p.M) keys[(size_t)row * p.n_groups + p.group] = key;
                }
            } else {
                float* C = PARTIAL ? p.part + (size_t)p.chunk * p.m_max * p.N : reinterpret_cast<float*>(p.Cout);
                // A row tile that lies wholly below M (all but the last one of a pass) is stored without row checks,
                // through a wavefront-uniform row pointer plus a 32-bit lane offset.
                const int tile_row = p.m0 + 32 * (wave + 4 * mi);
                unsigned char* tile = reinterpret_cast<unsigned char*>(C + (size_t)tile_row * p.N);
                const unsigned lane_bytes = ((unsigned)lr * (unsigned)p.N + (unsigned)(p.n0 + lc)) * 4u;
                if (tile_row + 32 <= p.M) {
#pragma unroll
                    for (int ni = 0; ni < NU; ni++) {
                        if (p.n0 + 32 * ni + lc >= p.N) continue;
#pragma unroll
                        for (int e = 0; e < 16; e++) {
                            unsigned char* rowp = tile + (size_t)(8 * (e >> 2) + (e & 3)) * p.N * 4;
                            float* dst = reinterpret_cast<float*>(rowp + (lane_bytes + 128u * ni));
                            if (!PARTIAL && EPI == HS_EPI_ADD_F32) *dst += acc[mi][ni][e];
                            else *dst = acc[mi][ni][e];
                        }
                    }
                } else {
#pragma unroll
                    for (int ni = 0; ni < NU; ni++) {
                        const int col = p.n0 + 32 * ni + lc;
                        if (col >= p.N) continue;
#pragma unroll
                        for (int e = 0; e < 16; e++) {
                            const int row = row0 + 8 * (e >> 2) + (e & 3);
                            if (row < p.M) {
                                float* dst = &C[(size_t)row * p.N + col];
                                if (!PARTIAL && EPI == HS_EPI_ADD_F32) *dst += acc[mi][ni][e];
                                else *dst = acc[mi][ni][e];
                            }
                        }
                    }
                }
            }
        }
    }
}

}  // namespace

// NU weight units per workgroup, MT row tiles per wavefront (128*MT rows per pass), SA / SW ring stages.
// (External linkage: the host takes the kernel's address to raise its dynamic LDS limit.)
template <int EPI, bool PARTIAL, int NU, int MT, int SA, int SW>
__global__ __launch_bounds__(256) void hs_gemm_stream(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                      const bf16_t* __restrict__ W2, void* __restrict__ Cout,
                                                      float* __restrict__ part, const int32_t* __restrict__ m_dev,
                                                      int m_max, int N, int K, int tpc, int n_groups, int n_pass) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const unsigned smem_off = (unsigned)(size_t)(lds_ptr_t)smem;
    constexpr int NCOLS = (EPI == HS_EPI_SWIGLU_BF16) ? 16 * NU : 32 * NU;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    stream_args p;
    p.M = *m_dev;
    p.A = reinterpret_cast<const unsigned char*>(A);
    p.wb[0] = reinterpret_cast<const unsigned char*>(W);
    p.wb[1] = reinterpret_cast<const unsigned char*>(EPI == HS_EPI_SWIGLU_BF16 ? W2 : W);
    p.Cout = Cout;
    p.part = part;
    p.m_max = m_max;
    p.N = N;
    p.K = K;
    // Workgroup id -> (weight group, row pass): ids are dealt round-robin to the 8 XCDs (each with its own L2).
    // Unsplit K: an XCD takes a weight group and runs its row passes back to back, so that the passes which stream
    // the same weight slab meet in one L2.
    // (With a single pass the id is the group: no padding of the grid, a workgroup that only exits still has to
    // wait for a compute unit with this kernel's LDS free.)
    int group = blockIdx.x, pass = 0, chunk = blockIdx.y;
    if (gridDim.y > 1) {
        // Split-K: the workgroups that land on one XCD (ids congruent mod 8) take consecutive (chunk, group, pass)
        // triples, pass fastest, i.e. one or two K chunks -- the slices of the activations they re-read then fit that
        // XCD's L2 (all chunks together, e.g. 8 MB for the down projection at 220 rows and 27 MB at 720, do not), and
        // the row passes that stream the same weight slice run side by side.  (grid.x = groups x passes, no padding.)
        const int total = gridDim.x * gridDim.y, id = blockIdx.x + gridDim.x * blockIdx.y;
        const int xcd = id & 7, slot = id >> 3;
        const int full = total >> 3, extra = total & 7;          // XCDs 0 .. extra-1 hold one workgroup more
        const int w = xcd * full + min(xcd, extra) + slot;
        chunk = w / (int)gridDim.x;
        const int rem = w - chunk * (int)gridDim.x;
        group = rem / n_pass;
        pass = rem - group * n_pass;
    } else if (n_pass > 1) {
        const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
        group = (local / n_pass) * 8 + xcd;
        pass = local % n_pass;
    }
    if (group >= n_groups) return;
    p.n0 = group * NCOLS;
    p.group = group;
    p.n_groups = n_groups;
    p.chunk = chunk;
    p.w_once = n_pass == 1;
    const int nk = K / BK;
    p.kt0 = chunk * tpc;
    p.kt1 = min(nk, p.kt0 + tpc);

    // Weight loader geometry: instruction j of wavefront w fills the 1 KB block (w + 4j) of a tile = rows 8w..8w+7
    // of unit j; lane i lands on row i/8, chunk position i%8 and therefore fetches chunk (i%8) ^ swz(row).  Rows
    // beyond N are clamped to the last valid row: their products are computed and never stored.
    // (32-bit byte offsets: the host checks that every operand stays below 4 GiB.)
    const int lrow = lane >> 3, lpos = lane & 7;
    unsigned w_off[NU];
#pragma unroll
    for (int j = 0; j < NU; j++) {
        const int row = 8 * wave + lrow;  // row within the unit
        const int gn = (EPI == HS_EPI_SWIGLU_BF16) ? p.n0 + 16 * j + 8 * (wave & 1) + lrow : p.n0 + 32 * j + row;
        w_off[j] = (unsigned)min(gn, N - 1) * (unsigned)(K * 2) + ((lpos ^ swz(row)) << 4);
    }

    // The weight-only hand-overs of the first chunk's prologue go out now: they do not depend on the row count,
    // whose load from device memory (first statement above) is still on its way -- nothing above has used it.
    {
        const unsigned char* w_mine = uniform_ptr((EPI == HS_EPI_SWIGLU_BF16 && wave >= 2) ? p.wb[1] : p.wb[0]);
#pragma unroll
        for (int h = -SW; h < -SA; h++)
            if (p.kt0 + h + SW < p.kt1) issue_weight_tile<NU, MT, SA, SW>(p, w_mine, smem_off, w_off, wave, p.kt0 + h + SW);
    }
    p.w_pre = 1;
    for (p.m0 = pass * 128 * MT; p.m0 < p.M; p.m0 += n_pass * 128 * MT) {
        int nmi = 0;
#pragma unroll
        for (int s = 0; s < MT; s++)
            if (p.m0 + 32 * (wave + 4 * s) < p.M) nmi = s + 1;
        nmi = __builtin_amdgcn_readfirstlane(nmi);
        if (nmi == 0) stream_chunk<EPI, PARTIAL, NU, MT, SA, SW, 0>(p, smem, smem_off, w_off, wave, lane);
        else if (nmi == 1) stream_chunk<EPI, PARTIAL, NU, MT, SA, SW, 1>(p, smem, smem_off, w_off, wave, lane);
        else if (MT >= 2 && nmi == 2)
            stream_chunk<EPI, PARTIAL, NU, MT, SA, SW, (MT >= 2 ? 2 : 1)>(p, smem, smem_off, w_off, wave, lane);
        else if (MT >= 3)
            stream_chunk<EPI, PARTIAL, NU, MT, SA, SW, (MT >= 3 ? 3 : 1)>(p, smem, smem_off, w_off, wave, lane);
        __syncthreads();  // the rings are reused by the next row pass
        p.w_pre = 0;
    }
    HS_WAIT_VMCNT(0);     // (a workgroup without rows leaves with its early weight loads landed)
}

namespace {

template <int EPI, bool PARTIAL, int NU, int MT, int SA, int SW>
void launch_stream(const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, float* part, const int32_t* m_dev,
                   int m_max, int n, int k, int chunks, int tpc, int rows_hint, hipStream_t st) {
    constexpr int NCOLS = (EPI == HS_EPI_SWIGLU_BF16) ? 16 * NU : 32 * NU;
    constexpr size_t lds = (size_t)(SA * 4 * MT + SW * NU) * TILE_BYTES;
    static_assert(lds <= 160 * 1024, "LDS of one compute unit");
    static_assert((SA - 1) * (4 * MT + NU) + NU <= 32, "wait counts");
    static bool configured = false;  // more than 64 KB of dynamic LDS has to be asked for once per kernel
    if (!configured) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&hs_gemm_stream<EPI, PARTIAL, NU, MT, SA, SW>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        configured = true;
    }
    // row passes in the grid: what the hint calls for (rows beyond are reached by the pass loop of the kernel)
    const int n_groups = (n + NCOLS - 1) / NCOLS;
    int n_pass = (rows_hint + 128 * MT - 1) / (128 * MT);
    if (n_pass < 1) n_pass = 1;
    if (n_pass > (m_max + 128 * MT - 1) / (128 * MT)) n_pass = (m_max + 128 * MT - 1) / (128 * MT);
    dim3 grid(chunks > 1 ? n_groups * n_pass : (n_pass > 1 ? ((n_groups + 7) / 8) * 8 * n_pass : n_groups), chunks);
    hipLaunchKernelGGL((hs_gemm_stream<EPI, PARTIAL, NU, MT, SA, SW>), grid, dim3(256), lds, st, a, w, w2, c, part,
                       m_dev, m_max, n, k, tpc, n_groups, n_pass);
}

#ifndef HS_WIDE_GROUP_ROWS
#define HS_WIDE_GROUP_ROWS 352   // measured cross-over at the 7B shape: 33 vs 40 us at 300 rows, 49 vs 37 us at 385
#endif

// Units per workgroup: the candidate that needs the fewest unit-times to cover the output on 256 compute units.
int choose_units(int units, int chunks) {
    int best = 4, best_cost = 1 << 30;
    for (int nu : {5, 4}) {
        const int wgs = ((units + nu - 1) / nu) * chunks;
        const int cost = ((wgs + 255) / 256) * nu;
        if (cost < best_cost) { best = nu; best_cost = cost; }
    }
    return best;
}

template <int EPI, bool PARTIAL>
void launch_stream_shape(const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, float* part,
                         const int32_t* m_dev, int m_max, int n, int k, int chunks, int tpc, int rows_hint,
                         hipStream_t st) {
    const int unit_cols = (EPI == HS_EPI_SWIGLU_BF16) ? 16 : 32;
    const int nu = choose_units((n + unit_cols - 1) / unit_cols, chunks);
    // Rows per pass: 256 leaves LDS for a deeper weight ring; 384 once the hint is within a factor 1.6 of 256 (the
    // row count of a speculative step swings by a third around its mean), so that a step above its average does
    // not pay a second pass over the weights.  Row tiles that do not exist cost nothing in either shape.
    const bool tall = rows_hint > 160;
#define HS_ARGS a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, rows_hint, st
    // The 64-row groups of the short-reduction split-K shapes (QKV, O) pay at a few hundred rows, where they halve the
    // partial sums; with many row passes every group re-reads the whole activation slab of its pass, and wider groups
    // (half as many re-reads) win.  The K chunking -- the reduction order -- is the shape's either way.
    if (PARTIAL && chunks > 1 && hs_gemm_narrow_groups(k) && rows_hint < HS_WIDE_GROUP_ROWS) {
        if (tall) launch_stream<EPI, PARTIAL, 2, 3, 2, 6>(HS_ARGS);
        else launch_stream<EPI, PARTIAL, 2, 2, 2, 8>(HS_ARGS);
    } else if (nu == 5) {
        if (tall) launch_stream<EPI, PARTIAL, 5, 3, 2, 3>(HS_ARGS);
        else launch_stream<EPI, PARTIAL, 5, 2, 2, 4>(HS_ARGS);
    } else {
        if (tall) launch_stream<EPI, PARTIAL, 4, 3, 2, 4>(HS_ARGS);
        else launch_stream<EPI, PARTIAL, 4, 2, 2, 5>(HS_ARGS);
    }
#undef HS_ARGS
}

}  // namespace

int hs_gemm_rowmax_groups(int n) {
    const int nu = choose_units((n + 31) / 32, 1);
    return (n + 32 * nu - 1) / (32 * nu);
}

void hs_launch_gemm_stream(int epi, const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, float* part,
                           const int32_t* m_dev, int m_max, int n, int k, int chunks, int tpc, int rows_hint,
                           hipStream_t st) {
#define HS_ARGS a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, rows_hint, st
    if (epi == HS_EPI_SWIGLU_BF16) {
        launch_stream_shape<HS_EPI_SWIGLU_BF16, false>(HS_ARGS);
    } else if (chunks > 1) {
        // partial sums: the ordered reduce applies the epilogue
        launch_stream_shape<HS_EPI_STORE_F32, true>(HS_ARGS);
    } else if (epi == HS_EPI_ROWMAX) {
        launch_stream_shape<HS_EPI_ROWMAX, false>(HS_ARGS);
    } else if (epi == HS_EPI_ADD_F32) {
        launch_stream_shape<HS_EPI_ADD_F32, false>(HS_ARGS);
    } else {
        launch_stream_shape<HS_EPI_STORE_F32, false>(HS_ARGS);
    }
#undef HS_ARGS
}
