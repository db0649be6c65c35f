// bf16 MFMA GEMMs for the dense projections of the verify forward pass (QKV, O, gate/up with SwiGLU epilogue,
// down, LM head):  C[M,N] (+)= A[M,K] . W[N,K]^T,  both operands K-contiguous, fp32 accumulation.
//
// Layout on gfx950: a workgroup of 4 wavefronts owns a BM x 128 output tile (BM = 64 * MI; 128 is what runs);
// each wavefront a (BM/2) x 64 quadrant as (BM/64) x 2 v_mfma_f32_32x32x16_bf16 tiles.  The operand tiles, 64
// deep in K, travel from global memory straight into LDS (global_load_lds_dwordx4: no staging registers) through
// two rings: activations, which come from L2 with a short latency, are double-buffered; weights, which stream from
// HBM exactly once, get SW stages, so that SW-1 weight tiles per workgroup are in flight while one is being
// multiplied.  At a few hundred rows these GEMMs live on weight bytes in flight and on every workgroup of the grid
// being resident at once (80 KB of LDS per workgroup: two per compute unit), not on matrix-core rate.  The
// load writes lane i's 16 bytes at LDS offset 16*i of a wavefront-uniform base, so a tile row is 128 unpadded
// bytes; bank conflicts of the fragment reads are avoided by an XOR swizzle of the 16-byte chunk index with bits of
// the row index, applied on the global side (which chunk a lane fetches).
//
// Reduction order.  K is cut into a fixed number of chunks that depends only on the GEMM's shape (N, K).  Each
// chunk is accumulated by the matrix cores on its own, and the chunk sums are added left to right in fp32.  This
// one definition is executed in two ways that give bit-identical results: "serial" (one workgroup walks all
// chunks, folding each finished chunk into a running total) and "split" (one workgroup per chunk writes its
// partial sum, a second kernel adds the partials in the same order), the latter where a row-tile grid alone
// cannot fill 256 compute units.  Which one runs, and which row-tile height, are pure performance choices steered
// by the caller's row hint; a row's result never depends on how many other rows share the launch (this is what
// makes speculative and one-token decoding agree bit for bit).
//
// The row count M lives on the device (number of draft-tree rows of this step).  The grid holds as many row tiles
// as the host-side row hint suggests; a workgroup walks row tiles with that stride until it passes M, so any M up
// to m_max is covered whatever the hint was.  Workgroup ids are spread so that all row tiles that read the same
// W tile run on the same XCD (ids are dealt round-robin to the 8 XCDs, each with its own L2).
#include "hs_gemm_common.h"

using namespace hs_gemm_detail;

namespace {

enum { MODE_PLAIN = 0, MODE_SERIAL = 1, MODE_SPLIT = 2 };

}  // namespace

// MI x NI = 32x32 MFMA tiles per wavefront: the workgroup tile is BM = 64 * MI rows by BN = 64 * NI weight rows.
// SW = stages of the weight ring (the activation ring has two).
// (External linkage: the host takes the kernel's address to raise its dynamic LDS limit.)
template <int EPI, int MODE, int MI, int NI, int SW>
__global__ __launch_bounds__(256) void hs_gemm_bf16_mfma(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                       const bf16_t* __restrict__ W2, void* __restrict__ Cout,
                                                       float* __restrict__ part, const int32_t* __restrict__ m_dev,
                                                       int m_max, int N, int K, int m_tiles, int n_tiles,
                                                       int tiles_per_chunk) {
    constexpr int BM = 64 * MI, BN = 64 * NI;
    constexpr int NLA = BM / 32;        // 1 KB load instructions per wavefront and k-tile for the A tile
    constexpr int NLB = BN / 32;        // ... and for the W tile
    constexpr int SA = 2;
    constexpr int A_BYTES = BM * ROW_BYTES, W_BYTES = BN * ROW_BYTES;
    constexpr int W_RING = SA * A_BYTES;  // byte offset of the weight ring
    static_assert(SW == 2 || SW == 3, "the wait counts below cover two or three weight stages");
    static_assert(MODE != MODE_SERIAL || MI * NI <= 4, "the serial execution keeps a second set of accumulators");
    static_assert(EPI != HS_EPI_SWIGLU_BF16 || NI % 2 == 0, "gate and up tiles come in pairs");
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    // LDS byte offset of the ring (what M0 carries): the 32-bit value of the pointer in the LDS address space
    const unsigned smem_off = (unsigned)(size_t)(lds_ptr_t)smem;

    const int M = *m_dev;
    // XCD-aware tile assignment: id -> (xcd, local); an XCD walks its column tiles with the row tile running
    // fastest, so the row tiles that share a weight tile run together on one L2.
    const int id = blockIdx.x;
    const int xcd = id & 7, local = id >> 3;
    const int n_tile = (local / m_tiles) * 8 + xcd;
    const int m_first = local % m_tiles;
    if (n_tile >= n_tiles) return;
    // SwiGLU: the tile's BN weight rows are BN/2 gate rows followed by the BN/2 up rows of the same output columns.
    constexpr int NCOLS = (EPI == HS_EPI_SWIGLU_BF16) ? BN / 2 : BN;
    const int n0 = n_tile * NCOLS;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    const int nk = K / BK;
    int kt0 = 0, kt1 = nk;
    if (MODE == MODE_SPLIT) {
        kt0 = blockIdx.y * tiles_per_chunk;
        kt1 = min(nk, kt0 + tiles_per_chunk);
    }

    // Load geometry: instruction j of wavefront w fills the 1 KB block (4j + w) of a tile = its rows 8(4j+w)..+7;
    // lane i lands on row i/8, chunk position i%8 and therefore fetches chunk (i%8) ^ swz(row).  Rows beyond M
    // (or N) are clamped to the last valid row: their products are computed and never stored.
    const int lrow = lane >> 3, lpos = lane & 7;
    // (32-bit byte offsets: the largest matrix of the supported shapes, vocab x d_model bf16, stays below 4 GiB;
    // the host checks it.)
    unsigned b_off[NLB];
    const unsigned char* b_base[NLB];
#pragma unroll
    for (int j = 0; j < NLB; j++) {
        const int r = (4 * j + wave) * 8 + lrow;
        int gn = n0 + r;
        b_base[j] = reinterpret_cast<const unsigned char*>(W);
        if (EPI == HS_EPI_SWIGLU_BF16) {
            gn = n0 + (r % (BN / 2));
            if ((4 * j + wave) * 8 >= BN / 2) b_base[j] = reinterpret_cast<const unsigned char*>(W2);  // uniform
        }
        b_off[j] = (unsigned)min(gn, N - 1) * (unsigned)(K * 2) + ((lpos ^ swz(r)) << 4);
    }

    // Fragment geometry: lane l reads tile row (row0 + l%32), k-chunk 2*ks + l/32, at its swizzled position.
    const int l32 = lane & 31, g = lane >> 5, fl = swz(l32);
    const int a_frag = (wm * (BM / 2) + l32) * ROW_BYTES;
    // weight tile ni of this wavefront: SwiGLU keeps NI/2 gate tiles then the NI/2 up tiles of the same columns
    int b_frag[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ni++) {
        const int trow = (EPI == HS_EPI_SWIGLU_BF16)
                             ? ((ni < NI / 2 ? 0 : BN / 2) + wn * (16 * NI) + 32 * (ni % (NI / 2 > 0 ? NI / 2 : 1)))
                             : (wn * (32 * NI) + 32 * ni);
        b_frag[ni] = (trow + l32) * ROW_BYTES;
    }

    for (int m_tile = m_first; m_tile * BM < M; m_tile += m_tiles) {
        const int m0 = m_tile * BM;
        unsigned a_off[NLA];
#pragma unroll
        for (int j = 0; j < NLA; j++) {
            const int r = (4 * j + wave) * 8 + lrow;
            a_off[j] = (unsigned)min(m0 + r, M - 1) * (unsigned)(K * 2) + ((lpos ^ swz(r)) << 4);
        }
#define HS_ISSUE_A(KT, SLOT)                                                                                     \
    {                                                                                                            \
        const unsigned dst_ = smem_off + (SLOT) * A_BYTES + wave * 1024;                                         \
        const unsigned char* base_ = reinterpret_cast<const unsigned char*>(A) + (size_t)(KT) * ROW_BYTES;       \
        _Pragma("unroll") for (int j = 0; j < NLA; j++) load_to_lds_16(base_, a_off[j], dst_ + j * 4096);        \
    }
#define HS_ISSUE_W(KT, SLOT)                                                                                     \
    {                                                                                                            \
        const unsigned dst_ = smem_off + W_RING + (SLOT) * W_BYTES + wave * 1024;                                \
        const size_t koff_ = (size_t)(KT) * ROW_BYTES;                                                           \
        _Pragma("unroll") for (int j = 0; j < NLB; j++) load_to_lds_16(b_base[j] + koff_, b_off[j], dst_ + j * 4096); \
    }

        f32x16 acc[MI][NI], total[MODE == MODE_SERIAL ? MI : 1][MODE == MODE_SERIAL ? NI : 1];
#pragma unroll
        for (int i = 0; i < MI; i++)
#pragma unroll
            for (int j = 0; j < NI; j++)
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    acc[i][j][e] = 0.f;
                    if (MODE == MODE_SERIAL) total[i][j][e] = 0.f;
                }

        // Prologue: activation tile kt0 and weight tiles kt0 .. kt0+SW-2 in flight.  Issue order matters for the
        // wait counts below: in every iteration the activation tile goes first, then the weight tile.
        HS_ISSUE_A(kt0, 0)
#pragma unroll
        for (int s = 0; s < SW - 1; s++)
            if (kt0 + s < kt1) HS_ISSUE_W(kt0 + s, s)

        int slot_a = 0, slot_w = 0;
        for (int kt = kt0; kt < kt1; kt++) {
            // Loads complete in issue order, and the last loads issued before this point are activation tile kt
            // followed by weight tile kt+SW-2 (if there is one).  So tile kt of both operands has landed once at
            // most that one weight tile is outstanding.  (The in-order rule also means that a third weight stage
            // is the deepest that pays: waiting for the young activation tile drains every older weight tile.)
            if (SW > 2 && kt + SW - 2 < kt1) {
                HS_WAIT_VMCNT(NLB);
            } else {
                HS_WAIT_VMCNT(0);
            }
            // Bare barrier: a fenced one would wait for every outstanding load, the tiles in flight included.
            // Everyone's part of tile kt is in LDS (each wavefront waited for its own loads above), and everyone
            // is done reading tile kt-1, whose slots are refilled next.
            __builtin_amdgcn_s_barrier();
            if (kt + 1 < kt1) HS_ISSUE_A(kt + 1, slot_a ^ 1)
            if (kt + SW - 1 < kt1) HS_ISSUE_W(kt + SW - 1, (slot_w == 0) ? SW - 1 : slot_w - 1)
            const unsigned char* sta = smem + slot_a * A_BYTES;
            const unsigned char* stw = smem + W_RING + slot_w * W_BYTES;
            // Fragment reads run two k-steps (of 16) ahead of the matrix cores: the first MFMAs start as soon as
            // their operands arrive and the rest of the LDS latency hides behind them.
            bf16x8 fa[BK / 16][MI], fb[BK / 16][NI];
#define HS_FRAGS(KS)                                                                                             \
    {                                                                                                            \
        const int pos_ = ((2 * (KS) + g) ^ fl) << 4;                                                             \
        _Pragma("unroll") for (int ni = 0; ni < NI; ni++)                                                        \
            fb[KS][ni] = *reinterpret_cast<const bf16x8*>(stw + b_frag[ni] + pos_);                              \
        _Pragma("unroll") for (int mi = 0; mi < MI; mi++)                                                        \
            fa[KS][mi] = *reinterpret_cast<const bf16x8*>(sta + a_frag + mi * 32 * ROW_BYTES + pos_);            \
    }
            HS_FRAGS(0)
            HS_FRAGS(1)
#pragma unroll
            for (int ks = 0; ks < BK / 16; ks++) {
                if (ks + 2 < BK / 16) HS_FRAGS(ks + 2)
                __builtin_amdgcn_sched_barrier(0);  // keep the reads ahead of the matrix-core block
#pragma unroll
                for (int mi = 0; mi < MI; mi++)
#pragma unroll
                    for (int ni = 0; ni < NI; ni++)
                        acc[mi][ni] =
                            __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[ks][mi], fb[ks][ni], acc[mi][ni], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
#undef HS_FRAGS
            if (MODE == MODE_SERIAL) {
                // end of a chunk: fold its sum into the running total (left-to-right chunk order)
                if ((kt + 1) % tiles_per_chunk == 0 || kt + 1 == nk) {
#pragma unroll
                    for (int i = 0; i < MI; i++)
#pragma unroll
                        for (int j = 0; j < NI; j++)
#pragma unroll
                            for (int e = 0; e < 16; e++) {
                                total[i][j][e] += acc[i][j][e];
                                acc[i][j][e] = 0.f;
                            }
                }
            }
            slot_a ^= 1;
            slot_w = (slot_w + 1 == SW) ? 0 : slot_w + 1;
        }
#undef HS_ISSUE_A
#undef HS_ISSUE_W

        // Epilogue.  Accumulator element e of a 32x32 tile: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
        const int lr = 4 * (lane >> 5), lc = lane & 31;
        if (EPI == HS_EPI_SWIGLU_BF16) {
            bf16_t* C = reinterpret_cast<bf16_t*>(Cout);
#pragma unroll
            for (int t = 0; t < NI / 2; t++) {
                const int col = n0 + wn * (16 * NI) + 32 * t + lc;
                if (col >= N) continue;
#pragma unroll
                for (int mi = 0; mi < MI; mi++)
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        int row = m0 + wm * (BM / 2) + mi * 32 + 8 * (e >> 2) + lr + (e & 3);
                        if (row < M) {
                            float gt = acc[mi][t][e], u = acc[mi][t + NI / 2][e];
                            float s = gt / (1.f + __expf(-gt));
                            C[(size_t)row * N + col] = f32_to_bf16(s * u);
                        }
                    }
            }
        } else {
            float* C =
                (MODE == MODE_SPLIT) ? part + (size_t)blockIdx.y * m_max * N : reinterpret_cast<float*>(Cout);
#pragma unroll
            for (int mi = 0; mi < MI; mi++)
#pragma unroll
                for (int ni = 0; ni < NI; ni++) {
                    const int col = n0 + wn * (32 * NI) + ni * 32 + lc;
                    if (col >= N) continue;
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        int row = m0 + wm * (BM / 2) + mi * 32 + 8 * (e >> 2) + lr + (e & 3);
                        if (row < M) {
                            float v = (MODE == MODE_SERIAL) ? total[MODE == MODE_SERIAL ? mi : 0][MODE == MODE_SERIAL ? ni : 0][e]
                                                             : acc[mi][ni][e];
                            float* p = &C[(size_t)row * N + col];
                            if (MODE != MODE_SPLIT && EPI == HS_EPI_ADD_F32) *p += v;
                            else *p = v;
                        }
                    }
                }
        }
        __syncthreads();  // the ring is reused by the next row tile
    }
}

namespace {

// Second pass of the split execution: add the chunk partials left to right, then store or add to the residual.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_split_reduce(const float* __restrict__ part, float* __restrict__ C,
                                                          const int32_t* __restrict__ m_dev, int m_max, int N,
                                                          int chunks) {
    const int c4 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c4 >= N) return;
    const int M = *m_dev;
    for (int row = blockIdx.y; row < M; row += gridDim.y) {
        const size_t off = (size_t)row * N + c4, stride = (size_t)m_max * N;
        float4 t = *reinterpret_cast<const float4*>(part + off);
        for (int s = 1; s < chunks; s++) {
            float4 p = *reinterpret_cast<const float4*>(part + s * stride + off);
            t.x += p.x; t.y += p.y; t.z += p.z; t.w += p.w;
        }
        float4* dst = reinterpret_cast<float4*>(C + off);
        if (EPI == HS_EPI_ADD_F32) {
            float4 o = *dst;
            o.x += t.x; o.y += t.y; o.z += t.z; o.w += t.w;
            *dst = o;
        } else {
            *dst = t;
        }
    }
}

// Plain kernel for debugging: one thread per output element, sequential fp32 dot product.
template <int EPI>
__global__ void gemm_bf16_plain(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                const bf16_t* __restrict__ W2, void* __restrict__ Cout,
                                const int32_t* __restrict__ m_dev, int N, int K) {
    const int M = *m_dev;
    int col = blockIdx.x * blockDim.x + threadIdx.x;
    int row = blockIdx.y;
    if (row >= M || col >= N) return;
    const bf16_t* a = A + (size_t)row * K;
    const bf16_t* w = W + (size_t)col * K;
    float s = 0.f;
    for (int k = 0; k < K; k++) s += bf16_to_f32(a[k]) * bf16_to_f32(w[k]);
    if (EPI == HS_EPI_SWIGLU_BF16) {
        const bf16_t* w2 = W2 + (size_t)col * K;
        float u = 0.f;
        for (int k = 0; k < K; k++) u += bf16_to_f32(a[k]) * bf16_to_f32(w2[k]);
        float g = s / (1.f + __expf(-s));
        reinterpret_cast<bf16_t*>(Cout)[(size_t)row * N + col] = f32_to_bf16(g * u);
    } else if (EPI == HS_EPI_ADD_F32) {
        reinterpret_cast<float*>(Cout)[(size_t)row * N + col] += s;
    } else {
        reinterpret_cast<float*>(Cout)[(size_t)row * N + col] = s;
    }
}

template <int EPI, int MODE, int MI, int NI, int SW>
void launch_tile(const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, float* part, const int32_t* m_dev,
                 int m_max, int n, int k, int chunks, int tpc, int rows_hint, hipStream_t st) {
    constexpr int BM = 64 * MI, BN = 64 * NI;
    constexpr int NCOLS = (EPI == HS_EPI_SWIGLU_BF16) ? BN / 2 : BN;
    constexpr size_t lds = (size_t)(2 * BM + SW * BN) * ROW_BYTES;
    static bool configured = false;  // more than 64 KB of dynamic LDS has to be asked for once per kernel
    if (!configured) {
        hipFuncSetAttribute(reinterpret_cast<const void*>(&hs_gemm_bf16_mfma<EPI, MODE, MI, NI, SW>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        configured = true;
    }
    // Row tiles in the grid: what the hint calls for, with an eighth of margin once there is more than one row
    // per sequence (the row count swings from step to step).  Not more: a workgroup of this kernel holds 80-160 KB
    // of LDS and is not free to dispatch even if it exits at once -- 256 unused ones cost 10 us.  Rows beyond the
    // grid are reached by the grid-stride loop of the kernel.
    const int m_tiles_all = (m_max + BM - 1) / BM;
    int m_main = MI == 2 && rows_hint <= BM ? 1 : (rows_hint + rows_hint / 8 + BM - 1) / BM;
    if (m_main < 1) m_main = 1;
    if (m_main > m_tiles_all) m_main = m_tiles_all;
    const int m_tiles = m_main;
    const int n_tiles = (n + NCOLS - 1) / NCOLS;
    const int blocks = ((n_tiles + 7) / 8) * m_tiles * 8;
    dim3 grid(blocks, MODE == MODE_SPLIT ? chunks : 1);
    hipLaunchKernelGGL((hs_gemm_bf16_mfma<EPI, MODE, MI, NI, SW>), grid, dim3(256), lds, st, a, w, w2, c, part, m_dev, m_max,
                       n, k, m_tiles, n_tiles, tpc);
}

template <int EPI>
void launch(const hs_ctx* ctx, const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, const int32_t* m_dev,
            int m_max, int n, int k, int rows_hint, hipStream_t st, int* pending) {
    if (pending) *pending = 0;
    if (ctx->flags & HS_FLAG_REFERENCE_KERNELS) {
        dim3 grid((n + 255) / 256, m_max);
        hipLaunchKernelGGL(gemm_bf16_plain<EPI>, grid, dim3(256), 0, st, a, w, w2, c, m_dev, n, k);
        return;
    }
    const int nk = k / BK;
    int chunks = (EPI == HS_EPI_SWIGLU_BF16) ? 1 : hs_gemm_chunks(n, k);
    const int tpc = (nk + chunks - 1) / chunks;
    chunks = (nk + tpc - 1) / tpc;  // no empty chunk
    float* part = reinterpret_cast<float*>(ctx->ws + ctx->lay.gemm_part);
    if (rows_hint <= HS_GEMM_STREAM_MAX_ROWS) {
        // few rows: the projection is a weight stream; one workgroup holds all rows against its weight slab
        hs_launch_gemm_stream(EPI, a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, rows_hint, st);
        if (chunks > 1) {
            if (pending) {
                *pending = chunks;
            } else {
                const int rows = rows_hint < 1 ? 1 : (2 * rows_hint > m_max ? m_max : 2 * rows_hint);
                hipLaunchKernelGGL((gemm_split_reduce<EPI>), dim3((n / 4 + 255) / 256, rows), dim3(256), 0, st, part,
                                   reinterpret_cast<float*>(c), m_dev, m_max, n, chunks);
            }
        }
        return;
    }
    // Launch shape from the row hint.  Tile height: 128 rows while all rows fit one tile, else 256.  Tile width:
    // 256 weight rows where the output is wide enough to put a workgroup on every compute unit anyway (the wider
    // tile re-reads half as many activation bytes per weight byte), else 128.  Narrow outputs run split over K
    // while the row tiles alone would leave compute units idle.
    const bool tall = rows_hint > 128;
#define HS_ARGS a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, rows_hint, st
    if constexpr (EPI == HS_EPI_SWIGLU_BF16) {
        if (tall) launch_tile<EPI, MODE_PLAIN, 4, 4, 3>(HS_ARGS);
        else launch_tile<EPI, MODE_PLAIN, 2, 4, 3>(HS_ARGS);
    } else if (chunks == 1) {
        if (tall) launch_tile<EPI, MODE_PLAIN, 4, 4, 3>(HS_ARGS);
        else launch_tile<EPI, MODE_PLAIN, 2, 4, 3>(HS_ARGS);
    } else if (rows_hint > 512) {
        launch_tile<EPI, MODE_SERIAL, 2, 2, 3>(HS_ARGS);
    } else {
        const int n128 = (n + 127) / 128;
        const int m_tiles = tall ? (rows_hint + 255) / 256 : 1;
        // workgroups that can be resident at once: two per compute unit with the 128 x 128 tile, else one
        const bool wide = n128 * chunks * m_tiles > (tall ? 256 : 512);
        if (tall) {
            if (wide) launch_tile<EPI, MODE_SPLIT, 4, 4, 3>(HS_ARGS);
            else launch_tile<EPI, MODE_SPLIT, 4, 2, 3>(HS_ARGS);
        } else {
            if (wide) launch_tile<EPI, MODE_SPLIT, 2, 4, 3>(HS_ARGS);
            else launch_tile<EPI, MODE_SPLIT, 2, 2, 3>(HS_ARGS);
        }
        if (pending) {
            *pending = chunks;
        } else {
            int rows = rows_hint < 1 ? 1 : (2 * rows_hint > m_max ? m_max : 2 * rows_hint);
            hipLaunchKernelGGL((gemm_split_reduce<EPI>), dim3((n / 4 + 255) / 256, rows), dim3(256), 0, st, part,
                               reinterpret_cast<float*>(c), m_dev, m_max, n, chunks);
        }
    }
#undef HS_ARGS
}

}  // namespace

// Number of K chunks of a projection: a function of the shape alone.  Narrow outputs get as many chunks as put
// about one workgroup of the weight-streaming execution (128 weight rows each) on every one of the 256 compute
// units; every chunk keeps at least 4 k-tiles.
int hs_gemm_chunks(int n, int k) {
    const int groups = (n + 127) / 128;
    int chunks = 256 / groups;
    const int nk = k / BK;
    if (chunks > nk / 4) chunks = nk / 4;
    if (chunks < 1) chunks = 1;
    return chunks;
}

void hs_launch_gemm(const hs_ctx* ctx, int epi, const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c,
                    const int32_t* m_dev, int m_max, int n, int k, int rows_hint, hipStream_t st, int* pending) {
    switch (epi) {
        case HS_EPI_STORE_F32:
            launch<HS_EPI_STORE_F32>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st, pending);
            break;
        case HS_EPI_ADD_F32:
            launch<HS_EPI_ADD_F32>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st, pending);
            break;
        default:
            launch<HS_EPI_SWIGLU_BF16>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st, pending);
            break;
    }
}
