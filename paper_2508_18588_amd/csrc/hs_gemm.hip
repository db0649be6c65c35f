// bf16 MFMA GEMMs for the dense projections of the verify forward pass (QKV, O, gate/up with SwiGLU epilogue,
// down, LM head):  C[M,N] (+)= A[M,K] . W[N,K]^T,  both operands K-contiguous, fp32 accumulation.
//
// Layout on gfx950: a workgroup of 4 wavefronts owns a BM x 128 output tile, BM = 128 or 256; each wavefront a
// (BM/2) x 64 quadrant as (BM/64) x 2 v_mfma_f32_32x32x16_bf16 tiles.  A and W tiles (64 deep in K) are staged
// through LDS with a padded row stride.  The weight stream comes from HBM and is kept two k-tiles ahead in
// registers; the activations come from L2 and are kept one k-tile ahead.  The 256-row tile reads every weight once
// for up to 256 rows -- the shape of a verify step with a few draft tokens per sequence, which is weight-streaming
// bound -- the 128-row tile serves one-token decoding (rows = sequences).
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
// The row count M lives on the device (number of draft-tree rows of this step); the grid covers m_max rows and
// workgroups whose rows start beyond M exit at once.  Workgroup ids are spread so that all M-tiles that read the
// same W-tile run on the same XCD (ids are dealt round-robin to the 8 XCDs, each with its own L2).
#include "hs_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // plain vector: stays in registers

namespace {

constexpr int BN = 128, BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // bf16 elements; 144-byte rows keep 16-byte reads conflict-free

enum { MODE_PLAIN = 0, MODE_SERIAL = 1, MODE_SPLIT = 2 };

// MI = 32-row MFMA tiles per wavefront in M: the workgroup tile is BM = 64 * MI rows.
template <int EPI, int MODE, int MI>
__global__ __launch_bounds__(256) void gemm_bf16_mfma(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                       const bf16_t* __restrict__ W2, void* __restrict__ Cout,
                                                       float* __restrict__ part, const int32_t* __restrict__ m_dev,
                                                       int m_max, int N, int K, int m_tiles, int n_tiles,
                                                       int tiles_per_chunk) {
    constexpr int BM = 64 * MI;
    constexpr int NA = BM / 32;  // 16-byte A chunks per thread and k-tile
    __shared__ __attribute__((aligned(16))) bf16_t sA[BM * LDS_STRIDE];
    __shared__ __attribute__((aligned(16))) bf16_t sB[BN * LDS_STRIDE];

    const int M = *m_dev;
    // XCD-aware tile assignment: id -> (xcd, local); an XCD walks its N-tiles, M fastest.
    const int id = blockIdx.x;
    const int xcd = id & 7, local = id >> 3;
    const int n_tile = (local / m_tiles) * 8 + xcd;
    const int m_tile = local % m_tiles;
    if (n_tile >= n_tiles) return;
    const int m0 = m_tile * BM;
    if (m0 >= M) return;
    // SwiGLU: the tile's 128 B-rows are 64 gate rows followed by the 64 up rows of the same output columns.
    constexpr int NCOLS = (EPI == HS_EPI_SWIGLU_BF16) ? 64 : 128;
    const int n0 = n_tile * NCOLS;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    const int nk = K / BK;
    int kt0 = 0, kt1 = nk;
    if (MODE == MODE_SPLIT) {
        kt0 = blockIdx.y * tiles_per_chunk;
        kt1 = min(nk, kt0 + tiles_per_chunk);
    }

    // Rows beyond M (or N) are clamped to the last valid row: their products are computed and never stored, so
    // every load is unconditional and the prefetch stays in registers.
    u32x4 ra[NA], rb0[4], rb1[4];
    const bf16_t* a_ptr[NA];
    const bf16_t* b_ptr[4];
    int sa_off[NA], sb_off[4];
#pragma unroll
    for (int i = 0; i < NA; i++) {
        int c = tid + 256 * i;
        int r = c >> 3, c8 = (c & 7) * 8;
        sa_off[i] = r * LDS_STRIDE + c8;
        a_ptr[i] = A + (size_t)min(m0 + r, M - 1) * K + c8;
    }
#pragma unroll
    for (int i = 0; i < 4; i++) {
        int c = tid + 256 * i;
        int r = c >> 3, c8 = (c & 7) * 8;
        sb_off[i] = r * LDS_STRIDE + c8;
        int gn;
        const bf16_t* wsrc = W;
        if (EPI == HS_EPI_SWIGLU_BF16) {
            gn = n0 + (r & 63);
            if (r >= 64) wsrc = W2;
        } else {
            gn = n0 + r;
        }
        b_ptr[i] = wsrc + (size_t)min(gn, N - 1) * K + c8;
    }
#define HS_FETCH_A(KT)                                                                     \
    _Pragma("unroll") for (int i = 0; i < NA; i++)                                         \
        ra[i] = *reinterpret_cast<const u32x4*>(a_ptr[i] + (size_t)(KT) * BK);
#define HS_FETCH_B(RB, KT)                                                                 \
    _Pragma("unroll") for (int i = 0; i < 4; i++)                                          \
        RB[i] = *reinterpret_cast<const u32x4*>(b_ptr[i] + (size_t)(KT) * BK);
#define HS_STAGE(RB)                                                                       \
    _Pragma("unroll") for (int i = 0; i < NA; i++)                                         \
        *reinterpret_cast<u32x4*>(&sA[sa_off[i]]) = ra[i];                                 \
    _Pragma("unroll") for (int i = 0; i < 4; i++)                                          \
        *reinterpret_cast<u32x4*>(&sB[sb_off[i]]) = RB[i];

    f32x16 acc[MI][2], total[MI][2];
#pragma unroll
    for (int i = 0; i < MI; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) {
                acc[i][j][e] = 0.f;
                if (MODE == MODE_SERIAL) total[i][j][e] = 0.f;
            }

    const int arow = wm * (BM / 2) + (lane & 31);
    const int brow0 = (EPI == HS_EPI_SWIGLU_BF16) ? (wn * 32 + (lane & 31)) : (wn * 64 + (lane & 31));
    const int brow1 = (EPI == HS_EPI_SWIGLU_BF16) ? (64 + wn * 32 + (lane & 31)) : (wn * 64 + 32 + (lane & 31));
    const int koff = (lane >> 5) * 8;

#define HS_COMPUTE(KT)                                                                                      \
    _Pragma("unroll") for (int ks = 0; ks < BK / 16; ks++) {                                                \
        bf16x8 fb0 = *reinterpret_cast<const bf16x8*>(&sB[brow0 * LDS_STRIDE + ks * 16 + koff]);            \
        bf16x8 fb1 = *reinterpret_cast<const bf16x8*>(&sB[brow1 * LDS_STRIDE + ks * 16 + koff]);            \
        _Pragma("unroll") for (int mi = 0; mi < MI; mi++) {                                                 \
            bf16x8 fa = *reinterpret_cast<const bf16x8*>(&sA[(arow + 32 * mi) * LDS_STRIDE + ks * 16 + koff]); \
            acc[mi][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb0, acc[mi][0], 0, 0, 0);             \
            acc[mi][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb1, acc[mi][1], 0, 0, 0);             \
        }                                                                                                   \
    }                                                                                                       \
    if (MODE == MODE_SERIAL) {                                                                              \
        /* end of a chunk: fold its sum into the running total (left-to-right chunk order) */               \
        if (((KT) + 1) % tiles_per_chunk == 0 || (KT) + 1 == nk) {                                          \
            _Pragma("unroll") for (int i = 0; i < MI; i++)                                                  \
            _Pragma("unroll") for (int j = 0; j < 2; j++)                                                   \
            _Pragma("unroll") for (int e = 0; e < 16; e++) {                                                \
                total[i][j][e] += acc[i][j][e];                                                             \
                acc[i][j][e] = 0.f;                                                                         \
            }                                                                                               \
        }                                                                                                   \
    }

    if (kt0 < kt1) { HS_FETCH_A(kt0) HS_FETCH_B(rb0, kt0) }
    if (kt0 + 1 < kt1) { HS_FETCH_B(rb1, kt0 + 1) }
    for (int kt = kt0; kt < kt1; kt += 2) {
        HS_STAGE(rb0)
        __syncthreads();
        if (kt + 1 < kt1) { HS_FETCH_A(kt + 1) }
        if (kt + 2 < kt1) { HS_FETCH_B(rb0, kt + 2) }
        HS_COMPUTE(kt)
        __syncthreads();
        if (kt + 1 < kt1) {
            HS_STAGE(rb1)
            __syncthreads();
            if (kt + 2 < kt1) { HS_FETCH_A(kt + 2) }
            if (kt + 3 < kt1) { HS_FETCH_B(rb1, kt + 3) }
            HS_COMPUTE(kt + 1)
            __syncthreads();
        }
    }
#undef HS_FETCH_A
#undef HS_FETCH_B
#undef HS_STAGE
#undef HS_COMPUTE

    // Epilogue.  Accumulator element e of a 32x32 tile: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
    const int lr = 4 * (lane >> 5), lc = lane & 31;
    if (EPI == HS_EPI_SWIGLU_BF16) {
        bf16_t* C = reinterpret_cast<bf16_t*>(Cout);
        const int col = n0 + wn * 32 + lc;
        if (col < N) {
#pragma unroll
            for (int mi = 0; mi < MI; mi++)
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    int row = m0 + wm * (BM / 2) + mi * 32 + 8 * (e >> 2) + lr + (e & 3);
                    if (row < M) {
                        float g = acc[mi][0][e], u = acc[mi][1][e];
                        float s = g / (1.f + __expf(-g));
                        C[(size_t)row * N + col] = f32_to_bf16(s * u);
                    }
                }
        }
    } else {
        float* C = (MODE == MODE_SPLIT) ? part + (size_t)blockIdx.y * m_max * N : reinterpret_cast<float*>(Cout);
#pragma unroll
        for (int mi = 0; mi < MI; mi++)
#pragma unroll
            for (int ni = 0; ni < 2; ni++) {
                const int col = n0 + wn * 64 + ni * 32 + lc;
                if (col >= N) continue;
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    int row = m0 + wm * (BM / 2) + mi * 32 + 8 * (e >> 2) + lr + (e & 3);
                    if (row < M) {
                        float v = (MODE == MODE_SERIAL) ? total[mi][ni][e] : acc[mi][ni][e];
                        float* p = &C[(size_t)row * N + col];
                        if (MODE != MODE_SPLIT && EPI == HS_EPI_ADD_F32) *p += v;
                        else *p = v;
                    }
                }
            }
    }
}

// Second pass of the split execution: add the chunk partials left to right, then store or add to the residual.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_split_reduce(const float* __restrict__ part, float* __restrict__ C,
                                                          const int32_t* __restrict__ m_dev, int m_max, int N,
                                                          int chunks) {
    const int row = blockIdx.y;
    if (row >= *m_dev) return;
    const int c4 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c4 >= N) return;
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

template <int EPI, int MODE, int MI>
void launch_tile(const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, float* part, const int32_t* m_dev,
                 int m_max, int n, int k, int chunks, int tpc, hipStream_t st) {
    constexpr int NCOLS = (EPI == HS_EPI_SWIGLU_BF16) ? 64 : 128;
    const int m_tiles = (m_max + 64 * MI - 1) / (64 * MI);
    const int n_tiles = (n + NCOLS - 1) / NCOLS;
    const int blocks = ((n_tiles + 7) / 8) * m_tiles * 8;
    dim3 grid(blocks, MODE == MODE_SPLIT ? chunks : 1);
    hipLaunchKernelGGL((gemm_bf16_mfma<EPI, MODE, MI>), grid, dim3(256), 0, st, a, w, w2, c, part, m_dev, m_max, n, k,
                       m_tiles, n_tiles, tpc);
}

template <int EPI>
void launch(const hs_ctx* ctx, const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, const int32_t* m_dev,
            int m_max, int n, int k, int rows_hint, hipStream_t st) {
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
    // Launch shape from the row hint: narrow outputs run split over K while the row tiles alone would leave compute
    // units idle.  The 256-row tile measured slower than two 128-row tiles at every row count tried (one wavefront
    // per SIMD cannot hide the staging), so it is compiled but not selected.
    const bool tall = false;
    const bool split = chunks > 1 && rows_hint <= 512;
    if (chunks == 1) {
        if (tall) launch_tile<EPI, MODE_PLAIN, 4>(a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, st);
        else launch_tile<EPI, MODE_PLAIN, 2>(a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, st);
    } else if (!split) {
        launch_tile<EPI, MODE_SERIAL, 2>(a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, st);
    } else {
        if (tall) launch_tile<EPI, MODE_SPLIT, 4>(a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, st);
        else launch_tile<EPI, MODE_SPLIT, 2>(a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, st);
        if (EPI != HS_EPI_SWIGLU_BF16)
            hipLaunchKernelGGL((gemm_split_reduce<EPI>), dim3((n / 4 + 255) / 256, m_max), dim3(256), 0, st, part,
                               reinterpret_cast<float*>(c), m_dev, m_max, n, chunks);
    }
}

}  // namespace

// Number of K chunks of a projection: a function of the shape alone.  Narrow outputs (few column tiles) get up
// to 8 chunks so that the split execution can put several hundred workgroups on the chip; every chunk keeps at
// least 4 k-tiles.
int hs_gemm_chunks(int n, int k) {
    const int n_tiles = (n + BN - 1) / BN;
    int chunks = (512 + n_tiles - 1) / n_tiles;
    if (chunks > 8) chunks = 8;
    const int nk = k / BK;
    if (chunks > nk / 4) chunks = nk / 4;
    if (chunks < 1) chunks = 1;
    return chunks;
}

void hs_launch_gemm(const hs_ctx* ctx, int epi, const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c,
                    const int32_t* m_dev, int m_max, int n, int k, int rows_hint, hipStream_t st) {
    switch (epi) {
        case HS_EPI_STORE_F32: launch<HS_EPI_STORE_F32>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st); break;
        case HS_EPI_ADD_F32: launch<HS_EPI_ADD_F32>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st); break;
        default: launch<HS_EPI_SWIGLU_BF16>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st); break;
    }
}
