// bf16 MFMA GEMMs for the dense projections of the verify forward pass (QKV, O, gate/up with SwiGLU epilogue,
// down, LM head):  C[M,N] (+)= A[M,K] . W[N,K]^T,  both operands K-contiguous, fp32 accumulation.
//
// Layout on gfx950: a workgroup of 4 wavefronts owns a 128x128 output tile; each wavefront a 64x64 quadrant as
// 2x2 v_mfma_f32_32x32x16_bf16 tiles.  A and W tiles (128 x 64 bf16) are staged through LDS with a padded row
// stride; the next k-tile is prefetched into registers while the current one feeds the matrix cores.  The
// accumulation order over K is the same for every row, whatever M is: a row's result does not depend on which
// other rows share the launch (this is what makes speculative and one-token decoding agree bit for bit).
//
// The row count M lives on the device (number of draft-tree rows of this step); the grid covers m_max rows and
// workgroups whose rows start beyond M exit at once.  Workgroup ids are spread so that all M-tiles that read the
// same W-tile run on the same XCD (ids are dealt round-robin to the 8 XCDs, each with its own L2).
#include "hs_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int LDS_STRIDE = BK + 8;  // bf16 elements; 144-byte rows keep 16-byte reads conflict-free

struct Chunk { uint4 v; };

template <int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_mfma(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W,
                                                       const bf16_t* __restrict__ W2, void* __restrict__ Cout,
                                                       const int32_t* __restrict__ m_dev, int N, int K, int m_tiles,
                                                       int n_tiles) {
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

    // global -> register staging: 4 x 16-byte chunks of A and of W per thread and k-tile
    Chunk ra[4], rb[4];
    const bf16_t* a_ptr[4];
    const bf16_t* b_ptr[4];
    bool a_ok[4], b_ok[4];
    int s_off[4];
#pragma unroll
    for (int i = 0; i < 4; i++) {
        int c = tid + 256 * i;
        int r = c >> 3, c8 = (c & 7) * 8;
        s_off[i] = r * LDS_STRIDE + c8;
        int gm = m0 + r;
        a_ok[i] = gm < M;
        a_ptr[i] = A + (size_t)(a_ok[i] ? gm : 0) * K + c8;
        int gn;
        const bf16_t* wsrc = W;
        if (EPI == HS_EPI_SWIGLU_BF16) {
            gn = n0 + (r & 63);
            if (r >= 64) wsrc = W2;
        } else {
            gn = n0 + r;
        }
        b_ok[i] = gn < N;
        b_ptr[i] = wsrc + (size_t)(b_ok[i] ? gn : 0) * K + c8;
    }
    const uint4 zero4 = make_uint4(0, 0, 0, 0);

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    const int nk = K / BK;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        ra[i].v = a_ok[i] ? *reinterpret_cast<const uint4*>(a_ptr[i]) : zero4;
        rb[i].v = b_ok[i] ? *reinterpret_cast<const uint4*>(b_ptr[i]) : zero4;
    }

    const int arow = wm * 64 + (lane & 31);
    const int brow0 = (EPI == HS_EPI_SWIGLU_BF16) ? (wn * 32 + (lane & 31)) : (wn * 64 + (lane & 31));
    const int brow1 = (EPI == HS_EPI_SWIGLU_BF16) ? (64 + wn * 32 + (lane & 31)) : (wn * 64 + 32 + (lane & 31));
    const int koff = (lane >> 5) * 8;

    for (int kt = 0; kt < nk; kt++) {
#pragma unroll
        for (int i = 0; i < 4; i++) {
            *reinterpret_cast<uint4*>(&sA[s_off[i]]) = ra[i].v;
            *reinterpret_cast<uint4*>(&sB[s_off[i]]) = rb[i].v;
        }
        __syncthreads();
        if (kt + 1 < nk) {
#pragma unroll
            for (int i = 0; i < 4; i++) {
                ra[i].v = a_ok[i] ? *reinterpret_cast<const uint4*>(a_ptr[i] + (size_t)(kt + 1) * BK) : zero4;
                rb[i].v = b_ok[i] ? *reinterpret_cast<const uint4*>(b_ptr[i] + (size_t)(kt + 1) * BK) : zero4;
            }
        }
#pragma unroll
        for (int ks = 0; ks < BK / 16; ks++) {
            bf16x8 fa0 = *reinterpret_cast<const bf16x8*>(&sA[arow * LDS_STRIDE + ks * 16 + koff]);
            bf16x8 fa1 = *reinterpret_cast<const bf16x8*>(&sA[(arow + 32) * LDS_STRIDE + ks * 16 + koff]);
            bf16x8 fb0 = *reinterpret_cast<const bf16x8*>(&sB[brow0 * LDS_STRIDE + ks * 16 + koff]);
            bf16x8 fb1 = *reinterpret_cast<const bf16x8*>(&sB[brow1 * LDS_STRIDE + ks * 16 + koff]);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0, fb0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa0, fb1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1, fb0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa1, fb1, acc[1][1], 0, 0, 0);
        }
        __syncthreads();
    }

    // Epilogue.  Accumulator element e of a 32x32 tile: row 8*(e/4) + 4*(lane/32) + e%4, column lane%32.
    const int lr = 4 * (lane >> 5), lc = lane & 31;
    if (EPI == HS_EPI_SWIGLU_BF16) {
        bf16_t* C = reinterpret_cast<bf16_t*>(Cout);
        const int col = n0 + wn * 32 + lc;
        if (col < N) {
#pragma unroll
            for (int mi = 0; mi < 2; mi++)
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    int row = m0 + wm * 64 + mi * 32 + 8 * (e >> 2) + lr + (e & 3);
                    if (row < M) {
                        float g = acc[mi][0][e], u = acc[mi][1][e];
                        float s = g / (1.f + __expf(-g));
                        C[(size_t)row * N + col] = f32_to_bf16(s * u);
                    }
                }
        }
    } else {
        float* C = reinterpret_cast<float*>(Cout);
#pragma unroll
        for (int mi = 0; mi < 2; mi++)
#pragma unroll
            for (int ni = 0; ni < 2; ni++) {
                const int col = n0 + wn * 64 + ni * 32 + lc;
                if (col >= N) continue;
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    int row = m0 + wm * 64 + mi * 32 + 8 * (e >> 2) + lr + (e & 3);
                    if (row < M) {
                        float* p = &C[(size_t)row * N + col];
                        if (EPI == HS_EPI_ADD_F32) *p += acc[mi][ni][e];
                        else *p = acc[mi][ni][e];
                    }
                }
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

template <int EPI>
void launch(const hs_ctx* ctx, const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, const int32_t* m_dev,
            int m_max, int n, int k, hipStream_t st) {
    if (ctx->flags & HS_FLAG_REFERENCE_KERNELS) {
        dim3 grid((n + 255) / 256, m_max);
        hipLaunchKernelGGL(gemm_bf16_plain<EPI>, grid, dim3(256), 0, st, a, w, w2, c, m_dev, n, k);
        return;
    }
    constexpr int NCOLS = (EPI == HS_EPI_SWIGLU_BF16) ? 64 : 128;
    int m_tiles = (m_max + BM - 1) / BM;
    int n_tiles = (n + NCOLS - 1) / NCOLS;
    int n_per_xcd = (n_tiles + 7) / 8;
    int blocks = n_per_xcd * m_tiles * 8;
    hipLaunchKernelGGL(gemm_bf16_mfma<EPI>, dim3(blocks), dim3(256), 0, st, a, w, w2, c, m_dev, n, k, m_tiles,
                       n_tiles);
}

}  // namespace

void hs_launch_gemm(const hs_ctx* ctx, int epi, const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c,
                    const int32_t* m_dev, int m_max, int n, int k, hipStream_t st) {
    switch (epi) {
        case HS_EPI_STORE_F32: launch<HS_EPI_STORE_F32>(ctx, a, w, w2, c, m_dev, m_max, n, k, st); break;
        case HS_EPI_ADD_F32: launch<HS_EPI_ADD_F32>(ctx, a, w, w2, c, m_dev, m_max, n, k, st); break;
        default: launch<HS_EPI_SWIGLU_BF16>(ctx, a, w, w2, c, m_dev, m_max, n, k, st); break;
    }
}
