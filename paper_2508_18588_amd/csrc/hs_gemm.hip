// Launcher of the dense projections of the verify forward pass (QKV, O, gate/up with SwiGLU epilogue, down, LM
// head):  C[M,N] (+)= A[M,K] . W[N,K]^T,  both operands bf16 and K-contiguous, fp32 accumulation.
//
// Reduction order.  K is cut into a fixed number of chunks that depends only on the projection's shape (N, K).  Each
// chunk is accumulated by the matrix cores on its own, and the chunk sums are added left to right in fp32
// (t = p0 + p1 + ...; then stored, or added to the residual).  A row's result therefore never depends on how many
// other rows share the launch or on the launch shape the row hint selects -- which is what makes speculative and
// one-token decoding agree bit for bit.  The MFMA kernel lives in hs_gemm_stream.hip; here are the ordered reduce
// of the chunk partials (used when no following kernel takes them over), the plain kernels (debugging, fp32
// activations), and the shape rules.
#include "hs_gemm_common.h"

using namespace hs_gemm_detail;

namespace {

// Second pass of the split execution: add the chunk partials left to right, then store or add to the residual.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_split_reduce(const float* __restrict__ part, float* __restrict__ C,
                                                          const int32_t* __restrict__ m_dev, int m_max, int N,
                                                          int chunks) {
    const int c4 = (blockIdx.x * 256 + threadIdx.x) * 4;
    if (c4 >= N) return;
    const int M = *m_dev;
    if ((N & 3) != 0) {
        // rows are not 16-byte aligned: element by element, same order of addition
        for (int row = blockIdx.y; row < M; row += gridDim.y) {
            for (int c = c4; c < min(c4 + 4, N); c++) {
                const size_t off = (size_t)row * N + c, stride = (size_t)m_max * N;
                float t = part[off];
                for (int s = 1; s < chunks; s++) t += part[s * stride + off];
                if (EPI == HS_EPI_ADD_F32) C[off] += t;
                else C[off] = t;
            }
        }
        return;
    }
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

// Plain kernels for debugging and for the fp32-activation mode: no matrix cores, no LDS.  One wavefront computes
// PR rows x PC output columns; its lanes split K (4 consecutive elements per lane and step, so both operands are
// read in coalesced runs), every lane accumulates its products in ACC precision in k order, and the 64 lane sums
// are combined by a fixed butterfly.  A row's result does not depend on the other rows of the launch.
// AT = activation type (bf16 bits or float); with AT = float nothing is rounded below fp32 anywhere and the sums
// are carried in fp64.
constexpr int PR = 8, PC = 2;

template <typename T> __device__ __forceinline__ float act_load(const T* p);
template <> __device__ __forceinline__ float act_load<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <> __device__ __forceinline__ float act_load<float>(const float* p) { return *p; }
template <typename T> __device__ __forceinline__ void act_store(T* p, float v);
template <> __device__ __forceinline__ void act_store<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }
template <> __device__ __forceinline__ void act_store<float>(float* p, float v) { *p = v; }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const int lo = __shfl_xor(__double2loint(v), o), hi = __shfl_xor(__double2hiint(v), o);
        v += __hiloint2double(hi, lo);
    }
    return v;
}

template <int EPI, typename AT, typename ACC>
__global__ __launch_bounds__(256) void gemm_plain(const AT* __restrict__ A, const bf16_t* __restrict__ W,
                                                   const bf16_t* __restrict__ W2, void* __restrict__ Cout,
                                                   const int32_t* __restrict__ m_dev, int N, int K) {
    constexpr int NW = EPI == HS_EPI_SWIGLU_BF16 ? 2 : 1;
    const int M = *m_dev;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c0 = (blockIdx.x * 4 + wave) * PC, r0 = blockIdx.y * PR;
    if (r0 >= M || c0 >= N) return;
    ACC acc[NW][PR][PC];
#pragma unroll
    for (int w = 0; w < NW; w++)
#pragma unroll
        for (int r = 0; r < PR; r++)
#pragma unroll
            for (int c = 0; c < PC; c++) acc[w][r][c] = 0;
    for (int k = lane * 4; k < K; k += 256) {
        float a[PR][4], b[NW][PC][4];
#pragma unroll
        for (int r = 0; r < PR; r++) {
            const AT* ap = A + (size_t)min(r0 + r, M - 1) * K + k;
#pragma unroll
            for (int e = 0; e < 4; e++) a[r][e] = act_load<AT>(ap + e);
        }
#pragma unroll
        for (int c = 0; c < PC; c++) {
            const size_t wo = (size_t)min(c0 + c, N - 1) * K + k;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                b[0][c][e] = bf16_to_f32(W[wo + e]);
                if (NW == 2) b[NW - 1][c][e] = bf16_to_f32(W2[wo + e]);
            }
        }
#pragma unroll
        for (int e = 0; e < 4; e++)
#pragma unroll
            for (int w = 0; w < NW; w++)
#pragma unroll
                for (int r = 0; r < PR; r++)
#pragma unroll
                    for (int c = 0; c < PC; c++) acc[w][r][c] += (ACC)a[r][e] * (ACC)b[w][c][e];
    }
#pragma unroll
    for (int r = 0; r < PR; r++)
#pragma unroll
        for (int c = 0; c < PC; c++) {
            const ACC s = wave_sum(acc[0][r][c]);
            ACC u = 0;
            if (NW == 2) u = wave_sum(acc[NW - 1][r][c]);
            if (lane != 0 || r0 + r >= M || c0 + c >= N) continue;
            const size_t o = (size_t)(r0 + r) * N + c0 + c;
            if (EPI == HS_EPI_SWIGLU_BF16) {
                // silu(gate) * up, in the accumulation precision
                const ACC g = s / ((ACC)1 + (ACC)exp(-(double)s));
                act_store<AT>(reinterpret_cast<AT*>(Cout) + o, (float)(g * u));
            } else if (EPI == HS_EPI_ADD_F32) {
                float* dst = reinterpret_cast<float*>(Cout) + o;
                *dst = (float)((ACC)*dst + s);
            } else {
                reinterpret_cast<float*>(Cout)[o] = (float)s;
            }
        }
}

template <int EPI>
void launch(const hs_ctx* ctx, const void* a_any, const bf16_t* w, const bf16_t* w2, void* c, const int32_t* m_dev,
            int m_max, int n, int k, int rows_hint, hipStream_t st, int* pending) {
    if (pending) *pending = 0;
    if (hs_plain_kernels(ctx)) {
        dim3 grid((n + 4 * PC - 1) / (4 * PC), (m_max + PR - 1) / PR);
        if (hs_fp32_activations(ctx))
            hipLaunchKernelGGL((gemm_plain<EPI, float, double>), grid, dim3(256), 0, st, (const float*)a_any, w, w2, c,
                               m_dev, n, k);
        else
            hipLaunchKernelGGL((gemm_plain<EPI, bf16_t, float>), grid, dim3(256), 0, st, (const bf16_t*)a_any, w, w2,
                               c, m_dev, n, k);
        return;
    }
    const bf16_t* a = (const bf16_t*)a_any;
    const int nk = k / BK;
    int chunks = (EPI == HS_EPI_SWIGLU_BF16 || EPI == HS_EPI_ROWMAX) ? 1 : hs_gemm_chunks(n, k);
    const int tpc = (nk + chunks - 1) / chunks;
    chunks = (nk + tpc - 1) / tpc;  // no empty chunk
    float* part = reinterpret_cast<float*>(ctx->ws + ctx->lay.gemm_part);
    hs_launch_gemm_stream(EPI, a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, rows_hint, st);
    if (chunks > 1) {
        if (pending) {
            *pending = chunks;  // the next kernel in line adds the partials up
        } else {
            const int rows = rows_hint < 1 ? 1 : (2 * rows_hint > m_max ? m_max : 2 * rows_hint);
            hipLaunchKernelGGL((gemm_split_reduce<EPI>), dim3(((n + 3) / 4 + 255) / 256, rows), dim3(256), 0, st, part,
                               reinterpret_cast<float*>(c), m_dev, m_max, n, chunks);
        }
    }
}

}  // namespace

// Number of K chunks of a projection: a function of the shape alone.  Narrow outputs get as many chunks as put
// about one workgroup of the weight-streaming execution on every one of the 256 compute units; every chunk keeps at
// least 4 k-tiles.  A workgroup takes 128 weight rows, or 64 when the reduction is short (hs_gemm_narrow_groups):
// with half as many chunks the projection writes -- and the kernel after it reads -- half the partial sums, and
// with K < 8192 the activation tile that every workgroup re-reads is small enough for that to pay.
bool hs_gemm_narrow_groups(int k) { return k < 8192; }

int hs_gemm_chunks(int n, int k) {
    const int groups = hs_gemm_narrow_groups(k) ? (n + 63) / 64 : (n + 127) / 128;
    int chunks = 256 / groups;
    const int nk = k / BK;
    if (chunks > nk / 4) chunks = nk / 4;
    if (chunks < 1) chunks = 1;
    return chunks;
}

void hs_launch_gemm(const hs_ctx* ctx, int epi, const void* a, const bf16_t* w, const bf16_t* w2, void* c,
                    const int32_t* m_dev, int m_max, int n, int k, int rows_hint, hipStream_t st, int* pending) {
    switch (epi) {
        case HS_EPI_STORE_F32:
            launch<HS_EPI_STORE_F32>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st, pending);
            break;
        case HS_EPI_ADD_F32:
            launch<HS_EPI_ADD_F32>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st, pending);
            break;
        case HS_EPI_ROWMAX:
            launch<HS_EPI_ROWMAX>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st, pending);
            break;
        default:
            launch<HS_EPI_SWIGLU_BF16>(ctx, a, w, w2, c, m_dev, m_max, n, k, rows_hint, st, pending);
            break;
    }
}
