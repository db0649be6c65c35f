// Launcher of the dense projections of the verify forward pass (QKV, O, gate/up with SwiGLU epilogue, down, LM
// head):  C[M,N] (+)= A[M,K] . W[N,K]^T,  both operands bf16 and K-contiguous, fp32 accumulation.
//
// Reduction order.  K is cut into a fixed number of chunks that depends only on the projection's shape (N, K).  Each
// chunk is accumulated by the matrix cores on its own, and the chunk sums are added left to right in fp32
// (t = p0 + p1 + ...; then stored, or added to the residual).  A row's result therefore never depends on how many
// other rows share the launch or on the launch shape the row hint selects -- which is what makes speculative and
// one-token decoding agree bit for bit.  The MFMA kernel lives in hs_gemm_stream.hip; here are the ordered reduce
// of the chunk partials (used when no following kernel takes them over), a plain reference kernel, and the shape
// rules.
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
    hs_launch_gemm_stream(EPI, a, w, w2, c, part, m_dev, m_max, n, k, chunks, tpc, rows_hint, st);
    if (chunks > 1) {
        if (pending) {
            *pending = chunks;  // the next kernel in line adds the partials up
        } else {
            const int rows = rows_hint < 1 ? 1 : (2 * rows_hint > m_max ? m_max : 2 * rows_hint);
            hipLaunchKernelGGL((gemm_split_reduce<EPI>), dim3((n / 4 + 255) / 256, rows), dim3(256), 0, st, part,
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
