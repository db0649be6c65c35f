// Helpers of the bf16 MFMA GEMM (launcher and kernel live in two translation units).
#pragma once
#include "hs_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace hs_gemm_detail {

constexpr int BK = 64;             // k-tile depth
constexpr int ROW_BYTES = BK * 2;  // one tile row in LDS: 8 chunks of 16 bytes

// vmcnt(n) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4 and lgkmcnt 11:8 left at their maxima)
#define HS_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))

// Chunk swizzle of tile row r: consecutive rows 0..15 map to the 16 distinct (row parity, chunk) bank groups, and
// rows 0..7 to even values, so that the two k-halves of a fragment read (chunks c and c^1) never collide either.
__device__ __forceinline__ int swz(int r) { return (((r >> 1) & 3) << 1) | ((r >> 3) & 1); }

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// 16 bytes per lane from global memory straight into LDS: lane i's data lands at LDS byte offset lds_off + 16 * i
// (lds_off is wavefront-uniform and travels in M0).  Counted by vmcnt like any other load.  Issued as inline
// assembly so that the compiler's wait-count bookkeeping does not see it: told about such a load it treats every
// later LDS read as possibly returning out of order and waits for all of them at once, which serialises fragment
// reads and matrix-core work; the kernels place the vmcnt waits for these loads themselves.  Any wait the compiler
// inserts for its own loads can only be stricter than needed, because loads complete in issue order.
// The source address is a wavefront-uniform base (scalar registers) plus a 32-bit unsigned byte offset per lane.
__device__ __forceinline__ void load_to_lds_16(const unsigned char* base, unsigned off, unsigned lds_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_off), "v"(off), "s"(base)
                 : "memory", "m0");
}

// The same for data that is read once per launch (the weight stream): non-temporal, so that it does not evict the
// activation tile that every workgroup re-reads from L2.
__device__ __forceinline__ void load_to_lds_16_stream(const unsigned char* base, unsigned off, unsigned lds_off) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                 :
                 : "s"(lds_off), "v"(off), "s"(base)
                 : "memory", "m0");
}

}  // namespace hs_gemm_detail

// Split-K projections with a short reduction run in groups of 64 weight rows (see hs_gemm_chunks).
bool hs_gemm_narrow_groups(int k);

// The MFMA kernel (defined in hs_gemm_stream.hip).  `chunks`/`tpc` are the K chunking of
// the shape (chunks > 1: chunk sums go to `part`, laid out [chunk][m_max][n], for the ordered reduce).
void hs_launch_gemm_stream(int epi, const bf16_t* a, const bf16_t* w, const bf16_t* w2, void* c, float* part,
                           const int32_t* m_dev, int m_max, int n, int k, int chunks, int tpc, int rows_hint,
                           hipStream_t st);
