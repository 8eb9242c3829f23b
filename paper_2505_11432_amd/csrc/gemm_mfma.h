// Shared definitions of the grouped MFMA GEMM (the paper's GroupedGEMM operator, Section 4.1; Section 7 names
// it, with its dynamic per-expert shapes, as the straggler of MoE layers): argument block, operand layouts,
// contraction modes, epilogues and the two LDS read primitives.  The kernel itself is in gemm_mfma_dma.h.
//   forward   C[rows, N] = A[rows, K] * W[e][N, K]^T     A K-major, B K-major, rows segmented by expert
//   dgrad     C[rows, N] = A[rows, K] * W[e][K, N]       A K-major, B N-major, rows segmented by expert
//   wgrad     C[e][M, N] = P[rows_e, M]^T * Q[rows_e, N] A M-major, B N-major, contraction segmented
#pragma once
#include "moe_common.h"

namespace moe {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) short s16x4;

enum Layout { KMAJOR = 0, MNMAJOR = 1 };
enum Mode { ROWSEG = 0, KSEG = 1, PLAIN = 2 };   // PLAIN: one dense GEMM, no expert segments
// EPI_SWIGLU_W / EPI_SWIGLU_BWD_W: the Section 4.1 operator order (gate weight multiplied right after SwiGLU; the
// forward one also selects its A rows through an index map, Section 4.2)
enum Epi { EPI_STORE = 0, EPI_SWIGLU = 1, EPI_SWIGLU_BWD = 2, EPI_BIAS_F32 = 3, EPI_SWIGLU_W = 4, EPI_SWIGLU_BWD_W = 5 };

typedef __attribute__((ext_vector_type(8))) int i32x8;

struct Args {
  const void* A; long lda;           // A operand: K-major [rows, K] or M-major [rows(k), M]; bf16, or e4m3 codes
  const void* B; long ldb; long b_es; // B operand per expert: K-major [N, K] or N-major [K, N] (strides in elements)
  void* C; long ldc; long c_es;      // output (c_es: per-expert stride, wgrad only)
  const int32_t* offsets; int E;
  int M;                             // ROWSEG: total rows in A/C (upper bound); KSEG: rows of C
  int N, K;                          // KSEG: K unused (segment length comes from offsets)
  int accumulate;
  // fused SwiGLU epilogues
  int f;                             // EPI_SWIGLU: B rows n and f+n are paired, N = f
  bf16* H;                           // EPI_SWIGLU: [rows, 2f] receives G|U;  EPI_SWIGLU_BWD: read G|U
  bf16* A_out;                       // [rows, f]: SwiGLU output (both fused epilogues)
  bf16* dH;                          // EPI_SWIGLU_BWD: [rows, 2f] receives dG|dU
  const float* bias;                 // EPI_BIAS_F32: per-column fp32 bias or NULL; C is fp32, any N
  const float* row_scale;            // e4m3 operands: per-row scale of A [rows] (NULL = 1)
  const float* col_scale; long cs_es; // e4m3 operands: per-output-channel scale of B [E, N(+f)] and its expert stride
  // e4m3 weight-gradient GEMM (KSEG): power-of-two group scales, one E8M0 byte per (128-k group, row) of each
  // operand, applied by the block-scaled MFMA; [groups, rows] with the given row counts as leading dimensions
  const uint8_t* a_e8m0; long a_e8_ld;
  const uint8_t* b_e8m0; long b_e8_ld;
  // Split-K for the last, partly filled round of tiles (ROWSEG, bf16 store epilogue only): when the tiles left
  // after the complete rounds fill at most half of the workgroups, each of them is cut into 2..4 parts along K
  // that run on different workgroups and write fp32 partial tiles here ([part][BM][BN]); splitk_fixup_kernel
  // adds the parts and writes C.  NULL: no splitting.
  float* splitk_ws;
  // Section 4.1 / 4.2 order (EPI_SWIGLU_W, EPI_SWIGLU_BWD_W)
  const int32_t* a_rowmap;           // EPI_SWIGLU_W: logical row r of A is row a_rowmap[r] of the buffer ([M] entries)
  int a_phys_rows;                   //   rows of that buffer (for the 32-bit offset check)
  const float* row_w;                // [M] gate weight of each row: A_out = w * SwiGLU(G, U) in both epilogues
  float* dw_part;                    // EPI_SWIGLU_BWD_W: [n-tiles * waves along n][M] partial sums of <dA'[r,:], A[r,:]>
};

__device__ __forceinline__ bf16x8 lds_read_b128(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }

__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
  typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
  const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
  return __builtin_bit_cast(bf16x4, r);
}

}  // namespace mfma
}  // namespace moe
