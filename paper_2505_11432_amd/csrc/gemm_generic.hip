// Generic strided grouped GEMM on the vector ALU (fp32 FMA, LDS-tiled 64x64x16).
//
// It is the arithmetic of the paper's GroupedGEMM operator (Section 4.1: one kernel for the
// per-expert matmuls of FC1 and FC2, and their gradients) for the cases the MFMA kernels do
// not cover: fp32 data (no fast fp32 matrix path is needed for the correctness-only
// configuration), the skinny router matmuls, and shapes the tuned tiles reject.
#include "moe_common.h"

namespace moe {
namespace {

constexpr int BM = 64, BN = 64, BK = 16, NT = 256;

template <typename TA, typename TB, typename TC>
__global__ void __launch_bounds__(NT) gemm_generic_kernel(GemmProblem p, int tiles_n, int tiles_m_fixed) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const TA* __restrict__ A = static_cast<const TA*>(p.A);
  const TB* __restrict__ B = static_cast<const TB*>(p.B);
  TC* __restrict__ C = static_cast<TC*>(p.C);

  const int tid = threadIdx.x;
  const int nt = blockIdx.x % tiles_n;
  int rest = blockIdx.x / tiles_n;
  int e = 0, m0, m_end, k0, k_end;
  if (p.mode == 0) {
    // rest = running tile index over all experts' row tiles
    int found = 0;
    for (e = 0; e < p.E; ++e) {
      const int lo = p.offsets[e], hi = p.offsets[e + 1];
      const int te = (hi - lo + BM - 1) / BM;
      if (rest < te) { m0 = lo + rest * BM; m_end = hi; found = 1; break; }
      rest -= te;
    }
    if (!found) return;
    k0 = 0; k_end = p.K;
  } else if (p.mode == 1) {
    e = rest / tiles_m_fixed;
    m0 = (rest % tiles_m_fixed) * BM; m_end = p.M;
    k0 = p.offsets[e]; k_end = p.offsets[e + 1];
  } else {
    m0 = rest * BM; m_end = p.M;
    k0 = 0; k_end = p.K;
  }
  const int n0 = nt * BN;
  const TB* Be = B + (long)e * p.b_es;
  TC* Ce = C + (long)e * p.c_es;

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;

  const int ty = tid / 16, tx = tid % 16;
  const bool a_kfast = (p.a_cs == 1);
  const bool b_nfast = (p.b_cs == 1);

  for (int kb = k0; kb < k_end; kb += BK) {
#pragma unroll
    for (int i = 0; i < (BM * BK) / NT; ++i) {
      const int idx = tid + i * NT;
      const int m = a_kfast ? idx / BK : idx % BM;
      const int k = a_kfast ? idx % BK : idx / BM;
      float v = 0.f;
      if (m0 + m < m_end && kb + k < k_end) v = to_f32(A[(long)(m0 + m) * p.a_rs + (long)(kb + k) * p.a_cs]);
      As[k][m] = v;
    }
#pragma unroll
    for (int i = 0; i < (BN * BK) / NT; ++i) {
      const int idx = tid + i * NT;
      const int n = b_nfast ? idx % BN : idx / BK;
      const int k = b_nfast ? idx / BN : idx % BK;
      float v = 0.f;
      if (n0 + n < p.N && kb + k < k_end) v = to_f32(Be[(long)(kb + k) * p.b_rs + (long)(n0 + n) * p.b_cs]);
      Bs[k][n] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= m_end) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= p.N) continue;
      float v = acc[i][j];
      if (p.bias) v += p.bias[n];
      TC* dst = Ce + (long)m * p.ldc + n;
      if (p.accumulate) v += to_f32(*dst);
      *dst = from_f32<TC>(v);
    }
  }
}

}  // namespace

int launch_gemm_generic(const GemmProblem& p, moe_dtype a_dt, moe_dtype b_dt, moe_dtype c_dt, hipStream_t s) {
  const int tiles_n = cdiv(p.N, BN);
  int tiles_m_fixed = 1;
  long blocks;
  if (p.mode == 0) {
    blocks = (long)tiles_n * (cdiv(p.M, BM) + p.E);
  } else if (p.mode == 1) {
    tiles_m_fixed = cdiv(p.M, BM);
    blocks = (long)tiles_n * tiles_m_fixed * p.E;
  } else {
    blocks = (long)tiles_n * cdiv(p.M, BM);
  }
  if (blocks <= 0 || p.N <= 0) return MOE_OK;
  if (blocks > 0x7fffffffL) return MOE_ERR_UNSUPPORTED;
  dim3 grid((unsigned)blocks), block(NT);
#define MOE_GEMM_CASE(DA, DB, DC, TA, TB, TC)                                          \
  if (a_dt == DA && b_dt == DB && c_dt == DC) {                                        \
    gemm_generic_kernel<TA, TB, TC><<<grid, block, 0, s>>>(p, tiles_n, tiles_m_fixed); \
    MOE_LAUNCH_CHECK();                                                                \
    return MOE_OK;                                                                     \
  }
  MOE_GEMM_CASE(MOE_F32, MOE_F32, MOE_F32, float, float, float)
  MOE_GEMM_CASE(MOE_BF16, MOE_BF16, MOE_BF16, bf16, bf16, bf16)
  MOE_GEMM_CASE(MOE_BF16, MOE_BF16, MOE_F32, bf16, bf16, float)
  MOE_GEMM_CASE(MOE_F32, MOE_BF16, MOE_F32, float, bf16, float)
  MOE_GEMM_CASE(MOE_F32, MOE_BF16, MOE_BF16, float, bf16, bf16)
#undef MOE_GEMM_CASE
  return MOE_ERR_UNSUPPORTED;
}

}  // namespace moe
