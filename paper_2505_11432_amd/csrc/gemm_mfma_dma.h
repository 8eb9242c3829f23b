// Grouped bf16 GEMM on the gfx950 matrix cores with an asynchronous global->LDS pipeline.
//
// Same contract and tile geometry as gemm_mfma.h (the paper's GroupedGEMM operator, Section 4.1, in
// its three contraction layouts), but operand tiles travel global -> LDS directly
// (global_load_lds_dwordx4) into an NSTAGE-deep ring, so loads for k-step s+NSTAGE-1 are in flight
// while k-step s is on the matrix cores, no VGPRs stage the tiles and no ds_write phase exists.
// One s_barrier per k-step: after it every wave's loads for the step have landed and every wave has
// left the previous step, whose buffer the new loads may overwrite.
//
// A direct-to-LDS load deposits the wave's 64 x 16 bytes contiguously, so the LDS swizzles are applied
// on the global side: the lane that owns physical chunk pc of a row fetches logical chunk pc ^ swz(row).
//   K-major tile [rows][BKT]:  swz = (row / rows_per_256B) mod chunks_per_row  -> ds_read_b128 conflict-free
//   M/N-major tile [BKT][cols]: swz = 4 * (k mod 4)                            -> ds_read_b64_tr_b16 conflict-free
// Loads that fall outside the contraction range fetch from a 16-byte zero block instead, which gives
// the exact zero fill that ragged expert segments (wgrad) and K tails need.
#pragma once
#include "gemm_mfma.h"

namespace moe {
namespace mfma {

static __device__ __attribute__((aligned(16))) const unsigned int g_zero_block[4] = {0u, 0u, 0u, 0u};

// One wave-wide direct-to-LDS load: lane i's 16 bytes land at lds_addr + 16*i.  lds_addr is wave-uniform.
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "memory", "m0");
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]; other counters left open
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <int ROWS, int BKT> struct KTile {        // K-major [ROWS][BKT] bf16
  static constexpr int ROW_BYTES = BKT * 2, CPR = ROW_BYTES / 16, RPL = 256 / ROW_BYTES;
  static constexpr int BYTES = ROWS * ROW_BYTES;
  static constexpr int ROWS_PER_DMA = 1024 / ROW_BYTES;
  __device__ static __forceinline__ int swz(int row) { return (row / RPL) % CPR; }
  __device__ static __forceinline__ int offset(int row, int chunk) { return row * ROW_BYTES + ((chunk ^ swz(row)) << 4); }
};
template <int COLS, int BKT> struct MNTile {       // M/N-major [BKT][COLS] bf16
  static constexpr int ROW_BYTES = COLS * 2, CPR = ROW_BYTES / 16;
  static constexpr int BYTES = BKT * ROW_BYTES;
  static constexpr int ROWS_PER_DMA = 1024 / ROW_BYTES;
  static_assert(ROW_BYTES <= 1024 && CPR >= 16, "M/N-major tiles are 128..512 columns wide");
  __device__ static __forceinline__ int swz(int krow) { return (krow & 3) << 2; }
};

template <Layout L, int EXTENT, int BKT> struct DmaTileBytes;
template <int EXTENT, int BKT> struct DmaTileBytes<KMAJOR, EXTENT, BKT> { static constexpr int value = KTile<EXTENT, BKT>::BYTES; };
template <int EXTENT, int BKT> struct DmaTileBytes<MNMAJOR, EXTENT, BKT> { static constexpr int value = MNTile<EXTENT, BKT>::BYTES; };

template <Layout L, int EXTENT, int BKT>
__device__ __forceinline__ bf16x8 read_frag_dma(const char* tile, int base, int kk, int lane) {
  if constexpr (L == KMAJOR) {
    const int row = base + (lane & 31);
    return lds_read_b128(tile + KTile<EXTENT, BKT>::offset(row, kk * 2 + (lane >> 5)));
  } else {
    using TL = MNTile<EXTENT, BKT>;
    const int g = lane >> 4, i = lane & 15;
    const int krow = kk * 16 + ((g >> 1) << 3) + (i >> 2);          // krow & 3 == (i >> 2)
    const int col = base + ((g & 1) << 4) + ((i & 3) << 2);
    const int chunk = (col >> 3) ^ TL::swz(krow);
    const char* p = tile + krow * TL::ROW_BYTES + (chunk << 4) + ((col & 7) << 1);
    const bf16x4 lo = lds_read_tr(p);
    const bf16x4 hi = lds_read_tr(p + 4 * TL::ROW_BYTES);             // krow + 4 has the same swizzle
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }
}

template <int BM, int BN, int BKT, int NSTAGE, int WM, int WN, Layout LA, Layout LB, Mode MODE, Epi EPI, typename TC,
          int PROBE = 0>   // PROBE (tuning only): 1 = no global loads, 2 = no LDS reads / MFMAs
__global__ void __launch_bounds__(WM * WN * 64) grouped_gemm_dma_kernel(Args p) {
  constexpr int NW = WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int A_BYTES = DmaTileBytes<LA, BM, BKT>::value, B_BYTES = DmaTileBytes<LB, BN, BKT>::value;
  constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int A_DMA = A_BYTES / 1024 / NW, B_DMA = B_BYTES / 1024 / NW;     // loads per wave per stage
  constexpr int LOADS = A_DMA + B_DMA;
  static_assert(A_BYTES % (1024 * NW) == 0 && B_BYTES % (1024 * NW) == 0, "tile does not split over the waves");
  static_assert(NSTAGE >= 2 && (NSTAGE - 2) * LOADS < 64, "pipeline depth exceeds the vmcnt range");
  static_assert(EPI != EPI_SWIGLU || TN % 2 == 0, "SwiGLU pairs gate/up MFMA tiles inside a wave");

  extern __shared__ __attribute__((aligned(16))) char smem[];
  const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)smem;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  // ---- which tile is mine -----------------------------------------------------------------
  // Workgroup b runs on XCD b % 8 and each XCD has its own L2, so XCD x is handed the x-th eighth of a
  // logical tile order in which 32 consecutive tiles (one per CU of the XCD) form a compact block of one
  // expert: all of GN adjacent n-tiles for a run of m-tiles.  Those tiles stream the same A and B panels
  // at the same k, which turns most of their loads into L2 hits.
  constexpr int BN_OUT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;
  constexpr int GN = 4, XCDS = 8;
  const int tiles_n = (p.N + BN_OUT - 1) / BN_OUT;
  const int tiles_m_fixed = (p.M + BM - 1) / BM;              // KSEG only
  int total_tiles;
  if constexpr (MODE == ROWSEG) {
    int mts = 0;
    for (int i = 0; i < p.E; ++i) mts += (p.offsets[i + 1] - p.offsets[i] + BM - 1) / BM;
    total_tiles = mts * tiles_n;
  } else if constexpr (MODE == KSEG) {
    total_tiles = p.E * tiles_m_fixed * tiles_n;
  } else {
    total_tiles = tiles_m_fixed * tiles_n;
  }
  const int per_xcd = (total_tiles + XCDS - 1) / XCDS;
  const int slot = blockIdx.x / XCDS;
  if (slot >= per_xcd) return;
  int l = (blockIdx.x % XCDS) * per_xcd + slot;                // logical tile index
  if (l >= total_tiles) return;
  int e, mt_e, m_lo, m_hi;
  if constexpr (MODE == ROWSEG) {
    for (e = 0; e < p.E; ++e) {
      m_lo = p.offsets[e]; m_hi = p.offsets[e + 1];
      mt_e = (m_hi - m_lo + BM - 1) / BM;
      if (l < mt_e * tiles_n) break;
      l -= mt_e * tiles_n;
    }
  } else {
    mt_e = tiles_m_fixed;
    e = l / (mt_e * tiles_n);          // always 0 in PLAIN mode
    l -= e * mt_e * tiles_n;
    m_lo = 0; m_hi = p.M;
  }
  const int ng = l / (mt_e * GN);
  const int r = l - ng * mt_e * GN;
  const int gw = min(GN, tiles_n - ng * GN);
  const int mt = r / gw;
  const int nt = ng * GN + (r - mt * gw);
  const int m0 = m_lo + mt * BM, m_end = m_hi;
  int k_begin, k_end;
  if constexpr (MODE == KSEG) { k_begin = p.offsets[e]; k_end = p.offsets[e + 1]; }
  else { k_begin = 0; k_end = p.K; }
  const int n0 = nt * BN_OUT;
  const bf16* __restrict__ Ag = p.A;
  const bf16* __restrict__ Bg = p.B + (long)e * p.b_es;
  const char* zero = reinterpret_cast<const char*>(g_zero_block);

  // ---- per-lane source pointers of this wave's loads (k-step 0), and what advances them ----------
  // load j of the wave covers DMA slot q = wave + j*NW of the tile (1 KiB of LDS each).
  const char* a_src[A_DMA];
  const char* b_src[B_DMA];
  int a_k[A_DMA], b_k[B_DMA];       // k coordinate (relative to the k-step start) this lane's chunk begins at
  long a_step, b_step;              // bytes to advance per k-step
#pragma unroll
  for (int j = 0; j < A_DMA; ++j) {
    const int q = wave + j * NW;
    if constexpr (LA == KMAJOR) {
      using TL = KTile<BM, BKT>;
      const int row = q * TL::ROWS_PER_DMA + lane / TL::CPR;
      const int lc = (lane % TL::CPR) ^ TL::swz(row);
      const int gr = min(m0 + row, p.M - 1);
      a_src[j] = reinterpret_cast<const char*>(Ag + (long)gr * p.lda + k_begin + lc * 8);
      a_k[j] = lc * 8;
    } else {
      using TL = MNTile<BM, BKT>;
      const int krow = q * TL::ROWS_PER_DMA + lane / TL::CPR;
      const int lc = (lane % TL::CPR) ^ TL::swz(krow);
      const int col = min(m0 + lc * 8, p.M - 8);
      a_src[j] = reinterpret_cast<const char*>(Ag + (long)(k_begin + krow) * p.lda + col);
      a_k[j] = krow;
    }
  }
  a_step = (LA == KMAJOR) ? (long)BKT * 2 : (long)BKT * p.lda * 2;
#pragma unroll
  for (int j = 0; j < B_DMA; ++j) {
    const int q = wave + j * NW;
    if constexpr (LB == KMAJOR) {
      using TL = KTile<BN, BKT>;
      const int row = q * TL::ROWS_PER_DMA + lane / TL::CPR;
      const int lc = (lane % TL::CPR) ^ TL::swz(row);
      int gr;
      if constexpr (EPI == EPI_SWIGLU) {
        const int qq = row >> 5;
        const int n = min(n0 + (qq >> 1) * 32 + (row & 31), p.f - 1);
        gr = (qq & 1) ? p.f + n : n;
      } else {
        gr = min(n0 + row, p.N - 1);
      }
      b_src[j] = reinterpret_cast<const char*>(Bg + (long)gr * p.ldb + k_begin + lc * 8);
      b_k[j] = lc * 8;
    } else {
      using TL = MNTile<BN, BKT>;
      const int krow = q * TL::ROWS_PER_DMA + lane / TL::CPR;
      const int lc = (lane % TL::CPR) ^ TL::swz(krow);
      const int col = min(n0 + lc * 8, p.N - 8);
      b_src[j] = reinterpret_cast<const char*>(Bg + (long)(k_begin + krow) * p.ldb + col);
      b_k[j] = krow;
    }
  }
  b_step = (LB == KMAJOR) ? (long)BKT * 2 : (long)BKT * p.ldb * 2;

  const int klen = k_end - k_begin;
  const int nk = (klen + BKT - 1) / BKT;

  // Issue the loads of k-step `ks` into ring slot ks % NSTAGE.  Only the last step can be ragged.
  auto issue = [&](int ks) {
    if constexpr (PROBE == 1) return;
    const unsigned stage = smem_lds + (unsigned)(ks % NSTAGE) * STAGE_BYTES;
    const int k_left = klen - ks * BKT;          // valid k in this step
    const bool full = k_left >= BKT;
#pragma unroll
    for (int j = 0; j < A_DMA; ++j) {
      const char* src = a_src[j] + (long)ks * a_step;
      if (!full && a_k[j] >= k_left) src = zero;
      dma16(src, stage + (unsigned)(wave + j * NW) * 1024u);
    }
#pragma unroll
    for (int j = 0; j < B_DMA; ++j) {
      const char* src = b_src[j] + (long)ks * b_step;
      if (!full && b_k[j] >= k_left) src = zero;
      dma16(src, stage + A_BYTES + (unsigned)(wave + j * NW) * 1024u);
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- pipeline ---------------------------------------------------------------------------------
#pragma unroll
  for (int s = 0; s < NSTAGE - 1; ++s)
    if (s < nk) issue(s);

  for (int kt = 0; kt < nk; ++kt) {
    // my loads for step kt have landed once at most the younger steps' loads are outstanding
    if (kt + NSTAGE - 2 < nk) wait_vmcnt<(NSTAGE - 2) * LOADS>();
    else wait_vmcnt<0>();
    __syncthreads();
    if (kt + NSTAGE - 1 < nk) issue(kt + NSTAGE - 1);

    const char* at = smem + (kt % NSTAGE) * STAGE_BYTES;
    const char* bt = at + A_BYTES;
    if constexpr (PROBE == 2) continue;
#pragma unroll
    for (int kk = 0; kk < BKT / 16; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = read_frag_dma<LA, BM, BKT>(at, wm * WTM + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = read_frag_dma<LB, BN, BKT>(bt, wn * WTN + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
  }

  // ---- epilogue (same register layout as gemm_mfma.h) ------------------------------------------
  const int lrow = lane & 31, lcol = (lane >> 5) << 2;
  if constexpr (EPI == EPI_STORE) {
    TC* __restrict__ Cg = static_cast<TC*>(p.C) + (long)e * p.c_es;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = m0 + wm * WTM + i * 32 + lrow;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + wn * WTN + j * 32 + q * 8 + lcol;
          if (n >= p.N) continue;
          TC* dst = Cg + (long)m * p.ldc + n;
          float v[4] = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
          Vec16<TC> o;
          if (p.accumulate) {
#pragma unroll
            for (int t = 0; t < 4; ++t) v[t] += to_f32(dst[t]);
          }
#pragma unroll
          for (int t = 0; t < 4; ++t) o.v[t] = from_f32<TC>(v[t]);
          if constexpr (sizeof(TC) == 4) *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<uint4*>(&o);
          else *reinterpret_cast<uint2*>(dst) = *reinterpret_cast<uint2*>(&o);
        }
      }
    }
  } else if constexpr (EPI == EPI_BIAS_F32) {
    float* __restrict__ Cg = static_cast<float*>(p.C);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = m0 + wm * WTM + i * 32 + lrow;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int n = n0 + wn * WTN + j * 32 + (r >> 2) * 8 + lcol + (r & 3);
          if (n < p.N) Cg[(long)m * p.ldc + n] = acc[i][j][r] + (p.bias ? p.bias[n] : 0.f);
        }
    }
  } else if constexpr (EPI == EPI_SWIGLU) {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = m0 + wm * WTM + i * 32 + lrow;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < TN; j += 2) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + ((wn * WTN + j * 32) >> 1) + q * 8 + lcol;
          if (n >= p.f) continue;
          bf16x4 g, u, a;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            g[t] = static_cast<bf16>(acc[i][j][4 * q + t]);
            u[t] = static_cast<bf16>(acc[i][j + 1][4 * q + t]);
            const float gf = static_cast<float>(g[t]);
            a[t] = static_cast<bf16>(gf * sigmoid_f32(gf) * static_cast<float>(u[t]));
          }
          *reinterpret_cast<bf16x4*>(p.H + (long)m * 2 * p.f + n) = g;
          *reinterpret_cast<bf16x4*>(p.H + (long)m * 2 * p.f + p.f + n) = u;
          *reinterpret_cast<bf16x4*>(p.A_out + (long)m * p.f + n) = a;
        }
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int m = m0 + wm * WTM + i * 32 + lrow;
      if (m >= m_end) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = n0 + wn * WTN + j * 32 + q * 8 + lcol;
          if (n >= p.N) continue;
          const bf16x4 g = *reinterpret_cast<const bf16x4*>(p.H + (long)m * 2 * p.N + n);
          const bf16x4 u = *reinterpret_cast<const bf16x4*>(p.H + (long)m * 2 * p.N + p.N + n);
          bf16x4 dg, du, a;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const float gf = static_cast<float>(g[t]), uf = static_cast<float>(u[t]);
            const float d = static_cast<float>(static_cast<bf16>(acc[i][j][4 * q + t]));
            const float s = sigmoid_f32(gf);
            dg[t] = static_cast<bf16>(d * uf * s * (1.0f + gf * (1.0f - s)));
            du[t] = static_cast<bf16>(d * gf * s);
            a[t] = static_cast<bf16>(gf * s * uf);
          }
          *reinterpret_cast<bf16x4*>(p.dH + (long)m * 2 * p.N + n) = dg;
          *reinterpret_cast<bf16x4*>(p.dH + (long)m * 2 * p.N + p.N + n) = du;
          if (p.A_out) *reinterpret_cast<bf16x4*>(p.A_out + (long)m * p.N + n) = a;
        }
      }
    }
  }
}

template <int BM, int BN, int BKT, int NSTAGE, Layout LA, Layout LB>
constexpr int dma_smem_bytes() {
  return NSTAGE * (DmaTileBytes<LA, BM, BKT>::value + DmaTileBytes<LB, BN, BKT>::value);
}

}  // namespace mfma
}  // namespace moe
