// Grouped GEMM on the gfx950 matrix cores (bf16 inputs, fp32 accumulate): the paper's GroupedGEMM
// operator for FC1 / FC2 and their gradients (Section 4.1; Section 7 names it, with its dynamic
// per-expert shapes, as the straggler of MoE layers).  One kernel template covers the three
// contraction layouts of the layer:
//   forward   C[rows, N] = A[rows, K] * W[e][N, K]^T     A K-major, B K-major, rows segmented by expert
//   dgrad     C[rows, N] = A[rows, K] * W[e][K, N]       A K-major, B N-major, rows segmented by expert
//   wgrad     C[e][M, N] = P[rows_e, M]^T * Q[rows_e, N] A M-major, B N-major, contraction segmented
// Expert row counts are read from `offsets` on the device; the grid is sized for the worst case and
// surplus blocks exit at once, so no call ever waits for the host to learn a shape.
//
// Tiling: BM x BN x 64 block tiles, WM x WN waves, each wave a grid of 32x32x16 MFMAs.  Operand tiles
// are staged global -> registers -> LDS (double buffered, one barrier per 64-wide k step).  K-major
// tiles sit in LDS as [row][64] with a 16-byte-chunk XOR swizzle and are read with ds_read_b128;
// M/N-major tiles sit as [k][cols] (padded rows) and are read with the transposing LDS load
// ds_read_b64_tr_b16, which hands every lane the four consecutive k it needs for its own column.
// The MFMA is issued with the weight fragment as the first operand, so each lane ends up holding four
// consecutive output columns of one output row and the epilogue stores 8- or 16-byte vectors.
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
enum Epi { EPI_STORE = 0, EPI_SWIGLU = 1, EPI_SWIGLU_BWD = 2, EPI_BIAS_F32 = 3 };

constexpr int BK = 64;
constexpr int MN_PAD = 32;   // bf16 elements of padding per k-row of an M/N-major tile (64 bytes)

struct Args {
  const bf16* A; long lda;           // A operand: K-major [rows, K] or M-major [rows(k), M]
  const bf16* B; long ldb; long b_es; // B operand per expert: K-major [N, K] or N-major [K, N]
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
  unsigned long long* clk_out;       // tuning aid (NULL in the library): per-block {core clocks, 100 MHz ticks}
};

template <int ROWS> struct KMajorTile {   // [ROWS][64] bf16, swizzled
  static constexpr int BYTES = ROWS * BK * 2;
  __device__ static __forceinline__ int offset(int row, int chunk) {
    return row * (BK * 2) + ((chunk ^ ((row >> 1) & 7)) << 4);
  }
};
template <int COLS> struct MNMajorTile {  // [64][COLS + pad] bf16
  static constexpr int STRIDE = (COLS + MN_PAD) * 2;
  static constexpr int BYTES = BK * STRIDE;
};

template <Layout L, int EXTENT> struct TileBytes {
  static constexpr int value = (L == KMAJOR) ? KMajorTile<EXTENT>::BYTES : MNMajorTile<EXTENT>::BYTES;
};

__device__ __forceinline__ bf16x8 lds_read_b128(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }

__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
  typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
  const s16x4 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(p));
  return __builtin_bit_cast(bf16x4, r);
}

// Fragment (32 rows/cols x 16 k) for one MFMA operand out of an LDS tile.
template <Layout L, int EXTENT>
__device__ __forceinline__ bf16x8 read_frag(const char* tile, int base, int kk, int lane) {
  if constexpr (L == KMAJOR) {
    const int row = base + (lane & 31);
    return lds_read_b128(tile + KMajorTile<EXTENT>::offset(row, kk * 2 + (lane >> 5)));
  } else {
    const int g = lane >> 4, i = lane & 15;
    const int krow = kk * 16 + ((g >> 1) << 3) + (i >> 2);
    const int col = base + ((g & 1) << 4) + ((i & 3) << 2);
    const char* p = tile + krow * MNMajorTile<EXTENT>::STRIDE + col * 2;
    const bf16x4 lo = lds_read_tr(p);
    const bf16x4 hi = lds_read_tr(p + 4 * MNMajorTile<EXTENT>::STRIDE);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }
}

template <int BM, int BN, int WM, int WN, Layout LA, Layout LB, Mode MODE, Epi EPI, typename TC>
__global__ void __launch_bounds__(WM * WN * 64) grouped_gemm_kernel(Args p) {
  constexpr int NT = WM * WN * 64;
  constexpr int WTM = BM / WM, WTN = BN / WN;          // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;          // MFMA tiles per wave
  constexpr int A_BYTES = TileBytes<LA, BM>::value, B_BYTES = TileBytes<LB, BN>::value;
  constexpr int A_VECS = BM * BK / 8 / NT, B_VECS = BN * BK / 8 / NT;   // 16-byte loads per thread
  static_assert(BM * BK / 8 % NT == 0 && BN * BK / 8 % NT == 0, "tile/threads mismatch");
  static_assert(EPI != EPI_SWIGLU || TN % 2 == 0, "SwiGLU pairs gate/up MFMA tiles inside a wave");

  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int STAGE_BYTES = A_BYTES + B_BYTES;   // stage s: A tile at s*STAGE_BYTES, B tile right after it

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  // ---- which tile is mine -----------------------------------------------------------------
  constexpr int BN_OUT = (EPI == EPI_SWIGLU) ? BN / 2 : BN;   // output columns covered per block
  const int tiles_n = (p.N + BN_OUT - 1) / BN_OUT;
  int e, m0, m_end, k_begin, k_end;
  const int nt = blockIdx.x % tiles_n;
  int rest = blockIdx.x / tiles_n;
  if constexpr (MODE == ROWSEG) {
    bool found = false;
    for (e = 0; e < p.E; ++e) {
      const int lo = p.offsets[e], hi = p.offsets[e + 1];
      const int te = (hi - lo + BM - 1) / BM;
      if (rest < te) { m0 = lo + rest * BM; m_end = hi; found = true; break; }
      rest -= te;
    }
    if (!found) return;
    k_begin = 0; k_end = p.K;
  } else {
    const int tiles_m = (p.M + BM - 1) / BM;
    e = rest / tiles_m;
    m0 = (rest % tiles_m) * BM; m_end = p.M;
    k_begin = p.offsets[e]; k_end = p.offsets[e + 1];
  }
  const int n0 = nt * BN_OUT;
  const bf16* __restrict__ Ag = p.A;
  const bf16* __restrict__ Bg = p.B + (long)e * p.b_es;

  // ---- global -> register staging -----------------------------------------------------------
  uint4 a_reg[A_VECS], b_reg[B_VECS];
  const int last_row_a = (MODE == ROWSEG) ? p.M - 1 : 0;

  auto load_tiles = [&](int k0) {
#pragma unroll
    for (int i = 0; i < A_VECS; ++i) {
      const int idx = tid + i * NT;
      uint4 v = make_uint4(0, 0, 0, 0);
      if constexpr (LA == KMAJOR) {
        const int row = idx >> 3, ch = idx & 7;
        const int gr = min(m0 + row, last_row_a);
        if (k0 + ch * 8 < k_end) v = *reinterpret_cast<const uint4*>(Ag + (long)gr * p.lda + k0 + ch * 8);
      } else {
        constexpr int CPR = BM / 8;
        const int kr = idx / CPR, ch = idx % CPR;
        if (k0 + kr < k_end && m0 + ch * 8 < m_end)
          v = *reinterpret_cast<const uint4*>(Ag + (long)(k0 + kr) * p.lda + m0 + ch * 8);
      }
      a_reg[i] = v;
    }
#pragma unroll
    for (int i = 0; i < B_VECS; ++i) {
      const int idx = tid + i * NT;
      uint4 v = make_uint4(0, 0, 0, 0);
      if constexpr (LB == KMAJOR) {
        const int row = idx >> 3, ch = idx & 7;
        int gr;
        if constexpr (EPI == EPI_SWIGLU) {
          const int q = row >> 5;
          const int n = min(n0 + (q >> 1) * 32 + (row & 31), p.f - 1);
          gr = (q & 1) ? p.f + n : n;
        } else {
          gr = min(n0 + row, p.N - 1);
        }
        if (k0 + ch * 8 < k_end) v = *reinterpret_cast<const uint4*>(Bg + (long)gr * p.ldb + k0 + ch * 8);
      } else {
        constexpr int CPR = BN / 8;
        const int kr = idx / CPR, ch = idx % CPR;
        if (k0 + kr < k_end && n0 + ch * 8 < p.N)
          v = *reinterpret_cast<const uint4*>(Bg + (long)(k0 + kr) * p.ldb + n0 + ch * 8);
      }
      b_reg[i] = v;
    }
  };

  auto store_tiles = [&](int buf) {
#pragma unroll
    for (int i = 0; i < A_VECS; ++i) {
      const int idx = tid + i * NT;
      int off;
      if constexpr (LA == KMAJOR) off = KMajorTile<BM>::offset(idx >> 3, idx & 7);
      else off = (idx / (BM / 8)) * MNMajorTile<BM>::STRIDE + (idx % (BM / 8)) * 16;
      *reinterpret_cast<uint4*>(smem + buf * STAGE_BYTES + off) = a_reg[i];
    }
#pragma unroll
    for (int i = 0; i < B_VECS; ++i) {
      const int idx = tid + i * NT;
      int off;
      if constexpr (LB == KMAJOR) off = KMajorTile<BN>::offset(idx >> 3, idx & 7);
      else off = (idx / (BN / 8)) * MNMajorTile<BN>::STRIDE + (idx % (BN / 8)) * 16;
      *reinterpret_cast<uint4*>(smem + buf * STAGE_BYTES + A_BYTES + off) = b_reg[i];
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- main loop ------------------------------------------------------------------------------
  const int nk = (k_end - k_begin + BK - 1) / BK;
  if (nk > 0) {
    load_tiles(k_begin);
    store_tiles(0);
    __syncthreads();
  }
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_tiles(k_begin + (kt + 1) * BK);
    const char* at = smem + buf * STAGE_BYTES;
    const char* bt = at + A_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = read_frag<LA, BM>(at, wm * WTM + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = read_frag<LB, BN>(bt, wn * WTN + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_tiles(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: lane holds output row m = base + lane%32 and columns 8q + 4(lane/32) + 0..3 ----
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
          Vec16<TC> o;   // only the first 4 elements are used
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
  } else if constexpr (EPI == EPI_SWIGLU) {
    // MFMA tile 2j holds G and tile 2j+1 holds U for the same 32 output columns.
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
    // acc = dA; read G|U, write dG|dU and the recomputed SwiGLU output
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

template <int BM, int BN, Layout LA, Layout LB>
constexpr int smem_bytes() { return 2 * (TileBytes<LA, BM>::value + TileBytes<LB, BN>::value); }

}  // namespace mfma
}  // namespace moe
