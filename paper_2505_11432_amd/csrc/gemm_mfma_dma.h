// Grouped bf16 GEMM on the gfx950 matrix cores with an asynchronous global->LDS pipeline.
//
// Same contract and tile geometry as gemm_mfma.h (the paper's GroupedGEMM operator, Section 4.1, in
// its three contraction layouts), but operand tiles travel global -> LDS directly
// (global_load_lds_dwordx4) into an NSTAGE-deep ring, so loads for k-step s+NSTAGE-1 are in flight
// while k-step s is on the matrix cores, no VGPRs stage the tiles and no ds_write phase exists.
// One s_barrier per k-step: after it every wave's loads for the step have landed and every wave has
// left the previous step, whose buffer the new loads may overwrite.
//
// The kernel is persistent: one workgroup per CU walks a static list of tiles.  When the last k-step of
// a tile is done the ring is free, so the first stages of the NEXT tile are put in flight before the
// current tile's epilogue runs; workgroup launch, tile lookup, pointer set-up and the cold first loads
// all disappear behind the epilogue's stores.
//
// A direct-to-LDS load deposits the wave's 64 x 16 bytes contiguously, so the LDS swizzles are applied
// on the global side: the lane that owns physical chunk pc of a row fetches logical chunk pc ^ swz(row).
//   K-major tile [rows][BKT]:  swz = (row / rows_per_256B) mod chunks_per_row  -> ds_read_b128 conflict-free
//   M/N-major tile [BKT][cols]: swz = 4 * (k mod 4)                            -> ds_read_b64_tr_b16 conflict-free
// Loads that fall outside the contraction range fetch from a 16-byte zero block instead, which gives
// the exact zero fill that ragged expert segments (wgrad) and K tails need.
#pragma once
#include <type_traits>

#include "gemm_mfma.h"

namespace moe {
namespace mfma {

static __device__ __attribute__((aligned(16))) const unsigned int g_zero_block[4] = {0u, 0u, 0u, 0u};

// One wave-wide direct-to-LDS load: lane i's 16 bytes land at lds_addr + 16*i.  lds_addr is wave-uniform.
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_addr) {
  // No "memory" clobber: the LDS write is asynchronous anyway and is ordered by wait_vmcnt + s_barrier, and
  // without it the compiler stays free to hoist LDS fragment reads of the current stage across the load.
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gptr), "s"(lds_addr) : "m0");
}

// The same load with the address split into a wave-uniform 64-bit base (scalar registers) and a 32-bit per-lane
// byte offset: the per-k-step address update is then scalar arithmetic, and issuing the load needs no vector ALU
// slot (those are what the SIMD partner's MFMAs compete for).
__device__ __forceinline__ void dma16s(const char* sbase, unsigned voff, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_addr) : "m0");
}

// One wave-wide 4-byte direct-to-LDS load whose data nobody reads (it lands in a dump area): its only effect is to
// bring the 64 lines it touches into this XCD's L2 ahead of the tile loads that need them.
__device__ __forceinline__ void touch4s(const char* sbase, unsigned voff, unsigned lds_dump) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_dump) : "m0");
}

// Sixteen of those loads in one block: eight from sbase_a, then eight from sbase_b, into LDS slots that lie a fixed
// 4 KiB apart from lds_first on (a 32 KiB A tile followed by the B tile, four loader waves).  M0 is stepped with
// scalar adds inside the block, so the sixteen slot addresses need no registers of their own (kept as sixteen
// loop-invariant scalars they were spilled to vector lanes and read back with v_readlane before every load).
__device__ __forceinline__ void dma16s_x16(const char* sbase_a, const char* sbase_b, const unsigned (&va)[8],
                                           const unsigned (&vb)[8], unsigned lds_first) {
  asm volatile(
      "s_mov_b32 m0, %18\n\t"
      "global_load_lds_dwordx4 %0, %16\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %1, %16\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %2, %16\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %3, %16\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %4, %16\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %5, %16\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %6, %16\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %7, %16\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %8, %17\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %9, %17\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %10, %17\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %11, %17\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %12, %17\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %13, %17\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %14, %17\n\ts_add_u32 m0, m0, 0x1000\n\t"
      "global_load_lds_dwordx4 %15, %17"
      ::"v"(va[0]), "v"(va[1]), "v"(va[2]), "v"(va[3]), "v"(va[4]), "v"(va[5]), "v"(va[6]), "v"(va[7]),
        "v"(vb[0]), "v"(vb[1]), "v"(vb[2]), "v"(vb[3]), "v"(vb[4]), "v"(vb[5]), "v"(vb[6]), "v"(vb[7]),
        "s"(sbase_a), "s"(sbase_b), "s"(lds_first)
      : "m0", "scc");
}

__device__ __forceinline__ const char* uniform_ptr(const char* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const char*>(((unsigned long long)hi << 32) | lo);
}

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  // gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]; other counters left open
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

template <int ROWS, int BKT, int ESZ = 2> struct KTile {        // K-major [ROWS][BKT] of ESZ-byte elements
  static constexpr int ROW_BYTES = BKT * ESZ, CPR = ROW_BYTES / 16, RPL = 256 / ROW_BYTES;
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

template <Layout L, int EXTENT, int BKT, int ESZ = 2> struct DmaTileBytes;
template <int EXTENT, int BKT, int ESZ> struct DmaTileBytes<KMAJOR, EXTENT, BKT, ESZ> { static constexpr int value = KTile<EXTENT, BKT, ESZ>::BYTES; };
template <int EXTENT, int BKT, int ESZ> struct DmaTileBytes<MNMAJOR, EXTENT, BKT, ESZ> {
  static_assert(ESZ == 2, "M/N-major tiles exist for bf16 only");
  static constexpr int value = MNTile<EXTENT, BKT>::BYTES;
};

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


// ---- epilogue staging --------------------------------------------------------------------------------
// After the MFMA (weight fragment first) a lane holds one output row (lane % 32) and columns
// 8q + 4*(lane/32) + 0..3 (q = 0..3) of a 32x32 tile: a direct store would touch 32 rows with 16 bytes
// each.  Each wave therefore owns a small LDS patch of 32 rows x 64 bytes; tiles pass through it so that
// global memory sees 16-byte lanes forming 64-byte row segments (4 lanes per row, 16 rows per instruction).
constexpr int STG_STRIDE = 80;                  // bytes per staged row (64 payload + 16 pad)
constexpr int STG_BYTES = 32 * STG_STRIDE;      // per wave

// Global accesses of the epilogues are raw buffer instructions on a descriptor that starts at the block's origin
// (wave-uniform): a lane outside the valid rows or columns gets an offset past the end of the buffer, which the
// hardware answers with zeros (loads) or drops (stores).  No lane-dependent branch surrounds a memory instruction, so
// every wave issues the same, known number of them and the compiler's s_waitcnt vmcnt(n) stay exact: with stores
// inside `if (valid)` blocks it has to assume that none was issued and waits for vmcnt(0), i.e. for every store of
// the previous block, before each read.
typedef unsigned int u32x4v __attribute__((ext_vector_type(4)));
constexpr unsigned BUF_SPAN = 0x40000000u;      // 1 GiB from the block origin; a 32-row block spans far less
constexpr unsigned BUF_OOB = 0x80000000u;       // offset of a masked lane
__device__ __forceinline__ __amdgpu_buffer_rsrc_t block_rsrc(const void* origin) {
  char* base = const_cast<char*>(uniform_ptr(static_cast<const char*>(origin)));
  return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)BUF_SPAN, 0x00020000);   // raw buffer, 32-bit data format
}
__device__ __forceinline__ unsigned block_offset(int r, int c, long ld, int esz, int rows_valid, int cols_valid) {
  return (r < rows_valid && c < cols_valid) ? (unsigned)(((long)r * ld + c) * esz) : BUF_OOB;
}

// 32 rows x 32 bf16 columns from registers to global memory (row-major, leading dimension ld elements).
__device__ __forceinline__ void stage_store_bf16(char* stg, const bf16x4 (&v)[4], bf16* g, long ld, int rows_valid,
                                                 int cols_valid, int lane) {
  const int row = lane & 31, h = lane >> 5;
#pragma unroll
  for (int q = 0; q < 4; ++q) *reinterpret_cast<bf16x4*>(stg + row * STG_STRIDE + (8 * q + 4 * h) * 2) = v[q];
  const __amdgpu_buffer_rsrc_t rs = block_rsrc(g);
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = pass * 16 + (lane >> 2), c = (lane & 3) * 8;
    const u32x4v val = *reinterpret_cast<const u32x4v*>(stg + r * STG_STRIDE + c * 2);
    __builtin_amdgcn_raw_buffer_store_b128(val, rs, block_offset(r, c, ld, 2, rows_valid, cols_valid), 0, 0);
  }
}

// 32 rows x 32 bf16 columns from global memory into registers (same lane layout as the accumulators).
__device__ __forceinline__ void stage_load_bf16(char* stg, bf16x4 (&v)[4], const bf16* g, long ld, int rows_valid,
                                                int cols_valid, int lane) {
  const __amdgpu_buffer_rsrc_t rs = block_rsrc(g);
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = pass * 16 + (lane >> 2), c = (lane & 3) * 8;
    const u32x4v val = __builtin_amdgcn_raw_buffer_load_b128(rs, block_offset(r, c, ld, 2, rows_valid, cols_valid), 0, 0);
    *reinterpret_cast<u32x4v*>(stg + r * STG_STRIDE + c * 2) = val;
  }
  const int row = lane & 31, h = lane >> 5;
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const bf16x4*>(stg + row * STG_STRIDE + (8 * q + 4 * h) * 2);
}

// The same load in two phases, so that the global reads of the next 32x32 block can be in flight while the
// current block is processed: fetch (global -> registers, zero where masked) and unpack (registers -> LDS patch ->
// accumulator lane layout).
struct StageFetch { u32x4v v[2]; };
__device__ __forceinline__ StageFetch stage_fetch_bf16(const bf16* g, long ld, int rows_valid, int cols_valid, int lane) {
  StageFetch f;
  const __amdgpu_buffer_rsrc_t rs = block_rsrc(g);
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = pass * 16 + (lane >> 2), c = (lane & 3) * 8;
    f.v[pass] = __builtin_amdgcn_raw_buffer_load_b128(rs, block_offset(r, c, ld, 2, rows_valid, cols_valid), 0, 0);
  }
  return f;
}
__device__ __forceinline__ void stage_unpack_bf16(char* stg, const StageFetch& f, bf16x4 (&v)[4], int lane) {
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = pass * 16 + (lane >> 2), c = (lane & 3) * 8;
    *reinterpret_cast<u32x4v*>(stg + r * STG_STRIDE + c * 2) = f.v[pass];
  }
  const int row = lane & 31, h = lane >> 5;
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const bf16x4*>(stg + row * STG_STRIDE + (8 * q + 4 * h) * 2);
}

// 32 rows x 32 fp32 columns, as two halves of 16 columns; optional read-modify-write accumulation.
__device__ __forceinline__ void stage_store_f32(char* stg, const f32x16& acc, float* g, long ld, int rows_valid,
                                                int cols_valid, bool accumulate, int lane) {
  const int row = lane & 31, h = lane >> 5;
  const __amdgpu_buffer_rsrc_t rs = block_rsrc(g);
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
      const int q = half * 2 + qq;
      const f32x4 t = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
      *reinterpret_cast<f32x4*>(stg + row * STG_STRIDE + (8 * qq + 4 * h) * 4) = t;
    }
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int r = pass * 16 + (lane >> 2), c = half * 16 + (lane & 3) * 4;
      f32x4 val = *reinterpret_cast<const f32x4*>(stg + r * STG_STRIDE + (lane & 3) * 16);
      const unsigned off = block_offset(r, c, ld, 4, rows_valid, cols_valid);
      if (accumulate) val += __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0));   // (uniform)
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4v, val), rs, off, 0, 0);
    }
  }
}

// ---- the same three with plain global accesses inside `if (valid)` (the e4m3 kernels: their register budget does
// not take the descriptors)
// 32 rows x 32 bf16 columns from registers to global memory (row-major, leading dimension ld elements).
__device__ __forceinline__ void stage_store_bf16_g(char* stg, const bf16x4 (&v)[4], bf16* g, long ld, int rows_valid,
                                                 int cols_valid, int lane) {
  const int row = lane & 31, h = lane >> 5;
#pragma unroll
  for (int q = 0; q < 4; ++q) *reinterpret_cast<bf16x4*>(stg + row * STG_STRIDE + (8 * q + 4 * h) * 2) = v[q];
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = pass * 16 + (lane >> 2), c = (lane & 3) * 8;
    const uint4 val = *reinterpret_cast<const uint4*>(stg + r * STG_STRIDE + c * 2);
    if (r < rows_valid && c < cols_valid) *reinterpret_cast<uint4*>(g + (long)r * ld + c) = val;
  }
}

// 32 rows x 32 bf16 columns from global memory into registers (same lane layout as the accumulators).
__device__ __forceinline__ void stage_load_bf16_g(char* stg, bf16x4 (&v)[4], const bf16* g, long ld, int rows_valid,
                                                int cols_valid, int lane) {
#pragma unroll
  for (int pass = 0; pass < 2; ++pass) {
    const int r = pass * 16 + (lane >> 2), c = (lane & 3) * 8;
    uint4 val = make_uint4(0, 0, 0, 0);
    if (r < rows_valid && c < cols_valid) val = *reinterpret_cast<const uint4*>(g + (long)r * ld + c);
    *reinterpret_cast<uint4*>(stg + r * STG_STRIDE + c * 2) = val;
  }
  const int row = lane & 31, h = lane >> 5;
#pragma unroll
  for (int q = 0; q < 4; ++q) v[q] = *reinterpret_cast<const bf16x4*>(stg + row * STG_STRIDE + (8 * q + 4 * h) * 2);
}

// 32 rows x 32 fp32 columns, as two halves of 16 columns; optional read-modify-write accumulation.
__device__ __forceinline__ void stage_store_f32_g(char* stg, const f32x16& acc, float* g, long ld, int rows_valid,
                                                int cols_valid, bool accumulate, int lane) {
  const int row = lane & 31, h = lane >> 5;
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int qq = 0; qq < 2; ++qq) {
      const int q = half * 2 + qq;
      const f32x4 t = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
      *reinterpret_cast<f32x4*>(stg + row * STG_STRIDE + (8 * qq + 4 * h) * 4) = t;
    }
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      const int r = pass * 16 + (lane >> 2), c = half * 16 + (lane & 3) * 4;
      f32x4 val = *reinterpret_cast<const f32x4*>(stg + r * STG_STRIDE + (lane & 3) * 16);
      if (r < rows_valid && c < cols_valid) {
        float* dst = g + (long)r * ld + c;
        if (accumulate) val += *reinterpret_cast<const f32x4*>(dst);
        *reinterpret_cast<f32x4*>(dst) = val;
      }
    }
  }
}

// e4m3 fragment (32 rows x 64 k, 32 bytes per lane) for the 32x32x64 f8f6f4 MFMA out of a K-major tile.
template <int EXTENT, int BKT>
__device__ __forceinline__ i32x8 read_frag_fp8(const char* tile, int base, int kk, int lane) {
  using TL = KTile<EXTENT, BKT, 1>;
  const int row = base + (lane & 31);
  const int c0 = kk * 4 + ((lane >> 5) << 1);
  const uint4 lo = *reinterpret_cast<const uint4*>(tile + TL::offset(row, c0));
  const uint4 hi = *reinterpret_cast<const uint4*>(tile + TL::offset(row, c0 + 1));
  i32x8 r = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, (int)hi.z, (int)hi.w};
  return r;
}

// Work list with the last round split along K: tiles [0, full_tiles) are whole; each of the remaining
// total_tiles - full_tiles tiles becomes `split` items.  No split unless it at least halves the last round.
__host__ __device__ __forceinline__ void splitk_plan(int total_tiles, int workgroups, int& full_tiles, int& split, int& total_items) {
  full_tiles = total_tiles / workgroups * workgroups;
  const int rem = total_tiles - full_tiles;
  split = 1;
  if (rem > 0 && workgroups / rem >= 2) split = workgroups / rem >= 4 ? 4 : workgroups / rem;
  if (split == 1) full_tiles = total_tiles;
  total_items = full_tiles + (total_tiles - full_tiles) * split;
}

// Adds the K parts of every split tile and writes the bf16 result with the tile's row / column masks.  Four
// workgroups per split tile; the tile list is rebuilt exactly as in the GEMM kernel (same grouping constants).
template <int BM, int BN>
__global__ void __launch_bounds__(256) splitk_fixup_kernel(const float* __restrict__ parts, const int32_t* __restrict__ offsets,
                                                           int E, int N, int gemm_workgroups, bf16* __restrict__ C, long ldc) {
  constexpr int GN = 8;
  __shared__ int cum_tiles[MOE_MAX_EXPERTS + 1];
  if (threadIdx.x == 0) {
    int run = 0;
    cum_tiles[0] = 0;
    for (int i = 0; i < E; ++i) {
      run += (offsets[i + 1] - offsets[i] + BM - 1) / BM;
      cum_tiles[i + 1] = run;
    }
  }
  __syncthreads();
  const int tiles_n = (N + BN - 1) / BN;
  const int total_tiles = cum_tiles[E] * tiles_n;
  int full_tiles, split, total_items;
  splitk_plan(total_tiles, gemm_workgroups, full_tiles, split, total_items);
  constexpr int SLICES = 4;                          // workgroups per split tile (each takes BM / SLICES rows)
  const int r_tile = blockIdx.x / SLICES, slice = blockIdx.x % SLICES;
  if (split == 1 || r_tile >= total_tiles - full_tiles) return;
  int l = full_tiles + r_tile;
  int lo = 0, hi = E;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cum_tiles[mid] * tiles_n <= l) lo = mid; else hi = mid;
  }
  const int e = lo;
  const int mt_e = cum_tiles[e + 1] - cum_tiles[e];
  l -= cum_tiles[e] * tiles_n;
  const int ng = l / (mt_e * GN);
  const int r = l - ng * mt_e * GN;
  const int gw = min(GN, tiles_n - ng * GN);
  const int mt = r / gw;
  const int nt = ng * GN + (r - mt * gw);
  const int m0 = offsets[e] + mt * BM, m_end = offsets[e + 1], n0 = nt * BN;
  const float* base = parts + (long)r_tile * split * (BM * BN);
  for (int i = threadIdx.x; i < (BM / SLICES) * BN / 8; i += blockDim.x) {
    const int row = slice * (BM / SLICES) + i / (BN / 8), col = (i % (BN / 8)) * 8;
    if (m0 + row >= m_end || n0 + col >= N) continue;          // N is a multiple of 8
    float v[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) v[q] = 0.f;
    for (int s = 0; s < split; ++s) {
      const f32x4 a = *reinterpret_cast<const f32x4*>(base + (long)s * (BM * BN) + row * BN + col);
      const f32x4 b = *reinterpret_cast<const f32x4*>(base + (long)s * (BM * BN) + row * BN + col + 4);
#pragma unroll
      for (int q = 0; q < 4; ++q) { v[q] += a[q]; v[4 + q] += b[q]; }
    }
    bf16x8 o;
#pragma unroll
    for (int q = 0; q < 8; ++q) o[q] = static_cast<bf16>(v[q]);
    *reinterpret_cast<bf16x8*>(C + (long)(m0 + row) * ldc + n0 + col) = o;
  }
}

template <int BM, int BN, int BKT, int NSTAGE, int WM, int WN, Layout LA, Layout LB, Mode MODE, Epi EPI, typename TC,
          typename TIN = bf16>   // TIN = uint8_t: e4m3 codes, K-major operands only
__global__ void __launch_bounds__(WM * WN * 64) grouped_gemm_dma_kernel(Args p) {
  constexpr int NW = WM * WN;
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int ESZ = sizeof(TIN);
  constexpr bool FP8 = ESZ == 1;
  constexpr int CHUNK = 16 / ESZ;                     // elements per 16-byte chunk
  static_assert(!FP8 || (LA == KMAJOR && LB == KMAJOR), "e4m3 operands are K-major");
  constexpr bool BSCALE = FP8 && MODE == KSEG;        // block-scaled contraction over tokens (weight gradients)
  static_assert(!BSCALE || (BKT == 128 && NSTAGE == 2), "one 128-token scale group per k-step; scale loads rely on the vmcnt(0) wait");
  constexpr int A_BYTES = DmaTileBytes<LA, BM, BKT, ESZ>::value, B_BYTES = DmaTileBytes<LB, BN, BKT, ESZ>::value;
  constexpr int STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int RING_BYTES = NSTAGE * STAGE_BYTES;
  // With 8 waves (two per SIMD; waves w and w + 4 share one) only the lower four issue loads: a wave stalls while
  // the texture-address queue is full (64 loads take ~1100 clocks), and this way its SIMD partner runs MFMAs
  // meanwhile.  Smaller workgroups (one wave per SIMD) let every wave load.
  constexpr bool SPLIT = (NW == 8);
  constexpr int NL = SPLIT ? NW / 2 : NW;                                      // loader waves
  constexpr int A_DMA = A_BYTES / 1024 / NL, B_DMA = B_BYTES / 1024 / NL;     // loads per loader wave per stage
  constexpr int LOADS = A_DMA + B_DMA;
  constexpr int KK = FP8 ? BKT / 64 : BKT / 16;    // MFMA sub-steps per k-step
  constexpr bool SWI = EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_W;              // FC1 + SwiGLU epilogue
  constexpr bool FOLD = EPI == EPI_SWIGLU_W || EPI == EPI_SWIGLU_BWD_W;       // gate weight folded in (Section 4.1)
  constexpr bool GATHER_A = EPI == EPI_SWIGLU_W;                              // A rows selected by index map (Section 4.2)
  static_assert(!FOLD || (!FP8 && MODE == ROWSEG && LA == KMAJOR), "the folded order exists for the bf16 row-segmented kernels");
  constexpr int BN_OUT = SWI ? BN / 2 : BN;
  // Store instructions a wave issues in the epilogue of a full tile (branch-free buffer stores, bf16 kernels): two
  // per 32x32 bf16 block, four per fp32 block; 0 = not known at compile time.
  constexpr bool PLAIN_EPI = FP8 && !(MODE == ROWSEG && (SWI || EPI == EPI_STORE));   // epilogue with plain (branchy) global accesses
  constexpr int EPI_STORES_RAW = PLAIN_EPI ? 0
                                 : EPI == EPI_STORE ? TM * TN * (sizeof(TC) == 4 ? 4 : 2)
                                 : SWI ? TM * TN * 3
                                 : EPI == EPI_SWIGLU_BWD ? TM * TN * 6
                                 : EPI == EPI_SWIGLU_BWD_W ? TM * TN * 6 + TM
                                 : 0;
  constexpr int EPI_STORES = (NSTAGE - 2) * LOADS + EPI_STORES_RAW <= 63 ? EPI_STORES_RAW : 0;   // vmcnt is a 6-bit field
  bool epi_stores = false;         // the previous tile's epilogue issued exactly EPI_STORES stores (wave-uniform)
  constexpr int GN = 8, XCDS = 8;   // GN n-tiles per group: a window of 32 tiles is 4 m-tiles x 8 n-tiles (measured against 8 x 4, 16 x 2, 2 x 16)
  static_assert(A_BYTES % (1024 * NL) == 0 && B_BYTES % (1024 * NL) == 0, "tile does not split over the loader waves");
  static_assert(NSTAGE >= 2 && (NSTAGE - 2) * LOADS < 64, "pipeline depth exceeds the vmcnt range");
  static_assert(!SWI || TN % 2 == 0, "SwiGLU pairs gate/up MFMA tiles inside a wave");
  static_assert(NW <= 8, "LDS is budgeted for at most 8 epilogue patches");

  extern __shared__ __attribute__((aligned(16))) char smem[];
  const unsigned smem_lds = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
  int* cum_tiles = reinterpret_cast<int*>(smem + RING_BYTES);          // [E+1] running count of m-tiles (ROWSEG)
  constexpr int TABLE_BYTES = (MOE_MAX_EXPERTS + 8) * 4;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;
  const char* zero = reinterpret_cast<const char*>(g_zero_block);
  char* stg = smem + RING_BYTES + TABLE_BYTES + wave * STG_BYTES;      // this wave's epilogue patch

  // ---- the tile list ------------------------------------------------------------------------------
  // Workgroup b runs on XCD b % 8 and each XCD has its own L2.  The logical tile order is cut into windows
  // of W = G/8 consecutive tiles (one per CU of an XCD); a window is a compact block of one expert -- GN
  // adjacent n-tiles for a run of m-tiles -- whose tiles stream the same A and B panels at the same k, so
  // most of their loads hit in L2.  Windows are dealt round-robin to the XCDs: at any moment the eight
  // XCDs work on eight neighbouring windows, mostly the next m-tiles of the same n-tiles, i.e. the same B
  // panels (shared through the Infinity Cache) and disjoint A panels.
  const int tiles_n = (p.N + BN_OUT - 1) / BN_OUT;
  const int tiles_m_fixed = (p.M + BM - 1) / BM;              // KSEG / PLAIN
  int total_tiles;
  if constexpr (MODE == ROWSEG) {
    if (tid == 0) {
      int run = 0;
      cum_tiles[0] = 0;
      for (int i = 0; i < p.E; ++i) {
        run += (p.offsets[i + 1] - p.offsets[i] + BM - 1) / BM;
        cum_tiles[i + 1] = run;
      }
    }
    __syncthreads();
    total_tiles = __builtin_amdgcn_readfirstlane(cum_tiles[p.E]) * tiles_n;
  } else if constexpr (MODE == KSEG) {
    total_tiles = p.E * tiles_m_fixed * tiles_n;
  } else {
    total_tiles = tiles_m_fixed * tiles_n;
  }
  // split-K plan for the partly filled last round (see Args::splitk_ws); identical arithmetic in splitk_fixup_kernel
  constexpr bool SPLITK = MODE == ROWSEG && EPI == EPI_STORE && sizeof(TC) == 2;
  int full_tiles = total_tiles, split = 1, total_items = total_tiles;
  if constexpr (SPLITK) {
    if (p.splitk_ws != nullptr) splitk_plan(total_tiles, (int)gridDim.x, full_tiles, split, total_items);
  }
  const int xcd = blockIdx.x % XCDS;
  const int window = gridDim.x / XCDS;           // tiles per window = CUs per XCD
  const int in_window = blockIdx.x / XCDS;
  int slot = 0;                                  // this XCD's window counter

  // tile state
  int e = 0, m0 = 0, m_end = 0, n0 = 0, klen = 0, nk = 0;
  int part_slot = -1;               // >= 0: this work item is one K part of a split tile; index of its partial tile
  const bool is_loader = !SPLIT || wave < NL;            // wave-uniform; the lower waves win issue arbitration
  const int lw = wave & (NL - 1);                        // loader index
  const char* a_base = zero;        // wave-uniform: operand origin of the open tile at its first k
  const char* b_base = zero;
  unsigned a_off[A_DMA], b_off[B_DMA];   // this lane's byte offset from the base, fixed over the k loop
  int a_k[A_DMA], b_k[B_DMA];       // k coordinate (relative to the k-step start) this lane's chunk begins at
  // L2 touches (bf16 kernels).  The workgroups of a window stream the same A and B panels at the same k, so every
  // new line is requested by several of them at once and all of them wait for the one fill.  At the end of k-step kt
  // the first wave that does not load (wave NL) touches this workgroup's quarter of the A-panel lines that the
  // loader waves request next (the n-tiles of a group share the A panel; quarter = position in the group mod 4).
  // Measured: touches at the start of a step queue behind the tile loads in the texture-address unit (kernel 16 %
  // slower); at the end of the step they gain 1.2 to 3 %; one or two steps further ahead: no change; touching the B
  // panel as well, or half of A, or from two waves: slower again (each touch instruction costs the address unit as
  // much as a 1 KB tile load).  Not for e4m3 operands: half the time per k-step for the same loads, touches cost 2 %.
  constexpr bool TOUCH = MODE == ROWSEG && NSTAGE == 2 && SPLIT && !FP8;
  // the same for the bf16 weight-gradient kernel (four stages of 32 k-rows): two k-steps per touch, every other step
  constexpr bool TOUCH_K = MODE == KSEG && !FP8 && SPLIT && LA == MNMAJOR && LB == MNMAJOR && NSTAGE == 4;
  constexpr bool TOUCH_K2 = MODE == KSEG && !FP8 && SPLIT && LA == MNMAJOR && LB == MNMAJOR && NSTAGE == 2 && BKT == 64;
  const bool is_toucher = (TOUCH || TOUCH_K || TOUCH_K2) && wave == NL;
  const unsigned lds_dump = smem_lds + RING_BYTES + TABLE_BYTES + 8 * STG_BYTES;
  const unsigned scale_lds = lds_dump + 256;                                   // block-scale ring: 2 stages x (256 + 256) bytes
  const char* scale_smem = smem + RING_BYTES + TABLE_BYTES + 8 * STG_BYTES + 256;
  unsigned ta_off = 0;
  // rotation of this workgroup's load order within the A / B tile (see open_tile); only where it pays: the e4m3
  // row-segmented kernels (in the others the extra scalar state pushes tile offsets out of registers)
  constexpr bool ROT = FP8 && MODE == ROWSEG;
  int rot_a = 0, rot_b = 0;
  // block scales of the current and the next k-step for this lane's fragment rows (byte 0 of each register)
  // Block scales (e4m3 weight gradients): the 256 + 256 E8M0 bytes of a k-step travel global -> LDS with the tiles
  // (two 4-byte direct-to-LDS loads by loader wave 0, into a two-stage ring of 512 bytes) and every wave reads its
  // rows' bytes from there.  Fetching them per lane from global memory took six more vector-memory instructions per
  // wave and k-step, 48 per workgroup next to the 64 tile loads, and the address unit is what the load issue is
  // bound by: the k-step was 0.4 us longer.
  static_assert(!BSCALE || (BM == 256 && BN == 256), "one 4-byte load per lane covers the 256 channels of a tile side");
  int sa_cur[TM], sb_cur[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) sa_cur[i] = 127;
#pragma unroll
  for (int j = 0; j < TN; ++j) sb_cur[j] = 127;
  const char* sa_base = nullptr;        // scale row of the tile's first k-step (wave-uniform)
  const char* sb_base = nullptr;
  unsigned sa_voff = 0, sb_voff = 0;    // this lane's four channels
  const long a_step = (LA == KMAJOR) ? (long)BKT * ESZ : (long)BKT * p.lda * ESZ;   // bytes per k-step
  const long b_step = (LB == KMAJOR) ? (long)BKT * ESZ : (long)BKT * p.ldb * ESZ;

  // Decode slot -> tile and set up this lane's source pointers.  Returns false when the list is exhausted.
  auto open_tile = [&](int sl) __attribute__((always_inline)) -> bool {
    int l = (sl * XCDS + xcd) * window + in_window;
    if (l >= total_items) return false;
    int part = 0;
    part_slot = -1;
    if (l >= full_tiles) {           // only with SPLITK: parts of one tile are neighbours in the list
      part_slot = l - full_tiles;
      part = part_slot % split;
      l = full_tiles + part_slot / split;
    }
    int mt_e, m_lo, m_hi;
    if constexpr (MODE == ROWSEG) {
      // binary search: largest ex with cum_tiles[ex] * tiles_n <= l
      int lo = 0, hi = p.E;
      while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cum_tiles[mid] * tiles_n <= l) lo = mid; else hi = mid;
      }
      // everything about the tile is wave-uniform: keep it in scalar registers
      e = __builtin_amdgcn_readfirstlane(lo);
      mt_e = __builtin_amdgcn_readfirstlane(cum_tiles[e + 1] - cum_tiles[e]);
      l = __builtin_amdgcn_readfirstlane(l - cum_tiles[e] * tiles_n);
      m_lo = p.offsets[e]; m_hi = p.offsets[e + 1];
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
    m0 = m_lo + mt * BM; m_end = m_hi; n0 = nt * BN_OUT;
    // Sharers of a panel start their loads at different quarters of it (the n-tiles of a group share A, the m-tiles
    // of a window share B), so that the first request for each new line, the one that starts its L2 fill, is spread
    // over the sharers and over the step instead of all of them queueing on the same line in the same order.
    if constexpr (ROT) {
      rot_a = __builtin_amdgcn_readfirstlane(((r - mt * gw) & 3) * A_DMA / 4);
      rot_b = __builtin_amdgcn_readfirstlane((mt & 3) * B_DMA / 4);
    }
    int k_begin, k_end;
    if constexpr (MODE == KSEG) { k_begin = p.offsets[e]; k_end = p.offsets[e + 1]; }
    else { k_begin = 0; k_end = p.K; }
    klen = k_end - k_begin;
    nk = (klen + BKT - 1) / BKT;
    if (part_slot >= 0) {            // this item covers k-steps [s0, s1) of the tile
      const int s0 = part * nk / split, s1 = (part + 1) * nk / split;
      k_begin += s0 * BKT;
      klen = min(klen, s1 * BKT) - s0 * BKT;
      nk = s1 - s0;
    }
    const char* Ag = static_cast<const char*>(p.A);
    const char* Bg = static_cast<const char*>(p.B) + (long)e * p.b_es * ESZ;
    // Base of each operand at the tile's first k (wave-uniform) and this lane's fixed byte offset from it.
    // Load j of loader wave lw fills DMA slot q = lw + j*NL of the tile (1 KiB of LDS each).
    if constexpr (GATHER_A) a_base = uniform_ptr(Ag + (long)k_begin * ESZ);          // row offsets are absolute
    else if constexpr (LA == KMAJOR) a_base = uniform_ptr(Ag + ((long)m0 * p.lda + k_begin) * ESZ);
    else a_base = uniform_ptr(Ag + (long)k_begin * p.lda * ESZ);
    if constexpr (LB == KMAJOR) b_base = uniform_ptr(Bg + (long)k_begin * ESZ);
    else b_base = uniform_ptr(Bg + (long)k_begin * p.ldb * ESZ);
#pragma unroll
    for (int j = 0; j < A_DMA; ++j) {
      const int q = lw + ((j + rot_a) % A_DMA) * NL;
      if constexpr (LA == KMAJOR) {
        using TL = KTile<BM, BKT, ESZ>;
        const int row = q * TL::ROWS_PER_DMA + lane / TL::CPR;
        const int lc = (lane % TL::CPR) ^ TL::swz(row);
        int rel = min(row, p.M - 1 - m0);                             // rows past the end of A repeat its last row
        if constexpr (GATHER_A) rel = p.a_rowmap[m0 + rel];           // < a_phys_rows: the launcher's contract
        a_off[j] = (unsigned)rel * (unsigned)(p.lda * ESZ) + (unsigned)(lc * 16);
        a_k[j] = lc * CHUNK;
      } else {
        using TL = MNTile<BM, BKT>;
        const int krow = q * TL::ROWS_PER_DMA + lane / TL::CPR;
        const int lc = (lane % TL::CPR) ^ TL::swz(krow);
        const int col = min(m0 + lc * 8, p.M - 8);
        a_off[j] = (unsigned)krow * (unsigned)(p.lda * ESZ) + (unsigned)(col * ESZ);
        a_k[j] = krow;
      }
    }
#pragma unroll
    for (int j = 0; j < B_DMA; ++j) {
      const int q = lw + ((j + rot_b) % B_DMA) * NL;
      if constexpr (LB == KMAJOR) {
        using TL = KTile<BN, BKT, ESZ>;
        const int row = q * TL::ROWS_PER_DMA + lane / TL::CPR;
        const int lc = (lane % TL::CPR) ^ TL::swz(row);
        int gr;
        if constexpr (SWI) {
          const int qq = row >> 5;
          const int n = min(n0 + (qq >> 1) * 32 + (row & 31), p.f - 1);
          gr = (qq & 1) ? p.f + n : n;
        } else {
          gr = min(n0 + row, p.N - 1);
        }
        b_off[j] = (unsigned)gr * (unsigned)(p.ldb * ESZ) + (unsigned)(lc * 16);     // < 4 GiB: checked by the launcher
        b_k[j] = lc * CHUNK;
      } else {
        using TL = MNTile<BN, BKT>;
        const int krow = q * TL::ROWS_PER_DMA + lane / TL::CPR;
        const int lc = (lane % TL::CPR) ^ TL::swz(krow);
        const int col = min(n0 + lc * 8, p.N - 8);
        b_off[j] = (unsigned)krow * (unsigned)(p.ldb * ESZ) + (unsigned)(col * ESZ);
        b_k[j] = krow;
      }
    }
    if constexpr (TOUCH) {
      // the gw n-tiles of a group share the A panel: quarter (position in the group mod 4) of its 256 rows, one line per lane
      const int qa = (r - mt * gw) & 3;
      int arow = min(qa * 64 + lane, p.M - 1 - m0);
      if constexpr (GATHER_A) arow = p.a_rowmap[m0 + arow];
      ta_off = (unsigned)arow * (unsigned)(p.lda * ESZ);
    }
    if constexpr (TOUCH_K2) {
      // weight gradient, 64-deep steps: this workgroup's quarter (16 k-rows x 4 lines) of the A tile of one k-step
      const int qa = (r - mt * gw) & 3;
      ta_off = (unsigned)(qa * 16 + (lane >> 2)) * (unsigned)(p.lda * ESZ) + (unsigned)(min(m0 + (lane & 3) * 64, p.M - 8) * ESZ);
    }
    if constexpr (TOUCH_K) {
      // weight gradient, 32-deep steps: lanes 0..31 take this workgroup's quarter (8 k-rows x 4 lines) of the A tile of one k-step,
      // lanes 32..63 the same quarter of the following k-step
      const int qa = (r - mt * gw) & 3;
      const int kr = (lane >> 5) * BKT + (((lane & 31) >> 2));
      ta_off = (unsigned)(kr + qa * 8) * (unsigned)(p.lda * ESZ) + (unsigned)(min(m0 + (lane & 3) * 64, p.M - 8) * ESZ);
    }
    if constexpr (BSCALE) {
      const long g0 = k_begin / BKT;
      sa_base = uniform_ptr(reinterpret_cast<const char*>(p.a_e8m0) + g0 * p.a_e8_ld);
      sb_base = uniform_ptr(reinterpret_cast<const char*>(p.b_e8m0) + g0 * p.b_e8_ld);
      // channels past the end repeat the last four (their rows and columns are masked when the tile is stored)
      sa_voff = (unsigned)min(m0 + 4 * lane, p.M - 4);
      sb_voff = (unsigned)min(n0 + 4 * lane, p.N - 4);
    }
    return true;
  };
  // Issue the loads of k-step `ks` of the open tile into ring slot ks % NSTAGE.  Only the last step can be ragged.
  auto issue = [&](int ks) __attribute__((always_inline)) {
    if (!is_loader) return;
    const unsigned stage = smem_lds + (unsigned)(ks % NSTAGE) * STAGE_BYTES;
    const int k_left = klen - ks * BKT;          // valid k in this step
    const char* ab = a_base + (long)ks * a_step;     // scalar arithmetic
    const char* bb = b_base + (long)ks * b_step;
    if constexpr (BSCALE) {
      if (lw == 0) {
        const unsigned dst = scale_lds + (unsigned)(ks % NSTAGE) * 512u;
        touch4s(sa_base + (long)ks * p.a_e8_ld, sa_voff, dst);
        touch4s(sb_base + (long)ks * p.b_e8_ld, sb_voff, dst + 256u);
      }
    }
    if (k_left >= BKT) {
      // the e4m3 weight-gradient kernel asks for the B tile first, the others for the A tile: measured
      constexpr bool B_FIRST = FP8 && MODE == KSEG;
      if constexpr (A_DMA == 8 && B_DMA == 8 && NL == 4 && A_BYTES == 8 * 4096 && !ROT && !B_FIRST) {
        dma16s_x16(ab, bb, a_off, b_off, stage + (unsigned)lw * 1024u);
      } else {
        if constexpr (B_FIRST) {
#pragma unroll
          for (int j = 0; j < B_DMA; ++j) dma16s(bb, b_off[j], stage + A_BYTES + (unsigned)(lw + ((j + rot_b) % B_DMA) * NL) * 1024u);
        }
#pragma unroll
        for (int j = 0; j < A_DMA; ++j) dma16s(ab, a_off[j], stage + (unsigned)(lw + ((j + rot_a) % A_DMA) * NL) * 1024u);
        if constexpr (!B_FIRST) {
#pragma unroll
          for (int j = 0; j < B_DMA; ++j) dma16s(bb, b_off[j], stage + A_BYTES + (unsigned)(lw + ((j + rot_b) % B_DMA) * NL) * 1024u);
        }
      }
    } else {
      // ragged last step: chunks past the end of the contraction come from the zero block.  The offsets pass
      // through an empty asm so that their 64-bit extensions are made here, in the cold path, instead of being
      // kept in register pairs across the whole k loop.
#pragma unroll
      for (int j = 0; j < A_DMA; ++j) {
        unsigned off = a_off[j];
        asm volatile("" : "+v"(off));
        dma16(a_k[j] >= k_left ? zero : ab + off, stage + (unsigned)(lw + ((j + rot_a) % A_DMA) * NL) * 1024u);
      }
#pragma unroll
      for (int j = 0; j < B_DMA; ++j) {
        unsigned off = b_off[j];
        asm volatile("" : "+v"(off));
        dma16(b_k[j] >= k_left ? zero : bb + off, stage + A_BYTES + (unsigned)(lw + ((j + rot_b) % B_DMA) * NL) * 1024u);
      }
    }
  };
  auto issue_prologue = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s)
      if (s < nk) issue(s);
  };

  if (!open_tile(slot)) return;
  issue_prologue();

  for (;;) {
    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // Wait until this wave's loads for step s have landed.  vmcnt counts loads and stores together, in issue order, so
    // the wait names how many younger operations may still be outstanding: the loads of the (NSTAGE - 2) following
    // steps, and, in the first NSTAGE - 1 steps of a tile (whose loads were issued before the previous tile's
    // epilogue), that epilogue's stores when their number is known (epi_stores; 0 = unknown: wait for everything).
    auto wait_step = [&](int s) __attribute__((always_inline)) {
      if (s + NSTAGE - 2 < nk) {
        if constexpr (EPI_STORES > 0) {
          if (s < NSTAGE - 1 && epi_stores) { wait_vmcnt<(NSTAGE - 2) * LOADS + EPI_STORES>(); return; }
        }
        if (s > 0) { wait_vmcnt<(NSTAGE - 2) * LOADS>(); return; }
      }
      wait_vmcnt<0>();
    };
    // ---- k loop ------------------------------------------------------------------------------------
    // bf16 kernels: the fragments of a sub-step are read one sub-step ahead, also across the step barrier.  The
    // barrier that opens step s+1 sits before the last sub-step's MFMAs of step s (whose fragments are in registers
    // by then), so the first fragment reads of a step, which all eight waves issue at once, overlap MFMAs instead of
    // leaving the matrix cores idle at every step start: -1.6 to -2.2 % on the forward kernels and dgrad1, -4 to -6 %
    // on the weight-gradient kernel with 64-deep steps (with 32-deep steps, two sub-steps each, it gains nothing).
    // The dgrad2 kernels gain from it as well (-2.4 % plain, -0.9 % of the fused-order backward) once their epilogue
    // ends with an explicit vmcnt wait (see there); before that a build with it measured no gain.  The e4m3 kernels
    // have no room for a second set of 32-byte fragments.
    constexpr bool XPIPE = !FP8 && (MODE != KSEG || NSTAGE == 2);
    if constexpr (XPIPE) {
      static_assert(KK % 2 == 0, "fragment sets alternate by sub-step parity");
      // opens step s: its loads have landed (at most the younger steps' loads are outstanding; the first step of a
      // tile also drains the previous tile's epilogue stores), every wave is done with step s-1, whose stage is
      // refilled right away
      auto open_step = [&](int s) __attribute__((always_inline)) {
        if (!is_toucher) {                  // (the touching wave has no tile loads of its own to wait for)
          wait_step(s);
        }
        __syncthreads();
        if (s + NSTAGE - 1 < nk) issue(s + NSTAGE - 1);
      };
      // A wave whose rows all lie past the expert's last row has nothing to multiply (wave-uniform; it still issues
      // its loads and takes part in the barriers).  In a nearly empty last tile of an expert only one or two waves
      // per CU then use the matrix cores, and the k-step shrinks to what the loads need.
      const bool wave_active = MODE != ROWSEG || m0 + wm * WTM < m_end;
      if (!wave_active) {
        for (int s = 0; s < nk; ++s) open_step(s);
      } else if (nk > 0) {
        bf16x8 af[2][TM], bfr[2][TN];
        auto read_frags = [&](const char* at, int kk, int set) __attribute__((always_inline)) {
          const char* bt = at + A_BYTES;
#pragma unroll
          for (int i = 0; i < TM; ++i) af[set][i] = read_frag_dma<LA, BM, BKT>(at, wm * WTM + i * 32, kk, lane);
#pragma unroll
          for (int j = 0; j < TN; ++j) bfr[set][j] = read_frag_dma<LB, BN, BKT>(bt, wn * WTN + j * 32, kk, lane);
        };
        open_step(0);
        read_frags(smem, 0, 0);
        for (int kt = 0; kt < nk; ++kt) {
          const char* at = smem + (kt % NSTAGE) * STAGE_BYTES;
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) {
            constexpr int TOUCH_AT = KK >= 2 ? KK - 2 : 0;      // one sub-step ahead of the refill it runs before (later: slower)
            if constexpr (TOUCH || TOUCH_K2) {
              if (kk == TOUCH_AT && is_toucher && (kt + NSTAGE + 1) * BKT <= klen) {   // whole k-steps only: every touched address exists
                touch4s(a_base + (long)(kt + NSTAGE) * a_step, ta_off, lds_dump);
              }
            }
            if (kk + 1 < KK) {
              read_frags(at, kk + 1, (kk + 1) & 1);
            } else if (kt + 1 < nk) {
              open_step(kt + 1);
              read_frags(smem + ((kt + 1) % NSTAGE) * STAGE_BYTES, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
              for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[kk & 1][j], af[kk & 1][i], acc[i][j], 0, 0, 0);
          }
        }
      }
    } else
    for (int kt = 0; kt < nk; ++kt) {
      // my loads for step kt have landed once at most the younger steps' loads are outstanding; the first
      // step of a tile also drains the previous tile's epilogue stores, which share the counter
      if (!is_toucher) {                    // (the touching wave has no tile loads of its own to wait for)
        wait_step(kt);
      }
      __syncthreads();
      if (kt + NSTAGE - 1 < nk) issue(kt + NSTAGE - 1);

      if constexpr (BSCALE) {
        // this step's scale bytes landed with its tiles (same wait, same barrier)
        const unsigned char* sc = reinterpret_cast<const unsigned char*>(scale_smem) + (kt % NSTAGE) * 512;
#pragma unroll
        for (int i = 0; i < TM; ++i) sa_cur[i] = sc[wm * WTM + i * 32 + (lane & 31)];
#pragma unroll
        for (int j = 0; j < TN; ++j) sb_cur[j] = sc[256 + wn * WTN + j * 32 + (lane & 31)];
      }
      const char* at = smem + (kt % NSTAGE) * STAGE_BYTES;
      const char* bt = at + A_BYTES;
      if constexpr (MODE == ROWSEG) {
        // A wave whose rows all lie past the expert's last row has nothing to multiply (wave-uniform; it still
        // issued its loads and takes part in the barriers).  In a nearly empty last tile of an expert only one or
        // two waves per CU then use the matrix cores, and the k-step shrinks to what the loads need.
        if (m0 + wm * WTM >= m_end) continue;
      }
#pragma unroll
      for (int kk = 0; kk < KK; ++kk) {
        if constexpr (TOUCH) {
          // late in the step, when the tile loads of this step have left the texture-address queue
          if (kk == KK - 1 && is_toucher && (kt + NSTAGE + 1) * BKT <= klen) {   // whole k-steps only: every touched address exists
            touch4s(a_base + (long)(kt + NSTAGE) * a_step, ta_off, lds_dump);
          }
        }
        if constexpr (TOUCH_K) {
          if (kk == KK - 1 && is_toucher && (kt & 1) == 0 && (kt + NSTAGE + 2) * BKT <= klen) {
            touch4s(a_base + (long)(kt + NSTAGE) * a_step, ta_off, lds_dump);
          }
        }
        if constexpr (FP8) {
          // 32x32x64 e4m3 x e4m3 (format selectors 0, 0), both block scales 2^0 (E8M0 code 127)
          i32x8 af[TM], bfr[TN];
#pragma unroll
          for (int i = 0; i < TM; ++i) af[i] = read_frag_fp8<BM, BKT>(at, wm * WTM + i * 32, kk, lane);
#pragma unroll
          for (int j = 0; j < TN; ++j) bfr[j] = read_frag_fp8<BN, BKT>(bt, wn * WTN + j * 32, kk, lane);
#pragma unroll
          for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
              if constexpr (BSCALE)
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bfr[j], af[i], acc[i][j], 0, 0, 0, sb_cur[j], 0, sa_cur[i]);
              else
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(bfr[j], af[i], acc[i][j], 0, 0, 0, 127, 0, 127);
        } else {
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
    }

    if constexpr (TOUCH || TOUCH_K || TOUCH_K2) {
      if (is_toucher) wait_vmcnt<0>();      // no touch may still be on its way into LDS when the patches are used
    }
    // ---- hand the ring to the next tile, then write this one out -------------------------------------
    const int ep_e = e, ep_m0 = m0, ep_m_end = m_end, ep_n0 = n0, ep_part_slot = part_slot;
    // a full tile that is no split-K part and does not read-modify-write issues every store of its epilogue
    epi_stores = EPI_STORES > 0 && part_slot < 0 && !p.accumulate && m0 + BM <= m_end &&
                 n0 + BN_OUT <= (SWI ? p.f : p.N);
    // SwiGLU' (bf16): the saved G and U of the wave's first block are asked for before the hand-over, ahead of the
    // next tile's first loads in the memory queue
    constexpr bool EARLY_GU = !FP8 && (EPI == EPI_SWIGLU_BWD || EPI == EPI_SWIGLU_BWD_W);
    StageFetch fg_first, fu_first;
    if constexpr (EARLY_GU) {
      const int mb = m0 + wm * WTM, nb = n0 + wn * WTN;
      const bf16* hrow = p.H + (long)mb * 2 * p.N + nb;
      fg_first = stage_fetch_bf16(hrow, 2L * p.N, m_end - mb, p.N - nb, lane);
      fu_first = stage_fetch_bf16(hrow + p.N, 2L * p.N, m_end - mb, p.N - nb, lane);
    }
    slot += 1;
    __syncthreads();                      // every wave has read its last fragments: the ring is free
    const bool has_next = open_tile(slot);
    if (has_next) {
      issue_prologue();
    }
    {
      const int e = ep_e, m0 = ep_m0, m_end = ep_m_end, n0 = ep_n0;
      (void)e;
      // e4m3 operands with per-row / per-output-channel scales: output = acc * scale of the row (token) * scale of
      // the output channel, applied block by block right before a block is written, so that only one block's 16
      // channel scales are live at a time
      auto dequant_block = [&](int i, int j) __attribute__((always_inline)) {
        if constexpr (FP8 && !BSCALE) {
          const int lrow = lane & 31, lcol = (lane >> 5) << 2;
          const int m = min(m0 + wm * WTM + i * 32 + lrow, p.M - 1);
          const float rs = p.row_scale ? p.row_scale[m] : 1.f;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            int n;
            if constexpr (SWI) {
              const int nn = min(n0 + ((wn * WTN + (j & ~1) * 32) >> 1) + q * 8 + lcol, p.f - 4);
              n = (j & 1) ? p.f + nn : nn;
            } else {
              n = min(n0 + wn * WTN + j * 32 + q * 8 + lcol, p.N - 4);
            }
            f32x4 cs = {1.f, 1.f, 1.f, 1.f};
            if (p.col_scale) cs = *reinterpret_cast<const f32x4*>(p.col_scale + (long)e * p.cs_es + n);
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[i][j][4 * q + t] *= rs * cs[t];
          }
        }
      };
      // every 32x32 MFMA tile goes through the wave's LDS patch (see stage_store_* above); bf16 kernels use the
      // branch-free buffer accesses, e4m3 kernels the plain ones
      auto store_bf16 = [&](const bf16x4 (&v)[4], bf16* g, long ld, int rv, int cv) __attribute__((always_inline)) {
        if constexpr (PLAIN_EPI) stage_store_bf16_g(stg, v, g, ld, rv, cv, lane); else stage_store_bf16(stg, v, g, ld, rv, cv, lane);
      };
      auto load_bf16 = [&](bf16x4 (&v)[4], const bf16* g, long ld, int rv, int cv) __attribute__((always_inline)) {
        if constexpr (PLAIN_EPI) stage_load_bf16_g(stg, v, g, ld, rv, cv, lane); else stage_load_bf16(stg, v, g, ld, rv, cv, lane);
      };
      auto store_f32 = [&](const f32x16& a, float* g, long ld, int rv, int cv, bool accumulate) __attribute__((always_inline)) {
        if constexpr (PLAIN_EPI) stage_store_f32_g(stg, a, g, ld, rv, cv, accumulate, lane); else stage_store_f32(stg, a, g, ld, rv, cv, accumulate, lane);
      };
      if (SPLITK && ep_part_slot >= 0) {
        // one K part of a split tile: the whole fp32 tile goes to the partial buffer, no masks
        float* part_tile = p.splitk_ws + (long)ep_part_slot * (BM * BN);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            dequant_block(i, j);
            store_f32(acc[i][j], part_tile + (long)(wm * WTM + i * 32) * BN + wn * WTN + j * 32, BN, 32, 32, false);
          }
      } else if constexpr (EPI == EPI_STORE) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int mb = m0 + wm * WTM + i * 32;
          const int rows_valid = m_end - mb;
          if (rows_valid <= 0) continue;
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const int nb = n0 + wn * WTN + j * 32;
            const int cols_valid = p.N - nb;
            if (cols_valid <= 0) continue;
            dequant_block(i, j);
            if constexpr (sizeof(TC) == 4) {
              float* g = static_cast<float*>(p.C) + (long)e * p.c_es + (long)mb * p.ldc + nb;
              store_f32(acc[i][j], g, p.ldc, rows_valid, cols_valid, p.accumulate != 0);
            } else {
              bf16* g = static_cast<bf16*>(p.C) + (long)e * p.c_es + (long)mb * p.ldc + nb;
              bf16x4 v[4];
              if (p.accumulate) {
                bf16x4 old[4];
                load_bf16(old, g, p.ldc, rows_valid, cols_valid);
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                  for (int t = 0; t < 4; ++t)
                    v[q][t] = static_cast<bf16>(acc[i][j][4 * q + t] + static_cast<float>(old[q][t]));
              } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                  for (int t = 0; t < 4; ++t) v[q][t] = static_cast<bf16>(acc[i][j][4 * q + t]);
              }
              store_bf16(v, g, p.ldc, rows_valid, cols_valid);
            }
          }
        }
      } else if constexpr (EPI == EPI_BIAS_F32) {
        const int lrow = lane & 31, lcol = (lane >> 5) << 2;
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
      } else if constexpr (SWI) {
        // MFMA tile 2j holds G and tile 2j+1 holds U for the same 32 output columns
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          const int mb = m0 + wm * WTM + i * 32;
          const int rows_valid = m_end - mb;
          if (rows_valid <= 0) continue;
          float w_row = 1.0f;                                   // this lane's row is lane % 32 of the block
          if constexpr (FOLD) w_row = p.row_w[min(mb + (lane & 31), p.M - 1)];
#pragma unroll
          for (int j = 0; j < TN; j += 2) {
            const int nb = n0 + ((wn * WTN + j * 32) >> 1);
            const int cols_valid = p.f - nb;
            if (cols_valid <= 0) continue;
            dequant_block(i, j);
            dequant_block(i, j + 1);
            bf16x4 g[4], u[4], a[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
              for (int t = 0; t < 4; ++t) {
                g[q][t] = static_cast<bf16>(acc[i][j][4 * q + t]);
                u[q][t] = static_cast<bf16>(acc[i][j + 1][4 * q + t]);
                const float gf = static_cast<float>(g[q][t]);
                a[q][t] = static_cast<bf16>(w_row * (gf * sigmoid_f32(gf) * static_cast<float>(u[q][t])));
              }
            bf16* hrow = p.H + (long)mb * 2 * p.f + nb;
            store_bf16(g, hrow, 2L * p.f, rows_valid, cols_valid);
            store_bf16(u, hrow + p.f, 2L * p.f, rows_valid, cols_valid);
            store_bf16(a, p.A_out + (long)mb * p.f + nb, p.f, rows_valid, cols_valid);
          }
        }
      } else {
        // acc = dA; read G|U, write dG|dU and the recomputed SwiGLU output.  Folded order (Section 4.1): acc is dA', the
        // gradient w.r.t. A' = w_r * A.  dG|dU are written for dA' as it is (the row's weight is applied downstream:
        // once per row in the combine of d_xp and in the rows handed to wgrad1, not per element here), the stored
        // FC2 input is A', and <dA'[r,:], A[r,:]> over this wave's columns goes to dw_part as one partial sum of the
        // gate-weight gradient of row r.
        auto swiglu_bwd_block = [&](const f32x16& dacc, const bf16x4 (&g)[4], const bf16x4 (&u)[4], int mb, int nb,
                                    int rows_valid, int cols_valid, float w_row, float& dw_sum) __attribute__((always_inline)) {
          bf16x4 dg[4], du[4], a[4];
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const float gf = static_cast<float>(g[q][t]), uf = static_cast<float>(u[q][t]);
              float d = static_cast<float>(static_cast<bf16>(dacc[4 * q + t]));
              const float sg = sigmoid_f32(gf);
              const float av = gf * sg * uf;
              if constexpr (FOLD) dw_sum += d * av;      // masked G, U are zero: columns past N and rows past the segment add 0
              dg[q][t] = static_cast<bf16>(d * uf * sg * (1.0f + gf * (1.0f - sg)));
              du[q][t] = static_cast<bf16>(d * gf * sg);
              a[q][t] = static_cast<bf16>(FOLD ? w_row * av : av);
            }
          bf16* drow = p.dH + (long)mb * 2 * p.N + nb;
          store_bf16(dg, drow, 2L * p.N, rows_valid, cols_valid);
          store_bf16(du, drow + p.N, 2L * p.N, rows_valid, cols_valid);
          if constexpr (FP8) {
            if (p.A_out) store_bf16(a, p.A_out + (long)mb * p.N + nb, p.N, rows_valid, cols_valid);
          } else {
            store_bf16(a, p.A_out + (long)mb * p.N + nb, p.N, p.A_out ? rows_valid : 0, cols_valid);   // no A_out: all lanes masked
          }
        };
        // lanes l and l + 32 hold the two column halves of row l.  Every row of the expert's segment gets exactly one
        // partial per (n-tile, wave along n); blocks past N contribute zero.
        auto row_weight = [&](int i) __attribute__((always_inline)) -> float {
          if constexpr (FOLD) return p.row_w[min(m0 + wm * WTM + i * 32 + (lane & 31), p.M - 1)];
          return 1.0f;
        };
        auto write_dw = [&](int i, float dw_sum) __attribute__((always_inline)) {
          if constexpr (FOLD) {
            const float tot = dw_sum + __shfl_xor(dw_sum, 32);
            const int mb = m0 + wm * WTM + i * 32;
            const __amdgpu_buffer_rsrc_t rs = block_rsrc(p.dw_part + (long)((n0 / BN) * WN + wn) * p.M + mb);
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned, tot), rs,
                                                  (lane < 32 && mb + lane < m_end) ? (unsigned)lane * 4u : BUF_OOB, 0, 0);
          }
        };
        if constexpr (FP8) {
          // (the e4m3 instantiation has no registers to spare for reading ahead)
#pragma unroll
          for (int i = 0; i < TM; ++i) {
            const int mb = m0 + wm * WTM + i * 32;
            const int rows_valid = m_end - mb;
            if (rows_valid <= 0) continue;
            float dw_sum = 0.f;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
              const int nb = n0 + wn * WTN + j * 32;
              const int cols_valid = p.N - nb;
              if (cols_valid <= 0) continue;
              bf16x4 g[4], u[4];
              const bf16* hrow = p.H + (long)mb * 2 * p.N + nb;
              load_bf16(g, hrow, 2L * p.N, rows_valid, cols_valid);
              load_bf16(u, hrow + p.N, 2L * p.N, rows_valid, cols_valid);
              dequant_block(i, j);
              swiglu_bwd_block(acc[i][j], g, u, mb, nb, rows_valid, cols_valid, 1.0f, dw_sum);
            }
          }
        } else {
          // The G and U reads of block b+1 are issued as soon as block b has been unpacked from the fetch registers,
          // so they are in flight while block b is computed and stored (one set of fetch registers: a second set
          // makes the compiler spill the loaders' tile offsets and reload them inside the k loop).
          constexpr int NB = TM * TN;
          auto block_geom = [&](int b, int& mb, int& nb, int& rows_valid, int& cols_valid) __attribute__((always_inline)) {
            const int i = b / TN, j = b % TN;
            mb = m0 + wm * WTM + i * 32;
            nb = n0 + wn * WTN + j * 32;
            rows_valid = m_end - mb;
            cols_valid = p.N - nb;
          };
          auto fetch_block = [&](int b, StageFetch& fg, StageFetch& fu) __attribute__((always_inline)) {
            int mb, nb, rows_valid, cols_valid;
            block_geom(b, mb, nb, rows_valid, cols_valid);
            const bf16* hrow = p.H + (long)mb * 2 * p.N + nb;
            fg = stage_fetch_bf16(hrow, 2L * p.N, rows_valid, cols_valid, lane);
            fu = stage_fetch_bf16(hrow + p.N, 2L * p.N, rows_valid, cols_valid, lane);
          };
          // Every block runs whether or not it has valid rows or columns (the masks live in the buffer offsets): a
          // uniform skip of single blocks would again make the number of stores in flight unknown to the compiler.
          // A wave without any valid row skips all of it.
          StageFetch fg = fg_first, fu = fu_first;
          float w_row = 1.0f, dw_sum = 0.f;
          if (m0 + wm * WTM < m_end)
#pragma unroll
          for (int b = 0; b < NB; ++b) {
            if (b % TN == 0) { w_row = row_weight(b / TN); dw_sum = 0.f; }
            int mb, nb, rows_valid, cols_valid;
            block_geom(b, mb, nb, rows_valid, cols_valid);
            bf16x4 g[4], u[4];
            stage_unpack_bf16(stg, fg, g, lane);
            stage_unpack_bf16(stg, fu, u, lane);
            if (b + 1 < NB) fetch_block(b + 1, fg, fu);
            __builtin_amdgcn_sched_barrier(0);      // the read-ahead stays ahead of this block's arithmetic and stores
            swiglu_bwd_block(acc[b / TN][b % TN], g, u, mb, nb, rows_valid, cols_valid, w_row, dw_sum);
            if (b % TN == TN - 1) write_dw(b / TN, dw_sum);
          }
          // Every wave leaves this epilogue with none of its vector memory operations in flight.  The first step of
          // the next tile would wait for them anyway (more stores than vmcnt can name), so this costs nothing; but
          // it has to be said here, once, on a path every wave takes.  The k loop has a path without any vmcnt wait
          // (the touching wave's), and when the compiler cannot rule out that the read-ahead loads of G and U above
          // are still writing their registers on that path, it guards the registers where they are reused: if the
          // allocation gives them to the fragments, that is a vmcnt wait in front of the fragment reads of every step
          // on every wave, which there also waits for the tile loads issued a moment before (seen: dgrad2 +20 % after
          // a change to the epilogue's arithmetic that moved the allocation).
          wait_vmcnt<0>();
        }
      }
    }
    if (!has_next) break;
  }
}

template <int BM, int BN, int BKT, int NSTAGE, Layout LA, Layout LB, int ESZ = 2>
constexpr int dma_smem_bytes() {
  // the ring, the per-expert tile table and one epilogue patch per wave (at most 8 waves)
  return NSTAGE * (DmaTileBytes<LA, BM, BKT, ESZ>::value + DmaTileBytes<LB, BN, BKT, ESZ>::value) + (MOE_MAX_EXPERTS + 8) * 4 +
         8 * STG_BYTES + 256 + 1024;       // + the dump area of the L2 touches + the block-scale ring
}

}  // namespace mfma
}  // namespace moe
