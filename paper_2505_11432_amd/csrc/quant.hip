// E4M3 cast of activations and gradients (Section 5 "Communication compression for FP8 training":
// E4M3 for all tensors, per-token quantisation forward, per-channel quantisation in groups of 128
// tokens backward; Section 7 "FP8 training": per-token 1 x h scales).
//
// Scale rule (the paper gives none): amax = max|v| of the group; amax == 0 -> scale 1, codes 0;
// else inv = 448/amax and scale = amax/448 (one fp32 division each), code = nearest-even e4m3 of
// clamp(fp32(v)*inv, -448, 448).  The clamp comes first because the gfx950 converter turns
// magnitudes of 465 and more into NaN instead of saturating.
#include "moe_common.h"

namespace moe {
namespace {

constexpr float kE4M3Max = 448.0f;
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float clamp448(float p) { return fminf(fmaxf(p, -kE4M3Max), kE4M3Max); }

// Four floats -> four packed codes (byte i = element i).
__device__ __forceinline__ unsigned pack4_e4m3(float a, float b, float c, float d) {
  int w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(a), clamp448(b), 0, false);
  w = __builtin_amdgcn_cvt_pk_fp8_f32(clamp448(c), clamp448(d), w, true);
  return (unsigned)w;
}

template <int THREADS>
__device__ __forceinline__ float block_max(float v, float* red) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = v;
  __syncthreads();
  v = red[0];
#pragma unroll
  for (int w = 1; w < THREADS / 64; ++w) v = fmaxf(v, red[w]);
  __syncthreads();
  return v;
}

// One block per row.  A row of up to THREADS x 8 vectors stays in registers between the amax pass and the
// convert pass, so HBM sees each element once (256 threads: 16384 bf16 columns; 1024 threads, used for wider
// rows: 65536); longer rows are read a second time (from L2).
template <typename T, int THREADS, int kHold = 8>
__global__ void __launch_bounds__(THREADS) quant_rows_kernel(const T* __restrict__ src, int rows, int cols,
                                                             uint8_t* __restrict__ codes, float* __restrict__ scales) {
  __shared__ float red[THREADS / 64];
  constexpr int V = 16 / sizeof(T);
  const int nvec = cols / V;
  const bool in_regs = nvec <= THREADS * kHold;
  for (int r = blockIdx.x; r < rows; r += gridDim.x) {
    const T* row = src + (long)r * cols;
    Vec16<T> hold[kHold];
    float amax = 0.f;
    if (in_regs) {
      // every load is issued before the first value is used; vectors past the row's end re-read its last vector
      // (same maximum, never stored), which keeps the loads unconditional
#pragma unroll
      for (int h = 0; h < kHold; ++h) {
        const int c = min((int)threadIdx.x + h * THREADS, nvec - 1);
        // streamed once: non-temporal
        hold[h] = __builtin_bit_cast(Vec16<T>, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + (long)c * V)));
      }
#pragma unroll
      for (int h = 0; h < kHold; ++h)
#pragma unroll
        for (int i = 0; i < V; ++i) amax = fmaxf(amax, fabsf(to_f32(hold[h].v[i])));
    } else {
      for (int c = threadIdx.x; c < nvec; c += THREADS) {
        const Vec16<T> v = *reinterpret_cast<const Vec16<T>*>(row + (long)c * V);
#pragma unroll
        for (int i = 0; i < V; ++i) amax = fmaxf(amax, fabsf(to_f32(v.v[i])));
      }
    }
    amax = block_max<THREADS>(amax, red);
    const float inv = amax > 0.f ? kE4M3Max / amax : 1.0f;
    if (threadIdx.x == 0) scales[r] = amax > 0.f ? amax / kE4M3Max : 1.0f;
    auto convert = [&](const Vec16<T>& v, int c) {
      unsigned out[V / 4];
#pragma unroll
      for (int i = 0; i < V / 4; ++i)
        out[i] = pack4_e4m3(to_f32(v.v[4 * i]) * inv, to_f32(v.v[4 * i + 1]) * inv, to_f32(v.v[4 * i + 2]) * inv,
                            to_f32(v.v[4 * i + 3]) * inv);
      uint8_t* dst = codes + (long)r * cols + (long)c * V;           // V bytes, V-byte aligned: one store
      typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
      if constexpr (V == 8) { const u32x2 o = {out[0], out[1]}; __builtin_nontemporal_store(o, reinterpret_cast<u32x2*>(dst)); }
      else __builtin_nontemporal_store(out[0], reinterpret_cast<unsigned*>(dst));
    };
    if (in_regs) {
#pragma unroll
      for (int h = 0; h < kHold; ++h) {
        const int c = threadIdx.x + h * THREADS;
        {
          // keep the row as the 16 raw bytes per vector between the two passes: without this the compiler holds
          // the fp32 values it made for the amax pass (4x the registers)
          u32x4 raw = __builtin_bit_cast(u32x4, hold[h]);
          asm volatile("" : "+v"(raw));
          hold[h] = __builtin_bit_cast(Vec16<T>, raw);
        }
        if (c < nvec) convert(hold[h], c);
      }
    } else {
      for (int c = threadIdx.x; c < nvec; c += THREADS) convert(*reinterpret_cast<const Vec16<T>*>(row + (long)c * V), c);
    }
  }
}

// One block per (128-row group, 64-column slab): thread (rg, cq) holds rows rg, rg+16, ... (8 rows) of the four
// columns 4*cq..4*cq+3 in registers; the column maxima are combined through LDS.
template <typename T>
__global__ void __launch_bounds__(256) quant_colgroup_kernel(const T* __restrict__ src, int rows, int cols,
                                                             uint8_t* __restrict__ codes,
                                                             float* __restrict__ scales, int slabs) {
  __shared__ float cmax[16][64];
  const int g = blockIdx.x / slabs;
  const int cq = threadIdx.x % 16, rg = threadIdx.x / 16;
  const int c = (blockIdx.x % slabs) * 64 + cq * 4;
  const int r0 = g * 128;
  const bool col_ok = c < cols;
  float v[8][4];
  float amax[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = r0 + rg + 16 * i;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[i][j] = 0.f;
    if (col_ok && r < rows) {
      const T* p = src + (long)r * cols + c;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        v[i][j] = to_f32(p[j]);
        amax[j] = fmaxf(amax[j], fabsf(v[i][j]));
      }
    }
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) cmax[rg][cq * 4 + j] = amax[j];
  __syncthreads();
  float inv[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float m = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) m = fmaxf(m, cmax[q][cq * 4 + j]);
    inv[j] = m > 0.f ? kE4M3Max / m : 1.0f;
    if (rg == 0 && col_ok) scales[(long)g * cols + c + j] = m > 0.f ? m / kE4M3Max : 1.0f;
  }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = r0 + rg + 16 * i;
    if (col_ok && r < rows)
      *reinterpret_cast<unsigned*>(codes + (long)r * cols + c) =
          pack4_e4m3(v[i][0] * inv[0], v[i][1] * inv[1], v[i][2] * inv[2], v[i][3] * inv[3]);
  }
}


// ---- backward-orientation cast for the weight-gradient GEMMs ---------------------------------------------
// Section 7 "FP8 training": per-channel quantisation within 128-token groups for the backward pass.  The
// contraction index of a weight-gradient GEMM is the token, so the codes are written transposed ([channel]
// [token], K-major for the matrix cores) and every expert's segment is padded with zero codes to a multiple
// of 128 tokens: a group never spans two experts, every k-step of the GEMM is one whole group, and the group
// scale is a power of two (E8M0 byte), which the block-scaled MFMA applies inside the contraction.
// Scale rule: k = smallest integer with amax * 2^-k <= 448 (448 = 1.75 * 2^8), k = 0 for amax = 0,
// clamped to [-126, 127]; byte = k + 127; code = nearest-even e4m3 of clamp(v * 2^-k, +-448).

// pad_offsets[e] = first padded token column of expert e (a multiple of 128); pad_offsets[E] = total.
__global__ void tgroup_offsets_kernel(const int32_t* __restrict__ offsets, int E, int32_t* __restrict__ pad_offsets) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    int run = 0;
    pad_offsets[0] = 0;
    for (int e = 0; e < E; ++e) {
      run += (offsets[e + 1] - offsets[e] + 127) / 128 * 128;
      pad_offsets[e + 1] = run;
    }
  }
}

// One block per (padded 128-token group, 128-channel slab).  Thread (rgrp, cq) holds eight consecutive tokens
// (rows 8*rgrp .. 8*rgrp+7) of eight consecutive channels: a wave's load touches four rows with 16 bytes per lane,
// and a channel's eight codes of those tokens are eight consecutive bytes of the transposed output, written to the
// LDS tile as one 8-byte word (16-byte chunks of a tile row are XOR-swizzled by the channel octet, so the sixteen
// threads of a row group do not meet in one bank).  Channel maxima are reduced over the wave's four row groups with
// shuffles and over the four waves through LDS.  Global memory sees 16-byte lanes forming 128-byte rows (one channel
// x 128 tokens).
template <typename T>
__global__ void __launch_bounds__(256) quant_tgroup_kernel(const T* __restrict__ src,
                                                           const float* __restrict__ src_row_scale, int cols,
                                                           const int32_t* __restrict__ offsets,
                                                           const int32_t* __restrict__ pad_offsets, int E,
                                                           uint8_t* __restrict__ codes_t, long ldt,
                                                           uint8_t* __restrict__ e8m0, int slabs) {
  constexpr int CH = 128;                           // channels per block
  __shared__ float cmax[4][CH];
  __shared__ __attribute__((aligned(16))) uint8_t tile[CH][128 + 16];
  const int g = blockIdx.x / slabs;
  const int tok0 = g * 128;                         // padded token column of this group
  if (tok0 >= pad_offsets[E]) return;
  int lo = 0, hi = E;                               // expert whose padded range holds tok0
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (pad_offsets[mid] <= tok0) lo = mid; else hi = mid;
  }
  const int e = lo;
  const int r0 = offsets[e] + (tok0 - pad_offsets[e]);      // first source row of the group
  const int r_end = offsets[e + 1];
  const int cq = threadIdx.x % 16, rgrp = threadIdx.x / 16;
  const int c0 = (blockIdx.x % slabs) * CH;
  const int c = c0 + cq * 8;
  const bool col_ok = c < cols;                     // cols is a multiple of 16: all eight channels or none
  float v[8][8];
  float amax[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) amax[j] = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = r0 + rgrp * 8 + i;
#pragma unroll
    for (int j = 0; j < 8; ++j) v[i][j] = 0.f;
    if (col_ok && r < r_end) {
      const T* p = src + (long)r * cols + c;
      if constexpr (sizeof(T) == 1) {
        // e4m3 codes with one scale per source row: the value is code * scale, rounded once to fp32
        const int2 w = *reinterpret_cast<const int2*>(p);
        const float rs = src_row_scale[r];
        v[i][0] = __builtin_amdgcn_cvt_f32_fp8(w.x, 0) * rs;
        v[i][1] = __builtin_amdgcn_cvt_f32_fp8(w.x, 1) * rs;
        v[i][2] = __builtin_amdgcn_cvt_f32_fp8(w.x, 2) * rs;
        v[i][3] = __builtin_amdgcn_cvt_f32_fp8(w.x, 3) * rs;
        v[i][4] = __builtin_amdgcn_cvt_f32_fp8(w.y, 0) * rs;
        v[i][5] = __builtin_amdgcn_cvt_f32_fp8(w.y, 1) * rs;
        v[i][6] = __builtin_amdgcn_cvt_f32_fp8(w.y, 2) * rs;
        v[i][7] = __builtin_amdgcn_cvt_f32_fp8(w.y, 3) * rs;
      } else if constexpr (sizeof(T) == 2) {
        typedef __bf16 bf16x8v __attribute__((ext_vector_type(8)));
        const bf16x8v w = *reinterpret_cast<const bf16x8v*>(p);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[i][j] = static_cast<float>(w[j]);
      } else {
        const float4 a = *reinterpret_cast<const float4*>(p);
        const float4 b = *reinterpret_cast<const float4*>(p + 4);
        v[i][0] = a.x; v[i][1] = a.y; v[i][2] = a.z; v[i][3] = a.w;
        v[i][4] = b.x; v[i][5] = b.y; v[i][6] = b.z; v[i][7] = b.w;
      }
#pragma unroll
      for (int j = 0; j < 8; ++j) amax[j] = fmaxf(amax[j], fabsf(v[i][j]));
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    amax[j] = fmaxf(amax[j], __shfl_xor(amax[j], 16));
    amax[j] = fmaxf(amax[j], __shfl_xor(amax[j], 32));
  }
  if ((threadIdx.x & 63) < 16) {
#pragma unroll
    for (int j = 0; j < 8; ++j) cmax[threadIdx.x >> 6][cq * 8 + j] = amax[j];
  }
  __syncthreads();
  float inv[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float m = fmaxf(fmaxf(cmax[0][cq * 8 + j], cmax[1][cq * 8 + j]), fmaxf(cmax[2][cq * 8 + j], cmax[3][cq * 8 + j]));
    int k = 0;
    if (m > 0.f) {
      const unsigned bits = __float_as_uint(m);
      k = (int)((bits >> 23) & 0xffu) - 127 - 8 + ((bits & 0x7fffffu) > 0x600000u ? 1 : 0);
      k = max(-126, min(127, k));
    }
    inv[j] = __uint_as_float((unsigned)(127 - k) << 23);          // 2^-k, exact
    if (rgrp == 0 && col_ok) e8m0[(long)g * cols + c + j] = (uint8_t)(k + 127);
  }
  const int chunk = ((rgrp >> 1) ^ (cq & 7)) << 4;                 // swizzled 16-byte chunk of the tile row
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    uint2 w;
    w.x = pack4_e4m3(v[0][j] * inv[j], v[1][j] * inv[j], v[2][j] * inv[j], v[3][j] * inv[j]);
    w.y = pack4_e4m3(v[4][j] * inv[j], v[5][j] * inv[j], v[6][j] * inv[j], v[7][j] * inv[j]);
    *reinterpret_cast<uint2*>(&tile[cq * 8 + j][chunk + ((rgrp & 1) << 3)]) = w;
  }
  __syncthreads();
#pragma unroll
  for (int pass = 0; pass < 4; ++pass) {
    const int ch = pass * 32 + threadIdx.x / 8, seg = threadIdx.x % 8;
    if (c0 + ch < cols)
      *reinterpret_cast<uint4*>(codes_t + (long)(c0 + ch) * ldt + tok0 + seg * 16) =
          *reinterpret_cast<const uint4*>(&tile[ch][(seg ^ ((ch >> 3) & 7)) << 4]);
  }
}

template <typename T>
__global__ void __launch_bounds__(256) dequant_kernel(const uint8_t* __restrict__ codes,
                                                      const float* __restrict__ scales, int rows, int cols, int mode,
                                                      T* __restrict__ dst) {
  const long nquad = (long)rows * cols / 4;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < nquad; i += (long)gridDim.x * blockDim.x) {
    const long el = i * 4;
    const int r = (int)(el / cols);
    const int c = (int)(el % cols);
    const int w = *reinterpret_cast<const int*>(codes + el);
    float s[4];
    if (mode == MOE_Q_ROW) {
      s[0] = s[1] = s[2] = s[3] = scales[r];
    } else {
      const float* sp = scales + (long)(r / 128) * cols + c;
      s[0] = sp[0]; s[1] = sp[1]; s[2] = sp[2]; s[3] = sp[3];
    }
    dst[el + 0] = from_f32<T>(__builtin_amdgcn_cvt_f32_fp8(w, 0) * s[0]);
    dst[el + 1] = from_f32<T>(__builtin_amdgcn_cvt_f32_fp8(w, 1) * s[1]);
    dst[el + 2] = from_f32<T>(__builtin_amdgcn_cvt_f32_fp8(w, 2) * s[2]);
    dst[el + 3] = from_f32<T>(__builtin_amdgcn_cvt_f32_fp8(w, 3) * s[3]);
  }
}

}  // namespace

int launch_quant_fp8(const void* src, moe_dtype src_dt, int rows, int cols, moe_qmode mode, uint8_t* codes,
                     float* scales, hipStream_t s) {
  if (rows == 0 || cols == 0) return MOE_OK;
  if (mode == MOE_Q_ROW) {
    const int grid = rows < 256 * 16 ? rows : 256 * 16;
    const bool wide = cols / (16 / (int)dtype_size(src_dt)) > 256 * 8;     // more vectors than 256 threads can hold
    if (src_dt == MOE_F32) {
      if (wide) quant_rows_kernel<float, 1024><<<grid, 1024, 0, s>>>((const float*)src, rows, cols, codes, scales);
      else quant_rows_kernel<float, 256><<<grid, 256, 0, s>>>((const float*)src, rows, cols, codes, scales);
    } else {
      const int nvec = cols / 8;
      if (wide && nvec <= 256 * 16) quant_rows_kernel<bf16, 256, 16><<<rows < 256 * 64 ? rows : 256 * 64, 256, 0, s>>>((const bf16*)src, rows, cols, codes, scales);
      else if (wide) quant_rows_kernel<bf16, 1024><<<grid, 1024, 0, s>>>((const bf16*)src, rows, cols, codes, scales);
      else quant_rows_kernel<bf16, 256><<<grid, 256, 0, s>>>((const bf16*)src, rows, cols, codes, scales);
    }
  } else {
    const int slabs = cdiv(cols, 64);
    const int grid = cdiv(rows, 128) * slabs;
    if (src_dt == MOE_F32) quant_colgroup_kernel<float><<<grid, 256, 0, s>>>((const float*)src, rows, cols, codes, scales, slabs);
    else quant_colgroup_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)src, rows, cols, codes, scales, slabs);
  }
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

int launch_tgroup_offsets(const int32_t* offsets, int E, int32_t* pad_offsets, hipStream_t s) {
  tgroup_offsets_kernel<<<1, 64, 0, s>>>(offsets, E, pad_offsets);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

int launch_quant_tgroup(const void* src, const float* src_row_scale, moe_dtype src_dt, int rows, int cols, const int32_t* offsets,
                        const int32_t* pad_offsets, int E, uint8_t* codes_t, long ldt, uint8_t* e8m0, hipStream_t s) {
  if (cols == 0) return MOE_OK;
  const int slabs = cdiv(cols, 128);
  const int groups = cdiv(rows, 128) + E;              // upper bound on the padded group count
  const long grid = (long)groups * slabs;
  if (grid <= 0 || grid > 0x7fffffffL) return MOE_ERR_UNSUPPORTED;
  if (src_dt == MOE_F32)
    quant_tgroup_kernel<float><<<(int)grid, 256, 0, s>>>((const float*)src, nullptr, cols, offsets, pad_offsets, E, codes_t, ldt, e8m0, slabs);
  else if (src_dt == MOE_BF16)
    quant_tgroup_kernel<bf16><<<(int)grid, 256, 0, s>>>((const bf16*)src, nullptr, cols, offsets, pad_offsets, E, codes_t, ldt, e8m0, slabs);
  else
    quant_tgroup_kernel<uint8_t><<<(int)grid, 256, 0, s>>>((const uint8_t*)src, src_row_scale, cols, offsets, pad_offsets, E, codes_t, ldt, e8m0, slabs);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

int launch_dequant_fp8(const uint8_t* codes, const float* scales, int rows, int cols, moe_qmode mode, void* dst,
                       moe_dtype dst_dt, hipStream_t s) {
  if (rows == 0 || cols == 0) return MOE_OK;
  long blocks = ((long)rows * cols / 4 + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
  if (dst_dt == MOE_F32) dequant_kernel<float><<<(int)blocks, 256, 0, s>>>(codes, scales, rows, cols, (int)mode, (float*)dst);
  else dequant_kernel<bf16><<<(int)blocks, 256, 0, s>>>(codes, scales, rows, cols, (int)mode, (bf16*)dst);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

}  // namespace moe
