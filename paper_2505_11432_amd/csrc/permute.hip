// Dispatch, combine and the gate-weight gradient (Section 3.2: scatter and gather operators that move
// rows according to a row map computed once from the routing result; Section 4.1: the weighted sum).
// All three are HBM-bound row movers: one wave walks one token's row in 16-byte vectors per lane, so
// every global access is a full 1 KiB wave-wide burst.  Token-centric on both sides: dispatch reads a
// token row once and writes its k copies; combine gathers k rows and writes one.
#include "moe_common.h"

namespace moe {
namespace {

constexpr int kWavesPerBlock = 4;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // 16 bytes for the nontemporal builtins

// Broadcast lane `src` (wave-uniform) of a per-lane value; reads the register whatever EXEC says.
__device__ __forceinline__ int bcast(int v, int src) { return __builtin_amdgcn_readlane(v, src); }
__device__ __forceinline__ float bcast(float v, int src) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src));
}

// One wave per token; CU chunks of 64 lanes x 16 bytes are read before their k copies are written.
template <typename T, bool kScaled, int CU>
__global__ void __launch_bounds__(64 * kWavesPerBlock) dispatch_kernel(const T* __restrict__ x,
                                                                       const float* __restrict__ x_scale,
                                                                       const int32_t* __restrict__ inv_perm,
                                                                       const float* __restrict__ row_mul, int T_, int k,
                                                                       int d, T* __restrict__ xp,
                                                                       float* __restrict__ xp_scale) {
  constexpr int V = 16 / sizeof(T);
  const int lane = threadIdx.x % 64;
  const int wave = blockIdx.x * kWavesPerBlock + threadIdx.x / 64;
  const int nwaves = gridDim.x * kWavesPerBlock;
  const int nvec = d / V;
  for (int t = wave; t < T_; t += nwaves) {
    int my_row = -1;
    float my_mul = 1.f;
    if (lane < k) {
      my_row = inv_perm[(long)t * k + lane];          // < 0: the expert is not local, no copy
      if constexpr (kScaled) my_mul = row_mul[(long)t * k + lane];
      if (x_scale != nullptr && my_row >= 0) xp_scale[my_row] = x_scale[t];
    }
    if (__ballot(my_row >= 0) == 0) continue;      // no local expert wants this token: do not read it
    for (int c0 = 0; c0 < nvec; c0 += 64 * CU) {
      Vec16<T> v[CU];
#pragma unroll
      for (int q = 0; q < CU; ++q) {
        const int c = c0 + q * 64 + lane;
        if (c < nvec) v[q] = *reinterpret_cast<const Vec16<T>*>(x + (long)t * d + (long)c * V);
      }
      for (int j = 0; j < k; ++j) {
        const int r = bcast(my_row, j);
        const float m = bcast(my_mul, j);
#pragma unroll
        for (int q = 0; q < CU; ++q) {
          const int c = c0 + q * 64 + lane;
          Vec16<T> o = v[q];
          if constexpr (kScaled) {
#pragma unroll
            for (int i = 0; i < V; ++i) o.v[i] = from_f32<T>(to_f32(v[q].v[i]) * m);
          }
          if (c < nvec && r >= 0)
            __builtin_nontemporal_store(__builtin_bit_cast(u32x4, o), reinterpret_cast<u32x4*>(xp + (long)r * d + (long)c * V));
        }
      }
    }
  }
}

// fp8 codes are bytes; they are decoded by the hardware converter (OCP e4m3 on gfx950).
template <typename TIN> struct RowLoader {
  static constexpr int V = 16 / sizeof(TIN);
  __device__ static void load(const TIN* p, float (&out)[V]) {
    const u32x4 raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));     // rows are streamed once
    const Vec16<TIN> v = __builtin_bit_cast(Vec16<TIN>, raw);
#pragma unroll
    for (int i = 0; i < V; ++i) out[i] = to_f32(v.v[i]);
  }
};
template <> struct RowLoader<uint8_t> {
  static constexpr int V = 16;
  __device__ static void load(const uint8_t* p, float (&out)[16]) {
    const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    const unsigned w[4] = {q[0], q[1], q[2], q[3]};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[4 * i + 0] = __builtin_amdgcn_cvt_f32_fp8((int)w[i], 0);
      out[4 * i + 1] = __builtin_amdgcn_cvt_f32_fp8((int)w[i], 1);
      out[4 * i + 2] = __builtin_amdgcn_cvt_f32_fp8((int)w[i], 2);
      out[4 * i + 3] = __builtin_amdgcn_cvt_f32_fp8((int)w[i], 3);
    }
  }
};

// Raw 16-byte chunk -> V floats (bf16 / fp32 rows: plain conversion; e4m3 codes: the hardware converter).
template <typename TIN> __device__ __forceinline__ void decode16(const u32x4& raw, float (&out)[RowLoader<TIN>::V]) {
  if constexpr (sizeof(TIN) == 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[4 * i + 0] = __builtin_amdgcn_cvt_f32_fp8((int)raw[i], 0);
      out[4 * i + 1] = __builtin_amdgcn_cvt_f32_fp8((int)raw[i], 1);
      out[4 * i + 2] = __builtin_amdgcn_cvt_f32_fp8((int)raw[i], 2);
      out[4 * i + 3] = __builtin_amdgcn_cvt_f32_fp8((int)raw[i], 3);
    }
  } else {
    const Vec16<TIN> v = __builtin_bit_cast(Vec16<TIN>, raw);
#pragma unroll
    for (int i = 0; i < RowLoader<TIN>::V; ++i) out[i] = to_f32(v.v[i]);
  }
}

// V floats -> TOUT, written as whole 16-byte vectors (streamed: nothing reads the row again soon).
template <typename TOUT, int V> __device__ __forceinline__ void store_row_chunk(TOUT* dst, const float (&acc)[V]) {
  constexpr int PER = 16 / sizeof(TOUT);
#pragma unroll
  for (int s = 0; s < V / PER; ++s) {
    Vec16<TOUT> o;
#pragma unroll
    for (int i = 0; i < PER; ++i) o.v[i] = from_f32<TOUT>(acc[s * PER + i]);
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4, o), reinterpret_cast<u32x4*>(dst + s * PER));
  }
}

// One wave per token.  The row is walked in groups of CU chunks of 64 lanes x 16 bytes; for each group the chunks of
// KU slots are all requested before the first of them is used, so a lane keeps KU * CU loads in flight (eight for every
// k) instead of one.  The k terms are still added in ascending slot order in fp32, whatever KU is.
template <typename TIN, typename TOUT, int KU, int CU>
__global__ void __launch_bounds__(64 * kWavesPerBlock) combine_kernel(const TIN* __restrict__ yp,
                                                                      const float* __restrict__ yp_scale,
                                                                      const int32_t* __restrict__ inv_perm,
                                                                      const float* __restrict__ topk_w, int T_, int k,
                                                                      int d, TOUT* __restrict__ y) {
  constexpr int V = RowLoader<TIN>::V;      // elements per lane per chunk
  const int lane = threadIdx.x % 64;
  const int wave = blockIdx.x * kWavesPerBlock + threadIdx.x / 64;
  const int nwaves = gridDim.x * kWavesPerBlock;
  const int nvec = d / V;
  for (int t = wave; t < T_; t += nwaves) {
    int my_row = -1;                         // lanes at or past k: a slot without a row
    float my_w = 1.f;
    if (lane < k) {
      my_row = inv_perm[(long)t * k + lane];
      if (topk_w != nullptr) my_w = topk_w[(long)t * k + lane];
      if (yp_scale != nullptr && my_row >= 0) my_w *= yp_scale[my_row];
    }
    for (int c0 = 0; c0 < nvec; c0 += 64 * CU) {
      float acc[CU][V];
#pragma unroll
      for (int q = 0; q < CU; ++q)
#pragma unroll
        for (int i = 0; i < V; ++i) acc[q][i] = 0.f;
      for (int j0 = 0; j0 < k; j0 += KU) {
        u32x4 raw[KU][CU];
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          const int r = bcast(my_row, j0 + u);      // r < 0: no local row (the term is left to another share) or j >= k
#pragma unroll
          for (int q = 0; q < CU; ++q) {
            const int c = c0 + q * 64 + lane;
            raw[u][q] = u32x4{0u, 0u, 0u, 0u};
            if (r >= 0 && c < nvec) raw[u][q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(yp + (long)r * d + (long)c * V));
          }
        }
#pragma unroll
        for (int u = 0; u < KU; ++u) {
          const int r = bcast(my_row, j0 + u);
          const float w = bcast(my_w, j0 + u);
          if (r >= 0) {                             // (wave-uniform) a skipped term leaves the sum untouched
#pragma unroll
            for (int q = 0; q < CU; ++q) {
              float v[V];
              decode16<TIN>(raw[u][q], v);
#pragma unroll
              for (int i = 0; i < V; ++i) acc[q][i] = fmaf(w, v[i], acc[q][i]);
            }
          }
        }
      }
#pragma unroll
      for (int q = 0; q < CU; ++q) {
        const int c = c0 + q * 64 + lane;
        if (c < nvec) store_row_chunk<TOUT, V>(y + (long)t * d + (long)c * V, acc[q]);
      }
    }
  }
}

// d_topk_w[t,j] = <dy[t,:], yp[row(t,j),:]>.  Same walk as the combine: per group of CU chunks the dy chunks and the
// chunks of KU slots are all requested before the first use.
template <typename TDY, typename TIN, int KU, int CU>
__global__ void __launch_bounds__(64 * kWavesPerBlock) gate_grad_kernel(const TDY* __restrict__ dy,
                                                                        const TIN* __restrict__ yp,
                                                                        const float* __restrict__ yp_scale,
                                                                        const int32_t* __restrict__ inv_perm, int T_,
                                                                        int k, int d, float* __restrict__ d_topk_w) {
  constexpr int V = RowLoader<TIN>::V;
  constexpr int DYV = 16 / sizeof(TDY);          // dy elements per 16-byte load
  constexpr int DYL = V / DYV;                   // 16-byte loads of dy per chunk of V elements
  static_assert(V % DYV == 0, "a chunk of yp covers whole 16-byte pieces of dy");
  const int lane = threadIdx.x % 64;
  const int wave = blockIdx.x * kWavesPerBlock + threadIdx.x / 64;
  const int nwaves = gridDim.x * kWavesPerBlock;
  const int nvec = d / V;
  for (int t = wave; t < T_; t += nwaves) {
    int my_row = -1;
    float my_scale = 1.f;
    if (lane < k) {
      my_row = inv_perm[(long)t * k + lane];
      if (yp_scale != nullptr && my_row >= 0) my_scale = yp_scale[my_row];
    }
    float acc[MOE_MAX_TOPK];
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j) acc[j] = 0.f;
    if (__ballot(my_row >= 0) != 0)              // no local row at all: every gradient of this token is 0
    for (int c0 = 0; c0 < nvec; c0 += 64 * CU) {
      u32x4 graw[CU][DYL];
#pragma unroll
      for (int q = 0; q < CU; ++q) {
        const int c = c0 + q * 64 + lane;
#pragma unroll
        for (int h = 0; h < DYL; ++h) {
          graw[q][h] = u32x4{0u, 0u, 0u, 0u};
          if (c < nvec) graw[q][h] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dy + (long)t * d + (long)c * V + h * DYV));
        }
      }
#pragma unroll
      for (int j0 = 0; j0 < MOE_MAX_TOPK; j0 += KU) {
        if (j0 < k) {
          u32x4 raw[KU][CU];
#pragma unroll
          for (int u = 0; u < KU; ++u) {
            const int r = bcast(my_row, j0 + u);
#pragma unroll
            for (int q = 0; q < CU; ++q) {
              const int c = c0 + q * 64 + lane;
              raw[u][q] = u32x4{0u, 0u, 0u, 0u};
              if (r >= 0 && c < nvec) raw[u][q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(yp + (long)r * d + (long)c * V));
            }
          }
#pragma unroll
          for (int q = 0; q < CU; ++q) {
            float g[V];
#pragma unroll
            for (int h = 0; h < DYL; ++h) {
              float part[DYV];
              decode16<TDY>(graw[q][h], part);
#pragma unroll
              for (int i = 0; i < DYV; ++i) g[h * DYV + i] = part[i];
            }
#pragma unroll
            for (int u = 0; u < KU; ++u) {
              float v[V];
              decode16<TIN>(raw[u][q], v);
              float sum = 0.f;
#pragma unroll
              for (int i = 0; i < V; ++i) sum = fmaf(g[i], v[i], sum);
              acc[j0 + u] += sum;                 // rows that were not loaded are all zero
            }
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < MOE_MAX_TOPK; ++j) {
      if (j < k) {
        float sum = acc[j];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
        sum *= bcast(my_scale, j);
        if (lane == 0) d_topk_w[(long)t * k + j] = sum;
      }
    }
  }
}

int row_grid(int T) {
  int blocks = cdiv(T, kWavesPerBlock);
  const int cap = 256 * 16;
  return blocks < 1 ? 1 : (blocks > cap ? cap : blocks);
}

}  // namespace

int launch_dispatch(const void* x, const float* x_scale, moe_dtype dt, const int32_t* inv_perm, const float* row_mul,
                    int T, int k, int d, void* xp, float* xp_scale, hipStream_t s) {
  const dim3 grid(row_grid(T)), block(64 * kWavesPerBlock);
  constexpr int CP = 4, CS = 4;      // chunks read before their copies are written (measured: 1, 2, 4)
  if (dt == MOE_F32) {
    if (row_mul) dispatch_kernel<float, true, CS><<<grid, block, 0, s>>>((const float*)x, nullptr, inv_perm, row_mul, T, k, d, (float*)xp, nullptr);
    else dispatch_kernel<float, false, CP><<<grid, block, 0, s>>>((const float*)x, nullptr, inv_perm, nullptr, T, k, d, (float*)xp, nullptr);
  } else if (dt == MOE_BF16) {
    if (row_mul) dispatch_kernel<bf16, true, CS><<<grid, block, 0, s>>>((const bf16*)x, nullptr, inv_perm, row_mul, T, k, d, (bf16*)xp, nullptr);
    else dispatch_kernel<bf16, false, CP><<<grid, block, 0, s>>>((const bf16*)x, nullptr, inv_perm, nullptr, T, k, d, (bf16*)xp, nullptr);
  } else {
    dispatch_kernel<uint8_t, false, CP><<<grid, block, 0, s>>>((const uint8_t*)x, x_scale, inv_perm, nullptr, T, k, d, (uint8_t*)xp, xp_scale);
  }
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

// ---- Section 4.1 / 4.2 operator order: per-row index map and gate weight; reduction of the gate-gradient partials ----

__global__ void __launch_bounds__(256) row_map_kernel(const int32_t* __restrict__ perm, const float* __restrict__ topk_w,
                                                      const int32_t* __restrict__ offsets, int E, int rows, int k,
                                                      int32_t* __restrict__ row_token, float* __restrict__ row_w) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= rows) return;
  int tok = 0;
  float w = 0.f;
  if (r < offsets[E]) {              // rows past the last segment exist only as padding: token 0, weight 0
    const int a = perm[r];
    tok = a / k;
    w = topk_w[a];
  }
  row_token[r] = tok;
  row_w[r] = w;
}

// d_topk_w[a] = sum over the parts, in a fixed order, of part[p][inv_perm[a]]; 0 for an assignment without a row.
// A workgroup handles 64 assignments; its four waves each add a quarter of the parts (unrolled, so the loads of one
// wave are in flight together), then wave 0 adds the four quarters in ascending order.
__global__ void __launch_bounds__(256) gate_grad_reduce_kernel(const float* __restrict__ part, int parts, long ld,
                                                               const int32_t* __restrict__ inv_perm, int n,
                                                               float* __restrict__ d_topk_w) {
  __shared__ float quarter[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const int a = blockIdx.x * 64 + lane;
  const int r = a < n ? inv_perm[a] : -1;
  const int per = (parts + 3) / 4;
  const int p0 = q * per, p1 = min(parts, p0 + per);
  float acc = 0.f;
  if (r >= 0) {
    int p = p0;
    for (; p + 8 <= p1; p += 8) {
      float v[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) v[i] = part[(long)(p + i) * ld + r];
#pragma unroll
      for (int i = 0; i < 8; ++i) acc += v[i];
    }
    for (; p < p1; ++p) acc += part[(long)p * ld + r];
  }
  quarter[q][lane] = acc;
  __syncthreads();
  if (q == 0 && a < n) d_topk_w[a] = ((quarter[0][lane] + quarter[1][lane]) + quarter[2][lane]) + quarter[3][lane];
}

int launch_row_map(const int32_t* perm, const float* topk_w, const int32_t* offsets, int E, int rows, int k,
                   int32_t* row_token, float* row_w, hipStream_t s) {
  if (rows == 0) return MOE_OK;
  row_map_kernel<<<dim3((unsigned)cdiv(rows, 256)), dim3(256), 0, s>>>(perm, topk_w, offsets, E, rows, k, row_token, row_w);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

int launch_gate_grad_reduce(const float* part, int parts, long ld, const int32_t* inv_perm, int n, float* d_topk_w,
                            hipStream_t s) {
  if (n == 0) return MOE_OK;
  gate_grad_reduce_kernel<<<dim3((unsigned)cdiv(n, 64)), dim3(256), 0, s>>>(part, parts, ld, inv_perm, n, d_topk_w);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

int launch_combine(const void* yp, const float* yp_scale, moe_dtype dt, const int32_t* inv_perm, const float* topk_w,
                   int T, int k, int d, void* y, moe_dtype y_dt, hipStream_t s) {
  const dim3 grid(row_grid(T)), block(64 * kWavesPerBlock);
// loads in flight per lane (slots x chunks), picked by measurement on 600 MB row buffers: 2 x 8, 4 x 4, 8 x 2
#define MOE_COMBINE_CASE(DI, DO, TI, TO)                                                                              \
  if (dt == DI && y_dt == DO) {                                                                                       \
    if (k <= 2) combine_kernel<TI, TO, 2, 8><<<grid, block, 0, s>>>((const TI*)yp, yp_scale, inv_perm, topk_w, T, k, d, (TO*)y);      \
    else if (k <= 4) combine_kernel<TI, TO, 4, 4><<<grid, block, 0, s>>>((const TI*)yp, yp_scale, inv_perm, topk_w, T, k, d, (TO*)y); \
    else combine_kernel<TI, TO, 8, 2><<<grid, block, 0, s>>>((const TI*)yp, yp_scale, inv_perm, topk_w, T, k, d, (TO*)y);             \
    MOE_LAUNCH_CHECK();                                                                                               \
    return MOE_OK;                                                                                                    \
  }
  MOE_COMBINE_CASE(MOE_F32, MOE_F32, float, float)
  MOE_COMBINE_CASE(MOE_BF16, MOE_BF16, bf16, bf16)
  MOE_COMBINE_CASE(MOE_BF16, MOE_F32, bf16, float)
  MOE_COMBINE_CASE(MOE_F8E4M3, MOE_BF16, uint8_t, bf16)
  MOE_COMBINE_CASE(MOE_F8E4M3, MOE_F32, uint8_t, float)
#undef MOE_COMBINE_CASE
  return MOE_ERR_UNSUPPORTED;
}

int launch_gate_grad(const void* dy, moe_dtype dy_dt, const void* yp, const float* yp_scale, moe_dtype dt,
                     const int32_t* inv_perm, int T, int k, int d, float* d_topk_w, hipStream_t s) {
  const dim3 grid(row_grid(T)), block(64 * kWavesPerBlock);
#define MOE_GG_CASE(DD, DI, TD, TI)                                                                                    \
  if (dy_dt == DD && dt == DI) {                                                                                       \
    if (k <= 2) gate_grad_kernel<TD, TI, 2, 4><<<grid, block, 0, s>>>((const TD*)dy, (const TI*)yp, yp_scale, inv_perm, T, k, d, d_topk_w);      \
    else if (k <= 4) gate_grad_kernel<TD, TI, 4, 1><<<grid, block, 0, s>>>((const TD*)dy, (const TI*)yp, yp_scale, inv_perm, T, k, d, d_topk_w); \
    else gate_grad_kernel<TD, TI, 8, 1><<<grid, block, 0, s>>>((const TD*)dy, (const TI*)yp, yp_scale, inv_perm, T, k, d, d_topk_w);             \
    MOE_LAUNCH_CHECK();                                                                                                \
    return MOE_OK;                                                                                                     \
  }
  MOE_GG_CASE(MOE_F32, MOE_F32, float, float)
  MOE_GG_CASE(MOE_BF16, MOE_BF16, bf16, bf16)
  MOE_GG_CASE(MOE_BF16, MOE_F8E4M3, bf16, uint8_t)
  MOE_GG_CASE(MOE_F32, MOE_F8E4M3, float, uint8_t)
#undef MOE_GG_CASE
  return MOE_ERR_UNSUPPORTED;
}

}  // namespace moe
