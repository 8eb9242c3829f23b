// SwiGLU between FC1 and FC2 (Section 4.1) and its derivative, as stand-alone HBM-bound
// kernels: A = G/(1+exp(-G)) * U on H = [G|U], and (dG, dU) from (G, U, dA).
// 16-byte vectors per lane, one row segment per block column; rows at or beyond *row_limit
// (the number of dispatched rows, read on the device) are left untouched.
#include "moe_common.h"

namespace moe {
namespace {

template <typename T>
__global__ void __launch_bounds__(256) swiglu_fwd_kernel(const T* __restrict__ H, T* __restrict__ A, int M, int f,
                                                         const int32_t* __restrict__ row_limit) {
  constexpr int V = 16 / sizeof(T);
  const int limit = row_limit ? min(*row_limit, M) : M;
  const int vec_per_row = f / V;
  const long total = (long)limit * vec_per_row;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const long r = i / vec_per_row;
    const int c = (int)(i % vec_per_row) * V;
    const Vec16<T> g = *reinterpret_cast<const Vec16<T>*>(H + r * 2 * f + c);
    const Vec16<T> u = *reinterpret_cast<const Vec16<T>*>(H + r * 2 * f + f + c);
    Vec16<T> a;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const float gf = to_f32(g.v[j]);
      a.v[j] = from_f32<T>(gf * sigmoid_f32(gf) * to_f32(u.v[j]));
    }
    *reinterpret_cast<Vec16<T>*>(A + r * f + c) = a;
  }
}

template <typename T>
__global__ void __launch_bounds__(256) swiglu_bwd_kernel(const T* __restrict__ H, const T* __restrict__ dA,
                                                         T* __restrict__ dH, int M, int f,
                                                         const int32_t* __restrict__ row_limit) {
  constexpr int V = 16 / sizeof(T);
  const int limit = row_limit ? min(*row_limit, M) : M;
  const int vec_per_row = f / V;
  const long total = (long)limit * vec_per_row;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const long r = i / vec_per_row;
    const int c = (int)(i % vec_per_row) * V;
    const Vec16<T> g = *reinterpret_cast<const Vec16<T>*>(H + r * 2 * f + c);
    const Vec16<T> u = *reinterpret_cast<const Vec16<T>*>(H + r * 2 * f + f + c);
    const Vec16<T> da = *reinterpret_cast<const Vec16<T>*>(dA + r * f + c);
    Vec16<T> dg, du;
#pragma unroll
    for (int j = 0; j < V; ++j) {
      const float gf = to_f32(g.v[j]), uf = to_f32(u.v[j]), d = to_f32(da.v[j]);
      const float s = sigmoid_f32(gf);
      dg.v[j] = from_f32<T>(d * uf * s * (1.0f + gf * (1.0f - s)));
      du.v[j] = from_f32<T>(d * gf * s);
    }
    *reinterpret_cast<Vec16<T>*>(dH + r * 2 * f + c) = dg;
    *reinterpret_cast<Vec16<T>*>(dH + r * 2 * f + f + c) = du;
  }
}

int grid_for(long work_items) {
  long blocks = (work_items + 255) / 256;
  if (blocks > 256L * 16) blocks = 256L * 16;
  return (int)(blocks < 1 ? 1 : blocks);
}

}  // namespace

int launch_swiglu_fwd(const void* H, void* A, int M, int f, const int32_t* row_limit, moe_dtype dt, hipStream_t s) {
  if (M == 0) return MOE_OK;
  if (dt == MOE_F32) {
    swiglu_fwd_kernel<float><<<grid_for((long)M * f / 4), 256, 0, s>>>((const float*)H, (float*)A, M, f, row_limit);
  } else if (dt == MOE_BF16) {
    swiglu_fwd_kernel<bf16><<<grid_for((long)M * f / 8), 256, 0, s>>>((const bf16*)H, (bf16*)A, M, f, row_limit);
  } else {
    return MOE_ERR_UNSUPPORTED;
  }
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

int launch_swiglu_bwd(const void* H, const void* dA, void* dH, int M, int f, const int32_t* row_limit,
                      moe_dtype dt, hipStream_t s) {
  if (M == 0) return MOE_OK;
  if (dt == MOE_F32) {
    swiglu_bwd_kernel<float><<<grid_for((long)M * f / 4), 256, 0, s>>>((const float*)H, (const float*)dA, (float*)dH,
                                                                        M, f, row_limit);
  } else if (dt == MOE_BF16) {
    swiglu_bwd_kernel<bf16><<<grid_for((long)M * f / 8), 256, 0, s>>>((const bf16*)H, (const bf16*)dA, (bf16*)dH, M,
                                                                       f, row_limit);
  } else {
    return MOE_ERR_UNSUPPORTED;
  }
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

}  // namespace moe
