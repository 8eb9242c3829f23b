// Batched matrix transpose, dst[b][c][r] = src[b][r][c].  Used once at set-up, outside the training step: the FP8
// backward (Section 7 "FP8 training": per-channel quantisation for the backward pass) contracts the weights along
// their other axis, so they are cast a second time from a transposed copy, W1[e]^T [d,2f] and W2[e]^T [f,d].
// 64x64 element tiles through LDS (padded rows: no bank conflicts), coalesced on both sides.
#include "moe_common.h"

namespace moe {
namespace {

template <typename T>
__global__ void __launch_bounds__(256) transpose_kernel(const T* __restrict__ src, int rows, int cols, T* __restrict__ dst) {
  __shared__ T tile[64][65];
  const long mat = (long)rows * cols;
  const T* s = src + blockIdx.z * mat;
  T* d = dst + blockIdx.z * mat;
  const int r0 = blockIdx.y * 64, c0 = blockIdx.x * 64;
  const int tx = threadIdx.x % 64, ty = threadIdx.x / 64;
  for (int i = ty; i < 64; i += 4) {
    const int r = r0 + i, c = c0 + tx;
    if (r < rows && c < cols) tile[i][tx] = s[(long)r * cols + c];
  }
  __syncthreads();
  for (int i = ty; i < 64; i += 4) {
    const int c = c0 + i, r = r0 + tx;
    if (r < rows && c < cols) d[(long)c * rows + r] = tile[tx][i];
  }
}

template <typename T>
int launch_t(const void* src, int batch, int rows, int cols, void* dst, hipStream_t s) {
  const dim3 grid((unsigned)cdiv(cols, 64), (unsigned)cdiv(rows, 64), (unsigned)batch);
  transpose_kernel<T><<<grid, dim3(256), 0, s>>>(static_cast<const T*>(src), rows, cols, static_cast<T*>(dst));
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

}  // namespace

int launch_transpose(const void* src, moe_dtype dt, int batch, int rows, int cols, void* dst, hipStream_t s) {
  if (dt == MOE_F32) return launch_t<uint32_t>(src, batch, rows, cols, dst, s);
  if (dt == MOE_BF16) return launch_t<uint16_t>(src, batch, rows, cols, dst, s);
  return launch_t<uint8_t>(src, batch, rows, cols, dst, s);
}

}  // namespace moe
