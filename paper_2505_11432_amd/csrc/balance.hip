// Device-level auxiliary balance loss (Section 3.2 "Load balance": the experts placed on one GPU form a group and
// the balance loss is computed per device rather than per expert, as in DeepSeek-V2).
//   s[t,e]  = softmax of the token's logits over all E experts (affinity)
//   f_e     = E / (k T) * (number of assignments to e),   P_e = mean_t s[t,e]
//   f'_g    = mean of f_e over the experts of device g,    P'_g = sum of P_e over them
//   loss    = alpha * sum_g f'_g P'_g
//   dz[t,c] = alpha / T * s[t,c] * (F_c - sum_e s[t,e] F_e),  F_e = f' of e's device (f is piecewise constant)
// P is reduced in two passes with a fixed order (per-chunk partial sums, then a sum over the chunks): no float
// atomics, so the loss is reproducible bit for bit.
#include "moe_common.h"

namespace moe {
namespace {

constexpr int kMaxVals = MOE_MAX_EXPERTS / 64;     // experts per lane when one wave holds a token's logits

// one wave per token; returns the lane's softmax values s[lane + 64 i]
__device__ __forceinline__ void token_softmax(const float* __restrict__ row, int E, int lane, float (&s)[kMaxVals]) {
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < kMaxVals; ++i) {
    const int e = lane + 64 * i;
    s[i] = e < E ? row[e] : -INFINITY;
    m = fmaxf(m, s[i]);
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
  float den = 0.f;
#pragma unroll
  for (int i = 0; i < kMaxVals; ++i) {
    s[i] = (lane + 64 * i < E) ? expf(s[i] - m) : 0.f;
    den += s[i];
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) den += __shfl_xor(den, off);
  const float inv = 1.0f / den;
#pragma unroll
  for (int i = 0; i < kMaxVals; ++i) s[i] *= inv;
}

// partial[chunk][e] = sum of s[t,e] over the chunk's tokens (4 waves per block, combined through LDS in wave order)
__global__ void __launch_bounds__(256) balance_partial_kernel(const float* __restrict__ logits, int T, int E,
                                                              int chunk_tokens, float* __restrict__ partial) {
  __shared__ float acc_lds[4][MOE_MAX_EXPERTS];
  const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  const int t_begin = blockIdx.x * chunk_tokens, t_end = min(t_begin + chunk_tokens, T);
  float acc[kMaxVals];
#pragma unroll
  for (int i = 0; i < kMaxVals; ++i) acc[i] = 0.f;
  for (int t = t_begin + wave; t < t_end; t += 4) {
    float s[kMaxVals];
    token_softmax(logits + (long)t * E, E, lane, s);
#pragma unroll
    for (int i = 0; i < kMaxVals; ++i) acc[i] += s[i];
  }
#pragma unroll
  for (int i = 0; i < kMaxVals; ++i) acc_lds[wave][lane + 64 * i] = acc[i];
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += blockDim.x)
    partial[(long)blockIdx.x * E + e] = ((acc_lds[0][e] + acc_lds[1][e]) + acc_lds[2][e]) + acc_lds[3][e];
}

// one block: P_e = sum over chunks (ascending) / T; group sums; the loss
__global__ void __launch_bounds__(256) balance_final_kernel(const float* __restrict__ partial, int nchunks,
                                                            const int32_t* __restrict__ counts, int T, int E, int k,
                                                            int n_groups, float alpha, float* __restrict__ loss,
                                                            float* __restrict__ group_f, float* __restrict__ group_p) {
  __shared__ float P[MOE_MAX_EXPERTS];
  __shared__ float gf[MOE_MAX_EXPERTS], gp[MOE_MAX_EXPERTS];
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    float s = 0.f;
    for (int c = 0; c < nchunks; ++c) s += partial[(long)c * E + e];
    P[e] = s / (float)T;
  }
  __syncthreads();
  const int per = E / n_groups;
  for (int g = threadIdx.x; g < n_groups; g += blockDim.x) {
    float fs = 0.f, ps = 0.f;
    for (int j = 0; j < per; ++j) {
      fs += (float)counts[g * per + j] * ((float)E / ((float)k * (float)T));
      ps += P[g * per + j];
    }
    gf[g] = fs / (float)per;
    gp[g] = ps;
    group_f[g] = gf[g];
    group_p[g] = gp[g];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float l = 0.f;
    for (int g = 0; g < n_groups; ++g) l += gf[g] * gp[g];
    loss[0] = alpha * l;
  }
}

// d_logits[t,c] += alpha/T * s_c * (F_c - sum_e s_e F_e); one wave per token
__global__ void __launch_bounds__(256) balance_bwd_kernel(const float* __restrict__ logits,
                                                          const float* __restrict__ group_f, int T, int E,
                                                          int per_group, float scale, float* __restrict__ d_logits) {
  const int lane = threadIdx.x % 64;
  const int wave = blockIdx.x * 4 + threadIdx.x / 64, nwaves = gridDim.x * 4;
  float F[kMaxVals];
#pragma unroll
  for (int i = 0; i < kMaxVals; ++i) {
    const int e = lane + 64 * i;
    F[i] = e < E ? group_f[e / per_group] : 0.f;
  }
  for (int t = wave; t < T; t += nwaves) {
    float s[kMaxVals];
    token_softmax(logits + (long)t * E, E, lane, s);
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < kMaxVals; ++i) dot += s[i] * F[i];
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off);
#pragma unroll
    for (int i = 0; i < kMaxVals; ++i) {
      const int e = lane + 64 * i;
      if (e < E) d_logits[(long)t * E + e] += scale * s[i] * (F[i] - dot);
    }
  }
}

}  // namespace

size_t balance_ws_bytes(int T, int E) {
  const int tb = route_chunk_tokens(T);
  return align_up((size_t)cdiv(T, tb) * E * sizeof(float), 256);
}

int launch_balance_loss(const float* logits, const int32_t* counts, int T, int E, int k, int n_groups, float alpha,
                        float* loss, float* group_f, float* group_p, void* ws, hipStream_t s) {
  const int tb = route_chunk_tokens(T);
  const int nchunks = cdiv(T, tb);
  float* partial = static_cast<float*>(ws);
  balance_partial_kernel<<<nchunks, 256, 0, s>>>(logits, T, E, tb, partial);
  MOE_LAUNCH_CHECK();
  balance_final_kernel<<<1, 256, 0, s>>>(partial, nchunks, counts, T, E, k, n_groups, alpha, loss, group_f, group_p);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

int launch_balance_loss_bwd(const float* logits, const float* group_f, int T, int E, int n_groups, float alpha,
                            float* d_logits, hipStream_t s) {
  int blocks = cdiv(T, 4);
  if (blocks > 256 * 8) blocks = 256 * 8;
  balance_bwd_kernel<<<blocks, 256, 0, s>>>(logits, group_f, T, E, E / n_groups, alpha / (float)T, d_logits);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

}  // namespace moe
