// Gating and row map (Section 2.1: top-k gate; Section 3.2 "Efficient operators": the mapping from
// input rows to output rows is computed once from the routing result; Section 4.2: rows ordered by
// expert, then by source).  The paper lists the "multitude of small operators" of the gate as a
// launch-latency straggler (Section 7); here the whole step is three launches and no host read-back:
//   1. route_topk_kernel   per token: k-fold arg-max under the total order (logit desc, id asc) with
//                          wave shuffles, softmax over the selected logits, per-chunk expert histogram
//   2. route_scan_kernel   exclusive scan of the histograms over chunks (per expert) and over experts
//   3. route_rank_kernel   stable rank of every assignment inside its expert via wave ballots
// No atomics decide an order, so perm / inv_perm are unique and reproducible bit for bit.
#include "moe_common.h"

namespace moe {
namespace {

constexpr int kMaxValsPerLane = MOE_MAX_EXPERTS / 64;

__device__ __forceinline__ bool better(float az, int ae, float bz, int be) {
  return az > bz || (az == bz && ae < be);
}

// G lanes cooperate on one token; lane `sub` holds experts sub, sub+G, sub+2G, ...
template <int G>
__global__ void __launch_bounds__(256) route_topk_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                         int renorm, int chunk_tokens, int32_t* __restrict__ topk_idx,
                                                         float* __restrict__ topk_w, int32_t* __restrict__ chunk_hist) {
  __shared__ int hist[MOE_MAX_EXPERTS];
  for (int e = threadIdx.x; e < MOE_MAX_EXPERTS; e += blockDim.x) hist[e] = 0;
  __syncthreads();

  const int sub = threadIdx.x % G;
  const int grp = threadIdx.x / G;
  const int ngroups = blockDim.x / G;
  const int t_begin = blockIdx.x * chunk_tokens;
  const int t_end = min(t_begin + chunk_tokens, T);
  const int vpl = (E + G - 1) / G;

  for (int t = t_begin + grp; t < t_end; t += ngroups) {
    float v[kMaxValsPerLane];
    unsigned taken = 0;
#pragma unroll
    for (int i = 0; i < kMaxValsPerLane; ++i) {
      const int e = sub + i * G;
      if (i < vpl && e < E) {
        v[i] = logits[(long)t * E + e];
      } else {
        v[i] = -INFINITY;
        taken |= 1u << i;
      }
    }
    float my_z = -INFINITY;
    int my_e = 0;
    float top_z = 0.f;
    for (int j = 0; j < k; ++j) {
      float bz = -INFINITY;
      int be = 0x7fffffff;
#pragma unroll
      for (int i = 0; i < kMaxValsPerLane; ++i) {
        const int e = sub + i * G;
        if (!((taken >> i) & 1u) && better(v[i], e, bz, be)) { bz = v[i]; be = e; }
      }
#pragma unroll
      for (int off = G / 2; off >= 1; off >>= 1) {
        const float oz = __shfl_xor(bz, off, G);
        const int oe = __shfl_xor(be, off, G);
        if (better(oz, oe, bz, be)) { bz = oz; be = oe; }
      }
      if (be % G == sub) taken |= 1u << (be / G);   // the owner retires the winner
      if (sub == j) { my_z = bz; my_e = be; }
      if (j == 0) top_z = bz;
    }
    const bool holds_slot = sub < k;
    const float ex = holds_slot ? expf(my_z - top_z) : 0.f;
    float den;
    if (renorm) {
      den = ex;
    } else {
      den = 0.f;
#pragma unroll
      for (int i = 0; i < kMaxValsPerLane; ++i)
        if (i < vpl && sub + i * G < E) den += expf(v[i] - top_z);
    }
#pragma unroll
    for (int off = G / 2; off >= 1; off >>= 1) den += __shfl_xor(den, off, G);
    if (holds_slot) {
      topk_idx[(long)t * k + sub] = my_e;
      topk_w[(long)t * k + sub] = ex / den;
      atomicAdd(&hist[my_e], 1);     // integer count: the sum does not depend on the order
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += blockDim.x) chunk_hist[(long)blockIdx.x * E + e] = hist[e];
}

// chunk_hist [nchunks, E] -> exclusive prefix over chunks, in place; counts, offsets.
__global__ void __launch_bounds__(MOE_MAX_EXPERTS) route_scan_kernel(int32_t* __restrict__ chunk_hist, int nchunks,
                                                                     int E, int32_t* __restrict__ counts,
                                                                     int32_t* __restrict__ offsets) {
  __shared__ int total[MOE_MAX_EXPERTS];
  const int e = threadIdx.x;
  if (e < E) {
    int run = 0;
    for (int c = 0; c < nchunks; ++c) {
      const int h = chunk_hist[(long)c * E + e];
      chunk_hist[(long)c * E + e] = run;
      run += h;
    }
    total[e] = run;
    counts[e] = run;
  }
  __syncthreads();
  if (e == 0) {
    int run = 0;
    for (int i = 0; i < E; ++i) { offsets[i] = run; run += total[i]; }
    offsets[E] = run;
  }
}

// One wave per chunk walks its assignments in order, 64 at a time.
__global__ void __launch_bounds__(64) route_rank_kernel(const int32_t* __restrict__ topk_idx, int T, int E, int k,
                                                        int chunk_tokens, const int32_t* __restrict__ chunk_base,
                                                        const int32_t* __restrict__ offsets,
                                                        int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm) {
  __shared__ int next_row[MOE_MAX_EXPERTS];
  const int lane = threadIdx.x;
  for (int e = lane; e < E; e += 64) next_row[e] = offsets[e] + chunk_base[(long)blockIdx.x * E + e];
  __syncthreads();
  const long a_begin = (long)blockIdx.x * chunk_tokens * k;
  const long a_end = min((long)(blockIdx.x + 1) * chunk_tokens, (long)T) * k;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  for (long base = a_begin; base < a_end; base += 64) {
    const long a = base + lane;
    const bool valid = a < a_end;
    const int e = valid ? topk_idx[a] : -1;
    bool pending = valid;
    unsigned long long todo = __ballot(pending);
    while (todo) {
      const int leader = __ffsll((long long)todo) - 1;
      const int e0 = __shfl(e, leader);
      const unsigned long long same = __ballot(pending && e == e0);
      const int start = next_row[e0];
      if (pending && e == e0) {
        const int r = start + __popcll(same & lt_mask);
        inv_perm[a] = r;
        perm[r] = (int)a;
        pending = false;
      }
      __syncthreads();                       // every lane has read next_row[e0]
      if (lane == leader) next_row[e0] = start + __popcll(same);
      __syncthreads();
      todo &= ~same;
    }
  }
}

__global__ void __launch_bounds__(256) route_bwd_kernel(const float* __restrict__ logits,
                                                        const int32_t* __restrict__ topk_idx,
                                                        const float* __restrict__ topk_w,
                                                        const float* __restrict__ d_topk_w, int T, int E, int k,
                                                        int renorm, float* __restrict__ d_logits) {
  const long total = (long)T * E;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const long t = i / E;
    const int e = (int)(i % E);
    float inner = 0.f, mine = 0.f;
    for (int j = 0; j < k; ++j) {
      const float w = topk_w[t * k + j], dw = d_topk_w[t * k + j];
      inner += w * dw;
      if (topk_idx[t * k + j] == e) mine = w * dw;
    }
    float out;
    if (renorm) {
      // selected: w_j*(dw_j - inner) = mine - w_j*inner; written as below to keep one expression
      float wj = 0.f;
      for (int j = 0; j < k; ++j)
        if (topk_idx[t * k + j] == e) wj = topk_w[t * k + j];
      out = mine - wj * inner;
    } else {
      float m = -INFINITY;
      for (int c = 0; c < E; ++c) m = fmaxf(m, logits[t * E + c]);
      float den = 0.f;
      for (int c = 0; c < E; ++c) den += expf(logits[t * E + c] - m);
      const float p = expf(logits[t * E + e] - m) / den;
      out = mine - p * inner;
    }
    d_logits[i] = out;
  }
}

template <int G>
int launch_topk(const float* logits, int T, int E, int k, int renorm, int chunk_tokens, int nchunks, int32_t* idx,
                float* w, int32_t* hist, hipStream_t s) {
  route_topk_kernel<G><<<nchunks, 256, 0, s>>>(logits, T, E, k, renorm, chunk_tokens, idx, w, hist);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

}  // namespace

size_t route_ws_bytes(int T, int E) {
  const int tb = route_chunk_tokens(T);
  return align_up((size_t)cdiv(T, tb) * E * sizeof(int32_t), 256);
}

int launch_route(const float* logits, int T, int E, int k, int renorm, int32_t* idx, float* w, int32_t* counts,
                 int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* ws, hipStream_t s) {
  const int tb = route_chunk_tokens(T);
  const int nchunks = cdiv(T, tb);
  int32_t* hist = static_cast<int32_t*>(ws);
  int rc;
  if (E <= 1) rc = launch_topk<1>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, s);
  else if (E <= 2) rc = launch_topk<2>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, s);
  else if (E <= 4) rc = launch_topk<4>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, s);
  else if (E <= 8) rc = launch_topk<8>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, s);
  else if (E <= 16) rc = launch_topk<16>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, s);
  else if (E <= 32) rc = launch_topk<32>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, s);
  else rc = launch_topk<64>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, s);
  if (rc != MOE_OK) return rc;
  route_scan_kernel<<<1, MOE_MAX_EXPERTS, 0, s>>>(hist, nchunks, E, counts, offsets);
  MOE_LAUNCH_CHECK();
  route_rank_kernel<<<nchunks, 64, 0, s>>>(idx, T, E, k, tb, hist, offsets, perm, inv_perm);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

int launch_route_bwd(const float* logits, const int32_t* idx, const float* w, const float* dw, int T, int E, int k,
                     int renorm, float* d_logits, hipStream_t s) {
  long blocks = ((long)T * E + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  route_bwd_kernel<<<(int)blocks, 256, 0, s>>>(logits, idx, w, dw, T, E, k, renorm, d_logits);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

}  // namespace moe
