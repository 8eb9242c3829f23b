// Gating and row map (Section 2.1: top-k gate; Section 3.2 "Efficient operators": the mapping from
// input rows to output rows is computed once from the routing result; Section 4.2: rows ordered by
// expert, then by source).  The paper lists the "multitude of small operators" of the gate as a
// launch-latency straggler (Section 7); here the whole step is three launches and no host read-back:
//   1. route_topk_kernel   per token: k-fold arg-max under the total order (logit desc, id asc) with
//                          shuffles inside groups of <= 16 lanes (4+ tokens per wave at a time), softmax
//                          over the selected logits, per-chunk expert histogram
//   2. route_scan_kernel   one wave per expert: exclusive scan of its per-chunk counts
//   3. route_rank_kernel   offsets = scan of the counts; stable rank of every assignment inside its
//                          expert: equal-expert lanes found with one ballot per bit of the expert id
// No atomics decide an order, so perm / inv_perm are unique and reproducible bit for bit.
#include "moe_common.h"

namespace moe {
namespace {

__device__ __forceinline__ bool better(float az, int ae, float bz, int be) {
  return az > bz || (az == bz && ae < be);
}

// G lanes (G <= 16) cooperate on one token, 64/G tokens per wave at a time; lane `sub` of a group holds the
// VPL experts sub, sub+G, sub+2G, ...  The per-chunk histogram is written transposed, [E][nchunks], so the
// scan kernel reads rows.
template <int G, int VPL>
__global__ void __launch_bounds__(256) route_topk_kernel(const float* __restrict__ logits, int T, int E, int k,
                                                         int renorm, int chunk_tokens, int nchunks,
                                                         int32_t* __restrict__ topk_idx, float* __restrict__ topk_w,
                                                         int32_t* __restrict__ chunk_hist,
                                                         float* __restrict__ score) {
  __shared__ int hist[MOE_MAX_EXPERTS];
  for (int e = threadIdx.x; e < MOE_MAX_EXPERTS; e += blockDim.x) hist[e] = 0;
  __syncthreads();

  const int sub = threadIdx.x % G;
  const int grp = threadIdx.x / G;
  const int ngroups = blockDim.x / G;
  const int t_begin = blockIdx.x * chunk_tokens;
  const int t_end = min(t_begin + chunk_tokens, T);

  // all groups of a wave run the same number of rounds (shuffles need the whole group active; a group past
  // the end of the chunk works on the last token again and skips the stores)
  const int rounds = (t_end - t_begin + ngroups - 1) / ngroups;
  for (int it = 0; it < rounds; ++it) {
    const int t_raw = t_begin + it * ngroups + grp;
    const bool live = t_raw < t_end;
    const int t = live ? t_raw : t_end - 1;
    float v[VPL];
    unsigned taken = 0;
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
      const int e = sub + i * G;
      if (e < E) {
        v[i] = logits[(long)t * E + e];
      } else {
        v[i] = -INFINITY;
        taken |= 1u << i;
      }
    }
    float my_z = -INFINITY, top_z = 0.f;
    int my_e = 0;
    for (int j = 0; j < k; ++j) {
      float bz = -INFINITY;
      int be = 0x7fffffff;
#pragma unroll
      for (int i = 0; i < VPL; ++i) {
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
      if (sub == j) { my_z = bz; my_e = be; }        // lane j keeps slot j (k <= min(E, 16) <= G)
      if (j == 0) top_z = bz;
    }
    // weights: softmax over the selected logits (renorm) or over all logits read at the selected ones
    const bool holds_slot = sub < k;
    const float ex = holds_slot ? expf(my_z - top_z) : 0.f;
    float den, den_all = 0.f;
    if (!renorm || score != nullptr) {
#pragma unroll
      for (int i = 0; i < VPL; ++i)
        if (sub + i * G < E) den_all += expf(v[i] - top_z);
#pragma unroll
      for (int off = G / 2; off >= 1; off >>= 1) den_all += __shfl_xor(den_all, off, G);
    }
    if (renorm) {
      den = ex;
#pragma unroll
      for (int off = G / 2; off >= 1; off >>= 1) den += __shfl_xor(den, off, G);
    } else {
      den = den_all;
    }
    if (live && holds_slot) {
      topk_idx[(long)t * k + sub] = my_e;
      topk_w[(long)t * k + sub] = ex / den;
      if (score != nullptr) score[(long)t * k + sub] = ex / den_all;     // affinity: softmax over all experts
      atomicAdd(&hist[my_e], 1);     // integer count: the sum does not depend on the order
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += blockDim.x) chunk_hist[(long)e * nchunks + blockIdx.x] = hist[e];
}

// One wave per expert: exclusive prefix of that expert's per-chunk counts, in place; counts[e] = total.
__global__ void __launch_bounds__(64) route_scan_kernel(int32_t* __restrict__ chunk_hist, int nchunks,
                                                        int32_t* __restrict__ counts) {
  const int e = blockIdx.x, lane = threadIdx.x;
  int32_t* row = chunk_hist + (long)e * nchunks;
  const int per_lane = (nchunks + 63) / 64;          // nchunks <= 1024 -> at most 16
  const int c0 = lane * per_lane;
  int vals[16];
  int sum = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    vals[i] = (i < per_lane && c0 + i < nchunks) ? row[c0 + i] : 0;
    sum += vals[i];
  }
  int incl = sum;                                    // inclusive scan of the lane sums across the wave
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_up(incl, off);
    if (lane >= off) incl += o;
  }
  int run = incl - sum;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    if (i < per_lane && c0 + i < nchunks) row[c0 + i] = run;
    run += vals[i];
  }
  if (lane == 63) counts[e] = incl;
}

// One wave per chunk walks its assignments in order, 64 at a time.  Lanes with the same expert are found with
// one ballot per bit of the expert id; the rank inside the group is a popcount of the lower lanes.
// Only experts in [e_lo, e_hi) get rows (one GPU's expert-parallel share: the local scatter of Section 3.2);
// assignments to other experts get inv_perm = -1.  offsets has e_hi - e_lo + 1 entries.
__global__ void __launch_bounds__(64) route_rank_kernel(const int32_t* __restrict__ topk_idx, int T, int E, int k,
                                                        int e_lo, int e_hi, int chunk_tokens, int nchunks,
                                                        const int32_t* __restrict__ chunk_base,
                                                        const int32_t* __restrict__ counts,
                                                        int32_t* __restrict__ offsets,
                                                        int32_t* __restrict__ perm, int32_t* __restrict__ inv_perm,
                                                        const uint8_t* __restrict__ keep) {
  __shared__ int next_row[MOE_MAX_EXPERTS];
  __shared__ int expert_off[MOE_MAX_EXPERTS + 1];
  const int lane = threadIdx.x;
  // offsets = exclusive scan of counts (every block recomputes it; block 0 publishes it)
  int run = 0;
  for (int e0 = 0; e0 < E; e0 += 64) {
    const int e = e0 + lane;
    const int c = (e >= e_lo && e < e_hi) ? counts[e] : 0;
    int incl = c;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int o = __shfl_up(incl, off);
      if (lane >= off) incl += o;
    }
    if (e < E) expert_off[e] = run + incl - c;
    run += __shfl(incl, 63);
  }
  if (lane == 0) expert_off[E] = run;
  __syncthreads();
  if (blockIdx.x == 0)
    for (int e = e_lo + lane; e <= e_hi; e += 64) offsets[e - e_lo] = expert_off[e];
  for (int e = lane; e < E; e += 64) next_row[e] = expert_off[e] + chunk_base[(long)e * nchunks + blockIdx.x];
  __syncthreads();

  int ebits = 0;
  while ((1 << ebits) < E) ++ebits;
  const long a_begin = (long)blockIdx.x * chunk_tokens * k;
  const long a_end = min((long)(blockIdx.x + 1) * chunk_tokens, (long)T) * k;
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  for (long base = a_begin; base < a_end; base += 64) {
    const long a = base + lane;
    const bool valid = a < a_end;
    const int e = valid ? topk_idx[a] : 0;
    const bool gets_row = valid && e >= e_lo && e < e_hi && (keep == nullptr || keep[a] != 0);
    unsigned long long same = __ballot(gets_row);
    for (int b = 0; b < ebits; ++b) {
      const unsigned long long mb = __ballot((e >> b) & 1);
      same &= ((e >> b) & 1) ? mb : ~mb;
    }
    if (valid) {
      if (gets_row) {
        const int start = next_row[e];
        const int r = start + __popcll(same & lt_mask);
        inv_perm[a] = r;
        perm[r] = (int)a;
        if ((same >> lane) >> 1 == 0) next_row[e] = start + __popcll(same);   // the group's highest lane advances the row
      } else {
        inv_perm[a] = -1;
      }
    }
    __syncthreads();
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


// ---- device-level token dropping (Section 3.2 "Load balance": capacity per device, the experts of one GPU form
// a group, as in DeepSeek-V2: when a device gets more than `capacity` assignments the ones with the lowest
// affinity are dropped) -------------------------------------------------------------------------------------
// Order of an assignment inside its device: key = affinity bits (positive floats order like integers) in the
// high word, ~assignment id in the low word, so larger key = kept first and equal affinities keep the lower id.
// The capacity-th largest key of every device is found by a most-significant-digit radix select, 8 bits per
// pass: one kernel counts the digit of every key that still matches the device's prefix (integer atomics: the
// counts do not depend on the order), one small kernel picks the digit and narrows the prefix.
struct SelectState {
  unsigned long long prefix[MOE_MAX_EXPERTS];     // high bits of the threshold found so far, per device
  int remaining[MOE_MAX_EXPERTS];                 // rank of the threshold among the keys that match the prefix
  int all_kept[MOE_MAX_EXPERTS];                  // device has no more than `capacity` assignments
  int hist[MOE_MAX_EXPERTS][256];
};

__device__ __forceinline__ unsigned long long drop_key(float score, long a) {
  return ((unsigned long long)__float_as_uint(score) << 32) | (unsigned long long)(0xffffffffu - (unsigned)a);
}

__global__ void __launch_bounds__(256) select_init_kernel(SelectState* st, int n_groups, int capacity) {
  for (int i = threadIdx.x; i < MOE_MAX_EXPERTS * 256; i += blockDim.x) (&st->hist[0][0])[i] = 0;
  for (int g = threadIdx.x; g < n_groups; g += blockDim.x) {
    st->prefix[g] = 0ull;
    st->remaining[g] = capacity;
    st->all_kept[g] = 0;
  }
}

// LDS_GROUPS > 0: the block counts into LDS first (up to 16 devices) and adds its totals once; otherwise straight
// into the global histogram.
template <int LDS_GROUPS>
__global__ void __launch_bounds__(256) select_count_kernel(const int32_t* __restrict__ topk_idx,
                                                           const float* __restrict__ score, long M, int per_group,
                                                           int n_groups, int pass, SelectState* st) {
  __shared__ int h[LDS_GROUPS > 0 ? LDS_GROUPS : 1][256];
  if constexpr (LDS_GROUPS > 0) {
    for (int i = threadIdx.x; i < LDS_GROUPS * 256; i += blockDim.x) (&h[0][0])[i] = 0;
    __syncthreads();
  }
  const int shift = 56 - 8 * pass;
  for (long a = blockIdx.x * (long)blockDim.x + threadIdx.x; a < M; a += (long)gridDim.x * blockDim.x) {
    const int g = topk_idx[a] / per_group;
    if (st->all_kept[g]) continue;
    const unsigned long long key = drop_key(score[a], a);
    const bool match = pass == 0 || (key >> (shift + 8)) == st->prefix[g];
    if (match) {
      const int digit = (int)((key >> shift) & 0xffull);
      if constexpr (LDS_GROUPS > 0) atomicAdd(&h[g][digit], 1);
      else atomicAdd(&st->hist[g][digit], 1);
    }
  }
  if constexpr (LDS_GROUPS > 0) {
    __syncthreads();
    for (int i = threadIdx.x; i < n_groups * 256; i += blockDim.x) {
      const int v = (&h[0][0])[i];
      if (v) atomicAdd(&st->hist[i / 256][i % 256], v);
    }
  }
}

// One wave per device: lane l holds the counts of digits 4l .. 4l+3; the digit that contains the threshold is the
// highest d with (keys in digits above d) + hist[d] >= remaining.
__global__ void __launch_bounds__(256) select_pick_kernel(SelectState* st, int n_groups, int pass) {
  const int lane = threadIdx.x % 64;
  const int g = blockIdx.x * 4 + threadIdx.x / 64;
  if (g >= n_groups || st->all_kept[g]) return;            // wave-uniform
  int c[4];
  int mine = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    c[i] = st->hist[g][4 * lane + i];
    st->hist[g][4 * lane + i] = 0;
    mine += c[i];
  }
  int incl = mine;                                          // inclusive suffix sum over lanes (lane 63 first)
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const int o = __shfl_down(incl, off);
    if (lane + off < 64) incl += o;
  }
  const int total = __shfl(incl, 0);
  const int remaining = st->remaining[g];
  if (pass == 0 && total <= remaining) {
    if (lane == 0) { st->all_kept[g] = 1; st->prefix[g] = 0ull; }   // threshold 0: every key passes
    return;
  }
  int cum = incl - mine;                                    // keys in digits above this lane's four
  int hit = -1, cum_at_hit = 0;
#pragma unroll
  for (int i = 3; i >= 0; --i) {
    if (hit < 0 && cum + c[i] >= remaining) { hit = 4 * lane + i; cum_at_hit = cum; }
    cum += c[i];
  }
  const unsigned long long hits = __ballot(hit >= 0);
  // remaining <= total here, so some lane hits; remaining = 0 (capacity 0) hits in lane 63 at digit 255
  const int winner = 63 - __builtin_clzll(hits);
  if (lane == winner) {
    st->prefix[g] = (st->prefix[g] << 8) | (unsigned long long)hit;
    st->remaining[g] = remaining - cum_at_hit;
  }
}

// keep[a] and the per-chunk expert histogram of the kept assignments (same layout as route_topk_kernel's)
__global__ void __launch_bounds__(256) keep_hist_kernel(const int32_t* __restrict__ topk_idx,
                                                        const float* __restrict__ score, int T, int E, int k,
                                                        int per_group, int chunk_tokens, int nchunks,
                                                        const SelectState* __restrict__ st,
                                                        uint8_t* __restrict__ keep, int32_t* __restrict__ chunk_hist) {
  __shared__ int hist[MOE_MAX_EXPERTS];
  for (int e = threadIdx.x; e < MOE_MAX_EXPERTS; e += blockDim.x) hist[e] = 0;
  __syncthreads();
  const long a_begin = (long)blockIdx.x * chunk_tokens * k;
  const long a_end = min((long)(blockIdx.x + 1) * chunk_tokens, (long)T) * k;
  for (long a = a_begin + threadIdx.x; a < a_end; a += blockDim.x) {
    const int e = topk_idx[a];
    const int g = e / per_group;
    const bool kp = st->all_kept[g] || drop_key(score[a], a) >= st->prefix[g];
    keep[a] = kp ? 1 : 0;
    if (kp) atomicAdd(&hist[e], 1);
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += blockDim.x) chunk_hist[(long)e * nchunks + blockIdx.x] = hist[e];
}

template <int G, int VPL>
int launch_topk(const float* logits, int T, int E, int k, int renorm, int chunk_tokens, int nchunks, int32_t* idx,
                float* w, int32_t* hist, float* score, hipStream_t s) {
  route_topk_kernel<G, VPL><<<nchunks, 256, 0, s>>>(logits, T, E, k, renorm, chunk_tokens, nchunks, idx, w, hist, score);
  MOE_LAUNCH_CHECK();
  return MOE_OK;
}

}  // namespace

size_t route_ws_bytes(int T, int E) {
  const int tb = route_chunk_tokens(T);
  return align_up((size_t)cdiv(T, tb) * E * sizeof(int32_t), 256);
}

size_t route_capacity_ws_bytes(int T, int E, int k) {
  return route_ws_bytes(T, E) + align_up(sizeof(SelectState), 256) + align_up((size_t)T * k, 256);
}

// n_groups = 0: no dropping.  Otherwise `score` [T,k] must be given and ws holds route_capacity_ws_bytes.
int launch_route(const float* logits, int T, int E, int k, int renorm, int e_lo, int e_hi, int n_groups, int capacity,
                 int32_t* idx, float* w, float* score, int32_t* counts, int32_t* offsets, int32_t* perm,
                 int32_t* inv_perm, void* ws, hipStream_t s) {
  const int tb = route_chunk_tokens(T);
  const int nchunks = cdiv(T, tb);
  int32_t* hist = static_cast<int32_t*>(ws);
  int rc;
  // lanes per token G = min(16, pow2 >= E) (so G >= k: one slot per lane); experts beyond 16 go VPL per lane
  if (E <= 1) rc = launch_topk<1, 1>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  else if (E <= 2) rc = launch_topk<2, 1>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  else if (E <= 4) rc = launch_topk<4, 1>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  else if (E <= 8) rc = launch_topk<8, 1>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  else if (E <= 16) rc = launch_topk<16, 1>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  else if (E <= 32) rc = launch_topk<16, 2>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  else if (E <= 64) rc = launch_topk<16, 4>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  else if (E <= 128) rc = launch_topk<16, 8>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  else rc = launch_topk<16, 16>(logits, T, E, k, renorm, tb, nchunks, idx, w, hist, score, s);
  if (rc != MOE_OK) return rc;
  const uint8_t* keep = nullptr;
  if (n_groups > 0) {
    char* base = static_cast<char*>(ws) + route_ws_bytes(T, E);
    SelectState* st = reinterpret_cast<SelectState*>(base);
    uint8_t* keep_w = reinterpret_cast<uint8_t*>(base + align_up(sizeof(SelectState), 256));
    const long M = (long)T * k;
    const int per_group = E / n_groups;
    long blocks = (M + 1023) / 1024;
    if (blocks > 512) blocks = 512;
    select_init_kernel<<<1, 256, 0, s>>>(st, n_groups, capacity);
    MOE_LAUNCH_CHECK();
    for (int pass = 0; pass < 8; ++pass) {
      if (n_groups <= 16) select_count_kernel<16><<<(int)blocks, 256, 0, s>>>(idx, score, M, per_group, n_groups, pass, st);
      else select_count_kernel<0><<<(int)blocks, 256, 0, s>>>(idx, score, M, per_group, n_groups, pass, st);
      MOE_LAUNCH_CHECK();
      select_pick_kernel<<<cdiv(n_groups, 4), 256, 0, s>>>(st, n_groups, pass);
      MOE_LAUNCH_CHECK();
    }
    keep_hist_kernel<<<nchunks, 256, 0, s>>>(idx, score, T, E, k, per_group, tb, nchunks, st, keep_w, hist);
    MOE_LAUNCH_CHECK();
    keep = keep_w;
  }
  route_scan_kernel<<<E, 64, 0, s>>>(hist, nchunks, counts);
  MOE_LAUNCH_CHECK();
  route_rank_kernel<<<nchunks, 64, 0, s>>>(idx, T, E, k, e_lo, e_hi, tb, nchunks, hist, counts, offsets, perm, inv_perm,
                                           keep);
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
