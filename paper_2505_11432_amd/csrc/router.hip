// Gradients of the router matmul (the "routing scores" operator, Section 7): d_w_r = d_logits^T x and
// dx += d_logits w_r.  Both are skinny (E <= 256 on one side), so they are HBM-bound on x / dx and run
// on the vector ALU with the gate gradient held in scalar registers:
//   d_w_r  two passes, no float atomics: each block owns a slab of 512 columns of x and a chunk of
//          tokens and keeps E x 2 fp32 sums per thread; a second kernel adds the per-chunk partials in
//          a fixed order, so the result is reproducible.
//   dx     one pass over dx: each thread owns 8 columns and walks the experts.
#include "moe_common.h"

namespace moe {
namespace {

constexpr int kETile = 64;        // experts per register tile
constexpr int kSlabCols = 512;    // 256 threads x 2 columns

template <typename T> struct Pair;
template <> struct Pair<float> { __device__ static float2 load(const float* p) { return *reinterpret_cast<const float2*>(p); } };
template <> struct Pair<bf16> {
  __device__ static float2 load(const bf16* p) {
    const unsigned u = *reinterpret_cast<const unsigned*>(p);
    return make_float2(__builtin_bit_cast(float, u << 16), __builtin_bit_cast(float, u & 0xffff0000u));
  }
};

// partial[chunk][e][col] = sum over the chunk's tokens of d_logits[t][e] * x[t][col]
template <typename T>
__global__ void __launch_bounds__(256) router_dwr_partial_kernel(const T* __restrict__ x,
                                                                 const float* __restrict__ d_logits, int Tn, int d,
                                                                 int E, int tokens_per_chunk,
                                                                 float* __restrict__ partial) {
  const int slabs = (d + kSlabCols - 1) / kSlabCols;
  const int slab = blockIdx.x % slabs, chunk = blockIdx.x / slabs;
  const int col = slab * kSlabCols + threadIdx.x * 2;
  const int t0 = chunk * tokens_per_chunk, t1 = min(t0 + tokens_per_chunk, Tn);
  const bool active = col < d;
  for (int e0 = 0; e0 < E; e0 += kETile) {
    float2 acc[kETile];
#pragma unroll
    for (int i = 0; i < kETile; ++i) acc[i] = make_float2(0.f, 0.f);
    for (int t = t0; t < t1; ++t) {
      const float2 xv = active ? Pair<T>::load(x + (long)t * d + col) : make_float2(0.f, 0.f);
      const float* g = d_logits + (long)t * E + e0;      // wave-uniform address: scalar loads
#pragma unroll
      for (int i = 0; i < kETile; ++i) {
        if (e0 + i < E) {
          const float gv = g[i];
          acc[i].x = fmaf(gv, xv.x, acc[i].x);
          acc[i].y = fmaf(gv, xv.y, acc[i].y);
        }
      }
    }
    if (active) {
#pragma unroll
      for (int i = 0; i < kETile; ++i)
        if (e0 + i < E) *reinterpret_cast<float2*>(partial + ((long)chunk * E + e0 + i) * d + col) = acc[i];
    }
  }
}

__global__ void __launch_bounds__(256) router_dwr_reduce_kernel(const float* __restrict__ partial, int chunks,
                                                                long n /* = E*d */, float* __restrict__ d_w_r) {
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < n; i += (long)gridDim.x * blockDim.x) {
    float s = 0.f;
    for (int c = 0; c < chunks; ++c) s += partial[(long)c * n + i];
    d_w_r[i] = s;
  }
}

// dx[t, cols] += sum_e d_logits[t][e] * w_r[e][cols]; a wave owns one token's 512-column slab at a time.
template <typename T>
__global__ void __launch_bounds__(256) router_dx_kernel(const T* __restrict__ w_r, const float* __restrict__ d_logits,
                                                        int Tn, int d, int E, T* __restrict__ dx) {
  constexpr int V = 16 / sizeof(T);
  const int nvec = d / V;
  const long total = (long)Tn * nvec;
  for (long i = blockIdx.x * (long)blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
    const long t = i / nvec;
    const int c = (int)(i % nvec) * V;
    Vec16<T> cur = *reinterpret_cast<const Vec16<T>*>(dx + t * d + c);
    float acc[V];
#pragma unroll
    for (int j = 0; j < V; ++j) acc[j] = to_f32(cur.v[j]);
    const float* g = d_logits + t * E;
    for (int e = 0; e < E; ++e) {
      const float gv = g[e];
      const Vec16<T> w = *reinterpret_cast<const Vec16<T>*>(w_r + (long)e * d + c);
#pragma unroll
      for (int j = 0; j < V; ++j) acc[j] = fmaf(gv, to_f32(w.v[j]), acc[j]);
    }
#pragma unroll
    for (int j = 0; j < V; ++j) cur.v[j] = from_f32<T>(acc[j]);
    *reinterpret_cast<Vec16<T>*>(dx + t * d + c) = cur;
  }
}

int dwr_chunks(int T) {
  int chunks = cdiv(T, 128);
  if (chunks > 128) chunks = 128;
  return chunks < 1 ? 1 : chunks;
}

}  // namespace

size_t router_bwd_ws_bytes(int T, int d, int E) { return align_up((size_t)dwr_chunks(T) * E * d * sizeof(float), 256); }

int launch_router_bwd(const void* x, const void* w_r, const float* d_logits, moe_dtype dt, int T, int d, int E,
                      float* d_w_r, void* dx, void* ws, hipStream_t s) {
  if (d_w_r) {
    const int chunks = dwr_chunks(T);
    const int tpc = cdiv(T, chunks);
    const int slabs = cdiv(d, kSlabCols);
    float* partial = static_cast<float*>(ws);
    if (dt == MOE_F32)
      router_dwr_partial_kernel<float><<<slabs * chunks, 256, 0, s>>>((const float*)x, d_logits, T, d, E, tpc, partial);
    else
      router_dwr_partial_kernel<bf16><<<slabs * chunks, 256, 0, s>>>((const bf16*)x, d_logits, T, d, E, tpc, partial);
    MOE_LAUNCH_CHECK();
    const long n = (long)E * d;
    long blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    router_dwr_reduce_kernel<<<(int)blocks, 256, 0, s>>>(partial, chunks, n, d_w_r);
    MOE_LAUNCH_CHECK();
  }
  if (dx && T > 0) {
    const long total = (long)T * d / (dt == MOE_F32 ? 4 : 8);
    long blocks = (total + 255) / 256;
    if (blocks > 256 * 16) blocks = 256 * 16;
    if (dt == MOE_F32) router_dx_kernel<float><<<(int)blocks, 256, 0, s>>>((const float*)w_r, d_logits, T, d, E, (float*)dx);
    else router_dx_kernel<bf16><<<(int)blocks, 256, 0, s>>>((const bf16*)w_r, d_logits, T, d, E, (bf16*)dx);
    MOE_LAUNCH_CHECK();
  }
  return MOE_OK;
}

}  // namespace moe
