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

// COLS consecutive elements of a row as fp32 (COLS * sizeof(T) bytes in one load)
template <typename T, int COLS> struct RowChunk {
  __device__ static void load(const T* p, float (&out)[COLS]) {
    struct alignas(COLS * sizeof(T)) Raw { T v[COLS]; };
    const Raw r = *reinterpret_cast<const Raw*>(p);
#pragma unroll
    for (int i = 0; i < COLS; ++i) out[i] = to_f32(r.v[i]);
  }
};

// partial[chunk][e][col] = sum over the chunk's tokens of d_logits[t][e] * x[t][col].
// A block owns 256 * COLS columns of x and one chunk of tokens; a thread keeps ETILE x COLS fp32 sums.  The
// chunk's gate gradients (up to 64 tokens x ETILE experts) are staged in LDS and read back as broadcasts.
// ETILE is the smallest of 8 / 16 / 32 / 64 that holds E (more than 64 experts: passes of 64), so that few
// experts do not pay for 64: with ETILE = 8 the kernel is bound by reading x, not by FMAs.
constexpr int kChunkTokens = 64;
constexpr int kTokUnroll = 8;         // rows of x in flight per thread

template <typename T, int ETILE, int COLS>
__global__ void __launch_bounds__(256) router_dwr_partial_kernel(const T* __restrict__ x,
                                                                 const float* __restrict__ d_logits, int Tn, int d,
                                                                 int E, int tokens_per_chunk,
                                                                 float* __restrict__ partial) {
  __shared__ __attribute__((aligned(16))) float g_lds[kChunkTokens][ETILE];
  constexpr int kSlab = 256 * COLS;
  const int slabs = (d + kSlab - 1) / kSlab;
  const int slab = blockIdx.x % slabs, chunk = blockIdx.x / slabs;
  const int col = slab * kSlab + threadIdx.x * COLS;
  const int t0 = chunk * tokens_per_chunk, t1 = min(t0 + tokens_per_chunk, Tn);
  const bool active = col < d;                 // d is a multiple of 16 >= COLS: a chunk is inside the row or outside
  for (int e0 = 0; e0 < E; e0 += ETILE) {
    float acc[ETILE][COLS];
#pragma unroll
    for (int i = 0; i < ETILE; ++i)
#pragma unroll
      for (int c = 0; c < COLS; ++c) acc[i][c] = 0.f;
    for (int ts = t0; ts < t1; ts += kChunkTokens) {
      const int te = min(ts + kChunkTokens, t1);
      __syncthreads();
      for (int i = threadIdx.x; i < kChunkTokens * ETILE; i += 256) {
        const int tt = i / ETILE, ee = i % ETILE;
        g_lds[tt][ee] = (ts + tt < te && e0 + ee < E) ? d_logits[(long)(ts + tt) * E + e0 + ee] : 0.f;   // zero rows past the chunk
      }
      __syncthreads();
      if (!active) continue;
      for (int tb = ts; tb < te; tb += kTokUnroll) {
        float xv[kTokUnroll][COLS];
#pragma unroll
        for (int u = 0; u < kTokUnroll; ++u) RowChunk<T, COLS>::load(x + (long)min(tb + u, Tn - 1) * d + col, xv[u]);
#pragma unroll
        for (int u = 0; u < kTokUnroll; ++u) {
          // rows past the chunk's end multiply zeros (tb + u - ts < kChunkTokens: both are multiples of 8 apart)
          const float4* g = reinterpret_cast<const float4*>(g_lds[tb + u - ts]);
#pragma unroll
          for (int i = 0; i < ETILE / 4; ++i) {
            const float4 gv = g[i];
#pragma unroll
            for (int c = 0; c < COLS; ++c) {
              acc[4 * i + 0][c] = fmaf(gv.x, xv[u][c], acc[4 * i + 0][c]);
              acc[4 * i + 1][c] = fmaf(gv.y, xv[u][c], acc[4 * i + 1][c]);
              acc[4 * i + 2][c] = fmaf(gv.z, xv[u][c], acc[4 * i + 2][c]);
              acc[4 * i + 3][c] = fmaf(gv.w, xv[u][c], acc[4 * i + 3][c]);
            }
          }
        }
      }
    }
    if (active) {
#pragma unroll
      for (int i = 0; i < ETILE; ++i)
        if (e0 + i < E) {
          float* dst = partial + ((long)chunk * E + e0 + i) * d + col;
#pragma unroll
          for (int c = 0; c < COLS; ++c) dst[c] = acc[i][c];
        }
    }
  }
}

// d_w_r[i] = sum over the chunks of partial[c][i] in a fixed order: a block owns 64 outputs, its four waves each add
// every fourth chunk (ascending), then the four sums are added in wave order.
__global__ void __launch_bounds__(256) router_dwr_reduce_kernel(const float* __restrict__ partial, int chunks,
                                                                long n /* = E*d */, float* __restrict__ d_w_r) {
  __shared__ float part[4][64];
  const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
  const long i = (long)blockIdx.x * 64 + lane;
  float s = 0.f;
  if (i < n) {
    int c = q;
    for (; c + 12 < chunks; c += 16) {
      const float v0 = partial[(long)c * n + i], v1 = partial[(long)(c + 4) * n + i];
      const float v2 = partial[(long)(c + 8) * n + i], v3 = partial[(long)(c + 12) * n + i];
      s = ((s + v0) + v1) + v2;
      s += v3;
    }
    for (; c < chunks; c += 4) s += partial[(long)c * n + i];
  }
  part[q][lane] = s;
  __syncthreads();
  if (q == 0 && i < n) d_w_r[i] = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
}

// dx[t, cols] += sum_e d_logits[t][e] * w_r[e][cols].  A block owns a slab of 512 columns (64 lanes x 8) and
// keeps that slab of w_r (up to 64 experts x 1 KiB) in LDS; its four waves walk the tokens.  More than 64
// experts are done in passes of 64 that each read-modify-write dx.
constexpr int kDxCols = 512;

template <typename T>
__global__ void __launch_bounds__(256) router_dx_kernel(const T* __restrict__ w_r, const float* __restrict__ d_logits,
                                                        int Tn, int d, int E, int token_groups, T* __restrict__ dx) {
  constexpr int V = 8;                                  // columns per lane
  __shared__ __attribute__((aligned(16))) T w_lds[kETile][kDxCols];
  const int slabs = (d + kDxCols - 1) / kDxCols;
  const int slab = blockIdx.x % slabs, tg = blockIdx.x / slabs;
  const int lane = threadIdx.x % 64, wave = threadIdx.x / 64;
  const int col = slab * kDxCols + lane * V;
  const bool active = col < d;
  for (int e0 = 0; e0 < E; e0 += kETile) {
    const int ne = min(kETile, E - e0);
    __syncthreads();
    for (int i = threadIdx.x; i < ne * (kDxCols / V); i += 256) {
      const int ee = i / (kDxCols / V), cc = (i % (kDxCols / V)) * V;
      Vec16<T> v;      // V elements of T fill 16 bytes for bf16; fp32 uses two 16-byte halves below
      if constexpr (sizeof(T) == 2) {
        if (slab * kDxCols + cc < d) v = *reinterpret_cast<const Vec16<T>*>(w_r + (long)(e0 + ee) * d + slab * kDxCols + cc);
        else for (int j = 0; j < V; ++j) v.v[j] = from_f32<T>(0.f);
        *reinterpret_cast<Vec16<T>*>(&w_lds[ee][cc]) = v;
      } else {
        for (int j = 0; j < V; ++j)
          w_lds[ee][cc + j] = (slab * kDxCols + cc + j < d) ? w_r[(long)(e0 + ee) * d + slab * kDxCols + cc + j] : from_f32<T>(0.f);
      }
    }
    __syncthreads();
    // a wave takes kTok tokens at a time: one LDS read of w_r feeds kTok x 8 FMAs
    constexpr int kTok = 4;
    for (int tb = (tg * 4 + wave) * kTok; tb < Tn; tb += token_groups * 4 * kTok) {
      if (!active) continue;
      float acc[kTok][V];
#pragma unroll
      for (int q = 0; q < kTok; ++q) {
        const int t = min(tb + q, Tn - 1);
        const T* src = dx + (long)t * d + col;
        if constexpr (sizeof(T) == 2) {
          const Vec16<T> cur = *reinterpret_cast<const Vec16<T>*>(src);
#pragma unroll
          for (int j = 0; j < V; ++j) acc[q][j] = to_f32(cur.v[j]);
        } else {
#pragma unroll
          for (int j = 0; j < V; ++j) acc[q][j] = to_f32(src[j]);
        }
      }
      for (int e = 0; e < ne; ++e) {
        float wv[V];
        if constexpr (sizeof(T) == 2) {
          const Vec16<T> w = *reinterpret_cast<const Vec16<T>*>(&w_lds[e][lane * V]);     // one ds_read_b128
#pragma unroll
          for (int j = 0; j < V; ++j) wv[j] = to_f32(w.v[j]);
        } else {
#pragma unroll
          for (int j = 0; j < V; ++j) wv[j] = to_f32(w_lds[e][lane * V + j]);
        }
#pragma unroll
        for (int q = 0; q < kTok; ++q) {
          const float gv = d_logits[(long)min(tb + q, Tn - 1) * E + e0 + e];     // wave-uniform: scalar load
#pragma unroll
          for (int j = 0; j < V; ++j) acc[q][j] = fmaf(gv, wv[j], acc[q][j]);
        }
      }
#pragma unroll
      for (int q = 0; q < kTok; ++q) {
        if (tb + q >= Tn) break;
        T* dst = dx + (long)(tb + q) * d + col;
        if constexpr (sizeof(T) == 2) {
          Vec16<T> out;
#pragma unroll
          for (int j = 0; j < V; ++j) out.v[j] = from_f32<T>(acc[q][j]);
          *reinterpret_cast<Vec16<T>*>(dst) = out;
        } else {
#pragma unroll
          for (int j = 0; j < V; ++j) dst[j] = from_f32<T>(acc[q][j]);
        }
      }
    }
  }
}

// ---- d_w_r on the matrix cores (many experts) -----------------------------------------------------------------
// d_w_r = d_logits^T x is a weight-gradient GEMM with the tokens as contraction index: E output rows, d columns.
// With 32 experts or more the vector-ALU kernel above is bound by its FMAs, so the grouped weight-gradient kernel is
// used instead, with token chunks in the role of the experts (one fp32 partial [E, d] per chunk, then the same
// fixed-order reduction).  The fp32 gate gradient enters as two bf16 matrices, hi = bf16(v) and lo = bf16(v - hi)
// (relative error of hi + lo: 2^-17), multiplied in two accumulating launches.
constexpr int kMfmaChunkTokens = 512;

int dwr_mfma_chunk_tokens(int T) {
  int tpc = kMfmaChunkTokens;
  while (cdiv(T, tpc) > MOE_MAX_EXPERTS) tpc *= 2;
  return tpc;
}
bool dwr_use_mfma(moe_dtype dt, int T, int d, int E) { return dt == MOE_BF16 && E >= 32 && E % 8 == 0 && d % 8 == 0 && T > 0; }

__global__ void __launch_bounds__(256) dlogits_split_kernel(const float* __restrict__ d_logits, long n, bf16* __restrict__ hi,
                                                            bf16* __restrict__ lo, int T, int tokens_per_chunk, int chunks,
                                                            int32_t* __restrict__ chunk_offsets) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i <= chunks) chunk_offsets[i] = (int32_t)min((long)T, i * tokens_per_chunk);
  if (i >= n) return;
  const float v = d_logits[i];
  const bf16 h = static_cast<bf16>(v);
  hi[i] = h;
  lo[i] = static_cast<bf16>(v - static_cast<float>(h));
}

int dwr_tokens_per_chunk(int T) {                // a multiple of the LDS staging size; at most 256 chunks
  int tpc = kChunkTokens;
  while (cdiv(T, tpc) > 256) tpc *= 2;
  return tpc;
}
int dwr_chunks(int T) {
  const int chunks = cdiv(T, dwr_tokens_per_chunk(T));
  return chunks < 1 ? 1 : chunks;
}

}  // namespace

static size_t dwr_mfma_ws_bytes(int T, int d, int E) {
  const size_t chunks = cdiv(T, dwr_mfma_chunk_tokens(T));
  return align_up(chunks * E * d * sizeof(float), 256) + 2 * align_up((size_t)T * E * 2, 256) + align_up((chunks + 1) * 4, 256);
}
size_t router_bwd_ws_bytes(int T, int d, int E) {
  const size_t valu = align_up((size_t)dwr_chunks(T) * E * d * sizeof(float), 256);
  const size_t mfma = T > 0 && E >= 32 && E % 8 == 0 ? dwr_mfma_ws_bytes(T, d, E) : 0;      // (any dtype: an upper bound)
  return valu > mfma ? valu : mfma;
}

int launch_router_bwd(const void* x, const void* w_r, const float* d_logits, moe_dtype dt, int T, int d, int E,
                      float* d_w_r, void* dx, void* ws, hipStream_t s) {
  const bool mfma_path = ws && dwr_use_mfma(dt, T, d, E) && (d_w_r || dx);     // dx alone may come without a workspace
  bf16* hi = nullptr;
  if (mfma_path) {
    const int tpc = dwr_mfma_chunk_tokens(T), chunks = cdiv(T, tpc);
    char* base = static_cast<char*>(ws);
    float* partial = reinterpret_cast<float*>(base);
    hi = reinterpret_cast<bf16*>(base + align_up((size_t)chunks * E * d * sizeof(float), 256));
    bf16* lo = reinterpret_cast<bf16*>(reinterpret_cast<char*>(hi) + align_up((size_t)T * E * 2, 256));
    int32_t* chunk_offsets = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(lo) + align_up((size_t)T * E * 2, 256));
    const long n = (long)T * E;
    dlogits_split_kernel<<<(int)((n + 255) / 256), 256, 0, s>>>(d_logits, n, hi, lo, T, tpc, chunks, chunk_offsets);
    MOE_LAUNCH_CHECK();
    if (d_w_r) {
      int rc = mfma_router_dwr(hi, x, chunk_offsets, chunks, E, d, partial, 0, s);
      if (rc != MOE_OK) return rc;
      rc = mfma_router_dwr(lo, x, chunk_offsets, chunks, E, d, partial, 1, s);
      if (rc != MOE_OK) return rc;
      const long nout = (long)E * d;
      router_dwr_reduce_kernel<<<(int)((nout + 63) / 64), 256, 0, s>>>(partial, chunks, nout, d_w_r);
      MOE_LAUNCH_CHECK();
    }
  } else if (d_w_r) {
    const int chunks = dwr_chunks(T);
    const int tpc = dwr_tokens_per_chunk(T);
    float* partial = static_cast<float*>(ws);
#define MOE_DWR_CASE(TT, ET, CO)                                                                                    \
  router_dwr_partial_kernel<TT, ET, CO><<<cdiv(d, 256 * CO) * chunks, 256, 0, s>>>((const TT*)x, d_logits, T, d, E, tpc, partial)
    if (dt == MOE_F32) {
      if (E <= 8) MOE_DWR_CASE(float, 8, 4);
      else if (E <= 16) MOE_DWR_CASE(float, 16, 4);
      else if (E <= 32) MOE_DWR_CASE(float, 32, 2);
      else MOE_DWR_CASE(float, 64, 2);
    } else {
      if (E <= 8) MOE_DWR_CASE(bf16, 8, 4);
      else if (E <= 16) MOE_DWR_CASE(bf16, 16, 4);
      else if (E <= 32) MOE_DWR_CASE(bf16, 32, 2);
      else MOE_DWR_CASE(bf16, 64, 2);
    }
#undef MOE_DWR_CASE
    MOE_LAUNCH_CHECK();
    const long n = (long)E * d;
    const long blocks = (n + 63) / 64;
    router_dwr_reduce_kernel<<<(int)blocks, 256, 0, s>>>(partial, chunks, n, d_w_r);
    MOE_LAUNCH_CHECK();
  }
  if (dx && mfma_path) {
    // dx is bf16: the hi part of the gate gradient alone is below its rounding (lo is 2^-9 of hi)
    const int rc = mfma_router_dx(hi, w_r, T, d, E, dx, s);
    if (rc != MOE_OK) return rc;
  } else if (dx && T > 0) {
    const int slabs = cdiv(d, kDxCols);
    int token_groups = cdiv(512, slabs);                 // about two blocks per CU
    if (token_groups > cdiv(T, 16)) token_groups = cdiv(T, 16);
    const int blocks = slabs * token_groups;
    if (dt == MOE_F32) router_dx_kernel<float><<<blocks, 256, 0, s>>>((const float*)w_r, d_logits, T, d, E, token_groups, (float*)dx);
    else router_dx_kernel<bf16><<<blocks, 256, 0, s>>>((const bf16*)w_r, d_logits, T, d, E, token_groups, (bf16*)dx);
    MOE_LAUNCH_CHECK();
  }
  return MOE_OK;
}

}  // namespace moe
