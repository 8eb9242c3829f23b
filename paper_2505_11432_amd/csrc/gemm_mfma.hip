// Launchers of the grouped MFMA GEMM (asynchronous global->LDS pipeline) for the bf16 expert FFN
// (Section 4.1: FC1 -> SwiGLU -> FC2 and the backward of each) and for the router matmul.
// Tile shapes, wave layouts and pipeline depths were picked by measurement on MI355X.
#include <atomic>
#include <vector>

#include "gemm_mfma_dma.h"

namespace moe {
namespace {

using namespace mfma;

constexpr int kMaxDevices = 64;

// One persistent workgroup per CU, in whole rounds of 8 (one per XCD).  The CU count of a device is looked up once;
// concurrent first calls may both look it up and store the same value.
int persistent_grid(int dev, int* grid) {
  static std::atomic<int> cached[kMaxDevices];
  int g = cached[dev].load(std::memory_order_acquire);
  if (g == 0) {
    int cus = 0;
    MOE_HIP_TRY(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    g = cus >= 8 ? cus / 8 * 8 : 8;
    cached[dev].store(g, std::memory_order_release);
  }
  *grid = g;
  return MOE_OK;
}

// Every kernel instantiation needs its dynamic-LDS limit raised once per device before its first launch.  Each
// instantiation registers its set-up function when the library is loaded, so that moe_init can run all of them
// ahead of time (a first call under graph capture must not be the one that sets the attribute).
typedef int (*configure_fn)(int dev);
std::vector<configure_fn>& configure_registry() {
  static std::vector<configure_fn> r;
  return r;
}

template <int BM, int BN, int BKT, int NS, int WM, int WN, Layout LA, Layout LB, Mode MODE, Epi EPI, typename TC, typename TIN>
struct KernelSetup {
  static constexpr int smem = dma_smem_bytes<BM, BN, BKT, NS, LA, LB, (int)sizeof(TIN)>();
  static auto kernel() { return grouped_gemm_dma_kernel<BM, BN, BKT, NS, WM, WN, LA, LB, MODE, EPI, TC, TIN>; }
  // Idempotent and safe to race: the attribute value is the same on every call, the per-device bit only saves work.
  static int configure(int dev) {
    static std::atomic<unsigned long long> done{0};
    const unsigned long long bit = 1ull << dev;
    if (done.load(std::memory_order_acquire) & bit) return MOE_OK;
    MOE_HIP_TRY(hipFuncSetAttribute((const void*)kernel(), hipFuncAttributeMaxDynamicSharedMemorySize, smem));
    done.fetch_or(bit, std::memory_order_release);
    return MOE_OK;
  }
  struct Registrar { Registrar() { configure_registry().push_back(&configure); } };
  static Registrar registrar;
};
template <int BM, int BN, int BKT, int NS, int WM, int WN, Layout LA, Layout LB, Mode MODE, Epi EPI, typename TC, typename TIN>
typename KernelSetup<BM, BN, BKT, NS, WM, WN, LA, LB, MODE, EPI, TC, TIN>::Registrar
    KernelSetup<BM, BN, BKT, NS, WM, WN, LA, LB, MODE, EPI, TC, TIN>::registrar;

template <int BM, int BN, int BKT, int NS, int WM, int WN, Layout LA, Layout LB, Mode MODE, Epi EPI, typename TC,
          typename TIN = bf16>
int launch(const Args& a, long tiles_upper_bound, hipStream_t s) {
  using Setup = KernelSetup<BM, BN, BKT, NS, WM, WN, LA, LB, MODE, EPI, TC, TIN>;
  (void)&Setup::registrar;           // instantiates the registration of this kernel
  if (tiles_upper_bound <= 0) return MOE_OK;
  {
    // the kernel addresses each operand as a 64-bit tile base plus a 32-bit per-lane byte offset
    const unsigned long long esz = sizeof(TIN), lim = 1ull << 32;
    const unsigned long long a_span = (EPI == EPI_SWIGLU_W) ? (unsigned long long)a.a_phys_rows * a.lda * esz   // absolute row offsets
                                      : (LA == KMAJOR)      ? (unsigned long long)BM * a.lda * esz
                                                            : ((unsigned long long)BKT * a.lda + a.M) * esz;
    const unsigned long long b_rows = (EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_W) ? 2ull * a.f : (unsigned long long)a.N;
    const unsigned long long b_span = (LB == KMAJOR) ? b_rows * a.ldb * esz : ((unsigned long long)BKT * a.ldb + a.N) * esz;
    if (a_span >= lim || b_span >= lim) return MOE_ERR_UNSUPPORTED;
  }
  int dev = 0;
  MOE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
  int blocks = 0;
  int rc = persistent_grid(dev, &blocks);
  if (rc != MOE_OK) return rc;
  rc = Setup::configure(dev);
  if (rc != MOE_OK) return rc;
  auto kern = Setup::kernel();
  constexpr int smem = Setup::smem;
  Args args = a;
  constexpr bool kSplitK = MODE == ROWSEG && EPI == EPI_STORE && sizeof(TC) == 2;
  if (!kSplitK || args.accumulate || blocks > MOE_SPLITK_MAX_PARTS) args.splitk_ws = nullptr;
  kern<<<dim3((unsigned)blocks), dim3(WM * WN * 64), smem, s>>>(args);
  MOE_LAUNCH_CHECK();
  if constexpr (kSplitK) {
    if (args.splitk_ws != nullptr) {
      // four workgroups per tile of the partly filled last round (fewer than `blocks` tiles); the others return at once
      splitk_fixup_kernel<BM, BN><<<dim3((unsigned)blocks * 4), dim3(256), 0, s>>>(args.splitk_ws, args.offsets, args.E, args.N, blocks,
                                                                              static_cast<bf16*>(args.C), args.ldc);
      MOE_LAUNCH_CHECK();
    }
  }
  return MOE_OK;
}

long rowseg_blocks(int M, int E, int N, int bm, int bn_out) {
  return (long)cdiv(N, bn_out) * (cdiv(M, bm) + E);
}

}  // namespace

// H[M,2f] = xp * w1[e]^T, A_out = SwiGLU(H)
int mfma_fc1_swiglu(const void* xp, const void* w1, const int32_t* offsets, int M, int d, int E, int f, void* H,
                    void* A_out, hipStream_t s) {
  Args a{};
  a.A = (const bf16*)xp; a.lda = d;
  a.B = (const bf16*)w1; a.ldb = d; a.b_es = 2L * f * d;
  a.offsets = offsets; a.E = E; a.M = M; a.N = f; a.K = d; a.f = f;
  a.H = (bf16*)H; a.A_out = (bf16*)A_out;
  return launch<256, 256, 64, 2, 4, 2, KMAJOR, KMAJOR, ROWSEG, EPI_SWIGLU, bf16>(a, rowseg_blocks(M, E, f, 256, 128), s);
}

// The same with the Section 4.1 / 4.2 operator order: row r of the A operand is row row_token[r] of x [T,d] (selected
// inside the kernel's loads, no dispatched copy), and A_out = row_w[r] * SwiGLU(H)
int mfma_fc1_swiglu_gather(const void* x, int T, const int32_t* row_token, const float* row_w, const void* w1,
                           const int32_t* offsets, int M, int d, int E, int f, void* H, void* A_out, hipStream_t s) {
  Args a{};
  a.A = (const bf16*)x; a.lda = d; a.a_rowmap = row_token; a.a_phys_rows = T; a.row_w = row_w;
  a.B = (const bf16*)w1; a.ldb = d; a.b_es = 2L * f * d;
  a.offsets = offsets; a.E = E; a.M = M; a.N = f; a.K = d; a.f = f;
  a.H = (bf16*)H; a.A_out = (bf16*)A_out;
  return launch<256, 256, 64, 2, 4, 2, KMAJOR, KMAJOR, ROWSEG, EPI_SWIGLU_W, bf16>(a, rowseg_blocks(M, E, f, 256, 128), s);
}

// C[M,N] = A[M,K] * W[e]^T with W[e] = [N,K]
int mfma_rowseg_nt(const void* A, const void* W, long w_es, const int32_t* offsets, int M, int N, int K, int E,
                   void* C, void* splitk_ws, hipStream_t s) {
  Args a{};
  a.splitk_ws = static_cast<float*>(splitk_ws);
  a.A = (const bf16*)A; a.lda = K;
  a.B = (const bf16*)W; a.ldb = K; a.b_es = w_es;
  a.C = C; a.ldc = N; a.offsets = offsets; a.E = E; a.M = M; a.N = N; a.K = K;
  return launch<256, 256, 64, 2, 4, 2, KMAJOR, KMAJOR, ROWSEG, EPI_STORE, bf16>(a, rowseg_blocks(M, E, N, 256, 256), s);
}

// C[M,N] = A[M,K] * W[e] with W[e] = [K,N]
int mfma_rowseg_nn(const void* A, const void* W, long w_es, const int32_t* offsets, int M, int N, int K, int E,
                   void* C, void* splitk_ws, hipStream_t s) {
  Args a{};
  a.splitk_ws = static_cast<float*>(splitk_ws);
  a.A = (const bf16*)A; a.lda = K;
  a.B = (const bf16*)W; a.ldb = N; a.b_es = w_es;
  a.C = C; a.ldc = N; a.offsets = offsets; a.E = E; a.M = M; a.N = N; a.K = K;
  return launch<256, 256, 64, 2, 2, 4, KMAJOR, MNMAJOR, ROWSEG, EPI_STORE, bf16>(a, rowseg_blocks(M, E, N, 256, 256), s);
}

// dA = d_yp * w2[e] fused with the SwiGLU derivative: reads H=[G|U], writes dH=[dG|dU] and (optionally) A
int mfma_dgrad2_swiglu_bwd(const void* d_yp, const void* w2, const int32_t* offsets, int M, int d, int E, int f,
                           const void* H, void* dH, void* A_out, hipStream_t s) {
  Args a{};
  a.A = (const bf16*)d_yp; a.lda = d;
  a.B = (const bf16*)w2; a.ldb = f; a.b_es = (long)d * f;
  a.offsets = offsets; a.E = E; a.M = M; a.N = f; a.K = d;
  a.H = (bf16*)const_cast<void*>(H); a.dH = (bf16*)dH; a.A_out = (bf16*)A_out;
  return launch<256, 256, 64, 2, 2, 4, KMAJOR, MNMAJOR, ROWSEG, EPI_SWIGLU_BWD, bf16>(a, rowseg_blocks(M, E, f, 256, 256), s);
}

// dgrad2 in the Section 4.1 order: d_yp holds the unweighted output gradient of each row; dH gets SwiGLU'(dA') (the
// row's weight is applied downstream), A_out = w_r * A, and dw_part [mfma_dgrad2_fold_parts(f)][M] the partial sums of <dA'[r,:], A[r,:]>
int mfma_dgrad2_fold_parts(int f) { return cdiv(f, 256) * 4; }
int mfma_dgrad2_swiglu_bwd_fold(const void* d_yp, const void* w2, const int32_t* offsets, int M, int d, int E, int f,
                                const void* H, void* dH, void* A_out, const float* row_w, float* dw_part, hipStream_t s) {
  Args a{};
  a.A = (const bf16*)d_yp; a.lda = d;
  a.B = (const bf16*)w2; a.ldb = f; a.b_es = (long)d * f;
  a.offsets = offsets; a.E = E; a.M = M; a.N = f; a.K = d;
  a.H = (bf16*)const_cast<void*>(H); a.dH = (bf16*)dH; a.A_out = (bf16*)A_out;
  a.row_w = row_w; a.dw_part = dw_part;
  return launch<256, 256, 64, 2, 2, 4, KMAJOR, MNMAJOR, ROWSEG, EPI_SWIGLU_BWD_W, bf16>(a, rowseg_blocks(M, E, f, 256, 256), s);
}

// C[e][Mo,N] (+)= P[rows_e, Mo]^T * Q[rows_e, N]
int mfma_wgrad(const void* P, const void* Q, const int32_t* offsets, int Mo, int N, int E, void* C, moe_dtype c_dt,
               int accumulate, hipStream_t s) {
  Args a{};
  a.A = (const bf16*)P; a.lda = Mo;
  a.B = (const bf16*)Q; a.ldb = N; a.b_es = 0;
  a.C = C; a.ldc = N; a.c_es = (long)Mo * N; a.offsets = offsets; a.E = E; a.M = Mo; a.N = N; a.K = 0;
  a.accumulate = accumulate;
  const long blocks = (long)E * cdiv(Mo, 256) * cdiv(N, 256);
  if (c_dt == MOE_F32) return launch<256, 256, 64, 2, 2, 4, MNMAJOR, MNMAJOR, KSEG, EPI_STORE, float>(a, blocks, s);
  return launch<256, 256, 64, 2, 2, 4, MNMAJOR, MNMAJOR, KSEG, EPI_STORE, bf16>(a, blocks, s);
}

// e4m3 operands (codes with per-row / per-output-channel scales), 32x32x64 f8f6f4 MFMA, bf16 results:
// H[M,2f] = (xp*sx) * (w1[e]*sw1)^T, A_out = SwiGLU(H)
int mfma_fc1_swiglu_fp8(const void* xp, const float* xp_scale, const void* w1, const float* w1_scale,
                        const int32_t* offsets, int M, int d, int E, int f, void* H, void* A_out, hipStream_t s) {
  Args a{};
  a.A = xp; a.lda = d;
  a.B = w1; a.ldb = d; a.b_es = 2L * f * d;
  a.offsets = offsets; a.E = E; a.M = M; a.N = f; a.K = d; a.f = f;
  a.H = (bf16*)H; a.A_out = (bf16*)A_out;
  a.row_scale = xp_scale; a.col_scale = w1_scale; a.cs_es = 2L * f;
  return launch<256, 256, 128, 2, 4, 2, KMAJOR, KMAJOR, ROWSEG, EPI_SWIGLU, bf16, uint8_t>(a, rowseg_blocks(M, E, f, 256, 128), s);
}

// C[M,N] = (A*sa) * (W[e]*sw)^T, bf16 out
int mfma_rowseg_nt_fp8(const void* A, const float* a_scale, const void* W, const float* w_scale, long w_es,
                       const int32_t* offsets, int M, int N, int K, int E, void* C, void* splitk_ws, hipStream_t s) {
  Args a{};
  a.splitk_ws = static_cast<float*>(splitk_ws);
  a.A = A; a.lda = K;
  a.B = W; a.ldb = K; a.b_es = w_es;
  a.C = C; a.ldc = N; a.offsets = offsets; a.E = E; a.M = M; a.N = N; a.K = K;
  a.row_scale = a_scale; a.col_scale = w_scale; a.cs_es = N;
  return launch<256, 256, 128, 2, 4, 2, KMAJOR, KMAJOR, ROWSEG, EPI_STORE, bf16, uint8_t>(a, rowseg_blocks(M, E, N, 256, 256), s);
}


// e4m3 dgrad2 fused with the SwiGLU derivative: dA = (d_yp*s_row) * (w2t[e]*s_ch)^T with w2t[e] = W2[e]^T stored
// [f, d] (second, transposed-orientation quantisation of the weights); reads H, writes dH (and A when asked)
int mfma_dgrad2_swiglu_bwd_fp8(const void* dyq, const float* dyq_scale, const void* w2t, const float* w2t_scale,
                               const int32_t* offsets, int M, int d, int E, int f, const void* H, void* dH, void* A_out,
                               hipStream_t s) {
  Args a{};
  a.A = dyq; a.lda = d;
  a.B = w2t; a.ldb = d; a.b_es = (long)f * d;
  a.offsets = offsets; a.E = E; a.M = M; a.N = f; a.K = d;
  a.H = (bf16*)const_cast<void*>(H); a.dH = (bf16*)dH; a.A_out = (bf16*)A_out;
  a.row_scale = dyq_scale; a.col_scale = w2t_scale; a.cs_es = f;
  return launch<256, 256, 128, 2, 4, 2, KMAJOR, KMAJOR, ROWSEG, EPI_SWIGLU_BWD, bf16, uint8_t>(a, rowseg_blocks(M, E, f, 256, 256), s);
}

// e4m3 weight gradient: C[e][Mo,N] (+)= P_t[Mo, tokens_e] * Q_t[N, tokens_e]^T on transposed (token-minor) codes
// whose expert segments are padded to whole 128-token groups (pad_offsets), with one power-of-two scale per
// (group, channel) applied by the block-scaled MFMA
int mfma_wgrad_fp8(const void* Pt, const uint8_t* p_e8m0, const void* Qt, const uint8_t* q_e8m0, long ldt,
                   const int32_t* pad_offsets, int Mo, int N, int E, void* C, moe_dtype c_dt, int accumulate,
                   hipStream_t s) {
  Args a{};
  a.A = Pt; a.lda = ldt;
  a.B = Qt; a.ldb = ldt; a.b_es = 0;
  a.C = C; a.ldc = N; a.c_es = (long)Mo * N; a.offsets = pad_offsets; a.E = E; a.M = Mo; a.N = N; a.K = 0;
  a.accumulate = accumulate;
  a.a_e8m0 = p_e8m0; a.a_e8_ld = Mo; a.b_e8m0 = q_e8m0; a.b_e8_ld = N;
  const long blocks = (long)E * cdiv(Mo, 256) * cdiv(N, 256);
  if (c_dt == MOE_F32) return launch<256, 256, 128, 2, 4, 2, KMAJOR, KMAJOR, KSEG, EPI_STORE, float, uint8_t>(a, blocks, s);
  return launch<256, 256, 128, 2, 4, 2, KMAJOR, KMAJOR, KSEG, EPI_STORE, bf16, uint8_t>(a, blocks, s);
}

// Router weight gradient as a weight-gradient GEMM over token chunks: partial[c][E, d] (+)= g_c^T * x_c
int mfma_router_dwr(const void* g, const void* x, const int32_t* chunk_offsets, int chunks, int E, int d, float* partial,
                    int accumulate, hipStream_t s) {
  Args a{};
  a.A = (const bf16*)g; a.lda = E;
  a.B = (const bf16*)x; a.ldb = d; a.b_es = 0;
  a.C = partial; a.ldc = d; a.c_es = (long)E * d; a.offsets = chunk_offsets; a.E = chunks; a.M = E; a.N = d; a.K = 0;
  a.accumulate = accumulate;
  const long blocks = (long)chunks * cdiv(E, 128) * cdiv(d, 256);
  return launch<128, 256, 32, 4, 2, 4, MNMAJOR, MNMAJOR, KSEG, EPI_STORE, float>(a, blocks, s);
}

// dx[T,d] += g[T,E] * w_r[E,d]: one dense GEMM with a very short contraction (K = E), bound by reading and writing dx
int mfma_router_dx(const void* g, const void* w_r, int T, int d, int E, void* dx, hipStream_t s) {
  Args a{};
  a.A = (const bf16*)g; a.lda = E;
  a.B = (const bf16*)w_r; a.ldb = d; a.b_es = 0;
  a.C = dx; a.ldc = d; a.E = 1; a.M = T; a.N = d; a.K = E;
  a.accumulate = 1;
  return launch<256, 256, 64, 2, 2, 4, KMAJOR, MNMAJOR, PLAIN, EPI_STORE, bf16>(a, (long)cdiv(T, 256) * cdiv(d, 256), s);
}

// logits[T,E] = x[T,d] * w_r[E,d]^T (+ bias), fp32 out
int mfma_router_fwd(const void* x, const void* w_r, const float* bias, int T, int d, int E, float* logits,
                    hipStream_t s) {
  Args a{};
  a.A = (const bf16*)x; a.lda = d;
  a.B = (const bf16*)w_r; a.ldb = d; a.b_es = 0;
  a.C = logits; a.ldc = E; a.E = 1; a.M = T; a.N = E; a.K = d; a.bias = bias;
  const long mt = cdiv(T, 256);
  // Few experts: the GEMM is a stream over x with almost no arithmetic, so what matters is how many workgroups pull
  // on memory and how deep each one's pipeline is: 64-row tiles (four times the workgroups) with an 8-stage ring
  // halve the time of 256-row tiles with two stages (cfg 2: 59 -> 30 us).
  if (E <= 32) return launch<64, 32, 64, 8, 2, 1, KMAJOR, KMAJOR, PLAIN, EPI_BIAS_F32, float>(a, cdiv(T, 64), s);
  if (E <= 64) return launch<64, 64, 64, 8, 2, 1, KMAJOR, KMAJOR, PLAIN, EPI_BIAS_F32, float>(a, cdiv(T, 64), s);
  return launch<256, 128, 64, 2, 4, 2, KMAJOR, KMAJOR, PLAIN, EPI_BIAS_F32, float>(a, mt * cdiv(E, 128), s);
}

// Sets up every grouped-GEMM kernel of this library for the current device (see moe_init).
int mfma_configure_all() {
  int dev = 0;
  MOE_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return MOE_ERR_UNSUPPORTED;
  int grid = 0;
  int rc = persistent_grid(dev, &grid);
  for (configure_fn fn : configure_registry()) {
    if (rc != MOE_OK) break;
    rc = fn(dev);
  }
  return rc;
}

}  // namespace moe
