// Shared host/device helpers of the gfx950 MoE kernels (internal; the public ABI is include/moe.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/moe.h"

namespace moe {

typedef __bf16 bf16;

// ---- host side -----------------------------------------------------------------------------
int record_hip_error(hipError_t e);          // remembers e for moe_last_hip_error, returns MOE_ERR_HIP

#define MOE_HIP_TRY(expr)                                   \
  do {                                                      \
    hipError_t _e = (expr);                                 \
    if (_e != hipSuccess) return ::moe::record_hip_error(_e); \
  } while (0)

// Call after every kernel launch: launch failures surface here, not at the next sync.
#define MOE_LAUNCH_CHECK() MOE_HIP_TRY(hipGetLastError())

static inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int cdiv(int a, int b) { return (a + b - 1) / b; }
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t dtype_size(moe_dtype t) { return t == MOE_F32 ? 4 : (t == MOE_BF16 ? 2 : 1); }

// Number of token chunks the routing kernels split T into (one histogram row per chunk).
static inline int route_chunk_tokens(int T) {
  int tb = 64;
  while ((T + tb - 1) / tb > 1024) tb *= 2;
  return tb;
}

// Workspace layouts, shared by moe_workspace_bytes and the calls that carve the buffer up.
size_t route_ws_bytes(int T, int E);
size_t ffn_fwd_ws_bytes(int M, int d, int f, moe_dtype act, moe_dtype out);
size_t ffn_bwd_ws_bytes(int M, int d, int f, moe_dtype dt);

// ---- device side ---------------------------------------------------------------------------
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return static_cast<float>(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return static_cast<bf16>(v); }

// 1 / (1 + 2^(-g * log2 e)) on the hardware exp2 and reciprocal (about 1 ulp each): an IEEE division costs ten
// more vector instructions per element, which the fused SwiGLU epilogues would pay 16 times per lane and tile.
// Saturates correctly: exp2 -> inf gives 0, exp2 -> 0 gives 1.
__device__ __forceinline__ float sigmoid_f32(float g) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(g * -1.44269504088896341f));
}

// Vector of 16 bytes of T for coalesced row traffic.
template <typename T> struct Vec16 { static constexpr int N = 16 / sizeof(T); T v[16 / sizeof(T)]; };

// ---- kernel launchers (one per translation unit) -------------------------------------------
// Generic strided grouped GEMM on the vector ALU (fp32 FMA); covers fp32 data and odd shapes.
struct GemmProblem {
  const void* A; long a_rs, a_cs;            // A(m,k) = A[m*a_rs + k*a_cs]
  const void* B; long b_es, b_rs, b_cs;      // B(e,k,n) = B[e*b_es + k*b_rs + n*b_cs]
  void* C; long c_es, ldc;                   // C(e,m,n) = C[e*c_es + m*ldc + n]
  const int32_t* offsets; int E;             // expert segments (device)
  int mode;                                  // 0: rows of A/C are segmented; 1: the contraction index is; 2: one plain GEMM
  int M, N, K;                               // mode 0: M = upper bound on rows; mode 1: K = upper bound
  int accumulate;                            // C += instead of C =
  const float* bias;                         // per-column fp32 bias added in the epilogue, or NULL
};
int launch_gemm_generic(const GemmProblem& p, moe_dtype a_dt, moe_dtype b_dt, moe_dtype c_dt, hipStream_t s);

int launch_route(const float* logits, int T, int E, int k, int renorm, int e_lo, int e_hi, int n_groups, int capacity,
                 int32_t* idx, float* w, float* score, int32_t* counts, int32_t* offsets, int32_t* perm,
                 int32_t* inv_perm, void* ws, hipStream_t s);
size_t route_capacity_ws_bytes(int T, int E, int k);
size_t balance_ws_bytes(int T, int E);
int launch_balance_loss(const float* logits, const int32_t* counts, int T, int E, int k, int n_groups, float alpha,
                        float* loss, float* group_f, float* group_p, void* ws, hipStream_t s);
int launch_balance_loss_bwd(const float* logits, const float* group_f, int T, int E, int n_groups, float alpha,
                            float* d_logits, hipStream_t s);
int launch_route_bwd(const float* logits, const int32_t* idx, const float* w, const float* dw, int T, int E, int k,
                     int renorm, float* d_logits, hipStream_t s);
int launch_dispatch(const void* x, const float* x_scale, moe_dtype dt, const int32_t* inv_perm, const float* row_mul,
                    int T, int k, int d, void* xp, float* xp_scale, hipStream_t s);
int launch_combine(const void* yp, const float* yp_scale, moe_dtype dt, const int32_t* inv_perm, const float* topk_w,
                   int T, int k, int d, void* y, moe_dtype y_dt, hipStream_t s);
int launch_gate_grad(const void* dy, moe_dtype dy_dt, const void* yp, const float* yp_scale, moe_dtype dt,
                     const int32_t* inv_perm, int T, int k, int d, float* d_topk_w, hipStream_t s);
int launch_row_map(const int32_t* perm, const float* topk_w, const int32_t* offsets, int E, int rows, int k,
                   int32_t* row_token, float* row_w, hipStream_t s);
int launch_gate_grad_reduce(const float* part, int parts, long ld, const int32_t* inv_perm, int n, float* d_topk_w,
                            hipStream_t s);
int launch_quant_fp8(const void* src, moe_dtype src_dt, int rows, int cols, moe_qmode mode, uint8_t* codes,
                     float* scales, hipStream_t s);
int launch_dequant_fp8(const uint8_t* codes, const float* scales, int rows, int cols, moe_qmode mode, void* dst,
                       moe_dtype dst_dt, hipStream_t s);
int launch_tgroup_offsets(const int32_t* offsets, int E, int32_t* pad_offsets, hipStream_t s);
// src_dt = MOE_F8E4M3: src holds e4m3 codes with one scale per row (src_row_scale [rows]); NULL otherwise
int launch_quant_tgroup(const void* src, const float* src_row_scale, moe_dtype src_dt, int rows, int cols, const int32_t* offsets,
                        const int32_t* pad_offsets, int E, uint8_t* codes_t, long ldt, uint8_t* e8m0, hipStream_t s);

// bf16 grouped GEMMs on the matrix cores (gemm_mfma.hip)
int mfma_fc1_swiglu(const void* xp, const void* w1, const int32_t* offsets, int M, int d, int E, int f, void* H,
                    void* A_out, hipStream_t s);
// splitk_ws: MOE_SPLITK_WS_BYTES of scratch for the partial tiles of a split last round, or NULL (no splitting)
constexpr int MOE_SPLITK_MAX_PARTS = 256;                               // at most one part per workgroup
static_assert(MOE_SPLITK_WS_BYTES == (size_t)MOE_SPLITK_MAX_PARTS * 256 * 256 * 4, "one 256x256 fp32 tile per part");
int mfma_rowseg_nt(const void* A, const void* W, long w_es, const int32_t* offsets, int M, int N, int K, int E,
                   void* C, void* splitk_ws, hipStream_t s);
int mfma_rowseg_nn(const void* A, const void* W, long w_es, const int32_t* offsets, int M, int N, int K, int E,
                   void* C, void* splitk_ws, hipStream_t s);
int mfma_dgrad2_swiglu_bwd(const void* d_yp, const void* w2, const int32_t* offsets, int M, int d, int E, int f,
                           const void* H, void* dH, void* A_out, hipStream_t s);
int mfma_wgrad(const void* P, const void* Q, const int32_t* offsets, int Mo, int N, int E, void* C, moe_dtype c_dt,
               int accumulate, hipStream_t s);
// Section 4.1 / 4.2 operator order
int mfma_fc1_swiglu_gather(const void* x, int T, const int32_t* row_token, const float* row_w, const void* w1,
                           const int32_t* offsets, int M, int d, int E, int f, void* H, void* A_out, hipStream_t s);
int mfma_dgrad2_fold_parts(int f);
int mfma_dgrad2_swiglu_bwd_fold(const void* d_yp, const void* w2, const int32_t* offsets, int M, int d, int E, int f,
                                const void* H, void* dH, void* A_out, const float* row_w, float* dw_part, hipStream_t s);

int mfma_fc1_swiglu_fp8(const void* xp, const float* xp_scale, const void* w1, const float* w1_scale,
                        const int32_t* offsets, int M, int d, int E, int f, void* H, void* A_out, hipStream_t s);
int mfma_rowseg_nt_fp8(const void* A, const float* a_scale, const void* W, const float* w_scale, long w_es,
                       const int32_t* offsets, int M, int N, int K, int E, void* C, void* splitk_ws, hipStream_t s);
int mfma_dgrad2_swiglu_bwd_fp8(const void* dyq, const float* dyq_scale, const void* w2t, const float* w2t_scale,
                               const int32_t* offsets, int M, int d, int E, int f, const void* H, void* dH, void* A_out,
                               hipStream_t s);
int mfma_wgrad_fp8(const void* Pt, const uint8_t* p_e8m0, const void* Qt, const uint8_t* q_e8m0, long ldt,
                   const int32_t* pad_offsets, int Mo, int N, int E, void* C, moe_dtype c_dt, int accumulate,
                   hipStream_t s);
int mfma_router_fwd(const void* x, const void* w_r, const float* bias, int T, int d, int E, float* logits,
                    hipStream_t s);
// partial[c][E][d] (+)= g[tokens of chunk c, E]^T * x[tokens of chunk c, d], g and x bf16, chunk_offsets [chunks+1]
int mfma_router_dwr(const void* g, const void* x, const int32_t* chunk_offsets, int chunks, int E, int d, float* partial,
                    int accumulate, hipStream_t s);
int mfma_router_dx(const void* g, const void* w_r, int T, int d, int E, void* dx, hipStream_t s);
size_t router_bwd_ws_bytes(int T, int d, int E);
int mfma_configure_all();          // per-device set-up of every grouped-GEMM kernel (moe_init)
int route_noalloc_prepare();       // looks up this device's static routing scratch (moe_init)
int launch_router_bwd(const void* x, const void* w_r, const float* d_logits, moe_dtype dt, int T, int d, int E,
                      float* d_w_r, void* dx, void* ws, hipStream_t s);

int launch_transpose(const void* src, moe_dtype dt, int batch, int rows, int cols, void* dst, hipStream_t s);

int launch_swiglu_fwd(const void* H, void* A, int M, int f, const int32_t* row_limit, moe_dtype dt, hipStream_t s);
int launch_swiglu_bwd(const void* H, const void* dA, void* dH, int M, int f, const int32_t* row_limit,
                      moe_dtype dt, hipStream_t s);

}  // namespace moe
