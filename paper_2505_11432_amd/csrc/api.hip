// extern "C" entry points: argument validation (before any HIP call), workspace carving and the
// sequencing of kernels for each call.  Declarations and contracts are in include/moe.h.
#include "moe_common.h"

namespace moe {

static thread_local int g_last_hip_error = 0;

int record_hip_error(hipError_t e) {
  g_last_hip_error = static_cast<int>(e);
  return MOE_ERR_HIP;
}

size_t ffn_fwd_ws_bytes(int M, int d, int f, moe_dtype act, moe_dtype out) {
  const size_t m = (size_t)M;
  if (act == MOE_F8E4M3) {
    // A in bf16, A codes, A scales, Y in bf16 (only when yp is written as codes)
    size_t b = align_up(m * f * 2, 256) + align_up(m * f, 256) + align_up(m * 4, 256);
    b += align_up(m * d * 2, 256);          // Y in bf16 (used only when yp is written as codes)
    (void)out;
    return b + MOE_SPLITK_WS_BYTES;
  }
  return align_up(m * f * dtype_size(act), 256) + (act == MOE_BF16 ? MOE_SPLITK_WS_BYTES : 0);
}

size_t ffn_bwd_ws_bytes(int M, int d, int f, moe_dtype dt) {
  (void)d;
  const size_t m = (size_t)M, es = dtype_size(dt);
  return align_up(m * f * es, 256) * 2 + align_up(m * 2 * f * es, 256) + (dt == MOE_BF16 ? MOE_SPLITK_WS_BYTES : 0);
}

static bool sizes_ok(int T, int d, int E, int k, int f) {
  return T >= 0 && d > 0 && f > 0 && E >= 1 && E <= MOE_MAX_EXPERTS && k >= 1 && k <= E && k <= MOE_MAX_TOPK &&
         (long)T * k <= 0x7fffffffL;
}

static int ffn_fwd_plain(const void* xp, const int32_t* offsets, const void* w1, const void* w2, moe_dtype dt, int M,
                         int d, int E, int f, void* h_save, void* yp, void* ws, hipStream_t s) {
  void* A = ws;
  GemmProblem g{};
  g.offsets = offsets; g.E = E; g.mode = 0; g.M = M; g.accumulate = 0; g.bias = nullptr;
  // FC1: H[M,2f] = xp[M,d] * w1[e]^T
  g.A = xp; g.a_rs = d; g.a_cs = 1;
  g.B = w1; g.b_es = 2L * f * d; g.b_rs = 1; g.b_cs = d;
  g.C = h_save; g.c_es = 0; g.ldc = 2L * f; g.N = 2 * f; g.K = d;
  int rc = launch_gemm_generic(g, dt, dt, dt, s);
  if (rc != MOE_OK) return rc;
  rc = launch_swiglu_fwd(h_save, A, M, f, offsets + E, dt, s);
  if (rc != MOE_OK) return rc;
  // FC2: yp[M,d] = A[M,f] * w2[e]^T
  g.A = A; g.a_rs = f; g.a_cs = 1;
  g.B = w2; g.b_es = (long)d * f; g.b_rs = 1; g.b_cs = f;
  g.C = yp; g.ldc = d; g.N = d; g.K = f;
  return launch_gemm_generic(g, dt, dt, dt, s);
}

// bf16: every GEMM on the matrix cores, SwiGLU and its derivative fused into the FC1 / dgrad2 epilogues.
static int ffn_fwd_bf16(const void* xp, const int32_t* offsets, const void* w1, const void* w2, int M, int d, int E,
                        int f, void* h_save, void* yp, void* a_out, void* ws, hipStream_t s) {
  void* A = a_out ? a_out : ws;        // the FC2 input: kept for the caller, or scratch
  int rc = mfma_fc1_swiglu(xp, w1, offsets, M, d, E, f, h_save, A, s);
  if (rc != MOE_OK) return rc;
  void* splitk = static_cast<char*>(ws) + align_up((size_t)M * f * 2, 256);
  return mfma_rowseg_nt(A, w2, (long)d * f, offsets, M, d, f, E, yp, splitk, s);
}

// fp8 (Section 5 / Section 7 "FP8 training"): e4m3 operands with per-token and per-output-channel scales on
// the 32x32x64 MFMA; the SwiGLU output is quantised per token before FC2; yp optionally per token as well.
static int ffn_fwd_fp8(const void* xp, const float* xp_scale, const int32_t* offsets, const void* w1,
                       const float* w1_scale, const void* w2, const float* w2_scale, int M, int d, int E, int f,
                       void* h_save, void* yp, float* yp_scale, moe_dtype out_dt, uint8_t* a_codes_out,
                       float* a_scale_out, void* ws, hipStream_t s) {
  char* base = static_cast<char*>(ws);
  void* A_bf16 = base;
  uint8_t* a_codes = a_codes_out ? a_codes_out : reinterpret_cast<uint8_t*>(base + align_up((size_t)M * f * 2, 256));
  float* a_scale = a_scale_out ? a_scale_out
                               : reinterpret_cast<float*>(base + align_up((size_t)M * f * 2, 256) + align_up((size_t)M * f, 256));
  void* y_bf16 = base + align_up((size_t)M * f * 2, 256) + align_up((size_t)M * f, 256) + align_up((size_t)M * 4, 256);
  int rc = mfma_fc1_swiglu_fp8(xp, xp_scale, w1, w1_scale, offsets, M, d, E, f, h_save, A_bf16, s);
  if (rc != MOE_OK) return rc;
  rc = launch_quant_fp8(A_bf16, MOE_BF16, M, f, MOE_Q_ROW, a_codes, a_scale, s);
  if (rc != MOE_OK) return rc;
  void* y_dst = out_dt == MOE_F8E4M3 ? y_bf16 : yp;
  void* splitk = static_cast<char*>(y_bf16) + align_up((size_t)M * d * 2, 256);
  rc = mfma_rowseg_nt_fp8(a_codes, a_scale, w2, w2_scale, (long)d * f, offsets, M, d, f, E, y_dst, splitk, s);
  if (rc != MOE_OK) return rc;
  if (out_dt == MOE_F8E4M3) rc = launch_quant_fp8(y_bf16, MOE_BF16, M, d, MOE_Q_ROW, static_cast<uint8_t*>(yp), yp_scale, s);
  return rc;
}

static int ffn_bwd_bf16(const void* xp, const void* h_save, const void* d_yp, const void* a_override,
                        const int32_t* offsets, const void* w1, const void* w2, int M, int d, int E, int f,
                        void* d_xp, void* d_w1, void* d_w2, moe_dtype grad_dt, int accumulate, void* ws,
                        hipStream_t s) {
  char* base = static_cast<char*>(ws);
  void* A = base;
  void* dH = base + 2 * align_up((size_t)M * f * 2, 256);
  int rc = mfma_dgrad2_swiglu_bwd(d_yp, w2, offsets, M, d, E, f, h_save, dH, a_override ? nullptr : A, s);
  if (rc != MOE_OK) return rc;
  rc = mfma_wgrad(d_yp, a_override ? a_override : A, offsets, d, f, E, d_w2, grad_dt, accumulate, s);
  if (rc != MOE_OK) return rc;
  void* splitk = base + 2 * align_up((size_t)M * f * 2, 256) + align_up((size_t)M * 2 * f * 2, 256);
  rc = mfma_rowseg_nn(dH, w1, 2L * f * d, offsets, M, d, 2 * f, E, d_xp, splitk, s);
  if (rc != MOE_OK) return rc;
  return mfma_wgrad(dH, xp, offsets, 2 * f, d, E, d_w1, grad_dt, accumulate, s);
}

static int ffn_bwd_plain(const void* xp, const void* h_save, const void* d_yp, const void* a_override,
                         const int32_t* offsets, const void* w1, const void* w2, moe_dtype dt, int M, int d, int E,
                         int f, void* d_xp, void* d_w1, void* d_w2, moe_dtype grad_dt, int accumulate, void* ws,
                         hipStream_t s) {
  const size_t es = dtype_size(dt);
  char* base = static_cast<char*>(ws);
  void* A = base;
  void* dA = base + align_up((size_t)M * f * es, 256);
  void* dH = base + 2 * align_up((size_t)M * f * es, 256);
  int rc;
  const void* A_used = a_override;
  if (a_override == nullptr) {
    rc = launch_swiglu_fwd(h_save, A, M, f, offsets + E, dt, s);     // recompute the FC2 input
    if (rc != MOE_OK) return rc;
    A_used = A;
  }
  GemmProblem g{};
  g.offsets = offsets; g.E = E; g.bias = nullptr;
  // dA[M,f] = d_yp[M,d] * w2[e]   (contraction over d)
  g.mode = 0; g.M = M; g.accumulate = 0;
  g.A = d_yp; g.a_rs = d; g.a_cs = 1;
  g.B = w2; g.b_es = (long)d * f; g.b_rs = f; g.b_cs = 1;
  g.C = dA; g.c_es = 0; g.ldc = f; g.N = f; g.K = d;
  rc = launch_gemm_generic(g, dt, dt, dt, s);
  if (rc != MOE_OK) return rc;
  rc = launch_swiglu_bwd(h_save, dA, dH, M, f, offsets + E, dt, s);
  if (rc != MOE_OK) return rc;
  // d_w2[e][d,f] = d_yp_e^T * A_e   (contraction over the expert's rows)
  g.mode = 1; g.accumulate = accumulate;
  g.A = d_yp; g.a_rs = 1; g.a_cs = d;
  g.B = A_used; g.b_es = 0; g.b_rs = f; g.b_cs = 1;
  g.C = d_w2; g.c_es = (long)d * f; g.ldc = f; g.M = d; g.N = f; g.K = M;
  rc = launch_gemm_generic(g, dt, dt, grad_dt, s);
  if (rc != MOE_OK) return rc;
  // d_xp[M,d] = dH[M,2f] * w1[e]   (contraction over 2f)
  g.mode = 0; g.accumulate = 0;
  g.A = dH; g.a_rs = 2L * f; g.a_cs = 1;
  g.B = w1; g.b_es = 2L * f * d; g.b_rs = d; g.b_cs = 1;
  g.C = d_xp; g.c_es = 0; g.ldc = d; g.M = M; g.N = d; g.K = 2 * f;
  rc = launch_gemm_generic(g, dt, dt, dt, s);
  if (rc != MOE_OK) return rc;
  // d_w1[e][2f,d] = dH_e^T * xp_e
  g.mode = 1; g.accumulate = accumulate;
  g.A = dH; g.a_rs = 1; g.a_cs = 2L * f;
  g.B = xp; g.b_es = 0; g.b_rs = d; g.b_cs = 1;
  g.C = d_w1; g.c_es = 2L * f * d; g.ldc = d; g.M = 2 * f; g.N = d; g.K = M;
  return launch_gemm_generic(g, dt, dt, grad_dt, s);
}

}  // namespace moe

using namespace moe;

extern "C" {

int moe_abi_version(void) { return MOE_ABI_VERSION; }
int moe_last_hip_error(void) { return g_last_hip_error; }

const char* moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_INVALID: return "invalid argument";
    case MOE_ERR_UNSUPPORTED: return "unsupported dtype, size or alignment";
    case MOE_ERR_WORKSPACE: return "workspace missing or too small";
    case MOE_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int moe_init(void) {
  const int rc = mfma_configure_all();
  if (rc != MOE_OK) return rc;
  return route_noalloc_prepare();
}

size_t moe_workspace_bytes(int T, int d, int E, int k, int f, moe_dtype act) {
  if (!sizes_ok(T, d, E, k, f)) return 0;
  if (act != MOE_F32 && act != MOE_BF16 && act != MOE_F8E4M3) return 0;
  const int M = T * k;
  const moe_dtype bwd_dt = act == MOE_F32 ? MOE_F32 : MOE_BF16;
  size_t b = route_ws_bytes(T, E);
  const size_t rb = router_bwd_ws_bytes(T, d, E);
  if (rb > b) b = rb;
  const size_t fw = ffn_fwd_ws_bytes(M, d, f, act, act);
  const size_t bw = ffn_bwd_ws_bytes(M, d, f, bwd_dt);
  if (fw > b) b = fw;
  if (bw > b) b = bw;
  return b + 256;
}

int moe_router_fwd(const void* x, const void* w_r, const float* bias, moe_dtype dt, int T, int d, int E,
                   float* logits, void* stream) {
  if (T < 0 || d <= 0 || E < 1 || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (T == 0) return MOE_OK;
  if (!x || !w_r || !logits) return MOE_ERR_INVALID;
  if (dt != MOE_F32 && dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (dt == MOE_BF16 && d % 8 == 0 && aligned16(x) && aligned16(w_r))
    return mfma_router_fwd(x, w_r, bias, T, d, E, logits, as_stream(stream));
  GemmProblem g{};
  g.mode = 2; g.E = 1; g.offsets = nullptr; g.accumulate = 0; g.bias = bias;
  g.A = x; g.a_rs = d; g.a_cs = 1;
  g.B = w_r; g.b_es = 0; g.b_rs = 1; g.b_cs = d;
  g.C = logits; g.c_es = 0; g.ldc = E; g.M = T; g.N = E; g.K = d;
  return launch_gemm_generic(g, dt, dt, MOE_F32, as_stream(stream));
}

int moe_router_bwd(const void* x, const void* w_r, const float* d_logits, moe_dtype dt, int T, int d, int E,
                   float* d_w_r, void* dx, void* workspace, size_t ws_bytes, void* stream) {
  if (T < 0 || d <= 0 || E < 1 || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (dt != MOE_F32 && dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (d % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (!d_logits && T > 0) return MOE_ERR_INVALID;
  if ((d_w_r && !x && T > 0) || (dx && !w_r)) return MOE_ERR_INVALID;
  if (!aligned16(x) || !aligned16(w_r) || !aligned16(dx) || !aligned16(d_w_r) || !aligned16(workspace))
    return MOE_ERR_UNSUPPORTED;
  const bool ws_ok = workspace && ws_bytes >= router_bwd_ws_bytes(T, d, E);
  if (d_w_r && !ws_ok) return MOE_ERR_WORKSPACE;
  return launch_router_bwd(x, w_r, d_logits, dt, T, d, E, d_w_r, dx, ws_ok ? workspace : nullptr, as_stream(stream));
}

int moe_route(const float* logits, int T, int E, int k, int renorm, int32_t* topk_idx, float* topk_w,
              int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm, void* workspace, size_t ws_bytes,
              void* stream) {
  if (!sizes_ok(T, 16, E, k, 16)) return MOE_ERR_INVALID;
  if (T == 0) return MOE_OK;
  if (!logits || !topk_idx || !topk_w || !counts || !offsets || !perm || !inv_perm) return MOE_ERR_INVALID;
  if (!workspace || ws_bytes < route_ws_bytes(T, E)) return MOE_ERR_WORKSPACE;
  return launch_route(logits, T, E, k, renorm != 0, 0, E, 0, 0, topk_idx, topk_w, nullptr, counts, offsets, perm, inv_perm,
                      workspace, as_stream(stream));
}

int moe_route_range(const float* logits, int T, int E, int k, int renorm, int e_lo, int e_hi, int32_t* topk_idx,
                    float* topk_w, int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                    void* workspace, size_t ws_bytes, void* stream) {
  if (!sizes_ok(T, 16, E, k, 16)) return MOE_ERR_INVALID;
  if (e_lo < 0 || e_hi > E || e_lo > e_hi) return MOE_ERR_INVALID;
  if (T == 0) return MOE_OK;
  if (!logits || !topk_idx || !topk_w || !counts || !offsets || !perm || !inv_perm) return MOE_ERR_INVALID;
  if (!workspace || ws_bytes < route_ws_bytes(T, E)) return MOE_ERR_WORKSPACE;
  return launch_route(logits, T, E, k, renorm != 0, e_lo, e_hi, 0, 0, topk_idx, topk_w, nullptr, counts, offsets, perm,
                      inv_perm, workspace, as_stream(stream));
}

int moe_balance_loss(const float* logits, const int32_t* counts, int T, int E, int k, int n_groups, float alpha,
                     float* loss, float* group_f, float* group_p, void* workspace, size_t ws_bytes, void* stream) {
  if (!sizes_ok(T, 16, E, k, 16)) return MOE_ERR_INVALID;
  if (n_groups < 1 || n_groups > E || E % n_groups != 0) return MOE_ERR_INVALID;
  if (!loss || !group_f || !group_p) return MOE_ERR_INVALID;
  if (T == 0) return MOE_ERR_INVALID;                 // the loss is a mean over tokens
  if (!logits || !counts) return MOE_ERR_INVALID;
  if (!workspace || ws_bytes < balance_ws_bytes(T, E)) return MOE_ERR_WORKSPACE;
  return launch_balance_loss(logits, counts, T, E, k, n_groups, alpha, loss, group_f, group_p, workspace, as_stream(stream));
}

int moe_balance_loss_bwd(const float* logits, const float* group_f, int T, int E, int n_groups, float alpha,
                         float* d_logits, void* stream) {
  if (T < 0 || E < 1 || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (n_groups < 1 || n_groups > E || E % n_groups != 0) return MOE_ERR_INVALID;
  if (T == 0) return MOE_OK;
  if (!logits || !group_f || !d_logits) return MOE_ERR_INVALID;
  return launch_balance_loss_bwd(logits, group_f, T, E, n_groups, alpha, d_logits, as_stream(stream));
}

size_t moe_route_capacity_workspace_bytes(int T, int E, int k) {
  if (!sizes_ok(T, 16, E, k, 16)) return 0;
  return route_capacity_ws_bytes(T, E, k);
}

int moe_route_capacity(const float* logits, int T, int E, int k, int renorm, int n_groups, int capacity,
                       int32_t* topk_idx, float* topk_w, float* score, int32_t* counts, int32_t* offsets,
                       int32_t* perm, int32_t* inv_perm, void* workspace, size_t ws_bytes, void* stream) {
  if (!sizes_ok(T, 16, E, k, 16)) return MOE_ERR_INVALID;
  if (n_groups < 1 || n_groups > E || E % n_groups != 0 || capacity < 0) return MOE_ERR_INVALID;
  if (T == 0) return MOE_OK;
  if (!logits || !topk_idx || !topk_w || !score || !counts || !offsets || !perm || !inv_perm) return MOE_ERR_INVALID;
  if (!workspace || ws_bytes < route_capacity_ws_bytes(T, E, k)) return MOE_ERR_WORKSPACE;
  return launch_route(logits, T, E, k, renorm != 0, 0, E, n_groups, capacity, topk_idx, topk_w, score, counts, offsets, perm,
                      inv_perm, workspace, as_stream(stream));
}

int moe_route_bwd(const float* logits, const int32_t* topk_idx, const float* topk_w, const float* d_topk_w, int T,
                  int E, int k, int renorm, float* d_logits, void* stream) {
  if (!sizes_ok(T, 16, E, k, 16)) return MOE_ERR_INVALID;
  if (T == 0) return MOE_OK;
  if (!topk_idx || !topk_w || !d_topk_w || !d_logits) return MOE_ERR_INVALID;
  if (!renorm && !logits) return MOE_ERR_INVALID;
  return launch_route_bwd(logits, topk_idx, topk_w, d_topk_w, T, E, k, renorm != 0, d_logits, as_stream(stream));
}

int moe_dispatch(const void* x, const float* x_scale, moe_dtype dt, const int32_t* inv_perm, const float* row_mul,
                 int T, int k, int d, void* xp, float* xp_scale, void* stream) {
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || d <= 0 || (long)T * k > 0x7fffffffL) return MOE_ERR_INVALID;
  if (dt != MOE_F32 && dt != MOE_BF16 && dt != MOE_F8E4M3) return MOE_ERR_UNSUPPORTED;
  if (d % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (T == 0) return MOE_OK;
  if (!x || !inv_perm || !xp) return MOE_ERR_INVALID;
  if (dt == MOE_F8E4M3) {
    if (row_mul) return MOE_ERR_UNSUPPORTED;
    if (!x_scale || !xp_scale) return MOE_ERR_INVALID;
  } else if (x_scale || xp_scale) {
    return MOE_ERR_INVALID;
  }
  if (!aligned16(x) || !aligned16(xp)) return MOE_ERR_UNSUPPORTED;
  return launch_dispatch(x, x_scale, dt, inv_perm, row_mul, T, k, d, xp, xp_scale, as_stream(stream));
}

int moe_combine(const void* yp, const float* yp_scale, moe_dtype dt, const int32_t* inv_perm, const float* topk_w,
                int T, int k, int d, void* y, moe_dtype y_dt, void* stream) {
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || d <= 0 || (long)T * k > 0x7fffffffL) return MOE_ERR_INVALID;
  if (d % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (dt != MOE_F32 && dt != MOE_BF16 && dt != MOE_F8E4M3) return MOE_ERR_UNSUPPORTED;
  if (y_dt != MOE_F32 && y_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (dt == MOE_F32 && y_dt != MOE_F32) return MOE_ERR_UNSUPPORTED;
  if (T == 0) return MOE_OK;
  if (!yp || !inv_perm || !y) return MOE_ERR_INVALID;
  if ((dt == MOE_F8E4M3) != (yp_scale != nullptr)) return MOE_ERR_INVALID;
  if (!aligned16(yp) || !aligned16(y)) return MOE_ERR_UNSUPPORTED;
  return launch_combine(yp, yp_scale, dt, inv_perm, topk_w, T, k, d, y, y_dt, as_stream(stream));
}

int moe_gate_grad(const void* dy, moe_dtype dy_dt, const void* yp, const float* yp_scale, moe_dtype dt,
                  const int32_t* inv_perm, int T, int k, int d, float* d_topk_w, void* stream) {
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || d <= 0 || (long)T * k > 0x7fffffffL) return MOE_ERR_INVALID;
  if (d % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (dy_dt != MOE_F32 && dy_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (dt != MOE_F8E4M3 && dt != dy_dt) return MOE_ERR_UNSUPPORTED;
  if (T == 0) return MOE_OK;
  if (!dy || !yp || !inv_perm || !d_topk_w) return MOE_ERR_INVALID;
  if ((dt == MOE_F8E4M3) != (yp_scale != nullptr)) return MOE_ERR_INVALID;
  if (!aligned16(yp) || !aligned16(dy)) return MOE_ERR_UNSUPPORTED;
  return launch_gate_grad(dy, dy_dt, yp, yp_scale, dt, inv_perm, T, k, d, d_topk_w, as_stream(stream));
}

int moe_expert_ffn_fwd(const void* xp, const float* xp_scale, moe_dtype act_dt, const int32_t* offsets,
                       const void* w1, const float* w1_scale, const void* w2, const float* w2_scale, moe_dtype w_dt,
                       int M, int d, int E, int f, void* h_save, void* yp, float* yp_scale, moe_dtype out_dt,
                       uint8_t* a_codes_out, float* a_scale_out, void* workspace, size_t ws_bytes, void* stream) {
  if (M < 0 || d <= 0 || f <= 0 || E < 1 || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (d % 16 != 0 || f % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (act_dt != w_dt) return MOE_ERR_UNSUPPORTED;
  if (act_dt != MOE_F32 && act_dt != MOE_BF16 && act_dt != MOE_F8E4M3) return MOE_ERR_UNSUPPORTED;
  if (act_dt != MOE_F8E4M3 && out_dt != act_dt) return MOE_ERR_UNSUPPORTED;
  if (act_dt == MOE_F8E4M3 && out_dt != MOE_F8E4M3 && out_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (M == 0) return MOE_OK;
  if (!xp || !offsets || !w1 || !w2 || !h_save || !yp) return MOE_ERR_INVALID;
  const bool fp8 = act_dt == MOE_F8E4M3;
  if (fp8 != (xp_scale != nullptr) || fp8 != (w1_scale != nullptr) || fp8 != (w2_scale != nullptr))
    return MOE_ERR_INVALID;
  if ((out_dt == MOE_F8E4M3) != (yp_scale != nullptr)) return MOE_ERR_INVALID;
  if (!aligned16(xp) || !aligned16(w1) || !aligned16(w2) || !aligned16(h_save) || !aligned16(yp) ||
      !aligned16(workspace))
    return MOE_ERR_UNSUPPORTED;
  if (!workspace || ws_bytes < ffn_fwd_ws_bytes(M, d, f, act_dt, out_dt)) return MOE_ERR_WORKSPACE;
  if (fp8 && (a_codes_out != nullptr) != (a_scale_out != nullptr)) return MOE_ERR_INVALID;
  if (!fp8 && (a_scale_out || (a_codes_out && act_dt != MOE_BF16))) return MOE_ERR_INVALID;
  if (!aligned16(a_codes_out)) return MOE_ERR_UNSUPPORTED;
  if (fp8) {
    // rows at or beyond offsets[E] are never read by the GEMMs, but the row quantisers walk all M rows
    return ffn_fwd_fp8(xp, xp_scale, offsets, w1, w1_scale, w2, w2_scale, M, d, E, f, h_save, yp, yp_scale, out_dt,
                       a_codes_out, a_scale_out, workspace, as_stream(stream));
  }
  if (act_dt == MOE_BF16)
    return ffn_fwd_bf16(xp, offsets, w1, w2, M, d, E, f, h_save, yp, a_codes_out, workspace, as_stream(stream));
  return ffn_fwd_plain(xp, offsets, w1, w2, act_dt, M, d, E, f, h_save, yp, workspace, as_stream(stream));
}

int moe_expert_ffn_bwd(const void* xp, const void* h_save, const void* d_yp, const void* a_override,
                       const int32_t* offsets, const void* w1, const void* w2, moe_dtype dt, int M, int d, int E,
                       int f, void* d_xp, void* d_w1, void* d_w2, moe_dtype grad_dt, int accumulate, void* workspace,
                       size_t ws_bytes, void* stream) {
  if (M < 0 || d <= 0 || f <= 0 || E < 1 || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (d % 16 != 0 || f % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (dt != MOE_F32 && dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (grad_dt != MOE_F32 && grad_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (dt == MOE_F32 && grad_dt != MOE_F32) return MOE_ERR_UNSUPPORTED;
  if (!offsets || !d_w1 || !d_w2) return MOE_ERR_INVALID;
  if (M > 0 && (!xp || !h_save || !d_yp || !w1 || !w2 || !d_xp)) return MOE_ERR_INVALID;
  if (!aligned16(xp) || !aligned16(h_save) || !aligned16(d_yp) || !aligned16(w1) || !aligned16(w2) ||
      !aligned16(d_xp) || !aligned16(d_w1) || !aligned16(d_w2) || !aligned16(a_override) || !aligned16(workspace))
    return MOE_ERR_UNSUPPORTED;
  if (M > 0 && (!workspace || ws_bytes < ffn_bwd_ws_bytes(M, d, f, dt))) return MOE_ERR_WORKSPACE;
  if (dt == MOE_BF16)
    return ffn_bwd_bf16(xp, h_save, d_yp, a_override, offsets, w1, w2, M, d, E, f, d_xp, d_w1, d_w2, grad_dt,
                        accumulate != 0, workspace, as_stream(stream));
  return ffn_bwd_plain(xp, h_save, d_yp, a_override, offsets, w1, w2, dt, M, d, E, f, d_xp, d_w1, d_w2, grad_dt,
                       accumulate != 0, workspace, as_stream(stream));
}

// ---- Section 4.1 / 4.2 operator order (bf16) ---------------------------------------------------------------
// workspace: A' [M,f] | dH [M,2f] | one [M,d] buffer (dY', later the re-dispatched FC1 input) | gate-gradient partials | split-K
static size_t fused_a_bytes(size_t m, int f) { return align_up(m * f * 2, 256); }
static size_t fused_dh_bytes(size_t m, int f) { return align_up(m * 2 * f * 2, 256); }
static size_t fused_rows_bytes(size_t m, int d) { return align_up(m * d * 2, 256); }
static size_t fused_part_bytes(size_t m, int f) { return align_up((size_t)mfma_dgrad2_fold_parts(f) * m * 4, 256); }

size_t moe_expert_ffn_fused_workspace_bytes(int T, int k, int d, int f) {
  if (T < 0 || k < 1 || d <= 0 || f <= 0) return 0;
  const size_t m = (size_t)T * k;
  return fused_a_bytes(m, f) + fused_dh_bytes(m, f) + fused_rows_bytes(m, d) + fused_part_bytes(m, f) + MOE_SPLITK_WS_BYTES + 256;
}

int moe_row_map(const int32_t* perm, const float* topk_w, const int32_t* offsets, int E, int T, int k,
                int32_t* row_token, float* row_w, void* stream) {
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || E < 1 || E > MOE_MAX_EXPERTS || (long)T * k > 0x7fffffffL) return MOE_ERR_INVALID;
  if (T == 0) return MOE_OK;
  if (!perm || !topk_w || !offsets || !row_token || !row_w) return MOE_ERR_INVALID;
  return launch_row_map(perm, topk_w, offsets, E, T * k, k, row_token, row_w, as_stream(stream));
}

static int fused_args_ok(int T, int k, int d, int E, int f) {
  if (T < 0 || k < 1 || k > MOE_MAX_TOPK || d <= 0 || f <= 0 || E < 1 || E > MOE_MAX_EXPERTS || (long)T * k > 0x7fffffffL)
    return MOE_ERR_INVALID;
  if (d % 16 != 0 || f % 16 != 0) return MOE_ERR_UNSUPPORTED;
  return MOE_OK;
}

int moe_expert_ffn_fused_fwd(const void* x, const int32_t* row_token, const float* row_w, const int32_t* offsets,
                             const void* w1, const void* w2, int T, int k, int d, int E, int f, void* h_save, void* ypw,
                             void* workspace, size_t ws_bytes, void* stream) {
  int rc = fused_args_ok(T, k, d, E, f);
  if (rc != MOE_OK) return rc;
  if (T == 0) return MOE_OK;
  if (!x || !row_token || !row_w || !offsets || !w1 || !w2 || !h_save || !ypw) return MOE_ERR_INVALID;
  if (!aligned16(x) || !aligned16(w1) || !aligned16(w2) || !aligned16(h_save) || !aligned16(ypw) || !aligned16(workspace))
    return MOE_ERR_UNSUPPORTED;
  if (!workspace || ws_bytes < moe_expert_ffn_fused_workspace_bytes(T, k, d, f)) return MOE_ERR_WORKSPACE;
  const int M = T * k;
  hipStream_t s = as_stream(stream);
  char* base = static_cast<char*>(workspace);
  void* Aw = base;
  void* splitk = base + fused_a_bytes(M, f) + fused_dh_bytes(M, f) + fused_rows_bytes(M, d) + fused_part_bytes(M, f);
  rc = mfma_fc1_swiglu_gather(x, T, row_token, row_w, w1, offsets, M, d, E, f, h_save, Aw, s);
  if (rc != MOE_OK) return rc;
  return mfma_rowseg_nt(Aw, w2, (long)d * f, offsets, M, d, f, E, ypw, splitk, s);
}

int moe_expert_ffn_fused_bwd(const void* x, const void* dy, const void* h_save, const int32_t* inv_perm,
                             const float* topk_w, const float* row_w, const int32_t* offsets, const void* w1, const void* w2, int T, int k,
                             int d, int E, int f, void* d_xp, void* d_w1, void* d_w2, moe_dtype grad_dt, int accumulate,
                             float* d_topk_w, void* workspace, size_t ws_bytes, void* stream) {
  int rc = fused_args_ok(T, k, d, E, f);
  if (rc != MOE_OK) return rc;
  if (grad_dt != MOE_F32 && grad_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (!offsets || !d_w1 || !d_w2) return MOE_ERR_INVALID;
  if (T > 0 && (!x || !dy || !h_save || !inv_perm || !topk_w || !row_w || !w1 || !w2 || !d_xp || !d_topk_w)) return MOE_ERR_INVALID;
  if (!aligned16(x) || !aligned16(dy) || !aligned16(h_save) || !aligned16(w1) || !aligned16(w2) || !aligned16(d_xp) ||
      !aligned16(d_w1) || !aligned16(d_w2) || !aligned16(workspace))
    return MOE_ERR_UNSUPPORTED;
  if (T > 0 && (!workspace || ws_bytes < moe_expert_ffn_fused_workspace_bytes(T, k, d, f))) return MOE_ERR_WORKSPACE;
  const int M = T * k;
  hipStream_t s = as_stream(stream);
  char* base = static_cast<char*>(workspace);
  void* Aw = base;
  void* dH = base + fused_a_bytes(M, f);
  void* rows = static_cast<char*>(dH) + fused_dh_bytes(M, f);
  float* part = reinterpret_cast<float*>(static_cast<char*>(rows) + fused_rows_bytes(M, d));
  void* splitk = reinterpret_cast<char*>(part) + fused_part_bytes(M, f);
  if (T > 0) {
    // dY'[r] = dy[token of r], unweighted: the weight now sits between SwiGLU and FC2
    rc = launch_dispatch(dy, nullptr, MOE_BF16, inv_perm, nullptr, T, k, d, rows, nullptr, s);
    if (rc != MOE_OK) return rc;
    rc = mfma_dgrad2_swiglu_bwd_fold(rows, w2, offsets, M, d, E, f, h_save, dH, Aw, row_w, part, s);
    if (rc != MOE_OK) return rc;
    rc = launch_gate_grad_reduce(part, mfma_dgrad2_fold_parts(f), M, inv_perm, M, d_topk_w, s);
    if (rc != MOE_OK) return rc;
  }
  rc = mfma_wgrad(rows, Aw, offsets, d, f, E, d_w2, grad_dt, accumulate != 0, s);
  if (rc != MOE_OK) return rc;
  if (T > 0) {
    rc = mfma_rowseg_nn(dH, w1, 2L * f * d, offsets, M, d, 2 * f, E, d_xp, splitk, s);
    if (rc != MOE_OK) return rc;
    // the FC1 input rows are produced again here instead of being kept since the forward (Section 4.1); they carry
    // the gate weight that dH was computed without
    rc = launch_dispatch(x, nullptr, MOE_BF16, inv_perm, topk_w, T, k, d, rows, nullptr, s);
    if (rc != MOE_OK) return rc;
  }
  return mfma_wgrad(dH, rows, offsets, 2 * f, d, E, d_w1, grad_dt, accumulate != 0, s);
}

int moe_quant_fp8(const void* src, moe_dtype src_dt, int rows, int cols, moe_qmode mode, uint8_t* codes,
                  float* scales, void* stream) {
  if (rows < 0 || cols < 0) return MOE_ERR_INVALID;
  if (src_dt != MOE_F32 && src_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (mode != MOE_Q_ROW && mode != MOE_Q_COLGROUP128) return MOE_ERR_INVALID;
  if (cols % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (rows == 0 || cols == 0) return MOE_OK;
  if (!src || !codes || !scales) return MOE_ERR_INVALID;
  if (!aligned16(src) || !aligned16(codes)) return MOE_ERR_UNSUPPORTED;
  return launch_quant_fp8(src, src_dt, rows, cols, mode, codes, scales, as_stream(stream));
}

int moe_dequant_fp8(const uint8_t* codes, const float* scales, int rows, int cols, moe_qmode mode, void* dst,
                    moe_dtype dst_dt, void* stream) {
  if (rows < 0 || cols < 0) return MOE_ERR_INVALID;
  if (dst_dt != MOE_F32 && dst_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (mode != MOE_Q_ROW && mode != MOE_Q_COLGROUP128) return MOE_ERR_INVALID;
  if (cols % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (rows == 0 || cols == 0) return MOE_OK;
  if (!codes || !scales || !dst) return MOE_ERR_INVALID;
  if (!aligned16(codes) || !aligned16(dst)) return MOE_ERR_UNSUPPORTED;
  return launch_dequant_fp8(codes, scales, rows, cols, mode, dst, dst_dt, as_stream(stream));
}

int moe_transpose(const void* src, moe_dtype dt, int batch, int rows, int cols, void* dst, void* stream) {
  if (batch < 0 || rows < 0 || cols < 0 || batch > 65535) return MOE_ERR_INVALID;
  if (dt != MOE_F32 && dt != MOE_BF16 && dt != MOE_F8E4M3) return MOE_ERR_UNSUPPORTED;
  if (batch == 0 || rows == 0 || cols == 0) return MOE_OK;
  if (!src || !dst || src == dst) return MOE_ERR_INVALID;
  if ((long)cdiv(rows, 64) > 65535) return MOE_ERR_UNSUPPORTED;
  return launch_transpose(src, dt, batch, rows, cols, dst, as_stream(stream));
}

size_t moe_tgroup_tokens(int rows, int E) {
  if (rows < 0 || E < 1) return 0;
  return ((size_t)(rows + 127) / 128 + (size_t)E) * 128;
}

int moe_quant_fp8_tgroup(const void* src, moe_dtype src_dt, int rows, int cols, const int32_t* offsets, int E,
                         int32_t* pad_offsets, uint8_t* codes_t, long ldt, uint8_t* e8m0, void* stream) {
  if (rows < 0 || cols < 0 || E < 1 || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (src_dt != MOE_F32 && src_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (cols % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (!offsets || !pad_offsets) return MOE_ERR_INVALID;
  if (ldt % 128 != 0 || ldt < (long)moe_tgroup_tokens(rows, E)) return MOE_ERR_INVALID;
  if (cols > 0 && (!codes_t || !e8m0 || (rows > 0 && !src))) return MOE_ERR_INVALID;
  if (!aligned16(src) || !aligned16(codes_t)) return MOE_ERR_UNSUPPORTED;
  int rc = launch_tgroup_offsets(offsets, E, pad_offsets, as_stream(stream));
  if (rc != MOE_OK) return rc;
  return launch_quant_tgroup(src, nullptr, src_dt, rows, cols, offsets, pad_offsets, E, codes_t, ldt, e8m0, as_stream(stream));
}

int moe_expert_ffn_bwd_fp8(const moe_ffn_bwd_fp8_args* a, void* stream) {
  if (!a) return MOE_ERR_INVALID;
  const int M = a->M, d = a->d, E = a->E, f = a->f;
  if (M < 0 || d <= 0 || f <= 0 || E < 1 || E > MOE_MAX_EXPERTS) return MOE_ERR_INVALID;
  if (d % 16 != 0 || f % 16 != 0) return MOE_ERR_UNSUPPORTED;
  if (a->grad_dt != MOE_F32 && a->grad_dt != MOE_BF16) return MOE_ERR_UNSUPPORTED;
  if (a->ldt % 128 != 0 || a->ldt < (long)moe_tgroup_tokens(M, E)) return MOE_ERR_INVALID;
  // the two forward operands: dequantised bf16 copies, or the codes and per-row scales themselves
  const bool x_codes = a->xp_codes != nullptr, a_codes = a->a_codes != nullptr;
  if (x_codes ? !a->xp_scale : !a->xp_deq) return MOE_ERR_INVALID;
  if (a_codes ? !a->a_scale : !a->a_deq) return MOE_ERR_INVALID;
  if (!aligned16(a->xp_codes) || !aligned16(a->a_codes)) return MOE_ERR_UNSUPPORTED;
  const void* ptrs[] = {a->d_yp, a->h_save, a->offsets, a->w1t, a->w1t_scale, a->w2t, a->w2t_scale,
                        a->d_xp, a->d_w1, a->d_w2, a->dy_codes, a->dy_scale, a->dh, a->dh_codes, a->dh_scale,
                        a->pad_offsets, a->dy_t, a->dy_e8m0, a->dh_t, a->dh_e8m0, a->a_t, a->a_e8m0, a->x_t, a->x_e8m0};
  for (const void* q : ptrs)
    if (!q) return MOE_ERR_INVALID;
  const void* vec[] = {a->d_yp, a->h_save, a->xp_deq, a->a_deq, a->w1t, a->w2t, a->d_xp, a->d_w1, a->d_w2, a->dy_codes,
                       a->dh, a->dh_codes, a->dy_t, a->dh_t, a->a_t, a->x_t, a->splitk_ws};
  for (const void* q : vec)
    if (!aligned16(q)) return MOE_ERR_UNSUPPORTED;
  hipStream_t s = as_stream(stream);
  const int acc = a->accumulate != 0;
  int rc = launch_quant_fp8(a->d_yp, MOE_BF16, M, d, MOE_Q_ROW, a->dy_codes, a->dy_scale, s);
  if (rc != MOE_OK) return rc;
  rc = mfma_dgrad2_swiglu_bwd_fp8(a->dy_codes, a->dy_scale, a->w2t, a->w2t_scale, a->offsets, M, d, E, f, a->h_save, a->dh,
                                  nullptr, s);
  if (rc != MOE_OK) return rc;
  rc = launch_quant_fp8(a->dh, MOE_BF16, M, 2 * f, MOE_Q_ROW, a->dh_codes, a->dh_scale, s);
  if (rc != MOE_OK) return rc;
  rc = mfma_rowseg_nt_fp8(a->dh_codes, a->dh_scale, a->w1t, a->w1t_scale, (long)d * 2 * f, a->offsets, M, d, 2 * f, E,
                          a->d_xp, a->splitk_ws, s);
  if (rc != MOE_OK) return rc;
  rc = launch_tgroup_offsets(a->offsets, E, a->pad_offsets, s);
  if (rc != MOE_OK) return rc;
  rc = launch_quant_tgroup(a->d_yp, nullptr, MOE_BF16, M, d, a->offsets, a->pad_offsets, E, a->dy_t, a->ldt, a->dy_e8m0, s);
  if (rc != MOE_OK) return rc;
  rc = a_codes ? launch_quant_tgroup(a->a_codes, a->a_scale, MOE_F8E4M3, M, f, a->offsets, a->pad_offsets, E, a->a_t, a->ldt, a->a_e8m0, s)
               : launch_quant_tgroup(a->a_deq, nullptr, MOE_BF16, M, f, a->offsets, a->pad_offsets, E, a->a_t, a->ldt, a->a_e8m0, s);
  if (rc != MOE_OK) return rc;
  rc = mfma_wgrad_fp8(a->dy_t, a->dy_e8m0, a->a_t, a->a_e8m0, a->ldt, a->pad_offsets, d, f, E, a->d_w2, a->grad_dt, acc, s);
  if (rc != MOE_OK) return rc;
  rc = launch_quant_tgroup(a->dh, nullptr, MOE_BF16, M, 2 * f, a->offsets, a->pad_offsets, E, a->dh_t, a->ldt, a->dh_e8m0, s);
  if (rc != MOE_OK) return rc;
  rc = x_codes ? launch_quant_tgroup(a->xp_codes, a->xp_scale, MOE_F8E4M3, M, d, a->offsets, a->pad_offsets, E, a->x_t, a->ldt, a->x_e8m0, s)
               : launch_quant_tgroup(a->xp_deq, nullptr, MOE_BF16, M, d, a->offsets, a->pad_offsets, E, a->x_t, a->ldt, a->x_e8m0, s);
  if (rc != MOE_OK) return rc;
  return mfma_wgrad_fp8(a->dh_t, a->dh_e8m0, a->x_t, a->x_e8m0, a->ldt, a->pad_offsets, 2 * f, d, E, a->d_w1, a->grad_dt, acc, s);
}

}  // extern "C"
