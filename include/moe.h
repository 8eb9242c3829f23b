/*
 * moe.h -- C ABI of the MI355X (gfx950) MoE expert-FFN hot path.
 *
 * One GPU's share of a mixture-of-experts FFN layer, forward and backward, after
 * MegaScale-MoE (arXiv 2505.11432): top-k gating, token dispatch into expert-contiguous
 * buffers, the expert grouped GEMMs with SwiGLU, the gate-weighted combine, and the E4M3
 * cast that stands in for the paper's communication compression.
 *
 * Conventions for every call
 *   - Every data pointer is a DEVICE pointer owned by the caller (16-byte aligned).  The
 *     library allocates nothing, frees nothing and keeps no pointer after it returns.
 *     Scratch comes from the caller's `workspace` (size from moe_workspace_bytes).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  A call only
 *     enqueues kernels on that stream and returns; it never synchronises and never copies
 *     device data to the host.  Expert row counts live on the device only, so grids are
 *     sized for the worst case and kernels read `offsets` themselves.
 *   - Return value: MOE_OK, or a negative moe_status.  Arguments are validated before any
 *     HIP call, so argument errors are reported on a machine without a GPU as well.
 *   - Matrices are row-major and dense.  Weights are "out, in": w1 [E, 2f, d] (gate
 *     projection in rows 0..f-1, up projection in rows f..2f-1), w2 [E, d, f], w_r [E_r, d].
 *   - T tokens, d model width (the paper's h), f expert width (h_ffn), E experts, k experts
 *     per token, M = T*k dispatched rows.  Assignment id a = t*k + j (token t, slot j).
 *   - d and f must be multiples of 16; 1 <= k <= E <= MOE_MAX_EXPERTS; k <= MOE_MAX_TOPK.
 *   - T = 0 is valid and does nothing.  Non-finite logits give an unspecified routing.
 *   - Calls on different streams or from different threads may run concurrently as long as
 *     their buffers (workspace included) do not overlap; the library keeps no mutable state
 *     beyond per-device set-up flags, which are atomic (see moe_init).
 */
#ifndef MOE_HIP_MOE_H
#define MOE_HIP_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_ABI_VERSION 1
#define MOE_MAX_EXPERTS 256
#define MOE_MAX_TOPK 16

typedef enum {
  MOE_OK = 0,
  MOE_ERR_INVALID = -1,      /* NULL pointer, negative size, k < 1, k > E, E too large */
  MOE_ERR_UNSUPPORTED = -2,  /* dtype combination or alignment the kernels do not cover */
  MOE_ERR_WORKSPACE = -3,    /* workspace missing or smaller than moe_workspace_bytes */
  MOE_ERR_HIP = -4           /* a HIP runtime call failed; see moe_last_hip_error */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1, MOE_F8E4M3 = 2 /* OCP e4m3fn, max 448 */ } moe_dtype;
typedef enum { MOE_Q_ROW = 0, MOE_Q_COLGROUP128 = 1 } moe_qmode;

int moe_abi_version(void);
/* hipError_t value of the last failed HIP call made by this thread (0 if none). */
int moe_last_hip_error(void);
const char* moe_status_string(int status);

/* Optional one-time set-up for the CURRENT device: raises the dynamic-LDS limit of every
 * grouped-GEMM kernel and looks up the static scratch of moe_route_noalloc.  Without it each
 * kernel does its own set-up on its first launch on a device (thread-safe, but not a stream
 * operation): a caller that records the calls of this library into a HIP graph either calls
 * moe_init() first or runs every call once, eagerly, before the capture starts.  Idempotent;
 * allocates nothing; call it again after switching to another device. */
int moe_init(void);

/* Bytes of scratch that the largest consumer (moe_expert_ffn_bwd) needs for these sizes;
 * valid for every call of this library with the same sizes.  0 on invalid sizes. */
size_t moe_workspace_bytes(int T, int d, int E, int k, int f, moe_dtype act);

/* ---- router matmul: the "routing scores" operator (Section 7, "MoE vs. dense") -------
 * logits[t,e] = sum_i x[t,i] * w_r[e,i] (+ bias[e]); fp32 accumulate, fp32 result.
 * x [T,d] and w_r [E,d] in `dt` (MOE_F32 or MOE_BF16); bias [E] fp32 or NULL. */
int moe_router_fwd(const void* x, const void* w_r, const float* bias, moe_dtype dt,
                   int T, int d, int E, float* logits /*[T,E]*/, void* stream);

/* Gradients of moe_router_fwd: d_w_r[e,i] = sum_t d_logits[t,e] * x[t,i] (fp32 [E,d],
 * overwritten; summed in a fixed order, so reproducible) and dx[t,i] += sum_e d_logits[t,e]
 * * w_r[e,i] (dx [T,d] in `dt`, read and written).  d_w_r or dx may be NULL to skip that
 * half.  d_w_r needs workspace (moe_workspace_bytes); dx alone runs without one.  With a
 * workspace, bf16 data and 32 experts or more, dx is computed on the matrix cores from the
 * gate gradient rounded to bf16 (relative 2^-9, below the rounding of the bf16 result). */
int moe_router_bwd(const void* x, const void* w_r, const float* d_logits, moe_dtype dt,
                   int T, int d, int E, float* d_w_r, void* dx,
                   void* workspace, size_t ws_bytes, void* stream);

/* ---- gating and row map (Section 2.1: top-k gate; Section 3.2 "Efficient operators":
 * the pre-computed mapping from input rows to output rows; Section 4.2: rows ordered by
 * expert, then by source, i.e. by assignment id on one rank) ---------------------------
 * Per token the k largest logits are selected (equal logits: lower expert id first; slot
 * j holds the (j+1)-th largest).  renorm=1: topk_w = softmax over the k selected logits;
 * renorm=0: softmax over all E logits read at the selected experts.
 * counts[e] = number of assignments to e; offsets = exclusive prefix sum, offsets[E] = M.
 * perm[r] = assignment id held by dispatched row r (stable: ascending a inside an
 * expert's segment); inv_perm[a] = r.  All outputs are fully written.  Integer outputs
 * are deterministic and unique.  Needs workspace. */
int moe_route(const float* logits /*[T,E]*/, int T, int E, int k, int renorm,
              int32_t* topk_idx /*[T,k]*/, float* topk_w /*[T,k]*/,
              int32_t* counts /*[E]*/, int32_t* offsets /*[E+1]*/,
              int32_t* perm /*[T*k]*/, int32_t* inv_perm /*[T*k]*/,
              void* workspace, size_t ws_bytes, void* stream);

/* ---- moe_route without a workspace, for callers that cannot allocate ---------------------------
 * For code under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: the
 * same computation and outputs as moe_route, bit for bit, but the scratch (the per-chunk expert
 * histograms) is a static device array of MOE_ROUTE_NOALLOC_SCRATCH_BYTES inside the library
 * instead of a caller workspace.  The call allocates nothing and frees nothing; the first call
 * on a device looks up that device's copy of the array (no allocation, but make it before a
 * graph capture starts).  Limit: ceil(T / c) * E * 4 <= MOE_ROUTE_NOALLOC_SCRATCH_BYTES, where
 * c = 64, 128, 256, ... is the smallest chunk with ceil(T / c) <= 1024 -- any T for E <= 64,
 * T <= 16384 for E = 256; beyond it the call returns MOE_ERR_UNSUPPORTED and moe_route is the
 * one to use.  All calls on one GPU share that GPU's array: two calls that overlap in time on
 * one GPU (different streams) race; calls on one stream, or on different GPUs, do not.  The
 * array keeps the last call's contents and nothing in it needs clearing: every entry a call
 * reads it has written itself. */
#define MOE_ROUTE_NOALLOC_SCRATCH_BYTES ((size_t)256 * 1024)
int moe_route_noalloc(const float* logits /*[T,E]*/, int T, int E, int k, int renorm,
                      int32_t* topk_idx /*[T,k]*/, float* topk_w /*[T,k]*/,
                      int32_t* counts /*[E]*/, int32_t* offsets /*[E+1]*/,
                      int32_t* perm /*[T*k]*/, int32_t* inv_perm /*[T*k]*/, void* stream);

/* The same for one GPU's expert-parallel share (Section 3.2: after the all-gather of the tokens a
 * local scatter keeps only those routed to local experts; Section 3.1: each rank holds E/n
 * experts).  The gate runs over all E experts; only assignments whose expert lies in
 * [e_lo, e_hi) get a row.  counts [E] stays global.  offsets has e_hi - e_lo + 1 entries and
 * covers the local experts (offsets[e_hi - e_lo] = number of local rows); perm [T*k] is written
 * for the local rows only; inv_perm [T*k] = -1 for an assignment without a row.  moe_dispatch,
 * moe_combine and moe_gate_grad skip such assignments: the combine then yields the partial sum
 * over the local experts (what a reduce-scatter adds up across ranks), the gate gradient is 0
 * there.  The expert FFN calls take the local weights, E = e_hi - e_lo and M = T*k as the row
 * bound (they touch no row at or past offsets[E]).  e_lo = 0, e_hi = E is moe_route. */
int moe_route_range(const float* logits, int T, int E, int k, int renorm, int e_lo, int e_hi,
                    int32_t* topk_idx, float* topk_w, int32_t* counts, int32_t* offsets,
                    int32_t* perm, int32_t* inv_perm, void* workspace, size_t ws_bytes,
                    void* stream);

/* ---- load balance (Section 3.2 "Load balance": auxiliary loss and token dropping, both per
 * device: the experts placed on one GPU form a group, as in DeepSeek-V2) --------------------
 * Device g holds the E / n_groups consecutive experts g*E/n_groups ...; E % n_groups = 0.
 *
 * moe_route_capacity: moe_route with device-level token dropping.  The affinity of an
 * assignment is the softmax of its token's logits over all E experts, read at the selected
 * expert (fp32; written to score [T,k]).  A device keeps at most `capacity` assignments; when
 * more arrive the ones with the lowest affinity are dropped, among equal affinities the higher
 * assignment id first.  A dropped assignment keeps its slot in topk_idx / topk_w (the weights
 * are not renormalised) and gets inv_perm = -1; counts [E], offsets [E+1] and perm cover the
 * kept assignments (perm past offsets[E] is not written).  Workspace:
 * moe_route_capacity_workspace_bytes(T, E, k). */
size_t moe_route_capacity_workspace_bytes(int T, int E, int k);
int moe_route_capacity(const float* logits, int T, int E, int k, int renorm, int n_groups,
                       int capacity, int32_t* topk_idx, float* topk_w, float* score,
                       int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                       void* workspace, size_t ws_bytes, void* stream);

/* Device-level balance loss.  With s[t,e] the affinity above, f_e = E/(k*T) * counts[e]
 * (counts = assignments per expert before any dropping, as moe_route writes them),
 * P_e = mean_t s[t,e]:  f'_g = mean of f_e over device g,  P'_g = sum of P_e over device g,
 * loss[0] = alpha * sum_g f'_g * P'_g; group_f [n_groups] = f', group_p [n_groups] = P'.
 * The sums over tokens run in a fixed order (reproducible).  workspace: moe_workspace_bytes.
 * moe_balance_loss_bwd ADDS d loss / d logits into d_logits [T,E], f' held constant:
 *   d_logits[t,c] += alpha/T * s[t,c] * (F_c - sum_e s[t,e] * F_e),  F_e = f' of e's device. */
int moe_balance_loss(const float* logits, const int32_t* counts, int T, int E, int k,
                     int n_groups, float alpha, float* loss, float* group_f, float* group_p,
                     void* workspace, size_t ws_bytes, void* stream);
int moe_balance_loss_bwd(const float* logits, const float* group_f, int T, int E, int n_groups,
                         float alpha, float* d_logits, void* stream);

/* Derivative of the gate weights w.r.t. the logits with the selection held constant.
 * d_logits [T,E] is fully written (zeros at unselected experts when renorm=1).
 * `logits` is only read when renorm=0 and may be NULL otherwise. */
int moe_route_bwd(const float* logits, const int32_t* topk_idx, const float* topk_w,
                  const float* d_topk_w, int T, int E, int k, int renorm,
                  float* d_logits, void* stream);

/* ---- dispatch / combine (Section 3.2: scatter and gather driven by the row map) -------
 * moe_dispatch: xp[inv_perm[t*k+j], :] = x[t, :] for every slot j, i.e. xp[r,:] =
 * x[perm[r] / k, :]  (* row_mul[t*k+j] if row_mul != NULL; with row_mul = topk_w this is
 * the backward of the weighted combine).  The rows of assignments that have a row (inv_perm >= 0) are
 * written; after moe_route that is every row below T*k; after moe_route_range or
 * moe_route_capacity the rows at or past offsets[E] are left untouched.
 * dt = MOE_F32 | MOE_BF16 | MOE_F8E4M3.  For MOE_F8E4M3 rows are 1-byte codes and the
 * per-token scale x_scale[t] is copied to xp_scale[row]; row_mul must then be NULL. */
int moe_dispatch(const void* x /*[T,d]*/, const float* x_scale /*[T] or NULL*/, moe_dtype dt,
                 const int32_t* inv_perm /*[T*k]*/, const float* row_mul /*[T*k] or NULL*/,
                 int T, int k, int d, void* xp /*[T*k,d]*/, float* xp_scale /*[T*k] or NULL*/,
                 void* stream);

/* moe_combine: y[t,:] = sum_j topk_w[t,j] * yp[inv_perm[t*k+j], :], summed in fp32 in
 * ascending j and rounded once to y_dt.  topk_w = NULL: unweighted (the backward of
 * dispatch).  For dt = MOE_F8E4M3 each row is dequantised with yp_scale[row] first. */
int moe_combine(const void* yp /*[T*k,d]*/, const float* yp_scale /*[T*k] or NULL*/, moe_dtype dt,
                const int32_t* inv_perm, const float* topk_w /*[T,k] or NULL*/,
                int T, int k, int d, void* y /*[T,d]*/, moe_dtype y_dt, void* stream);

/* d_topk_w[t,j] = <dy[t,:], yp[inv_perm[t*k+j], :]> in fp32 (derivative of the combine
 * w.r.t. the gate weights).  dy in dy_dt (MOE_F32|MOE_BF16); yp as in moe_combine. */
int moe_gate_grad(const void* dy /*[T,d]*/, moe_dtype dy_dt, const void* yp /*[T*k,d]*/,
                  const float* yp_scale, moe_dtype dt, const int32_t* inv_perm,
                  int T, int k, int d, float* d_topk_w /*[T,k]*/, void* stream);

/* ---- expert FFN (Section 4.1: FC1 GroupedGEMM -> SwiGLU -> FC2 GroupedGEMM) ----------
 * For expert e and its rows r in [offsets[e], offsets[e+1]):
 *   [G|U] = xp[r,:] * w1[e]^T,  A = G/(1+exp(-G)) * U,  yp[r,:] = A * w2[e]^T.
 * h_save [M,2f] receives [G|U] in the activation type (bf16 for MOE_BF16 and for the fp8
 * path, fp32 for MOE_F32); it is what the backward needs (the paper keeps the two FC1
 * outputs and recomputes the FC2 input).  fp32 accumulation throughout.
 * act_dt = w_dt = out_dt = MOE_F32 or MOE_BF16: plain path, scales must be NULL.
 * act_dt = w_dt = MOE_F8E4M3: xp holds codes with per-row scales xp_scale[M]; w1/w2 hold
 * codes with per-output-channel scales w1_scale [E,2f], w2_scale [E,d]; A is quantised per
 * row before FC2; out_dt = MOE_F8E4M3 writes yp as codes with per-row scales yp_scale[M],
 * out_dt = MOE_BF16 writes it unquantised.  a_codes_out [M,f] / a_scale_out [M] (both or neither)
 * receive the quantised FC2 input, which the backward dequantises and passes as a_override.
 * bf16 path: a_codes_out, if given (a_scale_out NULL), receives the FC2 input A [M,f] in bf16
 * instead of the workspace; passing it to moe_expert_ffn_bwd as a_override spares the backward
 * the second write of A (the paper recomputes the FC2 input, Section 4.1: keeping it trades
 * M*f*2 bytes for that write).  The plain paths touch no row >= offsets[E]; the fp8 path
 * requires offsets[E] = M. */
int moe_expert_ffn_fwd(const void* xp, const float* xp_scale, moe_dtype act_dt,
                       const int32_t* offsets /*[E+1], device*/,
                       const void* w1 /*[E,2f,d]*/, const float* w1_scale,
                       const void* w2 /*[E,d,f]*/, const float* w2_scale, moe_dtype w_dt,
                       int M, int d, int E, int f,
                       void* h_save /*[M,2f]*/, void* yp /*[M,d]*/, float* yp_scale,
                       moe_dtype out_dt, uint8_t* a_codes_out, float* a_scale_out,
                       void* workspace, size_t ws_bytes, void* stream);

/* Gradients of the expert FFN (Section 4.1, Fig. 8b: the FC2 backward takes the recomputed
 * FC2 input and the gradient of the FC2 output).  dt = MOE_F32 | MOE_BF16 for xp, h_save,
 * d_yp, w1, w2 and d_xp.  With A recomputed from h_save:
 *   dA = d_yp * w2[e];  d_w2[e] = d_yp_e^T * A_e;  (dG,dU) = SwiGLU'(G,U,dA);
 *   d_xp = [dG|dU] * w1[e];  d_w1[e] = [dG|dU]_e^T * xp_e.
 * a_override (or NULL): an [M,f] matrix in `dt` to use as A in d_w2 instead of the
 * recomputed one (the fp8 path passes the dequantised A that FC2 consumed).
 * grad_dt = MOE_F32 | MOE_BF16 is the type of d_w1 [E,2f,d] and d_w2 [E,d,f].
 * accumulate = 0: weight gradients are overwritten, experts without rows get exact zeros;
 * accumulate = 1: added into the existing values (fp32 main gradients kept across
 * micro-batches, Section 5). */
int moe_expert_ffn_bwd(const void* xp, const void* h_save, const void* d_yp,
                       const void* a_override, const int32_t* offsets,
                       const void* w1, const void* w2, moe_dtype dt,
                       int M, int d, int E, int f,
                       void* d_xp /*[M,d]*/, void* d_w1, void* d_w2, moe_dtype grad_dt,
                       int accumulate, void* workspace, size_t ws_bytes, void* stream);

/* ---- expert FFN in the Section 4.1 / 4.2 operator order (bf16 only) --------------------
 * The same layer with three changes of association, each the paper's: FC1 selects its input
 * rows from the token-order x through an index map inside the kernel's loads instead of
 * reading a dispatched copy (Section 4.2, "select rows of input data by the index mapping");
 * the gate weight is multiplied right after SwiGLU, so FC2 returns already weighted rows,
 * the combine is an unweighted sum (moe_combine with topk_w = NULL) and the FC2 output need
 * not be kept for the backward; the FC1 input rows are produced again in the backward
 * instead of being kept (Section 4.1, selective rematerialisation).  What stays resident
 * between forward and backward: x, h_save, the routing tables, row_token and row_w.
 *
 * moe_row_map: row_token[r] = perm[r] / k and row_w[r] = topk_w[perm[r]] for r < offsets[E];
 * token 0 and weight 0 for the remaining rows up to T*k. */
int moe_row_map(const int32_t* perm /*[T*k]*/, const float* topk_w /*[T,k]*/,
                const int32_t* offsets /*[E+1]*/, int E, int T, int k,
                int32_t* row_token /*[T*k]*/, float* row_w /*[T*k]*/, void* stream);

/* Bytes of workspace for the two calls below (0 on invalid sizes). */
size_t moe_expert_ffn_fused_workspace_bytes(int T, int k, int d, int f);

/* For row r of expert e: [G|U] = x[row_token[r],:] * w1[e]^T (written to h_save [T*k,2f]),
 * A' = row_w[r] * SwiGLU(G,U), ypw[r,:] = A' * w2[e]^T = row_w[r] * (the plain yp[r,:]).
 * x [T,d], w1, w2, h_save, ypw are bf16; T*d*2 bytes must stay below 4 GiB
 * (MOE_ERR_UNSUPPORTED otherwise).  Rows at or past offsets[E] are not written. */
int moe_expert_ffn_fused_fwd(const void* x, const int32_t* row_token, const float* row_w,
                             const int32_t* offsets, const void* w1, const void* w2,
                             int T, int k, int d, int E, int f, void* h_save, void* ypw /*[T*k,d]*/,
                             void* workspace, size_t ws_bytes, void* stream);

/* Backward of moe_expert_ffn_fused_fwd followed by the unweighted combine, from the
 * token-order output gradient dy [T,d]:  dY'[r] = dy[token of r];  dA' = dY' * w2[e];
 * d_topk_w[t,j] = <dA'[r,:], A[r,:]> for the row r of assignment (t,j), A recomputed from
 * h_save, 0 where the assignment has no row (summed in a fixed order: bit-reproducible);
 * d_w2[e] = dY'_e^T * A'_e.  The gate weight is linear in everything downstream of dA', so
 * it is applied once per row instead of once per element:
 *   (dG,dU) = SwiGLU'(G,U, dA');  d_xp[r,:] = [dG|dU] * w1[e]  -- WITHOUT the weight: the
 *   input gradient is dx[t,:] = sum_j topk_w[t,j] * d_xp[row(t,j),:], i.e. moe_combine WITH
 *   topk_w;  d_w1[e] = [dG|dU]_e^T * (row_w[r] * x[token of r]).
 * topk_w [T,k] and row_w [T*k] are the same weights by assignment and by row (moe_row_map).
 * grad_dt, accumulate: as in moe_expert_ffn_bwd. */
int moe_expert_ffn_fused_bwd(const void* x, const void* dy, const void* h_save,
                             const int32_t* inv_perm /*[T*k]*/, const float* topk_w,
                             const float* row_w, const int32_t* offsets,
                             const void* w1, const void* w2,
                             int T, int k, int d, int E, int f,
                             void* d_xp /*[T*k,d]*/, void* d_w1, void* d_w2, moe_dtype grad_dt,
                             int accumulate, float* d_topk_w /*[T,k]*/,
                             void* workspace, size_t ws_bytes, void* stream);

/* ---- E4M3 cast (Section 5 "Communication compression for FP8 training"; Section 7 "FP8
 * training": per-token 1 x h scales forward, per-channel scales in 128-token groups
 * backward) ---------------------------------------------------------------------------
 * MOE_Q_ROW: one scale per row.  MOE_Q_COLGROUP128: one scale per column inside each group
 * of 128 consecutive rows.  amax = max |v| of the group; amax = 0 gives scale 1 and codes 0;
 * otherwise scale = amax/448 and code = nearest-even e4m3 of clamp(fp32(v) * (448/amax)),
 * all in fp32.  src_dt / dst_dt = MOE_F32 | MOE_BF16. */
int moe_quant_fp8(const void* src, moe_dtype src_dt, int rows, int cols, moe_qmode mode,
                  uint8_t* codes /*[rows,cols]*/,
                  float* scales /*[rows] or [ceil(rows/128),cols]*/, void* stream);
int moe_dequant_fp8(const uint8_t* codes, const float* scales, int rows, int cols,
                    moe_qmode mode, void* dst, moe_dtype dst_dt, void* stream);

/* Batched transpose, dst[b][c][r] = src[b][r][c] for b < batch (src [batch,rows,cols], dst
 * [batch,cols,rows], dense, element type dt; MOE_F8E4M3 = bytes).  A set-up helper, not a step of
 * the layer: the FP8 backward (Section 7 "FP8 training", per-channel quantisation for the backward
 * pass) needs the weights cast along their other axis, i.e. moe_quant_fp8 over W1[e]^T and W2[e]^T.
 * src and dst must not overlap.  batch <= 65535, rows <= 64 * 65535. */
int moe_transpose(const void* src, moe_dtype dt, int batch, int rows, int cols, void* dst,
                  void* stream);

/* ---- FP8 backward GEMMs of the expert FFN (Section 7 "FP8 training": per-token quantisation
 * in the forward orientation, per-channel quantisation within 128-token groups for the
 * backward pass; Section 5: E4M3 for all tensors) -------------------------------------------
 * The four backward GEMMs on e4m3 operands with fp32 accumulation, straight-through casts:
 *   dA    = Qrow(d_yp) * w2t[e]^T      d_yp cast per token; w2t[e] = W2[e]^T as [f,d] codes with one
 *                                      scale per row (per input channel of W2: the second,
 *                                      transposed-orientation quantisation of the weights)
 *   dH    = SwiGLU'(h_save, dA)        bf16
 *   d_xp  = Qrow(dH) * w1t[e]^T        w1t[e] = W1[e]^T as [d,2f] codes, one scale per row
 *   d_w2[e] = Qg(d_yp_e)^T * Qg(a_deq_e),   d_w1[e] = Qg(dH_e)^T * Qg(xp_deq_e)
 * Qg is moe_quant_fp8_tgroup below.  Every buffer is device memory owned by the caller; the
 * intermediates are outputs too (they are what a parity check compares stage by stage) and
 * none may alias another.  Requires offsets[E] = M, d and f multiples of 16, ldt >=
 * moe_tgroup_tokens(M, E) and a multiple of 128.  Only enqueues work on `stream`. */
typedef struct moe_ffn_bwd_fp8_args {
  /* inputs */
  const void* d_yp;            /* [M,d]  bf16: gradient of the FC2 output (already gate-weighted) */
  const void* h_save;          /* [M,2f] bf16: [G|U] kept by the forward */
  const void* xp_deq;          /* [M,d]  bf16: the dispatched activations FC1 consumed, dequantised (or xp_codes below) */
  const void* a_deq;           /* [M,f]  bf16: the FC2 input the forward consumed, dequantised (or a_codes below) */
  const int32_t* offsets;      /* [E+1] */
  const uint8_t* w1t;          /* [E,d,2f] e4m3 codes of W1[e]^T */
  const float* w1t_scale;      /* [E,d] */
  const uint8_t* w2t;          /* [E,f,d] e4m3 codes of W2[e]^T */
  const float* w2t_scale;      /* [E,f] */
  int M, d, E, f;
  /* results */
  void* d_xp;                  /* [M,d] bf16 */
  void* d_w1;                  /* [E,2f,d] grad_dt */
  void* d_w2;                  /* [E,d,f]  grad_dt */
  moe_dtype grad_dt;           /* MOE_F32 | MOE_BF16 */
  int accumulate;              /* as in moe_expert_ffn_bwd */
  /* intermediates (all written) */
  uint8_t* dy_codes; float* dy_scale;     /* [M,d], [M]: Qrow(d_yp) */
  void* dh;                               /* [M,2f] bf16 */
  uint8_t* dh_codes; float* dh_scale;     /* [M,2f], [M]: Qrow(dH) */
  int32_t* pad_offsets;                   /* [E+1] */
  long ldt;                               /* token stride of the transposed code matrices */
  uint8_t* dy_t; uint8_t* dy_e8m0;        /* [d,ldt],  [ldt/128,d]  */
  uint8_t* dh_t; uint8_t* dh_e8m0;        /* [2f,ldt], [ldt/128,2f] */
  uint8_t* a_t;  uint8_t* a_e8m0;         /* [f,ldt],  [ldt/128,f]  */
  uint8_t* x_t;  uint8_t* x_e8m0;         /* [d,ldt],  [ldt/128,d]  */
  void* splitk_ws;                        /* MOE_SPLITK_WS_BYTES of scratch, or NULL: lets the d_xp GEMM split the
                                             tiles of a partly filled last round along K (faster, same result up
                                             to fp32 summation order) */
  /* optional inputs: the e4m3 codes and per-row scales the forward consumed.  When xp_codes
   * (a_codes) is given, the weight-gradient operand is cast from code * scale (one fp32
   * rounding) and xp_deq (a_deq) is not read and may be NULL. */
  const uint8_t* xp_codes; const float* xp_scale;   /* [M,d], [M] */
  const uint8_t* a_codes;  const float* a_scale;    /* [M,f], [M] */
} moe_ffn_bwd_fp8_args;
#define MOE_SPLITK_WS_BYTES ((size_t)256 * 256 * 256 * 4)
int moe_expert_ffn_bwd_fp8(const moe_ffn_bwd_fp8_args* args, void* stream);

/* Backward-orientation cast for the weight-gradient GEMMs (Section 7: per-channel quantisation
 * within 128-token groups).  src [rows,cols] holds dispatched rows in expert order
 * (offsets [E+1], offsets[E] = rows).  Groups are 128 consecutive rows inside one expert's
 * segment (a group never spans two experts; a segment's last group may be short).  The
 * paper gives no scale rule; here a group scale is the power of two 2^k with k the smallest
 * integer such that amax * 2^-k <= 448 (k = 0 when amax = 0, clamped to [-126,127]), stored
 * as the E8M0 byte k + 127, the form block-scaled matrix instructions apply inside the
 * contraction; code = nearest-even e4m3 of clamp(v * 2^-k, +-448).  Codes are written
 * transposed, codes_t[c*ldt + pad_offsets[e] + (r - offsets[e])], each expert's columns
 * padded with zero codes to a multiple of 128 (pad_offsets [E+1] is written by this call;
 * columns at or past pad_offsets[E] are not touched).  e8m0[(pad_offsets[e]/128 + j)*cols + c]
 * is the scale of group j of expert e, column c.  ldt >= moe_tgroup_tokens(rows, E), ldt % 128
 * = 0, cols % 16 = 0.  src_dt = MOE_F32 | MOE_BF16. */
size_t moe_tgroup_tokens(int rows, int E);
int moe_quant_fp8_tgroup(const void* src, moe_dtype src_dt, int rows, int cols,
                         const int32_t* offsets, int E, int32_t* pad_offsets,
                         uint8_t* codes_t, long ldt, uint8_t* e8m0, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_HIP_MOE_H */
