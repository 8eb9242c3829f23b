"""One MoE FFN layer on one GPU: buffers allocated once, then forward and backward as a fixed
sequence of C-ABI calls (router -> route -> dispatch -> expert FFN -> combine, and the reverse).

This is plumbing around the library: it owns device memory (torch tensors) and the call order,
and does no arithmetic of its own.  Operator order follows Section 4.1 of the paper (Fig. 8a/8b).
"""
from __future__ import annotations

import torch

from . import binding as B


class MoELayer:
    def __init__(self, T: int, d: int, E: int, k: int, f: int, dtype=torch.bfloat16, renorm: int = 1,
                 fp8: bool = False, grad_dtype=torch.float32, device="cuda:0", expert_range=None, capacity=None,
                 balance=None, fused: bool = False, keep_a: bool = False):
        """fused = True: the Section 4.1 / 4.2 operator order (bf16): FC1 selects its rows from x through the index
        map, the gate weight is applied right after SwiGLU, the combine is unweighted, the gate gradient comes out
        of the dgrad2 epilogue; neither the dispatched input nor the FC2 output is kept for the backward.

        keep_a = True (bf16, plain order): the FC2 input A is kept from the forward (M*f*2 bytes) and handed to the
        backward, which then does not write it again (the paper recomputes it, Section 4.1; this trades memory for time).

        expert_range = (e_lo, e_hi): this GPU's expert-parallel share (Section 3.2): x holds the all-gathered
        tokens, only rows routed to experts e_lo..e_hi-1 are dispatched, w1/w2 and their gradients hold those
        experts only, and y / dx are the partial sums over them.  Row buffers keep the bound T*k."""
        self.T, self.d, self.E, self.k, self.f = T, d, E, k, f
        self.M = T * k
        self.expert_range = expert_range
        # load balance (Section 3.2): capacity = (devices, rows per device) drops the lowest-affinity assignments of
        # an overloaded device; balance = (devices, alpha) adds the device-level auxiliary loss and its gradient
        self.capacity, self.balance = capacity, balance
        assert not (capacity is not None and (fp8 or expert_range is not None))
        self.E_local = E if expert_range is None else expert_range[1] - expert_range[0]
        assert not (fp8 and expert_range is not None), "the fp8 path needs offsets[E] = M"
        assert not (fp8 and balance is not None), "the fp8 path has no balance loss"
        self.dtype, self.renorm, self.fp8, self.device = dtype, renorm, fp8, device
        M = self.M
        dev = dict(device=device)
        i32 = dict(dtype=torch.int32, **dev)
        f32 = dict(dtype=torch.float32, **dev)
        act = dict(dtype=dtype, **dev)
        self.logits = torch.empty((T, E), **f32)
        self.topk_idx = torch.empty((T, k), **i32)
        self.topk_w = torch.empty((T, k), **f32)
        self.counts = torch.empty((E,), **i32)
        self.offsets = torch.empty((self.E_local + 1,), **i32)
        self.perm = torch.empty((M,), **i32)
        self.inv_perm = torch.empty((M,), **i32)
        self.h_save = torch.empty((M, 2 * f), **act)
        self.y = torch.empty((T, d), **act)
        self.d_topk_w = torch.empty((T, k), **f32)
        self.d_xp = torch.empty((M, d), **act)
        self.dx = torch.empty((T, d), **act)
        self.d_logits = torch.empty((T, E), **f32)
        self.d_w_r = torch.empty((E, d), **f32)
        self.d_w1 = torch.empty((self.E_local, 2 * f, d), dtype=grad_dtype, **dev)
        self.d_w2 = torch.empty((self.E_local, d, f), dtype=grad_dtype, **dev)
        if fp8:
            u8 = dict(dtype=torch.uint8, **dev)
            self.x_codes = torch.empty((T, d), **u8)
            self.x_scale = torch.empty((T,), **f32)
            self.xp = torch.empty((M, d), **u8)
            self.xp_scale = torch.empty((M,), **f32)
            self.yp = torch.empty((M, d), **u8)
            self.yp_scale = torch.empty((M,), **f32)
            self.xp_deq = torch.empty((M, d), **act)
            self.a_codes = torch.empty((M, f), **u8)
            self.a_scale = torch.empty((M,), **f32)
            self.a_deq = torch.empty((M, f), **act)
            self.w1_codes = self.w1_scale = self.w2_codes = self.w2_scale = None
            self.dy_codes = torch.empty((T, d), **u8)
            self.dy_scale = torch.empty(((T + 127) // 128, d), **f32)
            self.dy_deq = torch.empty((T, d), **act)
        elif fused:
            self.yp = torch.empty((M, d), **act)        # transient: FC2 output -> combine; not needed by the backward
        else:
            self.xp = torch.empty((M, d), **act)
            self.yp = torch.empty((M, d), **act)
        if not fused:
            self.d_yp = torch.empty((M, d), **act)
        if capacity is not None:
            self.score = torch.empty((T, k), **f32)
            self.route_ws = torch.empty((B.moe_route_capacity_workspace_bytes(T, E, k),), dtype=torch.uint8, **dev)
        if balance is not None:
            self.aux_loss = torch.zeros((1,), **f32)
            self.group_f = torch.empty((balance[0],), **f32)
            self.group_p = torch.empty((balance[0],), **f32)
        self.a_keep = None
        if keep_a:
            assert not fp8 and not fused and dtype == torch.bfloat16, "keep_a exists for the plain bf16 order"
            self.a_keep = torch.empty((M, f), **act)
        self.fused = fused
        if fused:
            assert not fp8 and dtype == torch.bfloat16, "the fused operator order exists for bf16"
            self.row_token = torch.empty((M,), **i32)
            self.row_w = torch.empty((M,), **f32)
            self.fused_ws = torch.empty((B.moe_expert_ffn_fused_workspace_bytes(T, k, d, f),), dtype=torch.uint8, **dev)
        self.timers = None      # set to a dict to collect (start, end) event pairs per call name
        self.timer_filter = None    # a set of call names: only these are bracketed (an event record between two calls
                                    # costs about 10 us of idle GPU, so timing every call slows the step by 0.6 %)
        code = B.F8E4M3 if fp8 else B.dtype_code(dtype)
        nbytes = B.moe_workspace_bytes(T, d, E, k, f, code)
        self.workspace = torch.empty((max(nbytes, 256),), dtype=torch.uint8, **dev)

    def _call(self, name, fn, *args):
        """Run one C-ABI call; with timers enabled, bracket it with events on the current stream."""
        if self.timers is None or (self.timer_filter is not None and name not in self.timer_filter):
            fn(*args)
            return
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        e0.record()
        fn(*args)
        e1.record()
        self.timers.setdefault(name, []).append((e0, e1))

    def timer_ms(self) -> dict:
        """Total milliseconds per call name over everything recorded so far (synchronises)."""
        torch.cuda.synchronize()
        return {k: sum(a.elapsed_time(b) for a, b in v) for k, v in (self.timers or {}).items()}

    def set_fp8_weights(self, w1, w2):
        """Per-output-channel E4M3 copies of the expert weights (kept across steps: the paper stores
        parameters in FP8, Section 7, so this cast is outside the timed loop)."""
        E, two_f, d = w1.shape
        f = two_f // 2
        dev = dict(device=w1.device)
        self.w1_codes = torch.empty((E, two_f, d), dtype=torch.uint8, **dev)
        self.w1_scale = torch.empty((E, two_f), dtype=torch.float32, **dev)
        self.w2_codes = torch.empty((E, d, f), dtype=torch.uint8, **dev)
        self.w2_scale = torch.empty((E, d), dtype=torch.float32, **dev)
        B.moe_quant_fp8(w1.view(E * two_f, d), B.Q_ROW, self.w1_codes.view(E * two_f, d), self.w1_scale.view(-1))
        B.moe_quant_fp8(w2.view(E * d, f), B.Q_ROW, self.w2_codes.view(E * d, f), self.w2_scale.view(-1))

    def set_fp8_backward_weights(self, w1, w2):
        """Second, transposed-orientation E4M3 copies of the weights for the dgrad GEMMs (one scale per input
        channel), also kept across steps, and the buffers the FP8 backward writes.  Set-up, not a step of the
        timed path."""
        E, two_f, d = w1.shape
        f = two_f // 2
        M = self.M
        dev = dict(device=w1.device)
        u8 = dict(dtype=torch.uint8, **dev)
        f32 = dict(dtype=torch.float32, **dev)
        w1t = torch.empty((E, d, two_f), dtype=w1.dtype, **dev)
        w2t = torch.empty((E, f, d), dtype=w2.dtype, **dev)
        B.moe_transpose(w1, w1t)
        B.moe_transpose(w2, w2t)
        self.w1t_codes = torch.empty((E, d, two_f), **u8)
        self.w1t_scale = torch.empty((E, d), **f32)
        self.w2t_codes = torch.empty((E, f, d), **u8)
        self.w2t_scale = torch.empty((E, f), **f32)
        B.moe_quant_fp8(w1t.view(E * d, two_f), B.Q_ROW, self.w1t_codes.view(E * d, two_f), self.w1t_scale.view(-1))
        B.moe_quant_fp8(w2t.view(E * f, d), B.Q_ROW, self.w2t_codes.view(E * f, d), self.w2t_scale.view(-1))
        del w1t, w2t
        ldt = B.moe_tgroup_tokens(M, E)
        G = ldt // 128
        self.bwd8 = dict(
            dy_codes=torch.empty((M, d), **u8), dy_scale=torch.empty((M,), **f32),
            dh=torch.empty((M, two_f), dtype=torch.bfloat16, **dev),
            dh_codes=torch.empty((M, two_f), **u8), dh_scale=torch.empty((M,), **f32),
            pad_offsets=torch.empty((E + 1,), dtype=torch.int32, **dev),
            dy_t=torch.zeros((d, ldt), **u8), dy_e8m0=torch.zeros((G, d), **u8),
            dh_t=torch.zeros((two_f, ldt), **u8), dh_e8m0=torch.zeros((G, two_f), **u8),
            a_t=torch.zeros((f, ldt), **u8), a_e8m0=torch.zeros((G, f), **u8),
            x_t=torch.zeros((d, ldt), **u8), x_e8m0=torch.zeros((G, d), **u8),
            splitk_ws=torch.empty((B.SPLITK_WS_BYTES,), **u8))

    def backward_fp8_gemm(self, x, w_r, dy, with_router: bool = True):
        """Backward of forward_fp8 with the four expert GEMMs on E4M3 operands (Section 7: per-channel
        quantisation within 128-token groups for the backward pass); everything else as in backward_fp8."""
        c = self._call
        c("quant_dy", B.moe_quant_fp8, dy, B.Q_COLGROUP128, self.dy_codes, self.dy_scale)
        c("dequant_dy", B.moe_dequant_fp8, self.dy_codes, self.dy_scale, B.Q_COLGROUP128, self.dy_deq)
        c("gate_grad", B.moe_gate_grad, self.dy_deq, self.yp, self.yp_scale, self.inv_perm, self.k, self.d_topk_w)
        c("dispatch_bwd_of_combine", B.moe_dispatch, self.dy_deq, None, self.inv_perm, self.topk_w.view(-1), self.k,
          self.d_yp, None)
        # the weight-gradient casts read the forward's codes and per-row scales directly (no dequantised copies)
        c("expert_ffn_bwd", B.moe_expert_ffn_bwd_fp8, self.d_yp, self.h_save, (self.xp, self.xp_scale),
          (self.a_codes, self.a_scale), self.offsets, self.w1t_codes, self.w1t_scale, self.w2t_codes, self.w2t_scale, self.d_xp, self.d_w1, self.d_w2, 0, self.bwd8)
        c("combine_bwd_of_dispatch", B.moe_combine, self.d_xp, None, self.inv_perm, None, self.k, self.dx)
        c("route_bwd", B.moe_route_bwd, self.logits, self.topk_idx, self.topk_w, self.d_topk_w, self.E,
          self.renorm, self.d_logits)
        if with_router:
            c("router_bwd", B.moe_router_bwd, x, w_r, self.d_logits, self.d_w_r, self.dx, self.workspace)
        return self.dx

    def forward_fp8(self, x, w_r, bias, logits=None):
        """Forward with E4M3 dispatched activations and returned expert outputs (per-token scales), e4m3 expert
        GEMMs, gate weight applied after FC2 on the dequantised outputs."""
        c = self._call
        if logits is None:
            c("router_fwd", B.moe_router_fwd, x, w_r, bias, self.logits)
        else:
            self.logits.copy_(logits)
        c("route", B.moe_route, self.logits, self.k, self.renorm, self.topk_idx, self.topk_w, self.counts,
          self.offsets, self.perm, self.inv_perm, self.workspace)
        c("quant_x", B.moe_quant_fp8, x, B.Q_ROW, self.x_codes, self.x_scale)
        c("dispatch", B.moe_dispatch, self.x_codes, self.x_scale, self.inv_perm, None, self.k, self.xp, self.xp_scale)
        c("expert_ffn_fwd", B.moe_expert_ffn_fwd, self.xp, self.xp_scale, self.offsets, self.w1_codes, self.w1_scale,
          self.w2_codes, self.w2_scale, self.h_save, self.yp, self.yp_scale, self.workspace, self.a_codes,
          self.a_scale)
        c("combine", B.moe_combine, self.yp, self.yp_scale, self.inv_perm, self.topk_w, self.k, self.y)
        return self.y

    def backward_fp8(self, x, w_r, w1, w2, dy, with_router: bool = True):
        """Straight-through backward of forward_fp8: dy cast per channel in 128-token groups, bf16 GEMMs on the
        master weights, the saved H and the dequantised xp / A that the forward GEMMs consumed."""
        c = self._call
        c("quant_dy", B.moe_quant_fp8, dy, B.Q_COLGROUP128, self.dy_codes, self.dy_scale)
        c("dequant_dy", B.moe_dequant_fp8, self.dy_codes, self.dy_scale, B.Q_COLGROUP128, self.dy_deq)
        c("gate_grad", B.moe_gate_grad, self.dy_deq, self.yp, self.yp_scale, self.inv_perm, self.k, self.d_topk_w)
        c("dispatch_bwd_of_combine", B.moe_dispatch, self.dy_deq, None, self.inv_perm, self.topk_w.view(-1), self.k,
          self.d_yp, None)
        c("dequant_xp", B.moe_dequant_fp8, self.xp, self.xp_scale, B.Q_ROW, self.xp_deq)
        c("dequant_a", B.moe_dequant_fp8, self.a_codes, self.a_scale, B.Q_ROW, self.a_deq)
        c("expert_ffn_bwd", B.moe_expert_ffn_bwd, self.xp_deq, self.h_save, self.d_yp, self.a_deq, self.offsets, w1,
          w2, self.d_xp, self.d_w1, self.d_w2, 0, self.workspace)
        c("combine_bwd_of_dispatch", B.moe_combine, self.d_xp, None, self.inv_perm, None, self.k, self.dx)
        c("route_bwd", B.moe_route_bwd, self.logits, self.topk_idx, self.topk_w, self.d_topk_w, self.E,
          self.renorm, self.d_logits)
        if with_router:
            c("router_bwd", B.moe_router_bwd, x, w_r, self.d_logits, self.d_w_r, self.dx, self.workspace)
        return self.dx

    # ---- forward: Fig. 8a ------------------------------------------------------------------
    def forward(self, x, w_r, bias, w1, w2, logits=None):
        """x [T,d]; w_r [E,d]; bias [E] fp32 or None; w1 [E,2f,d]; w2 [E,d,f].  `logits` overrides the
        router matmul (used by the parity tests to feed both sides the same fp32 bits)."""
        c = self._call
        if logits is None:
            c("router_fwd", B.moe_router_fwd, x, w_r, bias, self.logits)
        else:
            self.logits.copy_(logits)
        def balance_loss():
            # the loss counts every assignment, dropped or not, local or not: `counts` of moe_route / moe_route_range
            c("balance_loss", B.moe_balance_loss, self.logits, self.counts, self.k, self.balance[0], self.balance[1],
              self.aux_loss, self.group_f, self.group_p, self.workspace)

        if self.capacity is not None:
            if self.balance is not None:
                c("route", B.moe_route, self.logits, self.k, self.renorm, self.topk_idx, self.topk_w, self.counts,
                  self.offsets, self.perm, self.inv_perm, self.workspace)
                balance_loss()
            c("route", B.moe_route_capacity, self.logits, self.k, self.renorm, self.capacity[0], self.capacity[1],
              self.topk_idx, self.topk_w, self.score, self.counts, self.offsets, self.perm, self.inv_perm, self.route_ws)
        else:
            if self.expert_range is None:
                c("route", B.moe_route, self.logits, self.k, self.renorm, self.topk_idx, self.topk_w, self.counts,
                  self.offsets, self.perm, self.inv_perm, self.workspace)
            else:
                c("route", B.moe_route_range, self.logits, self.k, self.renorm, self.expert_range[0], self.expert_range[1],
                  self.topk_idx, self.topk_w, self.counts, self.offsets, self.perm, self.inv_perm, self.workspace)
            if self.balance is not None:
                balance_loss()
        if self.fused:
            c("row_map", B.moe_row_map, self.perm, self.topk_w, self.offsets, self.row_token, self.row_w)
            c("expert_ffn_fwd", B.moe_expert_ffn_fused_fwd, x, self.row_token, self.row_w, self.offsets, w1, w2, self.k,
              self.h_save, self.yp, self.fused_ws)
            c("combine", B.moe_combine, self.yp, None, self.inv_perm, None, self.k, self.y)
            return self.y
        c("dispatch", B.moe_dispatch, x, None, self.inv_perm, None, self.k, self.xp, None)
        c("expert_ffn_fwd", B.moe_expert_ffn_fwd, self.xp, None, self.offsets, w1, None, w2, None, self.h_save,
          self.yp, None, self.workspace, self.a_keep, None)
        c("combine", B.moe_combine, self.yp, None, self.inv_perm, self.topk_w, self.k, self.y)
        return self.y

    # ---- backward: Fig. 8b -----------------------------------------------------------------
    def backward(self, x, w_r, w1, w2, dy, with_router: bool = True):
        c = self._call
        if self.fused:
            c("expert_ffn_bwd", B.moe_expert_ffn_fused_bwd, x, dy, self.h_save, self.inv_perm, self.topk_w, self.row_w,
              self.offsets, w1, w2, self.k, self.d_xp, self.d_w1, self.d_w2, 0, self.d_topk_w, self.fused_ws)
        else:
            c("gate_grad", B.moe_gate_grad, dy, self.yp, None, self.inv_perm, self.k, self.d_topk_w)
            c("dispatch_bwd_of_combine", B.moe_dispatch, dy, None, self.inv_perm, self.topk_w.view(-1), self.k,
              self.d_yp, None)
            c("expert_ffn_bwd", B.moe_expert_ffn_bwd, self.xp, self.h_save, self.d_yp, self.a_keep, self.offsets, w1, w2,
              self.d_xp, self.d_w1, self.d_w2, 0, self.workspace)
        # fused order: d_xp comes without the gate weight, which this combine applies once per row
        c("combine_bwd_of_dispatch", B.moe_combine, self.d_xp, None, self.inv_perm, self.topk_w if self.fused else None,
          self.k, self.dx)
        c("route_bwd", B.moe_route_bwd, self.logits, self.topk_idx, self.topk_w, self.d_topk_w, self.E,
          self.renorm, self.d_logits)
        if self.balance is not None:
            c("balance_loss_bwd", B.moe_balance_loss_bwd, self.logits, self.group_f, self.balance[0], self.balance[1],
              self.d_logits)
        if with_router:
            c("router_bwd", B.moe_router_bwd, x, w_r, self.d_logits, self.d_w_r, self.dx, self.workspace)
        return self.dx
