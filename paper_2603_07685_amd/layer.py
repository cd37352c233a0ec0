"""One MoE expert layer as a fixed sequence of C-ABI calls on preallocated device buffers.

No arithmetic happens here: this module only allocates torch tensors as device
memory and issues the library calls in the order of the paper's four stages
(Sec. 2.1.1) and of the backward pass with the weight-/data-gradient split
(Sec. 4.2.3).  It is what the tests, the smoke check and the benchmark drive.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import workloads as wl


def host_inputs(cfg: wl.MoEConfig, shared_f: int | None = None) -> dict:
    """Seeded host inputs (fp32 arrays whose values are bf16-representable) for the small configs."""
    sf = cfg.shared_f if shared_f is None else shared_f
    s = cfg.seed
    _, _, logits = wl.router_logits(cfg.T, cfg.h, cfg.E_router, cfg.std, s)
    d = {
        "logits": logits,
        "X": wl.gaussian_bf16((cfg.T, cfg.h), cfg.std, s, 1),
        "W1": wl.gaussian_bf16((cfg.E, 2 * cfg.f, cfg.h), cfg.std, s, 2),
        "W2": wl.gaussian_bf16((cfg.E, cfg.h, cfg.f), cfg.std, s, 3),
        "dY": wl.gaussian_bf16((cfg.T, cfg.h), 1.0, s, 4),
    }
    if sf:
        d["Ws1"] = wl.gaussian_bf16((2 * sf, cfg.h), cfg.std, s, 5)
        d["Ws2"] = wl.gaussian_bf16((cfg.h, sf), cfg.std, s, 6)
    return d


def _dev_bf16(x: np.ndarray) -> torch.Tensor:
    bits = wl.f32_to_bf16_bits(np.ascontiguousarray(x, np.float32))
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


class LayerState:
    """Device buffers of one layer + the forward / backward call sequences."""

    def __init__(self, cfg: wl.MoEConfig, hin: dict | None = None, shared_f: int | None = None,
                 variant: str | None = None, wgrad_f32: bool = False, eq2: bool = False,
                 fused_quant: bool | None = None, epilogue_quant: bool | None = None, f32: bool = False,
                 fp8_wgrad: bool | None = None, gather: bool = False):
        self.cfg = cfg
        # bf16 only: the permute's row move fused into the GEMMs that read the permuted tensor (Sec. 4.3.3): fc1 and its
        # weight gradient fetch the rows of X through the row map, and under eq. (2), where the combine's backward is a
        # plain copy, fc2's two gradients fetch the rows of dY the same way; Xp (and then dO) are never stored
        self.gather = bool(gather)
        assert not self.gather or not (cfg.fp8 or cfg.mx or f32), "the gathered GEMMs are bf16 kernels"
        self.eq2 = bool(eq2)  # memory-efficient permutation (Sec. 4.1.2): weights applied before fc2
        self.fused_quant = None if fused_quant is None else bool(fused_quant)   # (resolved below, once fp8_wgrad is known)
        # blockwise fp8 (default there): the SwiGLU / SwiGLU-backward epilogues also emit the 1x128 codes of their
        # output, the next GEMM's operand (Sec. 5.4.2); off = stand-alone quantiser launches
        # (MXFP8: the 1x32 codes and the 32x1 copy for the weight gradients; row counts are on the 128-row grid there)
        self.epilogue_quant = bool(cfg.fp8 or cfg.mx) if epilogue_quant is None else bool(epilogue_quant)
        assert not self.epilogue_quant or cfg.fp8 or cfg.mx, "epilogue quantisation belongs to the one-byte recipes"
        # blockwise fp8 (default there): the weight gradients also run on E4M3 codes, quantised 128x1 down the token
        # dimension inside each expert's 128-aligned row range (Sec. 5.3.2, 5.4.1); off = weight gradients from the
        # bf16 tensors.  (MXFP8 always runs them on its 32x1 copies.)
        self.fp8_wgrad = (bool(cfg.fp8) and not cfg.mx) if fp8_wgrad is None else bool(fp8_wgrad)
        assert not self.fp8_wgrad or (cfg.fp8 and not cfg.mx and cfg.align % 128 == 0), \
            "blockwise fp8 weight gradients need the blockwise config with experts padded to 128 rows"
        # one-byte recipes whose weight gradients run on one-byte operands too: the permuted tokens and the combine's
        # backward are quantised straight from X / dY through the row map, in both directions, padding included
        # (Sec. 5.4.1, 5.4.2); Xp and dO are never stored in bf16
        if self.fused_quant is None:
            self.fused_quant = bool(cfg.mx) or self.fp8_wgrad
        assert not self.fused_quant or cfg.mx or self.fp8_wgrad, \
            "fused quantisation needs a recipe that keeps no bf16 copy for the weight gradients"
        T, k, E, h, f = cfg.T, cfg.k, cfg.E, cfg.h, cfg.f
        self.sf = sf = cfg.shared_f if shared_f is None else shared_f
        self.align = cfg.align
        Rcap = T * k + E * (cfg.align - 1)
        if cfg.mx or self.fp8_wgrad:  # the column-wise quantiser and the weight-gradient GEMM walk the rows in steps of 128
            Rcap = (Rcap + 127) // 128 * 128
        self.Rcap = Rcap
        self.ctx = B.Context(T, k, max(E, cfg.E_router), h, max(f, sf))
        # all-fp32 run (small layers, host inputs): every tensor and every call in fp32, for parity at the 1e-5 level
        self.f32 = bool(f32)
        assert not self.f32 or (hin is not None and not cfg.fp8 and not cfg.mx and not self.eq2), \
            "the all-fp32 run takes host inputs, eq. (1), no fp8"
        self.dt = B.F32 if self.f32 else B.BF16
        i32, f32 = torch.int32, torch.float32
        bf = f32 if self.f32 else torch.bfloat16   # storage type of activations, weights and gradients
        if self.f32:
            wgrad_f32 = True
        dev = "cuda"
        s = cfg.seed
        if hin is not None:
            put = (lambda x: torch.from_numpy(np.ascontiguousarray(x, np.float32)).cuda()) if self.f32 else _dev_bf16
            self.logits = torch.from_numpy(hin["logits"]).cuda()
            self.X, self.W1, self.W2, self.dY = (put(hin[n]) for n in ("X", "W1", "W2", "dY"))
            if sf:
                self.Ws1, self.Ws2 = put(hin["Ws1"]), put(hin["Ws2"])
        else:  # large configs: draw on the device
            g = torch.Generator(device=dev)
            g.manual_seed(s)
            self.logits = torch.empty((T, cfg.E_router), dtype=f32, device=dev).normal_(0.0, 0.03, generator=g)
            self.X = wl.device_gaussian_bf16((T, h), cfg.std, s, 1)
            self.W1 = wl.device_gaussian_bf16((E, 2 * f, h), cfg.std, s, 2)
            self.W2 = wl.device_gaussian_bf16((E, h, f), cfg.std, s, 3)
            self.dY = wl.device_gaussian_bf16((T, h), 1.0, s, 4)
            if sf:
                self.Ws1 = wl.device_gaussian_bf16((2 * sf, h), cfg.std, s, 5)
                self.Ws2 = wl.device_gaussian_bf16((h, sf), cfg.std, s, 6)
        b = wl.expert_bias(cfg)
        self.expert_bias = None if b is None else torch.from_numpy(b).cuda()
        # forced routing map (None: the router's own top-k drives the permute)
        forced = wl.routing_map(cfg, variant)
        self.forced_idx = None if forced is None else torch.from_numpy(forced).cuda()

        self.topk_idx = torch.empty((T, k), dtype=i32, device=dev)
        self.topk_prob = torch.empty((T, k), dtype=f32, device=dev)
        self.route_counts = torch.empty(cfg.E_router, dtype=i32, device=dev)
        self.row_of = torch.empty((T, k), dtype=i32, device=dev)
        self.src_of = torch.empty(Rcap, dtype=i32, device=dev)
        self.offsets = torch.empty(E + 1, dtype=i32, device=dev)
        self.counts = torch.empty(E, dtype=i32, device=dev)
        self.Xp = None if (self.fused_quant or self.gather) else torch.empty((Rcap, h), dtype=bf, device=dev)
        self.Z = torch.empty((Rcap, 2 * f), dtype=bf, device=dev)
        self.A = torch.empty((Rcap, f), dtype=bf, device=dev)
        self.O = torch.empty((Rcap, h), dtype=bf, device=dev)
        self.Y = torch.empty((T, h), dtype=bf, device=dev)
        # backward
        wdt = f32 if wgrad_f32 else bf
        self.wgrad_dt = B.F32 if wgrad_f32 else B.BF16
        self.dO = None if (self.fused_quant or (self.gather and self.eq2)) else torch.empty((Rcap, h), dtype=bf, device=dev)
        self.dprob = torch.empty((T, k), dtype=f32, device=dev)
        self.dZ = torch.empty((Rcap, 2 * f), dtype=bf, device=dev)
        self.dXp = torch.empty((Rcap, h), dtype=bf, device=dev)
        self.dX = torch.empty((T, h), dtype=bf, device=dev)
        self.dW1 = torch.empty((E, 2 * f, h), dtype=wdt, device=dev)
        self.dW2 = torch.empty((E, h, f), dtype=wdt, device=dev)
        if self.eq2:
            self.row_prob = torch.empty(Rcap, dtype=f32, device=dev)
            self.dprob_parts = 2 * ((f + 255) // 256)   # two partial sums per 256-column tile of the fc2 data gradient
            self.dprob_part = torch.empty((Rcap, self.dprob_parts), dtype=f32, device=dev)
        self.mx = bool(cfg.mx)                    # MXFP8: 1x32 blocks, E8M0 scales, scaling by the matrix instruction
        self.fp8 = bool(cfg.fp8) or self.mx       # one-byte operands in the forward / data-gradient GEMMs
        self.f8dt = B.MXFP8_E4M3 if self.mx else B.FP8_E4M3
        if self.fp8:
            u8 = torch.uint8
            mx = self.mx

            def codes(rows, cols):   # E4M3 codes + scales of a row-indexed tensor (1x128 fp32 / 1x32 E8M0)
                return (torch.empty((rows, cols), dtype=u8, device=dev),
                        torch.empty((rows, cols // 32), dtype=u8, device=dev) if mx else
                        torch.empty((rows, cols // 128), dtype=f32, device=dev))

            def wcodes(g, rows, cols):  # codes + scales of a weight stack read along its last dimension (forward)
                return (torch.empty((g, rows, cols), dtype=u8, device=dev),
                        torch.empty((g * rows, cols // 32), dtype=u8, device=dev) if mx else
                        torch.empty((g, rows // 128, cols // 128), dtype=f32, device=dev))

            def wcodes_col(g, rows, cols):  # MXFP8 only: the copy quantised along `rows` for the data gradient
                return (torch.empty((g, rows, cols), dtype=u8, device=dev),
                        torch.empty((g * rows // 128, cols, 4), dtype=u8, device=dev))

            def codes_col(rows, cols):  # the copy quantised down the rows for the weight gradient (32x1 E8M0 / 128x1 fp32)
                if not mx and not self.fp8_wgrad:
                    return None, None
                return (torch.empty((rows, cols), dtype=u8, device=dev),
                        torch.empty((rows // 128, cols, 4), dtype=u8, device=dev) if mx else
                        torch.empty((rows // 128, cols), dtype=f32, device=dev))

            self.qXp, self.sXp = codes(Rcap, h)
            self.qA, self.sA = codes(Rcap, f)
            self.qdO, self.sdO = codes(Rcap, h)
            self.qdZ, self.sdZ = codes(Rcap, 2 * f)
            if mx or self.fp8_wgrad:
                assert Rcap % 128 == 0 and T % 128 == 0, "fp8 weight gradients walk the rows in steps of 128"
            self.qXpc, self.sXpc = codes_col(Rcap, h)
            self.qAc, self.sAc = codes_col(Rcap, f)
            self.qdOc, self.sdOc = codes_col(Rcap, h)
            self.qdZc, self.sdZc = codes_col(Rcap, 2 * f)
            self.qW1, self.sW1 = wcodes(E, 2 * f, h)
            self.qW2, self.sW2 = wcodes(E, h, f)
            # data-gradient copies: the 128x128 blocks serve both directions; MXFP8 needs a second copy
            self.qW1d, self.sW1d = wcodes_col(E, 2 * f, h) if mx else (self.qW1, self.sW1)
            self.qW2d, self.sW2d = wcodes_col(E, h, f) if mx else (self.qW2, self.sW2)
            self.live_rows = self.offsets[E:E + 1]   # device int32: offsets[E]
            if sf:
                self.qX, self.sX = codes(T, h)
                self.qAs, self.sAs = codes(T, sf)
                self.qdY, self.sdY = codes(T, h)
                self.qdZs, self.sdZs = codes(T, 2 * sf)
                self.qXc, self.sXc = codes_col(T, h)
                self.qAsc, self.sAsc = codes_col(T, sf)
                self.qdYc, self.sdYc = codes_col(T, h)
                self.qdZsc, self.sdZsc = codes_col(T, 2 * sf)
                self.qWs1, self.sWs1 = wcodes(1, 2 * sf, h)
                self.qWs2, self.sWs2 = wcodes(1, h, sf)
                self.qWs1d, self.sWs1d = wcodes_col(1, 2 * sf, h) if mx else (self.qWs1, self.sWs1)
                self.qWs2d, self.sWs2d = wcodes_col(1, h, sf) if mx else (self.qWs2, self.sWs2)
        if sf:
            self.off_shared = torch.tensor([0, T], dtype=i32, device=dev)
            self.Zs = torch.empty((T, 2 * sf), dtype=bf, device=dev)
            self.As = torch.empty((T, sf), dtype=bf, device=dev)
            self.S = torch.empty((T, h), dtype=bf, device=dev)
            self.dZs = torch.empty((T, 2 * sf), dtype=bf, device=dev)
            self.dXs = torch.empty((T, h), dtype=bf, device=dev)
            self.dWs1 = torch.empty((2 * sf, h), dtype=wdt, device=dev)
            self.dWs2 = torch.empty((h, sf), dtype=wdt, device=dev)

    # ---- fp8 helpers: quantise a row-indexed tensor (1x128) / a weight stack (128x128) ----------
    def _q_rows(self, X, q, s, rows, cols, live=None, qc=None, sc=None):
        """Quantise a row-indexed tensor for the GEMM that contracts along its rows' elements (and, MXFP8, in the
        same pass the second copy, quantised down the rows, for the weight gradient)."""
        if self.mx:
            B.moe_mx_quantize_rowcol(self.ctx, X, rows, cols, live, q, s, qc, sc)
        elif self.fp8_wgrad:
            B.moe_fp8_quantize_rowcol(self.ctx, X, rows, cols, live, q, s, qc, sc)
        else:
            B.moe_fp8_quantize(self.ctx, X, B.Q_1x128, 1, rows, cols, live, q, s)

    def _q_gather(self, X, pair_scale, groups, rows, cols, q, s, qc, sc):
        """Both quantised copies of X's rows taken through the row map (the permuted tokens, or p * dY)."""
        fn = B.moe_mx_quantize_rowcol_gather if self.mx else B.moe_fp8_quantize_rowcol_gather
        fn(self.ctx, X, self.src_of, self.cfg.k, pair_scale, groups, rows, cols, self.live_rows, q, s, qc, sc)

    def _q_cols(self, X, qc, sc, rows, cols, live=None):
        """Blockwise recipe: the weight-gradient copy of a row-indexed tensor, 128x1 tiles down the rows (a tensor that
        two GEMMs read with different contraction dimensions is quantised once per direction, Sec. 5.3.3 / 5.4.1)."""
        if self.fp8_wgrad and not self.mx:
            B.moe_fp8_quantize_rowcol(self.ctx, X, rows, cols, live, None, None, qc, sc)

    def _q_weight(self, W, q, s, qd=None, sd=None):
        """Quantise a weight stack for the forward GEMM (and, MXFP8, the second copy for the data gradient)."""
        g, rows, cols = q.shape
        if self.mx:
            B.moe_mx_quantize_rowcol(self.ctx, W, g * rows, cols, None, q, s, qd, sd)
        else:
            B.moe_fp8_quantize(self.ctx, W, B.Q_128x128, g, rows, cols, None, q, s)

    def _route(self):
        cfg = self.cfg
        if cfg.grouped_router:
            B.moe_route_topk_grouped(self.ctx, self.logits, self.expert_bias, cfg.T, cfg.E_router, cfg.k, cfg.n_group,
                                     cfg.topk_group, cfg.score, cfg.norm_topk, cfg.route_scale,
                                     self.topk_idx, self.topk_prob, self.route_counts)
        else:
            B.moe_route_topk(self.ctx, self.logits, cfg.T, cfg.E_router, cfg.k, cfg.score, cfg.norm_topk,
                             cfg.route_scale, self.topk_idx, self.topk_prob, self.route_counts)

    def forward(self):
        return self._forward_fp8() if self.fp8 else self._forward_bf16()

    def backward(self):
        return self._backward_fp8() if self.fp8 else self._backward_bf16()

    # ---- the four forward stages --------------------------------------------------------------
    def _forward_bf16(self):
        c, cfg = self.ctx, self.cfg
        T, k, E, h, f, sf, Rcap = cfg.T, cfg.k, cfg.E, cfg.h, cfg.f, self.sf, self.Rcap
        self._route()
        idx = self.topk_idx if self.forced_idx is None else self.forced_idx
        B.moe_permute(c, None if self.gather else self.X, self.dt, idx, T, k, h, E, self.align, self.Xp, Rcap,
                      self.row_of, self.src_of, self.offsets, self.counts)
        row_prob = None
        if self.eq2:  # eq. (2): A = p * silu(gate) * up, plain-sum combine
            B.moe_gather_row_prob(c, self.topk_prob, self.src_of, Rcap, self.row_prob)
            row_prob = self.row_prob
        if self.gather:
            B.moe_grouped_gemm_fwd_gather(c, self.X, T, self.src_of, k, self.W1, self.offsets, E, 2 * f, h, Rcap,
                                          B.EPI_SWIGLU, row_prob, self.Z, self.A)
        else:
            B.moe_grouped_gemm_fwd_weighted(c, self.Xp, self.W1, self.offsets, E, 2 * f, h, Rcap, self.dt, B.EPI_SWIGLU,
                                            None, None, row_prob, self.Z, self.A)
        B.moe_grouped_gemm_fwd(c, self.A, self.W2, self.offsets, E, h, f, Rcap, self.dt, B.EPI_NONE,
                               None, None, self.O, None)
        if sf:
            B.moe_grouped_gemm_fwd(c, self.X, self.Ws1, self.off_shared, 1, 2 * sf, h, T, self.dt, B.EPI_SWIGLU,
                                   None, None, self.Zs, self.As)
            B.moe_grouped_gemm_fwd(c, self.As, self.Ws2, self.off_shared, 1, h, sf, T, self.dt, B.EPI_NONE,
                                   None, None, self.S, None)
        B.moe_unpermute_combine(c, self.O, self.dt, self.row_of, None if self.eq2 else self.topk_prob,
                                self.S if sf else None, T, k, h, self.Y)

    # ---- backward: combine, fc2 (wgrad, dgrad + SwiGLU'), fc1 (wgrad, dgrad), permute ---------
    def _backward_bf16(self):
        c, cfg = self.ctx, self.cfg
        T, k, E, h, f, sf, Rcap = cfg.T, cfg.k, cfg.E, cfg.h, cfg.f, self.sf, self.Rcap
        wdt = self.wgrad_dt
        if self.eq2 and self.gather:
            # dO would be plain copies of dY: both fc2 gradients fetch the rows of dY through the map instead
            B.moe_grouped_gemm_wgrad_gather(c, self.A, self.dY, B.GATHER_DC, T, self.src_of, k, self.offsets, E, h, f, Rcap,
                                            0, wdt, self.dW2)
            B.moe_grouped_gemm_dgrad_gather(c, self.dY, T, self.src_of, k, self.W2, self.offsets, E, h, f, Rcap, self.Z,
                                            self.row_prob, self.dZ, self.dprob_part)
            B.moe_scatter_row_dprob(c, self.dprob_part, self.dprob_parts, self.row_of, T, k, self.dprob)
        elif self.eq2:
            # dO = plain copies of dY (no weight, O is not read); dprob comes out of the fc2 data gradient
            B.moe_unpermute_combine_bwd(c, self.dY, None, self.dt, self.row_of, self.src_of, None,
                                        T, k, h, Rcap, self.dO, None)
            B.moe_grouped_gemm_wgrad(c, self.A, self.dO, self.offsets, E, h, f, Rcap, self.dt, None, None, 0, wdt,
                                     self.dW2)
            B.moe_grouped_gemm_dgrad_weighted(c, self.dO, self.W2, self.offsets, E, h, f, Rcap, self.dt, self.Z, None,
                                              None, self.row_prob, self.dZ, self.dprob_part)
            B.moe_scatter_row_dprob(c, self.dprob_part, self.dprob_parts, self.row_of, T, k, self.dprob)
        else:
            B.moe_unpermute_combine_bwd(c, self.dY, self.O, self.dt, self.row_of, self.src_of, self.topk_prob,
                                        T, k, h, Rcap, self.dO, self.dprob)
            B.moe_grouped_gemm_wgrad(c, self.A, self.dO, self.offsets, E, h, f, Rcap, self.dt, None, None, 0, wdt,
                                     self.dW2)
            B.moe_grouped_gemm_dgrad(c, self.dO, self.W2, self.offsets, E, h, f, Rcap, self.dt, self.Z, None, None,
                                     self.dZ)
        if self.gather:
            B.moe_grouped_gemm_wgrad_gather(c, self.X, self.dZ, B.GATHER_A, T, self.src_of, k, self.offsets, E, 2 * f, h,
                                            Rcap, 0, wdt, self.dW1)
        else:
            B.moe_grouped_gemm_wgrad(c, self.Xp, self.dZ, self.offsets, E, 2 * f, h, Rcap, self.dt, None, None, 0, wdt,
                                     self.dW1)
        B.moe_grouped_gemm_dgrad(c, self.dZ, self.W1, self.offsets, E, 2 * f, h, Rcap, self.dt, None, None, None,
                                 self.dXp)
        if sf:
            o1 = self.off_shared
            B.moe_grouped_gemm_wgrad(c, self.As, self.dY, o1, 1, h, sf, T, self.dt, None, None, 0, wdt, self.dWs2)
            B.moe_grouped_gemm_dgrad(c, self.dY, self.Ws2, o1, 1, h, sf, T, self.dt, self.Zs, None, None, self.dZs)
            B.moe_grouped_gemm_wgrad(c, self.X, self.dZs, o1, 1, 2 * sf, h, T, self.dt, None, None, 0, wdt, self.dWs1)
            B.moe_grouped_gemm_dgrad(c, self.dZs, self.Ws1, o1, 1, 2 * sf, h, T, self.dt, None, None, None, self.dXs)
        # dX[t] = sum of the k permuted-row gradients (+ the shared expert's dX): the plain-sum unpermute
        B.moe_unpermute_combine(c, self.dXp, self.dt, self.row_of, None, self.dXs if sf else None, T, k, h, self.dX)

    # ---- fp8 (blockwise, Sec. 5.3.2, or MXFP8, Sec. 5.3.3): forward and data-gradient GEMMs on E4M3 codes;
    # weights are re-quantised every step (MXFP8: in both directions, one pass); MXFP8 also runs the weight
    # gradients on one-byte operands, quantised down the token dimension in the same pass as the row-wise
    # copy; blockwise weight gradients run on 128x1 copies made by a second quantiser pass (fp8_wgrad off: on the bf16 tensors) ----
    def _forward_fp8(self):
        c, cfg = self.ctx, self.cfg
        T, k, E, h, f, sf, Rcap = cfg.T, cfg.k, cfg.E, cfg.h, cfg.f, self.sf, self.Rcap
        F8 = self.f8dt
        self._route()
        idx = self.topk_idx if self.forced_idx is None else self.forced_idx
        B.moe_permute(c, None if self.fused_quant else self.X, B.BF16, idx, T, k, h, E, self.align, self.Xp, Rcap,
                      self.row_of, self.src_of, self.offsets, self.counts)
        self._q_weight(self.W1, self.qW1, self.sW1, self.qW1d, self.sW1d)
        self._q_weight(self.W2, self.qW2, self.sW2, self.qW2d, self.sW2d)
        if self.fused_quant:
            self._q_gather(self.X, None, E, Rcap, h, self.qXp, self.sXp, self.qXpc, self.sXpc)
        else:
            self._q_rows(self.Xp, self.qXp, self.sXp, Rcap, h, self.live_rows, self.qXpc, self.sXpc)
        row_prob = None
        if self.eq2:
            B.moe_gather_row_prob(c, self.topk_prob, self.src_of, Rcap, self.row_prob)
            row_prob = self.row_prob
        eq = self.epilogue_quant
        self._fc1_fwd(self.qXp, self.qW1, self.offsets, E, 2 * f, h, Rcap, self.sXp, self.sW1, row_prob, self.Z, self.A,
                      self.qA, self.sA, self.qAc, self.sAc, self.live_rows)
        B.moe_grouped_gemm_fwd(c, self.qA, self.qW2, self.offsets, E, h, f, Rcap, F8, B.EPI_NONE,
                               self.sA, self.sW2, self.O, None)
        if sf:
            o1 = self.off_shared
            self._q_weight(self.Ws1.view(1, 2 * sf, h), self.qWs1, self.sWs1, self.qWs1d, self.sWs1d)
            self._q_weight(self.Ws2.view(1, h, sf), self.qWs2, self.sWs2, self.qWs2d, self.sWs2d)
            self._q_rows(self.X, self.qX, self.sX, T, h, None, self.qXc, self.sXc)
            self._fc1_fwd(self.qX, self.qWs1, o1, 1, 2 * sf, h, T, self.sX, self.sWs1, None, self.Zs, self.As,
                          self.qAs, self.sAs, self.qAsc, self.sAsc, None)
            B.moe_grouped_gemm_fwd(c, self.qAs, self.qWs2, o1, 1, h, sf, T, F8, B.EPI_NONE,
                                   self.sAs, self.sWs2, self.S, None)
        B.moe_unpermute_combine(c, self.O, B.BF16, self.row_of, None if self.eq2 else self.topk_prob,
                                self.S if sf else None, T, k, h, self.Y)

    def _backward_fp8(self):
        c, cfg = self.ctx, self.cfg
        T, k, E, h, f, sf, Rcap = cfg.T, cfg.k, cfg.E, cfg.h, cfg.f, self.sf, self.Rcap
        F8, wdt = self.f8dt, self.wgrad_dt
        if self.fused_quant:
            # dO = p * dY (eq. (2): plain copies of dY) goes from dY to its two quantised copies in one pass
            if not self.eq2:
                B.moe_unpermute_combine_bwd(c, self.dY, self.O, B.BF16, self.row_of, self.src_of, self.topk_prob,
                                            T, k, h, Rcap, None, self.dprob)
            self._q_gather(self.dY, None if self.eq2 else self.topk_prob, E, Rcap, h, self.qdO, self.sdO, self.qdOc, self.sdOc)
        else:
            if self.eq2:
                B.moe_unpermute_combine_bwd(c, self.dY, None, B.BF16, self.row_of, self.src_of, None,
                                            T, k, h, Rcap, self.dO, None)
            else:
                B.moe_unpermute_combine_bwd(c, self.dY, self.O, B.BF16, self.row_of, self.src_of, self.topk_prob,
                                            T, k, h, Rcap, self.dO, self.dprob)
            self._q_rows(self.dO, self.qdO, self.sdO, Rcap, h, self.live_rows, self.qdOc, self.sdOc)
        self._wgrad(self.A, self.dO, self.qAc, self.sAc, self.qdOc, self.sdOc, self.offsets, E, h, f, Rcap, self.dW2)
        self._fc2_dgrad(self.qdO, self.qW2d, self.offsets, E, h, f, Rcap, self.Z, self.sdO, self.sW2d,
                        self.row_prob if self.eq2 else None, self.dZ, self.dprob_part if self.eq2 else None,
                        self.qdZ, self.sdZ, self.qdZc, self.sdZc, self.live_rows)
        if self.eq2:
            B.moe_scatter_row_dprob(c, self.dprob_part, self.dprob_parts, self.row_of, T, k, self.dprob)
        self._wgrad(self.Xp, self.dZ, self.qXpc, self.sXpc, self.qdZc, self.sdZc, self.offsets, E, 2 * f, h, Rcap, self.dW1)
        B.moe_grouped_gemm_dgrad(c, self.qdZ, self.qW1d, self.offsets, E, 2 * f, h, Rcap, F8, None, self.sdZ, self.sW1d,
                                 self.dXp)
        if sf:
            o1 = self.off_shared
            self._q_rows(self.dY, self.qdY, self.sdY, T, h, None, self.qdYc, self.sdYc)
            self._wgrad(self.As, self.dY, self.qAsc, self.sAsc, self.qdYc, self.sdYc, o1, 1, h, sf, T, self.dWs2)
            self._fc2_dgrad(self.qdY, self.qWs2d, o1, 1, h, sf, T, self.Zs, self.sdY, self.sWs2d, None, self.dZs, None,
                            self.qdZs, self.sdZs, self.qdZsc, self.sdZsc, None)
            self._wgrad(self.X, self.dZs, self.qXc, self.sXc, self.qdZsc, self.sdZsc, o1, 1, 2 * sf, h, T, self.dWs1)
            B.moe_grouped_gemm_dgrad(c, self.qdZs, self.qWs1d, o1, 1, 2 * sf, h, T, F8, None, self.sdZs, self.sWs1d,
                                     self.dXs)
        B.moe_unpermute_combine(c, self.dXp, B.BF16, self.row_of, None, self.dXs if sf else None, T, k, h, self.dX)

    def _fc1_fwd(self, qX, qW, offsets, E, N, K, rows, sX, sW, row_prob, Z, A, qA, sA, qAc, sAc, live):
        """fc1 + SwiGLU and the quantised copies of the activation fc2 and its weight gradient read: from the GEMM's own
        epilogue (Sec. 5.4.2) where that is built and switched on, else by quantiser launches."""
        c, eq = self.ctx, self.epilogue_quant
        if eq and self.mx:
            B.moe_grouped_gemm_fwd_quant_mx(c, qX, qW, offsets, E, N, K, rows, sX, sW, row_prob, Z, A, qA, sA, qAc, sAc)
            return
        B.moe_grouped_gemm_fwd_quant(c, qX, qW, offsets, E, N, K, rows, self.f8dt, B.EPI_SWIGLU, sX, sW, row_prob, Z, A,
                                     qA if eq else None, sA if eq else None)
        if not eq:
            self._q_rows(A, qA, sA, rows, N // 2, live, qAc, sAc)
        else:
            self._q_cols(A, qAc, sAc, rows, N // 2, live)

    def _fc2_dgrad(self, qdO, qW, offsets, E, N, K, rows, Z, sdO, sW, row_prob, dZ, dprob_part, qdZ, sdZ, qdZc, sdZc, live):
        """fc2 data gradient + SwiGLU backward and the quantised copies of dZ, as in _fc1_fwd."""
        c, eq = self.ctx, self.epilogue_quant
        if eq and self.mx:
            B.moe_grouped_gemm_dgrad_quant_mx(c, qdO, qW, offsets, E, N, K, rows, Z, sdO, sW, row_prob, dZ, dprob_part,
                                              qdZ, sdZ, qdZc, sdZc)
            return
        B.moe_grouped_gemm_dgrad_quant(c, qdO, qW, offsets, E, N, K, rows, self.f8dt, Z, sdO, sW, row_prob, dZ, dprob_part,
                                       qdZ if eq else None, sdZ if eq else None)
        if not eq:
            self._q_rows(dZ, qdZ, sdZ, rows, 2 * K, live, qdZc, sdZc)
        else:
            self._q_cols(dZ, qdZc, sdZc, rows, 2 * K, live)

    def _wgrad(self, A, dC, qA, sA, qdC, sdC, offsets, E, N, K, rows, dW):
        """dW = dC^T A per expert: on the copies quantised down the rows (MXFP8: 32x1 blocks; blockwise: 128x1 tiles) or,
        with fp8_wgrad off, on the bf16 tensors."""
        if self.mx or self.fp8_wgrad:
            B.moe_grouped_gemm_wgrad(self.ctx, qA, qdC, offsets, E, N, K, rows, self.f8dt, sA, sdC, 0, self.wgrad_dt, dW)
        else:
            B.moe_grouped_gemm_wgrad(self.ctx, A, dC, offsets, E, N, K, rows, B.BF16, None, None, 0, self.wgrad_dt, dW)

    def step(self):
        self.forward()
        self.backward()
