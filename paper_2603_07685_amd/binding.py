"""ctypes binding of libmoe_hip.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/moe_hip.h.  Tensors are torch CUDA tensors used as device memory; the
current torch stream is passed as the HIP stream.  Nothing here computes: if
the library is missing the import of `lib()` raises, there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("MOE_HIP_LIB") or os.path.join(_PKG, "libmoe_hip.so")
_lib = None

BF16, FP8_E4M3, F32, MXFP8_E4M3 = 0, 1, 2, 3
SOFTMAX, SIGMOID = 0, 1
EPI_NONE, EPI_SWIGLU = 0, 1
Q_1x128, Q_128x1, Q_128x128 = 0, 1, 2
MX_1x32, MX_32x1 = 0, 1
GATHER_A, GATHER_DC = 0, 1

EXPORTS = [
    "moe_workspace_bytes", "moe_ctx_create", "moe_ctx_destroy", "moe_last_error", "moe_ctx_poll_error",
    "moe_route_topk", "moe_permute", "moe_grouped_gemm_fwd", "moe_grouped_gemm_dgrad", "moe_grouped_gemm_wgrad",
    "moe_unpermute_combine", "moe_unpermute_combine_bwd", "moe_fp8_quantize",
    "moe_grouped_gemm_fwd_weighted", "moe_grouped_gemm_dgrad_weighted", "moe_gather_row_prob", "moe_scatter_row_dprob",
    "moe_route_topk_bwd", "moe_mx_quantize", "moe_mx_quantize_rowcol",
    "moe_route_topk_grouped", "moe_aux_loss", "moe_mx_quantize_rowcol_gather",
    "moe_grouped_gemm_fwd_quant", "moe_grouped_gemm_dgrad_quant",
    "moe_grouped_gemm_fwd_quant_mx", "moe_grouped_gemm_dgrad_quant_mx", "moe_gate_gemm", "moe_permute_static",
    "moe_fp8_quantize_rowcol", "moe_fp8_quantize_rowcol_gather",
    "moe_grouped_gemm_fwd_gather", "moe_grouped_gemm_dgrad_gather", "moe_grouped_gemm_wgrad_gather",
]

_vp, _i, _i64, _f = C.c_void_p, C.c_int, C.c_int64, C.c_float


class MoeError(RuntimeError):
    pass


def lib() -> C.CDLL:
    """Load libmoe_hip.so (built by paper_2603_07685_amd.build / __graft_entry__.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise MoeError(f"{LIB_PATH} is not built: run `python -m paper_2603_07685_amd.build` first "
                           "(there is no CPU fallback)")
        L = C.CDLL(LIB_PATH)
        L.moe_workspace_bytes.restype = C.c_size_t
        L.moe_workspace_bytes.argtypes = [_i] * 5
        L.moe_ctx_create.argtypes = [C.POINTER(_vp), _i, C.c_size_t]
        L.moe_ctx_destroy.argtypes = [_vp]
        L.moe_last_error.restype = C.c_char_p
        L.moe_last_error.argtypes = [_vp]
        L.moe_ctx_poll_error.argtypes = [_vp, _vp, C.POINTER(_i)]
        L.moe_route_topk.argtypes = [_vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _vp, _vp, _vp]
        L.moe_permute.argtypes = [_vp, _vp, _vp, _i, _vp, _i, _i, _i, _i, _i, _vp, _i64, _vp, _vp, _vp, _vp]
        L.moe_permute_static.argtypes = [_vp, _vp, _i, _vp, _i, _i, _i, _i, _i, _vp, _i64, _vp, _vp, _vp, _vp]
        L.moe_grouped_gemm_fwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64, _i, _i, _vp, _vp, _vp, _vp]
        L.moe_grouped_gemm_dgrad.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64, _i, _vp, _vp, _vp, _vp]
        L.moe_grouped_gemm_wgrad.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64, _i, _vp, _vp, _i, _i, _vp]
        L.moe_unpermute_combine.argtypes = [_vp, _vp, _vp, _i, _vp, _vp, _vp, _i, _i, _i, _vp]
        L.moe_unpermute_combine_bwd.argtypes = [_vp, _vp, _vp, _vp, _i, _vp, _vp, _vp, _i, _i, _i, _i64, _vp, _vp]
        L.moe_fp8_quantize.argtypes = [_vp, _vp, _vp, _i, _i, _i64, _i, _vp, _vp, _vp]
        L.moe_grouped_gemm_fwd_weighted.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64, _i, _i, _vp, _vp, _vp, _vp, _vp]
        L.moe_grouped_gemm_dgrad_weighted.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64, _i, _vp, _vp, _vp, _vp, _vp, _vp]
        L.moe_mx_quantize.argtypes = [_vp, _vp, _vp, _i, _i, _i64, _i, _vp, _vp, _vp]
        L.moe_mx_quantize_rowcol.argtypes = [_vp, _vp, _vp, _i64, _i, _vp, _vp, _vp, _vp, _vp]
        L.moe_route_topk_grouped.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _i, _i, _f, _vp, _vp, _vp]
        L.moe_aux_loss.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _i, _f, _f, _i, _vp, _vp]
        L.moe_mx_quantize_rowcol_gather.argtypes = [_vp, _vp, _vp, _vp, _i, _vp, _i, _i64, _i, _vp, _vp, _vp, _vp, _vp]
        L.moe_grouped_gemm_fwd_quant.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64, _i, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
        L.moe_grouped_gemm_dgrad_quant.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64, _i, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
        L.moe_grouped_gemm_fwd_quant_mx.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64] + [_vp] * 9
        L.moe_grouped_gemm_dgrad_quant_mx.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i64] + [_vp] * 10
        L.moe_fp8_quantize_rowcol.argtypes = [_vp, _vp, _vp, _i64, _i, _vp, _vp, _vp, _vp, _vp]
        L.moe_fp8_quantize_rowcol_gather.argtypes = [_vp, _vp, _vp, _vp, _i, _vp, _i, _i64, _i, _vp, _vp, _vp, _vp, _vp]
        L.moe_gate_gemm.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _i, _vp]
        L.moe_grouped_gemm_fwd_gather.argtypes = [_vp, _vp, _vp, _i, _vp, _i, _vp, _vp, _i, _i, _i, _i64, _i, _vp, _vp, _vp]
        L.moe_grouped_gemm_dgrad_gather.argtypes = [_vp, _vp, _vp, _i, _vp, _i, _vp, _vp, _i, _i, _i, _i64, _vp, _vp, _vp, _vp]
        L.moe_grouped_gemm_wgrad_gather.argtypes = [_vp, _vp, _vp, _vp, _i, _i, _vp, _i, _vp, _i, _i, _i, _i64, _i, _i, _vp]
        L.moe_route_topk_bwd.argtypes = [_vp, _vp, _vp, _vp, _vp, _i, _i, _i, _i, _i, _f, _vp]
        L.moe_gather_row_prob.argtypes = [_vp, _vp, _vp, _vp, _i64, _vp]
        L.moe_scatter_row_dprob.argtypes = [_vp, _vp, _vp, _i, _vp, _i, _i, _vp]
        for name in EXPORTS:
            if name not in ("moe_workspace_bytes", "moe_last_error"):
                getattr(L, name).restype = _i
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


class Context:
    """Owns a moe_ctx (device workspace + error state)."""

    def __init__(self, T, k, E, h, f_max, device=0):
        L = lib()
        self.bytes = int(L.moe_workspace_bytes(T, k, E, h, f_max))
        h_ = _vp()
        st = L.moe_ctx_create(C.byref(h_), device, self.bytes)
        if st != 0:
            raise MoeError(f"moe_ctx_create failed with status {st}")
        self.h = h_

    def check(self, st, what):
        if st != 0:
            raise MoeError(f"{what}: status {st}: {lib().moe_last_error(self.h).decode()}")

    def poll_error(self) -> int:
        v = _i(0)
        self.check(lib().moe_ctx_poll_error(self.h, _stream(), C.byref(v)), "moe_ctx_poll_error")
        return v.value

    def close(self):
        if self.h:
            lib().moe_ctx_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def moe_workspace_bytes(T, k, E, h, f_max):
    return int(lib().moe_workspace_bytes(T, k, E, h, f_max))


def moe_route_topk(ctx, logits, T, E, k, fn, norm_topk, scale, topk_idx, topk_prob, counts):
    ctx.check(lib().moe_route_topk(ctx.h, _stream(), _ptr(logits), T, E, k, fn, int(norm_topk), scale,
                                   _ptr(topk_idx), _ptr(topk_prob), _ptr(counts)), "moe_route_topk")


def moe_route_topk_grouped(ctx, logits, expert_bias, T, E, k, n_group, topk_group, fn, norm_topk, scale,
                           topk_idx, topk_prob, counts):
    ctx.check(lib().moe_route_topk_grouped(ctx.h, _stream(), _ptr(logits), _ptr(expert_bias), T, E, k, n_group,
                                           topk_group, fn, int(norm_topk), float(scale), _ptr(topk_idx),
                                           _ptr(topk_prob), _ptr(counts)), "moe_route_topk_grouped")


def moe_aux_loss(ctx, logits, counts, T, E, k, fn, coeff, dloss, accumulate, loss, dlogits):
    ctx.check(lib().moe_aux_loss(ctx.h, _stream(), _ptr(logits), _ptr(counts), T, E, k, fn, float(coeff), float(dloss),
                                 int(bool(accumulate)), _ptr(loss), _ptr(dlogits)), "moe_aux_loss")


def moe_permute(ctx, X, dt, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts):
    ctx.check(lib().moe_permute(ctx.h, _stream(), _ptr(X), dt, _ptr(idx), T, k, h, E, align, _ptr(Xp), Rcap,
                                _ptr(row_of), _ptr(src_of), _ptr(offsets), _ptr(counts)), "moe_permute")


def moe_permute_static(X, dt, idx, T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts):
    st = lib().moe_permute_static(_stream(), _ptr(X), dt, _ptr(idx), T, k, h, E, align, _ptr(Xp), Rcap,
                                  _ptr(row_of), _ptr(src_of), _ptr(offsets), _ptr(counts))
    if st != 0:
        raise MoeError(f"moe_permute_static: status {st}: {lib().moe_last_error(None).decode()}")


def moe_grouped_gemm_fwd(ctx, A, B, offsets, E, N, K, Rcap, dt, epi, a_scale, b_scale, Cout, C_act):
    ctx.check(lib().moe_grouped_gemm_fwd(ctx.h, _stream(), _ptr(A), _ptr(B), _ptr(offsets), E, N, K, Rcap, dt, epi,
                                         _ptr(a_scale), _ptr(b_scale), _ptr(Cout), _ptr(C_act)),
              "moe_grouped_gemm_fwd")


def moe_grouped_gemm_dgrad(ctx, dC, B, offsets, E, N, K, Rcap, dt, Z_saved, dc_scale, b_scale, dA):
    ctx.check(lib().moe_grouped_gemm_dgrad(ctx.h, _stream(), _ptr(dC), _ptr(B), _ptr(offsets), E, N, K, Rcap, dt,
                                           _ptr(Z_saved), _ptr(dc_scale), _ptr(b_scale), _ptr(dA)),
              "moe_grouped_gemm_dgrad")


def moe_grouped_gemm_fwd_weighted(ctx, A, B, offsets, E, N, K, Rcap, dt, epi, a_scale, b_scale, row_prob, Cout, C_act):
    ctx.check(lib().moe_grouped_gemm_fwd_weighted(ctx.h, _stream(), _ptr(A), _ptr(B), _ptr(offsets), E, N, K, Rcap, dt,
                                                  epi, _ptr(a_scale), _ptr(b_scale), _ptr(row_prob), _ptr(Cout),
                                                  _ptr(C_act)),
              "moe_grouped_gemm_fwd_weighted")


def moe_grouped_gemm_dgrad_weighted(ctx, dC, B, offsets, E, N, K, Rcap, dt, Z_saved, dc_scale, b_scale, row_prob, dA,
                                    dprob_part):
    ctx.check(lib().moe_grouped_gemm_dgrad_weighted(ctx.h, _stream(), _ptr(dC), _ptr(B), _ptr(offsets), E, N, K, Rcap,
                                                    dt, _ptr(Z_saved), _ptr(dc_scale), _ptr(b_scale), _ptr(row_prob),
                                                    _ptr(dA), _ptr(dprob_part)),
              "moe_grouped_gemm_dgrad_weighted")


def moe_grouped_gemm_fwd_quant(ctx, A, B, offsets, E, N, K, Rcap, dt, epi, a_scale, b_scale, row_prob, Cout, C_act,
                               act_q, act_q_scale):
    ctx.check(lib().moe_grouped_gemm_fwd_quant(ctx.h, _stream(), _ptr(A), _ptr(B), _ptr(offsets), E, N, K, Rcap, dt, epi,
                                               _ptr(a_scale), _ptr(b_scale), _ptr(row_prob), _ptr(Cout), _ptr(C_act),
                                               _ptr(act_q), _ptr(act_q_scale)), "moe_grouped_gemm_fwd_quant")


def moe_grouped_gemm_dgrad_quant(ctx, dC, B, offsets, E, N, K, Rcap, dt, Z_saved, dc_scale, b_scale, row_prob, dA,
                                 dprob_part, dz_q, dz_q_scale):
    ctx.check(lib().moe_grouped_gemm_dgrad_quant(ctx.h, _stream(), _ptr(dC), _ptr(B), _ptr(offsets), E, N, K, Rcap, dt,
                                                 _ptr(Z_saved), _ptr(dc_scale), _ptr(b_scale), _ptr(row_prob), _ptr(dA),
                                                 _ptr(dprob_part), _ptr(dz_q), _ptr(dz_q_scale)),
              "moe_grouped_gemm_dgrad_quant")


def moe_grouped_gemm_fwd_quant_mx(ctx, A, B, offsets, E, N, K, Rcap, a_scale, b_scale, row_prob, Cout, C_act,
                                  act_q_row, act_e8_row, act_q_col, act_e8_col):
    ctx.check(lib().moe_grouped_gemm_fwd_quant_mx(ctx.h, _stream(), _ptr(A), _ptr(B), _ptr(offsets), E, N, K, Rcap,
                                                  _ptr(a_scale), _ptr(b_scale), _ptr(row_prob), _ptr(Cout), _ptr(C_act),
                                                  _ptr(act_q_row), _ptr(act_e8_row), _ptr(act_q_col), _ptr(act_e8_col)),
              "moe_grouped_gemm_fwd_quant_mx")


def moe_grouped_gemm_dgrad_quant_mx(ctx, dC, B, offsets, E, N, K, Rcap, Z_saved, dc_scale, b_scale, row_prob, dZ,
                                    dprob_part, dz_q_row, dz_e8_row, dz_q_col, dz_e8_col):
    ctx.check(lib().moe_grouped_gemm_dgrad_quant_mx(ctx.h, _stream(), _ptr(dC), _ptr(B), _ptr(offsets), E, N, K, Rcap,
                                                    _ptr(Z_saved), _ptr(dc_scale), _ptr(b_scale), _ptr(row_prob), _ptr(dZ),
                                                    _ptr(dprob_part), _ptr(dz_q_row), _ptr(dz_e8_row), _ptr(dz_q_col),
                                                    _ptr(dz_e8_col)), "moe_grouped_gemm_dgrad_quant_mx")


def moe_gate_gemm(ctx, X, Wr, T, E, h, logits):
    ctx.check(lib().moe_gate_gemm(ctx.h, _stream(), _ptr(X), _ptr(Wr), T, E, h, _ptr(logits)), "moe_gate_gemm")


def moe_route_topk_bwd(ctx, logits, topk_idx, dprob, T, E, k, fn, norm_topk, scale, dlogits):
    ctx.check(lib().moe_route_topk_bwd(ctx.h, _stream(), _ptr(logits), _ptr(topk_idx), _ptr(dprob), T, E, k, fn,
                                       int(norm_topk), float(scale), _ptr(dlogits)), "moe_route_topk_bwd")


def moe_gather_row_prob(ctx, prob, src_of, Rcap, row_prob):
    ctx.check(lib().moe_gather_row_prob(ctx.h, _stream(), _ptr(prob), _ptr(src_of), Rcap, _ptr(row_prob)),
              "moe_gather_row_prob")


def moe_scatter_row_dprob(ctx, dprob_part, parts, row_of, T, k, dprob):
    ctx.check(lib().moe_scatter_row_dprob(ctx.h, _stream(), _ptr(dprob_part), parts, _ptr(row_of), T, k, _ptr(dprob)),
              "moe_scatter_row_dprob")


def moe_grouped_gemm_wgrad(ctx, A, dC, offsets, E, N, K, Rcap, dt, a_scale, dc_scale, accumulate, out_dt, dB):
    ctx.check(lib().moe_grouped_gemm_wgrad(ctx.h, _stream(), _ptr(A), _ptr(dC), _ptr(offsets), E, N, K, Rcap, dt,
                                           _ptr(a_scale), _ptr(dc_scale), int(accumulate), out_dt, _ptr(dB)),
              "moe_grouped_gemm_wgrad")


def moe_grouped_gemm_fwd_gather(ctx, X, T, src_of, k, B, offsets, E, N, K, Rcap, epi, row_prob, Cout, C_act):
    ctx.check(lib().moe_grouped_gemm_fwd_gather(ctx.h, _stream(), _ptr(X), T, _ptr(src_of), k, _ptr(B), _ptr(offsets),
                                                E, N, K, Rcap, epi, _ptr(row_prob), _ptr(Cout), _ptr(C_act)),
              "moe_grouped_gemm_fwd_gather")


def moe_grouped_gemm_dgrad_gather(ctx, G, T, src_of, k, B, offsets, E, N, K, Rcap, Z_saved, row_prob, dA, dprob_part):
    ctx.check(lib().moe_grouped_gemm_dgrad_gather(ctx.h, _stream(), _ptr(G), T, _ptr(src_of), k, _ptr(B), _ptr(offsets),
                                                  E, N, K, Rcap, _ptr(Z_saved), _ptr(row_prob), _ptr(dA),
                                                  _ptr(dprob_part)), "moe_grouped_gemm_dgrad_gather")


def moe_grouped_gemm_wgrad_gather(ctx, A, dC, which, T, src_of, k, offsets, E, N, K, Rcap, accumulate, out_dt, dB):
    ctx.check(lib().moe_grouped_gemm_wgrad_gather(ctx.h, _stream(), _ptr(A), _ptr(dC), which, T, _ptr(src_of), k,
                                                  _ptr(offsets), E, N, K, Rcap, int(accumulate), out_dt, _ptr(dB)),
              "moe_grouped_gemm_wgrad_gather")


def moe_unpermute_combine(ctx, O, dt, row_of, prob, residual, T, k, h, Y):
    ctx.check(lib().moe_unpermute_combine(ctx.h, _stream(), _ptr(O), dt, _ptr(row_of), _ptr(prob), _ptr(residual),
                                          T, k, h, _ptr(Y)), "moe_unpermute_combine")


def moe_unpermute_combine_bwd(ctx, dY, O, dt, row_of, src_of, prob, T, k, h, Rcap, dO, dprob):
    ctx.check(lib().moe_unpermute_combine_bwd(ctx.h, _stream(), _ptr(dY), _ptr(O), dt, _ptr(row_of), _ptr(src_of),
                                              _ptr(prob), T, k, h, Rcap, _ptr(dO), _ptr(dprob)),
              "moe_unpermute_combine_bwd")


def moe_mx_quantize(ctx, X, block, groups, rows, cols, rows_dev, q, e8m0):
    ctx.check(lib().moe_mx_quantize(ctx.h, _stream(), _ptr(X), block, groups, rows, cols, _ptr(rows_dev), _ptr(q),
                                    _ptr(e8m0)), "moe_mx_quantize")


def moe_mx_quantize_rowcol(ctx, X, rows, cols, rows_dev, q_row, e8m0_row, q_col, e8m0_col):
    ctx.check(lib().moe_mx_quantize_rowcol(ctx.h, _stream(), _ptr(X), rows, cols, _ptr(rows_dev), _ptr(q_row),
                                           _ptr(e8m0_row), _ptr(q_col), _ptr(e8m0_col)), "moe_mx_quantize_rowcol")


def moe_mx_quantize_rowcol_gather(ctx, X, src_of, k, pair_scale, groups, rows, cols, rows_dev, q_row, e8m0_row, q_col,
                                  e8m0_col):
    ctx.check(lib().moe_mx_quantize_rowcol_gather(ctx.h, _stream(), _ptr(X), _ptr(src_of), k, _ptr(pair_scale), groups, rows, cols,
                                                  _ptr(rows_dev), _ptr(q_row), _ptr(e8m0_row), _ptr(q_col),
                                                  _ptr(e8m0_col)), "moe_mx_quantize_rowcol_gather")


def moe_fp8_quantize(ctx, X, block, groups, rows, cols, rows_dev, q, scale):
    ctx.check(lib().moe_fp8_quantize(ctx.h, _stream(), _ptr(X), block, groups, rows, cols, _ptr(rows_dev), _ptr(q),
                                     _ptr(scale)), "moe_fp8_quantize")


def moe_fp8_quantize_rowcol(ctx, X, rows, cols, rows_dev, q_row, scale_row, q_col, scale_col):
    ctx.check(lib().moe_fp8_quantize_rowcol(ctx.h, _stream(), _ptr(X), rows, cols, _ptr(rows_dev), _ptr(q_row),
                                            _ptr(scale_row), _ptr(q_col), _ptr(scale_col)), "moe_fp8_quantize_rowcol")


def moe_fp8_quantize_rowcol_gather(ctx, X, src_of, k, pair_scale, groups, rows, cols, rows_dev, q_row, scale_row, q_col,
                                   scale_col):
    ctx.check(lib().moe_fp8_quantize_rowcol_gather(ctx.h, _stream(), _ptr(X), _ptr(src_of), k, _ptr(pair_scale), groups, rows,
                                                   cols, _ptr(rows_dev), _ptr(q_row), _ptr(scale_row), _ptr(q_col),
                                                   _ptr(scale_col)), "moe_fp8_quantize_rowcol_gather")
