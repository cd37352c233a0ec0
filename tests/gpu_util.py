"""Helpers for the GPU parity tests: host<->device marshalling and error metrics (no layer arithmetic)."""
import numpy as np
import torch

from paper_2603_07685_amd import workloads as wl


def dev_bf16(x: np.ndarray) -> torch.Tensor:
    """fp32 host values (already bf16-representable or not) -> bf16 device tensor with the same RNE rounding."""
    bits = wl.f32_to_bf16_bits(np.ascontiguousarray(x, np.float32))
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def dev(x: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x)).cuda()


def rel_fro(got: np.ndarray, ref: np.ndarray) -> float:
    """Relative Frobenius error ||got - ref||_F / ||ref||_F (0 if both are zero)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    den = np.linalg.norm(ref.ravel())
    num = np.linalg.norm((got - ref).ravel())
    if den == 0:
        return 0.0 if num == 0 else float("inf")
    return float(num / den)


BF16_TOL = 2e-2   # relative Frobenius bound for bf16 outputs and gradients (fp32 accumulation): the contract
FP8_TOL = 6e-2    # same for the fp8 paths against the full-precision oracle
# Regression bounds, about three times what the kernels measure today (1.7e-3 .. 3.4e-3 for a bf16 call: one rounding
# of an fp32-accumulated result to 8 significant bits, 2^-9 at most per element; 2.5e-3 against the oracle's
# quantise-dequantise emulation of an fp8 call; 3e-7 for an fp32 call).  The contract bound stays what the tests
# promise; these catch a kernel that got worse without crossing it.
BF16_REG = 6e-3
FP8_EMUL_REG = 8e-3
F32_REG = 1e-5


def assert_close(got, ref, what="", tol=BF16_TOL, reg=BF16_REG, row_tol=None, row_floor=1e-6):
    """Element-level parity of one tensor against the oracle, three ways:
      * relative Frobenius error of the whole tensor <= tol (the contract) and <= reg (the regression bound);
      * every row r (last dimension) on its own: ||got_r - ref_r|| <= row_tol ||ref_r|| + floor, where the floor
        (row_floor = 1e-6 of the root-mean-square row norm) only absorbs rows that are zero or nearly so by
        construction.  A wrong or half-contracted row moves a pooled norm by 1/sqrt(rows) and hides in it; here it
        fails.  Tensors whose elements are sums with cancellation (dprob: a few dot products per row, error
        proportional to the operands, not to the result) pass a larger row_floor.
    Returns the pooled error."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.isfinite(got).all(), (what, "non-finite values")
    e = rel_fro(got, ref)
    assert e <= tol, (what, "pooled error above the contract bound", e, tol)
    if reg is not None:
        assert e <= reg, (what, "pooled error above the regression bound", e, reg)
    row_tol = tol if row_tol is None else row_tol
    if got.size:
        g2, r2 = got.reshape(-1, got.shape[-1]), ref.reshape(-1, ref.shape[-1])
        num = np.linalg.norm(g2 - r2, axis=1)
        den = np.linalg.norm(r2, axis=1)
        floor = row_floor * np.sqrt(np.mean(den ** 2))
        bad = np.nonzero(num > row_tol * den + floor)[0]
        if len(bad):
            w = bad[np.argmax(num[bad] / (den[bad] + floor))]
            raise AssertionError((what, f"{len(bad)} of {len(num)} rows above the per-row bound {row_tol}",
                                  f"worst row {int(w)}: error {num[w]:.3e}, norm {den[w]:.3e}"))
    return e


def permuted_rows(st, rows: torch.Tensor, cols=slice(None)) -> torch.Tensor:
    """Rows of the permuted-token tensor Xp: as stored, or, when the layer quantises straight from X (no bf16 Xp
    exists), what they are by definition: exact copies of the source tokens, zero for padding rows."""
    if st.Xp is not None:
        return st.Xp[rows][:, cols]
    s = st.src_of[rows].long()
    x = st.X[torch.div(s.clamp(min=0), st.cfg.k, rounding_mode="floor")][:, cols].clone()
    x[s < 0] = 0
    return x


def combine_bwd_rows(st, rows: torch.Tensor, cols=slice(None)) -> torch.Tensor:
    """Rows of dO = bf16(p * dY) (eq. (2): copies of dY): as stored, or rebuilt from dY when only its quantised
    copies exist (fp32 product rounded to bf16, the value the fused quantiser is defined on)."""
    if st.dO is not None:
        return st.dO[rows][:, cols]
    s = st.src_of[rows].long()
    x = st.dY[torch.div(s.clamp(min=0), st.cfg.k, rounding_mode="floor")][:, cols].float()
    if not st.eq2:
        x = x * st.topk_prob.reshape(-1)[s.clamp(min=0)][:, None]
    x = x.to(torch.bfloat16)
    x[s < 0] = 0
    return x
