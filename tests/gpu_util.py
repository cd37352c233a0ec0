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


BF16_TOL = 2e-2   # relative Frobenius bound for bf16 outputs and gradients (fp32 accumulation)
FP8_TOL = 6e-2    # same for the blockwise fp8 path


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
