"""GPU parity of the blockwise fp8 path (Sec. 5.3.2): quantisers bit-exact against the oracle, fp8 grouped
GEMMs against (a) the oracle run on the dequantised codes (tight: only accumulation order and the bf16
output rounding differ) and (b) the full-precision oracle (the 6e-2 bound of the fp8 recipe)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

EMU_TOL = 4e-3   # vs the oracle on the same codes: bf16 output rounding (2^-9) + fp32 accumulation order


@pytest.fixture(scope="module")
def B():
    from paper_2603_07685_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def ctx(B):
    c = B.Context(T=16384, k=8, E=256, h=7168, f_max=14336)
    yield c
    c.close()


def _quant(B, ctx, X, kind, rows_dev=None):
    """X: bf16 device tensor [rows, cols] or [G, rows, cols] -> (codes uint8, scales fp32) on the device."""
    if kind == B.Q_128x128:
        G, rows, cols = X.shape
        q = torch.empty((G, rows, cols), dtype=torch.uint8, device="cuda")
        s = torch.empty((G, rows // 128, cols // 128), dtype=torch.float32, device="cuda")
    else:
        G = 1
        rows, cols = X.shape
        q = torch.empty((rows, cols), dtype=torch.uint8, device="cuda")
        s = (torch.empty((rows, cols // 128), dtype=torch.float32, device="cuda") if kind == B.Q_1x128
             else torch.empty((rows // 128, cols), dtype=torch.float32, device="cuda"))
    B.moe_fp8_quantize(ctx, X, kind, G, rows, cols, rows_dev, q, s)
    return q, s


@pytest.mark.parametrize("rows,cols", [(256, 384), (1000, 128), (4096, 7168)])
def test_quantize_1x128_bit_exact(B, ctx, oracle, rows, cols):
    from gpu_util import dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(rows)
    Xh = wl.bf16_round((g.standard_normal((rows, cols)) * np.exp(g.uniform(-4, 2, (rows, 1)))).astype(np.float32))
    Xh[3, :128] = 0.0
    q, s = _quant(B, ctx, dev_bf16(Xh), B.Q_1x128)
    torch.cuda.synchronize()
    qo, so = oracle.fp8_quant_1x128(Xh)
    assert np.array_equal(s.cpu().numpy(), so)
    assert np.array_equal(q.cpu().numpy(), qo)


def test_quantize_128x1_and_rows_dev(B, ctx, oracle):
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(7)
    rows, cols = 640, 1160            # cols: two 512-column panels + a ragged third
    Xh = wl.bf16_round((g.standard_normal((rows, cols)) * np.exp(g.uniform(-3, 3, (1, cols)))).astype(np.float32))
    X = dev_bf16(Xh)
    q, s = _quant(B, ctx, X, B.Q_128x1)
    torch.cuda.synchronize()
    qo, so = oracle.fp8_quant_128x1(Xh)
    assert np.array_equal(s.cpu().numpy(), so) and np.array_equal(q.cpu().numpy(), qo)
    # live-row count on the device: only the first 384 rows are touched
    q2 = torch.full((rows, cols), 0x55, dtype=torch.uint8, device="cuda")
    s2 = torch.full((rows // 128, cols), -1.0, dtype=torch.float32, device="cuda")
    B.moe_fp8_quantize(ctx, X, B.Q_128x1, 1, rows, cols, dev(np.array([384], np.int32)), q2, s2)
    torch.cuda.synchronize()
    assert np.array_equal(q2.cpu().numpy()[:384], qo[:384]) and (q2[384:] == 0x55).all()
    assert np.array_equal(s2.cpu().numpy()[:3], so[:3]) and (s2[3:] == -1.0).all()


def test_quantize_128x128_bit_exact(B, ctx, oracle):
    from gpu_util import dev_bf16
    from paper_2603_07685_amd import workloads as wl
    Wh = wl.gaussian_bf16((3, 256, 384), 0.02, 5, 1)
    Wh[1, 128:, :128] = 0.0
    q, s = _quant(B, ctx, dev_bf16(Wh), B.Q_128x128)
    torch.cuda.synchronize()
    qo, so = oracle.fp8_quant_128x128(Wh)
    assert np.array_equal(s.cpu().numpy(), so) and np.array_equal(q.cpu().numpy(), qo)


def _offsets128(counts):
    pad = (np.asarray(counts) + 127) // 128 * 128
    return np.concatenate([[0], np.cumsum(pad)]).astype(np.int32)


@pytest.mark.parametrize("counts,N,K,swiglu", [
    ([300, 0, 257, 1, 700], 512, 256, False),
    ([130, 90], 256, 128, False),
    ([513, 128, 5], 768, 384, True),
    ([300, 0, 257, 1, 700], 512, 256, True),
])
def test_fp8_grouped_gemm_fwd(B, ctx, oracle, counts, N, K, swiglu):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, FP8_TOL
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets128(counts)
    R = int(off[-1])
    g = np.random.default_rng(N + K)
    Ah = wl.bf16_round((g.standard_normal((R, K)) * np.exp(g.uniform(-1, 1, (R, 1)))).astype(np.float32))
    for e, c in enumerate(counts):                     # padding rows are zero, as moe_permute leaves them
        Ah[off[e] + c: off[e + 1]] = 0.0
    Wh = wl.gaussian_bf16((E, N, K), 0.05, 61, N)
    qa, sa = _quant(B, ctx, dev_bf16(Ah), B.Q_1x128)
    qw, sw = _quant(B, ctx, dev_bf16(Wh), B.Q_128x128)
    C = torch.full((R, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    Act = torch.full((R, N // 2), float("nan"), dtype=torch.bfloat16, device="cuda") if swiglu else None
    B.moe_grouped_gemm_fwd(ctx, qa, qw, dev(off), E, N, K, R, B.FP8_E4M3, B.EPI_SWIGLU if swiglu else B.EPI_NONE,
                           sa, sw, C, Act)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    Ad = oracle.fp8_dequant(qa.cpu().numpy(), sa.cpu().numpy(), "1x128")
    Wd = oracle.fp8_dequant(qw.cpu().numpy(), sw.cpu().numpy(), "128x128")
    emu = oracle.grouped_gemm_nt(Ad, Wd, off)
    full = oracle.grouped_gemm_nt(Ah, Wh, off)
    got = host_f64(C)
    assert np.isfinite(got).all()
    assert rel_fro(got, emu) <= EMU_TOL
    assert rel_fro(got, full) <= FP8_TOL
    if swiglu:
        assert rel_fro(host_f64(Act), oracle.swiglu(emu)) <= 2 * EMU_TOL
        assert rel_fro(host_f64(Act), oracle.swiglu(full)) <= FP8_TOL


@pytest.mark.parametrize("counts,N,K,bwd", [
    ([300, 0, 257, 1, 700], 256, 512, False),
    ([130, 90], 128, 256, False),
    ([513, 128, 5], 384, 384, True),
])
def test_fp8_grouped_gemm_dgrad(B, ctx, oracle, counts, N, K, bwd):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, FP8_TOL
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets128(counts)
    R = int(off[-1])
    g = np.random.default_rng(N * 3 + K)
    dCh = wl.bf16_round((g.standard_normal((R, N)) * np.exp(g.uniform(-1, 1, (R, 1)))).astype(np.float32))
    for e, c in enumerate(counts):
        dCh[off[e] + c: off[e + 1]] = 0.0
    Wh = wl.gaussian_bf16((E, N, K), 0.05, 62, N)
    Zh = wl.gaussian_bf16((R, 2 * K), 1.5, 63, K) if bwd else None
    qd, sd = _quant(B, ctx, dev_bf16(dCh), B.Q_1x128)
    qw, sw = _quant(B, ctx, dev_bf16(Wh), B.Q_128x128)
    out = torch.full((R, 2 * K if bwd else K), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_dgrad(ctx, qd, qw, dev(off), E, N, K, R, B.FP8_E4M3, dev_bf16(Zh) if bwd else None, sd, sw, out)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    Dd = oracle.fp8_dequant(qd.cpu().numpy(), sd.cpu().numpy(), "1x128")
    Wd = oracle.fp8_dequant(qw.cpu().numpy(), sw.cpu().numpy(), "128x128")
    emu = oracle.grouped_gemm_nn(Dd, Wd, off)
    full = oracle.grouped_gemm_nn(dCh, Wh, off)
    if bwd:
        emu, full = oracle.swiglu_bwd(emu, Zh), oracle.swiglu_bwd(full, Zh)
    got = host_f64(out)
    assert np.isfinite(got).all()
    assert rel_fro(got, emu) <= (2 * EMU_TOL if bwd else EMU_TOL)
    assert rel_fro(got, full) <= FP8_TOL


def test_fp8_wgrad_is_refused(B, ctx):
    """fp8 weight gradients are not built: the call must fail loudly, not fall back."""
    z = torch.zeros((128, 128), dtype=torch.uint8, device="cuda")
    o = torch.zeros(2, dtype=torch.int32, device="cuda")
    with pytest.raises(B.MoeError):
        B.moe_grouped_gemm_wgrad(ctx, z, z, o, 1, 128, 128, 128, B.FP8_E4M3, None, None, 0, B.BF16, z)
