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


@pytest.mark.parametrize("rows,cols", [(256, 384), (640, 128), (1024, 2048)])
def test_quantize_rowcol_bit_exact(B, ctx, oracle, rows, cols):
    """Both blockwise copies from one pass over the input: each equal, bit for bit, to the oracle's separate 1x128 and
    128x1 quantisers; either copy alone; with a live-row count on the device, whole 128-row tiles beyond it are left
    alone; MOE_Q_128x1 through moe_fp8_quantize gives the same bits."""
    from gpu_util import dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(rows * 7 + cols)
    Xh = wl.bf16_round((g.standard_normal((rows, cols)) * np.exp(g.normal(size=(rows, cols)) * 2)).astype(np.float32))
    Xh[3, :128] = 0.0                      # an all-zero 1x128 block: scale 1, codes 0
    Xh[128:256, 5] = 0.0                   # an all-zero 128x1 block
    Xh[70, 40] = 448.0
    qr_o, sr_o = oracle.fp8_quant_1x128(Xh)
    qc_o, sc_o = oracle.fp8_quant_128x1(Xh)
    X = dev_bf16(Xh)
    for live_rows in (None, (rows // 256) * 128):
        qr = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
        sr = torch.zeros((rows, cols // 128), dtype=torch.float32, device="cuda")
        qc = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
        sc = torch.zeros((rows // 128, cols), dtype=torch.float32, device="cuda")
        live = None if live_rows is None else torch.tensor([live_rows], dtype=torch.int32, device="cuda")
        B.moe_fp8_quantize_rowcol(ctx, X, rows, cols, live, qr, sr, qc, sc)
        torch.cuda.synchronize()
        n = rows if live_rows is None else live_rows
        assert np.array_equal(qr.cpu().numpy()[:n], qr_o[:n]) and np.array_equal(sr.cpu().numpy()[:n], sr_o[:n])
        assert np.array_equal(qc.cpu().numpy()[:n], qc_o[:n]) and np.array_equal(sc.cpu().numpy()[:n // 128], sc_o[:n // 128])
        assert not qr[n:].any() and not qc[n:].any() and not sr[n:].any() and not sc[n // 128:].any()
    # one copy at a time
    qc = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
    sc = torch.zeros((rows // 128, cols), dtype=torch.float32, device="cuda")
    B.moe_fp8_quantize_rowcol(ctx, X, rows, cols, None, None, None, qc, sc)
    qr = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
    sr = torch.zeros((rows, cols // 128), dtype=torch.float32, device="cuda")
    B.moe_fp8_quantize_rowcol(ctx, X, rows, cols, None, qr, sr, None, None)
    q1, s1 = _quant(B, ctx, X, B.Q_128x1)
    torch.cuda.synchronize()
    assert np.array_equal(qc.cpu().numpy(), qc_o) and np.array_equal(sc.cpu().numpy(), sc_o)
    assert np.array_equal(qr.cpu().numpy(), qr_o) and np.array_equal(sr.cpu().numpy(), sr_o)
    assert np.array_equal(q1.cpu().numpy(), qc_o) and np.array_equal(s1.cpu().numpy(), sc_o)
    with pytest.raises(B.MoeError):
        B.moe_fp8_quantize_rowcol(ctx, X, rows, cols, None, qr, None, None, None)


@pytest.mark.parametrize("with_scale", [False, True])
def test_quantize_rowcol_gather_bit_exact(B, ctx, oracle, with_scale):
    """Blockwise quantisation fused into the permute (padding rows included) and into the combine's backward: the
    virtual tensor V[r] = (bf16(p[s] *)) X[s / k], s = src_of[r], zero where s < 0, quantised 1x128 and 128x1 without
    being stored."""
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(21 + with_scale)
    T, k, E, cols = 300, 3, 5, 384
    idx = g.integers(0, E, size=(T, k)).astype(np.int32)
    m = oracle.permute_maps(idx, E, 128, None)
    Rcap = (T * k + E * 127 + 127) // 128 * 128
    src = np.full(Rcap, -1, np.int32)
    src[:len(m.src_of)] = m.src_of
    R = int(m.offsets[-1])
    Xh = wl.bf16_round((g.standard_normal((T, cols)) * np.exp(g.normal(size=(T, cols)))).astype(np.float32))
    p = g.uniform(0.05, 1.0, size=T * k).astype(np.float32)
    V = Xh[np.maximum(src, 0) // k]
    if with_scale:
        V = wl.bf16_round(p[np.maximum(src, 0)][:, None] * V)
    V[src < 0] = 0
    qr = torch.zeros((Rcap, cols), dtype=torch.uint8, device="cuda")
    sr = torch.zeros((Rcap, cols // 128), dtype=torch.float32, device="cuda")
    qc = torch.zeros((Rcap, cols), dtype=torch.uint8, device="cuda")
    sc = torch.zeros((Rcap // 128, cols), dtype=torch.float32, device="cuda")
    live = torch.tensor([R], dtype=torch.int32, device="cuda")
    src_dev = dev(src)
    if with_scale:  # the map as a view that starts 4 bytes off a 16-byte boundary (padding lanes read spare map bytes)
        buf = torch.empty(Rcap + 1, dtype=torch.int32, device="cuda")
        buf[1:].copy_(src_dev)
        src_dev = buf[1:]
    B.moe_fp8_quantize_rowcol_gather(ctx, dev_bf16(Xh), src_dev, k, dev(p) if with_scale else None, E if with_scale else 1,
                                     Rcap, cols, live, qr, sr, qc, sc)
    torch.cuda.synchronize()
    qr_o, sr_o = oracle.fp8_quant_1x128(V)
    qc_o, sc_o = oracle.fp8_quant_128x1(V)
    assert np.array_equal(qr.cpu().numpy()[:R], qr_o[:R]) and np.array_equal(sr.cpu().numpy()[:R], sr_o[:R])
    assert np.array_equal(qc.cpu().numpy()[:R], qc_o[:R]) and np.array_equal(sc.cpu().numpy()[:R // 128], sc_o[:R // 128])
    assert (src[:R] < 0).any() and not qr.cpu().numpy()[:R][src[:R] < 0].any()      # padding rows: zero codes
    assert not qr[R:].any() and not qc[R:].any()                                     # beyond the live rows: untouched


def test_quantisers_one_division_per_block_bit_exact(B, ctx, oracle):
    """The quantisers divide once per block (r = 1 / scale) and correct the product x r with the exact residual; that
    must give the bits of the fp32 division x / scale the recipe is defined with.  Inputs chosen against it: block
    maxima from far below the range in which the short form is used (those blocks must take the plain division, also
    when they share a wave with ordinary ones) up to the top of the bf16 range; elements on and next to the halfway
    points between neighbouring E4M3 values (where one unit in the last place of the quotient changes the code);
    denormal elements inside ordinary blocks; all four kernels (1x128, 128x1, both in one pass, 128x128)."""
    from gpu_util import dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(99)
    rows, cols = 1024, 1024
    # E4M3 values and the midpoints between neighbours, as multiples of amax / 448
    e4 = np.array(sorted({(1 + m / 8) * 2.0 ** e for e in range(-6, 9) for m in range(8)} | {m / 8 * 2.0 ** -6 for m in range(8)}))
    e4 = e4[e4 <= 448]
    mids = (e4[1:] + e4[:-1]) / 2
    pts = np.concatenate([e4, mids, mids * (1 + 2.0 ** -8), mids * (1 - 2.0 ** -8)])
    X = g.choice(pts, size=(rows, cols)) * g.choice([-1.0, 1.0], size=(rows, cols)) / 448.0
    X = X * (1 + g.uniform(-1, 1, size=(rows, cols)) * 2.0 ** g.integers(-20, -6, size=(rows, cols)))   # small nudges
    # per 128x128 tile a magnitude: 2^-120 .. 2^126 (the short form is used from about 2^-31 up)
    mag = 2.0 ** g.choice([-120.0, -60.0, -41.0, -32.0, -31.0, -30.0, -10.0, 0.0, 3.0, 40.0, 100.0, 126.0], size=(rows // 128, cols // 128))
    X = X * np.kron(mag, np.ones((128, 128)))
    X[:, ::7] *= 448.0                                   # most rows and columns reach their block maximum somewhere
    X[5::64, 3::32] = 1e-40                              # denormal elements inside ordinary blocks
    X[256:384, 128:256] = 0.0                            # an all-zero tile
    with np.errstate(over="ignore"):
        Xh = wl.bf16_round(np.clip(X, -3e38, 3e38).astype(np.float32))
    Xd = dev_bf16(Xh)
    q, s = _quant(B, ctx, Xd, B.Q_1x128)
    qo, so = oracle.fp8_quant_1x128(Xh)
    assert np.array_equal(s.cpu().numpy(), so) and np.array_equal(q.cpu().numpy(), qo)
    q, s = _quant(B, ctx, Xd, B.Q_128x1)
    qc_o, sc_o = oracle.fp8_quant_128x1(Xh)
    assert np.array_equal(s.cpu().numpy(), sc_o) and np.array_equal(q.cpu().numpy(), qc_o)
    qr = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
    sr = torch.zeros((rows, cols // 128), dtype=torch.float32, device="cuda")
    qc = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
    sc = torch.zeros((rows // 128, cols), dtype=torch.float32, device="cuda")
    B.moe_fp8_quantize_rowcol(ctx, Xd, rows, cols, None, qr, sr, qc, sc)
    torch.cuda.synchronize()
    assert np.array_equal(qr.cpu().numpy(), qo) and np.array_equal(sr.cpu().numpy(), so)
    assert np.array_equal(qc.cpu().numpy(), qc_o) and np.array_equal(sc.cpu().numpy(), sc_o)
    W = Xh.reshape(1, rows, cols)
    q, s = _quant(B, ctx, dev_bf16(W), B.Q_128x128)
    torch.cuda.synchronize()
    qw_o, sw_o = oracle.fp8_quant_128x128(W)
    assert np.array_equal(s.cpu().numpy(), sw_o) and np.array_equal(q.cpu().numpy(), qw_o)
    # the inputs do what they were made for: codes of every magnitude class, blocks on both sides of the range
    assert len(np.unique(qo)) > 200 and (so < 2.0 ** -40).any() and (so > 2.0 ** 100).any()


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
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, FP8_TOL
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
    assert_close(got, emu, "vs emulation", tol=EMU_TOL, reg=None, row_tol=2e-2)     # every row: no wrong or mis-scaled row
    assert_close(got, full, "vs full precision", tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)
    if swiglu:
        assert_close(host_f64(Act), oracle.swiglu(emu), "A vs emulation", tol=2 * EMU_TOL, reg=None, row_tol=2e-2)
        assert_close(host_f64(Act), oracle.swiglu(full), "A vs full precision", tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)


@pytest.mark.parametrize("counts,N,K,bwd", [
    ([300, 0, 257, 1, 700], 256, 512, False),
    ([130, 90], 128, 256, False),
    ([513, 128, 5], 384, 384, True),
])
def test_fp8_grouped_gemm_dgrad(B, ctx, oracle, counts, N, K, bwd):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, FP8_TOL
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
    assert_close(got, emu, "vs emulation", tol=(2 * EMU_TOL if bwd else EMU_TOL), reg=None, row_tol=2e-2)
    assert_close(got, full, "vs full precision", tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)


@pytest.mark.parametrize("counts,N,K", [
    ([300, 0, 257, 1, 700], 512, 256),        # ragged experts (zero padding rows), an empty one, a one-row one
    ([128, 128], 128, 128),                   # one stage each, output smaller than a tile
    ([1300, 40, 0, 2049], 384, 640),          # odd and even stage counts, ragged output tiles in both directions
])
@pytest.mark.parametrize("out_f32", [False, True])
def test_fp8_grouped_gemm_wgrad(B, ctx, oracle, counts, N, K, out_f32):
    """Blockwise-fp8 weight gradient (Sec. 5.3.2; the 1x128 tiles run down the token dimension inside each expert's
    128-aligned row range, Sec. 5.4.1): dW_e = dC_e^T A_e from E4M3 codes with 128x1 fp32 scales on both operands,
    against the oracle's quantise-dequantise emulation (accumulation order and output rounding only) and against
    full precision (the format's noise).  The magnitude changes from row block to row block by up to e^8, so the
    per-stage rescaling of the accumulators is exercised in both directions."""
    from gpu_util import dev, dev_bf16, host_f64, assert_close, FP8_TOL
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets128(counts)
    R = int(off[-1])
    g = np.random.default_rng(N + 7 * K)
    mag = np.repeat(np.exp(g.uniform(-4, 4, (R // 128, 1))), 128, axis=0)
    dCh = wl.bf16_round((g.standard_normal((R, N)) * mag).astype(np.float32))
    Ah = wl.bf16_round((g.standard_normal((R, K)) * mag[::-1]).astype(np.float32))
    for e, c in enumerate(counts):                     # padding rows are zero, as moe_permute leaves them
        dCh[off[e] + c: off[e + 1]] = 0.0
        Ah[off[e] + c: off[e + 1]] = 0.0
    qd, sd = _quant(B, ctx, dev_bf16(dCh), B.Q_128x1)
    qa, sa = _quant(B, ctx, dev_bf16(Ah), B.Q_128x1)
    tdt = torch.float32 if out_f32 else torch.bfloat16
    dW = torch.full((E, N, K), float("nan"), dtype=tdt, device="cuda")
    odt = B.F32 if out_f32 else B.BF16
    doff = dev(off)
    B.moe_grouped_gemm_wgrad(ctx, qa, qd, doff, E, N, K, R, B.FP8_E4M3, sa, sd, 0, odt, dW)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    Dd = oracle.fp8_dequant(qd.cpu().numpy(), sd.cpu().numpy(), "128x1")
    Ad = oracle.fp8_dequant(qa.cpu().numpy(), sa.cpu().numpy(), "128x1")
    emu = oracle.grouped_gemm_tn(Dd, Ad, off)
    full = oracle.grouped_gemm_tn(dCh, Ah, off)
    got = host_f64(dW)
    assert np.isfinite(got).all()
    # (fp32 output: what is left is the matrix instruction's own accumulation of the 128 products of a stage, measured
    # at 1e-5 of the result, and the two roundings of the per-stage rescaling)
    assert_close(got, emu, "vs emulation", tol=(1e-4 if out_f32 else EMU_TOL), reg=None, row_tol=(1e-3 if out_f32 else 2e-2))
    assert_close(got, full, "vs full precision", tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)
    for e, c in enumerate(counts):
        if c == 0:
            assert np.all(got[e] == 0)                                  # zero-token expert: exact zeros
    # accumulate: dW += result
    B.moe_grouped_gemm_wgrad(ctx, qa, qd, doff, E, N, K, R, B.FP8_E4M3, sa, sd, 1, odt, dW)
    torch.cuda.synchronize()
    assert_close(host_f64(dW), 2 * emu, "accumulated", tol=(1e-4 if out_f32 else 2 * EMU_TOL), reg=None,
                 row_tol=(1e-3 if out_f32 else 2e-2))


def test_fp8_wgrad_needs_aligned_experts_and_scales(B, ctx):
    """A 128-row scale block must not straddle two experts: offsets that are not multiples of 128 raise the device
    error word and leave dW untouched; missing scale arrays are an argument error."""
    from gpu_util import dev
    qa = torch.zeros((256, 128), dtype=torch.uint8, device="cuda")
    qd = torch.zeros((256, 128), dtype=torch.uint8, device="cuda")
    sa = torch.ones((2, 128), dtype=torch.float32, device="cuda")
    dW = torch.full((2, 128, 128), 7.0, dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_wgrad(ctx, qa, qd, dev(np.array([0, 100, 256], np.int32)), 2, 128, 128, 256, B.FP8_E4M3, sa, sa, 0,
                             B.BF16, dW)
    assert ctx.poll_error() == 1
    assert ctx.poll_error() == 0
    assert (dW == 7.0).all()
    with pytest.raises(B.MoeError):
        B.moe_grouped_gemm_wgrad(ctx, qa, qd, dev(np.array([0, 128, 256], np.int32)), 2, 128, 128, 256, B.FP8_E4M3, None,
                                 None, 0, B.BF16, dW)


def test_fp8_block_scales_24_decades_apart(B, ctx, oracle):
    """The accumulators of the blockwise GEMMs are carried in units of the current block's scales: consecutive
    blocks whose scale products differ by 1e24 in either direction (the documented limit is 2^100) must neither
    overflow nor lose the large blocks.  Forward (row scale x weight-block scale) and weight gradient (row scale x
    column scale of the two 128x1-quantised operands), against the oracle's quantise-dequantise emulation."""
    from gpu_util import dev, dev_bf16, host_f64, assert_close
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(2024)
    E, R, N, K = 2, 512, 256, 512
    off = np.array([0, 256, 512], np.int32)
    # forward: contraction blocks alternate between 1e6 and 1e-6 in both operands; some rows start small, some big
    kmag = np.where(np.arange(K // 128) % 2 == 0, 1e6, 1e-6).repeat(128)
    flip = np.where(np.arange(R) % 3 == 0, 1.0, 0.0)[:, None]
    amag = np.where(flip > 0, kmag[::-1][None, :], kmag[None, :])
    Ah = wl.bf16_round((g.standard_normal((R, K)) * amag).astype(np.float32))
    Wh = wl.bf16_round((g.standard_normal((E, N, K)) * kmag[None, None, :]).astype(np.float32))
    qa, sa = _quant(B, ctx, dev_bf16(Ah), B.Q_1x128)
    qw, sw = _quant(B, ctx, dev_bf16(Wh), B.Q_128x128)
    C = torch.full((R, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_fwd(ctx, qa, qw, dev(off), E, N, K, R, B.FP8_E4M3, B.EPI_NONE, sa, sw, C, None)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    emu = oracle.grouped_gemm_nt(oracle.fp8_dequant(qa.cpu().numpy(), sa.cpu().numpy(), "1x128"),
                                 oracle.fp8_dequant(qw.cpu().numpy(), sw.cpu().numpy(), "128x128"), off)
    assert_close(host_f64(C), emu, "forward, 1e24 between blocks", tol=EMU_TOL, reg=None, row_tol=2e-2)
    # weight gradient: 128-row blocks alternate between 1e6 and 1e-6 in both operands
    rmag = np.where(np.arange(R // 128) % 2 == 0, 1e6, 1e-6).repeat(128)[:, None]
    dCh = wl.bf16_round((g.standard_normal((R, N)) * rmag).astype(np.float32))
    A2 = wl.bf16_round((g.standard_normal((R, K)) * rmag).astype(np.float32))
    qd, sd = _quant(B, ctx, dev_bf16(dCh), B.Q_128x1)
    q2, s2 = _quant(B, ctx, dev_bf16(A2), B.Q_128x1)
    dW = torch.full((E, N, K), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_grouped_gemm_wgrad(ctx, q2, qd, dev(off), E, N, K, R, B.FP8_E4M3, s2, sd, 0, B.F32, dW)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    emu = oracle.grouped_gemm_tn(oracle.fp8_dequant(qd.cpu().numpy(), sd.cpu().numpy(), "128x1"),
                                 oracle.fp8_dequant(q2.cpu().numpy(), s2.cpu().numpy(), "128x1"), off)
    assert_close(host_f64(dW), emu, "weight gradient, 1e24 between blocks", tol=1e-4, reg=None, row_tol=1e-3)
