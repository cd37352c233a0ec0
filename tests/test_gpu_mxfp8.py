"""GPU parity of the MXFP8 path (Sec. 5.3.3): E4M3 elements, 1x32 blocks, E8M0 scales applied by the matrix
instruction.  Quantisers bit-exact against the oracle; grouped GEMMs against the oracle's own
quantise-dequantise emulation (tight: accumulation order and bf16 output rounding only) and against the
full-precision result (6e-2)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

EMU_TOL = 4e-3


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


def _col_scales(e, G, N, K):
    """Column-wise E8M0 scales as the library stores them, [G*N/128, K, 4], in the oracle's order [G, K, N/32]."""
    e = e.cpu().numpy() if hasattr(e, "cpu") else e
    return np.ascontiguousarray(e.reshape(G, N // 128, K, 4).transpose(0, 2, 1, 3).reshape(G, K, N // 32))


def _mxq(B, ctx, X, kind, rows_dev=None):
    """X: device bf16 [rows, cols] (1x32) or [G, N, K] (32x1).  Returns (codes, e8m0) device tensors."""
    if kind == B.MX_1x32:
        rows, cols = X.shape
        q = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
        e = torch.zeros((rows, cols // 32), dtype=torch.uint8, device="cuda")
        B.moe_mx_quantize(ctx, X, kind, 1, rows, cols, rows_dev, q, e)
    else:
        G, N, K = X.shape
        q = torch.zeros((G, N, K), dtype=torch.uint8, device="cuda")
        e = torch.zeros((G * N // 128, K, 4), dtype=torch.uint8, device="cuda")
        B.moe_mx_quantize(ctx, X, kind, G, N, K, rows_dev, q, e)
    return q, e


@pytest.mark.parametrize("rows,cols", [(256, 384), (1000, 32), (77, 7168)])
def test_mx_quantize_1x32_bit_exact(B, ctx, oracle, rows, cols):
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(rows + cols)
    Xh = wl.bf16_round((g.standard_normal((rows, cols)) * np.exp(g.normal(size=(rows, cols)) * 2)).astype(np.float32))
    Xh[3, :32] = 0.0
    Xh[5, 0] = 448.0
    Xh[5, 1:32] = 1.0
    q, e = _mxq(B, ctx, dev_bf16(Xh), B.MX_1x32)
    torch.cuda.synchronize()
    qo, eo = oracle.mx_quant_1x32(Xh)
    assert np.array_equal(e.cpu().numpy(), eo)
    assert np.array_equal(q.cpu().numpy(), qo)
    # live-row count on the device: rows beyond it are left alone
    live = torch.tensor([rows // 2], dtype=torch.int32, device="cuda")
    q2, e2 = _mxq(B, ctx, dev_bf16(Xh), B.MX_1x32, live)
    torch.cuda.synchronize()
    assert np.array_equal(q2.cpu().numpy()[:rows // 2], qo[:rows // 2]) and not q2[rows // 2:].any()


def test_mx_quantize_32x1_bit_exact(B, ctx, oracle):
    from gpu_util import dev_bf16
    from paper_2603_07685_amd import workloads as wl
    Wh = wl.gaussian_bf16((3, 256, 1152), 0.02, 5, 1)
    Wh[1, 32:64, :100] = 0.0
    q, e = _mxq(B, ctx, dev_bf16(Wh), B.MX_32x1)
    torch.cuda.synchronize()
    qo, eo = oracle.mx_quant_32x1(Wh)
    assert np.array_equal(_col_scales(e, 3, 256, 1152), eo) and np.array_equal(q.cpu().numpy(), qo)


@pytest.mark.parametrize("rows,cols", [(128, 128), (640, 384), (256, 7168)])
def test_mx_quantize_rowcol_bit_exact(B, ctx, oracle, rows, cols):
    """Both copies from one pass over the input: each equal, bit for bit, to the oracle's separate quantisers; with a
    live-row count on the device, whole 128-row tiles beyond it are left alone."""
    from gpu_util import dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(rows * 7 + cols)
    Xh = wl.bf16_round((g.standard_normal((rows, cols)) * np.exp(g.normal(size=(rows, cols)) * 2)).astype(np.float32))
    Xh[3, :32] = 0.0
    Xh[32:64, 5] = 0.0
    Xh[70, 40] = 448.0
    qr_o, er_o = oracle.mx_quant_1x32(Xh)
    qc_o, ec_o = oracle.mx_quant_32x1(Xh[None])
    for live_rows in (None, (rows // 256) * 128):
        qr = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
        er = torch.zeros((rows, cols // 32), dtype=torch.uint8, device="cuda")
        qc = torch.zeros((rows, cols), dtype=torch.uint8, device="cuda")
        ec = torch.zeros((rows // 128, cols, 4), dtype=torch.uint8, device="cuda")
        live = None if live_rows is None else torch.tensor([live_rows], dtype=torch.int32, device="cuda")
        B.moe_mx_quantize_rowcol(ctx, dev_bf16(Xh), rows, cols, live, qr, er, qc, ec)
        torch.cuda.synchronize()
        n = rows if live_rows is None else live_rows
        assert np.array_equal(qr.cpu().numpy()[:n], qr_o[:n]) and np.array_equal(er.cpu().numpy()[:n], er_o[:n])
        assert np.array_equal(qc.cpu().numpy()[:n], qc_o[0, :n])
        assert np.array_equal(_col_scales(ec, 1, rows, cols)[0, :, :n // 32], ec_o[0, :, :n // 32])
        assert not qr[n:].any() and not qc[n:].any() and not er[n:].any() and not ec[n // 128:].any()


@pytest.mark.parametrize("with_scale", [False, True])
def test_mx_quantize_rowcol_gather_bit_exact(B, ctx, oracle, with_scale):
    """Quantisation fused into the permute (padding rows included) and into the combine's backward: the virtual
    tensor V[r] = (bf16(p[s] *)) X[s / k], s = src_of[r], zero where s < 0, quantised both ways without being stored."""
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(11 + with_scale)
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
    er = torch.zeros((Rcap, cols // 32), dtype=torch.uint8, device="cuda")
    qc = torch.zeros((Rcap, cols), dtype=torch.uint8, device="cuda")
    ec = torch.zeros((Rcap // 128, cols, 4), dtype=torch.uint8, device="cuda")
    live = torch.tensor([R], dtype=torch.int32, device="cuda")
    src_dev = dev(src)
    if with_scale:  # the map as a view that starts 4 bytes off a 16-byte boundary (padding lanes read spare map bytes)
        buf = torch.empty(Rcap + 1, dtype=torch.int32, device="cuda")
        buf[1:].copy_(src_dev)
        src_dev = buf[1:]
    B.moe_mx_quantize_rowcol_gather(ctx, dev_bf16(Xh), src_dev, k, dev(p) if with_scale else None, E if with_scale else 1,
                                    Rcap, cols, live, qr, er, qc, ec)
    torch.cuda.synchronize()
    qr_o, er_o = oracle.mx_quant_1x32(V)
    qc_o, ec_o = oracle.mx_quant_32x1(V[None])
    assert np.array_equal(qr.cpu().numpy()[:R], qr_o[:R]) and np.array_equal(er.cpu().numpy()[:R], er_o[:R])
    assert np.array_equal(qc.cpu().numpy()[:R], qc_o[0, :R])
    assert np.array_equal(_col_scales(ec, 1, Rcap, cols)[0, :, :R // 32], ec_o[0, :, :R // 32])
    assert (src[:R] < 0).any() and not qr.cpu().numpy()[:R][src[:R] < 0].any()      # padding rows: zero codes
    assert not qr[R:].any() and not qc[R:].any()                                     # beyond the live rows: untouched


def _offsets128(counts):
    pad = (np.asarray(counts) + 127) // 128 * 128
    return np.concatenate([[0], np.cumsum(pad)]).astype(np.int32)


@pytest.mark.parametrize("counts,N,K,swiglu", [
    ([300, 0, 257, 1, 700], 512, 256, False),
    ([130, 90], 256, 128, False),
    ([513, 128, 5], 768, 384, True),
    ([300, 0, 257, 1, 700], 512, 256, True),
])
def test_mx_grouped_gemm_fwd(B, ctx, oracle, counts, N, K, swiglu):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, FP8_TOL
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets128(counts)
    R = int(off[-1])
    g = np.random.default_rng(N + K)
    # per-element magnitudes spread over a few octaves so that neighbouring 32-blocks get different scales
    Ah = wl.bf16_round((g.standard_normal((R, K)) * np.exp(g.uniform(-2, 2, (R, K // 32)).repeat(32, axis=1))).astype(np.float32))
    for e, c in enumerate(counts):
        Ah[off[e] + c: off[e + 1]] = 0.0
    Wh = wl.bf16_round((g.standard_normal((E, N, K)) * 0.05 * np.exp(g.uniform(-2, 2, (E, N, K // 32)).repeat(32, axis=2))).astype(np.float32))
    qa, ea = _mxq(B, ctx, dev_bf16(Ah), B.MX_1x32)
    qw, ew = _mxq(B, ctx, dev_bf16(Wh.reshape(E * N, K)), B.MX_1x32)
    C = torch.full((R, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    Act = torch.full((R, N // 2), float("nan"), dtype=torch.bfloat16, device="cuda") if swiglu else None
    B.moe_grouped_gemm_fwd(ctx, qa, qw, dev(off), E, N, K, R, B.MXFP8_E4M3, B.EPI_SWIGLU if swiglu else B.EPI_NONE,
                           ea, ew, C, Act)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    Ad = oracle.mx_dequant(qa.cpu().numpy(), ea.cpu().numpy(), "1x32")
    Wd = oracle.mx_dequant(qw.cpu().numpy(), ew.cpu().numpy(), "1x32").reshape(E, N, K)
    emu = oracle.grouped_gemm_nt(Ad, Wd, off)
    full = oracle.grouped_gemm_nt(Ah, Wh, off)
    got = host_f64(C)
    assert np.isfinite(got).all()
    assert_close(got, emu, "vs emulation", tol=EMU_TOL, reg=None, row_tol=2e-2)
    assert_close(got, full, "vs full precision", tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)
    if swiglu:
        assert_close(host_f64(Act), oracle.swiglu(emu), "A vs emulation", tol=2 * EMU_TOL, reg=None, row_tol=2e-2)
        assert_close(host_f64(Act), oracle.swiglu(full), "A vs full precision", tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)


@pytest.mark.parametrize("counts,N,K,bwd", [
    ([300, 0, 257, 1, 700], 256, 512, False),
    ([130, 90], 128, 256, False),
    ([513, 128, 5], 384, 384, True),
])
def test_mx_grouped_gemm_dgrad(B, ctx, oracle, counts, N, K, bwd):
    """Data gradient: dC quantised along N (row-wise), the weights along N too (the column-wise copy)."""
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, FP8_TOL
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets128(counts)
    R = int(off[-1])
    g = np.random.default_rng(N * 3 + K)
    dCh = wl.bf16_round((g.standard_normal((R, N)) * np.exp(g.uniform(-2, 2, (R, N // 32)).repeat(32, axis=1))).astype(np.float32))
    for e, c in enumerate(counts):
        dCh[off[e] + c: off[e + 1]] = 0.0
    Wh = wl.bf16_round((g.standard_normal((E, N, K)) * 0.05 * np.exp(g.uniform(-2, 2, (E, N // 32, K)).repeat(32, axis=1))).astype(np.float32))
    qd, ed = _mxq(B, ctx, dev_bf16(dCh), B.MX_1x32)
    qw, ew = _mxq(B, ctx, dev_bf16(Wh), B.MX_32x1)
    Zh = wl.gaussian_bf16((R, 2 * K), 1.5, 35, K) if bwd else None
    out = torch.full((R, 2 * K if bwd else K), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_dgrad(ctx, qd, qw, dev(off), E, N, K, R, B.MXFP8_E4M3, dev_bf16(Zh) if bwd else None, ed, ew, out)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    dCd = oracle.mx_dequant(qd.cpu().numpy(), ed.cpu().numpy(), "1x32")
    Wd = oracle.mx_dequant(qw.cpu().numpy(), _col_scales(ew, E, N, K), "32x1")
    emu = oracle.grouped_gemm_nn(dCd, Wd, off)
    full = oracle.grouped_gemm_nn(dCh, Wh, off)
    if bwd:
        emu, full = oracle.swiglu_bwd(emu, Zh), oracle.swiglu_bwd(full, Zh)
    got = host_f64(out)
    assert np.isfinite(got).all()
    assert_close(got, emu, "vs emulation", tol=EMU_TOL, reg=None, row_tol=2e-2)
    assert_close(got, full, "vs full precision", tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)


@pytest.mark.parametrize("counts,N,K,out_f32,acc", [
    ([300, 0, 257, 1, 700], 256, 512, False, False),
    ([130, 90], 128, 256, True, True),
    ([513, 128, 5], 384, 640, False, True),
    ([0, 0, 1024], 512, 128, True, False),
])
def test_mx_grouped_gemm_wgrad(B, ctx, oracle, counts, N, K, out_f32, acc):
    """Weight gradient: both operands quantised down the token dimension (32x1), every expert's range a multiple
    of 128 rows.  An expert without rows gets zeros (or keeps its old value when accumulating)."""
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, FP8_TOL
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets128(counts)
    R = int(off[-1])
    g = np.random.default_rng(N * 5 + K)
    Ah = wl.bf16_round((g.standard_normal((R, K)) * np.exp(g.uniform(-2, 2, (R // 32, K)).repeat(32, axis=0))).astype(np.float32))
    dCh = wl.bf16_round((g.standard_normal((R, N)) * np.exp(g.uniform(-2, 2, (R // 32, N)).repeat(32, axis=0))).astype(np.float32))
    for e, c in enumerate(counts):
        Ah[off[e] + c: off[e + 1]] = 0.0
        dCh[off[e] + c: off[e + 1]] = 0.0
    qa, ea = _mxq(B, ctx, dev_bf16(Ah[None]), B.MX_32x1)
    qd, ed = _mxq(B, ctx, dev_bf16(dCh[None]), B.MX_32x1)
    odt = torch.float32 if out_f32 else torch.bfloat16
    old = wl.gaussian_bf16((E, N, K), 1.0, 77, N)
    dW = torch.tensor(old, dtype=odt, device="cuda") if acc else torch.full((E, N, K), float("nan"), dtype=odt, device="cuda")
    B.moe_grouped_gemm_wgrad(ctx, qa[0], qd[0], dev(off), E, N, K, R, B.MXFP8_E4M3, ea, ed, int(acc),
                             B.F32 if out_f32 else B.BF16, dW)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    Ad = oracle.mx_dequant(qa.cpu().numpy(), _col_scales(ea, 1, R, K), "32x1")[0]
    dCd = oracle.mx_dequant(qd.cpu().numpy(), _col_scales(ed, 1, R, N), "32x1")[0]
    emu = oracle.grouped_gemm_tn(dCd, Ad, off)
    full = oracle.grouped_gemm_tn(dCh, Ah, off)
    got = host_f64(dW)
    assert np.isfinite(got).all()
    if acc:
        got = got - old.astype(np.float64)
        for e in range(E):
            if off[e + 1] == off[e]:
                assert not got[e].any()
    assert_close(got, emu, "vs emulation", tol=(EMU_TOL if not acc or out_f32 else 2e-2), reg=None, row_tol=2e-2)   # bf16 accumulate rounds old + new
    assert_close(got, full, "vs full precision", tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)


def test_mx_wgrad_rejects_ranges_off_the_block_grid(B, ctx):
    """Expert ranges that do not start and end on multiples of 128 rows: the call raises the error word and leaves
    dB alone (a scale block would straddle two experts)."""
    from gpu_util import dev
    R = 512
    q = torch.zeros((R, 128), dtype=torch.uint8, device="cuda")
    e = torch.full((R // 128, 128, 4), 127, dtype=torch.uint8, device="cuda")
    dW = torch.full((2, 128, 128), 3.0, dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_wgrad(ctx, q, q, dev(np.array([0, 200, 512], np.int32)), 2, 128, 128, R, B.MXFP8_E4M3, e, e, 0,
                             B.BF16, dW)
    torch.cuda.synchronize()
    assert ctx.poll_error() != 0
    assert (dW == 3.0).all()


@pytest.mark.parametrize("counts,N,K,weighted,col", [
    ([300, 0, 257, 1, 700], 512, 256, False, True),
    ([513, 128, 5], 768, 384, True, True),
    ([130, 90], 256, 128, True, False),
])
def test_mx_quantising_epilogue_fwd_bit_exact(B, ctx, oracle, counts, N, K, weighted, col):
    """fc1 with the SwiGLU epilogue that also quantises (Sec. 5.4.2): Z and A are the plain call's bits, and the
    1x32 / 32x1 copies are the oracle's quantisers applied to the stored A, bit for bit; rows beyond offsets[E]
    are left alone."""
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets128(counts)
    R = int(off[-1])
    Rcap = R + 128
    g = np.random.default_rng(N + K + 1)
    Ah = wl.bf16_round((g.standard_normal((Rcap, K)) * np.exp(g.uniform(-2, 2, (Rcap, K // 32)).repeat(32, axis=1))).astype(np.float32))
    for e, c in enumerate(counts):
        Ah[off[e] + c: off[e + 1]] = 0.0
    Wh = wl.bf16_round((g.standard_normal((E, N, K)) * 0.05 * np.exp(g.uniform(-2, 2, (E, N, K // 32)).repeat(32, axis=2))).astype(np.float32))
    qa, ea = _mxq(B, ctx, dev_bf16(Ah), B.MX_1x32)
    qw, ew = _mxq(B, ctx, dev_bf16(Wh.reshape(E * N, K)), B.MX_1x32)
    rp = dev(g.uniform(0.05, 1.0, Rcap).astype(np.float32)) if weighted else None
    f = N // 2
    C0 = torch.zeros((Rcap, N), dtype=torch.bfloat16, device="cuda")
    A0 = torch.zeros((Rcap, f), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_fwd_weighted(ctx, qa, qw, dev(off), E, N, K, Rcap, B.MXFP8_E4M3, B.EPI_SWIGLU, ea, ew, rp, C0, A0)
    C1, A1 = torch.zeros_like(C0), torch.zeros_like(A0)
    qr = torch.full((Rcap, f), 7, dtype=torch.uint8, device="cuda")
    er = torch.full((Rcap, f // 32), 7, dtype=torch.uint8, device="cuda")
    qc = torch.full((Rcap, f), 7, dtype=torch.uint8, device="cuda") if col else None
    ec = torch.full((Rcap // 128, f, 4), 7, dtype=torch.uint8, device="cuda") if col else None
    B.moe_grouped_gemm_fwd_quant_mx(ctx, qa, qw, dev(off), E, N, K, Rcap, ea, ew, rp, C1, A1, qr, er, qc, ec)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    assert torch.equal(C0.view(torch.int16), C1.view(torch.int16)) and torch.equal(A0.view(torch.int16), A1.view(torch.int16))
    Ast = A1.float().cpu().numpy()
    qr_o, er_o = oracle.mx_quant_1x32(Ast)
    assert np.array_equal(er.cpu().numpy()[:R], er_o[:R]) and np.array_equal(qr.cpu().numpy()[:R], qr_o[:R])
    assert (qr[R:] == 7).all() and (er[R:] == 7).all()
    if col:
        qc_o, ec_o = oracle.mx_quant_32x1(Ast[None])
        assert np.array_equal(_col_scales(ec, 1, Rcap, f)[0, :, :R // 32], ec_o[0, :, :R // 32])
        assert np.array_equal(qc.cpu().numpy()[:R], qc_o[0, :R])
        assert (qc[R:] == 7).all() and (ec[R // 128:] == 7).all()


@pytest.mark.parametrize("counts,N,K,weighted,col", [
    ([300, 0, 257, 1, 700], 256, 512, False, True),
    ([513, 128, 5], 384, 384, True, True),
    ([130, 90], 128, 256, True, False),
])
def test_mx_quantising_epilogue_dgrad_bit_exact(B, ctx, oracle, counts, N, K, weighted, col):
    """fc2 data gradient with the SwiGLU-backward epilogue that also quantises dZ: dZ and the dprob partials are
    the plain call's bits, the two quantised copies the oracle's quantisers applied to the stored dZ."""
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets128(counts)
    R = int(off[-1])
    Rcap = R + 128
    g = np.random.default_rng(N * 3 + K + 1)
    dCh = wl.bf16_round((g.standard_normal((Rcap, N)) * np.exp(g.uniform(-2, 2, (Rcap, N // 32)).repeat(32, axis=1))).astype(np.float32))
    for e, c in enumerate(counts):
        dCh[off[e] + c: off[e + 1]] = 0.0
    Wh = wl.bf16_round((g.standard_normal((E, N, K)) * 0.05 * np.exp(g.uniform(-2, 2, (E, N // 32, K)).repeat(32, axis=1))).astype(np.float32))
    qd, ed = _mxq(B, ctx, dev_bf16(dCh), B.MX_1x32)
    qw, ew = _mxq(B, ctx, dev_bf16(Wh), B.MX_32x1)
    Z = dev_bf16(wl.gaussian_bf16((Rcap, 2 * K), 1.5, 35, K))
    rp = dev(g.uniform(0.05, 1.0, Rcap).astype(np.float32)) if weighted else None
    parts = 2 * ((K + 255) // 256)
    dZ0 = torch.zeros((Rcap, 2 * K), dtype=torch.bfloat16, device="cuda")
    dp0 = torch.zeros((Rcap, parts), dtype=torch.float32, device="cuda") if weighted else None
    B.moe_grouped_gemm_dgrad_weighted(ctx, qd, qw, dev(off), E, N, K, Rcap, B.MXFP8_E4M3, Z, ed, ew, rp, dZ0, dp0)
    dZ1 = torch.zeros_like(dZ0)
    dp1 = torch.zeros_like(dp0) if weighted else None
    qr = torch.full((Rcap, 2 * K), 7, dtype=torch.uint8, device="cuda")
    er = torch.full((Rcap, 2 * K // 32), 7, dtype=torch.uint8, device="cuda")
    qc = torch.full((Rcap, 2 * K), 7, dtype=torch.uint8, device="cuda") if col else None
    ec = torch.full((Rcap // 128, 2 * K, 4), 7, dtype=torch.uint8, device="cuda") if col else None
    B.moe_grouped_gemm_dgrad_quant_mx(ctx, qd, qw, dev(off), E, N, K, Rcap, Z, ed, ew, rp, dZ1, dp1, qr, er, qc, ec)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    assert torch.equal(dZ0.view(torch.int16), dZ1.view(torch.int16))
    if weighted:
        assert torch.equal(dp0, dp1)
    Zst = dZ1.float().cpu().numpy()
    qr_o, er_o = oracle.mx_quant_1x32(Zst)
    assert np.array_equal(er.cpu().numpy()[:R], er_o[:R]) and np.array_equal(qr.cpu().numpy()[:R], qr_o[:R])
    assert (qr[R:] == 7).all() and (er[R:] == 7).all()
    if col:
        qc_o, ec_o = oracle.mx_quant_32x1(Zst[None])
        assert np.array_equal(_col_scales(ec, 1, Rcap, 2 * K)[0, :, :R // 32], ec_o[0, :, :R // 32])
        assert np.array_equal(qc.cpu().numpy()[:R], qc_o[0, :R])
        assert (qc[R:] == 7).all() and (ec[R // 128:] == 7).all()


def test_mx_quantising_epilogue_rejects_bad_requests(B, ctx):
    """No row-wise outputs, the wrong epilogue, or a capacity off the 128-row grid with the 32x1 copy: refused on the
    host; expert ranges off the grid with the 32x1 copy: the device error word."""
    from gpu_util import dev
    R, N, K = 512, 256, 128
    q = torch.zeros((R, K), dtype=torch.uint8, device="cuda")
    e = torch.full((R, K // 32), 127, dtype=torch.uint8, device="cuda")
    qw = torch.zeros((2 * N, K), dtype=torch.uint8, device="cuda")
    ew = torch.full((2 * N, K // 32), 127, dtype=torch.uint8, device="cuda")
    A = torch.zeros((R, N // 2), dtype=torch.bfloat16, device="cuda")
    qr = torch.zeros((R, N // 2), dtype=torch.uint8, device="cuda")
    er = torch.zeros((R, N // 64), dtype=torch.uint8, device="cuda")
    ec = torch.zeros((R // 128, N // 2, 4), dtype=torch.uint8, device="cuda")
    off = dev(np.array([0, 256, 512], np.int32))
    with pytest.raises(B.MoeError):
        B.moe_grouped_gemm_fwd_quant_mx(ctx, q, qw, off, 2, N, K, R, e, ew, None, None, A, None, None, None, None)
    with pytest.raises(B.MoeError):
        B.moe_grouped_gemm_fwd_quant_mx(ctx, q, qw, off, 2, N, K, R, e, ew, None, None, A, qr, er, qr, None)
    with pytest.raises(B.MoeError):
        B.moe_grouped_gemm_fwd_quant_mx(ctx, q, qw, off, 2, N, K, R - 64, e, ew, None, None, A, qr, er, qr, ec)
    with pytest.raises(B.MoeError):   # the data gradient without saved pre-activations has nothing to quantise
        B.moe_grouped_gemm_dgrad_quant_mx(ctx, qr, qw, off, 2, N // 2, K, R, None, er, ew, None, A, None, qr, er, None, None)
    B.moe_grouped_gemm_fwd_quant_mx(ctx, q, qw, dev(np.array([0, 200, 512], np.int32)), 2, N, K, R, e, ew, None, None, A,
                                    qr, er, torch.zeros_like(qr), ec)
    torch.cuda.synchronize()
    assert ctx.poll_error() != 0


def test_mx_quantize_gather_source_rows_beyond_2_pow_24(B, ctx, oracle):
    """Map entries of 2^24 k and more (a source tensor of more than 16.7 million rows): the division of the entry by k
    must still be exact (a 2^40 / k constant would wrap around 64 bits there).  k = 1 and k = 3, 128 gathered rows."""
    from gpu_util import dev
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(77)
    cols, Rcap = 128, 128
    for k in (1, 3):
        T = (1 << 24) + 4096
        toks = np.sort(g.choice(np.arange((1 << 24) - 64, T), size=100, replace=False)).astype(np.int64)
        src = np.full(Rcap, -1, np.int32)
        src[:100] = (toks * k + g.integers(0, k, size=100)).astype(np.int32)
        rows = wl.bf16_round(g.standard_normal((100, cols)).astype(np.float32))
        X = torch.zeros((T, cols), dtype=torch.bfloat16, device="cuda")
        X[torch.from_numpy(toks).cuda()] = torch.from_numpy(rows).cuda().to(torch.bfloat16)
        V = np.zeros((Rcap, cols), np.float32)
        V[:100] = rows
        qr = torch.zeros((Rcap, cols), dtype=torch.uint8, device="cuda")
        er = torch.zeros((Rcap, cols // 32), dtype=torch.uint8, device="cuda")
        qc = torch.zeros((Rcap, cols), dtype=torch.uint8, device="cuda")
        ec = torch.zeros((Rcap // 128, cols, 4), dtype=torch.uint8, device="cuda")
        B.moe_mx_quantize_rowcol_gather(ctx, X, dev(src), k, None, 1, Rcap, cols, None, qr, er, qc, ec)
        torch.cuda.synchronize()
        qr_o, er_o = oracle.mx_quant_1x32(V)
        qc_o, _ = oracle.mx_quant_32x1(V[None])
        assert np.array_equal(qr.cpu().numpy(), qr_o) and np.array_equal(er.cpu().numpy(), er_o), k
        assert np.array_equal(qc.cpu().numpy(), qc_o[0]), k
        del X
