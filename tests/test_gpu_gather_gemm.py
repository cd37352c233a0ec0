"""GPU parity: the grouped GEMMs that fetch one operand through the row map (the permute's row move fused into
the operand fetch, Sec. 4.3.3) against the plain calls on the permuted copy (bit for bit) and against the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


@pytest.fixture(scope="module")
def B():
    from paper_2603_07685_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def ctx(B):
    c = B.Context(T=16384, k=8, E=64, h=1024, f_max=512)
    yield c
    c.close()


def _row_map(counts, align, T, k, seed, tail=5):
    """A permutation map as moe_permute builds it: expert e owns rows [off[e], off[e] + counts[e]) holding distinct
    flattened (token, slot) indices, padding rows up to off[e + 1] and the `tail` rows behind off[E] hold -1."""
    rng = np.random.default_rng(seed)
    pad = (np.asarray(counts) + align - 1) // align * align
    off = np.concatenate([[0], np.cumsum(pad)]).astype(np.int32)
    Rcap = int(off[-1]) + tail
    src = np.full(Rcap, -1, np.int32)
    picks = rng.choice(T * k, size=int(np.sum(counts)), replace=False)
    at = 0
    for e, c in enumerate(counts):
        src[off[e]:off[e] + c] = np.sort(picks[at:at + c])
        at += c
    return off, src, Rcap


def _gathered(Xh, src, k):
    out = Xh[np.maximum(src, 0) // k].copy()
    out[src < 0] = 0
    return out


def _bits(t):
    return t.view(torch.int32 if t.dtype == torch.float32 else torch.int16)


MAPS = [
    # counts, align, T, k
    ([300, 0, 257, 1, 700], 1, 400, 4),
    ([130, 90, 513], 16, 1000, 1),
    ([1000, 3, 0, 0, 513, 64], 128, 300, 8),
]


@pytest.mark.parametrize("counts,align,T,k", MAPS)
@pytest.mark.parametrize("f,K", [(256, 128), (384, 320)])
def test_fwd_gather_swiglu_and_plain(B, ctx, oracle, counts, align, T, k, f, K):
    from gpu_util import dev, dev_bf16, host_f64, assert_close
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off, src, Rcap = _row_map(counts, align, T, k, seed=f + K)
    R = int(off[-1])
    Xh = wl.gaussian_bf16((T, K), 1.0, 301, K)
    Wh = wl.gaussian_bf16((E, 2 * f, K), 0.1, 302, f)
    ph = np.random.default_rng(5).uniform(0.1, 1.0, Rcap).astype(np.float32)
    Xph = _gathered(Xh, src, k)
    X, Xp, W, doff, dsrc, p = dev_bf16(Xh), dev_bf16(Xph), dev_bf16(Wh), dev(off), dev(src), dev(ph)
    for prob in (None, p):
        Z0 = torch.full((Rcap, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
        A0 = torch.full((Rcap, f), float("nan"), dtype=torch.bfloat16, device="cuda")
        Z1, A1 = Z0.clone(), A0.clone()
        B.moe_grouped_gemm_fwd_weighted(ctx, Xp, W, doff, E, 2 * f, K, Rcap, B.BF16, B.EPI_SWIGLU, None, None, prob, Z0, A0)
        B.moe_grouped_gemm_fwd_gather(ctx, X, T, dsrc, k, W, doff, E, 2 * f, K, Rcap, B.EPI_SWIGLU, prob, Z1, A1)
        torch.cuda.synchronize()
        assert ctx.poll_error() == 0
        assert torch.equal(_bits(Z1[:R]), _bits(Z0[:R])) and torch.equal(_bits(A1[:R]), _bits(A0[:R]))
        assert torch.isnan(Z1[R:]).all() and torch.isnan(A1[R:]).all()      # rows beyond offsets[E] untouched
    Zref = oracle.grouped_gemm_nt(Xph[:R], Wh, off)
    assert_close(host_f64(Z1[:R]), Zref, "Z")
    assert_close(host_f64(A1[:R]), oracle.swiglu(Zref) * ph[:R, None], "A")
    # plain store epilogue
    C0 = torch.full((Rcap, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    C1 = C0.clone()
    B.moe_grouped_gemm_fwd(ctx, Xp, W, doff, E, 2 * f, K, Rcap, B.BF16, B.EPI_NONE, None, None, C0, None)
    B.moe_grouped_gemm_fwd_gather(ctx, X, T, dsrc, k, W, doff, E, 2 * f, K, Rcap, B.EPI_NONE, None, C1, None)
    torch.cuda.synchronize()
    assert torch.equal(_bits(C1[:R]), _bits(C0[:R])) and torch.isnan(C1[R:]).all()
    assert_close(host_f64(C1[:R]), Zref, "C")


@pytest.mark.parametrize("counts,align,T,k", MAPS)
@pytest.mark.parametrize("N,f", [(128, 128), (320, 192)])
def test_dgrad_gather(B, ctx, oracle, counts, align, T, k, N, f):
    """dC rows through the map: with the SwiGLU backward (weighted, with the dprob partial sums) and without."""
    from gpu_util import dev, dev_bf16, host_f64, assert_close
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off, src, Rcap = _row_map(counts, align, T, k, seed=N + f)
    R = int(off[-1])
    Gh = wl.gaussian_bf16((T, N), 1.0, 311, N)
    Wh = wl.gaussian_bf16((E, N, f), 0.1, 312, f)
    Zh = wl.gaussian_bf16((Rcap, 2 * f), 1.0, 313, f)
    ph = np.random.default_rng(6).uniform(0.1, 1.0, Rcap).astype(np.float32)
    Gph = _gathered(Gh, src, k)
    G, Gp, W, Zs, doff, dsrc, p = dev_bf16(Gh), dev_bf16(Gph), dev_bf16(Wh), dev_bf16(Zh), dev(off), dev(src), dev(ph)
    parts = 2 * ((f + 255) // 256)
    dZ0 = torch.full((Rcap, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    dZ1 = dZ0.clone()
    dp0 = torch.full((Rcap, parts), float("nan"), dtype=torch.float32, device="cuda")
    dp1 = dp0.clone()
    B.moe_grouped_gemm_dgrad_weighted(ctx, Gp, W, doff, E, N, f, Rcap, B.BF16, Zs, None, None, p, dZ0, dp0)
    B.moe_grouped_gemm_dgrad_gather(ctx, G, T, dsrc, k, W, doff, E, N, f, Rcap, Zs, p, dZ1, dp1)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    assert torch.equal(_bits(dZ1[:R]), _bits(dZ0[:R])) and torch.equal(_bits(dp1[:R]), _bits(dp0[:R]))
    assert torch.isnan(dZ1[R:]).all()
    dAref = oracle.grouped_gemm_nn(Gph[:R], Wh, off)
    dZref = oracle.swiglu_bwd(dAref, Zh[:R].astype(np.float64)) * ph[:R, None]
    assert_close(host_f64(dZ1[:R]), dZref, "dZ")
    dA0 = torch.full((Rcap, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    dA1 = dA0.clone()
    B.moe_grouped_gemm_dgrad(ctx, Gp, W, doff, E, N, f, Rcap, B.BF16, None, None, None, dA0)
    B.moe_grouped_gemm_dgrad_gather(ctx, G, T, dsrc, k, W, doff, E, N, f, Rcap, None, None, dA1, None)
    torch.cuda.synchronize()
    assert torch.equal(_bits(dA1[:R]), _bits(dA0[:R])) and torch.isnan(dA1[R:]).all()
    assert_close(host_f64(dA1[:R]), dAref, "dA")


WG_MAPS = MAPS + [([6000, 300, 257, 0, 700, 64, 1, 130], 1, 2000, 4)]     # the last one splits its contraction


@pytest.mark.parametrize("counts,align,T,k", WG_MAPS)
@pytest.mark.parametrize("N,K", [(256, 512), (320, 264)])
@pytest.mark.parametrize("out_f32", [False, True])
def test_wgrad_gather(B, ctx, oracle, counts, align, T, k, N, K, out_f32):
    """Either operand of the weight gradient through the map (A: the fc1 gradient reads X; dC: under eq. (2) the fc2
    gradient reads dY), with accumulation, on balanced and on skewed loads (split contraction)."""
    from gpu_util import dev, dev_bf16, host_f64, assert_close, F32_REG
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off, src, Rcap = _row_map(counts, align, T, k, seed=N + K)
    R = int(off[-1])
    tdt = torch.float32 if out_f32 else torch.bfloat16
    odt = B.F32 if out_f32 else B.BF16
    kw = dict(tol=1e-5, reg=F32_REG) if out_f32 else {}
    doff, dsrc = dev(off), dev(src)
    for which in (B.GATHER_A, B.GATHER_DC):
        cols_g, cols_o = (K, N) if which == B.GATHER_A else (N, K)
        Gh = wl.gaussian_bf16((T, cols_g), 1.0, 321 + which, N)          # the unpermuted operand
        Oh = wl.gaussian_bf16((Rcap, cols_o), 1.0, 323 + which, K)       # the other one, stored by permuted row
        Gph = _gathered(Gh, src, k)
        G, Gp, O = dev_bf16(Gh), dev_bf16(Gph), dev_bf16(Oh)
        Ap, dCp = (Gp, O) if which == B.GATHER_A else (O, Gp)
        Ag, dCg = (G, O) if which == B.GATHER_A else (O, G)
        d0 = torch.full((E, N, K), float("nan"), dtype=tdt, device="cuda")
        d1 = d0.clone()
        B.moe_grouped_gemm_wgrad(ctx, Ap, dCp, doff, E, N, K, Rcap, B.BF16, None, None, 0, odt, d0)
        B.moe_grouped_gemm_wgrad_gather(ctx, Ag, dCg, which, T, dsrc, k, doff, E, N, K, Rcap, 0, odt, d1)
        torch.cuda.synchronize()
        assert ctx.poll_error() == 0
        assert torch.equal(_bits(d1), _bits(d0))
        Aph, dCph = (Gph, Oh) if which == B.GATHER_A else (Oh, Gph)
        ref = oracle.grouped_gemm_tn(dCph[:R], Aph[:R], off)
        assert_close(host_f64(d1), ref, "dB", **kw)
        B.moe_grouped_gemm_wgrad_gather(ctx, Ag, dCg, which, T, dsrc, k, doff, E, N, K, Rcap, 1, odt, d1)
        torch.cuda.synchronize()
        assert_close(host_f64(d1), 2 * ref, "dB accumulated", **kw)


def test_gather_rejects_bad_requests(B, ctx):
    X = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    W = torch.zeros(1, 64, 64, dtype=torch.bfloat16, device="cuda")
    off = torch.tensor([0, 64], dtype=torch.int32, device="cuda")
    src = torch.zeros(64, dtype=torch.int32, device="cuda")
    C = torch.zeros(64, 64, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(B.MoeError):       # no map
        B.moe_grouped_gemm_fwd_gather(ctx, X, 64, None, 1, W, off, 1, 64, 64, 64, B.EPI_NONE, None, C, None)
    with pytest.raises(B.MoeError):       # k = 0
        B.moe_grouped_gemm_fwd_gather(ctx, X, 64, src, 0, W, off, 1, 64, 64, 64, B.EPI_NONE, None, C, None)
    with pytest.raises(B.MoeError):       # offsets inside the unpermuted tensor would not fit 32 bits
        B.moe_grouped_gemm_fwd_gather(ctx, X, 1 << 26, src, 1, W, off, 1, 64, 64, 64, B.EPI_NONE, None, C, None)
    with pytest.raises(B.MoeError):       # bad operand selector
        B.moe_grouped_gemm_wgrad_gather(ctx, X, X, 7, 64, src, 1, off, 1, 64, 64, 64, 0, B.BF16, C)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
