"""GPU parity: grouped GEMM forward / dgrad / wgrad against the CPU oracle on shapes that span
several 256x256 tiles, ragged row tails, empty experts and a one-row expert."""
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
    c = B.Context(T=16384, k=8, E=256, h=7168, f_max=14336)
    yield c
    c.close()


def _offsets(counts, align=1):
    pad = (np.asarray(counts) + align - 1) // align * align
    return np.concatenate([[0], np.cumsum(pad)]).astype(np.int32)


CASES = [
    # counts per expert, N, K
    ([300, 0, 257, 1, 700], 512, 128),
    ([256, 256], 256, 64),
    ([5], 128, 256),                      # N smaller than a tile (C1's fc2: N = h = 128)
    ([1000, 3, 0, 0, 513, 64], 768, 192),
]


@pytest.mark.parametrize("counts,N,K", CASES)
def test_grouped_gemm_fwd_plain(B, ctx, oracle, counts, N, K):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, BF16_TOL, F32_REG
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets(counts)
    R = int(off[-1])
    Rcap = R + 7
    Ah = wl.gaussian_bf16((Rcap, K), 1.0, 21, N)
    Bh = wl.gaussian_bf16((E, N, K), 1.0, 22, K)
    A, W = dev_bf16(Ah), dev_bf16(Bh)
    C = torch.full((Rcap, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_fwd(ctx, A, W, dev(off), E, N, K, Rcap, B.BF16, B.EPI_NONE, None, None, C, None)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    ref = oracle.grouped_gemm_nt(Ah[:R], Bh, off)
    got = host_f64(C)
    assert_close(got[:R], ref, "C")
    assert np.abs(got[:R] - ref).max() <= 0.02 * np.abs(ref).max() + 1e-6
    assert np.isnan(got[R:]).all()                                  # rows beyond offsets[E] untouched


@pytest.mark.parametrize("counts,f,K", [([300, 0, 257, 1, 700], 256, 128), ([130, 90], 128, 64),
                                         ([513], 384, 320)])
def test_grouped_gemm_fwd_swiglu(B, ctx, oracle, counts, f, K):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, BF16_TOL, F32_REG
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets(counts)
    R = int(off[-1])
    Rcap = R
    Ah = wl.gaussian_bf16((Rcap, K), 1.0, 23, f)
    Bh = wl.gaussian_bf16((E, 2 * f, K), 0.1, 24, K)
    A, W = dev_bf16(Ah), dev_bf16(Bh)
    Z = torch.full((Rcap, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    Act = torch.full((Rcap, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_fwd(ctx, A, W, dev(off), E, 2 * f, K, Rcap, B.BF16, B.EPI_SWIGLU, None, None, Z, Act)
    torch.cuda.synchronize()
    Zref = oracle.grouped_gemm_nt(Ah[:R], Bh, off)
    Aref = oracle.swiglu(Zref)
    assert_close(host_f64(Z), Zref, "Z")
    assert_close(host_f64(Act), Aref, "A")
    # Z may be skipped
    Act2 = torch.empty_like(Act)
    B.moe_grouped_gemm_fwd(ctx, A, W, dev(off), E, 2 * f, K, Rcap, B.BF16, B.EPI_SWIGLU, None, None, None, Act2)
    torch.cuda.synchronize()
    assert torch.equal(Act2.view(torch.int16), Act.view(torch.int16))


def test_grouped_gemm_bad_offsets_sets_error_word(B, ctx):
    """offsets[E] > Rcap: the kernel refuses to run and raises the device error word instead."""
    from gpu_util import dev
    A = torch.zeros((256, 64), dtype=torch.bfloat16, device="cuda")
    W = torch.zeros((1, 256, 64), dtype=torch.bfloat16, device="cuda")
    C = torch.full((256, 256), 7.0, dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_fwd(ctx, A, W, dev(np.array([0, 300], np.int32)), 1, 256, 64, 256, B.BF16, B.EPI_NONE,
                           None, None, C, None)
    assert ctx.poll_error() == 1
    assert ctx.poll_error() == 0
    assert (C == 7.0).all()


DG_CASES = [
    # counts, N (contraction), K (output columns)
    ([300, 0, 257, 1, 700], 128, 512),
    ([256, 256], 64, 256),
    ([5], 256, 128),                       # K smaller than a tile
    ([1000, 3, 0, 0, 513, 64], 192, 768),
]


@pytest.mark.parametrize("counts,N,K", DG_CASES)
def test_grouped_gemm_dgrad_plain(B, ctx, oracle, counts, N, K):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, BF16_TOL, F32_REG
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets(counts)
    R = int(off[-1])
    Rcap = R + 3
    dCh = wl.gaussian_bf16((Rcap, N), 1.0, 31, N)
    Bh = wl.gaussian_bf16((E, N, K), 1.0, 32, K)
    dC, W = dev_bf16(dCh), dev_bf16(Bh)
    dA = torch.full((Rcap, K), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_dgrad(ctx, dC, W, dev(off), E, N, K, Rcap, B.BF16, None, None, None, dA)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    ref = oracle.grouped_gemm_nn(dCh[:R], Bh, off)
    got = host_f64(dA)
    assert_close(got[:R], ref, "dA")
    assert np.abs(got[:R] - ref).max() <= 0.02 * np.abs(ref).max() + 1e-6
    assert np.isnan(got[R:]).all()


@pytest.mark.parametrize("counts,N,f", [([300, 0, 257, 1, 700], 128, 256), ([130, 90], 64, 128),
                                         ([513], 320, 384)])
def test_grouped_gemm_dgrad_swiglu_bwd(B, ctx, oracle, counts, N, f):
    """fc2 data gradient with the SwiGLU backward fused: dZ from dO, W2 and the saved pre-activation."""
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, BF16_TOL, F32_REG
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets(counts)
    R = int(off[-1])
    dOh = wl.gaussian_bf16((R, N), 1.0, 33, N)
    W2h = wl.gaussian_bf16((E, N, f), 0.1, 34, f)
    Zh = wl.gaussian_bf16((R, 2 * f), 1.5, 35, f)
    dZ = torch.full((R, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_dgrad(ctx, dev_bf16(dOh), dev_bf16(W2h), dev(off), E, N, f, R, B.BF16, dev_bf16(Zh), None, None,
                             dZ)
    torch.cuda.synchronize()
    dAref = oracle.grouped_gemm_nn(dOh, W2h, off)
    dZref = oracle.swiglu_bwd(dAref, Zh)
    assert_close(host_f64(dZ), dZref, "dZ")


@pytest.mark.parametrize("counts,N,f", [([300, 0, 257, 1, 700], 128, 256), ([130, 90], 64, 128),
                                         ([513], 320, 384), ([700, 40], 192, 640)])
def test_weighted_swiglu_forward_and_backward(B, ctx, oracle, counts, N, f):
    """Memory-efficient permutation (eq. (2)): the row weight multiplies the activation in the fc1 epilogue
    (the pre-activation stays unweighted); the fused fc2 data gradient scales dZ by it and emits the partial
    sums of <dA, silu(gate) * up> per row, which moe_scatter_row_dprob adds up per (token, slot)."""
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, BF16_TOL, F32_REG
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets(counts)
    R = int(off[-1])
    g = np.random.default_rng(R + f)
    ph = g.uniform(0.05, 1.0, size=R).astype(np.float32)
    p = dev(ph)
    # forward: Z = X W1^T, A = p * swiglu(Z)
    K = N
    Xh = wl.gaussian_bf16((R, K), 1.0, 51, K)
    W1h = wl.gaussian_bf16((E, 2 * f, K), 0.1, 52, f)
    Z = torch.full((R, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    A = torch.full((R, f), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_fwd_weighted(ctx, dev_bf16(Xh), dev_bf16(W1h), dev(off), E, 2 * f, K, R, B.BF16, B.EPI_SWIGLU,
                                    None, None, p, Z, A)
    torch.cuda.synchronize()
    Zref = oracle.grouped_gemm_nt(Xh, W1h, off)
    assert_close(host_f64(Z), Zref, "Z")                                # not weighted
    assert_close(host_f64(A), oracle.swiglu(Zref) * ph.astype(np.float64)[:, None], "A")
    # backward: dZ = p * swiglu_bwd(dO W2, Z); partials of <dA, swiglu(Z)>
    dOh = wl.gaussian_bf16((R, N), 1.0, 53, N)
    W2h = wl.gaussian_bf16((E, N, f), 0.1, 54, f)
    Zh = wl.gaussian_bf16((R, 2 * f), 1.5, 55, f)
    parts = 2 * ((f + 255) // 256)          # two entries per 256-column tile
    dZ = torch.full((R, 2 * f), float("nan"), dtype=torch.bfloat16, device="cuda")
    part = torch.full((R, parts), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_grouped_gemm_dgrad_weighted(ctx, dev_bf16(dOh), dev_bf16(W2h), dev(off), E, N, f, R, B.BF16, dev_bf16(Zh),
                                      None, None, p, dZ, part)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    dAref = oracle.grouped_gemm_nn(dOh, W2h, off)
    assert_close(host_f64(dZ), oracle.swiglu_bwd(dAref, Zh) * ph.astype(np.float64)[:, None], "dZ")
    dp_ref = (dAref * oracle.swiglu(Zh)).sum(axis=1)
    got = part.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    # per column tile, then summed
    tiles = (dAref * oracle.swiglu(Zh)).reshape(R, -1)
    for j in range(parts // 2):
        ref_j = tiles[:, 256 * j:256 * (j + 1)].sum(axis=1)
        assert rel_fro(got[:, 2 * j] + got[:, 2 * j + 1], ref_j) <= 1e-5, j
    assert rel_fro(got.sum(axis=1), dp_ref) <= 1e-5
    # scatter back to (token, slot): a synthetic map that visits the rows in reverse, with one skipped slot
    k = 2
    T = (R + k - 1) // k
    row_of = np.full((T, k), -1, np.int32)
    rows = np.arange(R - 1, -1, -1, dtype=np.int32)
    row_of.reshape(-1)[:R] = rows
    dprob = torch.full((T, k), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_scatter_row_dprob(ctx, part, parts, dev(row_of), T, k, dprob)
    torch.cuda.synchronize()
    g32 = got.astype(np.float32)[np.maximum(row_of, 0)]                 # [T, k, parts]: added in increasing part order, in fp32
    acc = np.zeros(row_of.shape, np.float32)
    for q in range(parts):
        acc = (acc + g32[..., q]).astype(np.float32)
    ref = np.where(row_of >= 0, acc, np.float32(0))
    np.testing.assert_array_equal(dprob.cpu().numpy(), ref)
    # gather: row weights from (token, slot) weights, zero for padding rows
    src_of = np.full(R + 3, -1, np.int32)
    src_of[:R] = g.permutation(T * k)[:R]
    probs = g.uniform(0, 1, size=(T, k)).astype(np.float32)
    rp = torch.full((R + 3,), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_gather_row_prob(ctx, dev(probs), dev(src_of), R + 3, rp)
    torch.cuda.synchronize()
    assert np.array_equal(rp.cpu().numpy(), oracle.gather_row_prob(probs, src_of).astype(np.float32))


WG_CASES = [
    # counts, N, K
    ([300, 0, 257, 1, 700], 256, 512),
    ([64, 128], 256, 256),
    ([5, 70], 128, 64),                    # output smaller than a tile in both directions
    ([1000, 3, 0, 0, 513, 64], 320, 264),  # ragged output tiles
]


@pytest.mark.parametrize("counts,N,K", WG_CASES)
@pytest.mark.parametrize("out_f32", [False, True])
def test_grouped_gemm_wgrad(B, ctx, oracle, counts, N, K, out_f32):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, BF16_TOL, F32_REG
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets(counts)
    R = int(off[-1])
    Rcap = R + 5
    dCh = wl.gaussian_bf16((Rcap, N), 1.0, 41, N)
    Ah = wl.gaussian_bf16((Rcap, K), 1.0, 42, K)
    tdt = torch.float32 if out_f32 else torch.bfloat16
    dB = torch.full((E, N, K), float("nan"), dtype=tdt, device="cuda")
    odt = B.F32 if out_f32 else B.BF16
    A, dC, doff = dev_bf16(Ah), dev_bf16(dCh), dev(off)
    B.moe_grouped_gemm_wgrad(ctx, A, dC, doff, E, N, K, Rcap, B.BF16, None, None, 0, odt, dB)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    ref = oracle.grouped_gemm_tn(dCh[:R], Ah[:R], off)
    got = host_f64(dB)
    kw = dict(tol=1e-5, reg=F32_REG) if out_f32 else {}
    assert_close(got, ref, "dB", **kw)
    for e, c in enumerate(counts):
        if c == 0:
            assert np.all(got[e] == 0)                              # zero-token expert: exact zeros
    # accumulate: dB += result
    B.moe_grouped_gemm_wgrad(ctx, A, dC, doff, E, N, K, Rcap, B.BF16, None, None, 1, odt, dB)
    torch.cuda.synchronize()
    assert_close(host_f64(dB), 2 * ref, "dB accumulated", **kw)


@pytest.mark.parametrize("counts", [[6000, 300, 257, 0, 700, 64, 1, 130], [9000, 5000, 100, 100, 100, 100, 100, 100, 100, 100]])
@pytest.mark.parametrize("out_f32", [False, True])
def test_grouped_gemm_wgrad_split_contraction(B, oracle, counts, out_f32):
    """Skewed loads: the contraction of experts far above the mean is split into pieces whose fp32 partial tiles are
    added in a fixed order by a second kernel.  Against the oracle (every element, every row), bit-identical from run
    to run, accumulate on top, and the same call on a context whose workspace has no room for partial tiles (no
    split) must agree with the oracle as well."""
    from gpu_util import dev, dev_bf16, host_f64, assert_close, F32_REG
    from paper_2603_07685_amd import workloads as wl
    E = len(counts)
    off = _offsets(counts)
    R = int(off[-1])
    N, K = 320, 264                                        # ragged output tiles in both directions
    dCh = wl.gaussian_bf16((R, N), 1.0, 81, E)
    Ah = wl.gaussian_bf16((R, K), 1.0, 82, E)
    A, dC, doff = dev_bf16(Ah), dev_bf16(dCh), dev(off)
    ref = oracle.grouped_gemm_tn(dCh, Ah, off)
    tdt = torch.float32 if out_f32 else torch.bfloat16
    odt = B.F32 if out_f32 else B.BF16
    kw = dict(tol=1e-5, reg=F32_REG) if out_f32 else {}
    big = B.Context(T=16384, k=8, E=E, h=512, f_max=256)    # room for 8 slices of partial tiles
    small = B.Context(T=16, k=1, E=E, h=0, f_max=0)         # none
    assert big.bytes >= 8 * 4 * 256 * 256 * 4 > small.bytes
    outs = []
    for ctx in (big, big, small):
        dB = torch.full((E, N, K), float("nan"), dtype=tdt, device="cuda")
        B.moe_grouped_gemm_wgrad(ctx, A, dC, doff, E, N, K, R, B.BF16, None, None, 0, odt, dB)
        torch.cuda.synchronize()
        assert ctx.poll_error() == 0
        assert_close(host_f64(dB), ref, "dB", **kw)
        outs.append(dB)
    assert torch.equal(outs[0].view(torch.int32 if out_f32 else torch.int16), outs[1].view(torch.int32 if out_f32 else torch.int16))
    assert not outs[0][counts.index(0)].any() if 0 in counts else True
    B.moe_grouped_gemm_wgrad(big, A, dC, doff, E, N, K, R, B.BF16, None, None, 1, odt, outs[0])
    torch.cuda.synchronize()
    assert_close(host_f64(outs[0]), 2 * ref, "dB accumulated", **kw)
    big.close()
    small.close()


@pytest.mark.parametrize("T,E,h", [(16384, 256, 7168), (1000, 8, 128), (300, 128, 4096), (1, 40, 64)])
def test_gate_gemm_and_router_on_its_logits(B, ctx, oracle, T, E, h):
    """logits = X Wr^T in fp32 from bf16 operands against the fp64 oracle; the router then selects on those logits
    exactly what the oracle selects on the same numbers."""
    from gpu_util import dev_bf16, rel_fro
    from paper_2603_07685_amd import workloads as wl
    Xh = wl.gaussian_bf16((T, h), 1.0, 31, T)
    Wh = wl.gaussian_bf16((E, h), 0.02, 32, E)
    logits = torch.full((T, E), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_gate_gemm(ctx, dev_bf16(Xh), dev_bf16(Wh), T, E, h, logits)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    got = logits.cpu().numpy()
    ref = oracle.grouped_gemm_nt(Xh, Wh[None], np.array([0, T], np.int32))
    assert np.isfinite(got).all()
    assert rel_fro(got, ref) <= 2e-6                        # fp32 accumulation of exact bf16 products
    k = min(8, E)
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    prob = torch.empty((T, k), dtype=torch.float32, device="cuda")
    B.moe_route_topk(ctx, logits, T, E, k, 0, False, 1.0, idx, prob, None)
    torch.cuda.synchronize()
    o_idx, o_prob, _ = oracle.route_topk(got, k, 0, False)
    assert np.array_equal(idx.cpu().numpy(), o_idx)


@pytest.mark.parametrize("E", [700, 1024])
def test_grouped_gemms_many_small_experts(B, ctx, oracle, E):
    """Hundreds of experts with 0..300 rows each (about a third of them empty): the device-side tile schedule, the
    expert search and the weight gradient's cost ordering beyond one pass of the workgroup's threads."""
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, BF16_TOL, F32_REG
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(E)
    counts = g.integers(0, 301, size=E)
    counts[g.random(E) < 0.33] = 0
    counts[E // 2] = 1500                                            # one expert far above the rest
    off = _offsets(counts)
    R = int(off[-1])
    N, K = 128, 64
    Ah = wl.gaussian_bf16((R, K), 1.0, 51, E)
    Wh = wl.gaussian_bf16((E, N, K), 1.0, 52, E)
    dCh = wl.gaussian_bf16((R, N), 1.0, 53, E)
    A, W, dC, doff = dev_bf16(Ah), dev_bf16(Wh), dev_bf16(dCh), dev(off)
    C = torch.full((R, N), float("nan"), dtype=torch.bfloat16, device="cuda")
    dA = torch.full((R, K), float("nan"), dtype=torch.bfloat16, device="cuda")
    dW = torch.full((E, N, K), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_grouped_gemm_fwd(ctx, A, W, doff, E, N, K, R, B.BF16, B.EPI_NONE, None, None, C, None)
    B.moe_grouped_gemm_dgrad(ctx, dC, W, doff, E, N, K, R, B.BF16, None, None, None, dA)
    B.moe_grouped_gemm_wgrad(ctx, A, dC, doff, E, N, K, R, B.BF16, None, None, 0, B.F32, dW)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    assert_close(host_f64(C), oracle.grouped_gemm_nt(Ah, Wh, off), "C")
    assert_close(host_f64(dA), oracle.grouped_gemm_nn(dCh, Wh, off), "dA")
    got = host_f64(dW)
    assert_close(got, oracle.grouped_gemm_tn(dCh, Ah, off), "dW", tol=1e-5, reg=F32_REG)
    assert not got[counts == 0].any()


def test_grouped_gemm_runs_are_bit_identical(B, ctx):
    """A determinism check (the kernel against itself: it says nothing about parity).  No result depends on timing: every workgroup walks its tiles through two LDS buffers that four waves fill and
    read under one barrier per stage, and no floating-point atomics are used, so two runs of a call must agree bit
    for bit.  Many tiles per workgroup (odd and even stage counts, ragged experts, an empty one), all three modes."""
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    counts = [1500, 0, 777, 2049, 130, 4096, 3, 900]
    E, N, K = len(counts), 1536, 1344          # K / 64 = 21 stages (odd), N / 64 = 24 (even)
    off = _offsets(counts)
    R = int(off[-1])
    Rcap = R + 3
    A = dev_bf16(wl.gaussian_bf16((Rcap, K), 1.0, 71, K))
    W = dev_bf16(wl.gaussian_bf16((E, N, K), 0.05, 72, K))
    dC = dev_bf16(wl.gaussian_bf16((Rcap, N), 1.0, 73, N))
    doff = dev(off)
    outs = []
    for rep in range(3):
        C = torch.zeros((Rcap, N), dtype=torch.bfloat16, device="cuda")
        dA = torch.zeros((Rcap, K), dtype=torch.bfloat16, device="cuda")
        dW = torch.zeros((E, N, K), dtype=torch.bfloat16, device="cuda")
        B.moe_grouped_gemm_fwd(ctx, A, W, doff, E, N, K, Rcap, B.BF16, B.EPI_NONE, None, None, C, None)
        B.moe_grouped_gemm_dgrad(ctx, dC, W, doff, E, N, K, Rcap, B.BF16, None, None, None, dA)
        B.moe_grouped_gemm_wgrad(ctx, A, dC, doff, E, N, K, Rcap, B.BF16, None, None, 0, B.BF16, dW)
        torch.cuda.synchronize()
        assert ctx.poll_error() == 0
        outs.append((C, dA, dW))
    for rep in (1, 2):
        for got, first in zip(outs[rep], outs[0]):
            assert torch.equal(got.view(torch.int16), first.view(torch.int16))
