"""GPU parity: router, row-ID map, permute, combine and its backward against the CPU oracle."""
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


def _route(B, ctx, logits, k, fn, norm, scale=1.0):
    from gpu_util import dev
    T, E = logits.shape
    d_log = dev(logits)
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    prob = torch.empty((T, k), dtype=torch.float32, device="cuda")
    counts = torch.empty(E, dtype=torch.int32, device="cuda")
    B.moe_route_topk(ctx, d_log, T, E, k, fn, norm, scale, idx, prob, counts)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), prob.cpu().numpy(), counts.cpu().numpy()


@pytest.mark.parametrize("T,E,k,fn,norm,scale", [
    (256, 8, 2, 0, False, 1.0),        # C1
    (8192, 8, 2, 0, False, 1.0),       # C2
    (16384, 128, 8, 0, False, 1.0),    # C3 router at its global shape
    (16384, 256, 8, 1, True, 1.0),     # C4/C5 router: sigmoid, normalised top-k
    (1000, 37, 5, 1, False, 2.5),      # ragged: E not a multiple of 64, T not a multiple of the block
    (333, 1024, 32, 0, True, 1.0),     # maximum E and k
    (64, 5, 5, 0, False, 1.0),         # k == E
])
def test_route_topk(B, ctx, oracle, T, E, k, fn, norm, scale):
    from paper_2603_07685_amd import workloads as wl
    _, _, logits = wl.router_logits(T, 64, E, 0.3, 77 + T + E)
    idx, prob, counts = _route(B, ctx, logits, k, fn, norm, scale)
    o_idx, o_prob, o_counts = oracle.route_topk(logits, k, fn, norm, scale)
    assert np.array_equal(idx, o_idx)            # bit-exact indices, slot order included
    assert np.array_equal(counts, o_counts)
    np.testing.assert_allclose(prob, o_prob, rtol=2e-6, atol=1e-9)


@pytest.mark.parametrize("T,E,k,fn,norm,scale", [
    (256, 8, 2, 0, False, 1.0),
    (1000, 128, 8, 0, True, 2.5),
    (4096, 256, 8, 1, True, 1.0),      # C4/C5 router
    (777, 300, 6, 1, False, 0.5),      # E not a multiple of 64
])
def test_route_topk_backward(B, ctx, oracle, T, E, k, fn, norm, scale):
    """dlogits from dweights with the selection frozen, every element, against the fp64 oracle."""
    from gpu_util import dev
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(T + E)
    logits = (g.normal(size=(T, E)) * 1.5).astype(np.float32)
    idx, _, _ = oracle.route_topk(logits, k, fn, norm, scale)
    dw = g.normal(size=(T, k)).astype(np.float32)
    out = torch.full((T, E), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_route_topk_bwd(ctx, dev(logits), dev(idx), dev(dw), T, E, k, fn, norm, scale, out)
    torch.cuda.synchronize()
    ref = oracle.route_topk_bwd(logits, idx, dw, fn, norm, scale)
    got = out.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    assert np.abs(got - ref).max() <= 2e-5 * np.abs(ref).max() + 1e-9
    if fn == 1:      # sigmoid: only the selected experts receive a gradient
        mask = np.zeros((T, E), bool)
        np.put_along_axis(mask, idx.astype(np.int64), True, axis=1)
        assert np.all(got[~mask] == 0)


def test_route_topk_ties_and_errors(B, ctx, oracle):
    g = np.random.default_rng(5)
    logits = g.integers(-2, 3, size=(512, 16)).astype(np.float32)     # many exact ties
    idx, prob, counts = _route(B, ctx, logits, 4, 1, True)
    o_idx, o_prob, o_counts = oracle.route_topk(logits, 4, 1, True)
    assert np.array_equal(idx, o_idx) and np.array_equal(counts, o_counts)
    np.testing.assert_allclose(prob, o_prob, rtol=2e-6)
    with pytest.raises(B.MoeError):
        _route(B, ctx, logits, 17, 0, False)                         # k > E


@pytest.mark.parametrize("T,E,k,ng,tg,fn,norm,scale,with_bias", [
    (16384, 256, 8, 8, 4, 1, True, 2.5, True),     # the published DeepSeek-V3 router at the C4 token count
    (4096, 128, 8, 8, 2, 0, True, 1.0, True),      # softmax scores, 16 experts per group, 4 per kept group
    (1000, 64, 6, 4, 2, 0, False, 1.0, False),
    (777, 96, 3, 8, 3, 1, False, 0.5, True),       # 12 per group: groups straddle lanes and register slots
    (500, 1024, 32, 64, 16, 1, True, 1.0, True),   # maximum E, k and group count
    (300, 40, 5, 1, 1, 1, True, 1.0, True),        # one group: only the bias differs from the plain router
    (64, 8, 8, 2, 2, 0, False, 1.0, False),        # k == E
])
def test_route_topk_grouped(B, ctx, oracle, T, E, k, ng, tg, fn, norm, scale, with_bias):
    """Group-limited, bias-corrected selection: indices (slot order included) and counts bit-exact."""
    from gpu_util import dev
    g = np.random.default_rng(T + E + k)
    logits = (g.normal(size=(T, E)) * 1.5).astype(np.float32)
    bias = (g.normal(size=E) * 0.1).astype(np.float32) if with_bias else None
    idx = torch.full((T, k), -7, dtype=torch.int32, device="cuda")
    prob = torch.full((T, k), float("nan"), dtype=torch.float32, device="cuda")
    counts = torch.full((E,), -7, dtype=torch.int32, device="cuda")
    B.moe_route_topk_grouped(ctx, dev(logits), None if bias is None else dev(bias), T, E, k, ng, tg, fn, norm, scale,
                             idx, prob, counts)
    torch.cuda.synchronize()
    o_idx, o_prob, o_counts = oracle.route_topk_grouped(logits, k, ng, tg, bias, fn, norm, scale)
    assert np.array_equal(idx.cpu().numpy(), o_idx)
    assert np.array_equal(counts.cpu().numpy(), o_counts)
    np.testing.assert_allclose(prob.cpu().numpy(), o_prob, rtol=2e-6, atol=1e-9)


def test_route_topk_grouped_ties_plain_equivalence_and_errors(B, ctx, oracle):
    from gpu_util import dev
    g = np.random.default_rng(6)
    T, E, k = 512, 32, 4
    logits = g.integers(-2, 3, size=(T, E)).astype(np.float32)          # many exact ties, in experts and in groups
    idx = torch.empty((T, k), dtype=torch.int32, device="cuda")
    prob = torch.empty((T, k), dtype=torch.float32, device="cuda")
    counts = torch.empty(E, dtype=torch.int32, device="cuda")
    B.moe_route_topk_grouped(ctx, dev(logits), None, T, E, k, 4, 2, 1, True, 1.0, idx, prob, counts)
    torch.cuda.synchronize()
    o_idx, o_prob, o_counts = oracle.route_topk_grouped(logits, k, 4, 2, None, 1, True, 1.0)
    assert np.array_equal(idx.cpu().numpy(), o_idx) and np.array_equal(counts.cpu().numpy(), o_counts)
    # one group, no bias: the plain router's selection
    B.moe_route_topk_grouped(ctx, dev(logits), None, T, E, k, 1, 1, 1, True, 1.0, idx, prob, counts)
    torch.cuda.synchronize()
    p_idx, p_prob, p_counts = _route(B, ctx, logits, k, 1, True)
    assert np.array_equal(idx.cpu().numpy(), p_idx) and np.array_equal(counts.cpu().numpy(), p_counts)
    np.testing.assert_allclose(prob.cpu().numpy(), p_prob, rtol=2e-6)
    for bad in [(3, 2), (4, 5), (64, 1)]:                                # E % n_group, topk_group > n_group, k/tg > E/ng
        with pytest.raises(B.MoeError):
            B.moe_route_topk_grouped(ctx, dev(logits), None, T, E, k, bad[0], bad[1], 1, True, 1.0, idx, prob, counts)


@pytest.mark.parametrize("T,E,k,fn", [
    (16384, 256, 8, 1),      # C4 router shape
    (16384, 128, 8, 0),      # C3
    (1000, 37, 5, 0),        # ragged
    (333, 1024, 32, 1),      # maximum E
    (1, 8, 2, 0),            # a single token
])
def test_aux_loss_and_gradient(B, ctx, oracle, T, E, k, fn):
    """Loss and d loss / d logits against the fp64 oracle; the gradient also accumulated onto an existing tensor;
    two runs give identical bits (fixed summation order)."""
    from gpu_util import dev
    g = np.random.default_rng(T + E + k)
    logits = (g.normal(size=(T, E)) * 1.5).astype(np.float32)
    counts = g.multinomial(T * k, g.dirichlet(np.ones(E) * 2.0)).astype(np.int32)
    coeff, dloss = 1e-2, 0.7
    ref_loss, ref_grad = oracle.aux_loss(logits, counts, k, fn, coeff)
    loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    dl = torch.full((T, E), float("nan"), dtype=torch.float32, device="cuda")
    B.moe_aux_loss(ctx, dev(logits), dev(counts), T, E, k, fn, coeff, dloss, 0, loss, dl)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    got = dl.cpu().numpy().astype(np.float64)
    assert abs(loss.item() - ref_loss) <= 2e-6 * abs(ref_loss)
    assert np.abs(got - dloss * ref_grad).max() <= 2e-5 * np.abs(dloss * ref_grad).max() + 1e-12
    # accumulate onto an existing gradient; loss only (dlogits NULL); bit-identical repeat
    base = g.normal(size=(T, E)).astype(np.float32)
    dl2 = dev(base)
    loss2 = torch.zeros(1, dtype=torch.float32, device="cuda")
    B.moe_aux_loss(ctx, dev(logits), dev(counts), T, E, k, fn, coeff, dloss, 1, loss2, dl2)
    loss3 = torch.zeros(1, dtype=torch.float32, device="cuda")
    B.moe_aux_loss(ctx, dev(logits), dev(counts), T, E, k, fn, coeff, dloss, 0, loss3, None)
    torch.cuda.synchronize()
    assert torch.equal(loss2, loss) and torch.equal(loss3, loss)
    np.testing.assert_allclose(dl2.cpu().numpy(), base + dl.cpu().numpy(), rtol=1e-6, atol=1e-9)   # fused multiply-add allowed
    # balanced load: the loss is coeff whatever the logits, the gradient vanishes
    if (T * k) % E == 0:
        bal = np.full(E, T * k // E, np.int32)
        B.moe_aux_loss(ctx, dev(logits), dev(bal), T, E, k, fn, coeff, 1.0, 0, loss, dl)
        torch.cuda.synchronize()
        assert abs(loss.item() - coeff) <= 2e-6 * coeff
        assert dl.abs().max().item() <= 1e-9


def _permute(B, ctx, X, idx, E, align, dt):
    from gpu_util import dev
    T, k = idx.shape
    h = X.shape[1]
    Rcap = T * k + E * (align - 1)
    Xp = torch.full((Rcap, h), float("nan"), dtype=X.dtype, device="cuda")
    row_of = torch.empty((T, k), dtype=torch.int32, device="cuda")
    src_of = torch.empty(Rcap, dtype=torch.int32, device="cuda")
    offsets = torch.empty(E + 1, dtype=torch.int32, device="cuda")
    counts = torch.empty(E, dtype=torch.int32, device="cuda")
    B.moe_permute(ctx, X, dt, dev(idx), T, k, h, E, align, Xp, Rcap, row_of, src_of, offsets, counts)
    torch.cuda.synchronize()
    return Xp, row_of, src_of, offsets, counts, Rcap


@pytest.mark.parametrize("T,k,E,h,align,f32", [
    (256, 2, 8, 128, 1, False),       # C1
    (256, 2, 8, 128, 1, True),
    (3000, 3, 7, 264, 16, False),     # ragged sizes, skipped ids, an empty expert
    (4096, 8, 32, 1024, 128, False),  # fp8-style padding
    (1, 1, 1, 8, 1, False),           # degenerate
    (2500, 8, 256, 72, 1, False),     # many experts, several chunks
])
def test_permute_maps_and_rows(B, ctx, oracle, T, k, E, h, align, f32):
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(T + E)
    idx = g.integers(-1 if E > 1 else 0, E + (1 if E > 1 else 0), size=(T, k)).astype(np.int32)
    if E > 4:
        idx[idx == 3] = 2                                             # expert 3 receives nothing
    Xh = wl.gaussian_bf16((T, h), 1.0, 11, T)
    X = dev(Xh) if f32 else dev_bf16(Xh)
    Xp, row_of, src_of, offsets, counts, Rcap = _permute(B, ctx, X, idx, E, align, B.F32 if f32 else B.BF16)
    m = oracle.permute_maps(idx, E, align, Rcap)
    assert np.array_equal(row_of.cpu().numpy(), m.row_of)
    assert np.array_equal(src_of.cpu().numpy(), m.src_of)
    assert np.array_equal(offsets.cpu().numpy(), m.offsets)
    assert np.array_equal(counts.cpu().numpy(), m.counts)
    ref = oracle.permute_rows(Xh, m.src_of[: m.Rtot], k, prec="f32")
    got = Xp[: m.Rtot].float().cpu().numpy()
    assert np.array_equal(got, ref)                                   # copies and zero padding are exact
    assert torch.isnan(Xp[m.Rtot:].float()).all()                     # rows beyond offsets[E] untouched


def test_permute_errors(B, ctx):
    from gpu_util import dev
    idx = dev(np.zeros((4, 2), np.int32))
    X = torch.zeros((4, 8), dtype=torch.bfloat16, device="cuda")
    Xp = torch.zeros((8, 8), dtype=torch.bfloat16, device="cuda")
    i32 = lambda n: torch.zeros(n, dtype=torch.int32, device="cuda")
    with pytest.raises(B.MoeError):   # Rcap too small for align = 4
        B.moe_permute(ctx, X, B.BF16, idx, 4, 2, 8, 2, 4, Xp, 8, i32(8), i32(8), i32(3), i32(2))
    with pytest.raises(B.MoeError):   # row size not a multiple of 16 bytes
        B.moe_permute(ctx, X, B.BF16, idx, 4, 2, 4, 2, 1, Xp, 8, i32(8), i32(8), i32(3), i32(2))


@pytest.mark.parametrize("T,k,E,h,align,f32,res", [
    (256, 2, 8, 128, 1, False, False),
    (256, 2, 8, 128, 1, True, True),
    (1500, 8, 32, 7168, 128, False, True),    # C4 row width, ragged tail of the 16-byte chunks
    (777, 5, 9, 200, 1, False, False),        # k not a multiple of 4
    (300, 1, 4, 64, 1, False, True),
])
def test_combine_and_backward(B, ctx, oracle, T, k, E, h, align, f32, res):
    from gpu_util import dev, dev_bf16, host_f64, rel_fro, assert_close, BF16_TOL
    from paper_2603_07685_amd import workloads as wl
    g = np.random.default_rng(T * 3 + k)
    idx = g.integers(-1, E, size=(T, k)).astype(np.int32)            # some slots not on this GPU
    m = oracle.permute_maps(idx, E, align)
    Rcap = T * k + E * (align - 1)
    Oh = wl.gaussian_bf16((Rcap, h), 1.0, 12, T)
    Sh = wl.gaussian_bf16((T, h), 1.0, 13, T) if res else None
    dYh = wl.gaussian_bf16((T, h), 1.0, 14, T)
    prob = wl.forced_probs(T, k, 15)
    mk = dev if f32 else dev_bf16
    dt = B.F32 if f32 else B.BF16
    tdt = torch.float32 if f32 else torch.bfloat16
    O, dY = mk(Oh), mk(dYh)
    S = mk(Sh) if res else None
    row_of, src_of, dprob_in = dev(m.row_of), dev(m.src_of), dev(prob)
    Y = torch.empty((T, h), dtype=tdt, device="cuda")
    B.moe_unpermute_combine(ctx, O, dt, row_of, dprob_in, S, T, k, h, Y)
    Yref = oracle.combine(Oh, m.row_of, prob, Sh)
    tol = 1e-5 if f32 else BF16_TOL
    kw = dict(tol=tol, reg=None, row_tol=1e-4) if f32 else {}
    assert_close(host_f64(Y), Yref, "Y", **kw)
    # plain-sum form (prob == NULL): the backward of permute
    B.moe_unpermute_combine(ctx, O, dt, row_of, None, None, T, k, h, Y)
    assert_close(host_f64(Y), oracle.combine(Oh, m.row_of, None, None), "plain sum", **kw)
    # backward
    dO = torch.full((Rcap, h), float("nan"), dtype=tdt, device="cuda")
    dprob = torch.empty((T, k), dtype=torch.float32, device="cuda")
    B.moe_unpermute_combine_bwd(ctx, dY, O, dt, row_of, src_of, dprob_in, T, k, h, Rcap, dO, dprob)
    torch.cuda.synchronize()
    dOref, dpref = oracle.combine_bwd(dYh, Oh, m.row_of, prob, Rcap)
    assert_close(host_f64(dO), dOref, "dO", **kw)                     # includes exact zeros on padding rows
    assert np.all(host_f64(dO)[m.src_of < 0] == 0)
    assert rel_fro(host_f64(dprob), dpref) <= (1e-5 if f32 else 1e-4)


def test_round_trip_is_identity(B, ctx, oracle):
    """permute then combine with w = 1/k returns X bit-exactly (k a power of two)."""
    from gpu_util import dev, dev_bf16
    from paper_2603_07685_amd import workloads as wl
    T, k, E, h = 2048, 4, 16, 512
    g = np.random.default_rng(3)
    idx = np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    X = dev_bf16(wl.gaussian_bf16((T, h), 1.0, 16, 0))
    Xp, row_of, src_of, offsets, counts, Rcap = _permute(B, ctx, X, idx, E, 1, B.BF16)
    assert int(counts.sum()) == T * k
    Y = torch.empty_like(X)
    w = torch.full((T, k), 0.25, dtype=torch.float32, device="cuda")
    B.moe_unpermute_combine(ctx, Xp, B.BF16, row_of, w, None, T, k, h, Y)
    torch.cuda.synchronize()
    assert torch.equal(Y.view(torch.int16), X.view(torch.int16))


def test_empty_batch_and_all_experts_empty(B, ctx, oracle):
    """Degenerate extents end to end: T = 0 through route / permute / combine, and grouped GEMMs whose offsets say
    that no expert has a row (forward and data gradient touch nothing, the weight gradient is exact zeros)."""
    from gpu_util import dev
    E, k, h, f = 4, 2, 64, 64
    # T = 0: nothing to read; counts and offsets are still written (all zero).  (One-row buffers stand in for the
    # empty tensors: torch gives a zero-size tensor a NULL data pointer, and a pointer must still be a pointer)
    empty = lambda cols, dt: torch.zeros((1, cols), dtype=dt, device="cuda")
    idx, prob = empty(k, torch.int32), empty(k, torch.float32)
    counts = torch.full((E,), 7, dtype=torch.int32, device="cuda")
    B.moe_route_topk(ctx, empty(E, torch.float32), 0, E, k, 0, False, 1.0, idx, prob, counts)
    Rcap = 8
    X = empty(h, torch.bfloat16)
    Xp = torch.full((Rcap, h), 3.0, dtype=torch.bfloat16, device="cuda")
    row_of = empty(k, torch.int32)
    src_of = torch.full((Rcap,), 5, dtype=torch.int32, device="cuda")
    offsets = torch.full((E + 1,), 9, dtype=torch.int32, device="cuda")
    cnt2 = torch.full((E,), 9, dtype=torch.int32, device="cuda")
    B.moe_permute(ctx, X, B.BF16, idx, 0, k, h, E, 1, Xp, Rcap, row_of, src_of, offsets, cnt2)
    Y = empty(h, torch.bfloat16)
    B.moe_unpermute_combine(ctx, Xp, B.BF16, row_of, prob, None, 0, k, h, Y)
    torch.cuda.synchronize()
    assert not counts.any() and not cnt2.any() and not offsets.any()
    assert (src_of == -1).all() and (Xp == 3.0).all()
    # all experts empty
    W = torch.ones((E, 2 * f, h), dtype=torch.bfloat16, device="cuda")
    A = torch.ones((Rcap, h), dtype=torch.bfloat16, device="cuda")
    Z = torch.full((Rcap, 2 * f), 3.0, dtype=torch.bfloat16, device="cuda")
    Act = torch.full((Rcap, f), 3.0, dtype=torch.bfloat16, device="cuda")
    dA = torch.full((Rcap, h), 3.0, dtype=torch.bfloat16, device="cuda")
    dW = torch.full((E, 2 * f, h), 3.0, dtype=torch.bfloat16, device="cuda")
    B.moe_grouped_gemm_fwd(ctx, A, W, offsets, E, 2 * f, h, Rcap, B.BF16, B.EPI_SWIGLU, None, None, Z, Act)
    B.moe_grouped_gemm_dgrad(ctx, Z, W, offsets, E, 2 * f, h, Rcap, B.BF16, None, None, None, dA)
    B.moe_grouped_gemm_wgrad(ctx, A, Z, offsets, E, 2 * f, h, Rcap, B.BF16, None, None, 0, B.BF16, dW)
    torch.cuda.synchronize()
    assert ctx.poll_error() == 0
    assert (Z == 3.0).all() and (Act == 3.0).all() and (dA == 3.0).all()
    assert not dW.any()
