"""GPU parity of the fp8 layer (config-5 recipe) at a reduced size, every element, per library call:
each GEMM output is compared with the full-precision oracle fed the same bf16 inputs the GPU call
consumed (bound 6e-2 for the fp8 GEMMs, 2e-2 for the bf16 parts), for the three load patterns of
config 5 (mild imbalance, four empty experts, one expert with 40 % of the rows)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _checkers():
    """(c8, c16): element-level checks of a one-byte GEMM's output against the full-precision oracle (6e-2 pooled; a
    row on its own fluctuates around the format's noise, hence 3 x for rows: a wrong row is off by its whole norm) and of a bf16 result (2e-2 pooled and
    per row, 6e-3 regression bound); dprob is a handful of dot products per row (sums with cancellation: the error
    scales with the operands, not with the result), so its rows are checked against the typical row."""
    from gpu_util import assert_close, BF16_TOL, FP8_TOL

    def c8(key, got, ref):
        return assert_close(got, ref, key, tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL, row_floor=0.3 if key == "dprob" else 1e-6)

    def c16(key, got, ref):
        return assert_close(got, ref, key, row_floor=0.05 if key == "dprob" else 1e-6)

    return c8, c16


@pytest.mark.parametrize("variant", [None, "zeros", "hot"])
def test_fp8_layer_every_element(oracle, variant):
    from gpu_util import rel_fro, BF16_TOL, FP8_TOL
    c8, c16 = _checkers()
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS["C5S"]
    hin = L.host_inputs(cfg)
    st = L.LayerState(cfg, hin, variant=variant, fused_quant=False)      # (per-call checks read the bf16 Xp and dO)
    assert st.fp8 and st.align == 128 and st.fp8_wgrad
    st.step()
    torch.cuda.synchronize()
    assert st.ctx.poll_error() == 0
    T, k, E, h, f = cfg.T, cfg.k, cfg.E, cfg.h, cfg.f

    o_idx, o_prob, _ = oracle.route_topk(hin["logits"], k, cfg.score, cfg.norm_topk)
    assert np.array_equal(st.topk_idx.cpu().numpy(), o_idx)
    idx = st.forced_idx.cpu().numpy()
    m = oracle.permute_maps(idx, E, 128, st.Rcap)
    for name, ref in (("row_of", m.row_of), ("src_of", m.src_of), ("offsets", m.offsets), ("counts", m.counts)):
        assert np.array_equal(getattr(st, name).cpu().numpy(), ref), name
    assert np.all(m.offsets % 128 == 0)
    if variant == "zeros":
        assert (m.counts == 0).sum() == 4
    if variant == "hot":
        assert m.counts.max() >= 0.39 * T * k
    R, off = m.Rtot, m.offsets
    Xp = oracle.permute_rows(hin["X"], m.src_of[:R], k)
    assert np.array_equal(_f64(st.Xp)[:R], Xp)                           # includes the zero padding rows

    W1, W2, Ws1, Ws2 = hin["W1"], hin["W2"], hin["Ws1"][None], hin["Ws2"][None]
    e8, e16 = {}, {}
    Zref = oracle.grouped_gemm_nt(Xp, W1, off)
    e8["Z"] = c8("Z", _f64(st.Z)[:R], Zref)
    e8["A"] = c8("A", _f64(st.A)[:R], oracle.swiglu(Zref))
    e8["O"] = c8("O", _f64(st.O)[:R], oracle.grouped_gemm_nt(_f64(st.A)[:R], W2, off))
    o1 = np.array([0, T], np.int32)
    e8["Zs"] = c8("Zs", _f64(st.Zs), oracle.grouped_gemm_nt(hin["X"], Ws1, o1))
    e8["S"] = c8("S", _f64(st.S), oracle.grouped_gemm_nt(_f64(st.As), Ws2, o1))
    prob = st.topk_prob.cpu().numpy().astype(np.float64)
    e16["Y"] = c16("Y", _f64(st.Y), oracle.combine(_f64(st.O)[:R], m.row_of, prob, _f64(st.S)))
    dOref, dpref = oracle.combine_bwd(hin["dY"], _f64(st.O)[:R], m.row_of, prob, R)
    e16["dO"] = c16("dO", _f64(st.dO)[:R], dOref)
    assert np.all(_f64(st.dO)[:R][m.src_of[:R] < 0] == 0)                 # padding rows of dO are exact zeros
    e16["dprob"] = c16("dprob", st.dprob.cpu().numpy(), dpref)
    dOg, Zg, dZg = _f64(st.dO)[:R], _f64(st.Z)[:R], _f64(st.dZ)[:R]
    cw = c8 if st.fp8_wgrad else c16                                       # the weight gradients run on E4M3 codes too
    ew = e8 if st.fp8_wgrad else e16
    ew["dW2"] = cw("dW2", _f64(st.dW2), oracle.grouped_gemm_tn(dOg, _f64(st.A)[:R], off))
    ew["dWs2"] = cw("dWs2", _f64(st.dWs2), oracle.grouped_gemm_tn(hin["dY"], _f64(st.As), o1)[0])
    e8["dZ"] = c8("dZ", dZg, oracle.swiglu_bwd(oracle.grouped_gemm_nn(dOg, W2, off), Zg))
    ew["dW1"] = cw("dW1", _f64(st.dW1), oracle.grouped_gemm_tn(dZg, Xp, off))
    e8["dXp"] = c8("dXp", _f64(st.dXp)[:R], oracle.grouped_gemm_nn(dZg, W1, off))
    e8["dZs"] = c8("dZs", _f64(st.dZs), oracle.swiglu_bwd(oracle.grouped_gemm_nn(hin["dY"], Ws2, o1), _f64(st.Zs)))
    e8["dXs"] = c8("dXs", _f64(st.dXs), oracle.grouped_gemm_nn(_f64(st.dZs), Ws1, o1))
    ew["dWs1"] = cw("dWs1", _f64(st.dWs1), oracle.grouped_gemm_tn(_f64(st.dZs), hin["X"], o1)[0])
    e16["dX"] = c16("dX", _f64(st.dX), oracle.combine(_f64(st.dXp)[:R], m.row_of, None, _f64(st.dXs)))
    for e in range(E):
        if m.counts[e] == 0:
            assert not st.dW1[e].any() and not st.dW2[e].any()
    print(variant, "fp8:", {k_: f"{v:.2e}" for k_, v in e8.items()}, "bf16:", {k_: f"{v:.2e}" for k_, v in e16.items()})
    for k_, v in e8.items():
        assert v <= FP8_TOL, (k_, v)
    for k_, v in e16.items():
        assert v <= BF16_TOL, (k_, v)
    # end-to-end against the full-precision layer (reported; the chain of three fp8 stages may sit near the bound)
    fw = oracle.layer_forward(hin["X"], idx, o_prob, W1, W2, E, 128, hin["Ws1"], hin["Ws2"])
    print("end-to-end Y vs full-precision oracle:", f"{rel_fro(_f64(st.Y), fw.Y):.2e}")
    assert rel_fro(_f64(st.Y), fw.Y) <= 0.1


def test_fp8_layer_eq2_per_call(oracle):
    """C5S in the memory-efficient permutation form (eq. (2)) with the fp8 GEMMs: the calls that differ from the
    standard form, each against the oracle on the tensors the GPU actually fed it."""
    from gpu_util import rel_fro, BF16_TOL, FP8_TOL
    c8, c16 = _checkers()
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS["C5S"]
    hin = L.host_inputs(cfg)
    st = L.LayerState(cfg, hin, eq2=True, fused_quant=False)
    st.step()
    torch.cuda.synchronize()
    assert st.ctx.poll_error() == 0
    T, k, E = cfg.T, cfg.k, cfg.E
    idx = st.forced_idx.cpu().numpy()
    m = oracle.permute_maps(idx, E, 128, st.Rcap)
    R, off = m.Rtot, m.offsets
    prob = st.topk_prob.cpu().numpy().astype(np.float64)
    row_p = oracle.gather_row_prob(prob, m.src_of[:R])
    np.testing.assert_array_equal(st.row_prob.cpu().numpy()[:R], row_p.astype(np.float32))
    Xp = oracle.permute_rows(hin["X"], m.src_of[:R], k)
    Zref = oracle.grouped_gemm_nt(Xp, hin["W1"], off)
    e8 = {"Z": c8("Z", _f64(st.Z)[:R], Zref),
          "A": c8("A", _f64(st.A)[:R], oracle.swiglu(Zref) * row_p[:, None])}
    assert np.all(_f64(st.A)[:R][m.src_of[:R] < 0] == 0)                  # padding rows carry weight 0
    Y = oracle.combine(_f64(st.O)[:R], m.row_of, None, _f64(st.S))
    e16 = {"Y": c8("Y", _f64(st.Y), Y)}
    dOref = oracle.permute_rows(hin["dY"], m.src_of[:R], k)
    assert np.array_equal(_f64(st.dO)[:R], dOref)
    dA = oracle.grouped_gemm_nn(dOref, hin["W2"], off)
    Zg = _f64(st.Z)[:R]
    e8["dZ"] = c8("dZ", _f64(st.dZ)[:R], oracle.swiglu_bwd(dA, Zg) * row_p[:, None])
    dp_row = (dA * oracle.swiglu(Zg)).sum(axis=1)
    dp = np.where(m.row_of >= 0, dp_row[np.maximum(m.row_of, 0)], 0.0)
    e8["dprob"] = c8("dprob", st.dprob.cpu().numpy(), dp)
    print("eq2 fp8:", {k_: f"{v:.2e}" for k_, v in e8.items()}, "bf16:", {k_: f"{v:.2e}" for k_, v in e16.items()})
    for k_, v in e8.items():
        assert v <= FP8_TOL, (k_, v)
    for k_, v in e16.items():
        assert v <= BF16_TOL, (k_, v)


def test_mxfp8_layer_per_call(oracle):
    """C6S: the layer with MXFP8 (1x32, E8M0) forward / data-gradient / weight-gradient GEMMs, every element, per call: each GPU
    result against the oracle applied to the tensors the GPU fed that call (bound 6e-2 for the fp8 calls)."""
    from gpu_util import rel_fro, BF16_TOL, FP8_TOL
    c8, c16 = _checkers()
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS["C6S"]
    hin = L.host_inputs(cfg)
    st = L.LayerState(cfg, hin, fused_quant=False)
    assert st.mx and st.fp8
    st.step()
    torch.cuda.synchronize()
    assert st.ctx.poll_error() == 0
    T, k, E = cfg.T, cfg.k, cfg.E
    idx = st.forced_idx.cpu().numpy()
    m = oracle.permute_maps(idx, E, 128, st.Rcap)
    R, off = m.Rtot, m.offsets
    Xp = oracle.permute_rows(hin["X"], m.src_of[:R], k)
    assert np.array_equal(_f64(st.Xp)[:R], Xp)
    # the quantised operands the GEMMs read, bit for bit
    qo, eo = oracle.mx_quant_1x32(Xp)
    assert np.array_equal(st.qXp.cpu().numpy()[:R], qo) and np.array_equal(st.sXp.cpu().numpy()[:R], eo)
    qo, eo = oracle.mx_quant_32x1(hin["W1"])
    f2, h_ = hin["W1"].shape[1:]
    col = lambda s_, G, N, K: s_.cpu().numpy().reshape(G, N // 128, K, 4).transpose(0, 2, 1, 3).reshape(G, K, N // 32)
    assert np.array_equal(st.qW1d.cpu().numpy(), qo) and np.array_equal(col(st.sW1d, E, f2, h_), eo)
    qo, eo = oracle.mx_quant_32x1(Xp[None])                   # the weight-gradient copy of the permuted tokens
    assert np.array_equal(st.qXpc.cpu().numpy()[:R], qo[0])
    assert np.array_equal(col(st.sXpc, 1, st.Rcap, h_)[0, :, :R // 32], eo[0])
    W1, W2, Ws1, Ws2 = hin["W1"], hin["W2"], hin["Ws1"][None], hin["Ws2"][None]
    o1 = np.array([0, T], np.int32)
    prob = st.topk_prob.cpu().numpy().astype(np.float64)
    Zref = oracle.grouped_gemm_nt(Xp, W1, off)
    dOg, Zg, dZg = _f64(st.dO)[:R], _f64(st.Z)[:R], _f64(st.dZ)[:R]
    e8 = {
        "Z": c8("Z", _f64(st.Z)[:R], Zref), "A": c8("A", _f64(st.A)[:R], oracle.swiglu(Zref)),
        "O": c8("O", _f64(st.O)[:R], oracle.grouped_gemm_nt(_f64(st.A)[:R], W2, off)),
        "Zs": c8("Zs", _f64(st.Zs), oracle.grouped_gemm_nt(hin["X"], Ws1, o1)),
        "S": c8("S", _f64(st.S), oracle.grouped_gemm_nt(_f64(st.As), Ws2, o1)),
        "dZ": c8("dZ", dZg, oracle.swiglu_bwd(oracle.grouped_gemm_nn(dOg, W2, off), Zg)),
        "dXp": c8("dXp", _f64(st.dXp)[:R], oracle.grouped_gemm_nn(dZg, W1, off)),
        "dZs": c8("dZs", _f64(st.dZs), oracle.swiglu_bwd(oracle.grouped_gemm_nn(hin["dY"], Ws2, o1), _f64(st.Zs))),
        "dXs": c8("dXs", _f64(st.dXs), oracle.grouped_gemm_nn(_f64(st.dZs), Ws1, o1)),
        "dW2": c8("dW2", _f64(st.dW2), oracle.grouped_gemm_tn(dOg, _f64(st.A)[:R], off)),
        "dW1": c8("dW1", _f64(st.dW1), oracle.grouped_gemm_tn(dZg, Xp, off)),
        "dWs2": c8("dWs2", _f64(st.dWs2), oracle.grouped_gemm_tn(hin["dY"], _f64(st.As), o1)[0]),
        "dWs1": c8("dWs1", _f64(st.dWs1), oracle.grouped_gemm_tn(_f64(st.dZs), hin["X"], o1)[0]),
    }
    e16 = {
        "Y": c16("Y", _f64(st.Y), oracle.combine(_f64(st.O)[:R], m.row_of, prob, _f64(st.S))),
        "dX": c16("dX", _f64(st.dX), oracle.combine(_f64(st.dXp)[:R], m.row_of, None, _f64(st.dXs))),
    }
    print("mxfp8:", {k_: f"{v:.2e}" for k_, v in e8.items()}, "bf16:", {k_: f"{v:.2e}" for k_, v in e16.items()})
    for k_, v in e8.items():
        assert v <= FP8_TOL, (k_, v)
    for k_, v in e16.items():
        assert v <= BF16_TOL, (k_, v)


@pytest.mark.parametrize("eq2", [False, True])
def test_mxfp8_fused_quantisation_is_bit_identical(oracle, eq2):
    """C6S: quantising the permuted tokens and the combine's backward straight from X / dY through the row map
    (no bf16 Xp or dO) gives the GEMMs the very same codes and scales, so every output of the step is bit-identical
    to the unfused path; the codes themselves are checked against the oracle."""
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS["C6S"]
    hin = L.host_inputs(cfg)
    a = L.LayerState(cfg, hin, eq2=eq2, fused_quant=False)
    b = L.LayerState(cfg, hin, eq2=eq2, fused_quant=True)
    assert b.Xp is None and b.dO is None
    for st in (a, b):
        st.step()
    torch.cuda.synchronize()
    assert a.ctx.poll_error() == 0 and b.ctx.poll_error() == 0
    R = int(a.offsets[-1].item())
    for n in ["qXp", "sXp", "qXpc", "qdO", "sdO", "qdOc"]:
        assert torch.equal(getattr(a, n)[:R], getattr(b, n)[:R]), n
    for n in ["sXpc", "sdOc"]:
        assert torch.equal(getattr(a, n)[:R // 128], getattr(b, n)[:R // 128]), n
    for n in ["Y", "dX", "dW1", "dW2", "dprob", "dWs1", "dWs2", "Z", "dZ"]:
        x, y = getattr(a, n), getattr(b, n)
        assert torch.equal(x[:R] if n in ("Z", "dZ") else x, y[:R] if n in ("Z", "dZ") else y), n
    # against the oracle: codes of the permuted tokens (padding rows included) and of dO = bf16(p * dY)
    idx = b.forced_idx.cpu().numpy()
    m = oracle.permute_maps(idx, cfg.E, 128, b.Rcap)
    Xp = oracle.permute_rows(hin["X"], m.src_of[:R], cfg.k)
    qo, eo = oracle.mx_quant_1x32(Xp)
    assert np.array_equal(b.qXp.cpu().numpy()[:R], qo) and np.array_equal(b.sXp.cpu().numpy()[:R], eo)
    src = m.src_of[:R]
    dO = hin["dY"].astype(np.float32)[np.maximum(src, 0) // cfg.k]
    if not eq2:
        dO = wl.bf16_round(dO * b.topk_prob.cpu().numpy().reshape(-1)[np.maximum(src, 0)][:, None])
    dO[src < 0] = 0
    qo, eo = oracle.mx_quant_1x32(dO)
    assert np.array_equal(b.qdO.cpu().numpy()[:R], qo) and np.array_equal(b.sdO.cpu().numpy()[:R], eo)
    qc, ec = oracle.mx_quant_32x1(dO[None])
    assert np.array_equal(b.qdOc.cpu().numpy()[:R], qc[0])
    ecg = b.sdOc.cpu().numpy().reshape(1, b.Rcap // 128, cfg.h, 4).transpose(0, 2, 1, 3).reshape(cfg.h, b.Rcap // 32)
    assert np.array_equal(ecg[:, :R // 32], ec[0])


@pytest.mark.parametrize("eq2", [False, True])
def test_fp8_fused_quantisation_is_bit_identical(oracle, eq2):
    """C5S, blockwise recipe: quantising the permuted tokens and the combine's backward straight from X / dY through
    the row map, 1x128 and 128x1 in one pass, padding included (no bf16 Xp or dO), gives the GEMMs the very same codes
    and scales, so every output of the step is bit-identical to the unfused path; the codes are checked against the
    oracle's quantisers."""
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS["C5S"]
    hin = L.host_inputs(cfg)
    a = L.LayerState(cfg, hin, eq2=eq2, fused_quant=False)
    b = L.LayerState(cfg, hin, eq2=eq2)
    assert b.fused_quant and b.fp8_wgrad and b.Xp is None and b.dO is None
    for st in (a, b):
        st.step()
    torch.cuda.synchronize()
    assert a.ctx.poll_error() == 0 and b.ctx.poll_error() == 0
    R = int(a.offsets[-1].item())
    for n in ["qXp", "sXp", "qXpc", "qdO", "sdO", "qdOc"]:
        assert torch.equal(getattr(a, n)[:R], getattr(b, n)[:R]), n
    for n in ["sXpc", "sdOc"]:
        assert torch.equal(getattr(a, n)[:R // 128], getattr(b, n)[:R // 128]), n
    for n in ["Y", "dX", "dW1", "dW2", "dprob", "dWs1", "dWs2", "Z", "dZ"]:
        x, y = getattr(a, n), getattr(b, n)
        assert torch.equal(x[:R] if n in ("Z", "dZ") else x, y[:R] if n in ("Z", "dZ") else y), n
    idx = b.forced_idx.cpu().numpy()
    m = oracle.permute_maps(idx, cfg.E, 128, b.Rcap)
    Xp = oracle.permute_rows(hin["X"], m.src_of[:R], cfg.k)
    qo, so = oracle.fp8_quant_1x128(Xp)
    assert np.array_equal(b.qXp.cpu().numpy()[:R], qo) and np.array_equal(b.sXp.cpu().numpy()[:R], so)
    qc, sc = oracle.fp8_quant_128x1(Xp)
    assert np.array_equal(b.qXpc.cpu().numpy()[:R], qc) and np.array_equal(b.sXpc.cpu().numpy()[:R // 128], sc)
    src = m.src_of[:R]
    dO = hin["dY"].astype(np.float32)[np.maximum(src, 0) // cfg.k]
    if not eq2:
        dO = wl.bf16_round(dO * b.topk_prob.cpu().numpy().reshape(-1)[np.maximum(src, 0)][:, None])
    dO[src < 0] = 0
    qo, so = oracle.fp8_quant_1x128(dO)
    assert np.array_equal(b.qdO.cpu().numpy()[:R], qo) and np.array_equal(b.sdO.cpu().numpy()[:R], so)
    qc, sc = oracle.fp8_quant_128x1(dO)
    assert np.array_equal(b.qdOc.cpu().numpy()[:R], qc) and np.array_equal(b.sdOc.cpu().numpy()[:R // 128], sc)


@pytest.mark.parametrize("eq2", [False, True])
def test_fp8_epilogue_quantisation_is_bit_identical(eq2):
    """C5S: the codes and scales the SwiGLU / SwiGLU-backward epilogues emit (routed and shared expert) equal those of
    the stand-alone 1x128 quantiser run on the stored bf16 tensor, so every output of the step is bit-identical."""
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS["C5S"]
    hin = L.host_inputs(cfg)
    a = L.LayerState(cfg, hin, eq2=eq2, epilogue_quant=False, fused_quant=False)
    b = L.LayerState(cfg, hin, eq2=eq2, epilogue_quant=True, fused_quant=False)
    for st in (a, b):
        for n in ("qA", "sA", "qdZ", "sdZ", "qAs", "sAs", "qdZs", "sdZs"):
            getattr(st, n).zero_()
        st.step()
    torch.cuda.synchronize()
    assert a.ctx.poll_error() == 0 and b.ctx.poll_error() == 0
    R = int(a.offsets[-1].item())
    for n in ("qA", "sA", "qdZ", "sdZ"):
        assert torch.equal(getattr(a, n)[:R], getattr(b, n)[:R]), n
    for n in ("qAs", "sAs", "qdZs", "sdZs", "Y", "dX", "dW1", "dW2", "dprob", "dWs1", "dWs2"):
        assert torch.equal(getattr(a, n), getattr(b, n)), n
    assert not b.qA[R:].any() and not b.qdZ[R:].any()          # rows beyond the live ones are not written


@pytest.mark.parametrize("eq2", [False, True])
def test_mxfp8_epilogue_quantisation_is_bit_identical(eq2):
    """C6S: the 1x32 and 32x1 copies of A and dZ (routed and shared expert) that the SwiGLU / SwiGLU-backward
    epilogues emit equal those of the stand-alone row+column quantiser run on the stored bf16 tensor, so every
    output of the step is bit-identical."""
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS["C6S"]
    hin = L.host_inputs(cfg)
    a = L.LayerState(cfg, hin, eq2=eq2, epilogue_quant=False)
    b = L.LayerState(cfg, hin, eq2=eq2, epilogue_quant=True)
    names = ("qA", "sA", "qAc", "sAc", "qdZ", "sdZ", "qdZc", "sdZc", "qAs", "sAs", "qAsc", "sAsc", "qdZs", "sdZs", "qdZsc", "sdZsc")
    for st in (a, b):
        for n in names:
            getattr(st, n).zero_()
        st.step()
    torch.cuda.synchronize()
    assert a.ctx.poll_error() == 0 and b.ctx.poll_error() == 0
    R = int(a.offsets[-1].item())
    for n in ("qA", "sA", "qAc", "qdZ", "sdZ", "qdZc"):
        assert torch.equal(getattr(a, n)[:R], getattr(b, n)[:R]), n
    for n in ("sAc", "sdZc"):
        assert torch.equal(getattr(a, n)[:R // 128], getattr(b, n)[:R // 128]), n
    for n in ("qAs", "sAs", "qAsc", "sAsc", "qdZs", "sdZs", "qdZsc", "sdZsc", "Y", "dX", "dW1", "dW2", "dprob", "dWs1", "dWs2"):
        assert torch.equal(getattr(a, n), getattr(b, n)), n
    assert not b.qA[R:].any() and not b.qdZ[R:].any() and not b.qAc[R:].any() and not b.qdZc[R:].any()
