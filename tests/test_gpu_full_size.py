"""GPU parity at the full benchmark sizes (C2, C3, C4 and the degenerate C4 load patterns, the fp8 and
MXFP8 configs), in the launch configuration bench.py times.

Integer results (routing indices, counts, row maps, offsets) are compared in full and bit-exactly.
Floating-point results are checked per library call on sampled outputs the oracle computes one by one
from the same bf16 input bits, per expert (nothing is pooled across experts):
  * rows of every forward / data-gradient tensor for EVERY live expert: at least 64 rows each (all rows of a
    smaller expert): both ends, the rows on either side of the first and last 256-row tile boundary, the
    ragged tail, random rows; for the largest expert, in addition one row in every 256-row band;
  * one 64x64 window of every weight gradient per expert, contracted over all rows of the expert; under the
    skewed loads (one expert with 40 % of the rows, Zipf) eight more windows in distinct 256x256 output tiles
    of the largest expert, whose tiles the kernel hands out dynamically;
  * the shared expert's tensors, including its activation and both weight gradients;
  * sampled tokens of the combine, its backward and the permute backward.
Bounds: per tensor and expert the relative Frobenius error (2e-2 bf16, 6e-2 one-byte operands against full
precision) and the same bound for every sampled row on its own.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

CASES = [("C2", None), ("C3", None), ("C4", None), ("C4", "zeros"), ("C4", "hot"),
         ("C5", None), ("C5", "zeros"), ("C5", "hot"), ("C6", None), ("C6", "zeros"), ("C6", "hot"), ("C4G", None)]
ROWS_PER_EXPERT = 64


def _f64(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def _sample_rows(lo, hi, g, n=ROWS_PER_EXPERT, every_band=False):
    """At least n rows of [lo, hi) (all of them if there are fewer): both ends, both sides of the first and the
    last 256-row tile boundary, the middle, random ones; every_band adds a random row in each 256-row band."""
    m = hi - lo
    if m <= n:
        return np.arange(lo, hi, dtype=np.int64)
    last = (m - 1) // 256 * 256
    cand = {lo, hi - 1, lo + min(255, m - 1), lo + min(256, m - 1), lo + last, lo + max(last - 1, 0), lo + m // 2}
    if every_band:
        cand |= {int(lo + b + g.integers(0, min(256, m - b))) for b in range(0, m, 256)}
    while len(cand) < n:
        cand |= {int(lo + v) for v in g.integers(0, m, size=n)}
    return np.array(sorted(c for c in cand if lo <= c < hi), dtype=np.int64)


@pytest.mark.parametrize("name,variant", CASES)
def test_full_size_sampled(oracle, name, variant):
    from gpu_util import assert_close, BF16_TOL, FP8_TOL, BF16_REG, permuted_rows, combine_bwd_rows
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS[name]
    g = np.random.default_rng(cfg.seed + (0 if variant is None else len(variant)))
    st = L.LayerState(cfg, None, variant=variant)
    st.step()
    torch.cuda.synchronize()
    assert st.ctx.poll_error() == 0
    T, k, E, h, f = cfg.T, cfg.k, cfg.E, cfg.h, cfg.f

    # ---- integer parts, in full ----
    logits = st.logits.cpu().numpy()
    if cfg.grouped_router:
        o_idx, o_prob, o_counts = oracle.route_topk_grouped(logits, k, cfg.n_group, cfg.topk_group, wl.expert_bias(cfg),
                                                            cfg.score, cfg.norm_topk, cfg.route_scale)
    else:
        o_idx, o_prob, o_counts = oracle.route_topk(logits, k, cfg.score, cfg.norm_topk, cfg.route_scale)
    assert np.array_equal(st.topk_idx.cpu().numpy(), o_idx)
    assert np.array_equal(st.route_counts.cpu().numpy(), o_counts)
    np.testing.assert_allclose(st.topk_prob.cpu().numpy(), o_prob, rtol=3e-6, atol=1e-9)
    idx = o_idx if st.forced_idx is None else st.forced_idx.cpu().numpy()
    m = oracle.permute_maps(idx, E, cfg.align, st.Rcap)
    assert np.array_equal(st.row_of.cpu().numpy(), m.row_of)
    assert np.array_equal(st.src_of.cpu().numpy(), m.src_of)
    assert np.array_equal(st.offsets.cpu().numpy(), m.offsets)
    assert np.array_equal(st.counts.cpu().numpy(), m.counts)
    assert int(m.counts.sum()) == T * k
    if variant == "zeros":
        assert int((m.counts == 0).sum()) == 4
    if variant == "hot":
        assert m.counts.max() >= 0.39 * T * k
    off = m.offsets

    one_byte = bool(cfg.fp8 or cfg.mx)
    # bounds per key: one-byte GEMM outputs against the full-precision oracle sit at the format's noise (3.6e-2 per
    # GEMM, 5e-2 behind the SwiGLU), so their regression bound is the contract bound itself; a row on its own
    # fluctuates around that figure by its 1/sqrt(columns), hence the wider row bound
    gemm_fwd_keys = {"Z", "A", "O", "dZ", "dXp", "Zs", "As", "S", "dZs", "dXs"}
    wgrad_keys = {"dW1", "dW2", "dWs1", "dWs2"}
    # which weight gradients run on one-byte operands: MXFP8 always, the blockwise recipe where the layer says so
    fp8_wgrad = bool(cfg.mx) or bool(getattr(st, "fp8_wgrad", False))

    def bounds(key):
        if one_byte and (key in gemm_fwd_keys or (key in wgrad_keys and fp8_wgrad)):
            return dict(tol=FP8_TOL, reg=None, row_tol=3 * FP8_TOL)
        return dict(tol=BF16_TOL, reg=BF16_REG, row_tol=BF16_TOL)

    # the row-wise quantiser of this config's recipe (for the layers that keep no bf16 copy of Xp and dO)
    row_quant = oracle.mx_quant_1x32 if cfg.mx else oracle.fp8_quant_1x128
    row_dequant = (lambda q, e: oracle.mx_dequant(q, e, "1x32")) if cfg.mx else (lambda q, e: oracle.fp8_dequant(q, e, "1x128"))
    worst = {}

    def chk(key, got, ref, tag, **kw):
        b = bounds(key)
        b.update(kw)
        e = assert_close(got, ref, f"{key} [{tag}]", **b)
        worst[key] = max(worst.get(key, 0.0), e)

    # ---- per-expert sampled rows and weight-gradient windows: every live expert ----
    live = [e for e in range(E) if m.counts[e] > 0]
    biggest = max(live, key=lambda e: m.counts[e])
    skewed = variant == "hot" or cfg.load == "zipf"
    one = lambda n: np.array([0, n], np.int32)
    n_rows_checked = 0
    for e in live:
        lo, hi = int(off[e]), int(off[e]) + int(m.counts[e])
        rows = _sample_rows(lo, hi, g, every_band=(e == biggest))
        assert len(rows) >= min(ROWS_PER_EXPERT, hi - lo)
        n_rows_checked += len(rows)
        rt = torch.from_numpy(rows).cuda()
        n = len(rows)
        tag = f"expert {e}"
        W1 = _f64(st.W1[e])[None]
        W2 = _f64(st.W2[e])[None]
        src_tok = m.src_of[rows] // k
        Xrows = _f64(st.X[torch.from_numpy(src_tok).cuda()])
        if st.Xp is not None:
            assert np.array_equal(_f64(st.Xp[rt]), Xrows)                   # permuted rows are exact copies
        else:                                                               # quantised straight from X: the codes are exact
            qo, eo = row_quant(Xrows)
            assert np.array_equal(st.qXp[rt].cpu().numpy(), qo) and np.array_equal(st.sXp[rt].cpu().numpy(), eo)
        Zref = oracle.grouped_gemm_nt(Xrows, W1, one(n))
        chk("Z", _f64(st.Z[rt]), Zref, tag)
        chk("A", _f64(st.A[rt]), oracle.swiglu(Zref), tag)
        Ag = _f64(st.A[rt])
        chk("O", _f64(st.O[rt]), oracle.grouped_gemm_nt(Ag, W2, one(n)), tag)
        dOg, Zg = _f64(combine_bwd_rows(st, rt)), _f64(st.Z[rt])
        if st.dO is None:
            qo, eo = row_quant(dOg)
            assert np.array_equal(st.qdO[rt].cpu().numpy(), qo) and np.array_equal(st.sdO[rt].cpu().numpy(), eo)
        chk("dZ", _f64(st.dZ[rt]), oracle.swiglu_bwd(oracle.grouped_gemm_nn(dOg, W2, one(n)), Zg), tag)
        chk("dXp", _f64(st.dXp[rt]), oracle.grouped_gemm_nn(_f64(st.dZ[rt]), W1, one(n)), tag)
        del W1, W2
        if one_byte:
            # the quantised copies the GEMMs read (made by quantiser launches or by the GEMM epilogues): bit for bit the
            # oracle's quantisers applied to the stored bf16 tensor -- the row-wise copies on the sampled rows, the
            # column-wise copies (the weight gradients' operands) on one 128-row group of the expert
            for nm, qn, sn in (("A", "qA", "sA"), ("dZ", "qdZ", "sdZ")):
                qo, eo = row_quant(_f64(getattr(st, nm)[rt]))
                assert np.array_equal(getattr(st, qn)[rt].cpu().numpy(), qo), (nm, tag, "row-wise codes")
                assert np.array_equal(getattr(st, sn)[rt].cpu().numpy(), eo), (nm, tag, "row-wise scales")
            if fp8_wgrad and cfg.align % 128 == 0:
                gi = int(g.integers(0, (int(off[e + 1]) - lo) // 128))
                r0 = lo + 128 * gi
                grp = torch.arange(r0, r0 + 128, device="cuda")
                # (256 columns of each tensor: a column's blocks do not depend on the other columns, and the oracle's
                # nearest-code search is slow)
                wcol = {"A": f, "dZ": 2 * f, "Xp": h, "dO": h}
                for nm, qn, sn in (("A", "qAc", "sAc"), ("dZ", "qdZc", "sdZc"), ("Xp", "qXpc", "sXpc"), ("dO", "qdOc", "sdOc")):
                    c0 = int(g.integers(0, wcol[nm] // 256)) * 256
                    cs = slice(c0, c0 + 256)
                    blk = {"A": lambda: st.A[grp, cs], "dZ": lambda: st.dZ[grp, cs], "Xp": lambda: permuted_rows(st, grp, cs),
                           "dO": lambda: combine_bwd_rows(st, grp, cs)}[nm]()
                    if cfg.mx:
                        qo, eo = oracle.mx_quant_32x1(_f64(blk)[None])
                        qo, eo = qo[0], eo[0]                  # [128, 256] codes, [256, 4] E8M0 bytes of the group
                    else:
                        qo, eo = oracle.fp8_quant_128x1(_f64(blk))
                        eo = eo[0]                             # [256] fp32 scales of the group
                    assert np.array_equal(getattr(st, qn)[grp, cs].cpu().numpy(), qo), (nm, tag, "column-wise codes")
                    assert np.array_equal(getattr(st, sn)[r0 // 128, cs].cpu().numpy(), eo), (nm, tag, "column-wise scales")
        # weight-gradient windows, contracted over every row of the expert
        hi_pad = hi
        allr = torch.arange(lo, hi_pad, device="cuda")
        wins2 = [(int(g.integers(0, h - 63)), int(g.integers(0, f - 63)))]
        wins1 = [(int(g.integers(0, 2 * f - 63)), int(g.integers(0, h - 63)))]
        if skewed and e == biggest:   # eight more windows, each in a different 256 x 256 output tile
            t2 = g.choice((h // 256) * (f // 256), size=8, replace=False)
            wins2 += [(int(t // (f // 256)) * 256 + int(g.integers(0, 193)), int(t % (f // 256)) * 256 + int(g.integers(0, 193))) for t in t2]
            t1 = g.choice((2 * f // 256) * (h // 256), size=8, replace=False)
            wins1 += [(int(t // (h // 256)) * 256 + int(g.integers(0, 193)), int(t % (h // 256)) * 256 + int(g.integers(0, 193))) for t in t1]
        for n0, k0 in wins2:
            ref = oracle.grouped_gemm_tn(_f64(combine_bwd_rows(st, allr, slice(n0, n0 + 64))), _f64(st.A[lo:hi_pad, k0:k0 + 64]),
                                         one(hi_pad - lo))[0]
            chk("dW2", _f64(st.dW2[e, n0:n0 + 64, k0:k0 + 64]), ref, f"{tag}, window ({n0}, {k0})")
        for n1, k1 in wins1:
            ref = oracle.grouped_gemm_tn(_f64(st.dZ[lo:hi_pad, n1:n1 + 64]), _f64(permuted_rows(st, allr, slice(k1, k1 + 64))),
                                         one(hi_pad - lo))[0]
            chk("dW1", _f64(st.dW1[e, n1:n1 + 64, k1:k1 + 64]), ref, f"{tag}, window ({n1}, {k1})")
    assert n_rows_checked >= min(ROWS_PER_EXPERT, int(m.counts[live].min())) * len(live)
    for e in range(E):                                                       # zero-token experts: exact zero gradients
        if m.counts[e] == 0:
            assert not st.dW1[e].any() and not st.dW2[e].any()

    # ---- shared expert (one group of T rows on the unpermuted tokens) ----
    if st.sf:
        sf = st.sf
        rows = _sample_rows(0, T, g, every_band=True)
        rt = torch.from_numpy(rows).cuda()
        n = len(rows)
        Ws1, Ws2 = _f64(st.Ws1)[None], _f64(st.Ws2)[None]
        Zs = oracle.grouped_gemm_nt(_f64(st.X[rt]), Ws1, one(n))
        chk("Zs", _f64(st.Zs[rt]), Zs, "shared")
        chk("As", _f64(st.As[rt]), oracle.swiglu(Zs), "shared")
        chk("S", _f64(st.S[rt]), oracle.grouped_gemm_nt(_f64(st.As[rt]), Ws2, one(n)), "shared")
        chk("dZs", _f64(st.dZs[rt]), oracle.swiglu_bwd(oracle.grouped_gemm_nn(_f64(st.dY[rt]), Ws2, one(n)), _f64(st.Zs[rt])), "shared")
        chk("dXs", _f64(st.dXs[rt]), oracle.grouped_gemm_nn(_f64(st.dZs[rt]), Ws1, one(n)), "shared")
        for _ in range(2):
            n0, k0 = int(g.integers(0, h - 63)), int(g.integers(0, sf - 63))
            chk("dWs2", _f64(st.dWs2[n0:n0 + 64, k0:k0 + 64]),
                oracle.grouped_gemm_tn(_f64(st.dY[:, n0:n0 + 64]), _f64(st.As[:, k0:k0 + 64]), one(T))[0], f"shared, window ({n0}, {k0})")
            n1, k1 = int(g.integers(0, 2 * sf - 63)), int(g.integers(0, h - 63))
            chk("dWs1", _f64(st.dWs1[n1:n1 + 64, k1:k1 + 64]),
                oracle.grouped_gemm_tn(_f64(st.dZs[:, n1:n1 + 64]), _f64(st.X[:, k1:k1 + 64]), one(T))[0], f"shared, window ({n1}, {k1})")

    # ---- combine, its backward and the permute backward on sampled tokens ----
    toks = np.unique(np.concatenate([[0, T - 1], g.integers(0, T, size=256)]))
    tt = torch.from_numpy(toks).cuda()
    r_of = m.row_of[toks]                                                    # [n, k]
    flat = torch.from_numpy(r_of.reshape(-1).astype(np.int64)).cuda()
    Osub = _f64(st.O[flat])
    dXpsub = _f64(st.dXp[flat])
    local_rows = np.arange(len(toks) * k, dtype=np.int32).reshape(len(toks), k)
    prob = st.topk_prob.cpu().numpy().astype(np.float64)[toks]
    S = _f64(st.S[tt]) if st.sf else None
    chk("Y", _f64(st.Y[tt]), oracle.combine(Osub, local_rows, prob, S), "tokens")
    dOref, dpref = oracle.combine_bwd(_f64(st.dY[tt]), Osub, local_rows, prob, len(toks) * k)
    if st.dO is not None:
        chk("dO", _f64(st.dO[flat]), dOref, "tokens")
    else:
        # only the quantised copies of dO exist: dequantise what the GPU wrote (the row-wise copy) and compare that with
        # the oracle's dO, at the format's bound
        deq = row_dequant(st.qdO[flat].cpu().numpy(), st.sdO[flat].cpu().numpy())
        chk("dO", deq, dOref, "tokens, dequantised codes", tol=FP8_TOL, reg=None, row_tol=FP8_TOL)
    chk("dprob", st.dprob.cpu().numpy().astype(np.float64)[toks], dpref, "tokens", row_floor=0.05)
    chk("dX", _f64(st.dX[tt]), oracle.combine(dXpsub, local_rows, None, _f64(st.dXs[tt]) if st.sf else None), "tokens")

    print(name, variant, f"{len(live)} experts, {n_rows_checked} rows;", {k_: f"{v:.2e}" for k_, v in worst.items()})


@pytest.mark.parametrize("name,variant,eq2", [("C4", None, False), ("C4", "hot", True), ("C3", None, False), ("C2", None, True)])
def test_full_size_gathered_operands_bit_identical(name, variant, eq2):
    """The permute's row move fused into the GEMMs (no Xp; with eq. (2) no dO): at the benchmark sizes, in the launch
    configuration bench.py times, every tensor of the step equals, bit for bit, that of the path with the stand-alone
    mover, which test_full_size_sampled holds against the oracle.  (hot / Zipf loads: the weight gradients split
    their contraction and hand tiles out dynamically.)"""
    from paper_2603_07685_amd import layer as L
    from paper_2603_07685_amd import workloads as wl
    cfg = wl.CONFIGS[name]
    a = L.LayerState(cfg, None, variant=variant, eq2=eq2)
    b = L.LayerState(cfg, None, variant=variant, eq2=eq2, gather=True)
    assert b.Xp is None and (b.dO is None) == eq2
    for st in (a, b):
        st.step()
    torch.cuda.synchronize()
    assert a.ctx.poll_error() == 0 and b.ctx.poll_error() == 0
    R = int(a.offsets[-1].item())
    for n in ["row_of", "src_of", "offsets", "counts"]:
        assert torch.equal(getattr(a, n), getattr(b, n)), n
    for n in ["Z", "A", "O", "dZ", "dXp"]:
        assert torch.equal(getattr(a, n)[:R].view(torch.int16), getattr(b, n)[:R].view(torch.int16)), n
    for n in ["Y", "dX", "dW1", "dW2"] + (["dWs1", "dWs2"] if a.sf else []):
        assert torch.equal(getattr(a, n).view(torch.int16), getattr(b, n).view(torch.int16)), n
    assert torch.equal(a.dprob.view(torch.int32), b.dprob.view(torch.int32))
