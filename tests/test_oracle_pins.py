"""Pins of the CPU oracle to things other than itself (CPU only).

Each test checks an oracle step against a closed form, an invariant, a library
routine on a special case, a brute-force restatement with a different structure,
or finite differences - chosen so that a dropped term, a wrong sign or index or
a transposed operand fails at least one of them.  Citations are to the paper's
sections / equations.
"""
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------------------
# Router (Sec. 1.1 definition; Sec. 2.1.2 item 2)
# ---------------------------------------------------------------------------
def test_router_closed_form_golden(oracle):
    """Worked closed-form cases stored in tests/golden/router_closed_form.txt."""
    path = os.path.join(HERE, "golden", "router_closed_form.txt")
    cases = []
    with open(path) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if not line:
                continue
            score, norm, k, ratios, idx, w = [s.strip() for s in line.split("|")]
            cases.append((int(score), int(norm), int(k), [float(v) for v in ratios.split()],
                          [int(v) for v in idx.split()], [float(v) for v in w.split()]))
    assert len(cases) >= 4
    for score, norm, k, ratios, idx_exp, w_exp in cases:
        r = np.array(ratios, np.float64)
        # softmax rows are given as odds e^l (l = ln r); sigmoid rows as odds s/(1-s) (l = ln r)
        logits = np.log(r).astype(np.float32)[None, :]
        idx, w, counts = oracle.route_topk(logits, k, score, bool(norm))
        assert idx[0].tolist() == idx_exp
        np.testing.assert_allclose(w[0], w_exp, rtol=2e-7)  # fp32 logits carry ~6e-8 relative error
        assert counts.sum() == k


@pytest.mark.parametrize("score", [0, 1])
@pytest.mark.parametrize("norm", [False, True])
def test_router_vs_bruteforce_sort(oracle, score, norm):
    g = _rng(3)
    T, E, k = 200, 37, 5
    logits = g.standard_normal((T, E)).astype(np.float32)
    idx, w, counts = oracle.route_topk(logits, k, score, norm, scale=2.5)
    l64 = logits.astype(np.float64)
    if score == 0:
        s = np.exp(l64 - l64.max(1, keepdims=True))
        s /= s.sum(1, keepdims=True)
        np.testing.assert_allclose(s.sum(1), 1.0, rtol=1e-14)
    else:
        s = 1.0 / (1.0 + np.exp(-l64))
    # selection on the scores (what the paper states) == selection on the logits (what the oracle does)
    order = np.argsort(-s, axis=1, kind="stable")[:, :k]
    assert np.array_equal(order, idx)
    ws = np.take_along_axis(s, order, 1)
    if norm:
        ws = ws / ws.sum(1, keepdims=True)
        np.testing.assert_allclose(w.sum(1), 2.5, rtol=1e-13)
    np.testing.assert_allclose(w, 2.5 * ws, rtol=1e-12)
    assert np.all(w >= 0)
    assert np.array_equal(counts, np.bincount(order.ravel(), minlength=E))
    assert counts.sum() == T * k
    # descending slot order
    assert np.all(np.diff(np.take_along_axis(l64, idx.astype(np.int64), 1), axis=1) <= 0)


def test_router_k_equals_E_and_ties(oracle):
    g = _rng(4)
    logits = g.standard_normal((16, 6)).astype(np.float32)
    idx, w, counts = oracle.route_topk(logits, 6, 0, False)
    assert np.all(np.sort(idx, 1) == np.arange(6))
    np.testing.assert_allclose(w.sum(1), 1.0, rtol=1e-14)      # softmax over all experts sums to one
    assert np.all(counts == 16)
    # ties: equal logits -> lower expert index first
    t = np.array([[1.0, 3.0, 3.0, 0.5, 3.0, 1.0]], np.float32)
    idx, w, _ = oracle.route_topk(t, 4, 1, True)
    assert idx[0].tolist() == [1, 2, 4, 0]
    np.testing.assert_allclose(w.sum(), 1.0, rtol=1e-14)
    assert w[0, 0] == w[0, 1] == w[0, 2]
    # f32 instantiation selects the same experts
    idx32, w32, _ = oracle.route_topk(logits, 3, 0, False, prec="f32")
    idx64, w64, _ = oracle.route_topk(logits, 3, 0, False, prec="f64")
    assert np.array_equal(idx32, idx64)
    np.testing.assert_allclose(w32, w64, rtol=1e-6)


# ---------------------------------------------------------------------------
# Router branches: group-limited top-k, expert bias, scaling (Sec. 4.3.4 item 1; Sec. 7)
# ---------------------------------------------------------------------------
def test_grouped_router_worked_examples(oracle):
    """Cases small enough to do by hand.  Sigmoid of ln(r) is r / (1 + r): logits ln 1, ln 3, ln(1/3), ln 9 give
    scores 1/2, 3/4, 1/4, 9/10."""
    ln = lambda r: float(np.log(r))
    # E = 4, two groups {0,1} and {2,3}, keep one group, k = 1: group scores (best single) 1/2 and 3/4 -> group 1
    lg = np.array([[ln(1), ln(1), ln(3), ln(1 / 3)]], np.float32)
    idx, w, cnt = oracle.route_topk_grouped(lg, 1, 2, 1, None, 1, False, 1.0)
    assert idx.tolist() == [[2]] and cnt.tolist() == [0, 0, 1, 0]
    np.testing.assert_allclose(w, [[0.75]], rtol=1e-7)
    # k = 2 from one group: group scores are sums of two: 1/2 + 1/2 = 1 = 3/4 + 1/4: the tie goes to group 0
    idx, w, _ = oracle.route_topk_grouped(lg, 2, 2, 1, None, 1, True, 2.0)
    assert idx.tolist() == [[0, 1]]
    np.testing.assert_allclose(w, [[1.0, 1.0]], rtol=1e-7)                 # (1/2) / 1 * 2
    # without the group limit the two best experts are 2 (3/4) and then 0 (1/2, lower index of the tie)
    idx, w, _ = oracle.route_topk_grouped(lg, 2, 1, 1, None, 1, True, 1.0)
    assert idx.tolist() == [[2, 0]]
    np.testing.assert_allclose(w, [[0.6, 0.4]], rtol=1e-7)
    # the group limit excludes the single best expert when its group loses: scores 9/10, 0 | 1/2, 1/2 with
    # two per group: sums 0.9 + ~0 < 1
    lg2 = np.array([[ln(9), -40.0, ln(1), ln(1)]], np.float32)
    idx, w, _ = oracle.route_topk_grouped(lg2, 2, 2, 1, None, 1, False, 1.0)
    assert idx.tolist() == [[2, 3]]
    # a bias decides the selection but not the weight: +1 on expert 3 (score 1/4) makes it the winner, weight 1/4
    b = np.array([0, 0, 0, 1], np.float32)
    idx, w, _ = oracle.route_topk_grouped(lg, 1, 1, 1, b, 1, False, 1.0)
    assert idx.tolist() == [[3]]
    np.testing.assert_allclose(w, [[0.25]], rtol=1e-7)
    # ... and moves the group choice too: {2,3} now scores 1.25 + 0.75
    idx, w, _ = oracle.route_topk_grouped(lg, 2, 2, 1, b, 1, True, 1.0)
    assert idx.tolist() == [[3, 2]]
    np.testing.assert_allclose(w, [[0.25, 0.75]], rtol=1e-7)
    # softmax: odds 1 : 2 : 3 : 4 -> probabilities 0.1 .. 0.4; groups {0,1} = 0.2 (best single), {2,3} = 0.4
    lg3 = np.log(np.array([[1, 2, 3, 4]], np.float64)).astype(np.float32)
    idx, w, _ = oracle.route_topk_grouped(lg3, 1, 2, 1, None, 0, False, 1.0)
    assert idx.tolist() == [[3]]
    np.testing.assert_allclose(w, [[0.4]], rtol=1e-6)
    with pytest.raises(ValueError):
        oracle.route_topk_grouped(lg, 3, 2, 1)          # k not a multiple of topk_group / more than the groups hold
    with pytest.raises(ValueError):
        oracle.route_topk_grouped(lg, 2, 3, 1)          # E not divisible into the groups


@pytest.mark.parametrize("score", [0, 1])
def test_grouped_router_reduces_to_plain_router(oracle, score):
    """One group and no bias (or a constant bias) is the plain router, which has its own pins."""
    g = _rng(41 + score)
    logits = g.standard_normal((300, 48)).astype(np.float32)
    i0, w0, c0 = oracle.route_topk(logits, 6, score, True, 2.5)
    i1, w1, c1 = oracle.route_topk_grouped(logits, 6, 1, 1, None, score, True, 2.5)
    assert np.array_equal(i0, i1) and np.array_equal(c0, c1)
    np.testing.assert_allclose(w1, w0, rtol=3e-7)       # grouped variant rounds the scores to fp32 first
    # all groups kept: the limit excludes nothing
    i2, w2, _ = oracle.route_topk_grouped(logits, 6, 6, 6, None, score, True, 2.5)
    assert np.array_equal(i0, i2)
    np.testing.assert_array_equal(w1, w2)


@pytest.mark.parametrize("score,E,ng,tg,k", [(1, 256, 8, 4, 8), (0, 64, 4, 2, 6), (1, 32, 8, 3, 3), (1, 16, 4, 1, 2)])
def test_grouped_router_vs_sort_based_statement(oracle, score, E, ng, tg, k):
    """The same selection stated with library sorts on the same fp32 decision values (independent of the oracle's
    loops): group score = sum of the k/tg largest c per group, keep the tg best groups, take the k largest c there."""
    g = _rng(E + k)
    T = 500
    logits = (g.standard_normal((T, E)) * 1.5).astype(np.float32)
    bias = (g.standard_normal(E) * 0.1).astype(np.float32)
    idx, w, counts = oracle.route_topk_grouped(logits, k, ng, tg, bias, score, True, 2.5)
    l64 = logits.astype(np.float64)
    if score == 0:
        ex = np.exp(l64 - l64.max(1, keepdims=True))
        s = (ex / ex.sum(1, keepdims=True)).astype(np.float32)
    else:
        s = (1.0 / (1.0 + np.exp(-l64))).astype(np.float32)
    c = s + bias[None, :]                                              # fp32 + fp32
    gs, m = E // ng, k // tg
    cg = c.reshape(T, ng, gs)
    top = -np.sort(-cg, axis=2)[:, :, :m]                              # descending
    gscore = top[:, :, 0].copy()
    for j in range(1, m):
        gscore = gscore + top[:, :, j]                                 # fp32, largest first
    keep = np.argsort(-gscore, axis=1, kind="stable")[:, :tg]
    mask = np.zeros((T, ng), bool)
    np.put_along_axis(mask, keep, True, 1)
    cm = np.where(np.repeat(mask, gs, axis=1), c, -np.inf)
    order = np.argsort(-cm, axis=1, kind="stable")[:, :k]
    assert np.array_equal(order, idx)
    assert np.all(np.take_along_axis(np.repeat(mask, gs, axis=1), idx.astype(np.int64), 1))
    assert max(len(set(r)) for r in (idx // gs).tolist()) <= tg          # at most tg groups per token
    ws = np.take_along_axis(s.astype(np.float64), order, 1)
    np.testing.assert_allclose(w, 2.5 * ws / ws.sum(1, keepdims=True), rtol=1e-12)
    np.testing.assert_allclose(w.sum(1), 2.5, rtol=1e-13)
    assert np.array_equal(counts, np.bincount(order.ravel(), minlength=E)) and counts.sum() == T * k
    # the bias steers the load: a large bias on one expert puts it into every token's selection, at its unbiased weight
    big = bias.copy()
    big[5] += 10.0
    idx_b, w_b, cnt_b = oracle.route_topk_grouped(logits, k, ng, tg, big, score, False, 1.0)
    assert cnt_b[5] == T and np.all(idx_b[:, 0] == 5)
    np.testing.assert_allclose(w_b[:, 0], s[:, 5].astype(np.float64), rtol=1e-12)
    # f32 instantiation: same decisions
    idx32, w32, _ = oracle.route_topk_grouped(logits, k, ng, tg, bias, score, True, 2.5, prec="f32")
    assert np.array_equal(idx32, idx)
    np.testing.assert_allclose(w32, w, rtol=1e-6)


# ---------------------------------------------------------------------------
# Load-balancing auxiliary loss (Sec. 4.3.4 items 2-3)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("score", [0, 1])
def test_aux_loss_closed_forms_and_gradient(oracle, score):
    g = _rng(60 + score)
    T, E, k, coeff = 96, 12, 3, 0.01
    logits = g.standard_normal((T, E)) * 2.0
    counts = g.multinomial(T * k, np.ones(E) / E)
    # 1. equal logits: every probability is 1/E, so sum_e f_e P_e = 1/E whatever the load: loss = coeff
    loss, grad = oracle.aux_loss(np.full((T, E), 0.7), counts, k, score, coeff)
    np.testing.assert_allclose(loss, coeff, rtol=1e-13)
    np.testing.assert_allclose(grad.sum(axis=1), 0.0, atol=1e-18)
    # 2. perfectly balanced load: f_e = 1/E and the probabilities of a token sum to one: loss = coeff for any logits,
    #    and the gradient vanishes (the loss does not depend on the logits at all)
    loss, grad = oracle.aux_loss(logits, np.full(E, T * k // E), k, score, coeff)
    np.testing.assert_allclose(loss, coeff, rtol=1e-13)
    np.testing.assert_allclose(grad, 0.0, atol=1e-17)
    # 3. collapse: every pair on expert 0 and (softmax) all probability there: f_0 = P_0 = 1, loss = coeff E
    if score == 0:
        hot = np.zeros((T, E))
        hot[:, 0] = 60.0
        c0 = np.zeros(E, np.int64)
        c0[0] = T * k
        np.testing.assert_allclose(oracle.aux_loss(hot, c0, k, score, coeff)[0], coeff * E, rtol=1e-12)
    # 4. the definition written as loops
    loss, grad = oracle.aux_loss(logits, counts, k, score, coeff)
    acc = 0.0
    for e in range(E):
        Pe = 0.0
        for t in range(T):
            v = np.exp(logits[t]) if score == 0 else 1.0 / (1.0 + np.exp(-logits[t]))
            Pe += v[e] / v.sum()
        acc += (counts[e] / (T * k)) * (Pe / T)
    np.testing.assert_allclose(loss, coeff * E * acc, rtol=1e-12)
    # 5. gradient by central differences (counts held fixed)
    for _ in range(12):
        t, e = int(g.integers(T)), int(g.integers(E))
        d = 1e-5
        lp, lm = logits.copy(), logits.copy()
        lp[t, e] += d
        lm[t, e] -= d
        fd = (oracle.aux_loss(lp, counts, k, score, coeff)[0] - oracle.aux_loss(lm, counts, k, score, coeff)[0]) / (2 * d)
        np.testing.assert_allclose(grad[t, e], fd, rtol=2e-6, atol=1e-12)
    # the most loaded expert has the largest weight w_e, above the p-weighted mean of the weights: descending the
    # loss lowers its logit for every token
    assert (grad[:, int(np.argmax(counts))] > 0).all()


# ---------------------------------------------------------------------------
# Row-ID map and permute (Sec. 4.3.3 "Preprocessing", "Permute"; Sec. 5.4.1 padding)
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("align", [1, 16, 128])
def test_maps_equal_stable_sort(oracle, align):
    g = _rng(5)
    T, k, E = 333, 3, 7
    idx = g.integers(-1, E + 1, size=(T, k)).astype(np.int32)   # includes -1 and E: "not on this GPU"
    idx[:, 0] = np.where(idx[:, 0] == 5, 4, idx[:, 0])           # make expert 5 rarer
    idx[idx == 3] = 2                                            # expert 3 gets no rows at all
    m = oracle.permute_maps(idx, E, align)
    flat = idx.ravel()
    valid = (flat >= 0) & (flat < E)
    counts = np.bincount(flat[valid], minlength=E)
    assert np.array_equal(m.counts, counts) and counts[3] == 0
    pad = (counts + align - 1) // align * align
    assert np.array_equal(m.offsets, np.concatenate([[0], np.cumsum(pad)]))
    assert m.Rtot == pad.sum()
    # textbook: stable sort of the flattened ids by expert
    order = np.argsort(np.where(valid, flat, E + 1), kind="stable")[: valid.sum()]
    pos = 0
    for e in range(E):
        seg = m.src_of[m.offsets[e]: m.offsets[e] + counts[e]]
        assert np.array_equal(seg, order[pos: pos + counts[e]])
        assert np.all(flat[seg] == e)
        assert np.all(np.diff(seg) > 0)
        assert np.all(m.src_of[m.offsets[e] + counts[e]: m.offsets[e + 1]] == -1)   # pad rows
        pos += counts[e]
    assert np.all(m.src_of[m.Rtot:] == -1)
    ro = m.row_of.ravel()
    assert np.all(ro[~valid] == -1)
    assert np.array_equal(m.src_of[ro[valid]], np.nonzero(valid)[0])
    # rows: copies of the source token, pad rows zero
    X = g.standard_normal((T, 10))
    Xp = oracle.permute_rows(X, m.src_of[: m.Rtot], k)
    live = m.src_of[: m.Rtot] >= 0
    assert np.array_equal(Xp[live], X[m.src_of[: m.Rtot][live] // k])
    assert np.all(Xp[~live] == 0)
    with pytest.raises(ValueError):
        oracle.permute_maps(idx, E, align, Rcap=m.Rtot - 1)


def test_permute_combine_round_trip(oracle):
    """Unpermute is the inverse of permute and sums the k copies (Sec. 4.3.3): w = 1/k returns X exactly."""
    g = _rng(6)
    T, k, E, h = 100, 4, 9, 24
    idx = np.stack([g.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    X = g.standard_normal((T, h))
    m = oracle.permute_maps(idx, E, 8)
    Xp = oracle.permute_rows(X, m.src_of[: m.Rtot], k)
    Y = oracle.combine(Xp, m.row_of, np.full((T, k), 0.25), None)
    assert np.array_equal(Y, X)
    res = g.standard_normal((T, h))
    Y1 = oracle.combine(Xp, m.row_of, None, res)            # w == 1, residual (shared expert slot) added
    np.testing.assert_allclose(Y1, 4 * X + res, rtol=1e-14, atol=1e-14)


# ---------------------------------------------------------------------------
# Expert GEMMs (Sec. 2.1.4, 4.3.2) against numpy on special cases
# ---------------------------------------------------------------------------
def _offsets(counts):
    return np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)


@pytest.mark.parametrize("prec,tol", [("f64", 1e-13), ("f32", 2e-5)])
def test_grouped_gemms_vs_numpy(oracle, prec, tol):
    g = _rng(7)
    counts = np.array([5, 0, 17, 1, 9])
    E, N, K = len(counts), 11, 13
    R = counts.sum()
    off = _offsets(counts)
    A = g.standard_normal((R, K))
    B = g.standard_normal((E, N, K))
    dC = g.standard_normal((R, N))
    Cm = oracle.grouped_gemm_nt(A, B, off, prec=prec)
    dA = oracle.grouped_gemm_nn(dC, B, off, prec=prec)
    dB = oracle.grouped_gemm_tn(dC, A, off, prec=prec)
    for e in range(E):
        s = slice(off[e], off[e + 1])
        np.testing.assert_allclose(Cm[s], A[s] @ B[e].T, rtol=tol, atol=tol)
        np.testing.assert_allclose(dA[s], dC[s] @ B[e], rtol=tol, atol=tol)
        np.testing.assert_allclose(dB[e], dC[s].T @ A[s], rtol=tol, atol=tol)
    assert np.all(dB[1] == 0)                                   # zero-token expert: exact zero gradient
    # row subset and output window agree with the full result
    rows = np.array([0, 4, 5, 21, 22, 31], np.int32)
    np.testing.assert_array_equal(oracle.grouped_gemm_nt(A, B, off, rows=rows, prec=prec), Cm[rows])
    np.testing.assert_array_equal(oracle.grouped_gemm_nn(dC, B, off, rows=rows, prec=prec), dA[rows])
    np.testing.assert_array_equal(oracle.grouped_gemm_tn(dC, A, off, window=(3, 4, 2, 7), prec=prec),
                                  dB[:, 3:7, 2:9])
    # E == 1 is an ordinary dense GEMM
    one = np.array([0, R], np.int32)
    np.testing.assert_allclose(oracle.grouped_gemm_nt(A, B[:1], one, prec=prec), A @ B[0].T, rtol=tol, atol=tol)


def test_swiglu_closed_form(oracle):
    # silu(0) = 0; silu(g) -> g for large g; silu(-g) = -g * sigmoid(-g); odd/even parts
    Z = np.array([[0.0, 40.0, -40.0, np.log(3.0), 7.0, 2.0, 3.0, -5.0]])
    A = oracle.swiglu(Z)
    np.testing.assert_allclose(A[0], [0.0, 80.0, -40.0 * np.exp(-40.0) / (1 + np.exp(-40.0)) * 3.0,
                                      np.log(3.0) * 0.75 * -5.0], rtol=1e-14, atol=0)
    g = _rng(8)
    Z = g.standard_normal((6, 10))
    gate, up = Z[:, :5], Z[:, 5:]
    np.testing.assert_allclose(oracle.swiglu(Z), gate / (1 + np.exp(-gate)) * up, rtol=1e-14)
    # silu(g) - silu(-g) = g
    Zm = Z.copy()
    Zm[:, :5] *= -1
    np.testing.assert_allclose(oracle.swiglu(Z) - oracle.swiglu(Zm), gate * up, rtol=1e-12, atol=1e-15)


# ---------------------------------------------------------------------------
# The whole layer against the definition written another way (Sec. 1.1; Sec. 4.1.2 eq. (1), (2))
# ---------------------------------------------------------------------------
def _dense_definition(X, idx, prob, W1, W2):
    """MoE(x) = sum_{i in TopK} p_i E_i(x): every expert applied to every token, then masked."""
    T, k = idx.shape
    E, f2, h = W1.shape
    f = f2 // 2
    Y = np.zeros((T, h))
    for e in range(E):
        Zd = X @ W1[e].T
        Ad = Zd[:, :f] / (1 + np.exp(-Zd[:, :f])) * Zd[:, f:]
        Od = Ad @ W2[e].T
        gatew = np.where(idx == e, prob, 0.0).sum(1)
        Y += gatew[:, None] * Od
    return Y


def _tiny_layer(seed, T=40, h=12, f=10, E=5, k=2, shared=True):
    g = _rng(seed)
    X = g.standard_normal((T, h))
    logits = g.standard_normal((T, E)).astype(np.float32)
    W1 = g.standard_normal((E, 2 * f, h)) * 0.4
    W2 = g.standard_normal((E, h, f)) * 0.4
    Ws1 = g.standard_normal((2 * 6, h)) * 0.4 if shared else None
    Ws2 = g.standard_normal((h, 6)) * 0.4 if shared else None
    dY = g.standard_normal((T, h))
    return X, logits, W1, W2, Ws1, Ws2, dY


@pytest.mark.parametrize("align", [1, 16])
def test_layer_equals_dense_definition(oracle, align):
    X, logits, W1, W2, Ws1, Ws2, _ = _tiny_layer(9)
    E = W1.shape[0]
    idx, prob, _ = oracle.route_topk(logits, 2, 1, True)
    fw = oracle.layer_forward(X, idx, prob, W1, W2, E, align)
    np.testing.assert_allclose(fw.Y, _dense_definition(X, idx, prob, W1, W2), rtol=1e-12, atol=1e-13)
    # shared expert: plain dense SwiGLU MLP of every token, added at the combine stage (Sec. 2.1.1 stage 4)
    fws = oracle.layer_forward(X, idx, prob, W1, W2, E, align, Ws1, Ws2)
    Zs = X @ Ws1.T
    fs = Ws1.shape[0] // 2
    S = (Zs[:, :fs] / (1 + np.exp(-Zs[:, :fs])) * Zs[:, fs:]) @ Ws2.T
    np.testing.assert_allclose(fws.Y, fw.Y + S, rtol=1e-12, atol=1e-13)
    # eq. (1) == eq. (2): weights applied before W2 with a plain-sum combine
    m = fw.maps
    p_row = np.zeros(fw.R)
    p_row[m.row_of.ravel()] = prob.ravel()
    O2 = oracle.grouped_gemm_nt(fw.A * p_row[:, None], W2, m.offsets)
    Y2 = oracle.combine(O2, m.row_of, None, None)
    np.testing.assert_allclose(Y2, fw.Y, rtol=1e-12, atol=1e-13)


def test_k1_p1_is_plain_mlp(oracle):
    X, logits, W1, W2, *_ = _tiny_layer(10)
    E, f2, _ = W1.shape
    idx, _, _ = oracle.route_topk(logits, 1, 0, False)
    fw = oracle.layer_forward(X, idx, np.ones_like(idx, dtype=np.float64), W1, W2, E)
    for t in range(X.shape[0]):
        e = idx[t, 0]
        z = W1[e] @ X[t]
        a = z[: f2 // 2] / (1 + np.exp(-z[: f2 // 2])) * z[f2 // 2:]
        np.testing.assert_allclose(fw.Y[t], W2[e] @ a, rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------------------
# Backward by central finite differences in double (routing frozen)
# ---------------------------------------------------------------------------
def test_backward_finite_differences(oracle):
    X, logits, W1, W2, Ws1, Ws2, dY = _tiny_layer(11, T=12, h=6, f=5, E=4, k=2)
    E = W1.shape[0]
    idx, prob, _ = oracle.route_topk(logits, 2, 0, False)
    # make one expert empty to cover the zero-token gradient
    idx[idx == 2] = 0
    idx[:, 1] = np.where(idx[:, 1] == idx[:, 0], (idx[:, 0] + 1) % 2, idx[:, 1])

    def loss(X_, p_, W1_, W2_, Ws1_, Ws2_):
        return float((oracle.layer_forward(X_, idx, p_, W1_, W2_, E, 4, Ws1_, Ws2_).Y * dY).sum())

    fw = oracle.layer_forward(X, idx, prob, W1, W2, E, 4, Ws1, Ws2)
    bw = oracle.layer_backward(fw, X, prob, W1, W2, dY, Ws1, Ws2)
    assert np.all(bw.dW1[2] == 0) and np.all(bw.dW2[2] == 0)
    args = [X, prob, W1, W2, Ws1, Ws2]
    grads = [bw.dX + bw.dX_shared, bw.dprob, bw.dW1, bw.dW2, bw.dWs1, bw.dWs2]
    g = _rng(12)
    eps = 1e-6
    for ai, (a, gr) in enumerate(zip(args, grads)):
        assert gr.shape == a.shape
        for _ in range(25):
            pos = tuple(g.integers(s) for s in a.shape)
            ap, am = a.copy(), a.copy()
            ap[pos] += eps
            am[pos] -= eps
            lp = loss(*[ap if j == ai else args[j] for j in range(6)])
            lm = loss(*[am if j == ai else args[j] for j in range(6)])
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - gr[pos]) <= 1e-6 * max(1.0, abs(fd)), (ai, pos, fd, gr[pos])


@pytest.mark.parametrize("score,norm", [(0, False), (0, True), (1, True), (1, False)])
def test_router_backward_finite_differences(oracle, score, norm):
    """dL/dlogits of the routing weights with the selection frozen, against central differences of the weight
    formula written out here (softmax over all experts / sigmoid, optional normalisation over the selected k),
    which is itself tied to the oracle's forward."""
    g = _rng(31 + 2 * score + norm)
    T, E, k, scale = 9, 11, 3, 1.7
    logits = g.normal(size=(T, E)).astype(np.float32)
    idx, prob, _ = oracle.route_topk(logits, k, score, norm, scale)
    dw = g.normal(size=(T, k))

    def weights(l):
        l = l.astype(np.float64)
        if score == 0:
            e = np.exp(l - l.max(axis=1, keepdims=True))
            sc = e / e.sum(axis=1, keepdims=True)
        else:
            sc = 1 / (1 + np.exp(-l))
        q = np.take_along_axis(sc, idx.astype(np.int64), axis=1)
        if norm:
            q = q / q.sum(axis=1, keepdims=True)
        return scale * q

    np.testing.assert_allclose(weights(logits), prob, rtol=1e-12, atol=1e-15)
    got = oracle.route_topk_bwd(logits, idx, dw, score, norm, scale)
    eps = 1e-5
    L64 = logits.astype(np.float64)
    for t in range(T):
        for e in range(E):
            lp, lm = L64.copy(), L64.copy()
            lp[t, e] += eps
            lm[t, e] -= eps
            fd = ((weights(lp) - weights(lm)) * dw).sum() / (2 * eps)
            assert abs(fd - got[t, e]) <= 1e-8 * max(1.0, abs(fd)) + 1e-9, (t, e, fd, got[t, e])
    if score == 0:   # softmax: a constant shift of the logits changes nothing
        np.testing.assert_allclose(got.sum(axis=1), 0.0, atol=1e-12)
    if norm:         # normalised weights sum to `scale`: a common factor on dw-direction 1 gives zero gradient
        ones = oracle.route_topk_bwd(logits, idx, np.ones((T, k)), score, norm, scale)
        np.testing.assert_allclose(ones, 0.0, atol=1e-12)


def test_eq2_layer_matches_eq1_and_finite_differences(oracle):
    """Memory-efficient permutation (Sec. 4.1.2): eq. (2) is an algebraic rearrangement of eq. (1), so its
    forward output and every gradient must equal eq. (1)'s (themselves pinned above), and its own loss must
    reproduce its dprob by central differences (dprob is the one gradient computed by a different formula)."""
    X, logits, W1, W2, Ws1, Ws2, dY = _tiny_layer(21, T=12, h=6, f=5, E=4, k=2)
    E = W1.shape[0]
    idx, prob, _ = oracle.route_topk(logits, 2, 1, True)
    idx[idx == 3] = 1
    idx[:, 1] = np.where(idx[:, 1] == idx[:, 0], (idx[:, 0] + 1) % 3, idx[:, 1])
    for align in (1, 4):
        f1 = oracle.layer_forward(X, idx, prob, W1, W2, E, align, Ws1, Ws2)
        b1 = oracle.layer_backward(f1, X, prob, W1, W2, dY, Ws1, Ws2)
        f2 = oracle.layer_forward_eq2(X, idx, prob, W1, W2, E, align, Ws1, Ws2)
        b2 = oracle.layer_backward_eq2(f2, X, prob, W1, W2, dY, Ws1, Ws2)
        np.testing.assert_allclose(f2.Y, f1.Y, rtol=1e-12, atol=1e-14)
        for name in ("dX", "dprob", "dW1", "dW2", "dWs1", "dWs2", "dX_shared"):
            np.testing.assert_allclose(getattr(b2, name), getattr(b1, name), rtol=1e-11, atol=1e-14, err_msg=name)
        assert np.all(b2.dW1[3] == 0) and np.all(b2.dW2[3] == 0)
        # padding rows: zero weight, zero gradient rows
        pad = f2.maps.src_of[:f2.R] < 0
        assert np.all(f2.row_prob[pad] == 0) and np.all(b2.dZ[pad] == 0) and np.all(f2.A[pad] == 0)
    g = _rng(22)
    eps = 1e-6
    for _ in range(20):
        pos = tuple(g.integers(s) for s in prob.shape)
        pp, pm = prob.copy(), prob.copy()
        pp[pos] += eps
        pm[pos] -= eps
        lp = float((oracle.layer_forward_eq2(X, idx, pp, W1, W2, E, 4, Ws1, Ws2).Y * dY).sum())
        lm = float((oracle.layer_forward_eq2(X, idx, pm, W1, W2, E, 4, Ws1, Ws2).Y * dY).sum())
        fd = (lp - lm) / (2 * eps)
        assert abs(fd - b2.dprob[pos]) <= 1e-6 * max(1.0, abs(fd)), (pos, fd, b2.dprob[pos])


def test_swiglu_bwd_and_combine_bwd_closed_forms(oracle):
    g = _rng(13)
    # d/dg silu(g) at g = 0 is 1/2; dZ_up = silu(g)
    Z = np.array([[0.0, 2.0, 3.0, 5.0]])
    dZ = oracle.swiglu_bwd(np.array([[1.0, 1.0]]), Z)
    s2 = 1 / (1 + np.exp(-2.0))
    np.testing.assert_allclose(dZ[0], [0.5 * 3.0, 5.0 * s2 * (1 + 2.0 * (1 - s2)), 0.0, 2.0 * s2], rtol=1e-14)
    # combine backward: dO = w * dY gathered, dprob = <dY, O>
    T, k, h, R = 7, 2, 5, 20
    row_of = g.permutation(R)[: T * k].reshape(T, k).astype(np.int32)
    row_of[2, 1] = -1
    O = g.standard_normal((R, h))
    dY = g.standard_normal((T, h))
    p = g.random((T, k))
    dO, dp = oracle.combine_bwd(dY, O, row_of, p, R)
    for t in range(T):
        for s in range(k):
            r = row_of[t, s]
            if r < 0:
                assert dp[t, s] == 0
                continue
            np.testing.assert_allclose(dO[r], p[t, s] * dY[t], rtol=1e-15)
            np.testing.assert_allclose(dp[t, s], dY[t] @ O[r], rtol=1e-13)
    untouched = np.setdiff1d(np.arange(R), row_of.ravel())
    assert np.all(dO[untouched] == 0)


# ---------------------------------------------------------------------------
# Blockwise FP8 (Sec. 5.3.2)
# ---------------------------------------------------------------------------
def test_e4m3_table(oracle):
    """All 256 codes against the OCP E4M3 definition and against torch's float8_e4m3fn."""
    vals = np.array([oracle.e4m3_decode(c) for c in range(256)])
    assert vals[0x7E] == 448.0 and vals[0xFE] == -448.0
    assert np.isnan(vals[0x7F]) and np.isnan(vals[0xFF])
    assert not np.any(np.isinf(vals))
    assert vals[0x01] == 2.0 ** -9 and vals[0x08] == 2.0 ** -6 and vals[0x38] == 1.0
    fin = vals[:0x7F]
    assert np.all(np.diff(fin) > 0)                              # codes are monotone in value
    torch = pytest.importorskip("torch")
    if hasattr(torch, "float8_e4m3fn"):
        tv = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).float().numpy()
        assert np.array_equal(np.nan_to_num(tv, nan=-1.0), np.nan_to_num(vals, nan=-1.0).astype(np.float32))
    # idempotence and rounding
    for c in list(range(0x7F)) + list(range(0x81, 0xFF)):
        assert oracle.e4m3_encode(vals[c]) == c
    assert oracle.e4m3_encode(1e9) == 0x7E and oracle.e4m3_encode(-1e9) == 0xFE      # saturating
    assert oracle.e4m3_encode(float("nan")) == 0x7F
    # ties to even: halfway between 1.0 (0x38) and 1.125 (0x39) -> 0x38; between 1.125 and 1.25 (0x3A) -> 0x3A
    assert oracle.e4m3_encode(1.0625) == 0x38 and oracle.e4m3_encode(1.1875) == 0x3A
    assert oracle.e4m3_encode(2.0 ** -10) == 0x00 and oracle.e4m3_encode(3 * 2.0 ** -10) == 0x02
    g = _rng(14)
    x = (g.standard_normal(4000) * np.exp(g.uniform(-6, 5, 4000))).astype(np.float32)
    x = x[np.abs(x) <= 448]
    codes = np.array([oracle.e4m3_encode(v) for v in x], np.uint8)
    if hasattr(torch, "float8_e4m3fn"):
        tc = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
        assert np.array_equal(tc & 0x7F, codes & 0x7F)
        nz = (codes & 0x7F) != 0
        assert np.array_equal(tc[nz], codes[nz])
    normal = np.abs(x) >= 2.0 ** -6
    rel = np.abs(vals[codes][normal] - x[normal]) / np.abs(x[normal])
    assert rel.max() <= 2.0 ** -4


def test_fp8_block_quantisers(oracle):
    g = _rng(15)
    X = (g.standard_normal((256, 384)) * np.exp(g.uniform(-3, 3, (256, 1)))).astype(np.float32)
    X[5, 128:256] = 0.0                                           # an all-zero tile: scale 1, codes 0
    for mode, fn in (("1x128", oracle.fp8_quant_1x128), ("128x1", oracle.fp8_quant_128x1)):
        q, s = fn(X)
        blocks = X.reshape(256, 3, 128) if mode == "1x128" else X.reshape(2, 128, 384).transpose(0, 2, 1)
        amax = np.abs(blocks).max(-1)
        np.testing.assert_array_equal(s, np.where(amax > 0, amax / np.float32(448), np.float32(1)))
        qb = q.reshape(256, 3, 128) if mode == "1x128" else q.reshape(2, 128, 384).transpose(0, 2, 1)
        assert np.all(((qb & 0x7F).max(-1) == 0x7E) | (amax == 0))   # the block's amax maps to +-448
        D = oracle.fp8_dequant(q, s, mode)
        sfull = np.repeat(s, 128, axis=1) if mode == "1x128" else np.repeat(s, 128, axis=0)
        assert np.all(np.abs(D - X) <= 2.0 ** -4 * np.abs(X) + sfull * 2.0 ** -10)
    q, s = oracle.fp8_quant_1x128(X)
    assert s[5, 1] == 1.0 and np.all(q[5, 128:256] == 0)
    W = g.standard_normal((2, 256, 128)).astype(np.float32)
    qw, sw = oracle.fp8_quant_128x128(W)
    amax = np.abs(W.reshape(2, 2, 128, 1, 128)).max((2, 4))
    np.testing.assert_array_equal(sw, amax / np.float32(448))
    Dw = oracle.fp8_dequant(qw, sw, "128x128")
    assert np.abs(Dw - W).max() <= 2.0 ** -4 * np.abs(W).max()
    # a transposed 1x128 quantisation equals the 128x1 quantisation
    qt, st = oracle.fp8_quant_1x128(np.ascontiguousarray(X.T))
    qc, sc = oracle.fp8_quant_128x1(X)
    assert np.array_equal(qt.T, qc) and np.array_equal(st.T, sc)


def test_fp8_blockwise_wgrad_emulation(oracle):
    """The quantise-dequantise emulation of the blockwise weight gradient (Sec. 5.3.2 with the 1x128 tiles running
    down the token dimension, Sec. 5.4.1): both operands quantised 128x1 inside an expert's 128-aligned row range,
    dequantised, then dW_e = dC_e^T A_e.  Pinned three ways: exact when the quantisation is exact; equal to the
    block-scaled form sum_b (s_dC[b, n] s_A[b, k]) (codes_dC_b^T codes_A_b) evaluated with numpy from the decoded
    codes (a wrong scale index, a transposed operand or a block that straddles experts breaks the equality); and
    within the format's error of the full-precision gradient."""
    g = _rng(21)
    counts = np.array([256, 0, 128, 384])
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R, N, K = int(off[-1]), 12, 20
    vals = np.array([oracle.e4m3_decode(c) for c in range(256)])
    finite = vals[np.isfinite(vals)]
    # (a) exactly representable operands: codes times a power-of-two scale per (128-row block, column); every block
    #     holds +-448, so amax / 448 is that power of two and the quantisation is the identity
    def exact(cols, seed):
        gg = _rng(seed)
        v = gg.choice(finite, size=(R, cols))
        v[::128] = 448.0 * gg.choice([-1.0, 1.0], size=(R // 128, cols))
        sc = 2.0 ** gg.integers(-12, 5, size=(R // 128, cols))
        return (v * np.repeat(sc, 128, axis=0)).astype(np.float32), sc
    dC, sdc = exact(N, 1)
    A, sa = exact(K, 2)
    qd, sd = oracle.fp8_quant_128x1(dC)
    qa, sA = oracle.fp8_quant_128x1(A)
    np.testing.assert_array_equal(sd, sdc.astype(np.float32))
    np.testing.assert_array_equal(sA, sa.astype(np.float32))
    Dd, Ad = oracle.fp8_dequant(qd, sd, "128x1"), oracle.fp8_dequant(qa, sA, "128x1")
    np.testing.assert_array_equal(Dd, dC.astype(np.float64))
    emu = oracle.grouped_gemm_tn(Dd, Ad, off)
    full = oracle.grouped_gemm_tn(dC, A, off)
    np.testing.assert_allclose(emu, full, rtol=1e-13, atol=0)
    assert not emu[1].any()                                            # the empty expert
    # (b) Gaussian operands with a different magnitude per row block: the block-scaled form, written with numpy
    mag = np.exp(g.uniform(-4, 4, (R // 128, 1)))
    dC = (g.standard_normal((R, N)) * np.repeat(mag, 128, axis=0)).astype(np.float32)
    A = (g.standard_normal((R, K)) * np.repeat(mag[::-1], 128, axis=0)).astype(np.float32)
    dC[128:256] = 0.0                                                   # a block of zero rows (padding): scale 1, codes 0
    qd, sd = oracle.fp8_quant_128x1(dC)
    qa, sA = oracle.fp8_quant_128x1(A)
    assert np.all(sd[1] == 1.0) and not qd[128:256].any()
    emu = oracle.grouped_gemm_tn(oracle.fp8_dequant(qd, sd, "128x1"), oracle.fp8_dequant(qa, sA, "128x1"), off)
    ref = np.zeros_like(emu)
    for e in range(len(counts)):
        for b in range(off[e] // 128, off[e + 1] // 128):
            cd, ca = vals[qd[128 * b:128 * b + 128]], vals[qa[128 * b:128 * b + 128]]
            ref[e] += np.outer(sd[b].astype(np.float64), sA[b].astype(np.float64)) * (cd.T @ ca)
    np.testing.assert_allclose(emu, ref, rtol=1e-12, atol=1e-300)
    # (c) against full precision: two quantised operands, each within 2^-4 per element
    full = oracle.grouped_gemm_tn(dC, A, off)
    err = np.linalg.norm(emu - full) / np.linalg.norm(full)
    assert 5e-3 < err < 6e-2, err


def test_mxfp8_quantisers(oracle):
    """MXFP8 (Sec. 5.3.3): E8M0 scale = smallest power of two that brings the block maximum inside +-448;
    1x32 blocks along the row (and along N for the column-wise weight copy)."""
    # scale exponent against the definition evaluated in exact rational arithmetic
    from fractions import Fraction
    g = _rng(41)
    for a in list(g.uniform(1e-6, 1e4, size=200)) + [448.0, 224.0, 448.0 * 2 ** -20, 449.0, 3.5, 1.75 * 2 ** -3, 1e-30, 3e38]:
        a32 = np.float32(a)
        e = oracle.e8m0_from_amax(float(a32)) - 127
        ratio = Fraction(float(a32)) / 448
        if -127 < e < 127:
            assert ratio <= Fraction(2) ** e and ratio > Fraction(2) ** (e - 1), (a, e)
    assert oracle.e8m0_from_amax(0.0) == 127
    # row-wise quantiser: per block amax/scale in (224, 448], no saturation, dequantisation error <= 2^-4 relative
    X = (g.normal(size=(7, 96)) * np.exp(g.normal(size=(7, 96)) * 3)).astype(np.float32)
    X[2, 32:64] = 0.0
    X[3, 5] = 448.0 * 2 ** 10                                   # block maximum exactly at the top of the range
    q, e8 = oracle.mx_quant_1x32(X)
    assert q.shape == X.shape and e8.shape == (7, 3)
    assert e8[2, 1] == 127 and not q[2, 32:64].any()
    dq = oracle.mx_dequant(q, e8, "1x32")
    for r in range(7):
        for b in range(3):
            blk = X[r, 32 * b:32 * b + 32].astype(np.float64)
            am = np.abs(blk).max()
            if am == 0:
                continue
            sc = 2.0 ** (int(e8[r, b]) - 127)
            assert 224 < am / sc <= 448, (r, b, am, sc)
            err = np.abs(dq[r, 32 * b:32 * b + 32] - blk)
            # normal E4M3 values: half an ulp = 2^-4 relative; below 2^-6 * scale: half the subnormal step
            assert np.all(err <= np.maximum(np.abs(blk) * 2.0 ** -4, sc * 2.0 ** -10) + 1e-300)
    assert q[3, 5] == 0x7E and e8[3, 0] == 127 + 10             # 448 * 2^10 -> largest code, scale 2^10
    # idempotence at the value level: representable values survive a second pass unchanged (codes may differ:
    # a block maximum that rounded down to exactly 224 * scale moves to the next smaller scale with doubled codes)
    q2, e2 = oracle.mx_quant_1x32(dq.astype(np.float32))
    big = np.abs(dq) >= np.repeat(2.0 ** (e8.astype(np.float64) - 127 - 5), 32, axis=1)   # not in the subnormal tail
    np.testing.assert_array_equal(oracle.mx_dequant(q2, e2, "1x32")[big], dq[big])
    # powers of two are exact
    P = (2.0 ** g.integers(-20, 20, size=(4, 64))).astype(np.float32)
    # (a block spanning more than 2^17 in magnitude underflows its small members: keep each block within range)
    P = (P.reshape(4, 2, 32) / P.reshape(4, 2, 32).max(axis=2, keepdims=True) * 2.0 ** g.integers(-5, 5, size=(4, 2, 1))).astype(np.float32)
    P = np.maximum(P, P.max(axis=2, keepdims=True) * 2.0 ** -12).reshape(4, 64)
    qp, ep = oracle.mx_quant_1x32(P)
    np.testing.assert_array_equal(oracle.mx_dequant(qp, ep, "1x32"), P.astype(np.float64))
    # column-wise copy of a weight stack == row-wise quantisation of the transposed matrices
    W = g.normal(size=(2, 64, 8)).astype(np.float32)
    qc, ec = oracle.mx_quant_32x1(W)
    assert qc.shape == W.shape and ec.shape == (2, 8, 2)
    for gi in range(2):
        qt, et = oracle.mx_quant_1x32(np.ascontiguousarray(W[gi].T))
        assert np.array_equal(qc[gi], qt.T) and np.array_equal(ec[gi], et)
    np.testing.assert_array_equal(oracle.mx_dequant(qc, ec, "32x1")[1],
                                  oracle.mx_dequant(*oracle.mx_quant_1x32(np.ascontiguousarray(W[1].T)), "1x32").T)


def test_assert_close_catches_a_wrong_row_that_a_pooled_norm_hides():
    """The helper the GPU parity tests use: a single wrong row (or a row that lost half its contraction) in a tensor of
    thousands passes a pooled 2e-2 Frobenius bound and must fail the per-row bound; the mistake is planted in a copy
    of a reference, on the CPU."""
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
    from gpu_util import assert_close, rel_fro, BF16_TOL
    g = np.random.default_rng(7)
    A = g.standard_normal((8192, 256))
    B = g.standard_normal((256, 256))
    ref = A @ B.T
    good = ref * (1.0 + 2e-3 * g.standard_normal(ref.shape))          # bf16-like rounding noise
    assert_close(good, ref, "good")
    half = good.copy()
    half[1234] = A[1234, :128] @ B[:, :128].T                            # one row with half its contraction
    assert rel_fro(half, ref) <= BF16_TOL                                # the pooled norm does not see it
    with pytest.raises(AssertionError, match="rows above the per-row bound"):
        assert_close(half, ref, "half a row", reg=None)
    wrong = good.copy()
    wrong[7] = good[8]                                                   # one row swapped for its neighbour
    assert rel_fro(wrong, ref) <= BF16_TOL
    with pytest.raises(AssertionError, match="rows above the per-row bound"):
        assert_close(wrong, ref, "wrong row", reg=None)
    drift = ref * (1.0 + 8e-3 * g.standard_normal(ref.shape))           # everywhere worse, still inside the contract
    with pytest.raises(AssertionError, match="regression bound"):
        assert_close(drift, ref, "drift")
    z = np.zeros((4, 8))
    assert_close(z, z, "zeros")                                          # empty experts: exact zeros pass


def test_fp8_blockwise_scales_far_apart(oracle):
    """Blocks 24 decades apart along one contraction: the oracle's quantise-dequantise has no dynamic-range limit
    of its own (each block is scaled by its own fp32 amax / 448): every element comes back within the format's
    half-ulp (2^-4 relative for normal codes), and the emulated product equals the block-scaled form
    sum_b s_A[r, b] s_W[b] (codes_A_b . codes_W_b) evaluated in exact rational arithmetic on a small case."""
    from fractions import Fraction
    g = _rng(77)
    R, K = 6, 512
    kmag = np.where(np.arange(K // 128) % 2 == 0, 1e12, 1e-12).repeat(128)
    A = (g.standard_normal((R, K)) * kmag).astype(np.float32)
    q, s = oracle.fp8_quant_1x128(A)
    assert s.shape == (R, K // 128) and np.all(s[:, 0] > 1e9) and np.all(s[:, 1] < 1e-13)
    Ad = oracle.fp8_dequant(q, s, "1x128")
    big = np.abs(A) >= (np.repeat(s, 128, axis=1) * 2.0 ** -6)           # normal codes only
    assert np.all(np.abs(Ad - A)[big] <= 2.0 ** -4 * np.abs(A)[big] * (1 + 1e-6))
    w = (g.standard_normal(K) * kmag).astype(np.float32)
    qw, sw = oracle.fp8_quant_1x128(w[None])
    wd = oracle.fp8_dequant(qw, sw, "1x128")[0]
    emu = Ad @ wd
    for r in range(R):
        tot = Fraction(0)
        for b in range(K // 128):
            blk = sum(Fraction(float(oracle.e4m3_decode(int(q[r, b * 128 + i])))) * Fraction(float(oracle.e4m3_decode(int(qw[0, b * 128 + i]))))
                      for i in range(128))
            tot += Fraction(float(s[r, b])) * Fraction(float(sw[0, b])) * blk
        assert abs(float(tot) - emu[r]) <= 1e-12 * abs(float(tot))
