"""numpy/ctypes front end of the C oracle (test infrastructure only).

`build()` compiles the two C files with gcc into `oracle/libmoe_oracle.so`
(the REAL-typed file twice: f64 = parity authority, f32 = the plain fp32 CPU
implementation whose time the benchmark reports).  Every wrapper takes and
returns host numpy arrays; `prec` selects the instantiation.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from types import SimpleNamespace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libmoe_oracle.so")
_lib = None

SOFTMAX, SIGMOID = 0, 1


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O3 -march=native -fopenmp, no fast-math)."""
    srcs = [os.path.join(_HERE, "moe_oracle.c"), os.path.join(_HERE, "fp8_oracle.c")]
    if not force and os.path.exists(_SO) and all(os.path.getmtime(_SO) >= os.path.getmtime(s) for s in srcs):
        return _SO
    flags = ["-O3", "-march=native", "-fopenmp", "-fPIC", "-std=c11", "-Wall"]
    objs = []
    for sfx, real, extra in (("f64", "double", ["-DORC_INTEGER_PARTS"]), ("f32", "float", [])):
        o = os.path.join(_HERE, f"moe_oracle_{sfx}.o")
        subprocess.check_call(["gcc", *flags, f"-DREAL={real}", f"-DSFX={sfx}", *extra, "-c", srcs[0], "-o", o])
        objs.append(o)
    o8 = os.path.join(_HERE, "fp8_oracle.o")
    subprocess.check_call(["gcc", *flags, "-c", srcs[1], "-o", o8])
    objs.append(o8)
    subprocess.check_call(["gcc", "-shared", "-fopenmp", *objs, "-o", _SO, "-lm"])
    for o in objs:
        os.remove(o)
    return _SO


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_SO)
        _lib.orc_permute_maps.restype = C.c_int64
        _lib.orc_e4m3_decode.restype = C.c_float
        _lib.orc_e4m3_decode.argtypes = [C.c_uint8]
        _lib.orc_e4m3_encode.restype = C.c_uint8
        _lib.orc_e4m3_encode.argtypes = [C.c_float]
        _lib.orc_e8m0_from_amax.restype = C.c_uint8
        _lib.orc_e8m0_from_amax.argtypes = [C.c_float]
    return _lib


def num_threads() -> int:
    """Threads the OpenMP loops use (OMP_NUM_THREADS or the cores the process may run on)."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        return int(v.split(",")[0])
    return len(os.sched_getaffinity(0))


def _dt(prec):
    return np.float64 if prec == "f64" else np.float32


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype):
    return None if a is None else np.ascontiguousarray(a, dtype=dtype)


def _fn(name, prec):
    return getattr(lib(), f"{name}_{prec}")


# ----------------------------------------------------------------------------
# steps
# ----------------------------------------------------------------------------
def route_topk(logits, k, score=SOFTMAX, norm_topk=False, scale=1.0, prec="f64"):
    logits = _arr(logits, np.float32)
    T, E = logits.shape
    idx = np.empty((T, k), np.int32)
    prob = np.empty((T, k), _dt(prec))
    counts = np.empty(E, np.int32)
    rc = _fn("orc_route_topk", prec)(_p(logits), T, E, k, int(score), int(bool(norm_topk)), C.c_double(scale),
                                     _p(idx), _p(prob), _p(counts))
    if rc != 0:
        raise ValueError("orc_route_topk: bad arguments")
    return idx, prob, counts


def route_topk_grouped(logits, k, n_group=1, topk_group=1, bias=None, score=SIGMOID, norm_topk=False, scale=1.0,
                       prec="f64"):
    """Group-limited top-k with an optional load-balancing expert bias (Sec. 4.3.4 item 1; Sec. 7)."""
    logits = _arr(logits, np.float32)
    T, E = logits.shape
    b = None if bias is None else _arr(bias, np.float32)
    idx = np.empty((T, k), np.int32)
    prob = np.empty((T, k), _dt(prec))
    counts = np.empty(E, np.int32)
    rc = _fn("orc_route_topk_grouped", prec)(_p(logits), None if b is None else _p(b), T, E, k, int(n_group),
                                             int(topk_group), int(score), int(bool(norm_topk)), C.c_double(scale),
                                             _p(idx), _p(prob), _p(counts))
    if rc != 0:
        raise ValueError("orc_route_topk_grouped: bad arguments")
    return idx, prob, counts


def aux_loss(logits, counts, k, score=SOFTMAX, coeff=1.0):
    """Load-balancing auxiliary loss and its gradient w.r.t. the logits (Sec. 4.3.4 items 2-3).

    The paper fuses the computation and cites the Switch-Transformer loss without restating it; that published
    form is taken: loss = coeff * E * sum_e f_e * P_e with f_e = counts[e] / (T k) the fraction of routed
    (token, slot) pairs that went to expert e and P_e = mean over tokens of p[t, e], where p is the score function
    over all E experts as Sec. 2.1.2 item 2 defines it (softmax, or sigmoid divided by its sum over the E experts).
    The counts are constants of the differentiation.  fp64 throughout.  Returns (loss, dloss/dlogits [T,E])."""
    l = np.asarray(logits, np.float64)
    c = np.asarray(counts, np.float64)
    T, E = l.shape
    if score == SOFTMAX:
        ex = np.exp(l - l.max(axis=1, keepdims=True))
        p = ex / ex.sum(axis=1, keepdims=True)
    else:
        sg = 1.0 / (1.0 + np.exp(-l))
        p = sg / sg.sum(axis=1, keepdims=True)
    f = c / (T * k)
    P = p.mean(axis=0)
    loss = coeff * E * float((f * P).sum())
    # d loss / d p[t,e] = coeff E f_e / T =: w_e, and p depends on the logits of its own token only
    w = coeff * E * f / T
    wp = (p * w[None, :]).sum(axis=1, keepdims=True)
    if score == SOFTMAX:
        grad = p * (w[None, :] - wp)                       # dp_e/dl_j = p_e ([e = j] - p_j)
    else:
        grad = (1.0 - sg) * p * (w[None, :] - wp)          # dp_e/dl_j = sg_j (1 - sg_j) ([e = j] - p_e) / S
    return loss, grad


def permute_maps(idx, E, align=1, Rcap=None):
    idx = _arr(idx, np.int32)
    T, k = idx.shape
    if Rcap is None:
        Rcap = T * k + E * (align - 1)
    row_of = np.empty((T, k), np.int32)
    src_of = np.empty(Rcap, np.int32)
    offsets = np.empty(E + 1, np.int32)
    counts = np.empty(E, np.int32)
    rtot = lib().orc_permute_maps(_p(idx), T, k, E, align, C.c_int64(Rcap), _p(row_of), _p(src_of), _p(offsets),
                                  _p(counts))
    if rtot < 0:
        raise ValueError("orc_permute_maps: Rcap too small or bad arguments")
    return SimpleNamespace(row_of=row_of, src_of=src_of, offsets=offsets, counts=counts, Rtot=int(rtot), k=k)


def permute_rows(X, src_of, k, prec="f64"):
    X = _arr(X, _dt(prec))
    src_of = _arr(src_of, np.int32)
    R, h = len(src_of), X.shape[1]
    Xp = np.empty((R, h), _dt(prec))
    _fn("orc_permute_rows", prec)(_p(X), _p(src_of), C.c_int64(R), k, h, _p(Xp))
    return Xp


def grouped_gemm_nt(A, B, offsets, rows=None, prec="f64"):
    """C[r,n] = sum_k A[r,k] B[e(r),n,k]; rows: optional list of row indices (result is [len(rows), N])."""
    A, B = _arr(A, _dt(prec)), _arr(B, _dt(prec))
    offsets = _arr(offsets, np.int32)
    E, N, K = B.shape
    assert A.shape[1] == K and len(offsets) == E + 1
    rows = _arr(rows, np.int32)
    n_out = len(rows) if rows is not None else A.shape[0]
    Cm = np.zeros((n_out, N), _dt(prec))
    _fn("orc_grouped_gemm_nt", prec)(_p(A), _p(B), _p(offsets), E, N, K, _p(rows),
                                     C.c_int64(0 if rows is None else len(rows)), _p(Cm))
    return Cm


def grouped_gemm_nn(dC, B, offsets, rows=None, prec="f64"):
    """dA[r,k] = sum_n dC[r,n] B[e(r),n,k]."""
    dC, B = _arr(dC, _dt(prec)), _arr(B, _dt(prec))
    offsets = _arr(offsets, np.int32)
    E, N, K = B.shape
    assert dC.shape[1] == N and len(offsets) == E + 1
    rows = _arr(rows, np.int32)
    n_out = len(rows) if rows is not None else dC.shape[0]
    dA = np.zeros((n_out, K), _dt(prec))
    _fn("orc_grouped_gemm_nn", prec)(_p(dC), _p(B), _p(offsets), E, N, K, _p(rows),
                                     C.c_int64(0 if rows is None else len(rows)), _p(dA))
    return dA


def grouped_gemm_tn(dC, A, offsets, window=None, prec="f64"):
    """dB[e,n,k] = sum_{r in e} dC[r,n] A[r,k]; window=(n0,nn,k0,kn) restricts the output block."""
    dC, A = _arr(dC, _dt(prec)), _arr(A, _dt(prec))
    offsets = _arr(offsets, np.int32)
    E, N, K = len(offsets) - 1, dC.shape[1], A.shape[1]
    n0, nn, k0, kn = window if window is not None else (0, N, 0, K)
    dB = np.zeros((E, nn, kn), _dt(prec))
    _fn("orc_grouped_gemm_tn", prec)(_p(dC), _p(A), _p(offsets), E, N, K, n0, nn, k0, kn, _p(dB))
    return dB


def swiglu(Z, prec="f64"):
    Z = _arr(Z, _dt(prec))
    R, f2 = Z.shape
    out = np.empty((R, f2 // 2), _dt(prec))
    _fn("orc_swiglu", prec)(_p(Z), C.c_int64(R), f2 // 2, _p(out))
    return out


def swiglu_bwd(dAct, Z, prec="f64"):
    dAct, Z = _arr(dAct, _dt(prec)), _arr(Z, _dt(prec))
    R, f2 = Z.shape
    dZ = np.empty((R, f2), _dt(prec))
    _fn("orc_swiglu_bwd", prec)(_p(dAct), _p(Z), C.c_int64(R), f2 // 2, _p(dZ))
    return dZ


def combine(O, row_of, prob=None, residual=None, prec="f64"):
    O = _arr(O, _dt(prec))
    row_of = _arr(row_of, np.int32)
    prob, residual = _arr(prob, _dt(prec)), _arr(residual, _dt(prec))
    T, k = row_of.shape
    h = O.shape[1]
    Y = np.empty((T, h), _dt(prec))
    _fn("orc_combine", prec)(_p(O), _p(row_of), _p(prob), _p(residual), T, k, h, _p(Y))
    return Y


def combine_bwd(dY, O, row_of, prob, R, prec="f64"):
    """Returns dO[R,h], dprob[T,k] for L = <dY, Y>."""
    dY, O = _arr(dY, _dt(prec)), _arr(O, _dt(prec))
    row_of, prob = _arr(row_of, np.int32), _arr(prob, _dt(prec))
    T, k = row_of.shape
    h = dY.shape[1]
    dO = np.empty((R, h), _dt(prec))
    dprob = np.empty((T, k), _dt(prec))
    _fn("orc_combine_bwd", prec)(_p(dY), _p(O), _p(row_of), _p(prob), T, k, h, C.c_int64(R), _p(dO), _p(dprob))
    return dO, dprob


# ----------------------------------------------------------------------------
# blockwise FP8 (fp32 decisions, independent of `prec`)
# ----------------------------------------------------------------------------
def e4m3_decode(code: int) -> float:
    return float(lib().orc_e4m3_decode(int(code)))


def e4m3_encode(x: float) -> int:
    return int(lib().orc_e4m3_encode(float(x)))


def fp8_quant_1x128(X):
    X = _arr(X, np.float32)
    rows, K = X.shape
    q = np.empty((rows, K), np.uint8)
    s = np.empty((rows, K // 128), np.float32)
    if lib().orc_fp8_quant_1x128(_p(X), C.c_int64(rows), K, _p(q), _p(s)) != 0:
        raise ValueError("K must be a multiple of 128")
    return q, s


def fp8_quant_128x1(X):
    X = _arr(X, np.float32)
    R, N = X.shape
    q = np.empty((R, N), np.uint8)
    s = np.empty((R // 128, N), np.float32)
    if lib().orc_fp8_quant_128x1(_p(X), C.c_int64(R), N, _p(q), _p(s)) != 0:
        raise ValueError("row count must be a multiple of 128")
    return q, s


def fp8_quant_128x128(W):
    W = _arr(W, np.float32)
    G, N, K = W.shape
    q = np.empty((G, N, K), np.uint8)
    s = np.empty((G, N // 128, K // 128), np.float32)
    if lib().orc_fp8_quant_128x128(_p(W), G, N, K, _p(q), _p(s)) != 0:
        raise ValueError("N and K must be multiples of 128")
    return q, s


def fp8_dequant(q, s, mode):
    """mode: '1x128' | '128x1' | '128x128' -> float64 array of q's shape."""
    q, s = _arr(q, np.uint8), _arr(s, np.float32)
    m = {"1x128": 0, "128x1": 1, "128x128": 2}[mode]
    if m == 2:
        G, rows, K = q.shape
    else:
        G, (rows, K) = 1, q.shape
    out = np.empty(q.shape, np.float64)
    lib().orc_fp8_dequant(_p(q), _p(s), m, G, C.c_int64(rows), K, _p(out))
    return out


# ----------------------------------------------------------------------------
# the layer, composed in the paper's order (Sec. 2.1.1)
# ----------------------------------------------------------------------------
def layer_forward(X, idx, prob, W1, W2, E, align=1, Ws1=None, Ws2=None, prec="f64"):
    """Permute -> fc1 -> SwiGLU -> fc2 -> weighted combine (+ shared expert).  Returns every intermediate."""
    m = permute_maps(idx, E, align)
    R = m.Rtot
    Xp = permute_rows(X, m.src_of[:R], m.k, prec)
    Z = grouped_gemm_nt(Xp, W1, m.offsets, prec=prec)
    A = swiglu(Z, prec)
    O = grouped_gemm_nt(A, W2, m.offsets, prec=prec)
    S = Zs = As = None
    if Ws1 is not None:
        off1 = np.array([0, X.shape[0]], np.int32)
        Zs = grouped_gemm_nt(X, Ws1[None], off1, prec=prec)
        As = swiglu(Zs, prec)
        S = grouped_gemm_nt(As, Ws2[None], off1, prec=prec)
    Y = combine(O, m.row_of, prob, S, prec)
    return SimpleNamespace(maps=m, R=R, Xp=Xp, Z=Z, A=A, O=O, S=S, Zs=Zs, As=As, Y=Y)


def layer_backward(fw, X, prob, W1, W2, dY, Ws1=None, Ws2=None, prec="f64"):
    """Backward of L = <dY, Y> through combine, fc2, SwiGLU, fc1, permute (routing frozen)."""
    m, R = fw.maps, fw.R
    dO, dprob = combine_bwd(dY, fw.O, m.row_of, prob, R, prec)
    dW2 = grouped_gemm_tn(dO, fw.A, m.offsets, prec=prec)
    dA = grouped_gemm_nn(dO, W2, m.offsets, prec=prec)
    dZ = swiglu_bwd(dA, fw.Z, prec)
    dW1 = grouped_gemm_tn(dZ, fw.Xp, m.offsets, prec=prec)
    dXp = grouped_gemm_nn(dZ, W1, m.offsets, prec=prec)
    dX = combine(dXp, m.row_of, None, None, prec)
    out = SimpleNamespace(dO=dO, dprob=dprob, dW2=dW2, dA=dA, dZ=dZ, dW1=dW1, dXp=dXp, dX=dX,
                          dWs1=None, dWs2=None, dX_shared=None)
    if Ws1 is not None:
        off1 = np.array([0, X.shape[0]], np.int32)
        out.dWs2 = grouped_gemm_tn(dY, fw.As, off1, prec=prec)[0]
        dAs = grouped_gemm_nn(dY, Ws2[None], off1, prec=prec)
        dZs = swiglu_bwd(dAs, fw.Zs, prec)
        out.dWs1 = grouped_gemm_tn(dZs, X, off1, prec=prec)[0]
        out.dX_shared = grouped_gemm_nn(dZs, Ws1[None], off1, prec=prec)
        out.dZs = dZs
    return out


# ----------------------------------------------------------------------------
# the same layer with the routing weight absorbed into the activation (Sec. 4.1.2, eq. (2))
# ----------------------------------------------------------------------------
def gather_row_prob(prob, src_of):
    """row_prob[r] = prob[t,s] of the slot that row r holds; 0 for padding rows."""
    flat = np.asarray(prob, np.float64).reshape(-1)
    src = np.asarray(src_of)
    return np.where(src >= 0, flat[np.maximum(src, 0)], 0.0)


def layer_forward_eq2(X, idx, prob, W1, W2, E, align=1, Ws1=None, Ws2=None, prec="f64"):
    """y = sum_i W2_i (p_i * phi(W1_i x)): weights applied before fc2, plain-sum combine."""
    m = permute_maps(idx, E, align)
    R = m.Rtot
    Xp = permute_rows(X, m.src_of[:R], m.k, prec)
    Z = grouped_gemm_nt(Xp, W1, m.offsets, prec=prec)
    row_p = gather_row_prob(prob, m.src_of[:R])
    A = swiglu(Z, prec) * row_p[:, None]
    O = grouped_gemm_nt(A, W2, m.offsets, prec=prec)
    S = Zs = As = None
    if Ws1 is not None:
        off1 = np.array([0, X.shape[0]], np.int32)
        Zs = grouped_gemm_nt(X, Ws1[None], off1, prec=prec)
        As = swiglu(Zs, prec)
        S = grouped_gemm_nt(As, Ws2[None], off1, prec=prec)
    Y = combine(O, m.row_of, None, S, prec)
    return SimpleNamespace(maps=m, R=R, Xp=Xp, Z=Z, A=A, O=O, S=S, Zs=Zs, As=As, Y=Y, row_prob=row_p)


def layer_backward_eq2(fw, X, prob, W1, W2, dY, Ws1=None, Ws2=None, prec="f64"):
    """Backward of L = <dY, Y> for eq. (2): dL/dp comes from the saved pre-activations, not from O."""
    m, R = fw.maps, fw.R
    dO = permute_rows(dY, m.src_of[:R], m.k, prec)              # plain copies of dY, zero rows for padding
    dW2 = grouped_gemm_tn(dO, fw.A, m.offsets, prec=prec)       # A already carries the weight
    dA = grouped_gemm_nn(dO, W2, m.offsets, prec=prec)          # gradient w.r.t. p * phi(z)
    act = swiglu(fw.Z, prec)                                    # phi(z), recomputed
    dprob_row = (dA * act).sum(axis=1)
    dZ = swiglu_bwd(dA, fw.Z, prec) * fw.row_prob[:, None]
    dW1 = grouped_gemm_tn(dZ, fw.Xp, m.offsets, prec=prec)
    dXp = grouped_gemm_nn(dZ, W1, m.offsets, prec=prec)
    dX = combine(dXp, m.row_of, None, None, prec)
    row_of = np.asarray(m.row_of)
    dprob = np.where(row_of >= 0, dprob_row[np.maximum(row_of, 0)], 0.0)
    out = SimpleNamespace(dO=dO, dprob=dprob, dprob_row=dprob_row, dW2=dW2, dA=dA, dZ=dZ, dW1=dW1, dXp=dXp, dX=dX,
                          dWs1=None, dWs2=None, dX_shared=None)
    if Ws1 is not None:
        off1 = np.array([0, X.shape[0]], np.int32)
        out.dWs2 = grouped_gemm_tn(dY, fw.As, off1, prec=prec)[0]
        dAs = grouped_gemm_nn(dY, Ws2[None], off1, prec=prec)
        dZs = swiglu_bwd(dAs, fw.Zs, prec)
        out.dWs1 = grouped_gemm_tn(dZs, X, off1, prec=prec)[0]
        out.dX_shared = grouped_gemm_nn(dZs, Ws1[None], off1, prec=prec)
        out.dZs = dZs
    return out


# ----------------------------------------------------------------------------
# router score function backward (Sec. 2.1.2 item 2): dL/dlogits from dL/dweights, selection frozen
# ----------------------------------------------------------------------------
def route_topk_bwd(logits, topk_idx, dprob, score=SOFTMAX, norm_topk=False, scale=1.0):
    """Weights are w_s = scale * q_s / D with q_s the score of the s-th selected expert and D = sum of the
    selected scores (norm_topk) or 1.  Chain rule through D, then through softmax (all E logits move every
    score) or sigmoid (a logit moves only its own score).  fp64, one token at a time."""
    L = np.asarray(logits, np.float64)
    T, E = L.shape
    out = np.zeros((T, E))
    for t in range(T):
        l = L[t]
        idx = np.asarray(topk_idx[t], np.int64)
        dw = np.asarray(dprob[t], np.float64)
        if score == SOFTMAX:
            ex = np.exp(l - l.max())
            sc = ex / ex.sum()
        else:
            sc = 1.0 / (1.0 + np.exp(-l))
        q = sc[idx]
        if norm_topk:
            D = q.sum()
            dq = scale * (dw / D - np.dot(dw, q) / (D * D))
        else:
            dq = scale * dw
        if score == SOFTMAX:
            g = np.zeros(E)
            g[idx] = dq
            out[t] = sc * (g - np.dot(dq, q))
        else:
            out[t, idx] = dq * q * (1.0 - q)
    return out


# ----------------------------------------------------------------------------
# MXFP8 (Sec. 5.3.3): E4M3 elements, 1x32 blocks, E8M0 scales
# ----------------------------------------------------------------------------
def mx_quant_1x32(X):
    """Row-wise: blocks of 32 along the last dimension.  Returns (codes [rows,K] u8, e8m0 [rows,K/32] u8)."""
    X = _arr(X, np.float32)
    rows, K = X.shape
    q = np.empty((rows, K), np.uint8)
    e = np.empty((rows, K // 32), np.uint8)
    if lib().orc_mx_quant_1x32(_p(X), C.c_int64(rows), K, _p(q), _p(e)) != 0:
        raise ValueError("K must be a multiple of 32")
    return q, e


def mx_quant_32x1(W):
    """Column-wise for a weight stack [G,N,K]: blocks of 32 along N.  Returns (codes [G,N,K], e8m0 [G,K,N/32])."""
    W = _arr(W, np.float32)
    G, N, K = W.shape
    q = np.empty((G, N, K), np.uint8)
    e = np.empty((G, K, N // 32), np.uint8)
    if lib().orc_mx_quant_32x1(_p(W), G, N, K, _p(q), _p(e)) != 0:
        raise ValueError("N must be a multiple of 32")
    return q, e


def mx_dequant(q, e, mode):
    """mode "1x32": q [rows,K], e [rows,K/32];  mode "32x1": q [G,N,K], e [G,K,N/32].  Returns float64."""
    q = _arr(q, np.uint8)
    e = _arr(e, np.uint8)
    out = np.empty(q.shape, np.float64)
    if mode == "1x32":
        rows, K = q.shape
        lib().orc_mx_dequant(_p(q), _p(e), 0, 1, C.c_int64(rows), K, _p(out))
    else:
        G, N, K = q.shape
        lib().orc_mx_dequant(_p(q), _p(e), 1, G, C.c_int64(N), K, _p(out))
    return out


def e8m0_from_amax(a: float) -> int:
    return int(lib().orc_e8m0_from_amax(C.c_float(a)))
