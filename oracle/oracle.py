"""CPU oracle for phantom parallelism -- TEST INFRASTRUCTURE, not part of the product.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use
this module.  It shares no code with the HIP path.

The per-rank, per-layer arithmetic is the plain fp64 C in phantom_oracle.c
(Section IV-A Eq. (ylq); Section IV-B Eq. (deltaL), (backprop), (bpb)-(bpD)).
This file puts those calls together the way the paper's pipeline does:

  * several ranks: the All-Gather of the phantom layers g^(i) (forward) and the
    Reduce-Scatter of dLoss/dg^(i,j) (backward) of Algorithm 1, done here as
    plain copies and sums in memory;
  * several layers: y_l feeds layer l+1, dLoss/dy_l comes back from layer l+1
    (Eq. (backprop));
  * the loss at the output (Section IV-B, "Local error at the output") and a
    plain SGD update.

Readings of the paper (it is silent on these):
  * MSE loss = 1/(2B) * sum_b sum_o (y_L - t)^2, so dLoss/dy_L = (y_L - t)/B:
    the paper's (y_L - y) per sample, averaged over the batch.  Summing over
    features keeps the loss additive over ranks as Section IV-B assumes.
  * the last layer is activated like the others (sigma_L appears in Eq. (deltaL)).
  * storage type bfloat16 ("bf16 in, fp32 accumulate"): tensors that are
    operands of a matrix product (layer inputs y_l, delta) and tensors that
    cross the rank boundary (g, dLoss/dg^(i,j), and their reduce-scatter sum)
    are rounded to bfloat16 when formed; sums and elementwise functions are
    exact.  With storage type fp32 nothing is rounded (fp64 throughout).
  * the sigma' factor of Eq. (deltaL) and Eq. (backprop) is sigma'(A_l) evaluated
    in fp64 on the unrounded pre-activation, for every storage type.
  * SGD: w <- w - lr * dLoss/dw for L, C, D, b of every layer, all gradients
    taken at the weights before the update.

Parity pins: tests/test_oracle_pins.py.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "phantom_oracle.c")
_LIB = os.path.join(_HERE, "libphantom_oracle.so")

ACTS = {"identity": 0, "relu": 1, "gelu": 2}

_lib = None


def build(force: bool = False) -> str:
    """Compile phantom_oracle.c with gcc (OpenMP) into oracle/libphantom_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.pho_round_bf16.restype = ctypes.c_double
        _lib.pho_round_bf16.argtypes = [ctypes.c_double]
        _lib.pho_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(lib().pho_num_threads())


def _c(a):
    """float64 C-contiguous view/copy and its pointer (None -> NULL)."""
    if a is None:
        return None, ctypes.c_void_p(0)
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _i(v):
    return ctypes.c_int64(int(v))


def round_bf16(a: np.ndarray) -> np.ndarray:
    out = np.array(a, dtype=np.float64, copy=True, order="C")
    lib().pho_round_bf16_array(out.ctypes.data_as(ctypes.c_void_p), _i(out.size))
    return out


def rd(a: np.ndarray, storage: str) -> np.ndarray:
    """Round to the storage type where the reading above says a tensor is stored."""
    if storage == "bf16":
        return round_bf16(a)
    if storage == "f32":
        return np.asarray(a, dtype=np.float64)
    raise ValueError(storage)


# ----------------------------------------------------------------------------
# one rank, one layer
# ----------------------------------------------------------------------------

def _vp(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else ctypes.c_void_p(0)


def compress(X, Cw):
    """g^(j) = C^(j) y^(j) for every sample: [B,s],[k,s] -> [B,k]."""
    B, s = X.shape
    k = Cw.shape[0]
    X_, pX = _c(X); Cw_, pC = _c(Cw)
    g = np.empty((B, k))
    lib().pho_compress(_i(B), _i(s), _i(k), pX, pC, _vp(g))
    return g


def layer_update(act, X, Lw, Dw, bias, G):
    """A = b + L y + sum_i D^(i,j) g^(i), Y = sigma(A) on one rank (Eq. (ylq))."""
    B, si = X.shape              # si inputs and so outputs of the layer on this rank (equal in the paper's text)
    so = Lw.shape[0]
    q = 0 if Dw is None else Dw.shape[0]
    k = Dw.shape[2] if q else 0
    X_, pX = _c(X); Lw_, pL = _c(Lw); b_, pb = _c(bias)
    Dw_, pD = _c(Dw if q else None); G_, pG = _c(G if q else None)
    if q:
        assert G_.shape == (q, B, k) and Dw_.shape == (q, so, k)
    assert Lw_.shape == (so, si) and b_.shape == (so,)
    A = np.empty((B, so)); Y = np.empty((B, so))
    lib().pho_layer_update(_i(B), _i(si), _i(so), _i(k), _i(q), ctypes.c_int(ACTS[act]),
                           pX, pL, pD, pb, pG, _vp(A), _vp(Y))
    return A, Y


def layer_fwd(act, X, Lw, Cw, Dw, bias, G):
    """Eq. (ylq) on one rank.  Returns A (pre-activation), Y, g_own (None when p = 1)."""
    q = 0 if Dw is None else Dw.shape[0]
    g = compress(X, Cw) if q else None
    A, Y = layer_update(act, X, Lw, Dw, bias, G)
    return {"A": A, "Y": Y, "g_own": g}


def delta_of(act, dY, A, storage="f32"):
    """delta = dY * sigma'(A), Eq. (deltaL); rounded to bfloat16 when that is the storage type."""
    B, s = dY.shape
    dY_, pdY = _c(dY); A_, pA = _c(A)
    d = np.empty((B, s))
    lib().pho_delta(_i(B), _i(s), ctypes.c_int(ACTS[act]), ctypes.c_int(int(storage == "bf16")),
                    pdY, pA, _vp(d))
    return d


def error_compress(Dw, delta):
    """dG_send[i] = (D^(i,j))^T delta^(j): the h of Eq. (backprop)."""
    q, s, k = Dw.shape
    B = delta.shape[0]
    Dw_, pD = _c(Dw); d_, pd = _c(delta)
    out = np.empty((q, B, k))
    lib().pho_error_compress(_i(B), _i(s), _i(k), _i(q), pD, pd, _vp(out))
    return out


def layer_grads(delta, X, Lw, Cw, G, dg_own, need_dX=True):
    """dX (braces of Eq. (backprop)) and Eq. (bpb)-(bpD) once dg_own is known."""
    B, si = X.shape
    so = Lw.shape[0]
    q = 0 if G is None else G.shape[0]
    k = Cw.shape[0] if q > 0 else 0
    d_, pd = _c(delta); X_, pX = _c(X); Lw_, pL = _c(Lw)
    Cw_, pC = _c(Cw if q else None); G_, pG = _c(G if q else None); h_, ph = _c(dg_own if q else None)
    assert d_.shape == (B, so) and Lw_.shape == (so, si)
    if q:
        assert G_.shape == (q, B, k) and h_.shape == (B, k) and Cw_.shape == (k, si)
    dX = np.empty((B, si)) if need_dX else None
    dLw = np.empty((so, si)); dCw = np.empty((k, si)); dDw = np.empty((q, so, k)); db = np.empty((so,))
    lib().pho_layer_grads(_i(B), _i(si), _i(so), _i(k), _i(q), pd, pX, pL, pC, pG, ph,
                          _vp(dX), _vp(dLw), _vp(dCw), _vp(dDw), _vp(db))
    return {"dX": dX, "dLw": dLw, "dCw": dCw if q else None, "dDw": dDw if q else None, "dbias": db}


def layer_bwd(act, dY, X, A, Lw, Cw, Dw, G, dg_own, storage="f32", need_dX=True):
    """Backward of one layer on one rank with the peers' reduce-scatter result dg_own given."""
    q = 0 if Dw is None else Dw.shape[0]
    delta = delta_of(act, dY, A, storage)
    out = layer_grads(delta, X, Lw, Cw, G, dg_own, need_dX)
    out["delta"] = delta
    out["dG_send"] = error_compress(Dw, delta) if q else None
    return out


# ----------------------------------------------------------------------------
# all p ranks together (Algorithm 1's gather / reduce-scatter done in memory)
# ----------------------------------------------------------------------------

def without_slot(a, j):
    """Slots i != j of a [p, ...] array, in increasing i: what rank j holds after the gather."""
    return np.concatenate([a[:j], a[j + 1:]], axis=0)


def all_ranks_fwd(act, X, P, storage="f32"):
    """X [p,B,s]; P = stacked weights Lw[p,s,s], Cw[p,k,s], Dw[p,p-1,s,k], bias[p,s].

    Returns A, Y [p,B,s] and the gathered phantom layers G_full [p,B,k]
    (rank j reads every slot but its own).
    """
    p, B, _ = X.shape
    so = P["Lw"].shape[1]
    A = np.empty((p, B, so)); Y = np.empty((p, B, so))
    if p == 1:
        A[0], Y[0] = layer_update(act, X[0], P["Lw"][0], None, P["bias"][0], None)
        return {"A": A, "Y": Y, "G_full": None}
    # compression on every rank, then the All-Gather (Algorithm 1, forward)
    G_full = rd(np.stack([compress(X[j], P["Cw"][j]) for j in range(p)]), storage)
    for j in range(p):
        A[j], Y[j] = layer_update(act, X[j], P["Lw"][j], P["Dw"][j], P["bias"][j], without_slot(G_full, j))
    return {"A": A, "Y": Y, "G_full": G_full}


def reduce_scatter(dG_send, storage="f32"):
    """dG_send [p(holder j), p-1(peer slot), B, k] -> dg_own [p(source i), B, k]:
    dLoss/dg^(i) = sum_{j != i} dLoss/dg^(i,j)  (Section IV-B, "Communication"; Algorithm 1, backward).
    On holder j, peer i sits in slot i if i < j, else i-1."""
    p = dG_send.shape[0]
    out = np.zeros(dG_send.shape[:1] + dG_send.shape[2:])
    for i in range(p):
        for j in range(p):
            if j != i:
                out[i] += dG_send[j, i if i < j else i - 1]
    return rd(out, storage)


def all_ranks_bwd(act, dY, X, A, P, G_full, storage="f32", need_dX=True):
    """Backward of one layer on all ranks.  dY, X, A: [p,B,s].  Returns stacked gradients."""
    p, B, s = X.shape
    delta = np.stack([delta_of(act, dY[j], A[j], storage) for j in range(p)])
    if p == 1:
        g = layer_grads(delta[0], X[0], P["Lw"][0], None, None, None, need_dX)
        return {"delta": delta, "dX": None if g["dX"] is None else g["dX"][None], "dLw": g["dLw"][None],
                "dbias": g["dbias"][None], "dCw": None, "dDw": None, "dG_send": None, "dg_own": None}
    # error compression on every holder, then the Reduce-Scatter
    dG_send = rd(np.stack([error_compress(P["Dw"][j], delta[j]) for j in range(p)]), storage)
    dg_own = reduce_scatter(dG_send, storage)
    per = [layer_grads(delta[j], X[j], P["Lw"][j], P["Cw"][j], without_slot(G_full, j), dg_own[j], need_dX)
           for j in range(p)]
    out = {name: (np.stack([r[name] for r in per]) if per[0][name] is not None else None) for name in per[0]}
    out.update(delta=delta, dG_send=dG_send, dg_own=dg_own)
    return out


# ----------------------------------------------------------------------------
# several layers, loss, SGD
# ----------------------------------------------------------------------------

def mse_loss(Y, T):
    """Reading stated in the module header: loss = 1/(2B) sum (Y-T)^2 over batch and features
    (and ranks, if Y has a leading rank axis); dLoss/dY = (Y-T)/B."""
    B = Y.shape[-2]
    diff = Y - T
    return float(0.5 * np.sum(diff * diff) / B), diff / B


GRAD_NAMES = ("Lw", "Cw", "Dw", "bias")


def ffn_forward(act, X0, layers, storage="f32", all_ranks=True):
    """Forward through every layer.  layers[l] holds the weights (stacked over ranks in
    all-ranks mode) and, in one-rank mode, the seeded peer buffer 'G'.
    Returns per-layer lists X (inputs), A, Y (unrounded outputs) and G."""
    Xs, As, Ys, Gs = [], [], [], []
    X = rd(X0, storage)
    for P in layers:
        if all_ranks:
            r = all_ranks_fwd(act, X, P, storage)
            G, g_own = r["G_full"], None
        else:
            q = P["Dw"].shape[0] if P.get("Dw") is not None else 0
            r = layer_fwd(act, X, P["Lw"], P["Cw"] if q else None, P["Dw"] if q else None, P["bias"],
                          P["G"] if q else None)
            G = P["G"] if q else None
        Xs.append(X); As.append(r["A"]); Ys.append(r["Y"]); Gs.append(G)
        X = rd(r["Y"], storage)      # y_l is the next layer's matrix-product operand
    return {"X": Xs, "A": As, "Y": Ys, "G": Gs, "out": X}


def ffn_step(act, X0, T, layers, lr, storage="f32", all_ranks=True):
    """One forward + backward + SGD step.  Returns the loss, per-layer gradients, updated
    weights, and the forward tensors.  In one-rank mode layers[l]['dg_own'] is the seeded
    reduce-scatter result of layer l."""
    fw = ffn_forward(act, X0, layers, storage, all_ranks)
    loss, dY = mse_loss(fw["out"], T)
    grads = [None] * len(layers)
    for l in reversed(range(len(layers))):
        P = layers[l]
        need_dX = l > 0
        if all_ranks:
            g = all_ranks_bwd(act, dY, fw["X"][l], fw["A"][l], P, fw["G"][l], storage, need_dX)
        else:
            q = P["Dw"].shape[0] if P.get("Dw") is not None else 0
            g = layer_bwd(act, dY, fw["X"][l], fw["A"][l], P["Lw"], P["Cw"] if q else None,
                          P["Dw"] if q else None, P["G"] if q else None, P["dg_own"] if q else None,
                          storage, need_dX)
        grads[l] = g
        dY = g["dX"]                 # dLoss/dy_{l-1}; the sigma' factor is applied by the next delta_of
    new_layers = []
    for P, g in zip(layers, grads):
        upd = dict(P)
        for name in GRAD_NAMES:
            if P.get(name) is not None and g.get("d" + name) is not None:
                upd[name] = P[name] - lr * g["d" + name]
        new_layers.append(upd)
    return {"loss": loss, "grads": grads, "layers": new_layers, "forward": fw}


# ----------------------------------------------------------------------------
# bookkeeping the paper prints: model size (Table 1) and operation counts (Section IV)
# ----------------------------------------------------------------------------

def param_shapes(n, p, k):
    """Shapes of everything ONE rank stores for one layer (Section IV-A, the three bullets, plus b)."""
    s = n // p
    shapes = {"Lw": (s, s), "bias": (s,)}
    if p > 1:
        shapes["Cw"] = (k, s)
        shapes["Dw"] = (p - 1, s, k)
    return shapes


def param_count(n, p, k, layers):
    """Trainable parameters of the whole phantom model: all ranks, all layers."""
    per_rank = sum(int(np.prod(shape)) for shape in param_shapes(n, p, k).values())
    return layers * p * per_rank


def mac_counts(n, p, k, batch):
    """Multiply-adds of one layer on one rank, counted term by term from the sums in
    pho_layer_fwd / pho_layer_bwd: returns (forward, backward)."""
    s, q = n // p, p - 1
    fwd = batch * (k * s * (q > 0) + s * (s + q * k))
    bwd = batch * (q * k * s          # error compression
                   + s * s + k * s * (q > 0)   # dX
                   + s * s + q * s * k          # dLw, dDw
                   + k * s * (q > 0))           # dCw
    return fwd, bwd
