"""Element-wise parity of the fused step, stage by stage.

phantom_ffn_step is run ONCE, as bench.py runs it, with its taps on (copies of y_l, g_l, delta_l, dG_send_l and
the reduce-scatter result, taken after the launch that finishes each).  Every stage of Eq. (ylq), Eq. (deltaL),
Eq. (backprop) and Eq. (bpb)-(bpD) is then recomputed by the oracle's single-stage functions FROM THE GPU'S OWN
TENSORS of the stage before, so that every bf16 rounding and every ReLU mask is decided on identical inputs on
both sides, and compared element by element at the parity bar.  Two correct implementations drift apart over
several bf16 layers (a value that rounds the other way nudges everything downstream); fed this way nothing
drifts, and a mistake in any launch of the step's schedule (riders, sum-on-read reduce-scatter, output error in
the update's epilogue, deferred SGD) shows in the stage it belongs to.
"""
import numpy as np
import torch

import paper_2508_00960_amd as ph
import phantom_inputs as pin
from oracle import oracle

from helpers import TOL, assert_close, empty, empty_f32, to_gpu, to_gpu_f32, to_np, workspace


def run_step_with_taps(prob, seed, lr, mode):
    dt, L, q, p, B = prob.dtype, prob.layers, prob.peers, prob.p, prob.batch
    all_ranks = prob.rank < 0
    lead = (p,) if all_ranks else ()
    data = pin.all_rank_step_inputs(prob, seed) if all_ranks else pin.one_rank_step_inputs(prob, seed)
    pc = ph.make_problem(prob.n, prob.p, prob.k, prob.batch, prob.layers, prob.act, prob.dtype, prob.rank,
                         widths=prob.widths, ks=prob.ks)
    ws = workspace(ph.workspace_bytes(pc))
    ws.fill_(0xFF)
    names = ["Lw", "bias"] + (["Cw", "Dw"] if q else [])
    train = mode != "forward"
    W = {nm: [to_gpu(P[nm], dt) for P in data["layers"]] for nm in names}
    M = {nm: [to_gpu_f32(P[nm]) for P in data["layers"]] for nm in names} if (dt == "bf16" and mode == "train") else {}
    Gd = {nm: [empty_f32(P[nm].shape) for P in data["layers"]] for nm in names} if train else {}
    G = [to_gpu(P["G"], dt) for P in data["layers"]] if (q and not all_ranks) else None
    dg = [to_gpu(P["dg_own"], dt) for P in data["layers"]] if (q and not all_ranks and train) else None
    taps = {"Y": [empty(lead + (B, prob.s_out(l)), dt) for l in range(L)]}
    if q:
        taps["g_own"] = [empty(lead + (B, prob.k_of(l)), dt) for l in range(L)]
    if train:
        taps["delta"] = [empty(lead + (B, prob.s_out(l)), dt) for l in range(L)]
        if q:
            taps["dG_send"] = [empty(lead + (q, B, prob.k_of(l)), dt) for l in range(L)]
            if all_ranks:
                taps["dg_own"] = [empty((p, B, prob.k_of(l)), dt) for l in range(L)]
    for per_layer in taps.values():
        for t in per_layer:
            t.view(torch.int16).fill_(0x7FC1)      # NaN patterns: a tap that is not written shows
    Y_out = empty(data["T"].shape, dt)
    loss = empty_f32((4,))
    ph.ffn_step(pc, to_gpu(data["X0"], dt), to_gpu(data["T"], dt) if train else None, W["Lw"], W.get("Cw"), W.get("Dw"),
                W["bias"], Lw_master=M.get("Lw"), Cw_master=M.get("Cw"), Dw_master=M.get("Dw"), bias_master=M.get("bias"),
                G=G, dg_own=dg, dLw=Gd.get("Lw"), dCw=Gd.get("Cw"), dDw=Gd.get("Dw"), dbias=Gd.get("bias"),
                Y_out=Y_out, loss=loss if train else None, lr=lr, mode=mode, workspace=ws, taps=taps)
    torch.cuda.synchronize()
    return data, W, M, Gd, taps, Y_out, (float(loss[0]) if train else None)


def check_stages(prob, seed=0, lr=1e-3, mode="train", rows=None):
    """Runs the step with taps and checks every stage against the oracle fed from the GPU's own tensors.
    rows: forward-only problems may check a sample of the batch rows (rows of a forward pass are independent).
    Returns the worst relative error per kind of tensor."""
    dt, L, q, p, B, act = prob.dtype, prob.layers, prob.peers, prob.p, prob.batch, prob.act
    all_ranks = prob.rank < 0
    ranks = range(p) if all_ranks else [0]
    train = mode != "forward"
    assert rows is None or not train
    data, W, M, Gd, taps, Y_out, loss = run_step_with_taps(prob, seed, lr, mode)
    worst = {}

    def close(kind, name, got, want, tol=None):
        worst[kind] = max(worst.get(kind, 0.0), assert_close(name, got, want, dt, tol))

    idx = np.arange(B) if rows is None else np.sort(np.random.default_rng(seed).choice(B, rows, replace=False))
    sel = torch.from_numpy(idx).cuda()

    def host(t):            # a GPU tensor (all batch rows or the sampled ones) as fp64, [ranks, rows, ...]
        a = to_np(t.index_select(t.dim() - 2, sel))
        return a if all_ranks else a[None]

    def per_rank(P, name, j):
        return P[name][j] if all_ranks else P[name]

    # ---- forward, Eq. (ylq): compression, then the update from the GPU's own gathered buffer --------------
    X0 = np.asarray(data["X0"])
    X = (X0[:, idx] if all_ranks else X0[idx][None])
    A_l, X_l = [], []
    for l in range(L):
        P = data["layers"][l]
        X_l.append(X)
        if q:
            g_gpu = host(taps["g_own"][l])
            g_ref = np.stack([oracle.compress(X[jj], per_rank(P, "Cw", j)) for jj, j in enumerate(ranks)])
            close("g_own", f"g_own[{l}]", torch.from_numpy(g_gpu), g_ref)
        A = []
        Y = []
        for jj, j in enumerate(ranks):
            if not q:
                gathered = None
            elif all_ranks:
                gathered = oracle.without_slot(g_gpu, j)
            else:
                gathered = np.asarray(P["G"])[:, idx]
            a, y = oracle.layer_update(act, X[jj], per_rank(P, "Lw", j), per_rank(P, "Dw", j) if q else None,
                                       per_rank(P, "bias", j), gathered)
            A.append(a); Y.append(y)
        A, Y = np.stack(A), np.stack(Y)
        y_gpu = host(taps["Y"][l])
        close("Y", f"Y[{l}]", torch.from_numpy(y_gpu), Y)
        A_l.append(A)
        X = y_gpu                                   # the next layer's operand: the GPU's own stored y_l
    assert torch.equal(Y_out, taps["Y"][L - 1])
    if not train:
        return worst

    # ---- output error, Eq. (deltaL) -----------------------------------------------------------------------
    T = np.asarray(data["T"]) if all_ranks else np.asarray(data["T"])[None]
    y_L = host(taps["Y"][L - 1])
    want_loss, dY = oracle.mse_loss(y_L, T)
    assert abs(loss - want_loss) <= (1e-5 if dt == "f32" else 1e-4) * abs(want_loss), (loss, want_loss)

    def sigma_arg(l):       # what sigma' is evaluated on: for ReLU the sign of the GPU's own stored output
        return host(taps["Y"][l]) if act == "relu" else A_l[l]

    delta = np.stack([oracle.delta_of(act, dY[jj], sigma_arg(L - 1)[jj], dt) for jj in range(len(ranks))])
    close("delta", f"delta[{L - 1}]", torch.from_numpy(host(taps["delta"][L - 1])), delta)

    # ---- backward, Eq. (backprop), (bpb)-(bpD), from the GPU's own delta_l ----------------------------------
    for l in reversed(range(L)):
        P = data["layers"][l]
        d_gpu = host(taps["delta"][l])
        if q:
            send_gpu = to_np(taps["dG_send"][l])
            send_gpu = send_gpu if all_ranks else send_gpu[None]
            send_ref = np.stack([oracle.error_compress(per_rank(P, "Dw", j), d_gpu[jj]) for jj, j in enumerate(ranks)])
            close("dG_send", f"dG_send[{l}]", torch.from_numpy(send_gpu), send_ref)
            if all_ranks:
                dg = to_np(taps["dg_own"][l])
                close("dg_own", f"dg_own[{l}]", torch.from_numpy(dg), oracle.reduce_scatter(send_gpu, dt))
                g_gpu = host(taps["g_own"][l])
            else:
                dg = np.asarray(P["dg_own"])[None]
        grads = []
        for jj, j in enumerate(ranks):
            gathered = None if not q else (oracle.without_slot(g_gpu, j) if all_ranks else np.asarray(P["G"]))
            grads.append(oracle.layer_grads(d_gpu[jj], X_l[l][jj], per_rank(P, "Lw", j), per_rank(P, "Cw", j) if q else None,
                                            gathered, dg[jj] if q else None, need_dX=l > 0))
        for nm in Gd:
            want = np.stack([g["d" + nm] for g in grads])
            got = Gd[nm][l] if all_ranks else Gd[nm][l][None]
            close("d" + nm, f"d{nm}[{l}]", got, want)
        if l > 0:
            below = np.stack([oracle.delta_of(act, grads[jj]["dX"], sigma_arg(l - 1)[jj], dt) for jj in range(len(ranks))])
            close("delta", f"delta[{l - 1}]", torch.from_numpy(host(taps["delta"][l - 1])), below)

    # ---- SGD: master <- master - lr * (the gradient the step produced); compute copy = bf16(master) ---------
    for l in range(L):
        for nm in W:
            start = to_gpu(data["layers"][l][nm], dt)
            if mode != "train":
                assert torch.equal(W[nm][l], start), f"{nm}[{l}] changed without an update"
                continue
            old = torch.from_numpy(np.asarray(data["layers"][l][nm]).astype(np.float32)).cuda()
            want = old - lr * Gd[nm][l]
            ulp = torch.finfo(torch.float32).eps * (old.abs() + (lr * Gd[nm][l]).abs())
            new = M[nm][l] if dt == "bf16" else W[nm][l]
            assert bool(((new - want).abs() <= 2 * ulp).all()), f"{nm}[{l}] update"
            if dt == "bf16":
                assert torch.equal(W[nm][l], M[nm][l].to(torch.bfloat16))
    return worst
