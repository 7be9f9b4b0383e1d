"""Parity of the HIP path with the CPU oracle, element by element, on the same seeded inputs.

Every call goes through the C ABI (paper_2508_00960_amd.binding).  Bars (tests/helpers.py):
max over elements of |gpu - ref| / max(|ref|, RMS(ref)) <= 1e-5 (fp32 storage) or 2e-2 (bf16
storage, fp32 accumulate).  The backward is always fed the same pre-activation on both sides, so
the ReLU mask is one decision taken on identical values.
"""
import numpy as np
import pytest
import torch

import paper_2508_00960_amd as ph
import phantom_inputs as pin
from oracle import oracle

from helpers import assert_close, empty, empty_f32, to_gpu, to_gpu_f32, to_np, workspace

pytestmark = pytest.mark.gpu


def _prob_c(prob: pin.Problem):
    return ph.make_problem(prob.n, prob.p, prob.k, prob.batch, prob.layers, prob.act, prob.dtype, prob.rank,
                           widths=prob.widths, ks=prob.ks)


# ----------------------------------------------------------------------------
# one layer, one rank
# ----------------------------------------------------------------------------

ONE_RANK_CASES = [
    # n, p, k, B, act, dtype, rank          (shards and batches that are not multiples of any tile)
    (256, 4, 8, 32, "relu", "f32", 0),            # the tiny fp32 configuration's layer shape
    (288, 4, 5, 37, "gelu", "f32", 2),
    (210, 3, 7, 130, "identity", "f32", 1),
    (64, 1, 0, 19, "relu", "f32", 0),             # p = 1: a plain dense layer
    (512, 4, 16, 192, "relu", "bf16", 3),
    (1056, 8, 24, 200, "gelu", "bf16", 5),        # shard 132: ragged in every tile dimension
    (520, 4, 3, 67, "relu", "bf16", 0),           # k not a multiple of any vector width
    (2048, 16, 64, 300, "gelu", "bf16", 7),
    (96, 1, 0, 50, "gelu", "bf16", 0),
    (512, 2, 256, 160, "relu", "bf16", 1),        # k = n/p
    (1024, 4, 4, 300, "relu", "bf16", 1),         # k = 4: 8-byte vectors
    (1032, 4, 6, 260, "gelu", "bf16", 2),         # shard 258, k = 6: 4-byte vectors
    (2048, 8, 32, 1100, "relu", "bf16", 0),       # several tiles in every dimension, split reduction
    (1536, 4, 16, 520, "identity", "bf16", 3),    # shard 384 = 3 tiles
    (2048, 8, 32, 4100, "gelu", "bf16", 0),       # few tiles, long batch (65 reduction steps in the weight gradients)
    (1032, 4, 6, 3000, "relu", "bf16", 1),        # the same with 4-byte vectors and ragged tiles
    (256, 1, 0, 4100, "relu", "bf16", 0),         # p = 1, 4 tiles, 65 reduction steps: weight gradients in split pieces (atomic adds)
    (520, 1, 0, 2100, "gelu", "bf16", 0),         # the same, ragged tiles (shard 520)
]


def run_layer_one_rank(prob: pin.Problem, seed: int):
    d = pin.one_rank_layer_inputs(prob, 0, seed)
    dt, q = prob.dtype, prob.peers
    B, si, so, k = prob.batch, prob.s_in(0), prob.s_out(0), prob.k_of(0)
    pc = _prob_c(prob)
    ws = workspace(ph.workspace_bytes(pc))
    has = q > 0

    f_ref = oracle.layer_fwd(prob.act, d["X"], d["Lw"], d["Cw"] if has else None, d["Dw"] if has else None,
                             d["bias"], d["G"] if has else None)
    X, Lw, bias = to_gpu(d["X"], dt), to_gpu(d["Lw"], dt), to_gpu(d["bias"], dt)
    Cw = to_gpu(d["Cw"], dt) if has else None
    Dw = to_gpu(d["Dw"], dt) if has else None
    G = to_gpu(d["G"], dt) if has else None
    Y, A = empty((B, so), dt), empty((B, so), dt)
    g_own = empty((B, k), dt) if has else None
    ph.layer_fwd(pc, X, Lw, Cw, Dw, bias, G, Y, g_own, A, ws)
    torch.cuda.synchronize()
    errs = {"Y": assert_close("Y", Y, f_ref["Y"], dt), "A": assert_close("A_save", A, f_ref["A"], dt)}
    if has:
        errs["g_own"] = assert_close("g_own", g_own, f_ref["g_own"], dt)

    # backward: both sides read the same stored pre-activation
    A_in = pin.round_to_storage(f_ref["A"], dt)
    b_ref = oracle.layer_bwd(prob.act, d["dY"], d["X"], A_in, d["Lw"], d["Cw"] if has else None,
                             d["Dw"] if has else None, d["G"] if has else None, d["dg_own"] if has else None,
                             storage=dt)
    dY, A_gpu = to_gpu(d["dY"], dt), to_gpu(A_in, dt)
    dg_own = to_gpu(d["dg_own"], dt) if has else None
    dX = empty((B, si), dt)
    dLw, dbias = empty_f32((so, si)), empty_f32((so,))
    dCw = empty_f32((k, si)) if has else None
    dDw = empty_f32((q, so, k)) if has else None
    dG_send = empty((q, B, k), dt) if has else None
    ph.layer_bwd(pc, dY, X, A_gpu, Lw, Cw, Dw, G, dg_own, dX, dLw, dCw, dDw, dbias, dG_send, ws)
    torch.cuda.synchronize()
    errs["dX"] = assert_close("dX", dX, b_ref["dX"], dt)
    errs["dLw"] = assert_close("dLw", dLw, b_ref["dLw"], dt)
    errs["dbias"] = assert_close("dbias", dbias, b_ref["dbias"], dt)
    if has:
        errs["dCw"] = assert_close("dCw", dCw, b_ref["dCw"], dt)
        errs["dDw"] = assert_close("dDw", dDw, b_ref["dDw"], dt)
        errs["dG_send"] = assert_close("dG_send", dG_send, b_ref["dG_send"], dt)
    if prob.act == "relu":
        # the backward accepts the layer output in place of the pre-activation
        Y_in = to_gpu(pin.round_to_storage(np.maximum(A_in, 0.0), dt), dt)
        dX2 = empty((B, si), dt)
        ph.layer_bwd(pc, dY, X, Y_in, Lw, Cw, Dw, G, dg_own, dX2, dLw, dCw, dDw, dbias, dG_send, ws)
        torch.cuda.synchronize()
        assert torch.equal(dX, dX2)
    return errs


@pytest.mark.parametrize("n,p,k,B,act,dtype,rank", ONE_RANK_CASES)
def test_layer_one_rank(n, p, k, B, act, dtype, rank):
    prob = pin.Problem(n=n, p=p, k=k, batch=B, layers=1, act=act, dtype=dtype, rank=rank)
    print(f"case one-rank n={n} p={p} k={k} B={B} {act} {dtype} rank={rank}", flush=True)
    run_layer_one_rank(prob, seed=1)


# a layer whose input and output widths differ (Section IV, first paragraph): n_in, n_out, p, k, B, act, dtype, rank
RECTANGULAR_CASES = [
    (96, 160, 4, 5, 37, "gelu", "f32", 2),
    (1024, 512, 4, 16, 200, "relu", "bf16", 1),        # narrowing: shard 256 -> 128
    (528, 1056, 4, 24, 300, "gelu", "bf16", 3),        # widening, shards 132 -> 264: ragged in every tile dimension
    (2048, 1024, 8, 32, 4100, "gelu", "bf16", 0),      # long batch
    (1032, 520, 4, 6, 260, "relu", "bf16", 2),         # shards 258 -> 130, k = 6: 4-byte vectors
]


@pytest.mark.parametrize("n_in,n_out,p,k,B,act,dtype,rank", RECTANGULAR_CASES)
def test_rectangular_layer_one_rank(n_in, n_out, p, k, B, act, dtype, rank):
    print(f"case one-rank {n_in}->{n_out} p={p} k={k} B={B} {act} {dtype} rank={rank}", flush=True)
    prob = pin.Problem(n=n_in, p=p, k=k, batch=B, layers=1, act=act, dtype=dtype, rank=rank, widths=(n_in, n_out), ks=(k,))
    run_layer_one_rank(prob, seed=1)


def test_first_layer_needs_no_input_gradient():
    prob = pin.Problem(n=256, p=4, k=8, batch=32, act="relu", dtype="f32", rank=1)
    d = pin.one_rank_layer_inputs(prob, 0, seed=5)
    pc = _prob_c(prob)
    ws = workspace(ph.workspace_bytes(pc))
    A_in = pin.round_to_storage(oracle.layer_fwd("relu", d["X"], d["Lw"], d["Cw"], d["Dw"], d["bias"], d["G"])["A"], "f32")
    ref = oracle.layer_bwd("relu", d["dY"], d["X"], A_in, d["Lw"], d["Cw"], d["Dw"], d["G"], d["dg_own"], need_dX=False)
    t = {k_: to_gpu(v, "f32") for k_, v in d.items()}
    dLw, dCw, dDw, dbias = empty_f32((64, 64)), empty_f32((8, 64)), empty_f32((3, 64, 8)), empty_f32((64,))
    dG_send = empty((3, 32, 8), "f32")
    ph.layer_bwd(pc, t["dY"], t["X"], to_gpu(A_in, "f32"), t["Lw"], t["Cw"], t["Dw"], t["G"], t["dg_own"], None,
                 dLw, dCw, dDw, dbias, dG_send, ws)
    torch.cuda.synchronize()
    assert_close("dLw", dLw, ref["dLw"], "f32")
    assert_close("dG_send", dG_send, ref["dG_send"], "f32")


# ----------------------------------------------------------------------------
# one layer, all ranks on the device (gather / reduce-scatter in memory)
# ----------------------------------------------------------------------------

ALL_RANK_CASES = [
    (256, 4, 8, 32, "relu", "f32"),
    (330, 5, 6, 45, "gelu", "f32"),
    (48, 1, 0, 20, "relu", "f32"),
    # a long batch in fp32: the weight gradients sum 6000 products per element and still have to meet 1e-5
    (288, 3, 48, 6000, "identity", "f32"),
    (1024, 8, 32, 136, "relu", "bf16"),
    (792, 6, 10, 70, "gelu", "bf16"),
    # many ranks on the device (grouped products with 16 / 64 groups, the skipped slot moves with the group)
    (2048, 16, 8, 200, "relu", "bf16"),
    (4096, 64, 4, 96, "gelu", "bf16"),
    # more tiles than compute units: two tiles per workgroup.  17 tile rows (an odd number, the last one ragged)
    # x 16 groups in the forward, the error compression and the input gradient ...
    (2048, 16, 8, 2100, "relu", "bf16"),
    # ... and 2 x 6 tiles x 32 groups in the weight gradients, with the compressor gradient beside them
    (8192, 32, 16, 200, "gelu", "bf16"),
]


@pytest.mark.parametrize("n,p,k,B,act,dtype", ALL_RANK_CASES)
def test_layer_all_ranks(n, p, k, B, act, dtype):
    print(f"case all-ranks n={n} p={p} k={k} B={B} {act} {dtype}", flush=True)
    run_layer_all_ranks(pin.Problem(n=n, p=p, k=k, batch=B, layers=1, act=act, dtype=dtype, rank=-1))


@pytest.mark.parametrize("n_in,n_out,p,k,B,act,dtype", [
    (96, 160, 4, 5, 37, "gelu", "f32"),
    (1024, 2048, 8, 16, 136, "relu", "bf16"),
    (1584, 792, 6, 10, 70, "gelu", "bf16"),
])
def test_rectangular_layer_all_ranks(n_in, n_out, p, k, B, act, dtype):
    print(f"case all-ranks {n_in}->{n_out} p={p} k={k} B={B} {act} {dtype}", flush=True)
    run_layer_all_ranks(pin.Problem(n=n_in, p=p, k=k, batch=B, layers=1, act=act, dtype=dtype, rank=-1,
                                    widths=(n_in, n_out), ks=(k,)))


def run_layer_all_ranks(prob):
    p, B, k, act, dtype = prob.p, prob.batch, prob.k_of(0), prob.act, prob.dtype
    dt, si, so, q = dtype, prob.s_in(0), prob.s_out(0), prob.peers
    P = pin.all_rank_params(prob, 0, seed=2)
    X0, T = pin.network_io(prob, seed=2)
    Xn = pin.shard_columns(X0, p)
    dYn = pin.shard_columns(pin.round_to_storage(T / B, dt), p)
    has = q > 0
    pc = _prob_c(prob)
    ws = workspace(ph.workspace_bytes(pc))

    f_ref = oracle.all_ranks_fwd(act, Xn, P, dt)
    X, Lw, bias = to_gpu(Xn, dt), to_gpu(P["Lw"], dt), to_gpu(P["bias"], dt)
    Cw = to_gpu(P["Cw"], dt) if has else None
    Dw = to_gpu(P["Dw"], dt) if has else None
    Y, A = empty((p, B, so), dt), empty((p, B, so), dt)
    G_full = empty((p, B, k), dt) if has else None
    ph.layer_fwd(pc, X, Lw, Cw, Dw, bias, None, Y, G_full, A, ws)
    torch.cuda.synchronize()
    assert_close("Y", Y, f_ref["Y"], dt)
    assert_close("A_save", A, f_ref["A"], dt)
    if has:
        assert_close("G_full", G_full, f_ref["G_full"], dt)

    A_in = pin.round_to_storage(f_ref["A"], dt)
    b_ref = oracle.all_ranks_bwd(act, dYn, Xn, A_in, P, f_ref["G_full"], dt)
    dY, A_gpu = to_gpu(dYn, dt), to_gpu(A_in, dt)
    G_in = to_gpu(f_ref["G_full"], dt) if has else None
    dX = empty((p, B, si), dt)
    dLw, dbias = empty_f32((p, so, si)), empty_f32((p, so))
    dCw = empty_f32((p, k, si)) if has else None
    dDw = empty_f32((p, q, so, k)) if has else None
    dG_send = empty((p, q, B, k), dt) if has else None
    dg_own = empty((p, B, k), dt) if has else None
    ph.layer_bwd(pc, dY, X, A_gpu, Lw, Cw, Dw, G_in, dg_own, dX, dLw, dCw, dDw, dbias, dG_send, ws)
    torch.cuda.synchronize()
    for name, t in (("dX", dX), ("dLw", dLw), ("dbias", dbias), ("dCw", dCw), ("dDw", dDw), ("dG_send", dG_send),
                    ("dg_own", dg_own)):
        if t is not None:
            assert_close(name, t, b_ref[name], dt)


# ----------------------------------------------------------------------------
# several layers: forward + MSE + backward + SGD in one call
# ----------------------------------------------------------------------------

def relu_margin(fw):
    """Smallest |pre-activation| / RMS over all layers of an oracle forward: how far the closest
    ReLU decision is from its kink."""
    return min(float(np.min(np.abs(A)) / np.sqrt(np.mean(A * A))) for A in fw["A"])


def run_step(prob: pin.Problem, seed: int, lr: float, with_grads: bool = True, ws=None, mode: str = "train"):
    dt, L, q = prob.dtype, prob.layers, prob.peers
    all_ranks = prob.rank < 0
    data = pin.all_rank_step_inputs(prob, seed) if all_ranks else pin.one_rank_step_inputs(prob, seed)
    ref = oracle.ffn_step(prob.act, data["X0"], data["T"], data["layers"], lr, storage=dt, all_ranks=all_ranks)
    has = q > 0
    pc = _prob_c(prob)
    if ws is None:
        ws = workspace(ph.workspace_bytes(pc))
    names = ["Lw", "bias"] + (["Cw", "Dw"] if has else [])
    W = {nm: [to_gpu(P[nm], dt) for P in data["layers"]] for nm in names}
    M = {nm: [to_gpu_f32(P[nm]) for P in data["layers"]] for nm in names} if dt == "bf16" else {}
    Gd = {nm: [empty_f32(P[nm].shape) for P in data["layers"]] for nm in names} if with_grads else {}
    G = [to_gpu(P["G"], dt) for P in data["layers"]] if (has and not all_ranks) else None
    dg = [to_gpu(P["dg_own"], dt) for P in data["layers"]] if (has and not all_ranks) else None
    X0, T = to_gpu(data["X0"], dt), to_gpu(data["T"], dt)
    Y_out = empty(data["T"].shape, dt)
    loss = empty_f32((4,))
    ph.ffn_step(pc, X0, T, W["Lw"], W.get("Cw"), W.get("Dw"), W["bias"],
                Lw_master=M.get("Lw"), Cw_master=M.get("Cw"), Dw_master=M.get("Dw"), bias_master=M.get("bias"),
                G=G, dg_own=dg, dLw=Gd.get("Lw"), dCw=Gd.get("Cw"), dDw=Gd.get("Dw"), dbias=Gd.get("bias"),
                Y_out=Y_out, loss=loss, lr=lr, mode=mode, workspace=ws)
    torch.cuda.synchronize()
    return data, ref, W, M, Gd, Y_out, float(loss[0])


def check_step(prob, data, ref, W, M, Gd, Y_out, loss, lr, grad_tol=None):
    dt = prob.dtype
    names = list(W.keys())
    assert_close("Y_L", Y_out, ref["forward"]["Y"][-1], dt)
    assert abs(loss - ref["loss"]) <= (1e-5 if dt == "f32" else 2e-2) * abs(ref["loss"]), (loss, ref["loss"])
    for l in range(prob.layers):
        for nm in names:
            assert_close(f"d{nm}[{l}]", Gd[nm][l], ref["grads"][l]["d" + nm], dt, grad_tol)
            new = ref["layers"][l][nm]
            if dt == "bf16":
                # the update itself: master_new = master_old - lr * (the gradient the GPU reports), in fp32
                old = torch.from_numpy(data["layers"][l][nm].astype(np.float32)).cuda()
                want = old - lr * Gd[nm][l]
                ulp = torch.finfo(torch.float32).eps * (old.abs() + (lr * Gd[nm][l]).abs())
                assert bool(((M[nm][l] - want).abs() <= 2 * ulp).all()), f"{nm}_master[{l}] update"
                assert_close(f"{nm}_master[{l}]", M[nm][l], new, dt)
                # compute copy = master rounded to bfloat16
                assert torch.equal(W[nm][l], M[nm][l].to(torch.bfloat16))
            else:
                assert_close(f"{nm}[{l}]", W[nm][l], new, dt)


def test_step_tiny_fp32_all_ranks():
    """benchmark configuration 1: n=256, p=4 (shard 64), k=8, batch 32, 2 layers, ReLU, MSE, SGD lr=1e-2."""
    prob = pin.Problem(n=256, p=4, k=8, batch=32, layers=2, act="relu", dtype="f32", rank=-1)
    data, ref, W, M, Gd, Y_out, loss = run_step(prob, seed=0, lr=1e-2)
    # no pre-activation of this seed sits within fp32 rounding of the ReLU kink (oracle-side check)
    assert relu_margin(ref["forward"]) > 1e-5
    check_step(prob, data, ref, W, M, Gd, Y_out, loss, 1e-2)


@pytest.mark.parametrize("n,p,k,B,L,act,dtype,rank", [
    (288, 4, 5, 37, 3, "gelu", "f32", -1),
    (288, 4, 5, 37, 2, "identity", "f32", 2),
    (96, 1, 0, 21, 2, "gelu", "f32", -1),
    (1024, 8, 16, 136, 3, "gelu", "bf16", -1),
    (792, 6, 10, 70, 2, "identity", "bf16", 3),
    (2048, 16, 32, 200, 4, "gelu", "bf16", 0),
    (2048, 16, 8, 136, 2, "gelu", "bf16", -1),
    (2048, 32, 4, 72, 2, "gelu", "bf16", -1),
])
def test_step_smooth_activations(n, p, k, B, L, act, dtype, rank):
    print(f"case step n={n} p={p} k={k} B={B} L={L} {act} {dtype} rank={rank}", flush=True)
    prob = pin.Problem(n=n, p=p, k=k, batch=B, layers=L, act=act, dtype=dtype, rank=rank)
    out = run_step(prob, seed=3, lr=0.05)
    check_step(prob, *out, 0.05)


@pytest.mark.parametrize("n,p,k,B,L,act,rank", [
    (2048, 8, 32, 4100, 2, "gelu", 0),       # one rank, long batch
    (1024, 8, 16, 136, 3, "gelu", -1),       # all ranks on the device
])
def test_step_without_gradient_outputs(n, p, k, B, L, act, rank):
    """A training step that is not asked for its gradients keeps them in the workspace: what the update
    moved the master weights by against the oracle's gradients, the bf16 copies against the masters.
    The workspace starts out full of NaN patterns, and is used for a second call as the first one left it."""
    print(f"case step/no grads n={n} p={p} k={k} B={B} L={L} {act} rank={rank}", flush=True)
    prob = pin.Problem(n=n, p=p, k=k, batch=B, layers=L, act=act, dtype="bf16", rank=rank)
    lr = 0.05
    ws = workspace(ph.workspace_bytes(_prob_c(prob)))
    ws.fill_(0xFF)                            # whatever the step expects to be zero, it has to clear itself
    for call in ("first call", "second call, same workspace"):
        data, ref, W, M, _, Y_out, loss = run_step(prob, seed=5, lr=lr, with_grads=False, ws=ws)
        assert_close("Y_L", Y_out, ref["forward"]["Y"][-1], "bf16")
        assert abs(loss - ref["loss"]) <= 2e-2 * abs(ref["loss"]), call
        for l in range(L):
            for nm in W:
                old = data["layers"][l][nm].astype(np.float32).astype(np.float64)
                # the step moved the master weight by -lr * gradient: compare the movement with the oracle's gradient
                moved = (M[nm][l].double().cpu().numpy() - old) / -lr
                assert_close(f"d{nm}[{l}] (from the update, {call})", torch.from_numpy(moved), ref["grads"][l]["d" + nm], "bf16")
                assert torch.equal(W[nm][l], M[nm][l].to(torch.bfloat16))


@pytest.mark.parametrize("widths,ks,p,B,act,dtype,rank", [
    ((288, 160, 96, 224), (5, 3, 7), 4, 37, "gelu", "f32", -1),
    ((288, 160, 96), (5, 3), 4, 37, "identity", "f32", 2),
    ((1024, 2048, 512, 1024), (16, 32, 8), 8, 136, "gelu", "bf16", -1),     # all ranks: thin compression, fused output error, riders
    ((2048, 1024, 3072), (32, 16), 16, 200, "gelu", "bf16", 0),             # one rank
    ((1032, 520, 1032), (6, 2), 4, 70, "identity", "bf16", 3),              # 4-byte vectors
    ((1056, 528, 1056), (24, 8), 8, 72, "gelu", "bf16", -1),                # shards 132, 66, 132: 4-byte vectors in the middle
])
def test_step_layers_of_different_widths(widths, ks, p, B, act, dtype, rank):
    """Section IV, first paragraph: widths n_l and phantom widths k_l per layer."""
    print(f"case step widths={widths} ks={ks} p={p} B={B} {act} {dtype} rank={rank}", flush=True)
    prob = pin.Problem(n=widths[0], p=p, k=ks[0], batch=B, layers=len(ks), act=act, dtype=dtype, rank=rank,
                       widths=widths, ks=ks)
    out = run_step(prob, seed=4, lr=0.05)
    check_step(prob, *out, 0.05)


@pytest.mark.parametrize("n,p,k,B,L,dtype,rank", [
    (2048, 16, 16, 300, 2, "bf16", 3),       # one rank: nothing but the weight-gradient launch can finish the loss
    (1024, 8, 16, 136, 2, "bf16", -1),       # all ranks: the reduce-scatter does
    (512, 1, 0, 200, 2, "bf16", 0),          # a dense stack
    (288, 4, 5, 37, 2, "f32", 1),
])
def test_step_without_update(n, p, k, B, L, dtype, rank):
    """mode no_update: loss and gradients as in a training step, the weights left as they were."""
    print(f"case step/no update n={n} p={p} k={k} B={B} L={L} {dtype} rank={rank}", flush=True)
    prob = pin.Problem(n=n, p=p, k=k, batch=B, layers=L, act="gelu", dtype=dtype, rank=rank)
    data, ref, W, M, Gd, Y_out, loss = run_step(prob, seed=6, lr=0.05, mode="no_update")
    assert_close("Y_L", Y_out, ref["forward"]["Y"][-1], dtype)
    assert abs(loss - ref["loss"]) <= (1e-5 if dtype == "f32" else 2e-2) * abs(ref["loss"]), (loss, ref["loss"])
    for l in range(L):
        for nm in W:
            assert_close(f"d{nm}[{l}]", Gd[nm][l], ref["grads"][l]["d" + nm], dtype)
            assert torch.equal(W[nm][l], to_gpu(data["layers"][l][nm], dtype)), f"{nm}[{l}] changed"


def test_training_several_steps_fp32():
    """Five SGD steps in a row (weights updated in place by one call feed the next) against the oracle
    taking the same five steps: the loss of every step and the final weights."""
    prob = pin.Problem(n=256, p=4, k=8, batch=40, layers=2, act="gelu", dtype="f32", rank=-1)
    lr, steps = 0.05, 5
    data = pin.all_rank_step_inputs(prob, seed=7)
    layers = [dict(P) for P in data["layers"]]
    want_loss = []
    for _ in range(steps):
        ref = oracle.ffn_step("gelu", data["X0"], data["T"], layers, lr, storage="f32", all_ranks=True)
        want_loss.append(ref["loss"])
        layers = ref["layers"]
    pc = _prob_c(prob)
    ws = workspace(ph.workspace_bytes(pc))
    names = ("Lw", "Cw", "Dw", "bias")
    W = {nm: [to_gpu(P[nm], "f32") for P in data["layers"]] for nm in names}
    X0, T = to_gpu(data["X0"], "f32"), to_gpu(data["T"], "f32")
    loss = empty_f32((4,))
    got_loss = []
    for _ in range(steps):
        ph.ffn_step(pc, X0, T, W["Lw"], W["Cw"], W["Dw"], W["bias"], loss=loss, lr=lr, workspace=ws)
        torch.cuda.synchronize()
        got_loss.append(float(loss[0]))
    assert want_loss[-1] < want_loss[0]                       # the oracle's own loss goes down
    for g, w in zip(got_loss, want_loss):
        assert abs(g - w) <= 1e-5 * abs(w), (got_loss, want_loss)
    for l in range(prob.layers):
        for nm in names:
            assert_close(f"{nm}[{l}] after {steps} steps", W[nm][l], layers[l][nm], "f32", 5e-5)


def test_step_forward_only():
    prob = pin.Problem(n=1024, p=8, k=16, batch=100, layers=3, act="relu", dtype="bf16", rank=0)
    data = pin.one_rank_step_inputs(prob, seed=4)
    fw = oracle.ffn_forward("relu", data["X0"], data["layers"], "bf16", all_ranks=False)
    pc = _prob_c(prob)
    ws = workspace(ph.workspace_bytes(pc))
    W = {nm: [to_gpu(P[nm], "bf16") for P in data["layers"]] for nm in ("Lw", "Cw", "Dw", "bias")}
    G = [to_gpu(P["G"], "bf16") for P in data["layers"]]
    Y_out = empty(data["X0"].shape, "bf16")
    ph.ffn_step(pc, to_gpu(data["X0"], "bf16"), None, W["Lw"], W["Cw"], W["Dw"], W["bias"], G=G, Y_out=Y_out,
                mode="forward", workspace=ws)
    torch.cuda.synchronize()
    assert_close("Y_L", Y_out, fw["Y"][-1], "bf16")


def test_binding_refuses_short_and_mistyped_tensors():
    """A buffer shorter than the problem's shape, of the wrong element size or not contiguous never reaches the library."""
    prob = ph.make_problem(256, 4, 8, 32, dtype="bf16")
    B, s, k, q = 32, 64, 8, 3
    X, Lw, Cw, Dw = empty((B, s), "bf16"), empty((s, s), "bf16"), empty((k, s), "bf16"), empty((q, s, k), "bf16")
    bias, G, Y, g_own = empty((s,), "bf16"), empty((q, B, k), "bf16"), empty((B, s), "bf16"), empty((B, k), "bf16")
    ws = workspace(ph.workspace_bytes(prob))
    with pytest.raises(ValueError, match="Y: 1984 elements, the problem needs 2048"):
        ph.layer_fwd(prob, X, Lw, Cw, Dw, bias, G, empty((B - 1, s), "bf16"), g_own, None, ws)
    with pytest.raises(ValueError, match="Lw: elements of 4 bytes, 2 expected"):
        ph.layer_fwd(prob, X, empty((s, s), "f32"), Cw, Dw, bias, G, Y, g_own, None, ws)
    with pytest.raises(ValueError, match="X: tensor is not contiguous"):
        ph.layer_fwd(prob, empty((s, B), "bf16").t(), Lw, Cw, Dw, bias, G, Y, g_own, None, ws)
    with pytest.raises(ValueError, match=r"dLw\[1\]: elements of 2 bytes, 4 expected"):
        two = ph.make_problem(256, 4, 8, 32, layers=2, dtype="bf16")
        ph.ffn_step(two, X, Y, [Lw, Lw], [Cw, Cw], [Dw, Dw], [bias, bias], G=[G, G], dg_own=[g_own, g_own],
                    dLw=[empty_f32((s, s)), Lw], mode="no_update", workspace=ws)
