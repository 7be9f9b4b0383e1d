"""Pins of the CPU oracle against things other than itself (no GPU needed).

What each pin fixes is stated in its docstring.  The independent side is always
one of: a dense layer computed with library matrix products and torch's
autograd (the phantom model is a dense model with structured off-diagonal
blocks, Section III-A / Eq. (ylq)); central finite differences; numbers the
paper prints (Table 1); library conversions (torch bfloat16, torch GELU).
"""
import math
import os

import numpy as np
import pytest
import torch

import phantom_inputs as pin
from oracle import oracle

torch.set_num_threads(4)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------------------
# helpers: the dense model that a phantom model is equal to, in torch fp64
# ----------------------------------------------------------------------------

def _t(a, grad=False):
    return torch.tensor(np.asarray(a), dtype=torch.float64, requires_grad=grad)


def _act_torch(act, a):
    if act == "relu":
        return torch.relu(a)
    if act == "gelu":
        return torch.nn.functional.gelu(a)          # exact erf form
    return a


def _dense_weight(Lw, Cw, Dw):
    """n x n matrix with block (j, j) = L^(j) and block (j, i) = D^(i,j) C^(i), i != j.
    Lw [p,s,s], Cw [p,k,s], Dw [p,p-1,s,k] (peer slots in increasing i, skipping j)."""
    p, s, _ = Lw.shape
    rows = []
    for j in range(p):
        blocks = []
        for i in range(p):
            if i == j:
                blocks.append(Lw[j])
            else:
                slot = i if i < j else i - 1
                blocks.append(Dw[j, slot] @ Cw[i])
        rows.append(torch.cat(blocks, dim=1))
    return torch.cat(rows, dim=0)


def _dense_reference(act, X0, T, layers, lr):
    """Loss, parameter gradients (autograd) and SGD-updated parameters of the dense-equivalent
    network.  X0, T: [p,B,s] shards; layers: stacked numpy weights per layer."""
    p, B, _ = X0.shape
    x = _t(X0).permute(1, 0, 2).reshape(B, -1)
    t = _t(T).permute(1, 0, 2).reshape(B, -1)
    leaves = []
    for P in layers:
        leaf = {name: _t(P[name], grad=True) for name in ("Lw", "Cw", "Dw", "bias") if P.get(name) is not None}
        leaves.append(leaf)
        if p > 1:
            W = _dense_weight(leaf["Lw"], leaf["Cw"], leaf["Dw"])
        else:
            W = leaf["Lw"][0]
        x = _act_torch(act, x @ W.T + leaf["bias"].reshape(-1))
    loss = 0.5 * torch.sum((x - t) ** 2) / B
    loss.backward()
    grads = [{name: v.grad.numpy() for name, v in leaf.items()} for leaf in leaves]
    y = x.detach().numpy().reshape(B, p, -1).transpose(1, 0, 2)
    return float(loss), grads, y


def _problem(n, p, k, B, L, act, widths=(), ks=()):
    return pin.Problem(n=n, p=p, k=k, batch=B, layers=L, act=act, dtype="f32", rank=-1, widths=widths, ks=ks)


def _close(a, b, tol=1e-11):
    a = np.asarray(a); b = np.asarray(b)
    scale = max(float(np.sqrt(np.mean(b * b))), 1e-300)
    assert a.shape == b.shape
    assert float(np.max(np.abs(a - b))) <= tol * scale, (float(np.max(np.abs(a - b))), scale)


# ----------------------------------------------------------------------------
# P1: p = 1 is a textbook dense layer
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("act", ["identity", "relu", "gelu"])
def test_p1_is_dense_layer(act):
    """With one rank there is no C, D or G: y = sigma(W x + b).  Pins the local update, the bias,
    the activation and its derivative, the loss scale and the SGD sign against torch autograd."""
    prob = _problem(n=24, p=1, k=1, B=7, L=2, act=act)
    data = pin.all_rank_step_inputs(prob, seed=3)
    layers = [{"Lw": P["Lw"], "bias": P["bias"], "Cw": None, "Dw": None} for P in data["layers"]]
    got = oracle.ffn_step(act, data["X0"], data["T"], layers, lr=0.05, storage="f32", all_ranks=True)
    loss, grads, y = _dense_reference(act, data["X0"], data["T"], layers, lr=0.05)
    assert abs(got["loss"] - loss) <= 1e-12 * abs(loss)
    _close(got["forward"]["out"], y)
    for l in range(prob.layers):
        _close(got["grads"][l]["dLw"], grads[l]["Lw"])
        _close(got["grads"][l]["dbias"], grads[l]["bias"])
        _close(got["layers"][l]["Lw"], layers[l]["Lw"] - 0.05 * grads[l]["Lw"])
        _close(got["layers"][l]["bias"], layers[l]["bias"] - 0.05 * grads[l]["bias"])


# ----------------------------------------------------------------------------
# P2: dense equivalence for any k, all ranks, several layers
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("n,p,k,B,L,act,widths,ks", [
    (12, 3, 2, 5, 2, "gelu", (), ()),
    (12, 3, 2, 5, 3, "relu", (), ()),
    (20, 4, 3, 6, 2, "identity", (), ()),
    (16, 2, 8, 4, 2, "relu", (), ()),        # k = s
    (30, 5, 1, 3, 1, "gelu", (), ()),        # a single ghost neuron
    # layers of different widths and phantom widths (Section IV, first paragraph): 12 -> 21 -> 6 -> 15 over 3 ranks
    (12, 3, 2, 5, 3, "gelu", (12, 21, 6, 15), (2, 3, 1)),
    (8, 2, 1, 4, 2, "relu", (8, 20, 4), (4, 2)),
])
def test_phantom_equals_structured_dense(n, p, k, B, L, act, widths, ks):
    check_structured_dense(n, p, k, B, L, act, widths, ks)


def check_structured_dense(n, p, k, B, L, act, widths=(), ks=()):
    """The phantom model is the dense model whose off-diagonal block (j,i) is D^(i,j) C^(i).
    torch autograd through that dense model gives the gradients of L, C, D and b directly.
    Pins: which D goes with which peer and which slot, that C^(i) is shared by all destinations,
    the gather and reduce-scatter index maps, the shapes of dD, the chaining over layers."""
    prob = _problem(n, p, k, B, L, act, widths, ks)
    data = pin.all_rank_step_inputs(prob, seed=11)
    got = oracle.ffn_step(act, data["X0"], data["T"], data["layers"], lr=0.01, storage="f32", all_ranks=True)
    loss, grads, y = _dense_reference(act, data["X0"], data["T"], data["layers"], lr=0.01)
    assert abs(got["loss"] - loss) <= 1e-12 * abs(loss)
    _close(got["forward"]["out"], y)
    for l in range(L):
        for name in ("Lw", "Cw", "Dw", "bias"):
            _close(got["grads"][l]["d" + name], grads[l][name])
            _close(got["layers"][l][name], data["layers"][l][name] - 0.01 * grads[l][name])


def test_identity_compressor_reproduces_dense_layer():
    """k = s, C^(i) = I and D^(i,j) = W_ji: the phantom layer IS the dense layer W."""
    p, s, B = 3, 4, 6
    n = p * s
    W = pin.normal((n, n), seed=5, tensor="W_dense")
    b = pin.normal((n,), seed=5, tensor="bias")
    X = pin.normal((B, n), seed=5, tensor="X")
    P = {"Lw": np.stack([W[j*s:(j+1)*s, j*s:(j+1)*s] for j in range(p)]),
         "Cw": np.stack([np.eye(s)] * p),
         "Dw": np.stack([np.stack([W[j*s:(j+1)*s, i*s:(i+1)*s] for i in range(p) if i != j]) for j in range(p)]),
         "bias": b.reshape(p, s)}
    r = oracle.all_ranks_fwd("relu", pin.shard_columns(X, p), P)
    want = np.maximum(X @ W.T + b, 0.0)
    _close(r["Y"], pin.shard_columns(want, p))


# ----------------------------------------------------------------------------
# P3: the emulation boundary: one rank fed with the buffers of an all-ranks run
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("storage,widths", [("f32", ()), ("bf16", ()), ("f32", (24, 40))])
def test_one_rank_reproduces_its_share_of_all_ranks(storage, widths):
    check_one_rank_vs_all_ranks(storage, widths)


def check_one_rank_vs_all_ranks(storage, widths=()):
    """Feeding rank j the gathered buffer (minus its slot) and its reduce-scatter result from an
    all-ranks run reproduces that rank's outputs exactly (same code, same order of sums)."""
    prob = pin.Problem(n=24, p=4, k=3, batch=5, layers=1, act="gelu", dtype=storage, rank=-1, widths=widths,
                       ks=(3,) if widths else ())
    P = pin.all_rank_params(prob, 0, seed=2)
    X0, T = pin.network_io(prob, seed=2)
    X = pin.shard_columns(X0, prob.p)
    dY = pin.shard_columns(pin.round_to_storage(T / prob.batch, storage), prob.p)
    fw = oracle.all_ranks_fwd("gelu", X, P, storage)
    bw = oracle.all_ranks_bwd("gelu", dY, X, fw["A"], P, fw["G_full"], storage)
    for j in range(prob.p):
        G = oracle.without_slot(fw["G_full"], j)
        f1 = oracle.layer_fwd("gelu", X[j], P["Lw"][j], P["Cw"][j], P["Dw"][j], P["bias"][j], G)
        assert np.array_equal(f1["Y"], fw["Y"][j]) and np.array_equal(f1["A"], fw["A"][j])
        assert np.array_equal(oracle.rd(f1["g_own"], storage), fw["G_full"][j])
        b1 = oracle.layer_bwd("gelu", dY[j], X[j], fw["A"][j], P["Lw"][j], P["Cw"][j], P["Dw"][j], G,
                              bw["dg_own"][j], storage)
        for name in ("dX", "dLw", "dCw", "dDw", "dbias"):
            assert np.array_equal(b1[name], bw[name][j]), name
        assert np.array_equal(oracle.rd(b1["dG_send"], storage), bw["dG_send"][j])


# ----------------------------------------------------------------------------
# P4: Table 1's model sizes
# ----------------------------------------------------------------------------

def test_parameter_count_matches_table_1():
    """One C per rank (not per peer), p-1 D's per rank, one bias per rank: L*(n^2/p + p*n*k + n)
    parameters; the dense (tensor-parallel) model has L*(n^2 + n).  Table 1 prints both in millions."""
    rows = [line.split() for line in open(os.path.join(GOLDEN, "table1_model_size.txt"))
            if line.strip() and not line.startswith("#")]
    assert len(rows) == 6
    for n, L, p, k, tp_m, pp_m in (map(int, r) for r in rows):
        count = oracle.param_count(n, p, k, L)
        assert count == L * (n * n // p + p * n * k + n)
        assert round(count / 1e6) == pp_m, (p, k, count)
        assert round(oracle.param_count(n, 1, 0, L) / 1e6) == tp_m
    # the shapes the count is made from are the shapes the generator and the oracle use
    prob = pin.Problem(n=32, p=4, k=3, batch=2, rank=0)
    got = {name: v.shape for name, v in pin.layer_params(prob, 0, 0, seed=0).items()}
    assert got == oracle.param_shapes(32, 4, 3)


# ----------------------------------------------------------------------------
# P5: finite differences (does not rely on torch)
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("act,widths,ks", [("gelu", (), ()), ("identity", (), ()), ("gelu", (12, 18, 6), (2, 3))])
def test_gradients_match_central_differences(act, widths, ks):
    check_central_differences(act, widths, ks)


def check_central_differences(act, widths=(), ks=()):
    """Central differences of the oracle's own forward + loss, for every parameter tensor of every
    layer and for the network input.  Pins the whole backward, incl. multi-layer chaining."""
    prob = _problem(n=12, p=3, k=2, B=3, L=2, act=act, widths=widths, ks=ks)
    data = pin.all_rank_step_inputs(prob, seed=7)
    layers = data["layers"]

    def loss_of(layers_, X0_):
        fw = oracle.ffn_forward(act, X0_, layers_, "f32", True)
        return oracle.mse_loss(fw["out"], data["T"])[0]

    step = oracle.ffn_step(act, data["X0"], data["T"], layers, lr=0.0)
    h = 1e-6
    rng = np.random.default_rng(0)
    for l in range(prob.layers):
        for name in ("Lw", "Cw", "Dw", "bias"):
            g = step["grads"][l]["d" + name]
            flat = rng.permutation(g.size)[: min(g.size, 40)]
            for idx in flat:
                pos = np.unravel_index(idx, g.shape)
                vals = []
                for sign in (+1, -1):
                    mod = [dict(P) for P in layers]
                    w = layers[l][name].copy(); w[pos] += sign * h
                    mod[l][name] = w
                    vals.append(loss_of(mod, data["X0"]))
                fd = (vals[0] - vals[1]) / (2 * h)
                assert abs(fd - g[pos]) <= 1e-7 * max(1.0, abs(g[pos])) + 2e-9, (l, name, pos, fd, g[pos])
    # input gradient: dX of layer 0 is not returned by ffn_step (not needed); ask for it directly
    fw = step["forward"]
    _, dY = oracle.mse_loss(fw["out"], data["T"])
    g1 = oracle.all_ranks_bwd(act, dY, fw["X"][1], fw["A"][1], layers[1], fw["G"][1])
    g0 = oracle.all_ranks_bwd(act, g1["dX"], fw["X"][0], fw["A"][0], layers[0], fw["G"][0])
    for idx in range(0, data["X0"].size, 5):
        pos = np.unravel_index(idx, data["X0"].shape)
        vals = []
        for sign in (+1, -1):
            x = data["X0"].copy(); x[pos] += sign * h
            vals.append(loss_of(layers, x))
        fd = (vals[0] - vals[1]) / (2 * h)
        assert abs(fd - g0["dX"][pos]) <= 1e-7 * max(1.0, abs(fd)) + 2e-9


# ----------------------------------------------------------------------------
# P6: the one-GEMM view (concatenation order of peers)
# ----------------------------------------------------------------------------

def test_concatenated_operands_give_the_same_layer():
    """A = [X | G_1 | ... ] [Lw | Dw_1 | ...]^T + b and the dense-layer backward on the concatenated
    operands agree with the per-peer sums (library matmul on one side, loops on the other)."""
    prob = pin.Problem(n=40, p=5, k=3, batch=9, act="gelu", dtype="f32", rank=2)
    d = pin.one_rank_layer_inputs(prob, 0, seed=4)
    q, s, k, B = prob.peers, prob.s, prob.k, prob.batch
    f = oracle.layer_fwd("gelu", d["X"], d["Lw"], d["Cw"], d["Dw"], d["bias"], d["G"])
    Xcat = np.concatenate([d["X"]] + [d["G"][i] for i in range(q)], axis=1)
    Wcat = np.concatenate([d["Lw"]] + [d["Dw"][i] for i in range(q)], axis=1)
    _close(f["A"], Xcat @ Wcat.T + d["bias"])
    _close(f["g_own"], d["X"] @ d["Cw"].T)
    b = oracle.layer_bwd("gelu", d["dY"], d["X"], f["A"], d["Lw"], d["Cw"], d["Dw"], d["G"], d["dg_own"])
    a_t = _t(f["A"], grad=True)
    torch.nn.functional.gelu(a_t).backward(_t(d["dY"]))
    delta = a_t.grad.numpy()
    _close(b["delta"], delta)
    dWcat = delta.T @ Xcat
    U = delta @ Wcat
    _close(b["dLw"], dWcat[:, :s])
    for i in range(q):
        _close(b["dDw"][i], dWcat[:, s + i * k: s + (i + 1) * k])
        _close(b["dG_send"][i], U[:, s + i * k: s + (i + 1) * k])
    _close(b["dX"], U[:, :s] + d["dg_own"] @ d["Cw"])
    _close(b["dCw"], d["dg_own"].T @ d["X"])
    _close(b["dbias"], delta.sum(axis=0))


# ----------------------------------------------------------------------------
# P7: operation counts (roofline numerator)
# ----------------------------------------------------------------------------

def test_mac_counts_by_brute_force():
    """Count one multiply-add per term of every sum of Eq. (ylq), (backprop), (bpL)-(bpD) with
    explicit loops; fwd + bwd = 3*B*s*(s + p*k), i.e. 6*B*s*(s+p*k) FLOP, which is the paper's
    O(n^2/p^2 + k n) per rank per layer."""
    n, p, k, B = 12, 3, 2, 4
    s, q = n // p, p - 1
    fwd = 0
    for b in range(B):
        for c in range(k):
            for m in range(s): fwd += 1                      # g = C y
        for o in range(s):
            for m in range(s): fwd += 1                      # L y
            for i in range(q):
                for c in range(k): fwd += 1                  # D g
    bwd = 0
    for b in range(B):
        for i in range(q):
            for c in range(k):
                for o in range(s): bwd += 1                  # D^T delta
        for m in range(s):
            for o in range(s): bwd += 1                      # L^T delta
            for c in range(k): bwd += 1                      # C^T dg
        for o in range(s):
            for m in range(s): bwd += 1                      # dL
            for i in range(q):
                for c in range(k): bwd += 1                  # dD
        for c in range(k):
            for m in range(s): bwd += 1                      # dC
    assert (fwd, bwd) == oracle.mac_counts(n, p, k, B)
    assert fwd == B * s * (s + p * k) and bwd == 2 * fwd
    assert 2 * (fwd + bwd) == 6 * B * s * (s + p * k)


# ----------------------------------------------------------------------------
# library pins of the two scalar functions
# ----------------------------------------------------------------------------

def test_bf16_rounding_matches_torch():
    """Nearest-even rounding to bfloat16 against torch's conversion, incl. exact ties."""
    vals = np.concatenate([
        pin.normal((4096,), seed=1, tensor="aux").astype(np.float32).astype(np.float64),
        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, 2.0 ** -20 * 1.00390625, 3.0, 255.5, 256.5 * 2]),
    ])
    want = torch.tensor(vals, dtype=torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(oracle.round_bf16(vals), want)
    assert np.array_equal(pin.round_to_storage(vals, "bf16"), want)


def test_sigma_prime_factor_of_a_bf16_step_is_unrounded():
    """Eq. (deltaL) / Eq. (backprop) multiply by sigma'(b + z) as it is: in a bfloat16-storage step the only
    rounding in delta_{l-1} is the one of the finished product, and the sigma' factor is torch's GELU
    derivative of the unrounded pre-activation (fp64), not a value on any coarser grid."""
    prob = pin.Problem(n=16, p=2, k=3, batch=4, layers=2, act="gelu", dtype="bf16", rank=-1)
    data = pin.all_rank_step_inputs(prob, seed=9)
    st = oracle.ffn_step("gelu", data["X0"], data["T"], data["layers"], lr=0.01, storage="bf16")
    A, dX = st["forward"]["A"][0], st["grads"][1]["dX"]
    at = _t(A, grad=True)
    torch.nn.functional.gelu(at).backward(torch.ones_like(at))
    want = oracle.round_bf16(dX * at.grad.numpy())
    got = st["grads"][0]["delta"]
    # the two evaluations of erf differ in the last bits of fp64: a product that lands within 1e-13 of a
    # bfloat16 tie could round either way; everything else is identical
    assert np.mean(got == want) > 0.99 and np.abs(got - want).max() <= 2.0 ** -7 * np.abs(want).max()
    assert not np.array_equal(A, oracle.round_bf16(A))


def test_gelu_and_its_derivative_match_torch():
    a = np.linspace(-6, 6, 241).reshape(1, -1)
    ones = np.ones_like(a)
    f = oracle.layer_update("gelu", a, np.eye(a.shape[1]), None, np.zeros(a.shape[1]), None)[1]
    at = _t(a, grad=True)
    y = torch.nn.functional.gelu(at)
    y.backward(torch.ones_like(y))
    _close(f, y.detach().numpy(), 1e-14)
    _close(oracle.delta_of("gelu", ones, a), at.grad.numpy(), 1e-13)
    # ReLU'(0) = 0
    assert oracle.delta_of("relu", np.ones((1, 3)), np.array([[-1.0, 0.0, 2.0]])).tolist() == [[0.0, 0.0, 1.0]]


def test_bf16_storage_rounds_operands_and_messages_only():
    """Storage type bfloat16: layer inputs, delta and the tensors that cross ranks sit on the bfloat16
    grid; gradients of weights are left unrounded."""
    prob = pin.Problem(n=16, p=2, k=3, batch=4, layers=2, act="gelu", dtype="bf16", rank=-1)
    data = pin.all_rank_step_inputs(prob, seed=9)
    st = oracle.ffn_step("gelu", data["X0"], data["T"], data["layers"], lr=0.01, storage="bf16")
    on_grid = lambda a: np.array_equal(a, oracle.round_bf16(a))
    fw = st["forward"]
    assert all(on_grid(x) for x in fw["X"]) and all(on_grid(g) for g in fw["G"])
    assert all(on_grid(g["delta"]) and on_grid(g["dG_send"]) and on_grid(g["dg_own"]) for g in st["grads"])
    assert not on_grid(st["grads"][0]["dLw"]) and not on_grid(fw["A"][0])


def test_generator_is_counter_based_and_seeded():
    a = pin.normal((5, 7), seed=1, tensor="X", layer=2, rank=3)
    b = pin.normal((35,), seed=1, tensor="X", layer=2, rank=3)
    assert np.array_equal(a.ravel(), b)
    assert not np.array_equal(a, pin.normal((5, 7), seed=2, tensor="X", layer=2, rank=3))
    assert not np.array_equal(a, pin.normal((5, 7), seed=1, tensor="X", layer=2, rank=4))
    big = pin.normal((200000,), seed=0, tensor="G")
    assert abs(big.mean()) < 0.01 and abs(big.std() - 1) < 0.01
    u = pin.uniform((200000,), -0.5, 0.5, seed=0, tensor="Lw")
    assert u.min() >= -0.5 and u.max() <= 0.5 and abs(u.std() - math.sqrt(1 / 12)) < 0.01
