"""phantom_ffn_step under HIP graph capture: every replay must do what the eager call does.

bench.py times replays of one captured step, so the step's launches (riders, fill kernels, deferred SGD) have to
survive capture.  A graph is replayed several times with unrelated eager work and synchronisations in between,
and each replay is checked against the same step run eagerly from the same state.  The bf16 path adds column
sums and loss partials with float atomics, whose order differs from run to run: replay and eager run agree to
rounding, not bit for bit, so the bound is a small multiple of the storage type's rounding.
"""
import pytest
import torch

import paper_2508_00960_amd as ph
import phantom_inputs as pin

from helpers import empty, empty_f32, to_gpu, to_gpu_f32, workspace

pytestmark = pytest.mark.gpu


class State:
    """Device tensors of one training run and a closure that launches one step on them."""

    def __init__(self, prob, data, lr, mode):
        dt, q = prob.dtype, prob.peers
        one_rank = prob.rank >= 0
        self.pc = ph.make_problem(prob.n, prob.p, prob.k, prob.batch, prob.layers, prob.act, prob.dtype, prob.rank)
        self.ws = workspace(ph.workspace_bytes(self.pc))
        names = ["Lw", "bias"] + (["Cw", "Dw"] if q else [])
        self.W = {nm: [to_gpu(P[nm], dt) for P in data["layers"]] for nm in names}
        self.M = {nm: [to_gpu_f32(P[nm]) for P in data["layers"]] for nm in names} if dt == "bf16" else {}
        self.Gd = {nm: [empty_f32(P[nm].shape) for P in data["layers"]] for nm in names}
        self.G = [to_gpu(P["G"], dt) for P in data["layers"]] if (q and one_rank) else None
        self.dg = [to_gpu(P["dg_own"], dt) for P in data["layers"]] if (q and one_rank) else None
        self.X0, self.T = to_gpu(data["X0"], dt), to_gpu(data["T"], dt)
        self.Y = empty(data["T"].shape, dt)
        self.loss = empty_f32((4,))
        self.lr, self.mode = lr, mode

    def step(self):
        W, M, Gd = self.W, self.M, self.Gd
        ph.ffn_step(self.pc, self.X0, self.T, W["Lw"], W.get("Cw"), W.get("Dw"), W["bias"],
                    Lw_master=M.get("Lw"), Cw_master=M.get("Cw"), Dw_master=M.get("Dw"), bias_master=M.get("bias"),
                    G=self.G, dg_own=self.dg, dLw=Gd["Lw"], dCw=Gd.get("Cw"), dDw=Gd.get("Dw"), dbias=Gd["bias"],
                    Y_out=self.Y, loss=self.loss, lr=self.lr, mode=self.mode, workspace=self.ws)

    def snapshot(self):
        torch.cuda.synchronize()
        out = {"loss": self.loss[:1].clone(), "Y": self.Y.float().clone()}
        for nm, per_layer in self.Gd.items():
            for l, t in enumerate(per_layer):
                out[f"d{nm}[{l}]"] = t.clone()
        for nm, per_layer in (self.M or self.W).items():
            for l, t in enumerate(per_layer):
                out[f"{nm}[{l}]"] = t.float().clone()
        return out


def assert_same(what, got, want, tol):
    for name, ref in want.items():
        scale = max(float(ref.abs().max()), 1e-30)
        err = float((got[name] - ref).abs().max()) / scale
        assert err <= tol, f"{what}: {name} differs by {err:.3e} of its largest magnitude (bound {tol:.1e})"


@pytest.mark.parametrize("n,p,k,B,L,act,dtype,rank,mode", [
    (1024, 8, 32, 256, 3, "relu", "bf16", -1, "train"),       # all ranks: riders on the weight-gradient launches
    (1024, 8, 32, 256, 3, "relu", "bf16", -1, "no_update"),
    (2048, 16, 32, 384, 3, "gelu", "bf16", 0, "train"),        # one rank: forward pair, deferred SGD
    (2048, 16, 32, 2304, 2, "gelu", "bf16", 0, "train"),       # one rank, long batch: weight gradients in pieces, SGD in their epilogues
    (288, 4, 5, 37, 2, "gelu", "f32", -1, "train"),            # fp32 kernels
])
def test_graph_replays_match_eager_steps(n, p, k, B, L, act, dtype, rank, mode):
    print(f"case graph n={n} p={p} k={k} B={B} L={L} {act} {dtype} rank={rank} {mode}", flush=True)
    prob = pin.Problem(n=n, p=p, k=k, batch=B, layers=L, act=act, dtype=dtype, rank=rank)
    data = pin.all_rank_step_inputs(prob, 11) if rank < 0 else pin.one_rank_step_inputs(prob, 11)
    tol = 1e-6 if dtype == "f32" else 4e-3
    replays = 4
    lr = 2e-4       # the loss sums over the outputs: steps of 1 / (layer width) or more diverge

    eager = State(prob, data, lr, mode)
    want = []
    for _ in range(replays):
        eager.step()
        want.append(eager.snapshot())

    captured = State(prob, data, lr, mode)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        captured.step()
    for i in range(replays):
        graph.replay()
        got = captured.snapshot()
        assert_same(f"replay {i}", got, want[i], tol * (i + 1))
        # the program's own eager work between replays: library calls on other tensors, a host read
        other = torch.randn(1 << 18, device="cuda")
        assert float((other * 2).sum().isfinite()) == 1.0
        torch.cuda.synchronize()
    if mode == "train":
        assert float(want[-1]["loss"]) < float(want[0]["loss"]), "the steps being compared do train"
