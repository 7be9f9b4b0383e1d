"""phantom_ffn_step_static (the step for callers that cannot allocate) against phantom_ffn_step.

Both entry points run the same kernels; the only difference is where the workspace lives.  The test calls the
new entry point through the C ABI twice in a row on one GPU, the second time with a smaller problem (so the array
still holds the first call's contents where the second one does not overwrite them), and checks every output of
each call against the same step through phantom_ffn_step: bit for bit where the step is deterministic (fp32
storage), to a small multiple of the storage type's rounding where float atomics decide the order of a sum
(bf16: column sums and loss partials), which is far inside the parity bar of 2e-2.  Problems beyond the
array's size are refused before any GPU call.
"""
import pytest
import torch

import paper_2508_00960_amd as ph
import phantom_inputs as pin

from helpers import empty, empty_f32, to_gpu, to_gpu_f32, workspace

pytestmark = pytest.mark.gpu


class Run:
    def __init__(self, prob, data, lr, mode):
        dt, q = prob.dtype, prob.peers
        one_rank = prob.rank >= 0
        self.pc = ph.make_problem(prob.n, prob.p, prob.k, prob.batch, prob.layers, prob.act, prob.dtype, prob.rank)
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

    def step(self, static):
        W, M, Gd = self.W, self.M, self.Gd
        kw = dict(Lw_master=M.get("Lw"), Cw_master=M.get("Cw"), Dw_master=M.get("Dw"), bias_master=M.get("bias"),
                  G=self.G, dg_own=self.dg, dLw=Gd["Lw"], dCw=Gd.get("Cw"), dDw=Gd.get("Dw"), dbias=Gd["bias"],
                  Y_out=self.Y, loss=self.loss, lr=self.lr, mode=self.mode)
        if static:
            ph.ffn_step_static(self.pc, self.X0, self.T, W["Lw"], W.get("Cw"), W.get("Dw"), W["bias"], **kw)
        else:
            ws = workspace(ph.workspace_bytes(self.pc))
            ph.ffn_step(self.pc, self.X0, self.T, W["Lw"], W.get("Cw"), W.get("Dw"), W["bias"], workspace=ws, **kw)
        torch.cuda.synchronize()

    def outputs(self):
        out = {"loss": self.loss[:1].clone(), "Y": self.Y.float().clone()}
        for nm, per_layer in self.Gd.items():
            for l, t in enumerate(per_layer):
                out[f"d{nm}[{l}]"] = t.clone()
        for nm, per_layer in (self.M or self.W).items():
            for l, t in enumerate(per_layer):
                out[f"{nm}[{l}]"] = t.float().clone()
        return out


def _compare(what, got, want, tol):
    for name, ref in want.items():
        assert torch.isfinite(got[name]).all(), f"{what}: {name} not finite"
        if tol == 0:
            assert torch.equal(got[name], ref), f"{what}: {name} differs"
        else:
            scale = max(float(ref.abs().max()), 1e-30)
            err = float((got[name] - ref).abs().max()) / scale
            assert err <= tol, f"{what}: {name} differs by {err:.3e} of its largest magnitude (bound {tol:.1e})"


@pytest.mark.parametrize("dtype,act,rank,first,second", [
    # (n, p, k, batch, layers) of the first call and of the second, smaller one
    ("bf16", "gelu", 0, (2048, 16, 32, 384, 3), (1024, 8, 16, 136, 2)),
    ("bf16", "relu", -1, (1024, 8, 32, 256, 3), (512, 4, 8, 72, 2)),
    ("f32", "gelu", -1, (288, 4, 5, 37, 3), (96, 3, 2, 19, 2)),
])
def test_static_step_matches_the_step_with_a_workspace(dtype, act, rank, first, second):
    tol = 0 if dtype == "f32" else 4e-3
    for call, (n, p, k, B, L) in (("first call", first), ("second call, smaller", second)):
        print(f"case no-alloc {call}: n={n} p={p} k={k} B={B} L={L} {act} {dtype} rank={rank}", flush=True)
        prob = pin.Problem(n=n, p=p, k=k, batch=B, layers=L, act=act, dtype=dtype, rank=min(rank, p - 1))
        assert ph.workspace_bytes(ph.make_problem(n, p, k, B, L, act, dtype, prob.rank)) <= ph.static_workspace_bytes()
        data = pin.all_rank_step_inputs(prob, 21) if prob.rank < 0 else pin.one_rank_step_inputs(prob, 21)
        a, b = Run(prob, data, 2e-4, "train"), Run(prob, data, 2e-4, "train")
        a.step(static=False)
        b.step(static=True)
        _compare(call, b.outputs(), a.outputs(), tol)


def test_static_step_refuses_what_does_not_fit():
    """Configuration 4 needs about half a gigabyte of workspace: refused, with the sizes in the message, and nothing
    is launched (the buffers handed over are far too small for the problem and stay untouched)."""
    big = ph.make_problem(16384, 16, 64, 4096, 8, "gelu", "bf16", 0)
    assert ph.workspace_bytes(big) > ph.static_workspace_bytes()
    ok = 0x1000
    eight = [ok] * 8
    with pytest.raises(ph.PhantomError) as e:
        ph.ffn_step_static(big, ok, ok, eight, eight, eight, eight, G=eight, dg_own=eight, loss=ok, mode="no_update")
    assert e.value.status == -3 and "scratch" in str(e.value)
