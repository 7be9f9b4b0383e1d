"""The fused step checked element by element, stage by stage (see stage_check.py), at the full sizes and in the
launch configurations that bench.py times, and on small problems that reach the launch schedules those do not."""
import pytest

import phantom_inputs as pin

from stage_check import check_stages

pytestmark = pytest.mark.gpu


def _report(name, worst):
    print(f"{name}: worst relative error per tensor kind: " + ", ".join(f"{k} {v:.1e}" for k, v in worst.items()), flush=True)


def test_config2_step_every_stage_full_size():
    """n=4096, p=8 (shard 512), k=32, batch 1024, 4 layers, ReLU, bf16, all 8 ranks: forward + MSE + backward."""
    print("case stages c2", flush=True)
    prob = pin.Problem(n=4096, p=8, k=32, batch=1024, layers=4, act="relu", dtype="bf16", rank=-1)
    _report("c2", check_stages(prob, seed=0, lr=0.0, mode="no_update"))


def test_config4_training_step_every_stage_full_size():
    """n=16384, p=16 (shard 1024), k=64, batch 4096, 8 layers, GELU, bf16, rank 0, seeded peers: training step."""
    print("case stages c4", flush=True)
    prob = pin.Problem(n=16384, p=16, k=64, batch=4096, layers=8, act="gelu", dtype="bf16", rank=0)
    _report("c4", check_stages(prob, seed=0, lr=1e-3, mode="train"))


def test_config3_step_every_stage_full_size():
    """n=32768, p=64 (shard 512), k=16, batch 2048, one layer, ReLU, bf16, rank 0: forward + MSE + backward."""
    print("case stages c3", flush=True)
    prob = pin.Problem(n=32768, p=64, k=16, batch=2048, layers=1, act="relu", dtype="bf16", rank=0)
    _report("c3", check_stages(prob, seed=0, lr=0.0, mode="no_update"))


@pytest.mark.parametrize("k", [4, 16, 64, 256])
def test_config5_forward_every_layer_full_size(k):
    """n=8192, p=8 (shard 1024), batch 8192, 6 layers, ReLU, bf16, rank 0, forward only: the GPU runs all 8192 rows,
    the oracle recomputes 768 sampled rows of every layer from the GPU's own previous layer."""
    print(f"case stages c5 k={k}", flush=True)
    prob = pin.Problem(n=8192, p=8, k=k, batch=8192, layers=6, act="relu", dtype="bf16", rank=0)
    _report(f"c5 k={k}", check_stages(prob, seed=2, mode="forward", rows=768))


@pytest.mark.parametrize("n,p,k,B,L,act,dtype,rank,mode", [
    (1024, 8, 16, 136, 3, "relu", "bf16", -1, "train"),        # ReLU, several bf16 layers, all ranks (sum-on-read reduce-scatter)
    (2048, 16, 32, 200, 4, "relu", "bf16", 0, "train"),        # ReLU, one rank
    (2048, 16, 8, 2100, 2, "relu", "bf16", -1, "train"),       # 272 output tiles: two-tile workgroups with the output error in the update
    (4096, 16, 16, 4300, 2, "gelu", "bf16", 0, "train"),       # one rank, 34 x 2 tiles and a ragged batch; compressor gradients cut in four along the batch
    (2048, 8, 32, 2050, 3, "relu", "bf16", 0, "train"),        # one rank: all layers' weight gradients in one launch, compressor gradients cut in two
    (1024, 4, 64, 3072, 2, "gelu", "bf16", 0, "no_update"),    # ... cut in three, no update
    (512, 4, 8, 40, 17, "relu", "bf16", 0, "train"),           # one rank, more layers than the launch's table holds: a launch per layer
    (16384, 8, 16, 200, 2, "gelu", "bf16", 0, "train"),        # one rank, 272 weight-gradient tiles per layer: a launch per layer
    (2048, 32, 4, 72, 2, "gelu", "bf16", -1, "no_update"),     # 32 ranks: the reduce-scatter kernel
    (520, 4, 3, 67, 3, "relu", "bf16", 1, "train"),            # k = 3: the shape-agnostic kernels in bf16
    (512, 1, 0, 300, 3, "relu", "bf16", 0, "train"),           # a dense stack
    (288, 4, 5, 37, 3, "relu", "f32", -1, "train"),            # fp32 kernels
    (288, 4, 5, 37, 2, "gelu", "f32", 2, "no_update"),
])
def test_step_every_stage(n, p, k, B, L, act, dtype, rank, mode):
    print(f"case stages n={n} p={p} k={k} B={B} L={L} {act} {dtype} rank={rank} {mode}", flush=True)
    prob = pin.Problem(n=n, p=p, k=k, batch=B, layers=L, act=act, dtype=dtype, rank=rank)
    _report("step", check_stages(prob, seed=8, lr=0.02, mode=mode))


@pytest.mark.parametrize("widths,ks,p,B,act,dtype,rank", [
    ((1024, 2048, 512, 1024), (16, 32, 8), 8, 136, "relu", "bf16", -1),
    ((2048, 1024, 3072), (32, 16), 16, 200, "gelu", "bf16", 0),
])
def test_step_every_stage_layers_of_different_widths(widths, ks, p, B, act, dtype, rank):
    print(f"case stages widths={widths} ks={ks} p={p} B={B} {act} {dtype} rank={rank}", flush=True)
    prob = pin.Problem(n=widths[0], p=p, k=ks[0], batch=B, layers=len(ks), act=act, dtype=dtype, rank=rank,
                       widths=widths, ks=ks)
    _report("widths", check_stages(prob, seed=4, lr=0.02, mode="train"))
