"""Seeded synthetic inputs for the phantom-layer hot path.

This module serves both the CPU oracle's tests and the HIP path's tests and
benchmark.  It holds no arithmetic of the method itself: only a counter-based
random generator, the rounding of generated values to the storage type the
caller asks for, and the shapes of the tensors a problem needs.

Generator: every tensor is identified by (seed, tensor name, layer, rank); its
element number i is drawn from splitmix64 applied to a key derived from that
identity plus i, so any element can be regenerated independently and the
values do not depend on the order in which tensors are requested.

Distributions follow the workload recipe of the paper's experiments as far as
it is stated (Section VI, "Data and Hardware": synthetic Gaussian data) and the
default initialisation of a linear layer for the weights: U(-1/sqrt(fan_in),
+1/sqrt(fan_in)) with fan_in = n/p (the layer's input shard) for the local matrix,
the compressor and the bias, and fan_in = k for the decompressors (shapes from
Section IV-A).
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

_MASK = np.uint64(0xFFFFFFFFFFFFFFFF)
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)

_TENSOR_IDS = {
    "X": 1, "T": 2, "Lw": 3, "Cw": 4, "Dw": 5, "bias": 6, "G": 7, "dY": 8,
    "dg_own": 9, "A": 10, "W_dense": 11, "aux": 12,
}


def _splitmix64(x: np.ndarray) -> np.ndarray:
    """One round of the splitmix64 output function on uint64 values."""
    with np.errstate(over="ignore"):
        z = (x + _GOLDEN) & _MASK
        z = ((z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)) & _MASK
        z = ((z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)) & _MASK
        return z ^ (z >> np.uint64(31))


def _key(seed: int, tensor: str, layer: int, rank: int) -> np.uint64:
    k = np.uint64(seed & 0xFFFFFFFFFFFFFFFF)
    for part in (_TENSOR_IDS[tensor], layer + 1, rank + 2):
        k = _splitmix64(np.asarray(k ^ np.uint64(part * 0x100000001B3 & 0xFFFFFFFFFFFFFFFF), dtype=np.uint64))
    return np.uint64(k)


def _u01(key: np.uint64, start: int, count: int) -> np.ndarray:
    """`count` doubles in (0, 1) for counters start .. start+count-1."""
    idx = np.arange(start, start + count, dtype=np.uint64)
    with np.errstate(over="ignore"):
        bits = _splitmix64((idx * _GOLDEN + key) & _MASK)
    # top 53 bits, shifted by half a step so that 0 is never produced
    return ((bits >> np.uint64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def uniform(shape, lo: float, hi: float, *, seed: int, tensor: str, layer: int = 0, rank: int = 0) -> np.ndarray:
    count = int(np.prod(shape)) if len(shape) else 1
    u = _u01(_key(seed, tensor, layer, rank), 0, count)
    return (lo + (hi - lo) * u).reshape(shape)


def normal(shape, *, seed: int, tensor: str, layer: int = 0, rank: int = 0, scale: float = 1.0) -> np.ndarray:
    """Standard normal values (Box-Muller on counter pairs 2i, 2i+1)."""
    count = int(np.prod(shape)) if len(shape) else 1
    key = _key(seed, tensor, layer, rank)
    u = _u01(key, 0, 2 * count)
    r = np.sqrt(-2.0 * np.log(u[0::2]))
    z = r * np.cos(2.0 * math.pi * u[1::2])
    return (scale * z).reshape(shape)


# ----------------------------------------------------------------------------
# storage types
# ----------------------------------------------------------------------------

def bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round to bfloat16 (nearest even, through float32) and return the 16-bit patterns."""
    f = np.ascontiguousarray(a, dtype=np.float32)
    u = f.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    u = bits.astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def round_to_storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """Values of `a` rounded to the storage type ('f32' or 'bf16'), returned as float64."""
    if dtype == "f32":
        return np.asarray(a, dtype=np.float32).astype(np.float64)
    if dtype == "bf16":
        return bf16_bits_to_f64(bf16_bits(a)).reshape(np.shape(a))
    raise ValueError(f"unknown storage dtype {dtype!r}")


# ----------------------------------------------------------------------------
# problem description and tensor recipes
# ----------------------------------------------------------------------------

@dataclass(frozen=True)
class Problem:
    """(n, p, k, batch, layers, activation) as in Section IV of the paper.

    rank >= 0: one rank's share, peers' buffers are seeded inputs.
    rank == -1: all p ranks held together; every tensor gains a leading [p] axis.

    widths, ks (optional): layer widths n_0 .. n_L (n_0 the network input, n_l the output of layer l)
    and phantom widths k_1 .. k_L, for a network whose layers differ (Section IV, first paragraph);
    empty = every width is n, every phantom width k.
    """
    n: int
    p: int
    k: int
    batch: int
    layers: int = 1
    act: str = "relu"          # 'identity' | 'relu' | 'gelu'
    dtype: str = "f32"         # 'f32' | 'bf16' (bf16 storage, fp32 accumulate)
    rank: int = 0
    widths: tuple = ()
    ks: tuple = ()

    def __post_init__(self):
        if self.widths:
            assert len(self.widths) == self.layers + 1 and (self.p == 1 or len(self.ks) == self.layers)
            assert all(w % self.p == 0 for w in self.widths)

    @property
    def s(self) -> int:
        return self.n // self.p

    @property
    def peers(self) -> int:
        return self.p - 1

    @property
    def kc(self) -> int:
        return self.s + self.peers * self.k

    def s_in(self, layer: int) -> int:
        """Inputs of layer `layer` (0-based) held by one rank."""
        return (self.widths[layer] if self.widths else self.n) // self.p

    def s_out(self, layer: int) -> int:
        return (self.widths[layer + 1] if self.widths else self.n) // self.p

    def k_of(self, layer: int) -> int:
        return self.ks[layer] if self.ks else self.k


def layer_params(prob: Problem, layer: int, rank: int, seed: int) -> dict:
    """Weights of one rank for one layer, rounded to the storage type."""
    si, so, k, q = prob.s_in(layer), prob.s_out(layer), prob.k_of(layer), prob.peers
    bs, bk = 1.0 / math.sqrt(si), 1.0 / math.sqrt(max(k, 1))
    out = {
        "Lw": uniform((so, si), -bs, bs, seed=seed, tensor="Lw", layer=layer, rank=rank),
        "bias": uniform((so,), -bs, bs, seed=seed, tensor="bias", layer=layer, rank=rank),
        "Cw": uniform((k, si), -bs, bs, seed=seed, tensor="Cw", layer=layer, rank=rank),
        "Dw": uniform((q, so, k), -bk, bk, seed=seed, tensor="Dw", layer=layer, rank=rank),
    }
    return {name: round_to_storage(v, prob.dtype) for name, v in out.items()}


def one_rank_layer_inputs(prob: Problem, layer: int, seed: int, *, with_backward: bool = True) -> dict:
    """Inputs of one phantom layer on rank prob.rank with seeded peer buffers.

    X, G ~ N(0,1); dY, dg_own ~ N(0,1)/batch (the scale of an MSE output error
    averaged over the batch).
    """
    B, k, q = prob.batch, prob.k_of(layer), prob.peers
    r = prob.rank
    d = layer_params(prob, layer, r, seed)
    d["X"] = normal((B, prob.s_in(layer)), seed=seed, tensor="X", layer=layer, rank=r)
    d["G"] = normal((q, B, k), seed=seed, tensor="G", layer=layer, rank=r)
    if with_backward:
        d["dY"] = normal((B, prob.s_out(layer)), seed=seed, tensor="dY", layer=layer, rank=r, scale=1.0 / B)
        d["dg_own"] = normal((B, k), seed=seed, tensor="dg_own", layer=layer, rank=r, scale=1.0 / B)
    for name in ("X", "G", "dY", "dg_own"):
        if name in d:
            d[name] = round_to_storage(d[name], prob.dtype)
    return d


def all_rank_params(prob: Problem, layer: int, seed: int) -> dict:
    """Weights of all p ranks for one layer, stacked on a leading [p] axis."""
    per = [layer_params(prob, layer, j, seed) for j in range(prob.p)]
    return {name: np.stack([d[name] for d in per]) for name in per[0]}


def network_io(prob: Problem, seed: int) -> tuple:
    """Network input and target, [batch, n] each, N(0,1), rounded to storage.

    In all-ranks mode the caller shards the columns: rank j owns columns
    j*s .. (j+1)*s-1.  In one-rank mode only that rank's columns are used.
    """
    n_in, n_out = prob.s_in(0) * prob.p, prob.s_out(prob.layers - 1) * prob.p
    X0 = normal((prob.batch, n_in), seed=seed, tensor="X", layer=-1, rank=0)
    T = normal((prob.batch, n_out), seed=seed, tensor="T", layer=-1, rank=0)
    return round_to_storage(X0, prob.dtype), round_to_storage(T, prob.dtype)


def shard_columns(a: np.ndarray, p: int) -> np.ndarray:
    """[B, n] -> [p, B, n/p] (copy)."""
    B, n = a.shape
    return np.ascontiguousarray(a.reshape(B, p, n // p).transpose(1, 0, 2))


def one_rank_step_inputs(prob: Problem, seed: int) -> dict:
    """Everything a multi-layer one-rank step needs: per-layer weights, seeded
    peer buffers G[l] and reduce-scatter results dg_own[l], the rank's columns
    of the network input and target."""
    B, q, r = prob.batch, prob.peers, prob.rank
    layers = []
    for l in range(prob.layers):
        k = prob.k_of(l)
        d = layer_params(prob, l, r, seed)
        d["G"] = round_to_storage(normal((q, B, k), seed=seed, tensor="G", layer=l, rank=r), prob.dtype)
        d["dg_own"] = round_to_storage(
            normal((B, k), seed=seed, tensor="dg_own", layer=l, rank=r, scale=1.0 / B), prob.dtype)
        layers.append(d)
    X0 = round_to_storage(normal((B, prob.s_in(0)), seed=seed, tensor="X", layer=-1, rank=r), prob.dtype)
    T = round_to_storage(normal((B, prob.s_out(prob.layers - 1)), seed=seed, tensor="T", layer=-1, rank=r), prob.dtype)
    return {"layers": layers, "X0": X0, "T": T}


def all_rank_step_inputs(prob: Problem, seed: int) -> dict:
    layers = [all_rank_params(prob, l, seed) for l in range(prob.layers)]
    X0, T = network_io(prob, seed)
    return {"layers": layers, "X0": shard_columns(X0, prob.p), "T": shard_columns(T, prob.p)}


def regression_task(n: int, samples: int, seed: int, dtype: str = "f32") -> tuple:
    """The data set of the paper's training experiments (Section VI, "Data and Hardware"):
    pairs (x_i, y_i), y_i = relu(W relu(x_i)), with one Gaussian n x n matrix W kept fixed.

    The paper says W is a standard Gaussian matrix and leaves the distribution of x open.  Here x ~ N(0, 1), and,
    as a deliberate departure from the paper's recipe, W ~ N(0, 1) / sqrt(n / 2): with the unscaled matrix the
    entries of y grow like sqrt(n / 2) (16 at n = 512) and the fixed learning rate of the tests would have to
    change with n; the scaled one keeps y of order one whatever n is.  The map itself (ReLU, fixed Gaussian W,
    ReLU) is the paper's.
    Returns (X, Y), [samples, n] each, rounded to the storage type.
    """
    W = normal((n, n), seed=seed, tensor="W_dense", layer=-2, rank=0, scale=1.0 / math.sqrt(n / 2.0))
    X = normal((samples, n), seed=seed, tensor="X", layer=-2, rank=0)
    Y = np.maximum(np.maximum(X, 0.0) @ W.T, 0.0)
    return round_to_storage(X, dtype), round_to_storage(Y, dtype)
