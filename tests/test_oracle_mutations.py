"""Do the pins of test_oracle_pins.py notice a mistake?  Each case below plants one plausible mistake
in the ORACLE (on the CPU, by replacing one of its functions with a wrong version for the duration of
the test) and expects at least one pin to fail.  A mistake that no pin notices would mean that the
oracle's parity claims rest on less than they say.

The pins run here are the ones that fix values from outside the oracle: torch autograd through an
ordinary dense network (Section III's tensor-parallel model that the phantom model must equal when its
off-diagonal blocks are D C), central differences of the oracle's own forward, and the agreement
between the one-rank and the all-ranks code paths.
"""
import numpy as np
import pytest

from oracle import oracle

import test_oracle_pins as pins


def _pins():
    """The pins as thunks (name, call)."""
    return [
        ("p=1 dense layer", lambda: pins.test_p1_is_dense_layer("gelu")),
        ("structured dense, gelu", lambda: pins.check_structured_dense(12, 3, 2, 5, 2, "gelu")),
        ("structured dense, relu, 3 layers", lambda: pins.check_structured_dense(12, 3, 2, 5, 3, "relu")),
        ("structured dense, 4 ranks", lambda: pins.check_structured_dense(20, 4, 3, 6, 2, "identity")),
        ("structured dense, layers of different widths",
         lambda: pins.check_structured_dense(12, 3, 2, 5, 3, "gelu", (12, 21, 6, 15), (2, 3, 1))),
        ("identity compressor", pins.test_identity_compressor_reproduces_dense_layer),
        ("one rank vs all ranks", lambda: pins.check_one_rank_vs_all_ranks("f32")),
        ("central differences", lambda: pins.check_central_differences("gelu")),
        ("concatenated operands", pins.test_concatenated_operands_give_the_same_layer),
    ]


def _failing_pins():
    failed = []
    for name, call in _pins():
        try:
            call()
        except AssertionError:
            failed.append(name)
        except Exception as exc:     # a shape error is also a way of noticing
            failed.append(f"{name} ({type(exc).__name__})")
    return failed


def test_unmutated_oracle_passes_every_pin():
    assert _failing_pins() == []


# ---- the planted mistakes ---------------------------------------------------------------

_orig = {name: getattr(oracle, name) for name in
         ("compress", "layer_update", "delta_of", "error_compress", "layer_grads", "without_slot", "reduce_scatter",
          "mse_loss")}


def _no_bias(act, X, Lw, Dw, bias, G):
    return _orig["layer_update"](act, X, Lw, Dw, np.zeros_like(bias), G)


def _last_peer_ignored(act, X, Lw, Dw, bias, G):
    if G is None:
        return _orig["layer_update"](act, X, Lw, Dw, bias, G)
    G2 = np.array(G, copy=True)
    G2[-1] = 0.0
    return _orig["layer_update"](act, X, Lw, Dw, bias, G2)


def _local_block_transposed(act, X, Lw, Dw, bias, G):
    return _orig["layer_update"](act, X, np.ascontiguousarray(Lw.T), Dw, bias, G)


def _peers_in_reverse_order(a, j):
    return _orig["without_slot"](a, j)[::-1].copy()


def _gather_keeps_own_slot(a, j):
    """Rank j drops slot j-1 instead of its own (an off-by-one in the skipped slot)."""
    jj = (j - 1) % a.shape[0]
    return _orig["without_slot"](a, jj)


def _compressor_rows_reversed(X, Cw):
    return _orig["compress"](X, Cw[::-1].copy())


def _derivative_at_the_output(act, dY, A, storage="f32"):
    """sigma' evaluated at sigma(A) instead of A (right for ReLU, wrong for a smooth activation)."""
    if act == "gelu":
        import math
        Y = 0.5 * A * (1.0 + np.vectorize(math.erf)(A / math.sqrt(2.0)))
        return _orig["delta_of"](act, dY, Y, storage)
    if act == "identity":
        return 2.0 * _orig["delta_of"](act, dY, A, storage)
    return _orig["delta_of"](act, dY, np.abs(A), storage)       # ReLU' = 1 everywhere but at 0


def _error_compression_peers_reversed(Dw, delta):
    return _orig["error_compress"](Dw, delta)[::-1].copy()


def _error_compression_without_transpose(Dw, delta):
    """Uses the first k columns of delta's product with D's first k rows: a transposed-operand slip."""
    out = _orig["error_compress"](Dw, delta)
    return out * 0.0 + np.einsum("bs,qsk->qbk", delta, Dw)[:, :, ::-1]


def _reduce_scatter_wrong_slot(dG_send, storage="f32"):
    p = dG_send.shape[0]
    out = np.zeros(dG_send.shape[:1] + dG_send.shape[2:])
    for i in range(p):
        for j in range(p):
            if j != i:
                out[i] += dG_send[j, j if j < i else j - 1]      # the holder's index where the source's belongs
    return oracle.rd(out, storage)


def _reduce_scatter_includes_nothing_from_last_rank(dG_send, storage="f32"):
    d = np.array(dG_send, copy=True)
    d[-1] = 0.0
    return _orig["reduce_scatter"](d, storage)


def _grads(change):
    def wrapped(delta, X, Lw, Cw, G, dg_own, need_dX=True):
        out = _orig["layer_grads"](delta, X, Lw, Cw, G, dg_own, need_dX)
        change(out, delta, X, Lw, Cw, G, dg_own, need_dX)
        return out
    return wrapped


def _dD_doubled(out, *_):
    if out["dDw"] is not None:
        out["dDw"] = 2.0 * out["dDw"]


def _dD_peers_reversed(out, *_):
    if out["dDw"] is not None:
        out["dDw"] = out["dDw"][::-1].copy()


def _dC_sign(out, *_):
    if out["dCw"] is not None:
        out["dCw"] = -out["dCw"]


def _dX_without_compressor_term(out, delta, X, Lw, Cw, G, dg_own, need_dX):
    if need_dX and dg_own is not None:
        out["dX"] = _orig["layer_grads"](delta, X, Lw, Cw, G, np.zeros_like(dg_own), True)["dX"]


def _dL_transposed(out, *_):
    out["dLw"] = np.ascontiguousarray(out["dLw"].T)


def _db_is_a_mean(out, delta, *_):
    out["dbias"] = out["dbias"] / delta.shape[0]


def _loss_without_the_half(Y, T):
    loss, dY = _orig["mse_loss"](Y, T)
    return 2.0 * loss, dY


def _output_error_not_averaged(Y, T):
    loss, dY = _orig["mse_loss"](Y, T)
    return loss, dY * Y.shape[-2]


MUTATIONS = [
    ("bias dropped from the update", "layer_update", _no_bias),
    ("last peer's phantom layer ignored", "layer_update", _last_peer_ignored),
    ("local block applied transposed", "layer_update", _local_block_transposed),
    ("gathered peers in reverse order", "without_slot", _peers_in_reverse_order),
    ("wrong slot skipped in the gathered buffer", "without_slot", _gather_keeps_own_slot),
    ("compressor rows reversed", "compress", _compressor_rows_reversed),
    ("activation derivative taken at the output", "delta_of", _derivative_at_the_output),
    ("error compression: peers reversed", "error_compress", _error_compression_peers_reversed),
    ("error compression: ghost index reversed", "error_compress", _error_compression_without_transpose),
    ("reduce-scatter reads the holder's slot", "reduce_scatter", _reduce_scatter_wrong_slot),
    ("reduce-scatter loses one sender", "reduce_scatter", _reduce_scatter_includes_nothing_from_last_rank),
    ("dD doubled", "layer_grads", _grads(_dD_doubled)),
    ("dD assigned to the wrong peers", "layer_grads", _grads(_dD_peers_reversed)),
    ("dC with the wrong sign", "layer_grads", _grads(_dC_sign)),
    ("dX without the compressor term", "layer_grads", _grads(_dX_without_compressor_term)),
    ("dL transposed", "layer_grads", _grads(_dL_transposed)),
    ("db averaged instead of summed", "layer_grads", _grads(_db_is_a_mean)),
    ("loss without the factor 1/2", "mse_loss", _loss_without_the_half),
    ("output error not averaged over the batch", "mse_loss", _output_error_not_averaged),
]


@pytest.mark.parametrize("what,name,wrong", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_a_planted_mistake_fails_a_pin(monkeypatch, what, name, wrong):
    monkeypatch.setattr(oracle, name, wrong)
    failed = _failing_pins()
    assert failed, f"no pin noticed: {what}"
