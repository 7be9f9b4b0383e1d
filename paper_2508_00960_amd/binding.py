"""ctypes binding of libphantom.so: argument marshalling only.

Every function has the name and argument order of its C entry point in
include/phantom.h.  Tensor arguments are torch tensors on the GPU (their
data_ptr() is passed), None (NULL), or plain integers (raw addresses, used by
the host-only argument-validation tests).  A tensor is checked against the
problem's shapes before the call (device memory, contiguous, element size, at
least as many elements as the argument has): the library sees an address only.
Nothing is computed here.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libphantom.so")

ACTS = {"identity": 0, "relu": 1, "gelu": 2}
DTYPES = {"f32": 0, "bf16": 1}
STEP_MODES = {"train": 0, "forward": 1, "no_update": 2}

PH_OK = 0


class PhantomError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"libphantom status {status}: {message}")
        self.status = status


class PhProblem(ctypes.Structure):
    _fields_ = [
        ("n", ctypes.c_int64), ("p", ctypes.c_int64), ("k", ctypes.c_int64), ("batch", ctypes.c_int64),
        ("layers", ctypes.c_int32), ("act", ctypes.c_int32), ("dtype", ctypes.c_int32), ("rank", ctypes.c_int32),
        ("widths", ctypes.POINTER(ctypes.c_int64)), ("ks", ctypes.POINTER(ctypes.c_int64)),
    ]

    @property
    def s(self) -> int:
        return self.n // self.p


_PP = ctypes.POINTER(ctypes.c_void_p)


class PhStepTaps(ctypes.Structure):
    _fields_ = [("Y", _PP), ("g_own", _PP), ("delta", _PP), ("dG_send", _PP), ("dg_own", _PP)]


class PhStepArgs(ctypes.Structure):
    _fields_ = [
        ("X0", ctypes.c_void_p), ("T", ctypes.c_void_p),
        ("Lw", _PP), ("Cw", _PP), ("Dw", _PP), ("bias", _PP),
        ("Lw_master", _PP), ("Cw_master", _PP), ("Dw_master", _PP), ("bias_master", _PP),
        ("G", _PP), ("dg_own", _PP),
        ("dLw", _PP), ("dCw", _PP), ("dDw", _PP), ("dbias", _PP),
        ("Y_out", ctypes.c_void_p), ("loss", ctypes.c_void_p),
        ("lr", ctypes.c_float), ("mode", ctypes.c_int32),
        ("taps", ctypes.POINTER(PhStepTaps)),
    ]


class PhProfileEntry(ctypes.Structure):
    _fields_ = [
        ("name", ctypes.c_char * 64), ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
        ("groups", ctypes.c_int32), ("calls", ctypes.c_int32), ("total_ms", ctypes.c_double),
        ("M2", ctypes.c_int64), ("N2", ctypes.c_int64), ("K2", ctypes.c_int64),
        ("M3", ctypes.c_int64), ("N3", ctypes.c_int64), ("K3", ctypes.c_int64),
        ("M4", ctypes.c_int64), ("N4", ctypes.c_int64), ("K4", ctypes.c_int64),
    ]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load():
    """Load libphantom.so.  It is never replaced by a fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    import torch  # noqa: F401  (brings the HIP runtime the library links against into the process first)
    if not os.path.exists(_LIB_PATH):
        from .build import build_library
        build_library(verbose=False)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    prob = ctypes.POINTER(PhProblem)
    lib.phantom_abi_version.restype = ctypes.c_int32
    lib.phantom_last_error.restype = ctypes.c_char_p
    lib.phantom_workspace_bytes.restype = ctypes.c_int
    lib.phantom_workspace_bytes.argtypes = [prob, ctypes.POINTER(sz)]
    lib.phantom_layer_fwd.restype = ctypes.c_int
    lib.phantom_layer_fwd.argtypes = [prob] + [vp] * 9 + [vp, sz, vp]
    lib.phantom_layer_bwd.restype = ctypes.c_int
    lib.phantom_layer_bwd.argtypes = [prob] + [vp] * 14 + [vp, sz, vp]
    lib.phantom_ffn_step.restype = ctypes.c_int
    lib.phantom_ffn_step.argtypes = [prob, ctypes.POINTER(PhStepArgs), vp, sz, vp]
    lib.phantom_ffn_step_static.restype = ctypes.c_int
    lib.phantom_ffn_step_static.argtypes = [prob, ctypes.POINTER(PhStepArgs), vp]
    lib.phantom_static_workspace_bytes.restype = ctypes.c_size_t
    lib.phantom_profile_begin.restype = ctypes.c_int
    lib.phantom_profile_begin.argtypes = [ctypes.c_int32]
    lib.phantom_profile_end.restype = ctypes.c_int
    lib.phantom_profile_end.argtypes = [ctypes.POINTER(PhProfileEntry), ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)]
    _lib = lib
    return lib


def profile_begin(max_launches: int = 4096) -> None:
    _check(load().phantom_profile_begin(int(max_launches)))


def profile_end(capacity: int = 256):
    """Returns a list of dicts: name, M, N, K, groups, calls, total_ms."""
    entries = (PhProfileEntry * capacity)()
    count = ctypes.c_int32(0)
    _check(load().phantom_profile_end(entries, capacity, ctypes.byref(count)))
    return [dict(name=e.name.decode(), M=e.M, N=e.N, K=e.K, groups=e.groups, calls=e.calls, total_ms=e.total_ms,
                 M2=e.M2, N2=e.N2, K2=e.K2, M3=e.M3, N3=e.N3, K3=e.K3, M4=e.M4, N4=e.N4, K4=e.K4)
            for e in entries[:count.value]]


def abi_version() -> int:
    return int(load().phantom_abi_version())


def last_error() -> str:
    return load().phantom_last_error().decode()


def make_problem(n: int, p: int, k: int, batch: int, layers: int = 1, act: str = "relu", dtype: str = "f32",
                 rank: int = 0, widths=(), ks=()) -> PhProblem:
    """widths (n_0 .. n_L) and ks (k_1 .. k_L): layers of different widths; empty = every layer n and k."""
    prob = PhProblem(n, p, k, batch, layers, ACTS[act], DTYPES[dtype], rank, None, None)
    if widths:
        prob._widths = (ctypes.c_int64 * len(widths))(*widths)      # kept alive by the struct object
        prob.widths = ctypes.cast(prob._widths, ctypes.POINTER(ctypes.c_int64))
        if ks:
            prob._ks = (ctypes.c_int64 * len(ks))(*ks)
            prob.ks = ctypes.cast(prob._ks, ctypes.POINTER(ctypes.c_int64))
    return prob


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _layer_shape(prob: PhProblem, layer: int):
    """(si, so, k) of one layer per rank: inputs, outputs, phantom width."""
    if prob.widths:
        si, so = prob.widths[layer] // prob.p, prob.widths[layer + 1] // prob.p
        k = prob.ks[layer] if prob.ks else prob.k
    else:
        si = so = prob.n // prob.p
        k = prob.k
    return si, so, (k if prob.p > 1 else 0)


def _expect(name: str, t, elems: int, elem_bytes: int) -> None:
    """A tensor handed over for `name` must live on the GPU, be contiguous and hold at least `elems` elements of
    `elem_bytes` bytes: the library sees an address only and would read or write past a shorter buffer.  Raw
    addresses and None pass through (the library checks for NULL where an argument is required)."""
    if t is None or isinstance(t, int) or elems <= 0:
        return
    if not t.is_cuda:
        raise ValueError(f"{name}: tensor is on {t.device}, the library needs device memory")
    if not t.is_contiguous():
        raise ValueError(f"{name}: tensor is not contiguous")
    if t.element_size() != elem_bytes:
        raise ValueError(f"{name}: elements of {t.element_size()} bytes, {elem_bytes} expected ({t.dtype})")
    if t.numel() < elems:
        raise ValueError(f"{name}: {t.numel()} elements, the problem needs {elems}")


def _check_layer_tensors(prob: PhProblem, layer: int, named: dict) -> None:
    """named: argument name -> (tensor, kind); kind says which of the layer's shapes the argument has."""
    si, so, k = _layer_shape(prob, layer)
    B, q = prob.batch, prob.p - 1
    groups = prob.p if prob.rank < 0 else 1
    esz = 2 if prob.dtype == DTYPES["bf16"] else 4
    counts = {
        "in": groups * B * si, "out": groups * B * so, "L": groups * so * si, "C": groups * k * si,
        "D": groups * q * so * k, "b": groups * so, "g": groups * B * k, "send": groups * q * B * k,
        "gathered": (prob.p if prob.rank < 0 else q) * B * k, "scalar": 1,
    }
    for name, (t, kind) in named.items():
        grad = kind.endswith("32")                      # gradients, master weights, the loss: float
        _expect(name, t, counts[kind[:-2] if grad else kind], 4 if grad else esz)


def _nbytes(t) -> int:
    if t is None:
        return 0
    if isinstance(t, tuple):
        return t[1]
    return t.numel() * t.element_size()


def _stream(stream) -> Optional[int]:
    if stream is not None:
        return stream if isinstance(stream, int) else stream.cuda_stream
    import torch
    if torch.cuda.is_available():
        return torch.cuda.current_stream().cuda_stream
    return None


def _check(status: int):
    if status != PH_OK:
        raise PhantomError(status, last_error())


def _ws(workspace):
    """workspace: a torch uint8 tensor, None, or (address, bytes)."""
    if workspace is None:
        return None, 0
    if isinstance(workspace, tuple):
        return workspace
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def workspace_bytes(prob: PhProblem) -> int:
    out = ctypes.c_size_t(0)
    _check(load().phantom_workspace_bytes(ctypes.byref(prob), ctypes.byref(out)))
    return int(out.value)


def layer_fwd(prob, X, Lw, Cw, Dw, bias, G, Y, g_own, A_save, workspace=None, stream=None):
    wp, wb = _ws(workspace)
    _check_layer_tensors(prob, 0, {"X": (X, "in"), "Lw": (Lw, "L"), "Cw": (Cw, "C"), "Dw": (Dw, "D"), "bias": (bias, "b"),
                                   "G": (G if prob.rank >= 0 else None, "gathered"), "Y": (Y, "out"),
                                   "g_own": (g_own, "g"), "A_save": (A_save, "out")})
    _check(load().phantom_layer_fwd(ctypes.byref(prob), _ptr(X), _ptr(Lw), _ptr(Cw), _ptr(Dw), _ptr(bias), _ptr(G),
                                    _ptr(Y), _ptr(g_own), _ptr(A_save), wp, wb, _stream(stream)))


def layer_bwd(prob, dY, X, A_or_Y, Lw, Cw, Dw, G, dg_own, dX, dLw, dCw, dDw, dbias, dG_send, workspace=None,
              stream=None):
    wp, wb = _ws(workspace)
    _check_layer_tensors(prob, 0, {"dY": (dY, "out"), "X": (X, "in"), "A_or_Y": (A_or_Y, "out"), "Lw": (Lw, "L"),
                                   "Cw": (Cw, "C"), "Dw": (Dw, "D"), "G": (G, "gathered"), "dg_own": (dg_own, "g"),
                                   "dX": (dX, "in"), "dLw": (dLw, "L32"), "dCw": (dCw, "C32"), "dDw": (dDw, "D32"),
                                   "dbias": (dbias, "b32"), "dG_send": (dG_send, "send")})
    _check(load().phantom_layer_bwd(ctypes.byref(prob), _ptr(dY), _ptr(X), _ptr(A_or_Y), _ptr(Lw), _ptr(Cw), _ptr(Dw),
                                    _ptr(G), _ptr(dg_own), _ptr(dX), _ptr(dLw), _ptr(dCw), _ptr(dDw), _ptr(dbias),
                                    _ptr(dG_send), wp, wb, _stream(stream)))


def _ptr_array(tensors: Optional[Sequence], layers: int):
    if tensors is None:
        return None, None
    if len(tensors) != layers:
        raise ValueError(f"expected {layers} per-layer tensors, got {len(tensors)}")
    arr = (ctypes.c_void_p * layers)(*[_ptr(t) for t in tensors])
    return ctypes.cast(arr, _PP), arr


def ffn_step(prob, X0, T, Lw, Cw, Dw, bias, *, Lw_master=None, Cw_master=None, Dw_master=None, bias_master=None,
             G=None, dg_own=None, dLw=None, dCw=None, dDw=None, dbias=None, Y_out=None, loss=None, lr=0.0,
             mode="train", workspace=None, stream=None, taps=None, static=False):
    """phantom_ffn_step; per-layer arguments are sequences of prob.layers tensors (or None).
    taps: dict with any of "Y", "g_own", "delta", "dG_send", "dg_own" -> sequence of prob.layers tensors (ph_step_taps)."""
    L = prob.layers
    keep = []
    kinds = {"Lw": "L", "Cw": "C", "Dw": "D", "bias": "b", "Lw_master": "L32", "Cw_master": "C32", "Dw_master": "D32",
             "bias_master": "b32", "G": "gathered", "dg_own": "g", "dLw": "L32", "dCw": "C32", "dDw": "D32", "dbias": "b32"}
    per_layer = {"Lw": Lw, "Cw": Cw, "Dw": Dw, "bias": bias, "Lw_master": Lw_master, "Cw_master": Cw_master,
                 "Dw_master": Dw_master, "bias_master": bias_master, "G": G, "dg_own": dg_own, "dLw": dLw, "dCw": dCw,
                 "dDw": dDw, "dbias": dbias}
    for layer in range(L):
        named = {f"{name}[{layer}]": (val[layer], kinds[name]) for name, val in per_layer.items()
                 if val is not None and len(val) == L and not (prob.rank < 0 and name in ("G", "dg_own"))}
        if layer == 0:
            named["X0"] = (X0, "in")
        if layer == L - 1:
            named.update({"T": (T, "out"), "Y_out": (Y_out, "out"), "loss": (loss, "scalar32")})
        _check_layer_tensors(prob, layer, named)
    args = PhStepArgs()
    args.X0, args.T, args.Y_out, args.loss = _ptr(X0), _ptr(T), _ptr(Y_out), _ptr(loss)
    for name, val in (("Lw", Lw), ("Cw", Cw), ("Dw", Dw), ("bias", bias), ("Lw_master", Lw_master),
                      ("Cw_master", Cw_master), ("Dw_master", Dw_master), ("bias_master", bias_master),
                      ("G", G), ("dg_own", dg_own), ("dLw", dLw), ("dCw", dCw), ("dDw", dDw), ("dbias", dbias)):
        ptr, arr = _ptr_array(val, L)
        keep.append(arr)
        if ptr is not None:
            setattr(args, name, ptr)
    args.lr = float(lr)
    args.mode = STEP_MODES[mode]
    if taps:
        tap_kinds = {"Y": "out", "g_own": "g", "delta": "out", "dG_send": "send", "dg_own": "g"}
        tp = PhStepTaps()
        for name, val in taps.items():
            for layer in range(L):
                _check_layer_tensors(prob, layer, {f"taps.{name}[{layer}]": (val[layer], tap_kinds[name])})
            ptr, arr = _ptr_array(val, L)
            keep.append(arr)
            setattr(tp, name, ptr)
        keep.append(tp)
        args.taps = ctypes.pointer(tp)
    if static:
        _check(load().phantom_ffn_step_static(ctypes.byref(prob), ctypes.byref(args), _stream(stream)))
        return
    wp, wb = _ws(workspace)
    _check(load().phantom_ffn_step(ctypes.byref(prob), ctypes.byref(args), wp, wb, _stream(stream)))


def ffn_step_static(prob, X0, T, Lw, Cw, Dw, bias, **kwargs):
    """phantom_ffn_step_static: the step on the library's own scratch array (no workspace argument)."""
    assert "workspace" not in kwargs
    ffn_step(prob, X0, T, Lw, Cw, Dw, bias, static=True, **kwargs)


def static_workspace_bytes() -> int:
    return int(load().phantom_static_workspace_bytes())
