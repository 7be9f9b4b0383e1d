"""Shared by the GPU parity tests: moving seeded numpy inputs to the GPU in the storage type,
bringing results back as float64, and the error measure of the parity bar."""
import numpy as np
import torch

import phantom_inputs as pin

# parity bar: max over elements of |gpu - ref| / max(|ref|, RMS(ref)), per tensor
TOL = {"f32": 1e-5, "bf16": 2e-2}


def to_gpu(a, dtype):
    """float64 numpy array holding storage-representable values -> GPU tensor in the storage type."""
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if dtype == "f32":
        return torch.from_numpy(a.astype(np.float32)).cuda()
    bits = pin.bf16_bits(a).reshape(a.shape)
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def to_gpu_f32(a):
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a).astype(np.float32)).cuda()


def empty(shape, dtype):
    return torch.empty(tuple(int(x) for x in shape), device="cuda",
                       dtype=torch.float32 if dtype == "f32" else torch.bfloat16)


def empty_f32(shape):
    return torch.empty(tuple(int(x) for x in shape), device="cuda", dtype=torch.float32)


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got, ref):
    got = np.asarray(got, dtype=np.float64); ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    denom = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / denom))


def assert_close(name, got_tensor, ref, dtype, tol=None):
    assert torch.isfinite(got_tensor.float()).all(), f"{name}: non-finite values"
    err = rel_err(to_np(got_tensor), ref)
    bar = TOL[dtype] if tol is None else tol
    assert err <= bar, f"{name}: max relative error {err:.3e} > {bar:.1e}"
    return err


def workspace(nbytes):
    return torch.empty(max(int(nbytes), 256), device="cuda", dtype=torch.uint8)
