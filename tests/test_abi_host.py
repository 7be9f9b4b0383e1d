"""Host-only checks of the C ABI: the library loads, exports everything include/phantom.h declares,
and rejects bad arguments before touching a GPU."""
import ctypes
import os
import re

import pytest

import paper_2508_00960_amd as ph

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "phantom.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(phantom_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(ph.library_path()) if os.path.exists(ph.library_path()) else ph.load()
    names = declared_functions()
    assert {"phantom_layer_fwd", "phantom_layer_bwd", "phantom_ffn_step", "phantom_workspace_bytes",
            "phantom_last_error"} <= set(names)
    for name in names:
        assert hasattr(lib, name), name
    assert ph.abi_version() == 4


def test_struct_layout_matches_header():
    assert ctypes.sizeof(ph.PhProblem) == 4 * 8 + 4 * 4 + 2 * 8
    from paper_2508_00960_amd.binding import PhStepArgs
    assert ctypes.sizeof(PhStepArgs) == 18 * 8 + 8 + 8
    from paper_2508_00960_amd.binding import PhStepTaps
    assert ctypes.sizeof(PhStepTaps) == 5 * 8
    from paper_2508_00960_amd.binding import PhProfileEntry
    assert ctypes.sizeof(PhProfileEntry) == 64 + 3 * 8 + 2 * 4 + 8 + 9 * 8


@pytest.mark.parametrize("kwargs,fragment", [
    (dict(n=255, p=4, k=8, batch=32), "multiples of p"),
    (dict(n=256, p=0, k=8, batch=32), "p ="),
    (dict(n=256, p=4, k=0, batch=32), "k ="),
    (dict(n=256, p=4, k=65, batch=32), "k ="),
    (dict(n=256, p=4, k=8, batch=0), "batch"),
    (dict(n=256, p=4, k=8, batch=32, rank=4), "rank"),
    (dict(n=256, p=4, k=8, batch=32, layers=0), "layers"),
    (dict(n=256, p=4, k=8, batch=32, layers=2, widths=(256, 130, 64), ks=(8, 8)), "multiples of p"),
    (dict(n=256, p=4, k=8, batch=32, layers=2, widths=(256, 128, 64), ks=(8, 33)), "k ="),
    (dict(n=256, p=4, k=8, batch=32, layers=2, widths=(256, 128, 64)), "widths without ks"),
])
def test_bad_problems_are_rejected(kwargs, fragment):
    prob = ph.make_problem(**kwargs)
    with pytest.raises(ph.PhantomError) as e:
        ph.workspace_bytes(prob)
    assert e.value.status == -1 and fragment in str(e.value)


def test_bad_enums_are_rejected():
    prob = ph.make_problem(256, 4, 8, 32)
    prob.act = 7
    with pytest.raises(ph.PhantomError, match="activation"):
        ph.workspace_bytes(prob)
    prob.act, prob.dtype = 0, 5
    with pytest.raises(ph.PhantomError, match="dtype"):
        ph.workspace_bytes(prob)


def test_null_and_misaligned_pointers_are_rejected_before_any_launch():
    prob = ph.make_problem(256, 4, 8, 32)
    ok = 0x1000
    with pytest.raises(ph.PhantomError, match="X is NULL"):
        ph.layer_fwd(prob, None, ok, ok, ok, ok, ok, ok, ok, None)
    with pytest.raises(ph.PhantomError, match="Y is not 16-byte aligned"):
        ph.layer_fwd(prob, ok, ok, ok, ok, ok, ok, ok + 8, ok, None)
    with pytest.raises(ph.PhantomError, match="G is NULL"):
        ph.layer_fwd(prob, ok, ok, ok, ok, ok, None, ok, ok, None)
    # p == 1 needs no C, D, G
    with pytest.raises(ph.PhantomError, match="dLw is NULL"):
        ph.layer_bwd(ph.make_problem(64, 1, 0, 8), ok, ok, ok, ok, None, None, None, None, ok, None, None, None, ok,
                     None, workspace=(0x2000, 1 << 30))
    with pytest.raises(ph.PhantomError) as e:
        ph.layer_bwd(prob, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, workspace=(0x2000, 16))
    assert e.value.status == -3 and "workspace" in str(e.value)


def test_step_checks_per_layer_pointer_arrays():
    prob = ph.make_problem(256, 4, 8, 32, layers=2, dtype="bf16")
    ok = 0x1000
    two = [ok, ok]
    with pytest.raises(ph.PhantomError, match=r"Lw_master"):
        ph.ffn_step(prob, ok, ok, two, two, two, two, G=two, dg_own=two, loss=ok, lr=0.1, workspace=(0x2000, 1 << 40))
    with pytest.raises(ph.PhantomError, match=r"Dw\[1\] is NULL"):
        ph.ffn_step(prob, ok, ok, two, two, [ok, None], two, G=two, mode="forward", workspace=(0x2000, 1 << 40))
    with pytest.raises(ValueError):
        ph.ffn_step(prob, ok, ok, [ok], two, two, two)


def test_capability_limits_are_found_before_any_launch():
    """A problem that is valid but beyond what the kernels index (PH_ERR_UNSUPPORTED) is refused from its shapes
    alone, on a host without a GPU: nothing can have been launched."""
    ok = 0x1000
    # 2^22 batch rows x 64 ranks of 2^22 neurons: 2^15 x 2^15 x 64 output tiles in the layer update
    huge = ph.make_problem((1 << 22) * 64, 64, 8, 1 << 22, dtype="bf16", rank=-1)
    with pytest.raises(ph.PhantomError) as e:
        ph.workspace_bytes(huge)
    assert e.value.status == -2 and "output tiles" in str(e.value)
    with pytest.raises(ph.PhantomError) as e:
        ph.layer_fwd(huge, ok, ok, ok, ok, ok, ok, ok, ok, None)
    assert e.value.status == -2
    with pytest.raises(ph.PhantomError) as e:
        ph.ffn_step(huge, ok, ok, [ok], [ok], [ok], [ok], loss=ok, mode="no_update", workspace=(0x2000, 1 << 40))
    assert e.value.status == -2
    wide = ph.make_problem((1 << 23) * 2, 2, 8, 16, dtype="bf16")      # n/p beyond 2^22
    with pytest.raises(ph.PhantomError) as e:
        ph.workspace_bytes(wide)
    assert e.value.status == -2


def test_production_library_reads_no_tuning_variable(monkeypatch):
    """The switches that force a launch schedule exist only in a build made for measurements."""
    data = open(ph.library_path(), "rb").read()
    for name in (b"PHANTOM_DUAL", b"PHANTOM_TAIL_DUAL", b"PHANTOM_PAIR", b"PHANTOM_FWD_PAIR", b"PHANTOM_RS_ON_READ"):
        assert name not in data, name


def test_step_taps_are_checked():
    prob = ph.make_problem(256, 4, 8, 32, layers=2, dtype="bf16")
    ok = 0x1000
    two = [ok, ok]
    with pytest.raises(ph.PhantomError, match=r"taps.delta\[1\] is not 16-byte aligned"):
        ph.ffn_step(prob, ok, ok, two, two, two, two, G=two, dg_own=two, loss=ok, mode="no_update",
                    workspace=(0x2000, 1 << 40), taps={"delta": [ok, ok + 4]})


def test_static_step_refuses_a_problem_beyond_its_scratch_array_on_the_host():
    big = ph.make_problem(16384, 16, 64, 4096, 8, "gelu", "bf16", 0)
    assert ph.workspace_bytes(big) > ph.static_workspace_bytes() == 64 << 20
    ok = 0x1000
    eight = [ok] * 8
    with pytest.raises(ph.PhantomError) as e:
        ph.ffn_step_static(big, ok, ok, eight, eight, eight, eight, G=eight, dg_own=eight, loss=ok, mode="no_update")
    assert e.value.status == -3 and "scratch" in str(e.value)


def test_workspace_grows_with_the_problem():
    small = ph.workspace_bytes(ph.make_problem(256, 4, 8, 32, layers=2))
    big = ph.workspace_bytes(ph.make_problem(4096, 8, 32, 1024, layers=4, dtype="bf16", rank=-1))
    assert 0 < small < big


def test_binding_refuses_host_tensors():
    """The library gets addresses only: the binding stops a tensor that is not device memory before the call."""
    import torch
    prob = ph.make_problem(256, 4, 8, 32)
    ok = 0x1000
    with pytest.raises(ValueError, match="X: tensor is on cpu"):
        ph.layer_fwd(prob, torch.zeros(32, 64), ok, ok, ok, ok, ok, ok, ok, None)
