"""MI355X-native phantom-layer operators (forward, backward, training step).

Thin binding over libphantom.so; see include/phantom.h for the contract.
"""
from .binding import (  # noqa: F401
    ACTS, DTYPES, STEP_MODES, PhantomError, PhProblem, abi_version, ffn_step, ffn_step_static, layer_bwd, layer_fwd, last_error,
    library_path, load, make_problem, profile_begin, profile_end, static_workspace_bytes, workspace_bytes,
)
