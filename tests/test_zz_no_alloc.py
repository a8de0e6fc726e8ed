"""wersa_forward_static (the forward with the library's built-in scratch as its workspace, for
callers that cannot allocate) against wersa_forward on the same inputs: same kernels, same
reduction order, so every output must agree bit for bit, which is inside the bf16 / float32
tolerance by a wide margin.  Two calls in a row share the scratch array, the second on a smaller
problem (stale contents of the first must not leak into it)."""
import ctypes

import numpy as np
import pytest

from paper_2507_08637_amd import workloads
from tests import helpers as hp

pytestmark = pytest.mark.gpu


def _run_both(cfg, flags=0):
    import torch
    from paper_2507_08637_amd import binding
    p = workloads.make_inputs(**cfg)
    t = hp.to_device(p, cfg["dtype"])
    L = cfg["L"]
    args = (t["Q"], t["K"], t["V"], t["Omega"], t["sigma"], t["Wg"], t["bg"], t["omega"], L)
    ref_out, ref_saved = binding.wersa_forward(*args, flags=flags)
    desc = binding.make_desc(t["Q"], L, cfg["m"], flags=flags)
    out = torch.full_like(t["Q"], float("nan"))
    saved = torch.full((binding.wersa_saved_bytes(desc) // 4,), float("nan"), dtype=torch.float32, device="cuda")
    binding.wersa_forward_static(*args, out, saved, flags=flags)
    torch.cuda.synchronize()
    assert torch.equal(out, ref_out), "O differs from wersa_forward"
    a, b = binding.saved_views(desc, saved), binding.saved_views(desc, ref_saved)
    for name in ("S", "z", "qbar", "s", "F", "D"):
        assert torch.equal(a[name], b[name]), name
    # and the oracle agrees with both (the bar of the parity tests)
    ref = hp.oracle_forward(p, cfg, keep=("O",))
    e = hp.rel_err(out, ref["O"])
    assert e < (1e-4 if cfg["dtype"] == "f32" else 2e-2), e
    return out, saved


def test_forward_static_matches_forward_twice_in_a_row_second_call_smaller():
    from paper_2507_08637_amd import binding
    lib = binding.load_library()
    assert lib.wersa_static_scratch_bytes() == 40 << 20
    big = dict(B=2, H=4, n=8192, d=64, L=6, m=256, dtype="bf16", flavour="plain", seed_base=6100, q_mean=0.3)
    small = dict(B=1, H=2, n=1000, d=64, L=5, m=128, dtype="bf16", flavour="plain", seed_base=6200, q_mean=0.3)
    _run_both(big)
    _run_both(small)
    _run_both(dict(B=1, H=2, n=700, d=48, L=3, m=80, dtype="f32", flavour="plain", seed_base=6300, q_mean=0.3))   # generic path
    _run_both(dict(B=1, H=2, n=2048, d=128, L=6, m=256, dtype="bf16", flavour="plain", seed_base=6400))            # head dimension 128


def test_forward_static_rejects_what_does_not_fit():
    """A problem whose workspace exceeds the built-in scratch is refused before anything runs."""
    import torch
    from paper_2507_08637_amd import binding
    lib = binding.load_library()
    q = torch.zeros(1, 8, 131072, 64, dtype=torch.bfloat16, device="cuda")
    desc = binding.make_desc(q, 6, 256, flags=binding.FLAG_GENERIC_PATH)   # generic path at this size: gigabytes of workspace
    assert lib.wersa_workspace_bytes(ctypes.byref(desc), 0) > lib.wersa_static_scratch_bytes()
    one = ctypes.c_void_p(q.data_ptr())
    assert lib.wersa_forward_static(ctypes.byref(desc), *([one] * 10), None) == 3
    # benchmark configuration 4 on the MFMA path fits
    fits = binding.make_desc(q, 6, 256)
    assert 0 < lib.wersa_workspace_bytes(ctypes.byref(fits), 0) <= lib.wersa_static_scratch_bytes()
