"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and turns bad arguments into error codes before anything is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2507_08637_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2507_08637_amd import build
        build.build()
    return binding.load_library()


def _desc(**kw):
    from paper_2507_08637_amd.binding import WersaDesc
    base = dict(B=1, H=2, n=256, d=64, L=3, m=64, dtype=0, eps=1e-6, bw_floor=1e-6,
                stride_b=2 * 256 * 64, stride_h=256 * 64, stride_n=64, flags=0)
    base.update(kw)
    return WersaDesc(**base)


def test_header_symbols_are_exported(lib):
    with open(os.path.join(ROOT, "include", "wersa.h")) as f:
        text = f.read()
    declared = set(re.findall(r"\b(wersa_[a-z_]+)\s*\(", text))
    assert declared, "no declarations found"
    from paper_2507_08637_amd import binding
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_sizes_and_status_strings(lib):
    d = _desc()
    assert lib.wersa_saved_bytes(ctypes.byref(d)) > 0
    assert lib.wersa_workspace_bytes(ctypes.byref(d), 1) >= lib.wersa_workspace_bytes(ctypes.byref(d), 0) > 0
    offs = [lib.wersa_saved_offset(ctypes.byref(d), w) for w in range(6)]
    assert offs == sorted(offs) and offs[0] == 0
    assert lib.wersa_saved_offset(ctypes.byref(d), 6) == -1
    assert lib.wersa_status_string(0) == b"ok"
    assert lib.wersa_version() >= 100


@pytest.mark.parametrize("kw,status", [
    (dict(B=0), 1), (dict(n=0), 1), (dict(L=-1), 1), (dict(dtype=7), 1), (dict(bw_floor=0.0), 1),
    (dict(stride_n=32), 1), (dict(stride_h=0), 1), (dict(flags=1 << 20), 1),
    (dict(L=21, n=1024), 2), (dict(d=40), 2), (dict(m=72), 2), (dict(d=512, stride_n=512), 2),
])
def test_bad_descriptors_are_rejected_before_launch(lib, kw, status):
    assert lib.wersa_saved_bytes(ctypes.byref(_desc(n=100, L=3))) > 0   # any n: padding is done in-kernel
    d = _desc(**kw)
    one = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    args = [one] * 4 + [one] * 4 + [one, one, one, 1 << 40, None]
    assert lib.wersa_forward(ctypes.byref(d), *args) == status
    assert lib.wersa_saved_bytes(ctypes.byref(d)) == 0
    assert lib.wersa_workspace_bytes(ctypes.byref(d), 0) == 0


def test_null_pointers_and_small_workspace(lib):
    d = _desc()
    one = ctypes.c_void_p(256)
    assert lib.wersa_forward(None, *([one] * 11), 1 << 40, None) == 1
    assert lib.wersa_forward(ctypes.byref(d), None, *([one] * 10), 1 << 40, None) == 1
    assert lib.wersa_forward(ctypes.byref(d), *([one] * 11), 16, None) == 3          # too small
    assert lib.wersa_forward(ctypes.byref(d), *([one] * 10), ctypes.c_void_p(264), 1 << 40, None) == 3
    bw = [one] * 4 + [one] * 4 + [one] * 3 + [one] * 3 + [None] * 4
    assert lib.wersa_backward(ctypes.byref(d), *bw, one, 16, None) == 3
    assert lib.wersa_backward(ctypes.byref(d), *([one] * 4 + [one] * 4 + [one, None, one] + [one] * 3 + [None] * 4),
                              one, 1 << 40, None) == 1
    assert lib.wersa_haar_filter(ctypes.byref(d), None, one, one, None) == 1
    # the stage entry point: no workspace needed up to six levels, a deeper transform needs one
    assert lib.wersa_haar_filter_workspace_bytes(ctypes.byref(d)) == 0
    assert lib.wersa_haar_filter_ws(ctypes.byref(d), None, one, one, None, 0, None) == 1
    deep = _desc(n=8192, L=9, stride_b=2 * 8192 * 64, stride_h=8192 * 64)
    need = lib.wersa_haar_filter_workspace_bytes(ctypes.byref(deep))
    assert need == 2 * 128 * 64 * 4          # one approximation row per 64-row tile, per slice and column
    assert lib.wersa_haar_filter(ctypes.byref(deep), one, one, one, None) == 2             # unsupported without
    assert lib.wersa_haar_filter_ws(ctypes.byref(deep), one, one, one, None, 0, None) == 3
    assert lib.wersa_haar_filter_ws(ctypes.byref(deep), one, one, one, one, need - 4, None) == 3
    assert lib.wersa_haar_filter_ws(ctypes.byref(deep), one, one, one, ctypes.c_void_p(264), need, None) == 3


def test_stated_limits_alignment_and_block_strides(lib):
    """What the header states: at most 1023 slices and 2^22 rows; on the MFMA path the tensor
    pointers are 16-byte aligned (checked before anything is enqueued); the block entry points
    ignore the descriptor's stride fields."""
    from paper_2507_08637_amd.binding import WersaDesc
    big = _desc(B=64, H=16, stride_b=16 * 256 * 64)
    assert lib.wersa_saved_bytes(ctypes.byref(big)) == 0 and lib.wersa_selected_path(ctypes.byref(big)) == -1
    assert lib.wersa_selected_path(ctypes.byref(_desc(B=33, H=31, stride_b=31 * 256 * 64))) == 0
    long = _desc(n=(1 << 22) + 1, stride_h=((1 << 22) + 1) * 64, stride_b=2 * ((1 << 22) + 1) * 64)
    assert lib.wersa_saved_bytes(ctypes.byref(long)) == 0
    # MFMA path (bf16, d = 64, m % 128 == 0): a pointer that is 2-byte but not 16-byte aligned
    fast = _desc(dtype=1, m=128)
    assert lib.wersa_selected_path(ctypes.byref(fast)) == 1
    ok, odd = ctypes.c_void_p(256), ctypes.c_void_p(258)
    huge = 1 << 40
    fwd = lambda q=ok, out=ok: lib.wersa_forward(ctypes.byref(fast), q, ok, ok, ok, ok, ok, ok, ok, out, ok, ok, huge, None)
    assert fwd(q=odd) == 1 and fwd(out=odd) == 1
    bwd = [ok] * 4 + [ok] * 4 + [ok, ok, ok] + [ok, odd, ok] + [None] * 4
    assert lib.wersa_backward(ctypes.byref(fast), *bwd, ok, huge, None) == 1
    # the same pointers on the generic path pass validation up to the workspace check
    gen = _desc(dtype=1, m=128, flags=1)
    assert lib.wersa_forward(ctypes.byref(gen), odd, ok, ok, ok, ok, ok, ok, ok, ok, ok, ok, 16, None) == 3
    # attention block: strides left at zero by a C caller
    blk = WersaDesc(B=2, H=4, n=256, d=64, L=3, m=128, dtype=1, eps=1e-6, bw_floor=1e-6, stride_b=0, stride_h=0,
                    stride_n=0, flags=0)
    assert lib.wersa_block_saved_bytes(ctypes.byref(blk)) > 0
    assert lib.wersa_block_workspace_bytes(ctypes.byref(blk), 1) > 0
    with_strides = WersaDesc(B=2, H=4, n=256, d=64, L=3, m=128, dtype=1, eps=1e-6, bw_floor=1e-6,
                             stride_b=256 * 256, stride_h=64, stride_n=256, flags=0)
    assert lib.wersa_block_saved_bytes(ctypes.byref(blk)) == lib.wersa_block_saved_bytes(ctypes.byref(with_strides))
    assert lib.wersa_block_forward(ctypes.byref(blk), *([ok] * 13), 16, None) == 3   # reaches the workspace check
    # the microbenchmarks refuse bad arguments without touching the device
    assert lib.wersa_peak_copy(None, ok, 1 << 20, 1, None) == -1.0
    assert lib.wersa_peak_mfma(None, 1, None) == -1.0
