"""ctypes binding of libwersa.so: argument marshalling only.

Function names mirror the C entry points of include/wersa.h.  Tensors are torch CUDA tensors
(torch supplies device memory and the stream; every step of the computation runs inside the
library's HIP kernels).  There is no CPU fallback: if the shared library is missing, loading
raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libwersa.so")

WERSA_F32, WERSA_BF16 = 0, 1
WERSA_FLAG_GENERIC_PATH = 1
EXPORTS = ["wersa_workspace_bytes", "wersa_saved_bytes", "wersa_forward", "wersa_backward",
           "wersa_forward_static", "wersa_static_scratch_bytes",
           "wersa_haar_filter", "wersa_haar_filter_ws", "wersa_haar_filter_workspace_bytes", "wersa_saved_offset", "wersa_selected_path", "wersa_status_string", "wersa_version",
           "wersa_profile_enable", "wersa_profile_only", "wersa_profile_reset", "wersa_profile_collect", "wersa_profile_get",
           "wersa_peak_copy", "wersa_peak_mfma",
           "wersa_block_workspace_bytes", "wersa_block_saved_bytes", "wersa_block_saved_offset",
           "wersa_block_workspace_offset",
           "wersa_block_forward", "wersa_block_backward"]


class WersaDesc(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("n", ctypes.c_int32),
                ("d", ctypes.c_int32), ("L", ctypes.c_int32), ("m", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("eps", ctypes.c_float), ("bw_floor", ctypes.c_float),
                ("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64),
                ("stride_n", ctypes.c_int64), ("flags", ctypes.c_int32)]


class WersaError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"wersa status {status}: {text}")
        self.status = status


_lib = None


def load_library():
    """Load libwersa.so (built by paper_2507_08637_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2507_08637_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, fp, dp = ctypes.c_void_p, ctypes.c_void_p, ctypes.POINTER(WersaDesc)
    lib.wersa_workspace_bytes.restype = ctypes.c_size_t
    lib.wersa_workspace_bytes.argtypes = [dp, ctypes.c_int]
    lib.wersa_saved_bytes.restype = ctypes.c_size_t
    lib.wersa_saved_bytes.argtypes = [dp]
    lib.wersa_selected_path.restype = ctypes.c_int32
    lib.wersa_selected_path.argtypes = [dp]
    lib.wersa_saved_offset.restype = ctypes.c_int64
    lib.wersa_saved_offset.argtypes = [dp, ctypes.c_int]
    lib.wersa_forward.restype = ctypes.c_int
    lib.wersa_forward.argtypes = [dp, vp, vp, vp, vp, fp, fp, fp, fp, vp, vp, vp, ctypes.c_size_t, vp]
    lib.wersa_forward_static.restype = ctypes.c_int
    lib.wersa_forward_static.argtypes = [dp, vp, vp, vp, vp, fp, fp, fp, fp, vp, vp, vp]
    lib.wersa_static_scratch_bytes.restype = ctypes.c_size_t
    lib.wersa_static_scratch_bytes.argtypes = []
    lib.wersa_backward.restype = ctypes.c_int
    lib.wersa_backward.argtypes = [dp] + [vp] * 4 + [fp] * 4 + [vp] * 3 + [vp] * 3 + [fp] * 4 + \
        [vp, ctypes.c_size_t, vp]
    lib.wersa_haar_filter.restype = ctypes.c_int
    lib.wersa_haar_filter.argtypes = [dp, vp, fp, vp, vp]
    lib.wersa_haar_filter_workspace_bytes.restype = ctypes.c_size_t
    lib.wersa_haar_filter_workspace_bytes.argtypes = [dp]
    lib.wersa_haar_filter_ws.restype = ctypes.c_int
    lib.wersa_haar_filter_ws.argtypes = [dp, vp, fp, vp, vp, ctypes.c_size_t, vp]
    lib.wersa_block_workspace_bytes.restype = ctypes.c_size_t
    lib.wersa_block_workspace_bytes.argtypes = [dp, ctypes.c_int]
    lib.wersa_block_saved_bytes.restype = ctypes.c_size_t
    lib.wersa_block_saved_bytes.argtypes = [dp]
    lib.wersa_block_saved_offset.restype = ctypes.c_int64
    lib.wersa_block_saved_offset.argtypes = [dp, ctypes.c_int]
    lib.wersa_block_workspace_offset.restype = ctypes.c_int64
    lib.wersa_block_workspace_offset.argtypes = [dp, ctypes.c_int]
    lib.wersa_block_forward.restype = ctypes.c_int
    lib.wersa_block_forward.argtypes = [dp] + [vp] * 6 + [fp] * 4 + [vp, vp, vp, ctypes.c_size_t, vp]
    lib.wersa_block_backward.restype = ctypes.c_int
    lib.wersa_block_backward.argtypes = [dp] + [vp] * 6 + [fp] * 4 + [vp, vp, vp] + [fp] * 8 + \
        [vp, ctypes.c_size_t, vp]
    lib.wersa_status_string.restype = ctypes.c_char_p
    lib.wersa_status_string.argtypes = [ctypes.c_int]
    lib.wersa_version.restype = ctypes.c_int32
    lib.wersa_version.argtypes = []
    lib.wersa_profile_enable.restype = None
    lib.wersa_profile_enable.argtypes = [ctypes.c_int]
    lib.wersa_profile_only.restype = None
    lib.wersa_profile_only.argtypes = [ctypes.c_char_p]
    lib.wersa_profile_reset.restype = None
    lib.wersa_profile_reset.argtypes = []
    lib.wersa_profile_collect.restype = ctypes.c_int32
    lib.wersa_profile_collect.argtypes = []
    lib.wersa_profile_get.restype = ctypes.c_int32
    lib.wersa_profile_get.argtypes = [ctypes.c_int32, ctypes.c_char_p, ctypes.c_int32,
                                      ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
    lib.wersa_peak_copy.restype = ctypes.c_double
    lib.wersa_peak_copy.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int32, vp]
    lib.wersa_peak_mfma.restype = ctypes.c_double
    lib.wersa_peak_mfma.argtypes = [fp, ctypes.c_int32, vp]
    _lib = lib
    return lib


def _check(status):
    if status != 0:
        raise WersaError(status, load_library().wersa_status_string(status).decode())


def wersa_path_name(desc):
    return {1: "mfma", 0: "generic"}.get(load_library().wersa_selected_path(ctypes.byref(desc)), "rejected")


def make_desc(x, L, m, eps=1e-6, bw_floor=1e-6, flags=0):
    """Descriptor for a (B, H, n, d) tensor x (last dim contiguous)."""
    assert x.dim() == 4 and x.stride(3) == 1, "expect (B, H, n, d) with contiguous last dim"
    B, H, n, d = x.shape
    if x.dtype == torch.float32:
        dt = WERSA_F32
    elif x.dtype == torch.bfloat16:
        dt = WERSA_BF16
    else:
        raise TypeError("dtype must be float32 or bfloat16")
    return WersaDesc(B, H, n, d, L, m, dt, eps, bw_floor, x.stride(0), x.stride(1), x.stride(2), flags)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _nbytes(t):
    return t.numel() * t.element_size()


def _scratch(nbytes, like, stream):
    """Temporary device buffer for one call.  The kernels that use it are only queued when the call
    returns, so the buffer must not go back to torch's allocator for reuse before they have run:
    with an explicit `stream` it is tied to that stream (the caching allocator then waits for the
    stream's queued work before handing the block to anyone else)."""
    buf = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=like.device)
    if stream is not None:
        buf.record_stream(stream)
    return buf


def _same_layout(ref, *others):
    for t in others:
        assert t.shape == ref.shape and t.stride() == ref.stride() and t.dtype == ref.dtype, \
            "q, k, v, out and gradients must share shape, strides and dtype"


FLAG_GENERIC_PATH = 1
FLAG_SEPARATE_OMEGA = 2
FLAG_POOLED_GATE = 4
FLAG_LAYERNORM = 8


def _check_omega(omega_rf, q, flags):
    """(d, m), or (2, d, m) with FLAG_SEPARATE_OMEGA: the query-side matrix, then the key-side one."""
    d = q.shape[3]
    assert omega_rf.is_contiguous() and omega_rf.dtype == q.dtype
    if flags & FLAG_SEPARATE_OMEGA:
        assert omega_rf.dim() == 3 and omega_rf.shape[0] == 2 and omega_rf.shape[1] == d
    else:
        assert omega_rf.dim() == 2 and omega_rf.shape[0] == d


def wersa_workspace_bytes(desc, for_backward):
    return load_library().wersa_workspace_bytes(ctypes.byref(desc), int(for_backward))


def wersa_saved_bytes(desc):
    return load_library().wersa_saved_bytes(ctypes.byref(desc))


def saved_views(desc, saved):
    """Named float32 views into the saved buffer: S, z, qbar, s, F, D."""
    lib = load_library()
    sl = desc.B * desc.H
    shapes = [("S", (sl, desc.m, desc.d)), ("z", (sl, desc.m)), ("qbar", (sl, desc.d)),
              ("s", (sl, desc.L + 1)), ("F", (sl, desc.L + 1)), ("D", (sl, desc.n))]
    out = {}
    for which, (name, shape) in enumerate(shapes):
        off = lib.wersa_saved_offset(ctypes.byref(desc), which)
        cnt = 1
        for s in shape:
            cnt *= s
        out[name] = saved[off:off + cnt].view(*shape)
    return out


def alloc_like(desc, ref, for_backward):
    """Allocate (saved, workspace) float32 buffers on ref's device."""
    lib = load_library()
    sb = lib.wersa_saved_bytes(ctypes.byref(desc))
    wb = lib.wersa_workspace_bytes(ctypes.byref(desc), int(for_backward))
    if sb == 0 or wb == 0:
        raise WersaError(2, "descriptor rejected (invalid or unsupported shape)")
    saved = torch.empty(sb // 4, dtype=torch.float32, device=ref.device)
    ws = torch.empty(wb // 4, dtype=torch.float32, device=ref.device)
    return saved, ws


def wersa_forward(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps=1e-6, bw_floor=1e-6,
                  out=None, saved=None, workspace=None, stream=None, flags=0):
    """Returns (out, saved).  All tensor arguments live on one CUDA device."""
    lib = load_library()
    _same_layout(q, k, v)
    desc = make_desc(q, L, omega_rf.shape[-1], eps, bw_floor, flags)
    _check_omega(omega_rf, q, flags)
    for p in (sigma, gate_w, gate_b, scale_w):
        assert p.dtype == torch.float32 and p.is_contiguous()
    if out is None:
        out = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    else:
        _same_layout(q, out)
    sb = lib.wersa_saved_bytes(ctypes.byref(desc))
    if sb == 0:
        _check(_probe(desc))
    if saved is None:
        saved = torch.empty(sb // 4, dtype=torch.float32, device=q.device)
    else:   # the C ABI takes no size for `saved`: checked here
        assert _nbytes(saved) >= sb, f"saved buffer holds {_nbytes(saved)} bytes, wersa_saved_bytes asks for {sb}"
    wb = lib.wersa_workspace_bytes(ctypes.byref(desc), 0)
    if workspace is None:
        workspace = _scratch(wb, q, stream)
    _check(lib.wersa_forward(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(omega_rf), _ptr(sigma),
                             _ptr(gate_w), _ptr(gate_b), _ptr(scale_w), _ptr(out), _ptr(saved),
                             _ptr(workspace), _nbytes(workspace), _stream(stream)))
    return out, saved


def wersa_forward_static(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, L, out, saved, eps=1e-6,
                         bw_floor=1e-6, stream=None, flags=0):
    """wersa_forward with the library's built-in scratch as the workspace: `out` and `saved` come
    from the caller and nothing is allocated here or in the library.  Returns (out, saved)."""
    lib = load_library()
    _same_layout(q, k, v, out)
    desc = make_desc(q, L, omega_rf.shape[-1], eps, bw_floor, flags)
    _check_omega(omega_rf, q, flags)
    sb = lib.wersa_saved_bytes(ctypes.byref(desc))
    assert sb == 0 or _nbytes(saved) >= sb, f"saved buffer holds {_nbytes(saved)} bytes, wersa_saved_bytes asks for {sb}"
    _check(lib.wersa_forward_static(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(omega_rf), _ptr(sigma),
                                    _ptr(gate_w), _ptr(gate_b), _ptr(scale_w), _ptr(out), _ptr(saved),
                                    _stream(stream)))
    return out, saved


def _probe(desc):
    # wersa_saved_bytes returned 0: ask the forward entry point for the precise status
    return load_library().wersa_forward(ctypes.byref(desc), *([None] * 11), 0, None)


def wersa_backward(q, k, v, omega_rf, sigma, gate_w, gate_b, scale_w, out, dout, saved, L,
                   eps=1e-6, bw_floor=1e-6, workspace=None, stream=None, param_grads=True, grads=None,
                   flags=0):
    """Returns dict(dq, dk, dv, dgate_w, dgate_b, dscale_w, dsigma).

    `grads` may be a dict from an earlier call: its tensors are then overwritten in place."""
    lib = load_library()
    _same_layout(q, k, v, out, dout)
    desc = make_desc(q, L, omega_rf.shape[-1], eps, bw_floor, flags)
    _check_omega(omega_rf, q, flags)
    if grads is not None:
        dq, dk, dv = grads["dq"], grads["dk"], grads["dv"]
        _same_layout(q, dq, dk, dv)
        dgw, dgb, dsw, dsg = grads["dgate_w"], grads["dgate_b"], grads["dscale_w"], grads["dsigma"]
    else:
        dq = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
        dk = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
        dv = torch.empty_strided(q.shape, q.stride(), dtype=q.dtype, device=q.device)
    if grads is not None:
        pass
    elif param_grads:
        dgw = torch.empty_like(gate_w)
        dgb = torch.empty_like(gate_b)
        dsw = torch.empty_like(scale_w)
        dsg = torch.empty(1, dtype=torch.float32, device=q.device)
    else:
        dgw = dgb = dsw = dsg = None
    wb = lib.wersa_workspace_bytes(ctypes.byref(desc), 1)
    if workspace is None:
        workspace = _scratch(wb, q, stream)
    sb = lib.wersa_saved_bytes(ctypes.byref(desc))
    assert sb == 0 or _nbytes(saved) >= sb, f"saved buffer holds {_nbytes(saved)} bytes, wersa_saved_bytes asks for {sb}"
    _check(lib.wersa_backward(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(omega_rf), _ptr(sigma),
                              _ptr(gate_w), _ptr(gate_b), _ptr(scale_w), _ptr(out), _ptr(dout),
                              _ptr(saved), _ptr(dq), _ptr(dk), _ptr(dv), _ptr(dgw), _ptr(dgb),
                              _ptr(dsw), _ptr(dsg), _ptr(workspace), _nbytes(workspace),
                              _stream(stream)))
    return dict(dq=dq, dk=dk, dv=dv, dgate_w=dgw, dgate_b=dgb, dscale_w=dsw, dsigma=dsg)


def wersa_haar_filter(x, filt, L, out=None, stream=None):
    """X_F = W^-1(F (.) W X) for x (B, H, n, d) and filt (B*H, L+1) float32."""
    lib = load_library()
    desc = make_desc(x, L, 16)
    assert filt.dtype == torch.float32 and filt.is_contiguous() and filt.numel() == x.shape[0] * x.shape[1] * (L + 1)
    if out is None:
        out = torch.empty_strided(x.shape, x.stride(), dtype=x.dtype, device=x.device)
    wb = lib.wersa_haar_filter_workspace_bytes(ctypes.byref(desc))
    if wb == 0:
        _check(lib.wersa_haar_filter(ctypes.byref(desc), _ptr(x), _ptr(filt), _ptr(out), _stream(stream)))
    else:   # levels above 6: the tiles' approximation coefficients go through a workspace
        ws = _scratch(wb, x, stream)
        _check(lib.wersa_haar_filter_ws(ctypes.byref(desc), _ptr(x), _ptr(filt), _ptr(out), _ptr(ws), wb,
                                        _stream(stream)))
    return out


def make_block_desc(x, H, L, m, eps=1e-6, bw_floor=1e-6, flags=0):
    """Descriptor for the attention block on x (B, n, hidden), hidden = H * d, dense bf16."""
    assert x.dim() == 3 and x.is_contiguous() and x.shape[2] % H == 0
    if x.dtype != torch.bfloat16:
        raise TypeError("the attention block takes bfloat16 tensors")
    B, n, hidden = x.shape
    d = hidden // H
    return WersaDesc(B, H, n, d, L, m, WERSA_BF16, eps, bw_floor, n * hidden, d, hidden, flags)


def block_saved_views(desc, saved):
    """bf16 views (B, n, hidden) of Q', K', V', A inside the block's saved byte buffer, and the
    core's saved buffer as float32."""
    lib = load_library()
    B, n, hidden = desc.B, desc.n, desc.H * desc.d
    out = {}
    for which, name in enumerate(("Qp", "Kp", "Vp", "A")):
        off = lib.wersa_block_saved_offset(ctypes.byref(desc), which)
        out[name] = saved[off:off + B * n * hidden * 2].view(torch.bfloat16).view(B, n, hidden)
    off = lib.wersa_block_saved_offset(ctypes.byref(desc), 4)
    out["core"] = saved[off:].view(torch.float32)
    return out


def block_workspace_views(desc, workspace):
    """bf16 views (B, n, hidden) of dA, dQ', dK', dV' left in the backward workspace."""
    lib = load_library()
    B, n, hidden = desc.B, desc.n, desc.H * desc.d
    out = {}
    for which, name in enumerate(("dA", "dQp", "dKp", "dVp")):
        off = lib.wersa_block_workspace_offset(ctypes.byref(desc), which)
        out[name] = workspace[off:off + B * n * hidden * 2].view(torch.bfloat16).view(B, n, hidden)
    return out


def _block_check_args(x, weights, omega_rf, params):
    hidden = x.shape[2]
    for w in weights:
        assert w.shape == (hidden, hidden) and w.is_contiguous() and w.dtype == x.dtype
    assert omega_rf.is_contiguous() and omega_rf.dtype == x.dtype
    for p in params:
        assert p.dtype == torch.float32 and p.is_contiguous()


def wersa_block_forward(x, wq, wk, wv, wo, H, omega_rf, sigma, gate_w, gate_b, scale_w, L, eps=1e-6,
                        bw_floor=1e-6, y=None, saved=None, workspace=None, stream=None, flags=0):
    """Returns (y, saved): y (B, n, hidden) bf16, saved a uint8 buffer for wersa_block_backward."""
    lib = load_library()
    desc = make_block_desc(x, H, L, omega_rf.shape[1], eps, bw_floor, flags)
    _block_check_args(x, (wq, wk, wv, wo), omega_rf, (sigma, gate_w, gate_b, scale_w))
    sb = lib.wersa_block_saved_bytes(ctypes.byref(desc))
    wb = lib.wersa_block_workspace_bytes(ctypes.byref(desc), 0)
    if sb == 0 or wb == 0:
        _check(lib.wersa_block_forward(ctypes.byref(desc), *([None] * 13), 0, None) or 2)
    if y is None:
        y = torch.empty_like(x)
    if saved is None:
        saved = torch.empty(sb, dtype=torch.uint8, device=x.device)
    else:
        assert _nbytes(saved) >= sb, f"saved buffer holds {_nbytes(saved)} bytes, wersa_block_saved_bytes asks for {sb}"
    if workspace is None:
        workspace = _scratch(wb, x, stream)
    _check(lib.wersa_block_forward(ctypes.byref(desc), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo),
                                   _ptr(omega_rf), _ptr(sigma), _ptr(gate_w), _ptr(gate_b), _ptr(scale_w),
                                   _ptr(y), _ptr(saved), _ptr(workspace), _nbytes(workspace), _stream(stream)))
    return y, saved


def wersa_block_backward(x, wq, wk, wv, wo, H, omega_rf, sigma, gate_w, gate_b, scale_w, dy, saved, L,
                         eps=1e-6, bw_floor=1e-6, workspace=None, stream=None, grads=None, flags=0):
    """Returns dict(dx, dwq, dwk, dwv, dwo, dgate_w, dgate_b, dscale_w, dsigma); weight gradients are
    float32.  `grads` may be a dict from an earlier call: its tensors are then overwritten."""
    lib = load_library()
    desc = make_block_desc(x, H, L, omega_rf.shape[1], eps, bw_floor, flags)
    _block_check_args(x, (wq, wk, wv, wo), omega_rf, (sigma, gate_w, gate_b, scale_w))
    assert dy.shape == x.shape and dy.is_contiguous() and dy.dtype == x.dtype
    wb = lib.wersa_block_workspace_bytes(ctypes.byref(desc), 1)
    if wb == 0:
        _check(lib.wersa_block_backward(ctypes.byref(desc), *([None] * 21), 0, None) or 2)
    if grads is None:
        f32 = dict(dtype=torch.float32, device=x.device)
        grads = dict(dx=torch.empty_like(x), dwq=torch.empty(wq.shape, **f32), dwk=torch.empty(wq.shape, **f32),
                     dwv=torch.empty(wq.shape, **f32), dwo=torch.empty(wq.shape, **f32),
                     dgate_w=torch.empty_like(gate_w), dgate_b=torch.empty_like(gate_b),
                     dscale_w=torch.empty_like(scale_w), dsigma=torch.empty(1, **f32))
    if workspace is None:
        workspace = _scratch(wb, x, stream)
    sb = lib.wersa_block_saved_bytes(ctypes.byref(desc))
    assert _nbytes(saved) >= sb, f"saved buffer holds {_nbytes(saved)} bytes, wersa_block_saved_bytes asks for {sb}"
    g = grads
    _check(lib.wersa_block_backward(ctypes.byref(desc), _ptr(x), _ptr(wq), _ptr(wk), _ptr(wv), _ptr(wo),
                                    _ptr(omega_rf), _ptr(sigma), _ptr(gate_w), _ptr(gate_b), _ptr(scale_w),
                                    _ptr(dy), _ptr(saved), _ptr(g["dx"]), _ptr(g["dwq"]), _ptr(g["dwk"]),
                                    _ptr(g["dwv"]), _ptr(g["dwo"]), _ptr(g["dgate_w"]), _ptr(g["dgate_b"]),
                                    _ptr(g["dscale_w"]), _ptr(g["dsigma"]), _ptr(workspace),
                                    _nbytes(workspace), _stream(stream)))
    return grads


def wersa_profile_enable(on, only=None):
    """Switch the event bracketing on or off; `only` restricts it to one kernel name."""
    lib = load_library()
    lib.wersa_profile_reset()
    lib.wersa_profile_only(only.encode() if only else None)
    lib.wersa_profile_enable(int(bool(on)))


def wersa_profile_collect():
    """{kernel name: (total_ms, launches)} for everything recorded since the last collect."""
    lib = load_library()
    cnt = lib.wersa_profile_collect()
    out = {}
    buf = ctypes.create_string_buffer(128)
    ms, launches = ctypes.c_double(), ctypes.c_int32()
    for i in range(cnt):
        if lib.wersa_profile_get(i, buf, 128, ctypes.byref(ms), ctypes.byref(launches)) == 0:
            out[buf.value.decode()] = (ms.value, launches.value)
    return out


def wersa_peak_copy(dst, src, reps=10, stream=None):
    """GB/s (read + written) of a plain streaming copy src -> dst, measured now on this device."""
    assert dst.is_contiguous() and src.is_contiguous() and dst.numel() * dst.element_size() == src.numel() * src.element_size()
    return load_library().wersa_peak_copy(_ptr(dst), _ptr(src), src.numel() * src.element_size() // 16 * 16, reps,
                                          _stream(stream))


def wersa_peak_mfma(reps=3, stream=None):
    """TFLOP/s of a loop of independent bf16 32x32x16 matrix instructions on every compute unit."""
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    return load_library().wersa_peak_mfma(_ptr(sink), reps, _stream(stream))
