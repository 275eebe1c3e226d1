"""ctypes binding for libvla.so: argument marshalling only.

Every step of the recurrence runs in the HIP kernels behind the C ABI
(include/vla.h); there is no Python or CPU fallback -- if the shared library is
missing, loading raises.
"""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libvla.so"

VLA_F32, VLA_BF16 = 0, 1
MODE_AUTO, MODE_SCAN, MODE_CHUNKED, MODE_TWO_PHASE, MODE_TIME_PARALLEL = 0, 1, 2, 3, 4

EXPORTS = ("vla_default_opts", "vla_forward_workspace_bytes", "vla_forward", "vla_forward_static",
           "vla_decode_step", "vla_status_string", "vla_version", "vla_resolve_mode")


class VlaError(RuntimeError):
    def __init__(self, status, name):
        super().__init__(f"vla_forward failed: {name} ({status})")
        self.status = status


class VlaOpts(ctypes.Structure):
    _fields_ = [("lambda0", ctypes.c_float), ("eps", ctypes.c_float), ("mode", ctypes.c_int),
                ("u", ctypes.c_void_p), ("u_scale", ctypes.c_float), ("refresh_period", ctypes.c_int),
                ("refresh_eta", ctypes.c_float), ("step_offset", ctypes.c_int),
                ("normalise_output", ctypes.c_int), ("feature_map", ctypes.c_int),
                ("zkey0", ctypes.c_void_p), ("zkey_T", ctypes.c_void_p), ("segments", ctypes.c_int)]


_lib = None


def lib_path() -> str:
    return os.path.join(HERE, _LIB_NAME)


def load_library():
    """Load libvla.so (built in-tree by paper_2605_11196_amd/build.py). Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch owns the device memory and the streams handed to the library, so libvla must bind
    # to the HIP runtime instance torch has loaded: import torch before dlopen-ing libvla.so
    # (loading in the other order would bring a second, separate copy of the runtime).
    import torch  # noqa: F401

    path = lib_path()
    if not os.path.exists(path):
        raise FileNotFoundError(
            f"{path} not found: build it with `python -m paper_2605_11196_amd.build` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    P, I = ctypes.c_void_p, ctypes.c_int
    OP = ctypes.POINTER(VlaOpts)
    lib.vla_default_opts.argtypes = [OP]
    lib.vla_default_opts.restype = None
    lib.vla_forward_workspace_bytes.argtypes = [I] * 6 + [OP]
    lib.vla_forward_workspace_bytes.restype = ctypes.c_size_t
    lib.vla_forward.argtypes = [P] * 8 + [I] * 6 + [OP, P, ctypes.c_size_t, P]
    lib.vla_forward.restype = I
    lib.vla_forward_static.argtypes = [P] * 8 + [I] * 6 + [OP, P]
    lib.vla_forward_static.restype = I
    lib.vla_decode_step.argtypes = [P] * 6 + [I] * 5 + [OP, P]
    lib.vla_decode_step.restype = I
    lib.vla_status_string.argtypes = [I]
    lib.vla_status_string.restype = ctypes.c_char_p
    lib.vla_version.argtypes = []
    lib.vla_version.restype = I
    lib.vla_resolve_mode.argtypes = [I] * 6 + [OP]
    lib.vla_resolve_mode.restype = I
    _lib = lib
    return lib


def version() -> int:
    return int(load_library().vla_version())


def status_string(status: int) -> str:
    return load_library().vla_status_string(int(status)).decode()


def _opts(lambda0, eps, mode, extra=None):
    o = VlaOpts()
    load_library().vla_default_opts(ctypes.byref(o))
    if lambda0 is not None:
        o.lambda0 = float(lambda0)
    if eps is not None:
        o.eps = float(eps)
    if mode is not None:
        o.mode = int(mode)
    for key, val in (extra or {}).items():   # u, u_scale, refresh_period, ... (addresses as int)
        if val is not None:
            setattr(o, key, val)
    return o


def vla_forward_workspace_bytes(B, H, T, d_k, d_v, io_dtype, *, lambda0=None, eps=None,
                                mode=None, segments=None, **extra) -> int:
    """`extra`: further vla_opts fields by name, as in vla_forward_raw."""
    o = _opts(lambda0, eps, mode, dict(extra, segments=segments))
    return int(load_library().vla_forward_workspace_bytes(B, H, T, d_k, d_v, io_dtype,
                                                          ctypes.byref(o)))


def resolve_mode(B, H, T, d_k, d_v, io_dtype, *, mode=None, **extra) -> int:
    """`extra`: further vla_opts fields by name, as in vla_forward_raw."""
    o = _opts(None, None, mode, extra)
    return int(load_library().vla_resolve_mode(B, H, T, d_k, d_v, io_dtype, ctypes.byref(o)))


def vla_forward_raw(q, k, v, S0, A0, o, S_T, A_T, B, H, T, d_k, d_v, io_dtype, *, lambda0=None,
                    eps=None, mode=None, workspace=0, workspace_bytes=0, stream=0, **extra) -> int:
    """Direct call with integer device addresses (0 = NULL); returns the vla_status.
    `extra`: further vla_opts fields by name (u, zkey0, zkey_T as integer addresses)."""
    op = _opts(lambda0, eps, mode, extra)
    n = lambda x: ctypes.c_void_p(int(x) if x else None)
    return int(load_library().vla_forward(n(q), n(k), n(v), n(S0), n(A0), n(o), n(S_T), n(A_T),
                                          B, H, T, d_k, d_v, io_dtype, ctypes.byref(op),
                                          n(workspace), int(workspace_bytes), n(stream)))


def vla_forward_static_raw(q, k, v, S0, A0, o, S_T, A_T, B, H, T, d_k, d_v, io_dtype, *, lambda0=None,
                           eps=None, mode=None, stream=0, **extra) -> int:
    """vla_forward_raw without a workspace: the library's static array serves the modes that need one."""
    op = _opts(lambda0, eps, mode, extra)
    n = lambda x: ctypes.c_void_p(int(x) if x else None)
    return int(load_library().vla_forward_static(n(q), n(k), n(v), n(S0), n(A0), n(o), n(S_T), n(A_T),
                                                 B, H, T, d_k, d_v, io_dtype, ctypes.byref(op), n(stream)))


def vla_decode_step_raw(q, k, v, S, A, o, B, H, d_k, d_v, io_dtype, *, eps=None, stream=0, **extra) -> int:
    """Direct call with integer device addresses; returns the vla_status."""
    op = _opts(None, eps, None, extra)
    n = lambda x: ctypes.c_void_p(int(x) if x else None)
    return int(load_library().vla_decode_step(n(q), n(k), n(v), n(S), n(A), n(o), B, H, d_k, d_v,
                                              io_dtype, ctypes.byref(op), n(stream)))


def vla_decode_step(q, k, v, S, A, *, eps=None, stream=None, u=None, u_scale=None, refresh_period=None,
                    refresh_eta=None, step_offset=None, normalise_output=None, feature_map=None, zkey=None):
    """One token for every head: q, k, v [B,H,d] on the GPU (float32 or bfloat16); S, A [B,H,d,d] float32 are
    updated in place, and so is `zkey` [B,H,d] float32 (the running key sum of the normalised read-out) when
    given.  The optional lines of Algorithm 1 are switched on as in vla_forward; this call is step
    step_offset + 1 of the refresh schedule.  Returns o [B,H,d]."""
    import torch

    if not (q.is_cuda and k.is_cuda and v.is_cuda and S.is_cuda and A.is_cuda):
        raise ValueError("all tensors must be on the GPU (no CPU path exists)")
    if q.dtype == torch.float32:
        io = VLA_F32
    elif q.dtype == torch.bfloat16:
        io = VLA_BF16
    else:
        raise ValueError(f"unsupported dtype {q.dtype}")
    if k.dtype != q.dtype or v.dtype != q.dtype or q.dim() != 3 or k.shape != q.shape or v.shape[:2] != q.shape[:2]:
        raise ValueError("expected q,k [B,H,d_k] and v [B,H,d_v] of one dtype")
    B, H, dk = q.shape
    dv = v.shape[-1]
    for name, x, shape in (("S", S, (B, H, dv, dk)), ("A", A, (B, H, dk, dk)), ("zkey", zkey, (B, H, dk))):
        if x is not None and (x.dtype != torch.float32 or tuple(x.shape) != shape or not x.is_contiguous()
                              or x.device != q.device):
            raise ValueError(f"{name} must be a contiguous float32 tensor of shape {shape} on {q.device}")
    if u is not None and (u.dtype != q.dtype or tuple(u.shape) != tuple(q.shape) or u.device != q.device):
        raise ValueError("u must match q in dtype, shape and device")
    q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
    u = None if u is None else u.contiguous()
    p = lambda x: None if x is None else x.data_ptr()
    with torch.cuda.device(q.device):
        o = torch.empty((B, H, dv), dtype=q.dtype, device=q.device)
        st = stream if stream is not None else torch.cuda.current_stream(q.device)
        handle = st.cuda_stream if hasattr(st, "cuda_stream") else int(st)
        if isinstance(st, torch.cuda.Stream):
            o.record_stream(st)
        extra = dict(u=p(u), u_scale=u_scale, refresh_period=refresh_period, refresh_eta=refresh_eta,
                     step_offset=step_offset,
                     normalise_output=None if normalise_output is None else int(bool(normalise_output)),
                     feature_map=None if feature_map is None else int(bool(feature_map)),
                     zkey0=p(zkey), zkey_T=p(zkey))
        rc = vla_decode_step_raw(q.data_ptr(), k.data_ptr(), v.data_ptr(), S.data_ptr(), A.data_ptr(),
                                 o.data_ptr(), B, H, dk, dv, io, eps=eps, stream=handle, **extra)
    if rc != 0:
        raise VlaError(rc, status_string(rc))
    return o


def vla_forward(q, k, v, S0=None, A0=None, *, lambda0=None, eps=None, mode=None, stream=None,
                return_state=True, u=None, u_scale=None, refresh_period=None, refresh_eta=None,
                step_offset=None, normalise_output=None, feature_map=None, zkey0=None,
                return_zkey=False, segments=None):
    """Torch-tensor front end: q,k [B,H,T,d_k], v [B,H,T,d_v] on the GPU (float32 or bfloat16).

    Allocates o (and S_T, A_T, workspace) with torch, enqueues the kernels on `stream`
    (a torch.cuda.Stream; default: torch's current stream) and returns (o, S_T, A_T).  The outputs are ready
    when the work on `stream` is: a caller that reads them on another stream orders the two itself.
    """
    import torch

    if not (q.is_cuda and k.is_cuda and v.is_cuda):
        raise ValueError("q, k, v must be GPU tensors (no CPU path exists)")
    if q.dtype == torch.float32:
        io = VLA_F32
    elif q.dtype == torch.bfloat16:
        io = VLA_BF16
    else:
        raise ValueError(f"unsupported dtype {q.dtype}")
    if k.dtype != q.dtype or v.dtype != q.dtype:
        raise ValueError("q, k, v must share a dtype")
    if q.dim() != 4 or k.shape != q.shape or v.shape[:3] != q.shape[:3]:
        raise ValueError("expected q,k [B,H,T,d_k] and v [B,H,T,d_v]")
    q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
    B, H, T, dk = q.shape
    dv = v.shape[-1]
    dev = q.device
    for name, s, shape in (("S0", S0, (B, H, dv, dk)), ("A0", A0, (B, H, dk, dk))):
        if s is not None and (s.dtype != torch.float32 or tuple(s.shape) != shape
                              or not s.is_contiguous() or s.device != dev):
            raise ValueError(f"{name} must be a contiguous float32 tensor of shape {shape} on {dev}")
    st = stream if stream is not None else torch.cuda.current_stream(dev)
    handle = st.cuda_stream if hasattr(st, "cuda_stream") else int(st)
    p = lambda x: 0 if x is None else x.data_ptr()
    if u is not None:
        if u.dtype != q.dtype or tuple(u.shape) != tuple(q.shape) or u.device != dev:
            raise ValueError("u must match q in dtype, shape and device")
        u = u.contiguous()
    if zkey0 is not None and (zkey0.dtype != torch.float32 or tuple(zkey0.shape) != (B, H, dk)
                              or not zkey0.is_contiguous() or zkey0.device != dev):
        raise ValueError(f"zkey0 must be a contiguous float32 tensor of shape {(B, H, dk)} on {dev}")
    with torch.cuda.device(dev):
        o = torch.empty((B, H, T, dv), dtype=q.dtype, device=dev)
        S_T = torch.empty((B, H, dv, dk), dtype=torch.float32, device=dev) if return_state else None
        A_T = torch.empty((B, H, dk, dk), dtype=torch.float32, device=dev) if return_state else None
        zkey_T = torch.empty((B, H, dk), dtype=torch.float32, device=dev) if return_zkey else None
        extra = dict(u=p(u) or None, u_scale=u_scale, refresh_period=refresh_period,
                     refresh_eta=refresh_eta, step_offset=step_offset,
                     normalise_output=None if normalise_output is None else int(bool(normalise_output)),
                     feature_map=None if feature_map is None else int(bool(feature_map)),
                     zkey0=p(zkey0) or None, zkey_T=p(zkey_T) or None, segments=segments)
        # the same options as the call, so that the query resolves AUTO to the mode the call will run
        need = vla_forward_workspace_bytes(B, H, T, dk, dv, io, lambda0=lambda0, eps=eps, mode=mode, **extra)
        ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=dev) if need else None
        # These tensors come from the allocator of torch's current stream while the kernels run on `st`: tell the
        # allocator, so that memory dropped here (the workspace when this function returns) is not handed to
        # other work before the kernels on `st` are done with it.
        if isinstance(st, torch.cuda.Stream):
            for t in (o, S_T, A_T, zkey_T, ws):
                if t is not None:
                    t.record_stream(st)
        rc = vla_forward_raw(p(q), p(k), p(v), p(S0), p(A0), p(o), p(S_T), p(A_T), B, H, T, dk, dv,
                             io, lambda0=lambda0, eps=eps, mode=mode, workspace=p(ws),
                             workspace_bytes=need, stream=handle, **extra)
    if rc != 0:
        raise VlaError(rc, status_string(rc))
    if return_zkey:
        return o, S_T, A_T, zkey_T
    return o, S_T, A_T
