"""ctypes binding of ``libsdtw_hip.so`` (the C-ABI of ``include/sdtw.h``).

Argument marshalling only: every function here checks shapes and dtypes, passes device
pointers through, and raises :class:`SdtwError` on a non-zero status.  PyTorch supplies
device memory and the current stream; nothing is computed in Python and there is no
fallback: if the library has not been built, the first call raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libsdtw_hip.so")
_lib = None

UNFUSED = 0
FUSED = 1
FLAG_VALUE_ONLY = 1
FLAG_MIN_MEMORY = 2
FLAG_DENSE_E = 4
EXPORT_COST, EXPORT_R, EXPORT_E = 0, 1, 2

STATUS_OK = 0
STATUS_INVALID_ARG = 1
STATUS_WORKSPACE = 2
STATUS_UNSUPPORTED = 3
STATUS_STATE = 4
STATUS_HIP = 5
STATUS_TIMEOUT = 6


class SdtwError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: status %d (%s)" % (where, status, sdtw_status_string(status)))


class Desc(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("N", ctypes.c_int32), ("M", ctypes.c_int32), ("D", ctypes.c_int32),
        ("gamma", ctypes.c_float), ("mode", ctypes.c_int32),
        ("x_batch_stride", ctypes.c_int64), ("y_batch_stride", ctypes.c_int64),
        ("bandwidth", ctypes.c_int32), ("flags", ctypes.c_uint32),
    ]


class BaryDesc(ctypes.Structure):
    _fields_ = [
        ("K", ctypes.c_int32), ("Lz", ctypes.c_int32), ("Lx", ctypes.c_int32), ("D", ctypes.c_int32),
        ("gamma", ctypes.c_float), ("mode", ctypes.c_int32),
        ("lr", ctypes.c_float), ("beta1", ctypes.c_float), ("beta2", ctypes.c_float), ("eps", ctypes.c_float),
        ("step", ctypes.c_int32), ("flags", ctypes.c_uint32),
    ]


EXPORTED_SYMBOLS = (
    "sdtw_version", "sdtw_status_string", "sdtw_workspace_bytes", "sdtw_forward", "sdtw_backward",
    "sdtw_barycenter_workspace_bytes", "sdtw_barycenter_step", "sdtw_workspace_status",
    "sdtw_normalized_workspace_bytes", "sdtw_normalized_forward", "sdtw_normalized_backward",
    "sdtw_forward_ragged", "sdtw_backward_ragged",
    "sdtw_debug_export", "sdtw_debug_lane_shift", "sdtw_debug_set_spin_limit",
    "sdtw_debug_profile", "sdtw_debug_profile_read", "sdtw_debug_force_workgroup_shape",
    "sdtw_debug_rate_probe", "sdtw_forward_static_scratch", "sdtw_debug_set_pool_blocks",
    "sdtw_half_workspace_bytes", "sdtw_forward_half", "sdtw_backward_half",
)


def library_path():
    return _LIB_PATH


def load_library():
    """Loads the HIP library; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            "libsdtw_hip.so is missing at %s: run `python -c 'import __graft_entry__ as g; g.build()'` "
            "from the repository root" % _LIB_PATH)
    # PyTorch first: its wheel brings a HIP runtime of its own, and the tensors this binding hands over
    # live in that runtime.  Loaded after it, this library binds to the same one; loaded before it, the
    # process would end up with two (the calls then fail with a HIP runtime error).
    import torch  # noqa: F401

    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    lib.sdtw_version.restype = i32
    lib.sdtw_status_string.restype = ctypes.c_char_p
    lib.sdtw_status_string.argtypes = [i32]
    lib.sdtw_workspace_bytes.restype = sz
    lib.sdtw_workspace_bytes.argtypes = [ctypes.POINTER(Desc)]
    lib.sdtw_forward.restype = i32
    lib.sdtw_forward.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, sz, vp]
    lib.sdtw_forward_static_scratch.restype = i32
    lib.sdtw_forward_static_scratch.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp]
    lib.sdtw_backward.restype = i32
    lib.sdtw_backward.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sdtw_barycenter_workspace_bytes.restype = sz
    lib.sdtw_barycenter_workspace_bytes.argtypes = [ctypes.POINTER(BaryDesc)]
    lib.sdtw_barycenter_step.restype = i32
    lib.sdtw_barycenter_step.argtypes = [ctypes.POINTER(BaryDesc), vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sdtw_forward_ragged.restype = i32
    lib.sdtw_forward_ragged.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sdtw_backward_ragged.restype = i32
    lib.sdtw_backward_ragged.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sdtw_normalized_workspace_bytes.restype = sz
    lib.sdtw_normalized_workspace_bytes.argtypes = [ctypes.POINTER(Desc)]
    lib.sdtw_normalized_forward.restype = i32
    lib.sdtw_normalized_forward.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, sz, vp]
    lib.sdtw_normalized_backward.restype = i32
    lib.sdtw_normalized_backward.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.sdtw_workspace_status.restype = i32
    lib.sdtw_workspace_status.argtypes = [vp, sz, vp, ctypes.POINTER(ctypes.c_int32)]
    lib.sdtw_debug_export.restype = i32
    lib.sdtw_debug_export.argtypes = [ctypes.POINTER(Desc), vp, sz, i32, vp, vp]
    lib.sdtw_debug_lane_shift.restype = i32
    lib.sdtw_debug_lane_shift.argtypes = [vp, vp]
    lib.sdtw_debug_set_spin_limit.restype = i32
    lib.sdtw_debug_set_spin_limit.argtypes = [ctypes.c_uint32]
    lib.sdtw_debug_force_workgroup_shape.restype = i32
    lib.sdtw_debug_force_workgroup_shape.argtypes = [i32]
    lib.sdtw_debug_profile.restype = i32
    lib.sdtw_debug_profile.argtypes = [i32]
    lib.sdtw_debug_profile_read.restype = i32
    lib.sdtw_debug_profile_read.argtypes = [ctypes.c_char_p, sz, ctypes.POINTER(ctypes.c_float), i32,
                                            ctypes.POINTER(ctypes.c_int)]
    lib.sdtw_half_workspace_bytes.restype = sz
    lib.sdtw_half_workspace_bytes.argtypes = [ctypes.POINTER(Desc)]
    lib.sdtw_forward_half.restype = i32
    lib.sdtw_forward_half.argtypes = [ctypes.POINTER(Desc), vp, vp, i32, vp, vp, sz, vp]
    lib.sdtw_backward_half.restype = i32
    lib.sdtw_backward_half.argtypes = [ctypes.POINTER(Desc), vp, vp, vp, vp, vp, sz, vp]
    lib.sdtw_debug_set_pool_blocks.restype = i32
    lib.sdtw_debug_set_pool_blocks.argtypes = [ctypes.c_longlong]
    lib.sdtw_debug_rate_probe.restype = i32
    lib.sdtw_debug_rate_probe.argtypes = [i32, i32, i32, i32, vp, sz, ctypes.POINTER(ctypes.c_float), vp]
    _lib = lib
    return lib


def sdtw_version():
    return int(load_library().sdtw_version())


def sdtw_status_string(status):
    return load_library().sdtw_status_string(int(status)).decode()


def make_desc(B, N, M, D, gamma, mode, x_shared=False, y_shared=False, bandwidth=0, flags=0):
    return Desc(B, N, M, D, float(gamma), int(mode), 0 if x_shared else N * D, 0 if y_shared else M * D,
                bandwidth, flags)


def sdtw_workspace_bytes(desc):
    return int(load_library().sdtw_workspace_bytes(ctypes.byref(desc)))


def sdtw_barycenter_workspace_bytes(bdesc):
    return int(load_library().sdtw_barycenter_workspace_bytes(ctypes.byref(bdesc)))


def _stream_ptr(stream):
    if stream is not None:
        return ctypes.c_void_p(int(stream))
    import torch

    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype=None, shape=None, name="tensor"):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return ctypes.c_void_p(0)
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("%s must be a contiguous device tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise ValueError("%s must have dtype %s" % (name, dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return ctypes.c_void_p(t.data_ptr())


class Workspace:
    """A device buffer of ``sdtw_workspace_bytes(desc)`` bytes allocated through PyTorch."""

    def __init__(self, nbytes, device="cuda"):
        import torch

        self.nbytes = int(nbytes)
        # torch's caching allocator returns 512-byte aligned blocks
        self.buffer = torch.empty(self.nbytes, dtype=torch.uint8, device=device)
        assert self.buffer.data_ptr() % 256 == 0

    @property
    def ptr(self):
        return ctypes.c_void_p(self.buffer.data_ptr())


def _desc_for(x, y, gamma, mode, check_dtype=True):
    import torch

    if x.dim() == 2:
        N, D = x.shape
        x_shared = True
    else:
        _, N, D = x.shape
        x_shared = False
    if y.dim() == 2:
        M = y.shape[0]
        y_shared = True
    else:
        M = y.shape[1]
        y_shared = False
    if x_shared and y_shared:
        B = 1
    else:
        B = y.shape[0] if not y_shared else x.shape[0]
    if y.shape[-1] != D:
        raise ValueError("x and y must have the same feature dimension")
    if not x_shared and not y_shared and x.shape[0] != y.shape[0]:
        raise ValueError("x and y must have the same batch size")
    assert not check_dtype or (x.dtype == torch.float32 and y.dtype == torch.float32)
    return make_desc(B, N, M, D, gamma, mode, x_shared, y_shared)


def sdtw_forward(x, y, gamma, mode=FUSED, workspace=None, value=None, stream=None, value_only=False,
                 bandwidth=0, min_memory=False):
    """value[b] = sdtw_gamma(x_b, y_b).  Returns (value, desc, workspace); keep the last two for
    :func:`sdtw_backward`.  x [B,N,D] or [N,D]; y [B,M,D] or [M,D]; float32 device tensors.
    ``value_only=True`` sets SDTW_FLAG_VALUE_ONLY: no backward call will follow.
    ``bandwidth`` w > 0: only cells with |i-j| <= w belong to the grid."""
    import torch

    lib = load_library()
    desc = _desc_for(x, y, gamma, mode)
    desc.bandwidth = int(bandwidth)
    if value_only:
        desc.flags |= FLAG_VALUE_ONLY
    if min_memory:
        desc.flags |= FLAG_MIN_MEMORY
    if workspace is None:
        nbytes = sdtw_workspace_bytes(desc)
        if nbytes == 0:
            raise SdtwError(STATUS_INVALID_ARG, "sdtw_workspace_bytes")
        workspace = Workspace(nbytes, x.device)
    if value is None:
        value = torch.empty(desc.B, dtype=torch.float32, device=x.device)
    rc = lib.sdtw_forward(ctypes.byref(desc), _ptr(x, torch.float32, name="x"), _ptr(y, torch.float32, name="y"),
                          _ptr(value, torch.float32, (desc.B,), "value"), workspace.ptr, workspace.nbytes,
                          _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_forward")
    return value, desc, workspace


def sdtw_forward_desc(desc, x, y, workspace, value, stream=None):
    """sdtw_forward with a descriptor the caller made (make_desc): nothing is allocated here."""
    import torch

    rc = load_library().sdtw_forward(ctypes.byref(desc), _ptr(x, torch.float32, name="x"), _ptr(y, torch.float32, name="y"),
                                     _ptr(value, torch.float32, (desc.B,), "value"), workspace.ptr, workspace.nbytes,
                                     _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_forward")
    return value


STATIC_SCRATCH_BYTES = 64 << 20


def sdtw_forward_static_scratch(desc, x, y, value, stream=None):
    """sdtw_forward's values through the entry point that uses the library's own scratch buffer
    (nothing is allocated, here or in the library).  Returns the status code."""
    import torch

    return int(load_library().sdtw_forward_static_scratch(
        ctypes.byref(desc), _ptr(x, torch.float32, name="x"), _ptr(y, torch.float32, name="y"),
        _ptr(value, torch.float32, (desc.B,), "value"), _stream_ptr(stream)))


def sdtw_backward(desc, x, y, workspace, grad_value=None, want_dx=True, want_dy=True, want_E=False,
                  dx=None, dy=None, E=None, stream=None):
    """Gradients of the values produced by the forward call that filled ``workspace``.
    Returns (dx [B,N,D] or None, dy [B,M,D] or None, E [B,N,M] or None)."""
    import torch

    lib = load_library()
    dev = x.device
    if want_dx and dx is None:
        dx = torch.empty((desc.B, desc.N, desc.D), dtype=torch.float32, device=dev)
    if want_dy and dy is None:
        dy = torch.empty((desc.B, desc.M, desc.D), dtype=torch.float32, device=dev)
    if want_E and E is None:
        E = torch.empty((desc.B, desc.N, desc.M), dtype=torch.float32, device=dev)
    rc = lib.sdtw_backward(
        ctypes.byref(desc), _ptr(x, torch.float32, name="x"), _ptr(y, torch.float32, name="y"),
        _ptr(grad_value, torch.float32, (desc.B,), "grad_value"),
        _ptr(dx, torch.float32, (desc.B, desc.N, desc.D), "dx"),
        _ptr(dy, torch.float32, (desc.B, desc.M, desc.D), "dy"),
        _ptr(E, torch.float32, (desc.B, desc.N, desc.M), "E"),
        workspace.ptr, workspace.nbytes, _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_backward")
    return dx, dy, E


def sdtw_forward_ragged(x, y, x_len, y_len, gamma, mode=FUSED, workspace=None, value=None, stream=None,
                        bandwidth=0, min_memory=False):
    """As :func:`sdtw_forward` for pairs of individual lengths: x_len, y_len are int32 device tensors
    [B] (or None).  Returns (value, desc, workspace)."""
    import torch

    lib = load_library()
    desc = _desc_for(x, y, gamma, mode)
    desc.bandwidth = int(bandwidth)
    if min_memory:
        desc.flags |= FLAG_MIN_MEMORY
    if workspace is None:
        nbytes = sdtw_workspace_bytes(desc)
        if nbytes == 0:
            raise SdtwError(STATUS_INVALID_ARG, "sdtw_workspace_bytes")
        workspace = Workspace(nbytes, x.device)
    if value is None:
        value = torch.empty(desc.B, dtype=torch.float32, device=x.device)
    rc = lib.sdtw_forward_ragged(ctypes.byref(desc), _ptr(x, torch.float32, name="x"), _ptr(y, torch.float32, name="y"),
                                 _ptr(x_len, torch.int32, (desc.B,), "x_len"), _ptr(y_len, torch.int32, (desc.B,), "y_len"),
                                 _ptr(value, torch.float32, (desc.B,), "value"), workspace.ptr, workspace.nbytes,
                                 _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_forward_ragged")
    return value, desc, workspace


def sdtw_backward_ragged(desc, x, y, x_len, y_len, workspace, grad_value=None, want_E=False, dx=None, dy=None,
                         E=None, stream=None):
    """Gradients for :func:`sdtw_forward_ragged` (same length vectors).  Returns (dx, dy, E or None)."""
    import torch

    lib = load_library()
    dev = x.device
    if dx is None:
        dx = torch.empty((desc.B, desc.N, desc.D), dtype=torch.float32, device=dev)
    if dy is None:
        dy = torch.empty((desc.B, desc.M, desc.D), dtype=torch.float32, device=dev)
    if want_E and E is None:
        E = torch.empty((desc.B, desc.N, desc.M), dtype=torch.float32, device=dev)
    rc = lib.sdtw_backward_ragged(
        ctypes.byref(desc), _ptr(x, torch.float32, name="x"), _ptr(y, torch.float32, name="y"),
        _ptr(x_len, torch.int32, (desc.B,), "x_len"), _ptr(y_len, torch.int32, (desc.B,), "y_len"),
        _ptr(grad_value, torch.float32, (desc.B,), "grad_value"),
        _ptr(dx, torch.float32, (desc.B, desc.N, desc.D), "dx"),
        _ptr(dy, torch.float32, (desc.B, desc.M, desc.D), "dy"),
        _ptr(E, torch.float32, (desc.B, desc.N, desc.M), "E"),
        workspace.ptr, workspace.nbytes, _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_backward_ragged")
    return dx, dy, E


def sdtw_normalized_workspace_bytes(desc):
    return int(load_library().sdtw_normalized_workspace_bytes(ctypes.byref(desc)))


def sdtw_normalized_forward(x, y, gamma, mode=FUSED, workspace=None, value=None, stream=None, min_memory=False):
    """value[b] = sdtw(x_b,y_b) - (sdtw(x_b,x_b) + sdtw(y_b,y_b)) / 2.  Returns (value, desc, workspace)."""
    import torch

    lib = load_library()
    desc = _desc_for(x, y, gamma, mode)
    if min_memory:
        desc.flags |= FLAG_MIN_MEMORY
    if workspace is None:
        nbytes = sdtw_normalized_workspace_bytes(desc)
        if nbytes == 0:
            raise SdtwError(STATUS_INVALID_ARG, "sdtw_normalized_workspace_bytes")
        workspace = Workspace(nbytes, x.device)
    if value is None:
        value = torch.empty(desc.B, dtype=torch.float32, device=x.device)
    rc = lib.sdtw_normalized_forward(ctypes.byref(desc), _ptr(x, torch.float32, name="x"),
                                     _ptr(y, torch.float32, name="y"), _ptr(value, torch.float32, (desc.B,), "value"),
                                     workspace.ptr, workspace.nbytes, _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_normalized_forward")
    return value, desc, workspace


def sdtw_normalized_backward(desc, x, y, workspace, grad_value=None, want_dx=True, want_dy=True, dx=None, dy=None,
                             stream=None):
    """Gradients of the normalised values.  Returns (dx [B,N,D] or None, dy [B,M,D] or None)."""
    import torch

    lib = load_library()
    dev = x.device
    if want_dx and dx is None:
        dx = torch.empty((desc.B, desc.N, desc.D), dtype=torch.float32, device=dev)
    if want_dy and dy is None:
        dy = torch.empty((desc.B, desc.M, desc.D), dtype=torch.float32, device=dev)
    rc = lib.sdtw_normalized_backward(
        ctypes.byref(desc), _ptr(x, torch.float32, name="x"), _ptr(y, torch.float32, name="y"),
        _ptr(grad_value, torch.float32, (desc.B,), "grad_value"),
        _ptr(dx, torch.float32, (desc.B, desc.N, desc.D), "dx"),
        _ptr(dy, torch.float32, (desc.B, desc.M, desc.D), "dy"),
        workspace.ptr, workspace.nbytes, _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_normalized_backward")
    return dx, dy


def make_bary_desc(K, Lz, Lx, D, gamma, mode, lr, beta1, beta2, eps, step, flags=0):
    return BaryDesc(K, Lz, Lx, D, float(gamma), int(mode), float(lr), float(beta1), float(beta2), float(eps),
                    int(step), int(flags))


def sdtw_barycenter_step(z, X, adam_m, adam_v, gamma, step, lr=0.05, beta1=0.9, beta2=0.999, eps=1e-8,
                         mode=FUSED, workspace=None, loss=None, dz=None, want_dz=False, stream=None, min_memory=False):
    """One in-place Adam step on z [Lz,D] against X [K,Lx,D].  Returns (loss [1], dz or None, workspace)."""
    import torch

    lib = load_library()
    K, Lx, D = X.shape
    Lz = z.shape[0]
    bdesc = make_bary_desc(K, Lz, Lx, D, gamma, mode, lr, beta1, beta2, eps, step, FLAG_MIN_MEMORY if min_memory else 0)
    if workspace is None:
        nbytes = sdtw_barycenter_workspace_bytes(bdesc)
        if nbytes == 0:
            raise SdtwError(STATUS_INVALID_ARG, "sdtw_barycenter_workspace_bytes")
        workspace = Workspace(nbytes, z.device)
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=z.device)
    if want_dz and dz is None:
        dz = torch.empty((Lz, D), dtype=torch.float32, device=z.device)
    rc = lib.sdtw_barycenter_step(
        ctypes.byref(bdesc), _ptr(z, torch.float32, (Lz, D), "z"), _ptr(X, torch.float32, name="X"),
        _ptr(adam_m, torch.float32, (Lz, D), "adam_m"), _ptr(adam_v, torch.float32, (Lz, D), "adam_v"),
        _ptr(loss, torch.float32, (1,), "loss"), _ptr(dz, torch.float32, (Lz, D), "dz"),
        workspace.ptr, workspace.nbytes, _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_barycenter_step")
    return loss, dz, workspace


def workspace_status(workspace, stream=None):
    """Synchronises and returns the device-side status word of a workspace."""
    out = ctypes.c_int32(-1)
    rc = load_library().sdtw_workspace_status(workspace.ptr, workspace.nbytes, _stream_ptr(stream), ctypes.byref(out))
    if rc != 0:
        raise SdtwError(rc, "sdtw_workspace_status")
    return int(out.value)


def debug_export(desc, workspace, what, stream=None):
    """Row-major copy of an intermediate (cost: float32, R: float64, E: float32), shape [B,N,M]."""
    import torch

    dtype = torch.float64 if what == EXPORT_R else torch.float32
    out = torch.empty((desc.B, desc.N, desc.M), dtype=dtype, device=workspace.buffer.device)
    rc = load_library().sdtw_debug_export(ctypes.byref(desc), workspace.ptr, workspace.nbytes, int(what),
                                          ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_debug_export")
    return out


def debug_lane_shift(stream=None):
    import torch

    out = torch.empty(128, dtype=torch.int32, device="cuda")
    rc = load_library().sdtw_debug_lane_shift(ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_debug_lane_shift")
    return out


def debug_set_spin_limit(polls):
    load_library().sdtw_debug_set_spin_limit(int(polls))


def debug_profile(enable):
    load_library().sdtw_debug_profile(1 if enable else 0)


def debug_profile_read(max_entries=4096):
    """[(kernel label, milliseconds)] of every launch since profiling was switched on."""
    names = ctypes.create_string_buffer(64 * max_entries)
    ms = (ctypes.c_float * max_entries)()
    count = ctypes.c_int(0)
    rc = load_library().sdtw_debug_profile_read(names, len(names), ms, max_entries, ctypes.byref(count))
    if rc != 0:
        raise SdtwError(rc, "sdtw_debug_profile_read")
    labels = names.value.decode().split(";")[:count.value]
    return [(labels[i], float(ms[i])) for i in range(count.value)]


def debug_force_workgroup_shape(bands_per_workgroup):
    rc = load_library().sdtw_debug_force_workgroup_shape(int(bands_per_workgroup))
    if rc != 0:
        raise SdtwError(rc, "sdtw_debug_force_workgroup_shape")


RATE_PROBE_SCRATCH_BYTES = 16 << 20


def debug_rate_probe(probe, variant, waves_per_simd, iters, scratch, stream=None):
    """Milliseconds one calibration micro-kernel took (see sdtw_debug_rate_probe in sdtw.h)."""
    ms = ctypes.c_float(0.0)
    rc = load_library().sdtw_debug_rate_probe(int(probe), int(variant), int(waves_per_simd), int(iters), scratch.ptr,
                                              scratch.nbytes, ctypes.byref(ms), _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_debug_rate_probe")
    return float(ms.value)


def debug_set_pool_blocks(blocks):
    load_library().sdtw_debug_set_pool_blocks(int(blocks))


INPUT_F16, INPUT_BF16 = 1, 2


def sdtw_forward_half(x, y, gamma, mode=FUSED, workspace=None, value=None, stream=None, min_memory=False):
    """sdtw_forward for float16 or bfloat16 device tensors x [B,N,D] / [N,D], y [B,M,D] / [M,D] (same dtype).
    Returns (value float32 [B], desc, workspace); keep the last two for :func:`sdtw_backward_half`."""
    import torch

    lib = load_library()
    if x.dtype != y.dtype or x.dtype not in (torch.float16, torch.bfloat16):
        raise ValueError("x and y must both be float16 or both bfloat16")
    desc = _desc_for(x, y, gamma, mode, check_dtype=False)
    if min_memory:
        desc.flags |= FLAG_MIN_MEMORY
    if workspace is None:
        nbytes = int(lib.sdtw_half_workspace_bytes(ctypes.byref(desc)))
        if nbytes == 0:
            raise SdtwError(STATUS_INVALID_ARG, "sdtw_half_workspace_bytes")
        workspace = Workspace(nbytes, x.device)
    if value is None:
        value = torch.empty(desc.B, dtype=torch.float32, device=x.device)
    kind = INPUT_F16 if x.dtype == torch.float16 else INPUT_BF16
    rc = lib.sdtw_forward_half(ctypes.byref(desc), _ptr(x, name="x"), _ptr(y, name="y"), kind,
                               _ptr(value, torch.float32, (desc.B,), "value"), workspace.ptr, workspace.nbytes,
                               _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_forward_half")
    return value, desc, workspace


def sdtw_backward_half(desc, workspace, grad_value=None, want_dx=True, want_dy=True, want_E=False, stream=None):
    """Gradients (float32) of the values :func:`sdtw_forward_half` produced.  Returns (dx, dy, E or None)."""
    import torch

    lib = load_library()
    dev = workspace.buffer.device
    dx = torch.empty((desc.B, desc.N, desc.D), dtype=torch.float32, device=dev) if want_dx else None
    dy = torch.empty((desc.B, desc.M, desc.D), dtype=torch.float32, device=dev) if want_dy else None
    E = torch.empty((desc.B, desc.N, desc.M), dtype=torch.float32, device=dev) if want_E else None
    rc = lib.sdtw_backward_half(ctypes.byref(desc), _ptr(grad_value, torch.float32, (desc.B,), "grad_value"),
                                _ptr(dx), _ptr(dy), _ptr(E), workspace.ptr, workspace.nbytes, _stream_ptr(stream))
    if rc != 0:
        raise SdtwError(rc, "sdtw_backward_half")
    return dx, dy, E
