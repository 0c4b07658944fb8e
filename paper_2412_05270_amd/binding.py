"""ctypes marshalling for libapollo_mi355x.so (the C ABI of include/apollo.h).

The functions carry the names of the C entry points and do nothing but convert arguments.
If the shared library has not been built the import of the library fails loudly: there is no
fallback implementation.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libapollo_mi355x.so"

APOLLO_OK, APOLLO_EINVAL, APOLLO_ENOMEM, APOLLO_ESTATE, APOLLO_EHIP, APOLLO_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
APOLLO_F32, APOLLO_BF16, APOLLO_Q8 = 0, 1, 2
APOLLO_ROUND_NEAREST, APOLLO_ROUND_STOCHASTIC = 0, 1
APOLLO_SCHEDULE_SERIAL, APOLLO_SCHEDULE_OVERLAP, APOLLO_SCHEDULE_CHUNKED = 0, 1, 2
APOLLO_CHANNEL, APOLLO_TENSOR = 0, 1
APOLLO_SIDE_AUTO, APOLLO_SIDE_LEFT, APOLLO_SIDE_RIGHT = 0, 1, 2
APOLLO_PROJ_RANDOM, APOLLO_PROJ_IDENTITY = 0, 1
APOLLO_PATH_RANK1, APOLLO_PATH_MATRIX_CORE, APOLLO_PATH_GENERAL, APOLLO_PATH_NONE = 0, 1, 2, 3
(APOLLO_DBG_M, APOLLO_DBG_V, APOLLO_DBG_S, APOLLO_DBG_NORM, APOLLO_DBG_C, APOLLO_DBG_R,
 APOLLO_DBG_COLSQ) = range(7)


class ApolloShape(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("grad_dtype", C.c_int32), ("reserved", C.c_int32)]


class ApolloConfig(C.Structure):
    _fields_ = [("rank", C.c_int32), ("mode", C.c_int32), ("seed", C.c_uint64),
                ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("scale", C.c_float), ("weight_decay", C.c_float), ("nl_gamma", C.c_float),
                ("refresh_interval", C.c_int32), ("bias_correction", C.c_int32),
                ("side", C.c_int32), ("weight_dtype", C.c_int32), ("state_dtype", C.c_int32),
                ("projection", C.c_int32), ("weight_rounding", C.c_int32), ("schedule", C.c_int32)]


class ApolloTensor(C.Structure):
    _fields_ = [("w", C.c_void_p), ("g", C.c_void_p), ("w_meta", C.c_void_p)]


class ApolloFlatShape(C.Structure):
    _fields_ = [("numel", C.c_int64), ("grad_dtype", C.c_int32), ("store_dtype", C.c_int32)]


class ApolloAdamwConfig(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("weight_decay", C.c_float),
                ("bias_correction", C.c_int32), ("reserved", C.c_int32)]


class ApolloError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("apollo status %d: %s" % (status, message))
        self.status = status


_lib = None


def library_path():
    return os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Loads the in-tree shared library (built by `python -m paper_2412_05270_amd.build`)."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise ImportError("%s is not built: run `python -m paper_2412_05270_amd.build` "
                          "(there is no fallback implementation)" % path)
    lib = C.CDLL(path)
    vp, i32, i64, u32, sz, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_size_t, C.c_float
    cfgp, shp = C.POINTER(ApolloConfig), C.POINTER(ApolloShape)
    lib.apollo_state_bytes.restype = sz
    lib.apollo_state_bytes.argtypes = [cfgp, shp, i32]
    lib.apollo_workspace_bytes.restype = sz
    lib.apollo_workspace_bytes.argtypes = [cfgp, shp, i32]
    lib.apollo_state_offsets.restype = i32
    lib.apollo_state_offsets.argtypes = [cfgp, shp, i32, i32, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
    lib.apollo_init.restype = i32
    lib.apollo_init.argtypes = [C.POINTER(vp), cfgp, shp, i32, vp, sz, vp, sz, i32, vp]
    lib.apollo_step.restype = i32
    lib.apollo_step.argtypes = [vp, C.POINTER(ApolloTensor), i32, i64, f32, vp]
    lib.apollo_step_prepare.restype = i32
    lib.apollo_step_prepare.argtypes = [vp, i64, f32, vp]
    lib.apollo_step_launch.restype = i32
    lib.apollo_step_launch.argtypes = [vp, C.POINTER(ApolloTensor), i32, vp]
    lib.apollo_step_noalloc.restype = i32
    lib.apollo_step_noalloc.argtypes = [cfgp, shp, C.POINTER(ApolloTensor), i32, vp, sz, i32, i64, f32, vp]
    lib.apollo_debug_fill_projection.restype = i32
    lib.apollo_debug_fill_projection.argtypes = [vp, i32, i64, vp, i32, vp]
    lib.apollo_debug_get.restype = i32
    lib.apollo_debug_get.argtypes = [vp, i32, i32, vp, sz, vp]
    lib.apollo_debug_philox.restype = i32
    lib.apollo_debug_philox.argtypes = [vp, u32, u32, vp, i64, vp]
    lib.apollo_debug_gauss_parts.restype = i32
    lib.apollo_debug_gauss_parts.argtypes = [u32, i64, vp, vp, vp, vp]
    lib.apollo_debug_copy.restype = i32
    lib.apollo_debug_copy.argtypes = [vp, vp, sz, vp]
    lib.apollo_debug_path.restype = i32
    lib.apollo_debug_path.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32)]
    lib.apollo_profile_enable.restype = i32
    lib.apollo_profile_enable.argtypes = [vp, i32]
    lib.apollo_profile_read.restype = i32
    lib.apollo_profile_read.argtypes = [vp, C.POINTER(f32), C.POINTER(i32)]
    lib.apollo_last_error.restype = C.c_char_p
    lib.apollo_last_error.argtypes = [vp]
    lib.apollo_destroy.restype = None
    lib.apollo_destroy.argtypes = [vp]
    fsp, acp = C.POINTER(ApolloFlatShape), C.POINTER(ApolloAdamwConfig)
    lib.apollo_adamw_state_bytes.restype = sz
    lib.apollo_adamw_state_bytes.argtypes = [fsp, i32]
    lib.apollo_adamw_workspace_bytes.restype = sz
    lib.apollo_adamw_workspace_bytes.argtypes = [fsp, i32]
    lib.apollo_adamw_state_offsets.restype = i32
    lib.apollo_adamw_state_offsets.argtypes = [fsp, i32, i32, C.POINTER(sz), C.POINTER(sz)]
    lib.apollo_adamw_init.restype = i32
    lib.apollo_adamw_init.argtypes = [C.POINTER(vp), acp, fsp, i32, vp, sz, vp, sz, i32, vp]
    lib.apollo_adamw_step.restype = i32
    lib.apollo_adamw_step.argtypes = [vp, C.POINTER(ApolloTensor), i32, i64, f32, vp]
    lib.apollo_adamw_last_error.restype = C.c_char_p
    lib.apollo_adamw_last_error.argtypes = [vp]
    lib.apollo_adamw_destroy.restype = None
    lib.apollo_adamw_destroy.argtypes = [vp]
    _lib = lib
    return lib


def _shape_array(shapes):
    arr = (ApolloShape * len(shapes))()
    for i, s in enumerate(shapes):
        if isinstance(s, ApolloShape):
            arr[i] = s
        else:
            rows, cols, dt = s
            arr[i] = ApolloShape(rows, cols, dt, 0)
    return arr


def apollo_last_error(handle=None):
    return (load_library().apollo_last_error(handle) or b"").decode()


def apollo_state_bytes(cfg, shapes):
    return load_library().apollo_state_bytes(C.byref(cfg), _shape_array(shapes), len(shapes))


def apollo_workspace_bytes(cfg, shapes):
    return load_library().apollo_workspace_bytes(C.byref(cfg), _shape_array(shapes), len(shapes))


def apollo_state_offsets(cfg, shapes, tensor):
    m, v, nm = C.c_size_t(), C.c_size_t(), C.c_size_t()
    rc = load_library().apollo_state_offsets(C.byref(cfg), _shape_array(shapes), len(shapes), tensor,
                                             C.byref(m), C.byref(v), C.byref(nm))
    return rc, m.value, v.value, nm.value


def apollo_init(cfg, shapes, state_ptr, state_bytes, workspace_ptr, workspace_bytes, zero_state=1, stream=None):
    """Returns (status, handle)."""
    h = C.c_void_p()
    rc = load_library().apollo_init(C.byref(h), C.byref(cfg) if cfg is not None else None,
                                    _shape_array(shapes) if shapes is not None else None,
                                    len(shapes) if shapes is not None else 0,
                                    state_ptr, state_bytes, workspace_ptr, workspace_bytes, zero_state, stream)
    return rc, (h if h.value else None)


def apollo_step(handle, tensors, step, lr, stream=None, n_tensors=None):
    """tensors: a ctypes array of ApolloTensor (or a list of (w_ptr, g_ptr))."""
    if tensors is not None and not isinstance(tensors, C.Array):
        arr = (ApolloTensor * len(tensors))()
        for i, t in enumerate(tensors):
            arr[i] = ApolloTensor(*t)        # (w, g) or (w, g, w_meta)
        tensors = arr
    n = n_tensors if n_tensors is not None else (len(tensors) if tensors is not None else 0)
    return load_library().apollo_step(handle, tensors, n, step, lr, stream)


def apollo_step_prepare(handle, step, lr, stream=None):
    return load_library().apollo_step_prepare(handle, step, lr, stream)


def apollo_step_launch(handle, tensors, stream=None, n_tensors=None):
    """tensors: a ctypes array of ApolloTensor."""
    n = n_tensors if n_tensors is not None else (len(tensors) if tensors is not None else 0)
    return load_library().apollo_step_launch(handle, tensors, n, stream)


APOLLO_NOALLOC_SCRATCH_BYTES = 32 * 1024 * 1024
APOLLO_NOALLOC_MAX_TENSORS = 64


def apollo_step_noalloc(cfg, shapes, tensors, state_ptr, state_bytes, zero_state, step, lr, stream=None):
    """tensors: a ctypes array of ApolloTensor (or a list of (w_ptr, g_ptr[, w_meta_ptr]))."""
    if tensors is not None and not isinstance(tensors, C.Array):
        arr = (ApolloTensor * len(tensors))()
        for i, t in enumerate(tensors):
            arr[i] = ApolloTensor(*t)
        tensors = arr
    return load_library().apollo_step_noalloc(C.byref(cfg) if cfg is not None else None,
                                              _shape_array(shapes) if shapes is not None else None, tensors,
                                              len(shapes) if shapes is not None else 0, state_ptr, state_bytes,
                                              1 if zero_state else 0, step, lr, stream)


def apollo_debug_fill_projection(handle, tensor, step, out_ptr, dtype, stream=None):
    return load_library().apollo_debug_fill_projection(handle, tensor, step, out_ptr, dtype, stream)


def apollo_debug_get(handle, tensor, what, out_ptr, nbytes, stream=None):
    return load_library().apollo_debug_get(handle, tensor, what, out_ptr, nbytes, stream)


def apollo_debug_path(handle, tensor):
    """-> (status, APOLLO_PATH_*, padded_copy)"""
    path, padded = C.c_int32(-1), C.c_int32(0)
    rc = load_library().apollo_debug_path(handle, tensor, C.byref(path), C.byref(padded))
    return rc, path.value, padded.value


def apollo_debug_philox(ctr_ptr, key0, key1, out_ptr, count, stream=None):
    return load_library().apollo_debug_philox(ctr_ptr, key0, key1, out_ptr, count, stream)


def apollo_debug_gauss_parts(first, count, radius_ptr, cos_ptr, sin_ptr, stream=None):
    return load_library().apollo_debug_gauss_parts(first, count, radius_ptr, cos_ptr, sin_ptr, stream)


def apollo_debug_copy(dst_ptr, src_ptr, nbytes, stream=None):
    return load_library().apollo_debug_copy(dst_ptr, src_ptr, nbytes, stream)


def apollo_profile_enable(handle, on):
    return load_library().apollo_profile_enable(handle, 1 if on else 0)


def apollo_profile_read(handle):
    """Returns (status, [ms of the five phases], n_steps)."""
    ms = (C.c_float * 5)()
    n = C.c_int32()
    rc = load_library().apollo_profile_read(handle, ms, C.byref(n))
    return rc, list(ms), n.value


def apollo_destroy(handle):
    load_library().apollo_destroy(handle)


def _flat_shape_array(shapes):
    arr = (ApolloFlatShape * len(shapes))()
    for i, s in enumerate(shapes):
        arr[i] = s if isinstance(s, ApolloFlatShape) else ApolloFlatShape(s[0], s[1], s[2] if len(s) > 2 else APOLLO_F32)
    return arr


def apollo_adamw_last_error(handle=None):
    return (load_library().apollo_adamw_last_error(handle) or b"").decode()


def apollo_adamw_state_bytes(shapes):
    return load_library().apollo_adamw_state_bytes(_flat_shape_array(shapes) if shapes is not None else None,
                                                   len(shapes) if shapes is not None else 0)


def apollo_adamw_workspace_bytes(shapes):
    return load_library().apollo_adamw_workspace_bytes(_flat_shape_array(shapes) if shapes is not None else None,
                                                       len(shapes) if shapes is not None else 0)


def apollo_adamw_state_offsets(shapes, tensor):
    m, v = C.c_size_t(), C.c_size_t()
    rc = load_library().apollo_adamw_state_offsets(_flat_shape_array(shapes), len(shapes), tensor, C.byref(m), C.byref(v))
    return rc, m.value, v.value


def apollo_adamw_init(cfg, shapes, state_ptr, state_bytes, workspace_ptr, workspace_bytes, zero_state=1, stream=None):
    """Returns (status, handle)."""
    h = C.c_void_p()
    rc = load_library().apollo_adamw_init(C.byref(h), C.byref(cfg) if cfg is not None else None,
                                          _flat_shape_array(shapes) if shapes is not None else None,
                                          len(shapes) if shapes is not None else 0,
                                          state_ptr, state_bytes, workspace_ptr, workspace_bytes, zero_state, stream)
    return rc, (h if h.value else None)


def apollo_adamw_step(handle, tensors, step, lr, stream=None, n_tensors=None):
    if tensors is not None and not isinstance(tensors, C.Array):
        arr = (ApolloTensor * len(tensors))()
        for i, (w, g) in enumerate(tensors):
            arr[i] = ApolloTensor(w, g)
        tensors = arr
    n = n_tensors if n_tensors is not None else (len(tensors) if tensors is not None else 0)
    return load_library().apollo_adamw_step(handle, tensors, n, step, lr, stream)


def apollo_adamw_destroy(handle):
    load_library().apollo_adamw_destroy(handle)


class AdamwStepper:
    """Owner of the device buffers (torch tensors) around one AdamW handle; calls go to the C ABI."""

    def __init__(self, cfg, weights, grads, device="cuda:0", zero_state=True):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.weights, self.grads = list(weights), list(grads)
        self.shapes = []
        for w, g in zip(self.weights, self.grads):
            # a bfloat16 weight tensor keeps its moments in bfloat16 as well (store_dtype)
            assert w.dtype in (torch.float32, torch.bfloat16) and w.is_contiguous() and g.is_contiguous()
            assert g.shape == w.shape and g.dtype in (torch.float32, torch.bfloat16)
            self.shapes.append((w.numel(), APOLLO_BF16 if g.dtype == torch.bfloat16 else APOLLO_F32,
                                APOLLO_BF16 if w.dtype == torch.bfloat16 else APOLLO_F32))
        sb = apollo_adamw_state_bytes(self.shapes)
        wb = apollo_adamw_workspace_bytes(self.shapes)
        if sb == 0 or wb == 0:
            raise ApolloError(APOLLO_EINVAL, apollo_adamw_last_error())
        self.state = torch.empty(sb, dtype=torch.uint8, device=device)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=device)
        self.device = self.state.device
        rc, self.handle = apollo_adamw_init(cfg, self.shapes, self.state.data_ptr(), sb, self.workspace.data_ptr(), wb,
                                            1 if zero_state else 0, self._stream())
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_adamw_last_error())
        self._tensors = (ApolloTensor * len(self.weights))()
        for i, (w, g) in enumerate(zip(self.weights, self.grads)):
            self._tensors[i] = ApolloTensor(w.data_ptr(), g.data_ptr())

    def _stream(self):
        """torch's current stream on the buffers' device, looked up at every call: the work is
        ordered after whatever the caller has queued there (its gradients), on whichever stream
        the caller has made current."""
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def step(self, step, lr):
        rc = apollo_adamw_step(self.handle, self._tensors, step, lr, self._stream())
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_adamw_last_error(self.handle))

    def moments(self, tensor):
        """(M, V) of one tensor as views into the state buffer, in the tensor's storage type."""
        rc, mo, vo = apollo_adamw_state_offsets(self.shapes, tensor)
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_adamw_last_error())
        n = self.shapes[tensor][0]
        if self.shapes[tensor][2] == APOLLO_BF16:
            f, e = self.state.view(self.torch.bfloat16), 2
        else:
            f, e = self.state.view(self.torch.float32), 4
        return f[mo // e: mo // e + n], f[vo // e: vo // e + n]

    def close(self):
        if self.handle is not None:
            apollo_adamw_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class ApolloStepper:
    """Convenience owner of the device buffers (torch tensors) around one handle.

    Only allocation and pointer bookkeeping live here; every call goes to the C ABI.
    """

    def __init__(self, cfg, weights, grads, device="cuda:0", zero_state=True, metas=None):
        """metas: with 8-bit weights (weights then are uint8 code tensors), one fp32 tensor of
        (scale, zero) pairs per tensor, shape (rows * cols / 128, 2)."""
        import torch
        self.torch = torch
        self.cfg = cfg
        self.weights = list(weights)
        self.grads = list(grads)
        self.metas = list(metas) if metas is not None else [None] * len(self.weights)
        self.shapes = []
        wdt = {APOLLO_BF16: torch.bfloat16, APOLLO_Q8: torch.uint8}.get(cfg.weight_dtype, torch.float32)
        for w, mt in zip(self.weights, self.metas):
            assert (mt is None) == (cfg.weight_dtype != APOLLO_Q8)
            assert mt is None or (mt.dtype == torch.float32 and mt.is_contiguous() and mt.numel() == w.numel() // 64)
        for w, g in zip(self.weights, self.grads):
            assert w.dtype == wdt and w.dim() == 2 and w.is_contiguous() and g.is_contiguous()
            assert g.shape == w.shape and g.dtype in (torch.float32, torch.bfloat16)
            self.shapes.append((w.shape[0], w.shape[1], APOLLO_BF16 if g.dtype == torch.bfloat16 else APOLLO_F32))
        sb = apollo_state_bytes(cfg, self.shapes)
        wb = apollo_workspace_bytes(cfg, self.shapes)
        if sb == 0 or wb == 0:
            raise ApolloError(APOLLO_EINVAL, apollo_last_error())
        self.state = torch.empty(sb, dtype=torch.uint8, device=device)
        self.workspace = torch.empty(wb, dtype=torch.uint8, device=device)
        self.device = self.state.device
        rc, self.handle = apollo_init(cfg, self.shapes, self.state.data_ptr(), sb, self.workspace.data_ptr(), wb,
                                      1 if zero_state else 0, self._stream())
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_last_error())
        self._tensors = (ApolloTensor * len(self.weights))()
        self.set_tensors(self.weights, self.grads, self.metas)

    def set_tensors(self, weights, grads, metas=None):
        self.weights, self.grads = list(weights), list(grads)
        self.metas = list(metas) if metas is not None else [None] * len(self.weights)
        for i, (w, g, mt) in enumerate(zip(self.weights, self.grads, self.metas)):
            self._tensors[i] = ApolloTensor(w.data_ptr(), g.data_ptr(), mt.data_ptr() if mt is not None else None)

    def _stream(self):
        """torch's current stream on the buffers' device, looked up at every call (see AdamwStepper)."""
        return self.torch.cuda.current_stream(self.device).cuda_stream

    def step(self, step, lr):
        rc = apollo_step(self.handle, self._tensors, step, lr, self._stream())
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_last_error(self.handle))

    def prepare(self, step, lr):
        """The scalars of one step into device memory (for a step replayed from a graph)."""
        rc = apollo_step_prepare(self.handle, step, lr, self._stream())
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_last_error(self.handle))

    def launch(self):
        """The kernels of one step, reading what prepare() left: this is the call to capture."""
        rc = apollo_step_launch(self.handle, self._tensors, self._stream())
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_last_error(self.handle))

    def channels(self, tensor):
        rows, cols, _ = self.shapes[tensor]
        left = self.cfg.side == APOLLO_SIDE_LEFT or (self.cfg.side == APOLLO_SIDE_AUTO and rows <= cols)
        return (cols if left else rows), (rows if left else cols)

    def debug(self, tensor, what):
        torch = self.torch
        n, _ = self.channels(tensor)
        r = self.cfg.rank
        if what in (APOLLO_DBG_M, APOLLO_DBG_V) and self.cfg.projection == APOLLO_PROJ_IDENTITY:
            # without a projection the moments have the tensor's own layout
            out = torch.empty(self.shapes[tensor][:2], dtype=torch.float32, device=self.state.device)
        elif what in (APOLLO_DBG_M, APOLLO_DBG_V, APOLLO_DBG_R):
            out = torch.empty((r, n), dtype=torch.float32, device=self.state.device)
        elif what == APOLLO_DBG_COLSQ or (what == APOLLO_DBG_S and self.cfg.mode == APOLLO_CHANNEL):
            out = torch.empty(n, dtype=torch.float32, device=self.state.device)
        else:
            out = torch.empty(1, dtype=torch.float32, device=self.state.device)
        rc = apollo_debug_get(self.handle, tensor, what, out.data_ptr(), out.numel() * 4, self._stream())
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_last_error(self.handle))
        return out

    def path(self, tensor):
        """(APOLLO_PATH_*, padded_copy) of one tensor."""
        rc, path, padded = apollo_debug_path(self.handle, tensor)
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_last_error(self.handle))
        return path, padded

    def projection(self, tensor, step, bf16):
        torch = self.torch
        _, m = self.channels(tensor)
        out = torch.empty((self.cfg.rank, m), dtype=torch.bfloat16 if bf16 else torch.float32,
                          device=self.state.device)
        rc = apollo_debug_fill_projection(self.handle, tensor, step, out.data_ptr(),
                                          APOLLO_BF16 if bf16 else APOLLO_F32, self._stream())
        if rc != APOLLO_OK:
            raise ApolloError(rc, apollo_last_error(self.handle))
        return out

    def close(self):
        if self.handle is not None:
            apollo_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
