"""ctypes binding of libkavg.so: the same calls as include/kavg.h, argument
marshalling only.  PyTorch supplies device memory and the stream; every step
of the method runs inside the library's HIP kernels.  There is no fallback:
if the library is missing or a call fails, an exception is raised.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkavg.so")

KAVG_OK, KAVG_EINVAL, KAVG_ENOMEM, KAVG_EDEVICE, KAVG_ESTATE = 0, 1, 2, 3, 4
KAVG_FP32, KAVG_BF16 = 0, 1
_CODES = {1: "KAVG_EINVAL", 2: "KAVG_ENOMEM", 3: "KAVG_EDEVICE", 4: "KAVG_ESTATE"}

EXPORTS = [
    "kavg_num_params", "kavg_workspace_bytes", "kavg_init", "kavg_set_params", "kavg_set_state",
    "kavg_set_data", "kavg_set_indices", "kavg_local_steps", "kavg_meta_update", "kavg_params",
    "kavg_momentum", "kavg_replica", "kavg_losses", "kavg_indices", "kavg_round", "kavg_last_error",
    "kavg_destroy", "kavg_meta_update_flat", "kavg_profile", "kavg_profile_read",
    "kavg_velocity_bytes", "kavg_set_learner_momentum", "kavg_velocity", "kavg_graph", "kavg_init_static", "kavg_probe", "kavg_refresh_bytes", "kavg_set_refresh",
    "kavg_num_params_conv", "kavg_workspace_bytes_conv", "kavg_init_conv", "kavg_fused", "kavg_set_fused", "kavg_set_wait_limit",
]
STATIC_WORKSPACE_BYTES = 32 << 20
CLASS_NAMES = ["index", "forward", "loss", "backward", "update", "meta", "head", "correction"]


class KavgError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("%s: %s" % (_CODES.get(code, code), text))
        self.code = code


_lib = None


def load_library():
    """Load libkavg.so built in-tree; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch owns the device memory and the stream this library works on, so both must
    # talk to ONE HIP runtime: import torch first, its libamdhip64 is then the one
    # libkavg.so binds to (same SONAME) instead of a second copy from the ROCm tree.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(
            "%s not found: build it with `python -m paper_2110_00625_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_f, c_sz, c_vp = ctypes.c_int, ctypes.c_float, ctypes.c_size_t, ctypes.c_void_p
    ip = ctypes.POINTER(ctypes.c_int)
    lib.kavg_num_params.restype = c_sz
    lib.kavg_num_params.argtypes = [c_int, ip]
    lib.kavg_workspace_bytes.restype = c_sz
    lib.kavg_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, ip, c_int]
    lib.kavg_num_params_conv.restype = c_sz
    lib.kavg_num_params_conv.argtypes = [c_int, c_int, c_int, ip, c_int, ip]
    lib.kavg_workspace_bytes_conv.restype = c_sz
    lib.kavg_workspace_bytes_conv.argtypes = [c_int, c_int, c_int, c_int, c_int, c_int, ip, c_int, ip]
    lib.kavg_init_conv.restype = c_int
    lib.kavg_init_conv.argtypes = [ctypes.POINTER(c_vp), c_int, c_int, c_f, c_f, c_int, c_int, c_int, ip, c_int, ip,
                                   c_int, ctypes.c_uint64, c_vp, c_sz, c_vp]
    lib.kavg_set_wait_limit.restype = c_int
    lib.kavg_set_wait_limit.argtypes = [c_vp, ctypes.c_uint]
    lib.kavg_fused.restype = c_int
    lib.kavg_fused.argtypes = [c_vp]
    lib.kavg_set_fused.restype = c_int
    lib.kavg_set_fused.argtypes = [c_vp, c_int]
    lib.kavg_init.restype = c_int
    lib.kavg_init.argtypes = [ctypes.POINTER(c_vp), c_int, c_int, c_f, c_f, c_int, ip, c_int, c_int,
                              ctypes.c_uint64, c_vp, c_sz, c_vp]
    lib.kavg_init_static.restype = c_int
    lib.kavg_init_static.argtypes = [ctypes.POINTER(c_vp), c_int, c_int, c_f, c_f, c_int, ip, c_int, c_int,
                                     ctypes.c_uint64, c_vp]
    for name, args in {
        "kavg_set_params": [c_vp, c_vp],
        "kavg_set_state": [c_vp, c_vp, c_vp, ctypes.c_uint64],
        "kavg_set_data": [c_vp, c_vp, c_vp, ctypes.c_int64],
        "kavg_set_indices": [c_vp, c_vp],
        "kavg_local_steps": [c_vp],
        "kavg_meta_update": [c_vp],
        "kavg_params": [c_vp, c_vp, c_sz],
        "kavg_momentum": [c_vp, c_vp, c_sz],
        "kavg_replica": [c_vp, c_int, c_vp, c_sz],
        "kavg_losses": [c_vp, c_vp],
        "kavg_indices": [c_vp, c_vp],
        "kavg_destroy": [c_vp],
        "kavg_set_learner_momentum": [c_vp, c_f, c_vp, c_sz],
        "kavg_velocity": [c_vp, c_int, c_vp, c_sz],
        "kavg_profile": [c_vp, ctypes.c_uint, ctypes.c_uint],
        "kavg_profile_read": [c_vp, c_vp, c_vp],
        "kavg_graph": [c_vp, c_int],
        "kavg_set_refresh": [c_vp, c_int, c_vp, c_sz],
        "kavg_meta_update_flat": [c_vp, c_vp, c_vp, c_sz, c_vp, c_sz, c_int, c_sz, c_f, c_vp],
        "kavg_probe": [c_int, c_vp, c_vp, c_sz, c_int, c_vp, c_vp, ctypes.POINTER(ctypes.c_double)],
    }.items():
        fn = getattr(lib, name)
        fn.restype = c_int
        fn.argtypes = args
    lib.kavg_velocity_bytes.restype = c_sz
    lib.kavg_velocity_bytes.argtypes = [c_vp]
    lib.kavg_refresh_bytes.restype = c_sz
    lib.kavg_refresh_bytes.argtypes = [c_vp, c_int]
    lib.kavg_round.restype = ctypes.c_uint64
    lib.kavg_round.argtypes = [c_vp]
    lib.kavg_last_error.restype = ctypes.c_char_p
    lib.kavg_last_error.argtypes = [c_vp]
    _lib = lib
    return lib


def _dims_array(dims):
    return (ctypes.c_int * len(dims))(*[int(d) for d in dims])


def _check(lib, ctx, rc):
    if rc != KAVG_OK:
        raise KavgError(rc, lib.kavg_last_error(ctx).decode())


def kavg_num_params(dims):
    return int(load_library().kavg_num_params(len(dims) - 1, _dims_array(dims)))


def kavg_workspace_bytes(P, K, B, dims, dtype):
    return int(load_library().kavg_workspace_bytes(P, K, B, len(dims) - 1, _dims_array(dims), dtype))


def kavg_meta_update_flat(w_tilde, v, replicas, mu, shadow=None, stream=None):
    """Fused meta step on caller tensors: w_tilde [n], v [n], replicas [P][stride>=n] (fp32,
    device); shadow None or int16/bfloat16 [P][sstride]."""
    import torch
    lib = load_library()
    P, n = replicas.shape[0], w_tilde.numel()
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    rc = lib.kavg_meta_update_flat(w_tilde.data_ptr(), v.data_ptr(), replicas.data_ptr(),
                                   replicas.stride(0), None if shadow is None else shadow.data_ptr(),
                                   0 if shadow is None else shadow.stride(0), P, n, float(mu), st)
    if rc != KAVG_OK:
        raise KavgError(rc, "kavg_meta_update_flat rejected its arguments" if rc == KAVG_EINVAL
                        else "HIP launch failed")


PROBE_READ, PROBE_WRITE, PROBE_COPY, PROBE_MFMA = 0, 1, 2, 3


def kavg_probe(kind, a=None, b=None, iters=1, sink=None, stream=None):
    """One probe launch on the current stream; returns the bytes moved / flops done by it."""
    import torch
    lib = load_library()
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    work = ctypes.c_double(0.0)
    nbytes = 0 if a is None else a.numel() * a.element_size()
    rc = lib.kavg_probe(int(kind), None if a is None else a.data_ptr(), None if b is None else b.data_ptr(),
                        nbytes, int(iters), sink.data_ptr(), st, ctypes.byref(work))
    if rc != KAVG_OK:
        raise KavgError(rc, "kavg_probe rejected its arguments" if rc == KAVG_EINVAL else "HIP launch failed")
    return work.value


class MAvg:
    """One kavg_ctx plus the torch tensors it borrows (workspace, data set, indices)."""

    def __init__(self, P, K, lr, mu, dims, B, dtype=KAVG_FP32, index_seed=0, device="cuda:0",
                 static_workspace=False, conv=None):
        """static_workspace: work in the library's own device block (kavg_init_static) instead of a
        torch allocation.  conv = (H, W, channels): 3x3 convolutions in front of the MLP
        (kavg_init_conv; bf16 only)."""
        import torch
        self._torch = torch
        self.lib = load_library()
        self.P, self.K, self.B, self.dims, self.dtype = P, K, B, tuple(int(d) for d in dims), dtype
        self.device = torch.device(device)
        self.ctx = ctypes.c_void_p()
        self.conv = None
        if conv is not None:
            H, W, channels = conv
            self.conv = (int(H), int(W), tuple(int(ch) for ch in channels))
            assert dtype == KAVG_BF16 and not static_workspace
            n_conv, ch = len(self.conv[2]) - 1, _dims_array(self.conv[2])
            nbytes = int(self.lib.kavg_workspace_bytes_conv(P, K, B, H, W, n_conv, ch, len(self.dims) - 1,
                                                            _dims_array(self.dims)))
        else:
            nbytes = kavg_workspace_bytes(P, K, B, self.dims, dtype)
        if nbytes == 0:
            raise KavgError(KAVG_EINVAL, "kavg_workspace_bytes rejected the configuration")
        torch.cuda.set_device(self.device)
        self.stream = torch.cuda.current_stream(self.device)
        if conv is not None:
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            rc = self.lib.kavg_init_conv(ctypes.byref(self.ctx), P, K, float(lr), float(mu), H, W, n_conv, ch,
                                         len(self.dims) - 1, _dims_array(self.dims), B, int(index_seed),
                                         self.workspace.data_ptr(), nbytes, self.stream.cuda_stream)
        elif static_workspace:
            self.workspace = None
            rc = self.lib.kavg_init_static(ctypes.byref(self.ctx), P, K, float(lr), float(mu), len(self.dims) - 1,
                                           _dims_array(self.dims), B, dtype, int(index_seed),
                                           self.stream.cuda_stream)
        else:
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            rc = self.lib.kavg_init(ctypes.byref(self.ctx), P, K, float(lr), float(mu), len(self.dims) - 1,
                                    _dims_array(self.dims), B, dtype, int(index_seed),
                                    self.workspace.data_ptr(), nbytes, self.stream.cuda_stream)
        if rc != KAVG_OK:
            raise KavgError(rc, self.lib.kavg_last_error(None).decode())
        self.n = kavg_num_params(self.dims)
        if self.conv is not None:
            self.n = int(self.lib.kavg_num_params_conv(self.conv[0], self.conv[1], len(self.conv[2]) - 1,
                                                       _dims_array(self.conv[2]), len(self.dims) - 1,
                                                       _dims_array(self.dims)))
        self._keep = {}

    # -- inputs -----------------------------------------------------------
    def set_params(self, w0):
        w0 = np.ascontiguousarray(w0, dtype=np.float32)
        assert w0.size == self.n
        _check(self.lib, self.ctx, self.lib.kavg_set_params(self.ctx, w0.ctypes.data))

    def set_state(self, w, v, round_):
        w = np.ascontiguousarray(w, dtype=np.float32)
        v = np.ascontiguousarray(v, dtype=np.float32)
        assert w.size == self.n and v.size == self.n
        _check(self.lib, self.ctx, self.lib.kavg_set_state(self.ctx, w.ctypes.data, v.ctypes.data, int(round_)))

    def set_data(self, X_dev, y_dev):
        """X_dev: device tensor [N][d0], float32 (fp32 mode) or bfloat16/int16 bit patterns (bf16 mode);
        y_dev: device int32 [N]."""
        torch = self._torch
        assert X_dev.is_cuda and y_dev.is_cuda and X_dev.is_contiguous() and y_dev.is_contiguous()
        assert y_dev.dtype == torch.int32
        if self.conv is None:
            assert X_dev.shape[1] == self.dims[0]
        else:
            assert tuple(X_dev.shape[1:]) == (self.conv[0], self.conv[1], self.conv[2][0])
        if self.dtype == KAVG_FP32:
            assert X_dev.dtype == torch.float32
        else:
            assert X_dev.dtype in (torch.bfloat16, torch.int16, torch.uint16)
        self._keep["X"], self._keep["y"] = X_dev, y_dev
        _check(self.lib, self.ctx, self.lib.kavg_set_data(self.ctx, X_dev.data_ptr(), y_dev.data_ptr(),
                                                          X_dev.shape[0]))

    def set_indices(self, idx_dev):
        if idx_dev is None:
            self._keep.pop("idx", None)
            _check(self.lib, self.ctx, self.lib.kavg_set_indices(self.ctx, None))
            return
        assert idx_dev.is_cuda and idx_dev.dtype == self._torch.int32 and idx_dev.is_contiguous()
        assert idx_dev.numel() == self.P * self.K * self.B
        self._keep["idx"] = idx_dev
        _check(self.lib, self.ctx, self.lib.kavg_set_indices(self.ctx, idx_dev.data_ptr()))

    def set_learner_momentum(self, beta):
        """Heavy-ball momentum inside every learner (0 switches it off); allocates the velocity block."""
        if beta == 0:
            _check(self.lib, self.ctx, self.lib.kavg_set_learner_momentum(self.ctx, 0.0, None, 0))
            self._keep.pop("vel", None)
            return
        nbytes = int(self.lib.kavg_velocity_bytes(self.ctx))
        vel = self._torch.empty(nbytes, dtype=self._torch.uint8, device=self.device)
        self._keep["vel"] = vel
        _check(self.lib, self.ctx, self.lib.kavg_set_learner_momentum(self.ctx, float(beta), vel.data_ptr(), nbytes))

    def velocity(self, j):
        return self._out(self.lib.kavg_velocity, int(j))

    @property
    def fused(self):
        """True when kavg_local_steps runs all K steps of this context in one launch."""
        return bool(self.lib.kavg_fused(self.ctx))

    def set_fused(self, on):
        _check(self.lib, self.ctx, self.lib.kavg_set_fused(self.ctx, 1 if on else 0))

    def set_wait_limit(self, polls):
        _check(self.lib, self.ctx, self.lib.kavg_set_wait_limit(self.ctx, int(polls)))

    def set_refresh(self, m):
        """Bring the stored replicas up to date every m local steps only (1 = every step, the default);
        allocates the history block."""
        if m == 1:
            _check(self.lib, self.ctx, self.lib.kavg_set_refresh(self.ctx, 1, None, 0))
            self._keep.pop("hist", None)
            return
        nbytes = int(self.lib.kavg_refresh_bytes(self.ctx, int(m)))
        if nbytes == 0:
            raise KavgError(KAVG_EINVAL, "kavg_refresh_bytes rejected refresh period %d" % m)
        hist = self._torch.empty(nbytes, dtype=self._torch.uint8, device=self.device)
        _check(self.lib, self.ctx, self.lib.kavg_set_refresh(self.ctx, int(m), hist.data_ptr(), nbytes))
        self._keep["hist"] = hist

    # -- the hot path -------------------------------------------------------
    def local_steps(self):
        _check(self.lib, self.ctx, self.lib.kavg_local_steps(self.ctx))

    def meta_update(self):
        _check(self.lib, self.ctx, self.lib.kavg_meta_update(self.ctx))

    # -- outputs ----------------------------------------------------------
    def _out(self, fn, *pre):
        out = np.empty(self.n, dtype=np.float32)
        _check(self.lib, self.ctx, fn(self.ctx, *pre, out.ctypes.data, self.n))
        return out

    def params(self):
        return self._out(self.lib.kavg_params)

    def momentum(self):
        return self._out(self.lib.kavg_momentum)

    def replica(self, j):
        return self._out(self.lib.kavg_replica, int(j))

    def losses(self):
        out = np.empty((self.K, self.P), dtype=np.float32)
        _check(self.lib, self.ctx, self.lib.kavg_losses(self.ctx, out.ctypes.data))
        return out

    def indices(self):
        out = np.empty((self.P, self.K, self.B), dtype=np.int32)
        _check(self.lib, self.ctx, self.lib.kavg_indices(self.ctx, out.ctypes.data))
        return out

    def profile(self, classes, every=1):
        """Bracket one launch in `every` of the named kernel classes with HIP events (() = off)."""
        mask = 0
        for name in classes:
            mask |= 1 << CLASS_NAMES.index(name)
        _check(self.lib, self.ctx, self.lib.kavg_profile(self.ctx, mask, int(every)))

    def graph(self, on=True):
        """Replay the K local steps as one HIP graph (needs a non-default current stream at construction)."""
        _check(self.lib, self.ctx, self.lib.kavg_graph(self.ctx, 1 if on else 0))

    def profile_read(self):
        """{class: (total ms, launches)} since the last profile() call."""
        ms = (ctypes.c_double * len(CLASS_NAMES))()
        cnt = (ctypes.c_longlong * len(CLASS_NAMES))()
        _check(self.lib, self.ctx, self.lib.kavg_profile_read(self.ctx, ms, cnt))
        return {n: (ms[i], int(cnt[i])) for i, n in enumerate(CLASS_NAMES)}

    def round(self):
        return int(self.lib.kavg_round(self.ctx))

    def close(self):
        if self.ctx:
            self.lib.kavg_destroy(self.ctx)
            self.ctx = ctypes.c_void_p()
            self._keep.clear()
            self.workspace = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
