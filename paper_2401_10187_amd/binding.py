"""ctypes binding of the C-ABI in include/kronmatmul.h.  Argument marshalling only: every step of
the computation runs in the HIP library.  There is no fallback: a missing library is an error."""
import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libkronmatmul.so")

KM_F32, KM_F64 = 0, 1
KM_OK, KM_EINVAL, KM_ENOMEM, KM_ELAUNCH, KM_EUNSUPPORTED = 0, 1, 2, 3, 4
KM_KERNEL_GENERIC, KM_KERNEL_FUSED, KM_KERNEL_MFMA, KM_KERNEL_SHUFFLE, KM_KERNEL_ROWS, KM_KERNEL_MFMA_ANY = 0, 1, 2, 3, 4, 5
KM_BUF_X, KM_BUF_Y, KM_BUF_WS0, KM_BUF_WS1 = 0, 1, 2, 3
KM_OPT_KERNELS, KM_OPT_MAX_FUSE, KM_OPT_PROFILE, KM_OPT_PREFER_TILE, KM_OPT_PREFER_THREADS, KM_OPT_TILES_PER_WG, KM_OPT_PAIR_INTERLEAVE, KM_OPT_TILE_ORDER = 0, 1, 2, 3, 4, 5, 6, 7
KM_OPT_PREFER_INSTANCE, KM_OPT_INSTANCE_COUNT, KM_OPT_KEEP_MIB = 8, 9, 10

EXPORTS = [
    "kronmatmul_workspace_size", "kronmatmul", "kronmatmul_ws", "kronmatmul_plan",
    "kronmatmul_store_column", "kronmatmul_cost", "kronmatmul_set_option", "kronmatmul_get_option",
    "kronmatmul_last_profile", "kronmatmul_mean_profile", "kronmatmul_release", "kronmatmul_status_string",
    "kronmatmul_kernel_name", "kronmatmul_tune",
    "kronmatmul_transposed_workspace_size", "kronmatmul_transposed", "kronmatmul_transposed_ws",
    "kronmatmul_clock_probe", "kronmatmul_prepare", "kronmatmul_static",
]
KM_STATIC_SCRATCH_BYTES = 16 << 20


class PlanStep(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int), ("first_factor", ctypes.c_int), ("num_factors", ctypes.c_int),
                ("tile_slices", ctypes.c_int), ("k_in", ctypes.c_longlong), ("k_out", ctypes.c_longlong),
                ("src", ctypes.c_int), ("dst", ctypes.c_int), ("grid", ctypes.c_longlong),
                ("block", ctypes.c_int), ("lds_bytes", ctypes.c_int), ("variant", ctypes.c_int),
                ("tiles_per_wg", ctypes.c_int), ("tile_order", ctypes.c_int), ("tile_rows", ctypes.c_int)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class KronMatmulError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__("%s: %s" % (what, status_string(status)))


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("HIP library %s is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                               "(there is no CPU fallback)" % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        ci, vp, ip = ctypes.c_int, ctypes.c_void_p, ctypes.POINTER(ctypes.c_int)
        ll = ctypes.c_longlong
        L.kronmatmul_workspace_size.restype = ci
        L.kronmatmul_workspace_size.argtypes = [ci, ci, ip, ip, ci, ctypes.POINTER(ctypes.c_size_t)]
        L.kronmatmul.restype = ci
        L.kronmatmul.argtypes = [ci, ci, ip, ip, vp, vp, vp, ci, vp]
        L.kronmatmul_static.restype = ci
        L.kronmatmul_static.argtypes = [ci, ci, ip, ip, vp, vp, vp, ci, vp]
        L.kronmatmul_prepare.restype = ci
        L.kronmatmul_prepare.argtypes = [ci, ci, ip, ip, ci]
        L.kronmatmul_ws.restype = ci
        L.kronmatmul_ws.argtypes = [ci, ci, ip, ip, vp, vp, vp, ci, vp, ctypes.c_size_t, vp]
        L.kronmatmul_transposed_workspace_size.restype = ci
        L.kronmatmul_transposed_workspace_size.argtypes = [ci, ci, ip, ip, ci, ctypes.POINTER(ctypes.c_size_t)]
        L.kronmatmul_transposed.restype = ci
        L.kronmatmul_transposed.argtypes = [ci, ci, ip, ip, vp, vp, vp, ci, vp]
        L.kronmatmul_transposed_ws.restype = ci
        L.kronmatmul_transposed_ws.argtypes = [ci, ci, ip, ip, vp, vp, vp, ci, vp, ctypes.c_size_t, vp]
        L.kronmatmul_plan.restype = ci
        L.kronmatmul_plan.argtypes = [ci, ci, ip, ip, ci, ctypes.POINTER(PlanStep), ci, ip]
        L.kronmatmul_tune.restype = ci
        L.kronmatmul_tune.argtypes = [ci, ci, ip, ip, ci, vp, ctypes.POINTER(ctypes.c_float),
                                      ctypes.POINTER(ctypes.c_float)]
        L.kronmatmul_store_column.restype = ll
        L.kronmatmul_store_column.argtypes = [ll, ll, ll, ll, ll]
        L.kronmatmul_cost.restype = ci
        L.kronmatmul_cost.argtypes = [ci, ci, ip, ip, ci, ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double)]
        L.kronmatmul_set_option.restype = ci
        L.kronmatmul_set_option.argtypes = [ci, ci]
        L.kronmatmul_get_option.restype = ci
        L.kronmatmul_get_option.argtypes = [ci, ip]
        L.kronmatmul_last_profile.restype = ci
        L.kronmatmul_last_profile.argtypes = [ctypes.POINTER(ctypes.c_float), ci, ip]
        L.kronmatmul_mean_profile.restype = ci
        L.kronmatmul_mean_profile.argtypes = [ctypes.POINTER(ctypes.c_float), ci, ip, ip]
        L.kronmatmul_clock_probe.restype = ci
        L.kronmatmul_clock_probe.argtypes = [vp, ci, vp]
        L.kronmatmul_release.restype = ci
        L.kronmatmul_release.argtypes = []
        L.kronmatmul_status_string.restype = ctypes.c_char_p
        L.kronmatmul_status_string.argtypes = [ci]
        L.kronmatmul_kernel_name.restype = ctypes.c_char_p
        L.kronmatmul_kernel_name.argtypes = [ci]
        _lib = L
    return _lib


def status_string(status):
    return lib().kronmatmul_status_string(int(status)).decode()


def kernel_name(kernel):
    return lib().kronmatmul_kernel_name(int(kernel)).decode()


def _check(status, what):
    if status != KM_OK:
        raise KronMatmulError(status, what)


def _shapes(P, Q):
    P = [int(p) for p in P]
    Q = [int(q) for q in Q]
    if len(P) != len(Q):
        raise ValueError("P and Q differ in length")
    n = len(P)
    return n, (ctypes.c_int * max(n, 1))(*P), (ctypes.c_int * max(n, 1))(*Q)


def _dtype_code(dtype):
    name = str(dtype).replace("torch.", "")
    if name in ("float32", "f32", "0"):
        return KM_F32
    if name in ("float64", "f64", "1"):
        return KM_F64
    raise TypeError("unsupported dtype %r (float32 and float64 only)" % (dtype,))


def workspace_size(M, P, Q, dtype, transposed=False):
    """Bytes of workspace kronmatmul_ws (or, with transposed=True, kronmatmul_transposed_ws) needs."""
    n, p, q = _shapes(P, Q)
    out = ctypes.c_size_t(0)
    fn = lib().kronmatmul_transposed_workspace_size if transposed else lib().kronmatmul_workspace_size
    _check(fn(int(M), n, p, q, _dtype_code(dtype), ctypes.byref(out)), "kronmatmul_workspace_size")
    return int(out.value)


def prepare(M, P, Q, dtype):
    """Set-up on the current device: plan the problem and set its kernels' attributes (before graph capture)."""
    n, p, q = _shapes(P, Q)
    _check(lib().kronmatmul_prepare(int(M), n, p, q, _dtype_code(dtype)), "kronmatmul_prepare")


def plan(M, P, Q, dtype):
    """List of dicts, one per kernel launch, in launch order."""
    n, p, q = _shapes(P, Q)
    cap = 64
    steps = (PlanStep * cap)()
    cnt = ctypes.c_int(0)
    _check(lib().kronmatmul_plan(int(M), n, p, q, _dtype_code(dtype), steps, cap, ctypes.byref(cnt)),
           "kronmatmul_plan")
    return [steps[i].as_dict() for i in range(min(cnt.value, cap))]


def tune(M, P, Q, dtype, stream=None):
    """Measures the compiled kernel instances for this problem on the current device and keeps the
    fastest plan for later calls.  Returns (kept_ms, cost_model_ms) per call."""
    import torch
    n, p, q = _shapes(P, Q)
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    kept, model = ctypes.c_float(0), ctypes.c_float(0)
    _check(lib().kronmatmul_tune(int(M), n, p, q, _dtype_code(dtype), ctypes.c_void_p(stream),
                                 ctypes.byref(kept), ctypes.byref(model)), "kronmatmul_tune")
    return float(kept.value), float(model.value)


def cost(M, P, Q, dtype):
    """(flops, planned_bytes)."""
    n, p, q = _shapes(P, Q)
    fl, by = ctypes.c_double(0), ctypes.c_double(0)
    _check(lib().kronmatmul_cost(int(M), n, p, q, _dtype_code(dtype), ctypes.byref(fl), ctypes.byref(by)),
           "kronmatmul_cost")
    return fl.value, by.value


def store_column(k_in, p_group, tile_k, tile_index, local_col):
    return int(lib().kronmatmul_store_column(int(k_in), int(p_group), int(tile_k), int(tile_index),
                                             int(local_col)))


def set_option(option, value):
    _check(lib().kronmatmul_set_option(int(option), int(value)), "kronmatmul_set_option")


def get_option(option):
    v = ctypes.c_int(0)
    _check(lib().kronmatmul_get_option(int(option), ctypes.byref(v)), "kronmatmul_get_option")
    return v.value


def last_profile():
    """Milliseconds per launch of the last call made with KM_OPT_PROFILE = 1."""
    cap = 64
    ms = (ctypes.c_float * cap)()
    cnt = ctypes.c_int(0)
    _check(lib().kronmatmul_last_profile(ms, cap, ctypes.byref(cnt)), "kronmatmul_last_profile")
    return [float(ms[i]) for i in range(min(cnt.value, cap))]


def mean_profile():
    """(list of mean milliseconds per launch, number of calls averaged) since profiling was enabled."""
    cap = 64
    ms = (ctypes.c_float * cap)()
    cnt, calls = ctypes.c_int(0), ctypes.c_int(0)
    _check(lib().kronmatmul_mean_profile(ms, cap, ctypes.byref(cnt), ctypes.byref(calls)),
           "kronmatmul_mean_profile")
    return [float(ms[i]) for i in range(min(cnt.value, cap))], calls.value


def clock_probe(ticks, micros, stream):
    """Enqueue the clock probe on `stream` (a torch stream): `ticks` is a CUDA int64 tensor of two
    elements that receives the shader-clock and 100 MHz-clock advances over about `micros` us."""
    import torch
    if ticks.dtype != torch.int64 or ticks.numel() < 2 or not ticks.is_cuda or not ticks.is_contiguous():
        raise ValueError("ticks must be a contiguous CUDA int64 tensor of two elements")
    _check(lib().kronmatmul_clock_probe(ctypes.c_void_p(ticks.data_ptr()), int(micros),
                                        ctypes.c_void_p(stream.cuda_stream)), "kronmatmul_clock_probe")


def release():
    _check(lib().kronmatmul_release(), "kronmatmul_release")


class Prepared:
    """A Kron-Matmul call with its arguments already checked and marshalled: calling it only crosses
    the C-ABI (for iterative callers that repeat one small problem, where marshalling would cost
    more than the kernels).  Keeps references to the tensors it was built from."""

    def __init__(self, X, Fs, Y=None, workspace=None, transposed=False):
        import torch
        self._torch = torch
        self.Y, self._args, self._ws_call, fptr = _marshal(X, Fs, Y, workspace, transposed)
        self._keep = (X, list(Fs), workspace, fptr)
        self._device = X.device
        self._what = _entry_name(self._ws_call, transposed)
        self._fn = getattr(lib(), self._what)

    def __call__(self, stream=None):
        """Enqueue on `stream` (a raw hipStream_t value; default: torch's current stream).  The
        tensors' device must be the current device."""
        if stream is None:
            stream = self._torch.cuda.current_stream(self._device).cuda_stream
        st = self._fn(*self._args, ctypes.c_void_p(stream))
        if st != KM_OK:
            raise KronMatmulError(st, self._what)
        return self.Y


def _entry_name(with_ws, transposed, static=False):
    if static:
        return "kronmatmul_static"
    return "kronmatmul" + ("_transposed" if transposed else "") + ("_ws" if with_ws else "")


def _marshal(X, Fs, Y, workspace, transposed=False):
    """Checks the tensors and returns (Y, C argument tuple without the stream, uses_workspace, the
    pointer array the tuple refers to)."""
    import torch
    if not X.is_cuda or X.dim() != 2 or not X.is_contiguous():
        raise ValueError("X must be a contiguous 2-D CUDA tensor")
    P, Q = [], []
    for F in Fs:
        if not F.is_cuda or F.dim() != 2 or not F.is_contiguous() or F.dtype != X.dtype or F.device != X.device:
            raise ValueError("factors must be contiguous 2-D CUDA tensors of X's dtype and device")
        P.append(F.shape[1] if transposed else F.shape[0])
        Q.append(F.shape[0] if transposed else F.shape[1])
    n, p, q = _shapes(P, Q)
    kin = kout = 1
    for a, b in zip(P, Q):
        kin *= a
        kout *= b
    M = X.shape[0]
    if X.shape[1] != kin:
        raise ValueError("X has %d columns, the factors need %d" % (X.shape[1], kin))
    if Y is None:
        Y = torch.empty((M, kout), dtype=X.dtype, device=X.device)
    elif (not Y.is_cuda or not Y.is_contiguous() or Y.dtype != X.dtype or tuple(Y.shape) != (M, kout)
          or Y.device != X.device):
        raise ValueError("Y must be a contiguous CUDA tensor of shape (%d, %d)" % (M, kout))
    code = _dtype_code(X.dtype)
    fptr = (ctypes.c_void_p * max(n, 1))(*[F.data_ptr() for F in Fs])
    head = (M, n, p, q, X.data_ptr(), ctypes.cast(fptr, ctypes.c_void_p), Y.data_ptr(), code)
    if workspace is None:
        return Y, head, False, fptr
    if not workspace.is_cuda or not workspace.is_contiguous() or workspace.device != X.device:
        raise ValueError("workspace must be a contiguous CUDA tensor on X's device")
    nbytes = workspace.numel() * workspace.element_size()
    return Y, head + (workspace.data_ptr(), nbytes), True, fptr


def kronmatmul(X, Fs, Y=None, workspace=None, stream=None, transposed=False, static=False):
    """Y = X (Fs[0] (x) ... (x) Fs[-1]) on the GPU.  X, Fs, Y and workspace are torch CUDA tensors
    (contiguous, same dtype).  With workspace=None the library's own cached workspace is used.
    With transposed=True every Fs[i] holds the transpose of the factor applied (shape Q_i x P_i).
    With static=True the call goes to kronmatmul_static (no allocation; Y must then be given, or the
    binding's own torch.empty allocates it).
    Returns Y.  The call is asynchronous on `stream` (default: torch's current stream)."""
    import torch
    if static and (workspace is not None or transposed):
        raise ValueError("static=True takes neither a workspace nor transposed factors")
    Y, args, with_ws, _fptr = _marshal(X, Fs, Y, workspace, transposed)
    if stream is None:
        stream = torch.cuda.current_stream(X.device).cuda_stream
    name = _entry_name(with_ws, transposed, static)
    with torch.cuda.device(X.device):
        _check(getattr(lib(), name)(*args, ctypes.c_void_p(stream)), name)
    return Y
