"""ctypes binding of libintsgd.so -- same names as include/intsgd.h, marshalling only.

Tensors are torch tensors on the current HIP device (torch.cuda); every call
enqueues on torch's current stream unless ``stream`` (a raw hipStream_t handle,
e.g. ``torch.cuda.Stream().cuda_stream``) is given.  A non-OK status raises
IntSGDError.  There is no fallback: if the library is missing, importing fails.
"""
import ctypes as C
import os

import torch

__all__ = [
    "IntSGDError", "Desc", "ROUND_NEAREST_EVEN", "ROUND_STOCHASTIC", "WIRE_INT8", "WIRE_INT32",
    "MAX_WORKERS", "default_clip", "library_path", "intsgd_workspace_bytes", "intsgd_prepare",
    "intsgd_release", "intsgd_compress", "intsgd_int_sum", "intsgd_decode_update",
    "intsgd_update_norm", "intsgd_next_alpha", "intsgd_next_alpha_host", "intsgd_compress_sum",
    "intsgd_decode_update_norm", "intsgd_step_fused", "intsgd_step_fused_next_alpha",
    "intsgd_step_fused_static", "STATIC_SCRATCH_BYTES",
    "intsgd_decode_update_momentum", "intsgd_step_momentum", "intsgd_diana_step",
    "intsgd_heuristic_alpha", "intsgd_fused_step_form", "intsgd_status_string", "new_workspace",
    "EXPORTED_SYMBOLS", "LaunchOpts",
]

ROUND_NEAREST_EVEN = 0
ROUND_STOCHASTIC = 1
WIRE_INT8 = 8
WIRE_INT32 = 32
MAX_WORKERS = 128
STATIC_SCRATCH_BYTES = 32 << 20

EXPORTED_SYMBOLS = [
    "intsgd_workspace_bytes", "intsgd_prepare", "intsgd_release",
    "intsgd_compress", "intsgd_step_fused_next_alpha", "intsgd_decode_update_momentum",
    "intsgd_step_momentum", "intsgd_diana_step", "intsgd_heuristic_alpha",
    "intsgd_int_sum", "intsgd_decode_update", "intsgd_update_norm", "intsgd_next_alpha",
    "intsgd_next_alpha_host", "intsgd_compress_sum", "intsgd_decode_update_norm",
    "intsgd_step_fused", "intsgd_fused_step_form", "intsgd_status_string", "intsgd_last_hip_error",
    "intsgd_step_fused_static",
]


def library_path() -> str:
    """The in-tree build; INTSGD_LIBRARY names another build of the same sources (e.g. one
    whose host code is compiled with sanitizers)."""
    override = os.environ.get("INTSGD_LIBRARY")
    if override:
        return override
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libintsgd.so")


def _load():
    path = library_path()
    if not os.path.exists(path):
        raise ImportError(
            "%s is not built; run `python paper_2102_08374_amd/build.py` "
            "(or __graft_entry__.build()) first" % path)
    return C.CDLL(path)


_lib = _load()


class _CLaunchOpts(C.Structure):
    _fields_ = [("tile_coords", C.c_uint32), ("max_workgroups", C.c_uint32),
                ("workgroups_per_cu", C.c_uint32), ("two_phase", C.c_uint32),
                ("start_event", C.c_void_p), ("stop_event", C.c_void_p)]


class _CDesc(C.Structure):
    _fields_ = [("d", C.c_uint64), ("n", C.c_uint32), ("num_blocks", C.c_uint32),
                ("block_offsets", C.POINTER(C.c_uint64)), ("rounding", C.c_int32),
                ("wire", C.c_int32), ("clip", C.c_int32), ("step", C.c_uint32),
                ("seed", C.c_uint64), ("launch", C.POINTER(_CLaunchOpts)),
                ("largest_sum", C.c_void_p)]


_P = C.c_void_p
_DP = C.POINTER(_CDesc)
_PP = C.POINTER(C.c_void_p)
_lib.intsgd_workspace_bytes.argtypes = [_DP]
_lib.intsgd_workspace_bytes.restype = C.c_size_t
_lib.intsgd_prepare.argtypes = [_DP]
_lib.intsgd_release.argtypes = []
_lib.intsgd_release.restype = None
_lib.intsgd_compress.argtypes = [_DP, _PP, _P, _PP, _P, _P, C.c_size_t, _P]
_lib.intsgd_int_sum.argtypes = [_DP, _PP, _P, _P]
_lib.intsgd_decode_update.argtypes = [_DP, _P, _P, C.c_double, _P, _P, _P]
_lib.intsgd_update_norm.argtypes = [_DP, _P, _P, _P, _P, C.c_size_t, _P]
_lib.intsgd_next_alpha.argtypes = [_DP, _P, _P, C.c_double, C.c_double, C.c_double, _P, _P]
_lib.intsgd_next_alpha_host.argtypes = [_DP, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                        C.c_double, C.c_double, C.c_double, C.POINTER(C.c_float)]
_lib.intsgd_compress_sum.argtypes = [_DP, _PP, _P, _P, _P, _P, C.c_size_t, _P]
_lib.intsgd_decode_update_norm.argtypes = [_DP, _P, _P, C.c_double, _P, _P, _P, C.c_size_t, _P]
_lib.intsgd_step_fused.argtypes = [_DP, _PP, _P, C.c_double, _P, _P, _P, _P, C.c_size_t, _P]
_lib.intsgd_step_fused_next_alpha.argtypes = [_DP, _PP, _P, C.c_double, C.c_double, _P, _P,
                                              C.c_double, C.c_double, _P, _P, _P, C.c_size_t, _P]
_lib.intsgd_step_fused_static.argtypes = [_DP, _PP, _P, C.c_double, C.c_double, _P, _P, C.c_double,
                                          C.c_double, _P, _P, _P]
_lib.intsgd_decode_update_momentum.argtypes = [_DP, _P, _P, C.c_double, C.c_double, C.c_double, _P,
                                               _P, _P, _P, C.c_size_t, _P]
_lib.intsgd_diana_step.argtypes = [_DP, _PP, _PP, _P, C.c_double, C.c_double, _P, _P, _P, C.c_double,
                                   C.c_double, _P, _P, _P, C.c_size_t, _P]
_lib.intsgd_heuristic_alpha.argtypes = [_DP, _PP, C.c_uint32, _P, _P, C.c_size_t, _P]
_lib.intsgd_step_momentum.argtypes = [_DP, _PP, _P, C.c_double, C.c_double, C.c_double, C.c_double,
                                      _P, _P, _P, C.c_double, C.c_double, _P, _P, _P, C.c_size_t, _P]
_lib.intsgd_fused_step_form.argtypes = [_DP]
_lib.intsgd_fused_step_form.restype = C.c_int
_lib.intsgd_status_string.argtypes = [C.c_int]
_lib.intsgd_status_string.restype = C.c_char_p
_lib.intsgd_last_hip_error.argtypes = []
_lib.intsgd_last_hip_error.restype = C.c_char_p
for _name in ("intsgd_prepare", "intsgd_compress", "intsgd_int_sum", "intsgd_decode_update",
              "intsgd_update_norm", "intsgd_next_alpha", "intsgd_next_alpha_host",
              "intsgd_compress_sum", "intsgd_decode_update_norm", "intsgd_step_fused",
              "intsgd_step_fused_next_alpha", "intsgd_step_fused_static",
              "intsgd_decode_update_momentum", "intsgd_step_momentum", "intsgd_diana_step",
              "intsgd_heuristic_alpha"):
    getattr(_lib, _name).restype = C.c_int


class IntSGDError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        msg = _lib.intsgd_status_string(self.status).decode()
        if self.status == -4:
            msg += " (" + _lib.intsgd_last_hip_error().decode() + ")"
        super().__init__("%s: %s [%d]" % (where, msg, self.status))


def _check(status, where):
    if status != 0:
        raise IntSGDError(status, where)


def default_clip(n: int, wire: int = WIRE_INT32) -> int:
    """Largest per-worker bound whose n-fold sum fits the wire type (Section 5.1)."""
    return ((1 << (wire - 1)) - 1) // max(1, int(n))


class LaunchOpts:
    """include/intsgd.h's intsgd_launch_opts: per-descriptor launch options (0 = automatic)
    and the optional pair of raw hipEvent_t handles that bracket a call's streaming kernel."""

    def __init__(self, tile_coords=0, max_workgroups=0, workgroups_per_cu=0, two_phase=0,
                 start_event=None, stop_event=None):
        self.c = _CLaunchOpts(int(tile_coords), int(max_workgroups), int(workgroups_per_cu),
                              int(two_phase), start_event or None, stop_event or None)

    def set_events(self, start_event, stop_event):
        """Raw hipEvent_t handles (ints), or None / None to detach."""
        self.c.start_event = start_event or None
        self.c.stop_event = stop_event or None

    def as_tuple(self):
        return (self.c.tile_coords, self.c.max_workgroups, self.c.workgroups_per_cu, self.c.two_phase)


class Desc:
    """Problem statement of include/intsgd.h's intsgd_desc (keeps the offsets and the launch
    options alive)."""

    def __init__(self, d, n, *, rounding=ROUND_NEAREST_EVEN, wire=WIRE_INT32, clip=None, seed=0,
                 step=0, block_offsets=None, opts=None, largest_sum=None):
        self._offsets = None
        num_blocks = 1
        ptr = None
        if block_offsets is not None:
            vals = [int(v) for v in block_offsets]
            num_blocks = len(vals) - 1
            self._offsets = (C.c_uint64 * len(vals))(*vals)
            ptr = C.cast(self._offsets, C.POINTER(C.c_uint64))
        if clip is None:
            clip = default_clip(n, WIRE_INT32)
        self.c = _CDesc(int(d), int(n), int(num_blocks), ptr, int(rounding), int(wire), int(clip),
                        int(step) & 0xFFFFFFFF, int(seed) & 0xFFFFFFFFFFFFFFFF, None, None)
        self.opts = opts
        self.largest_sum = largest_sum

    d = property(lambda self: self.c.d)
    n = property(lambda self: self.c.n)
    num_blocks = property(lambda self: self.c.num_blocks)
    wire = property(lambda self: self.c.wire)

    @property
    def step(self):
        return self.c.step

    @step.setter
    def step(self, k):
        self.c.step = int(k) & 0xFFFFFFFF

    @property
    def opts(self):
        return self._opts

    @opts.setter
    def opts(self, opts):
        """A LaunchOpts (kept alive by this object) or None = automatic."""
        self._opts = opts
        self.c.launch = C.pointer(opts.c) if opts is not None else None

    @property
    def largest_sum(self):
        return self._largest_sum

    @largest_sum.setter
    def largest_sum(self, t):
        """Optional output of the calls whose sweep forms the aggregate: a device int32 tensor
        of B elements that receives max |S_j| per block (read it as unsigned), or None.  Kept
        alive by this object."""
        if t is not None:
            assert t.is_cuda and t.is_contiguous() and t.dtype == torch.int32, "largest_sum: int32 on the device"
            assert t.numel() >= self.c.num_blocks, "largest_sum: one element per block"
        self._largest_sum = t
        self.c.largest_sum = None if t is None else t.data_ptr()

    def ref(self):
        return C.byref(self.c)


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream().cuda_stream
    return C.c_void_p(int(stream))


def _ptr(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


_ITEMSIZE = {torch.float32: 4, torch.int32: 4, torch.int8: 1, torch.float64: 8, torch.int64: 8,
             torch.uint8: 1}


def _need(t, numel, dtypes, what):
    """Shape guard: a device tensor of one of `dtypes` with at least `numel` elements
    (the C ABI sees raw pointers and cannot check extents itself)."""
    if t is None:
        return
    if not isinstance(dtypes, tuple):
        dtypes = (dtypes,)
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise ValueError("%s must be a contiguous device tensor" % what)
    if t.dtype not in dtypes:
        raise ValueError("%s has dtype %s, expected %s" % (what, t.dtype, dtypes))
    if t.numel() < numel:
        raise ValueError("%s has %d elements, needs %d" % (what, t.numel(), numel))


def _need_rows(desc, tensors, dtypes, what):
    if len(tensors) != desc.n:
        raise ValueError("%s: expected %d tensors, got %d" % (what, desc.n, len(tensors)))
    for i, t in enumerate(tensors):
        _need(t, desc.d, dtypes, "%s[%d]" % (what, i))


def _wire_dtype(desc):
    return torch.int8 if desc.wire == WIRE_INT8 else torch.int32


def _ptr_array(tensors):
    return (C.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])


def _ws(workspace):
    if workspace is None:
        return C.c_void_p(0), 0
    _need(workspace, 0, torch.uint8, "workspace")
    return C.c_void_p(workspace.data_ptr()), workspace.numel() * workspace.element_size()


def intsgd_workspace_bytes(desc: Desc) -> int:
    return int(_lib.intsgd_workspace_bytes(desc.ref()))


def new_workspace(desc: Desc, device="cuda") -> torch.Tensor:
    nbytes = intsgd_workspace_bytes(desc)
    if nbytes == 0:
        raise IntSGDError(-1, "intsgd_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def intsgd_prepare(desc: Desc):
    _check(_lib.intsgd_prepare(desc.ref()), "intsgd_prepare")


def intsgd_release():
    _lib.intsgd_release()


def intsgd_compress(desc, grads, alpha, q_out, sat_count, workspace, stream=None):
    _need_rows(desc, grads, torch.float32, "grads")
    _need_rows(desc, q_out, _wire_dtype(desc), "q_out")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(sat_count, desc.n, torch.int64, "sat_count")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_compress(desc.ref(), _ptr_array(grads), _ptr(alpha), _ptr_array(q_out),
                                _ptr(sat_count), w, wb, _stream(stream)), "intsgd_compress")


def intsgd_int_sum(desc, q, sum_out, stream=None):
    _need_rows(desc, q, _wire_dtype(desc), "q")
    _need(sum_out, desc.d, torch.int32, "sum_out")
    _check(_lib.intsgd_int_sum(desc.ref(), _ptr_array(q), _ptr(sum_out), _stream(stream)),
           "intsgd_int_sum")


def intsgd_decode_update(desc, sum_, alpha, eta, x, gtilde_out=None, stream=None):
    _need(sum_, desc.d, torch.int32, "sum")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(x, desc.d, torch.float32, "x")
    _need(gtilde_out, desc.d, torch.float32, "gtilde_out")
    _check(_lib.intsgd_decode_update(desc.ref(), _ptr(sum_), _ptr(alpha), float(eta), _ptr(x),
                                     _ptr(gtilde_out), _stream(stream)), "intsgd_decode_update")


def intsgd_update_norm(desc, x_new, x_old, norm_sq_out, workspace, stream=None):
    _need(x_new, desc.d, torch.float32, "x_new")
    _need(x_old, desc.d, torch.float32, "x_old")
    _need(norm_sq_out, desc.num_blocks, torch.float64, "norm_sq_out")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_update_norm(desc.ref(), _ptr(x_new), _ptr(x_old), _ptr(norm_sq_out), w, wb,
                                   _stream(stream)), "intsgd_update_norm")


def intsgd_next_alpha(desc, norm_sq, r, beta, eps, eta, alpha_out, stream=None):
    _need(norm_sq, desc.num_blocks, torch.float64, "norm_sq")
    _need(r, desc.num_blocks, torch.float64, "r")
    _need(alpha_out, desc.num_blocks, torch.float32, "alpha_out")
    _check(_lib.intsgd_next_alpha(desc.ref(), _ptr(norm_sq), _ptr(r), float(beta), float(eps),
                                  float(eta), _ptr(alpha_out), _stream(stream)),
           "intsgd_next_alpha")


def intsgd_next_alpha_host(desc, norm_sq, r, beta, eps, eta):
    """Host twin: lists/arrays of B doubles -> (status, r_new list, alpha list of fp32 values)."""
    B = desc.num_blocks
    ns = (C.c_double * B)(*[float(v) for v in norm_sq])
    rr = (C.c_double * B)(*[float(v) for v in r])
    al = (C.c_float * B)()
    st = _lib.intsgd_next_alpha_host(desc.ref(), ns, rr, float(beta), float(eps), float(eta), al)
    return int(st), list(rr), list(al)


def intsgd_compress_sum(desc, grads, alpha, sum_out, sat_count, workspace, stream=None):
    _need_rows(desc, grads, torch.float32, "grads")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(sum_out, desc.d, torch.int32, "sum_out")
    _need(sat_count, desc.n, torch.int64, "sat_count")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_compress_sum(desc.ref(), _ptr_array(grads), _ptr(alpha), _ptr(sum_out),
                                    _ptr(sat_count), w, wb, _stream(stream)),
           "intsgd_compress_sum")


def intsgd_decode_update_norm(desc, sum_, alpha, eta, x, norm_sq_out, workspace, stream=None):
    _need(sum_, desc.d, torch.int32, "sum")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(x, desc.d, torch.float32, "x")
    _need(norm_sq_out, desc.num_blocks, torch.float64, "norm_sq_out")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_decode_update_norm(desc.ref(), _ptr(sum_), _ptr(alpha), float(eta), _ptr(x),
                                          _ptr(norm_sq_out), w, wb, _stream(stream)),
           "intsgd_decode_update_norm")


def intsgd_step_fused(desc, grads, alpha, eta, x, norm_sq_out, sat_count, workspace, stream=None):
    _need_rows(desc, grads, torch.float32, "grads")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(x, desc.d, torch.float32, "x")
    _need(norm_sq_out, desc.num_blocks, torch.float64, "norm_sq_out")
    _need(sat_count, desc.n, torch.int64, "sat_count")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_step_fused(desc.ref(), _ptr_array(grads), _ptr(alpha), float(eta), _ptr(x),
                                  _ptr(norm_sq_out), _ptr(sat_count), w, wb, _stream(stream)),
           "intsgd_step_fused")


def intsgd_step_fused_next_alpha(desc, grads, alpha, eta, x, r, beta, eps, norm_sq_out, sat_count,
                                 workspace, stream=None, eta_next=None):
    """eta_next: the next step's stepsize (None = the same eta)."""
    _need_rows(desc, grads, torch.float32, "grads")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(x, desc.d, torch.float32, "x")
    _need(r, desc.num_blocks, torch.float64, "r")
    _need(norm_sq_out, desc.num_blocks, torch.float64, "norm_sq_out")
    _need(sat_count, desc.n, torch.int64, "sat_count")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_step_fused_next_alpha(desc.ref(), _ptr_array(grads), _ptr(alpha), float(eta),
                                             float(eta if eta_next is None else eta_next),
                                             _ptr(x), _ptr(r), float(beta), float(eps),
                                             _ptr(norm_sq_out), _ptr(sat_count), w, wb,
                                             _stream(stream)), "intsgd_step_fused_next_alpha")


def intsgd_step_fused_static(desc, grads, alpha, eta, x, r, beta, eps, norm_sq_out, sat_count,
                             stream=None, eta_next=None):
    """intsgd_step_fused_next_alpha on the library's static scratch: no workspace, no allocation."""
    _need_rows(desc, grads, torch.float32, "grads")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(x, desc.d, torch.float32, "x")
    _need(r, desc.num_blocks, torch.float64, "r")
    _need(norm_sq_out, desc.num_blocks, torch.float64, "norm_sq_out")
    _need(sat_count, desc.n, torch.int64, "sat_count")
    _check(_lib.intsgd_step_fused_static(desc.ref(), _ptr_array(grads), _ptr(alpha), float(eta),
                                         float(eta if eta_next is None else eta_next), _ptr(x),
                                         _ptr(r), float(beta), float(eps), _ptr(norm_sq_out),
                                         _ptr(sat_count), _stream(stream)),
           "intsgd_step_fused_static")


def intsgd_decode_update_momentum(desc, sum_, alpha, eta, mu, weight_decay, x, m, norm_sq_out,
                                  workspace, stream=None):
    _need(sum_, desc.d, torch.int32, "sum")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(x, desc.d, torch.float32, "x")
    _need(m, desc.d, torch.float32, "m")
    _need(norm_sq_out, desc.num_blocks, torch.float64, "norm_sq_out")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_decode_update_momentum(desc.ref(), _ptr(sum_), _ptr(alpha), float(eta),
                                              float(mu), float(weight_decay), _ptr(x), _ptr(m),
                                              _ptr(norm_sq_out), w, wb, _stream(stream)),
           "intsgd_decode_update_momentum")


def intsgd_step_momentum(desc, grads, alpha, eta, mu, weight_decay, x, m, r, beta, eps, norm_sq_out,
                         sat_count, workspace, stream=None, eta_next=None):
    """r may be None: alpha is then only read (no a8).  eta_next: the next step's stepsize."""
    _need_rows(desc, grads, torch.float32, "grads")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(x, desc.d, torch.float32, "x")
    _need(m, desc.d, torch.float32, "m")
    _need(r, desc.num_blocks, torch.float64, "r")
    _need(norm_sq_out, desc.num_blocks, torch.float64, "norm_sq_out")
    _need(sat_count, desc.n, torch.int64, "sat_count")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_step_momentum(desc.ref(), _ptr_array(grads), _ptr(alpha), float(eta),
                                     float(eta if eta_next is None else eta_next),
                                     float(mu), float(weight_decay), _ptr(x), _ptr(m), _ptr(r),
                                     float(beta), float(eps), _ptr(norm_sq_out), _ptr(sat_count),
                                     w, wb, _stream(stream)), "intsgd_step_momentum")


def intsgd_diana_step(desc, grads, h_local, alpha, eta, x, h, r, beta, eps, norm_sq_out, sat_count,
                      workspace, stream=None, eta_next=None):
    """IntDIANA step; r may be None (alpha only read).  eta_next: the next step's stepsize."""
    _need_rows(desc, grads, torch.float32, "grads")
    _need_rows(desc, h_local, torch.float32, "h_local")
    _need(alpha, desc.num_blocks, torch.float32, "alpha")
    _need(x, desc.d, torch.float32, "x")
    _need(h, desc.d, torch.float32, "h")
    _need(r, desc.num_blocks, torch.float64, "r")
    _need(norm_sq_out, desc.num_blocks, torch.float64, "norm_sq_out")
    _need(sat_count, desc.n, torch.int64, "sat_count")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_diana_step(desc.ref(), _ptr_array(grads), _ptr_array(h_local), _ptr(alpha),
                                  float(eta), float(eta if eta_next is None else eta_next), _ptr(x), _ptr(h), _ptr(r), float(beta), float(eps),
                                  _ptr(norm_sq_out), _ptr(sat_count), w, wb, _stream(stream)),
           "intsgd_diana_step")


def intsgd_heuristic_alpha(desc, grads, nb, alpha_out, workspace, stream=None):
    _need_rows(desc, grads, torch.float32, "grads")
    _need(alpha_out, desc.num_blocks, torch.float32, "alpha_out")
    w, wb = _ws(workspace)
    _check(_lib.intsgd_heuristic_alpha(desc.ref(), _ptr_array(grads), int(nb), _ptr(alpha_out), w, wb,
                                       _stream(stream)), "intsgd_heuristic_alpha")


def intsgd_fused_step_form(desc: "Desc") -> int:
    """1 = tile sweep, 2 = two-phase sweep (what the fused step would launch now)."""
    return int(_lib.intsgd_fused_step_form(desc.ref()))


def intsgd_status_string(status: int) -> str:
    return _lib.intsgd_status_string(int(status)).decode()
