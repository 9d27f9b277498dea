"""Thin ctypes binding of libftp.so: argument marshalling only, same names as the C ABI.

Every step of the path runs in the library's HIP kernels.  If the library has not been built,
importing this module raises: there is no fallback.  Device buffers are passed as integer
addresses (e.g. torch.Tensor.data_ptr()) and the stream as a hipStream_t value
(torch.cuda.current_stream().cuda_stream).
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libftp.so")

FTP_CONV, FTP_MAXPOOL = 0, 1
FTP_F32, FTP_BF16 = 0, 1
FTP_RECT_OWN, FTP_RECT_FWD, FTP_RECT_BWD = 0, 1, 2
FTP_OK, FTP_EINVAL, FTP_EUNSUPPORTED, FTP_EGRID, FTP_EGROUPS, FTP_ENOMEM, FTP_EHIP, FTP_ECHANNELS, FTP_ETOOLARGE = 0, -1, -2, -3, -4, -5, -6, -7, -8
FTP_STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024


class ftp_layer(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("k", ctypes.c_int32), ("stride", ctypes.c_int32), ("pad", ctypes.c_int32),
                ("cin", ctypes.c_int32), ("cout", ctypes.c_int32), ("leaky_slope", ctypes.c_float),
                ("has_bias", ctypes.c_int32)]


class ftp_kernel_time(ctypes.Structure):
    _fields_ = [("pass_", ctypes.c_int32), ("layer", ctypes.c_int32), ("launches", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("total_ms", ctypes.c_double), ("flops_per_launch", ctypes.c_double),
                ("bytes_per_launch", ctypes.c_double), ("kernel", ctypes.c_char * 96),
                ("executed_flops_per_launch", ctypes.c_double)]


PASS_NAMES = {0: "conv_fwd", 1: "conv_bwd_data", 2: "wgrad", 3: "reduce", 4: "pool_fwd", 5: "pool_bwd", 6: "scale_dy", 7: "update", 8: "wgrad_sum"}


class FtpError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        msg = _lib.ftp_strerror(code).decode()
        if code == FTP_EHIP:
            msg += " (hipError %d)" % _lib.ftp_last_hip_error()
        super().__init__("%s: %s [%d]" % (where, msg, code))


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError("libftp.so is not built: run `python -m paper_2409_09083_amd.build` "
                          "(or __graft_entry__.build()); there is no CPU fallback")
    # One HIP runtime per process: PyTorch ships its own libamdhip64 (same soname as ROCm's).  Load that
    # copy first, so that libftp binds to it whether or not torch has been imported yet; a second runtime
    # instance in the process would not see the device torch allocated the buffers on.
    try:
        import importlib.util
        spec = importlib.util.find_spec("torch")
        if spec is not None and spec.origin:
            hip = os.path.join(os.path.dirname(spec.origin), "lib", "libamdhip64.so")
            if os.path.exists(hip):
                ctypes.CDLL(hip, mode=ctypes.RTLD_GLOBAL)
    except Exception:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.ftp_plan.argtypes = [ctypes.POINTER(ftp_layer), i32, i32, i32, i32, i32, i32, i32,
                             ctypes.POINTER(i32), i32, ctypes.c_int, ctypes.POINTER(vp)]
    lib.ftp_plan.restype = ctypes.c_int
    lib.ftp_plan_destroy.argtypes = [vp]
    lib.ftp_plan_destroy.restype = None
    lib.ftp_plan_rect.argtypes = [vp, i32, i32, i32, i32, ctypes.c_int, ctypes.POINTER(i32)]
    lib.ftp_plan_map_shape.argtypes = [vp, i32, ctypes.POINTER(i32)]
    lib.ftp_plan_sizes.argtypes = [vp, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)]
    lib.ftp_plan_work.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                  ctypes.POINTER(ctypes.c_double)]
    lib.ftp_plan_buffer.argtypes = [vp, i32, ctypes.c_int, ctypes.POINTER(ctypes.c_int64)]
    lib.ftp_forward.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp, vp]
    lib.ftp_forward_static.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), vp, vp]
    lib.ftp_backward.argtypes = [vp, vp, vp, ctypes.POINTER(vp), vp, vp, vp, vp]
    lib.ftp_reduce_wgrad.argtypes = [vp, vp, vp, vp]
    lib.ftp_sgd_step.argtypes = [vp, vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.c_float, vp, vp]
    lib.ftp_profile.argtypes = [vp, i32]
    lib.ftp_set_overlap.argtypes = [vp, i32]
    lib.ftp_profile_read.argtypes = [vp, ctypes.POINTER(ftp_kernel_time), i32, ctypes.POINTER(i32)]
    lib.ftp_strerror.argtypes = [ctypes.c_int]
    lib.ftp_strerror.restype = ctypes.c_char_p
    lib.ftp_last_hip_error.restype = ctypes.c_int
    for f in ("ftp_profile", "ftp_profile_read", "ftp_set_overlap", "ftp_plan_buffer", "ftp_plan_rect", "ftp_plan_map_shape", "ftp_plan_sizes", "ftp_plan_work", "ftp_forward",
              "ftp_forward_static", "ftp_backward", "ftp_reduce_wgrad", "ftp_sgd_step"):
        getattr(lib, f).restype = ctypes.c_int
    return lib


_lib = _load()

EXPORTS = ("ftp_profile", "ftp_profile_read", "ftp_set_overlap", "ftp_plan", "ftp_plan_destroy", "ftp_plan_buffer", "ftp_plan_rect", "ftp_plan_map_shape", "ftp_plan_sizes", "ftp_plan_work",
           "ftp_forward", "ftp_forward_static", "ftp_backward", "ftp_reduce_wgrad", "ftp_sgd_step", "ftp_strerror", "ftp_last_hip_error")


def _check(rc, where):
    if rc != 0:
        raise FtpError(rc, where)


def _ptr_array(ptrs, n):
    if ptrs is None:
        return None
    arr = (ctypes.c_void_p * n)()
    for i, p in enumerate(ptrs):
        arr[i] = None if not p else int(p)
    return arr


def ftp_plan(layers, batch, in_c, in_h, in_w, grid_rows, grid_cols, group_ends, dtype=FTP_F32):
    """layers: sequence of objects/tuples (kind, k, stride, pad, cin, cout, slope[, has_bias]).  Returns a plan handle."""
    n = len(layers)
    arr = (ftp_layer * max(n, 1))()
    for i, ly in enumerate(layers):
        if isinstance(ly, (tuple, list)):
            kind, k, stride, pad, cin, cout, slope = ly[:7]
            has_bias = ly[7] if len(ly) > 7 else 0
        else:
            kind, k, stride, pad, cin, cout, slope = ly.kind, ly.k, ly.stride, ly.pad, ly.cin, ly.cout, ly.slope
            has_bias = int(getattr(ly, "has_bias", 0))
        arr[i] = ftp_layer(kind, k, stride, pad, cin, cout, slope, has_bias)
    ge = (ctypes.c_int32 * max(len(group_ends), 1))(*group_ends)
    out = ctypes.c_void_p()
    _check(_lib.ftp_plan(arr, n, batch, in_c, in_h, in_w, grid_rows, grid_cols, ge, len(group_ends), dtype,
                         ctypes.byref(out)), "ftp_plan")
    return out


def ftp_plan_destroy(plan):
    _lib.ftp_plan_destroy(plan)


def ftp_plan_rect(plan, group, boundary, ti, tj, kind):
    out = (ctypes.c_int32 * 4)()
    _check(_lib.ftp_plan_rect(plan, group, boundary, ti, tj, kind, out), "ftp_plan_rect")
    return tuple(out)


def ftp_plan_map_shape(plan, boundary):
    out = (ctypes.c_int32 * 3)()
    _check(_lib.ftp_plan_map_shape(plan, boundary, out), "ftp_plan_map_shape")
    return tuple(out)


def ftp_plan_sizes(plan):
    ws, pb, npar = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    split = (ctypes.c_size_t * 4)()
    _check(_lib.ftp_plan_sizes(plan, ctypes.byref(ws), ctypes.byref(pb), ctypes.byref(npar), split), "ftp_plan_sizes")
    return {"workspace_bytes": ws.value, "wgrad_partial_bytes": pb.value, "n_params": npar.value,
            "per_stack_split": tuple(split)}


def ftp_plan_work(plan):
    u, e = ctypes.c_double(), ctypes.c_double()
    halo = (ctypes.c_double * 2)()
    _check(_lib.ftp_plan_work(plan, ctypes.byref(u), ctypes.byref(e), halo), "ftp_plan_work")
    return {"useful_macs": u.value, "executed_macs": e.value, "halo_bytes_fwd": halo[0], "halo_bytes_bwd": halo[1]}


FTP_BUF_ACT, FTP_BUF_MASK, FTP_BUF_DELTA, FTP_BUF_SIGN = 0, 1, 2, 3


def ftp_plan_buffer(plan, boundary, which):
    out = (ctypes.c_int64 * 8)()
    _check(_lib.ftp_plan_buffer(plan, boundary, which, out), "ftp_plan_buffer")
    keys = ("location", "offset", "per_stack", "slot_w", "slot_h", "channels", "rect_kind", "group")
    return dict(zip(keys, [int(v) for v in out]))


def ftp_forward(plan, x, weights, biases, workspace, y, stream=0):
    n = len(weights)
    _check(_lib.ftp_forward(plan, x, _ptr_array(weights, n), _ptr_array(biases, n), workspace, y, stream), "ftp_forward")


def ftp_forward_static(plan, x, weights, biases, y, stream=0):
    n = len(weights)
    _check(_lib.ftp_forward_static(plan, x, _ptr_array(weights, n), _ptr_array(biases, n), y, stream), "ftp_forward_static")


def ftp_backward(plan, dy, x, weights, workspace, dx, wgrad_partials, stream=0):
    n = len(weights)
    _check(_lib.ftp_backward(plan, dy, x, _ptr_array(weights, n), workspace, dx, wgrad_partials, stream), "ftp_backward")


def ftp_reduce_wgrad(plan, wgrad_partials, wgrad, stream=0):
    _check(_lib.ftp_reduce_wgrad(plan, wgrad_partials, wgrad, stream), "ftp_reduce_wgrad")


def ftp_sgd_step(plan, wgrad_partials, weights, biases, lr, wgrad=0, stream=0):
    n = len(weights)
    _check(_lib.ftp_sgd_step(plan, wgrad_partials, _ptr_array(weights, n), _ptr_array(biases, n), lr, wgrad, stream), "ftp_sgd_step")


def ftp_set_overlap(plan, enable):
    _check(_lib.ftp_set_overlap(plan, 1 if enable else 0), "ftp_set_overlap")


def ftp_profile(plan, enable):
    _check(_lib.ftp_profile(plan, 1 if enable else 0), "ftp_profile")


def ftp_profile_read(plan, capacity=256):
    out = (ftp_kernel_time * capacity)()
    n = ctypes.c_int32()
    _check(_lib.ftp_profile_read(plan, out, capacity, ctypes.byref(n)), "ftp_profile_read")
    return [{"pass": PASS_NAMES[r.pass_], "layer": r.layer, "launches": r.launches, "total_ms": r.total_ms,
             "flops_per_launch": r.flops_per_launch, "bytes_per_launch": r.bytes_per_launch,
             "kernel": r.kernel.decode(), "executed_flops_per_launch": r.executed_flops_per_launch}
            for r in out[:min(n.value, capacity)]]


def ftp_strerror(code):
    return _lib.ftp_strerror(code).decode()


def ftp_last_hip_error():
    return _lib.ftp_last_hip_error()
