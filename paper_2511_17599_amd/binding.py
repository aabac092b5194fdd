"""ctypes binding of libflce.so: the same names and arguments as include/flce.h.

Argument marshalling only.  Pointers may be given as integers (device
addresses) or as objects with a ``data_ptr()`` method (torch tensors); streams
as integers or objects with a ``cuda_stream`` attribute.  A missing library
raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libflce.so")

FLCE_OK, FLCE_ERR_BAD_ARG, FLCE_ERR_BAD_SHAPE, FLCE_ERR_WORKSPACE = 0, 1, 2, 3
FLCE_ERR_TARGET_RANGE, FLCE_ERR_UNSUPPORTED, FLCE_ERR_HIP = 4, 5, 6
FLCE_DTYPE_BF16, FLCE_DTYPE_F32 = 0, 1
FLCE_REDUCE_MEAN, FLCE_REDUCE_SUM = 0, 1
FLCE_STATIC_SCRATCH_BYTES = 16 << 20

EXPORTS = ("flce_version", "flce_tuning_reload", "flce_status_string", "flce_workspace_bytes", "flce_plan_describe", "flce_forward", "flce_backward", "flce_forward_static",
           "flce_forward_with_grads", "flce_scale", "flce_forward_rows", "flce_backward_rows", "flce_forward_partial", "flce_merge_workspace_bytes",
           "flce_merge_partials", "flce_backward_partial", "flce_last_device_status", "flce_profile_enable",
           "flce_profile_collect", "flce_probe")
PROF_CLASSES = ("fwd_tiles", "fwd_epilogue", "bwd_prep", "recompute", "contract_dW", "contract_dH", "scale")

_lib = None


def lib():
    """The loaded library (opened on first use)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_17599_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        c = ctypes
        L.flce_version.restype = c.c_char_p
        L.flce_version.argtypes = []
        L.flce_tuning_reload.restype = None
        L.flce_tuning_reload.argtypes = []
        L.flce_status_string.restype = c.c_char_p
        L.flce_status_string.argtypes = [c.c_int]
        L.flce_workspace_bytes.restype = c.c_size_t
        L.flce_workspace_bytes.argtypes = [c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_int]
        L.flce_plan_describe.restype = c.c_int
        L.flce_plan_describe.argtypes = [c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_char_p, c.c_size_t]
        L.flce_forward.restype = c.c_int
        L.flce_forward.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_int64,
                                   c.c_int, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
        L.flce_forward_static.restype = c.c_int
        L.flce_forward_static.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64,
                                          c.c_int64, c.c_int, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p,
                                          c.c_void_p, c.c_void_p]
        L.flce_backward.restype = c.c_int
        L.flce_backward.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64,
                                    c.c_int64, c.c_int, c.c_int, c.c_float, c.c_void_p, c.c_void_p, c.c_void_p,
                                    c.c_size_t, c.c_void_p]
        L.flce_forward_with_grads.restype = c.c_int
        L.flce_forward_with_grads.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64,
                                              c.c_int64, c.c_int, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p,
                                              c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
        L.flce_scale.restype = c.c_int
        L.flce_scale.argtypes = [c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_int,
                                 c.c_float, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p]
        L.flce_forward_rows.restype = c.c_int
        L.flce_forward_rows.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_int64,
                                        c.c_float, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t,
                                        c.c_void_p]
        L.flce_backward_rows.restype = c.c_int
        L.flce_backward_rows.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64,
                                         c.c_int64, c.c_int64, c.c_int64, c.c_float, c.c_int, c.c_void_p, c.c_void_p,
                                         c.c_void_p, c.c_size_t, c.c_void_p]
        L.flce_forward_partial.restype = c.c_int
        L.flce_forward_partial.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64,
                                           c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_void_p, c.c_void_p,
                                           c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
        L.flce_merge_workspace_bytes.restype = c.c_size_t
        L.flce_merge_workspace_bytes.argtypes = [c.c_int64]
        L.flce_merge_partials.restype = c.c_int
        L.flce_merge_partials.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_int, c.c_void_p, c.c_int64,
                                          c.c_int64, c.c_int64, c.c_int, c.c_void_p, c.c_void_p, c.c_void_p,
                                          c.c_size_t, c.c_void_p]
        L.flce_backward_partial.restype = c.c_int
        L.flce_backward_partial.argtypes = [c.c_void_p, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64,
                                            c.c_int64, c.c_int64, c.c_int64, c.c_int64, c.c_int, c.c_int, c.c_float,
                                            c.c_void_p, c.c_void_p, c.c_void_p, c.c_size_t, c.c_void_p]
        L.flce_last_device_status.restype = c.c_int
        L.flce_last_device_status.argtypes = [c.c_void_p, c.c_void_p, c.POINTER(c.c_int64)]
        L.flce_profile_enable.restype = c.c_int
        L.flce_profile_enable.argtypes = [c.c_int]
        L.flce_profile_collect.restype = c.c_int
        L.flce_profile_collect.argtypes = [c.POINTER(c.c_double), c.POINTER(c.c_int64)]
        L.flce_probe.restype = c.c_int
        L.flce_probe.argtypes = [c.c_int, c.c_void_p, c.c_void_p, c.c_void_p, c.c_int64, c.c_int64, c.c_int64, c.c_int,
                                 c.c_int, c.c_void_p, c.c_void_p]
        _lib = L
    return _lib


def _ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def _stream(s):
    if s is None:
        return None
    if hasattr(s, "cuda_stream"):
        return s.cuda_stream
    return int(s)


def flce_version():
    return lib().flce_version().decode()


def flce_tuning_reload():
    lib().flce_tuning_reload()


def flce_status_string(status):
    return lib().flce_status_string(int(status)).decode()


def flce_workspace_bytes(N, d, V, dt, for_backward):
    return int(lib().flce_workspace_bytes(N, d, V, dt, int(bool(for_backward))))


def flce_plan_describe(N, d, V, dt):
    buf = ctypes.create_string_buffer(512)
    n = lib().flce_plan_describe(N, d, V, dt, buf, len(buf))
    if n < 0:
        raise ValueError("unsupported shape")
    return buf.value.decode()


def flce_forward(H, W, targets, N, d, V, ignore_index, reduction, dt, loss_out, lse_out, workspace, workspace_bytes,
                 hip_stream=None):
    return lib().flce_forward(_ptr(H), _ptr(W), _ptr(targets), N, d, V, ignore_index, reduction, dt, _ptr(loss_out),
                              _ptr(lse_out), _ptr(workspace), workspace_bytes, _stream(hip_stream))


def flce_forward_static(H, W, targets, N, d, V, ignore_index, reduction, dt, loss_out, lse_out, status_out=None,
                        n_valid_out=None, hip_stream=None):
    return lib().flce_forward_static(_ptr(H), _ptr(W), _ptr(targets), N, d, V, ignore_index, reduction, dt,
                                     _ptr(loss_out), _ptr(lse_out), _ptr(status_out), _ptr(n_valid_out),
                                     _stream(hip_stream))


def flce_backward(H, W, targets, lse, N, d, V, ignore_index, reduction, dt, grad_loss, dH_out, dW_out, workspace,
                  workspace_bytes, hip_stream=None):
    return lib().flce_backward(_ptr(H), _ptr(W), _ptr(targets), _ptr(lse), N, d, V, ignore_index, reduction, dt,
                               float(grad_loss), _ptr(dH_out), _ptr(dW_out), _ptr(workspace), workspace_bytes,
                               _stream(hip_stream))


def flce_forward_with_grads(H, W, targets, N, d, V, ignore_index, reduction, dt, loss_out, lse_out, dH_partial,
                            dW_partial, workspace, workspace_bytes, hip_stream=None):
    return lib().flce_forward_with_grads(_ptr(H), _ptr(W), _ptr(targets), N, d, V, ignore_index, reduction, dt,
                                         _ptr(loss_out), _ptr(lse_out), _ptr(dH_partial), _ptr(dW_partial),
                                         _ptr(workspace), workspace_bytes, _stream(hip_stream))


def flce_scale(dH_partial, dW_partial, N, d, V, reduction, dt, grad_loss, workspace, dH_out, dW_out, hip_stream=None):
    return lib().flce_scale(_ptr(dH_partial), _ptr(dW_partial), N, d, V, reduction, dt, float(grad_loss),
                            _ptr(workspace), _ptr(dH_out), _ptr(dW_out), _stream(hip_stream))


def flce_forward_rows(H, W, targets, N, d, V, ignore_index, label_smoothing, dt, loss_rows_out, lse_out, workspace,
                      workspace_bytes, hip_stream=None):
    return lib().flce_forward_rows(_ptr(H), _ptr(W), _ptr(targets), N, d, V, ignore_index, float(label_smoothing), dt,
                                   _ptr(loss_rows_out), _ptr(lse_out), _ptr(workspace), workspace_bytes,
                                   _stream(hip_stream))


def flce_backward_rows(H, W, targets, lse, grad_rows, N, d, V, ignore_index, label_smoothing, dt, dH_out, dW_out,
                       workspace, workspace_bytes, hip_stream=None):
    return lib().flce_backward_rows(_ptr(H), _ptr(W), _ptr(targets), _ptr(lse), _ptr(grad_rows), N, d, V,
                                    ignore_index, float(label_smoothing), dt, _ptr(dH_out), _ptr(dW_out),
                                    _ptr(workspace), workspace_bytes, _stream(hip_stream))


def flce_forward_partial(H, W_slice, targets, N, d, V_slice, v_begin, V_total, ignore_index, dt, m_out, a_out, zt_out,
                         workspace, workspace_bytes, hip_stream=None):
    return lib().flce_forward_partial(_ptr(H), _ptr(W_slice), _ptr(targets), N, d, V_slice, v_begin, V_total,
                                      ignore_index, dt, _ptr(m_out), _ptr(a_out), _ptr(zt_out), _ptr(workspace),
                                      workspace_bytes, _stream(hip_stream))


def flce_merge_workspace_bytes(N):
    return int(lib().flce_merge_workspace_bytes(N))


def flce_merge_partials(m_parts, a_parts, zt_parts, n_parts, targets, N, V_total, ignore_index, reduction, loss_out,
                        lse_out, workspace, workspace_bytes, hip_stream=None):
    return lib().flce_merge_partials(_ptr(m_parts), _ptr(a_parts), _ptr(zt_parts), n_parts, _ptr(targets), N,
                                     V_total, ignore_index, reduction, _ptr(loss_out), _ptr(lse_out),
                                     _ptr(workspace), workspace_bytes, _stream(hip_stream))


def flce_backward_partial(H, W_slice, targets, lse, N, d, V_slice, v_begin, V_total, ignore_index, reduction, dt,
                          grad_loss, dH_partial_out, dW_slice_out, workspace, workspace_bytes, hip_stream=None):
    return lib().flce_backward_partial(_ptr(H), _ptr(W_slice), _ptr(targets), _ptr(lse), N, d, V_slice, v_begin,
                                       V_total, ignore_index, reduction, dt, float(grad_loss), _ptr(dH_partial_out),
                                       _ptr(dW_slice_out), _ptr(workspace), workspace_bytes, _stream(hip_stream))


def flce_last_device_status(workspace, hip_stream=None):
    """Returns (status, n_valid)."""
    nv = ctypes.c_int64(0)
    st = lib().flce_last_device_status(_ptr(workspace), _stream(hip_stream), ctypes.byref(nv))
    return st, nv.value


def flce_profile_enable(on):
    return lib().flce_profile_enable(int(bool(on)))


def flce_profile_collect():
    """Returns (status, {class: milliseconds}, {class: launches}) and clears the recording."""
    n = len(PROF_CLASSES)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_int64 * n)()
    st = lib().flce_profile_collect(ms, cnt)
    return st, dict(zip(PROF_CLASSES, list(ms))), dict(zip(PROF_CLASSES, list(cnt)))


PROBE_MODES = ("mfma_only", "loop_kc_kr", "loop_kc_kc", "data_kc_kr", "data_kc_kc", "free_run_kc_kr",
               "loop_kc_kr_softmax", "half_kc_kr", "half_kc_kr_softmax", "loop_kc_kr_cold", "mfma_16x16x32_only", "loop_kc_packed",
               "loop_kr_kr", "loop_packed_kr", "loop_kr_kc", "loop_kr_packed", "loop_packed_packed")


def flce_probe(mode, A, B, BT, a_rows, b_rows, k_elems, workgroups, tiles_per_workgroup, sink, hip_stream=None):
    return lib().flce_probe(int(mode), _ptr(A), _ptr(B), _ptr(BT), a_rows, b_rows, k_elems, workgroups,
                            tiles_per_workgroup, _ptr(sink), _stream(hip_stream))
