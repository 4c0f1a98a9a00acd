"""ctypes binding of the C ABI in include/monet.h and include/monet_kernels.h.

Argument marshalling only: every step of the path runs inside libmonet.so.  There is no
fallback: if the library is missing, loading raises.
"""
import ctypes as C
import os

import numpy as np

ALLOC, FREE, RUN_FWD, RUN_RECOMPUTE, RUN_BWD, SAVE, ALIAS = range(7)

EVENT_DTYPE = np.dtype([("kind", "<i4"), ("stage", "<i4"), ("node", "<i4"), ("impl", "<i4"), ("aux", "<i4"),
                        ("reserved", "<i4"), ("bytes", "<i8"), ("live_after", "<i8")])

_LIB = None


class LaunchInfo(C.Structure):
    _fields_ = [("kind", C.c_int32), ("id", C.c_int32), ("impl", C.c_int32), ("flags", C.c_uint32),
                ("flops", C.c_double), ("bytes", C.c_double), ("issued_flops", C.c_double), ("label", C.c_char * 32)]


class MonetError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"monet error {code}: {msg}")
        self.code = code


def library_path():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmonet.so")


def load_library():
    global _LIB
    if _LIB is not None:
        return _LIB
    # PyTorch ships its own HIP runtime; it has to be the one already in the process when
    # libmonet.so resolves its HIP symbols, or kernels and device memory end up in two runtimes.
    import torch  # noqa: F401
    path = library_path()
    if not os.path.exists(path):
        raise FileNotFoundError(f"{path} is not built: run `python -m paper_2010_14501_amd.build`")
    lib = C.CDLL(path)
    vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int, C.c_size_t
    lib.monet_last_error.restype = C.c_char_p
    lib.monet_plan_load.argtypes = [C.c_char_p, sz, C.c_char_p, sz, C.POINTER(vp)]
    lib.monet_plan_load.restype = i32
    for name in ("monet_plan_exact_peak", "monet_plan_predicted_peak", "monet_plan_predicted_peak_tight", "monet_plan_arena_bytes",
                 "monet_plan_persistent_bytes"):
        getattr(lib, name).argtypes = [vp]
        getattr(lib, name).restype = i64
    for name in ("monet_plan_num_params", "monet_plan_num_inputs"):
        getattr(lib, name).argtypes = [vp]
        getattr(lib, name).restype = i32
    lib.monet_plan_bind_arena.argtypes = [vp, vp, sz]
    lib.monet_plan_bind_arena.restype = i32
    lib.monet_step.argtypes = [vp, vp, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp), vp]
    lib.monet_step.restype = i64
    lib.monet_plan_trace.argtypes = [vp, C.POINTER(vp), C.POINTER(sz)]
    lib.monet_plan_trace.restype = i32
    lib.monet_plan_set_poison.argtypes = [vp, i32]
    lib.monet_plan_set_poison.restype = i32
    lib.monet_plan_set_stop_after.argtypes = [vp, i64]
    lib.monet_plan_set_stop_after.restype = i32
    lib.monet_plan_tensor_offset.argtypes = [vp, sz, i32, i32]
    lib.monet_plan_tensor_offset.restype = i64
    lib.monet_plan_bn_stats_offset.argtypes = [vp, i32]
    lib.monet_plan_bn_stats_offset.restype = i64
    lib.monet_plan_num_launches.argtypes = [vp]
    lib.monet_plan_num_launches.restype = i32
    lib.monet_plan_launch_info.argtypes = [vp, sz, C.POINTER(LaunchInfo)]
    lib.monet_plan_launch_info.restype = i32
    lib.monet_plan_set_fusion.argtypes = [vp, i32]
    lib.monet_plan_set_fusion.restype = i32
    lib.monet_plan_set_timing.argtypes = [vp, i32]
    lib.monet_plan_set_timing.restype = i32
    lib.monet_plan_read_timing.argtypes = [vp, C.POINTER(C.c_float), sz]
    lib.monet_plan_read_timing.restype = i32
    lib.monet_free.argtypes = [vp]
    lib.monet_free.restype = None
    f = C.c_float
    lib.monet_conv_fwd.argtypes = [vp, vp, vp, vp] + [i32] * 10 + [vp, sz]
    lib.monet_conv_fwd_bn_stats.argtypes = [vp, vp, vp, vp] + [i32] * 9 + [vp, sz, vp, f, vp, sz]
    lib.monet_conv_fwd_bn_apply.argtypes = [vp, vp, vp, vp] + [i32] * 10 + [vp, sz, vp, vp, vp]
    lib.monet_conv_fwd_bn_apply.restype = i32
    lib.monet_conv_fwd_bn_relu.argtypes = [vp, vp, vp, vp] + [i32] * 10 + [vp, sz, vp, vp, vp, i32, vp, vp]
    lib.monet_conv_fwd_bn_relu.restype = i32
    lib.monet_conv_winograd.argtypes = [vp, vp, vp, vp] + [i32] * 8 + [vp, sz]
    lib.monet_conv_winograd_fused.argtypes = [vp, vp, vp, vp] + [i32] * 7 + [vp, sz]
    lib.monet_conv_winograd_fused.restype = i32
    lib.monet_conv_winograd_fused_workspace_bytes.argtypes = [i32] * 6
    lib.monet_conv_winograd_fused_workspace_bytes.restype = i64
    lib.monet_conv_winograd_wgrad.argtypes = [vp, vp, vp, vp] + [i32] * 6 + [vp, sz]
    lib.monet_conv_im2col_fwd.argtypes = [vp, vp, vp, vp] + [i32] * 10 + [vp, sz]
    lib.monet_conv_im2col_fwd.restype = i32
    lib.monet_conv_im2col_wgrad.argtypes = [vp, vp, vp, vp] + [i32] * 9 + [vp, sz]
    lib.monet_conv_im2col_wgrad.restype = i32
    lib.monet_conv_stem_fwd.argtypes = [vp, vp, vp, vp] + [i32] * 8
    lib.monet_conv_stem_fwd.restype = i32
    lib.monet_conv_stem_wgrad.argtypes = [vp, vp, vp, vp] + [i32] * 9 + [vp, sz]
    lib.monet_conv_stem_wgrad.restype = i32
    lib.monet_conv_pointwise_wgrad.argtypes = [vp, vp, vp, vp] + [i32] * 6 + [vp, sz]
    lib.monet_conv_pointwise_wgrad.restype = i32
    lib.monet_conv_im2col_workspace_bytes.argtypes = [i32] * 10
    lib.monet_conv_im2col_workspace_bytes.restype = i64
    lib.monet_conv_winograd_wgrad_workspace_bytes.argtypes = [i32] * 6
    lib.monet_conv_winograd_wgrad_workspace_bytes.restype = i64
    lib.monet_conv_winograd_workspace_bytes.argtypes = [i32] * 6
    lib.monet_conv_winograd_workspace_bytes.restype = i64
    lib.monet_conv_workspace_bytes.argtypes = [i32] * 11
    lib.monet_conv_workspace_bytes.restype = i64
    lib.monet_conv_dgrad.argtypes = [vp, vp, vp, vp] + [i32] * 11 + [vp, sz]
    lib.monet_conv_wgrad.argtypes = [vp, vp, vp, vp] + [i32] * 10 + [vp, sz]
    lib.monet_conv_reset_arrivals.argtypes = [vp]
    lib.monet_conv_reset_arrivals.restype = i32
    lib.monet_bn_stats.argtypes = [vp, vp, vp, i64, i32, f, vp, sz]
    lib.monet_bn_stats_static.argtypes = [vp, vp, vp, i64, i32, f]
    lib.monet_bn_apply.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32]
    lib.monet_bn_bwd.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, vp, i64, i32, i32, vp, sz]
    lib.monet_relu_fwd.argtypes = [vp, vp, vp, vp, i64, i32]
    lib.monet_relu_bwd.argtypes = [vp, vp, vp, i32, vp, i64, i32, i32]
    lib.monet_maxpool_fwd.argtypes = [vp, vp, vp, vp] + [i32] * 7
    lib.monet_maxpool_bwd.argtypes = [vp, vp, vp, vp, vp] + [i32] * 8
    lib.monet_copy.argtypes = [vp, vp, vp, i64]
    lib.monet_conv_force_tile.argtypes = [i32]
    lib.monet_conv_force_tile.restype = i32
    lib.monet_tconv_fwd.argtypes = [vp, vp, vp, vp] + [i32] * 8
    lib.monet_tconv_dgrad.argtypes = [vp, vp, vp, vp] + [i32] * 9
    lib.monet_tconv_wgrad.argtypes = [vp, vp, vp, vp] + [i32] * 9 + [vp, sz]
    lib.monet_dwconv_fwd.argtypes = [vp, vp, vp, vp] + [i32] * 8
    lib.monet_dwconv_dgrad.argtypes = [vp, vp, vp, vp] + [i32] * 9
    lib.monet_dwconv_wgrad.argtypes = [vp, vp, vp, vp] + [i32] * 8 + [vp, sz]
    lib.monet_column_copy.argtypes = [vp, vp, i64, vp, i64, i32, i64, i32]
    lib.monet_softmaxce_rows_fwd.argtypes = [vp, vp, vp, vp, i64, i32, vp, sz]
    lib.monet_softmaxce_rows_bwd.argtypes = [vp, vp, vp, vp, i64, i32, i32]
    for name in ("monet_conv_fwd", "monet_conv_dgrad", "monet_conv_wgrad", "monet_bn_stats", "monet_bn_stats_static", "monet_bn_apply", "monet_bn_bwd",
                 "monet_relu_fwd", "monet_relu_bwd", "monet_maxpool_fwd", "monet_maxpool_bwd", "monet_copy",
                 "monet_tconv_fwd", "monet_tconv_dgrad", "monet_tconv_wgrad", "monet_dwconv_fwd", "monet_dwconv_dgrad",
                 "monet_dwconv_wgrad", "monet_column_copy", "monet_softmaxce_rows_fwd", "monet_softmaxce_rows_bwd"):
        getattr(lib, name).restype = i32
    _LIB = lib
    return lib


def _check(rc):
    if rc < 0:
        raise MonetError(rc, load_library().monet_last_error().decode())
    return rc


def call(name, *args):
    """Call a per-kernel entry point; pointers are passed as ints (e.g. tensor.data_ptr())."""
    return _check(getattr(load_library(), name)(*args))


def _ptr_array(ptrs):
    arr = (C.c_void_p * len(ptrs))()
    for i, p in enumerate(ptrs):
        arr[i] = p
    return arr


class Plan:
    """A loaded (graph, schedule) pair.  Device memory is the caller's (e.g. a torch tensor)."""

    def __init__(self, graph_text, schedule_text):
        self._lib = load_library()
        self._h = C.c_void_p()
        gt, st = graph_text.encode(), schedule_text.encode()
        _check(self._lib.monet_plan_load(gt, len(gt), st, len(st), C.byref(self._h)))

    def close(self):
        if self._h:
            self._lib.monet_free(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    exact_peak = property(lambda s: _check(s._lib.monet_plan_exact_peak(s._h)))
    predicted_peak = property(lambda s: _check(s._lib.monet_plan_predicted_peak(s._h)))
    predicted_peak_tight = property(lambda s: _check(s._lib.monet_plan_predicted_peak_tight(s._h)))
    arena_bytes = property(lambda s: _check(s._lib.monet_plan_arena_bytes(s._h)))
    persistent_bytes = property(lambda s: _check(s._lib.monet_plan_persistent_bytes(s._h)))
    num_params = property(lambda s: _check(s._lib.monet_plan_num_params(s._h)))
    num_inputs = property(lambda s: _check(s._lib.monet_plan_num_inputs(s._h)))

    def trace(self):
        ev, n = C.c_void_p(), C.c_size_t()
        _check(self._lib.monet_plan_trace(self._h, C.byref(ev), C.byref(n)))
        buf = (C.c_char * (n.value * EVENT_DTYPE.itemsize)).from_address(ev.value)
        return np.frombuffer(buf, dtype=EVENT_DTYPE).copy()

    def trace_tuples(self):
        return [(int(e["kind"]), int(e["stage"]), int(e["node"]), int(e["impl"]), int(e["aux"]), int(e["bytes"]),
                 int(e["live_after"])) for e in self.trace()]

    def bind_arena(self, dev_ptr, nbytes):
        _check(self._lib.monet_plan_bind_arena(self._h, dev_ptr, nbytes))

    def set_poison(self, on):
        _check(self._lib.monet_plan_set_poison(self._h, 1 if on else 0))

    def set_stop_after(self, event_index):
        _check(self._lib.monet_plan_set_stop_after(self._h, event_index))

    def tensor_offset(self, event_index, node, is_grad=False):
        return self._lib.monet_plan_tensor_offset(self._h, event_index, node, 1 if is_grad else 0)

    def bn_stats_offset(self, node):
        return self._lib.monet_plan_bn_stats_offset(self._h, node)

    def launches(self, issued=False):
        """[(label, kind, id, impl, flops, bytes)] per operator launch, in execution order (with issued=True a seventh
        entry: the flop the kernels issue, which a Winograd implementation cuts below the algorithmic count)."""
        out = []
        for i in range(_check(self._lib.monet_plan_num_launches(self._h))):
            li = LaunchInfo()
            _check(self._lib.monet_plan_launch_info(self._h, i, C.byref(li)))
            rec = (li.label.decode(), li.kind, li.id, li.impl, li.flops, li.bytes)
            out.append(rec + (li.issued_flops,) if issued else rec)
        return out

    def set_fusion(self, on):
        _check(self._lib.monet_plan_set_fusion(self._h, 1 if on else 0))

    def set_timing(self, on):
        _check(self._lib.monet_plan_set_timing(self._h, 1 if on else 0))

    def read_timing(self):
        n = _check(self._lib.monet_plan_num_launches(self._h))
        buf = (C.c_float * n)()
        _check(self._lib.monet_plan_read_timing(self._h, buf, n))
        return np.frombuffer(buf, dtype=np.float32).copy()

    def step(self, stream, input_ptrs, weight_ptrs, grad_ptrs, loss_ptr=None):
        """Enqueue one training step; returns the peak logical live bytes."""
        return _check(self._lib.monet_step(self._h, stream, _ptr_array(input_ptrs), _ptr_array(weight_ptrs),
                                           _ptr_array(grad_ptrs), loss_ptr))
