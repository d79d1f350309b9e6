"""Thin ctypes binding of libsolon (argument marshalling only; every step runs in the HIP kernels).

Function names mirror the C ABI declared in include/solon.h.  Tensors are torch CUDA tensors used
for device memory only; the stream is torch's current stream unless one is given.  There is no
CPU fallback: if the shared library is missing, loading raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsolon.so")

SOLON_OK, SOLON_E_INVAL, SOLON_E_BOUND, SOLON_E_POINTS, SOLON_E_DECODE, SOLON_E_NUMERIC, SOLON_E_HIP = 0, -1, -2, -3, -4, -5, -6
SOLON_F32, SOLON_BF16 = 0, 1
SOLON_Q_GROUPS, SOLON_Q_REDUNDANCY, SOLON_Q_MESSAGE_LEN, SOLON_Q_MAX_GROUP, SOLON_Q_WORKSPACE, SOLON_Q_HAS_DEVICE = range(6)
SOLON_Q_LAST_REDO, SOLON_Q_LIMIT_GROUP, SOLON_Q_LIMIT_M, SOLON_Q_LAST_ONE_PASS = 6, 7, 8, 9

EXPORTS = [
    "solon_plan_create", "solon_plan_destroy", "solon_plan_query", "solon_plan_groups", "solon_plan_points",
    "solon_default_points", "solon_encode", "solon_locate", "solon_decode", "solon_locate_decode", "solon_decode_majority",
    "solon_decode_status", "solon_locate_static", "solon_decode_update", "solon_draw_projection",
    "solon_tune",
    "solon_last_error",
]

_lib = None


class SolonError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("solon status %d: %s" % (code, msg))
        self.code = code


def lib():
    """Load libsolon.so (built in-tree by __graft_entry__.build()); fails loudly when it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libsolon.so is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    # torch ships its own HIP runtime; load it first so that libsolon.so binds to that same runtime
    # (two HIP runtimes in one process do not see the device).
    import torch  # noqa: F401
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    L.solon_plan_create.argtypes = [ctypes.POINTER(vp), i32, i32, i32, i32, i64, i32, vp, vp, vp]
    L.solon_plan_create.restype = i32
    L.solon_plan_destroy.argtypes = [vp]
    L.solon_plan_destroy.restype = None
    L.solon_plan_query.argtypes = [vp, i32, ctypes.POINTER(i64)]
    L.solon_plan_query.restype = i32
    L.solon_plan_groups.argtypes = [vp, vp]
    L.solon_plan_groups.restype = i32
    L.solon_plan_points.argtypes = [vp, vp]
    L.solon_plan_points.restype = i32
    L.solon_default_points.argtypes = [i32, vp]
    L.solon_default_points.restype = i32
    L.solon_encode.argtypes = [vp, vp, i64, vp, i64, vp]
    L.solon_encode.restype = i32
    L.solon_locate.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp]
    L.solon_locate.restype = i32
    L.solon_decode.argtypes = [vp, vp, i64, vp, i32, vp, vp]
    L.solon_decode.restype = i32
    L.solon_draw_projection.argtypes = [ctypes.c_uint64, i64, vp, vp]
    L.solon_draw_projection.restype = i32
    L.solon_decode_update.argtypes = [vp, vp, i64, vp, i32, vp, ctypes.c_float, vp]
    L.solon_decode_update.restype = i32
    L.solon_locate_decode.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp, vp]
    L.solon_locate_decode.restype = i32
    L.solon_decode_majority.argtypes = [vp, vp, i64, vp, vp, vp, vp]
    L.solon_decode_majority.restype = i32
    L.solon_locate_static.argtypes = [vp, vp, i64, vp, vp, vp, vp, vp]
    L.solon_locate_static.restype = i32
    L.solon_decode_status.argtypes = [vp, vp]
    L.solon_decode_status.restype = i32
    L.solon_tune.argtypes = [ctypes.c_char_p, i32]
    L.solon_tune.restype = i32
    L.solon_last_error.argtypes = []
    L.solon_last_error.restype = ctypes.c_char_p
    _lib = L
    return L


def _check(rc):
    if rc != SOLON_OK:
        raise SolonError(rc, lib().solon_last_error().decode())


def _stream(stream):
    if stream is not None:
        return ctypes.c_void_p(int(stream))
    import torch
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _np_ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


def solon_default_points(r_g):
    out = np.empty(r_g, dtype=np.float32)
    _check(lib().solon_default_points(int(r_g), _np_ptr(out)))
    return out


def solon_tune(key, value):
    _check(lib().solon_tune(key.encode(), int(value)))


class Plan:
    """Owner of a solon_plan handle."""

    def __init__(self, P, s, m, d, B=None, dtype=SOLON_F32, group_of_node=None, group_of_batch=None, w=None):
        self.P, self.s, self.m, self.d, self.B, self.dtype = P, s, m, d, (P if B is None else B), dtype
        gon = None if group_of_node is None else np.ascontiguousarray(group_of_node, dtype=np.int32)
        gob = None if group_of_batch is None else np.ascontiguousarray(group_of_batch, dtype=np.int32)
        wv = None if w is None else np.ascontiguousarray(w, dtype=np.float32)
        h = ctypes.c_void_p()
        self._h = None
        _check(lib().solon_plan_create(ctypes.byref(h), P, self.B, s, m, d, dtype, _np_ptr(gon), _np_ptr(gob), _np_ptr(wv)))
        self._h = h
        self.q = self.query(SOLON_Q_GROUPS)
        self.r = self.query(SOLON_Q_REDUNDANCY)
        self.d_c = self.query(SOLON_Q_MESSAGE_LEN)

    def query(self, what):
        v = ctypes.c_int64()
        _check(lib().solon_plan_query(self._h, what, ctypes.byref(v)))
        return int(v.value)

    def groups(self):
        out = np.empty(self.P, dtype=np.int32)
        _check(lib().solon_plan_groups(self._h, _np_ptr(out)))
        return out

    def points(self):
        out = np.empty(self.P, dtype=np.float32)
        _check(lib().solon_plan_points(self._h, _np_ptr(out)))
        return out

    def close(self):
        if self._h is not None:
            lib().solon_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _dev_ptr(t):
    return ctypes.c_void_p(t.data_ptr())


def solon_encode(plan, G, Z, stream=None):
    """G: [B, d] CUDA tensor (fp32 or bf16), Z: [P, d_c] fp32 CUDA tensor (written)."""
    assert G.is_cuda and Z.is_cuda and G.stride(1) == 1 and Z.stride(1) == 1
    _check(lib().solon_encode(plan._h, _dev_ptr(G), G.stride(0), _dev_ptr(Z), Z.stride(0), _stream(stream)))


def solon_locate(plan, R, f, want_host=True, want_rho=False, stream=None):
    """Returns (sorted list of located node indices, rho or None); with want_host=False returns (None, None)
    and leaves the result on the device for solon_decode."""
    assert R.is_cuda and f.is_cuda and R.stride(1) == 1 and f.is_contiguous()
    if not want_host and not want_rho:
        _check(lib().solon_locate(plan._h, _dev_ptr(R), R.stride(0), _dev_ptr(f), None, None, None, _stream(stream)))
        return None, None
    idx = np.full(max(1, plan.q * plan.s), -1, dtype=np.int32)
    n = ctypes.c_int32(0)
    rho = np.empty(plan.P, dtype=np.float64) if want_rho else None
    rc = lib().solon_locate(plan._h, _dev_ptr(R), R.stride(0), _dev_ptr(f), _np_ptr(idx), ctypes.byref(n), _np_ptr(rho),
                            _stream(stream))
    _check(rc)
    return idx[: n.value].tolist(), rho


def solon_decode(plan, R, u, byz=None, stream=None):
    """u: [d] fp32 CUDA tensor (written).  byz=None uses the device-side result of the preceding solon_locate."""
    assert R.is_cuda and u.is_cuda and R.stride(1) == 1 and u.is_contiguous()
    if byz is None:
        _check(lib().solon_decode(plan._h, _dev_ptr(R), R.stride(0), None, -1, _dev_ptr(u), _stream(stream)))
    else:
        idx = np.ascontiguousarray(byz, dtype=np.int32)
        _check(lib().solon_decode(plan._h, _dev_ptr(R), R.stride(0), _np_ptr(idx), len(idx), _dev_ptr(u), _stream(stream)))


def solon_draw_projection(seed, f, stream=None):
    """Fills the fp32 CUDA tensor f with the projection vector of this seed (1 + standard normal, counter-based)."""
    assert f.is_cuda and f.is_contiguous()
    _check(lib().solon_draw_projection(ctypes.c_uint64(int(seed) & (2 ** 64 - 1)), f.numel(), _dev_ptr(f), _stream(stream)))


def solon_decode_update(plan, R, params, step, byz=None, stream=None):
    """params: [d] fp32 CUDA tensor, updated in place: params -= step * (decoded aggregate).  byz as for solon_decode."""
    assert R.is_cuda and params.is_cuda and R.stride(1) == 1 and params.is_contiguous()
    if byz is None:
        _check(lib().solon_decode_update(plan._h, _dev_ptr(R), R.stride(0), None, -1, _dev_ptr(params), float(step), _stream(stream)))
    else:
        idx = np.ascontiguousarray(byz, dtype=np.int32)
        _check(lib().solon_decode_update(plan._h, _dev_ptr(R), R.stride(0), _np_ptr(idx), len(idx), _dev_ptr(params), float(step),
                                         _stream(stream)))


def solon_locate_decode(plan, R, f, u, want_host=True, want_rho=False, stream=None):
    """solon_locate + solon_decode in one pass over R.  Returns (located list or None, rho or None)."""
    assert R.is_cuda and f.is_cuda and u.is_cuda and R.stride(1) == 1 and f.is_contiguous() and u.is_contiguous()
    if not want_host and not want_rho:
        _check(lib().solon_locate_decode(plan._h, _dev_ptr(R), R.stride(0), _dev_ptr(f), _dev_ptr(u), None, None, None, _stream(stream)))
        return None, None
    idx = np.full(max(1, plan.q * plan.s), -1, dtype=np.int32)
    n = ctypes.c_int32(0)
    rho = np.empty(plan.P, dtype=np.float64) if want_rho else None
    _check(lib().solon_locate_decode(plan._h, _dev_ptr(R), R.stride(0), _dev_ptr(f), _dev_ptr(u), _np_ptr(idx), ctypes.byref(n),
                                     _np_ptr(rho), _stream(stream)))
    return idx[: n.value].tolist(), rho


def solon_decode_majority(plan, R, u, want_host=True, stream=None):
    """m = 1 only.  Returns the sorted list of nodes that differ from their group's majority (None if want_host=False)."""
    assert R.is_cuda and u.is_cuda and R.stride(1) == 1 and u.is_contiguous()
    if not want_host:
        _check(lib().solon_decode_majority(plan._h, _dev_ptr(R), R.stride(0), _dev_ptr(u), None, None, _stream(stream)))
        return None
    idx = np.full(plan.P, -1, dtype=np.int32)
    n = ctypes.c_int32(0)
    _check(lib().solon_decode_majority(plan._h, _dev_ptr(R), R.stride(0), _dev_ptr(u), _np_ptr(idx), ctypes.byref(n), _stream(stream)))
    return idx[: n.value].tolist()


def solon_locate_static(plan, R, f, located, status, rho=None, stream=None):
    """The allocation-free locate: located int32[P], status int32[q] and (optional) rho float64[P] are CUDA tensors (written)."""
    assert R.is_cuda and f.is_cuda and located.is_cuda and status.is_cuda and R.stride(1) == 1 and f.is_contiguous()
    assert located.is_contiguous() and status.is_contiguous() and (rho is None or (rho.is_cuda and rho.is_contiguous()))
    _check(lib().solon_locate_static(plan._h, _dev_ptr(R), R.stride(0), _dev_ptr(f), _dev_ptr(located), _dev_ptr(status),
                                     _dev_ptr(rho) if rho is not None else None, _stream(stream)))


def solon_decode_status(plan, stream=None):
    return lib().solon_decode_status(plan._h, _stream(stream))
