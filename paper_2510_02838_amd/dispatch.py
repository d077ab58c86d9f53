"""ctypes binding of the dispatcher entry points declared in include/dispatch.h (argument
marshalling only; the arithmetic and the search run in the C++ library)."""
import ctypes as C

import numpy as np

from .binding import lib

TDS_OK, TDS_LIMIT, TDS_EINVAL = 0, 1, -1
_d, _u8, _ip = C.POINTER(C.c_double), C.POINTER(C.c_ubyte), C.POINTER(C.c_int)
_SIGS = {
    "tds_reward_weights": (C.c_int, [C.c_int, C.c_int, C.c_int, _d, _u8, _d, C.c_double, C.c_double, C.c_double,
                                     C.c_double, _d]),
    "tds_comm_penalty": (C.c_int, [C.c_int, C.c_int, _d, _d, _d]),
    "tds_dispatch_solve": (C.c_int, [C.c_int, C.c_int, C.c_int, _ip, _d, _d, _u8, _ip, _d, _d, C.c_double,
                                     C.c_longlong, C.c_double, _ip, _ip, _u8, _d, _d, C.POINTER(C.c_longlong)]),
}
EXPORTS = sorted(_SIGS)
for _name, (_res, _args) in _SIGS.items():
    _f = getattr(lib, _name)
    _f.restype, _f.argtypes = _res, _args
    globals()[_name] = _f


def _dp(a):
    return a.ctypes.data_as(_d)


def reward_weights(t, feas, deadline, tau, c_on=1000.0, c_late=200.0, alpha=5.0):
    t = np.ascontiguousarray(t, np.float64)
    feas = np.ascontiguousarray(feas, np.uint8)
    dl = np.ascontiguousarray(deadline, np.float64)
    R, I, K = t.shape
    W = np.empty(R)
    st = tds_reward_weights(R, I, K, _dp(t), feas.ctypes.data_as(_u8), _dp(dl), tau, c_on, c_late, alpha, _dp(W))
    if st != TDS_OK:
        raise ValueError("tds_reward_weights: invalid arguments")
    return W


def comm_penalty(length, beta=(0.0, 1e-6, 5e-6, 6e-6)):
    l = np.ascontiguousarray(length, np.float64)
    b = np.ascontiguousarray(beta, np.float64)
    Q = np.empty((l.size, b.size))
    if tds_comm_penalty(l.size, b.size, _dp(l), _dp(b), _dp(Q)) != TDS_OK:
        raise ValueError("tds_comm_penalty: invalid arguments")
    return Q


def solve(W, Q, feas, B, t, deadline, tau, degrees=(1, 2, 4, 8), node_limit=0, gap_abs=0.0):
    """Returns dict(status, choice=[(type, degree) or None], D, objective, upper_bound, nodes)."""
    W = np.ascontiguousarray(W, np.float64)
    Q = np.ascontiguousarray(Q, np.float64)
    feas = np.ascontiguousarray(feas, np.uint8)
    t = np.ascontiguousarray(t, np.float64)
    dl = np.ascontiguousarray(deadline, np.float64)
    Bv = np.ascontiguousarray(B, np.int32)
    dg = np.ascontiguousarray(degrees, np.int32)
    R, I, K = feas.shape
    ct, cd = np.empty(R, np.int32), np.empty(R, np.int32)
    D = np.empty(R, np.uint8)
    obj, ub, nodes = C.c_double(), C.c_double(), C.c_longlong()
    st = tds_dispatch_solve(R, I, K, dg.ctypes.data_as(_ip), _dp(W), _dp(Q), feas.ctypes.data_as(_u8),
                            Bv.ctypes.data_as(_ip), _dp(t), _dp(dl), tau, node_limit, gap_abs,
                            ct.ctypes.data_as(_ip), cd.ctypes.data_as(_ip), D.ctypes.data_as(_u8),
                            C.byref(obj), C.byref(ub), C.byref(nodes))
    if st == TDS_EINVAL:
        raise ValueError("tds_dispatch_solve: invalid arguments")
    choice = [None if ct[r] < 0 else (int(ct[r]), int(cd[r])) for r in range(R)]
    return dict(status=st, choice=choice, D=D.tolist(), objective=obj.value, upper_bound=ub.value, nodes=nodes.value)
