"""ctypes wrapper of the CPU oracle (dpsgd_oracle.c).  TEST INFRASTRUCTURE ONLY.

May be imported by tests/, by the smoke check and by the benchmark's cpu_baseline
leg, and by nothing else.  It imports nothing from the GPU package.  Models are
the plain dict descriptions the callers pass in (duck-typed; see the keys read
in `_to_c_model`).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dpsgd_oracle.c")
_LIB = os.path.join(_HERE, "libdpsgd_oracle.so")

_KIND = {"dense": 0, "conv2d": 1, "maxpool2d": 2, "embedding": 3, "lstm_last": 4, "seq_mean": 5,
         "lstm_seq": 6, "avgpool2d": 7}
_ACT = {"none": 0, "relu": 1, "tanh": 2}


class _Layer(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("kind", "act", "d_in", "d_out", "c_in", "c_out", "kh", "kw", "stride", "pad", "vocab", "dim")]


class _Model(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("layers", C.POINTER(_Layer)), ("in_c", C.c_int), ("in_h", C.c_int),
                ("in_w", C.c_int), ("seq_len", C.c_int), ("n_classes", C.c_int)]


def build(force=False):
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        L.oracle_num_params.restype = C.c_long
        L.oracle_num_params.argtypes = [C.POINTER(_Model)]
        L.oracle_example_loss.restype = C.c_double
        L.oracle_example_loss.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p, C.c_int]
        L.oracle_example_grad.restype = C.c_double
        L.oracle_example_grad.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p, C.c_int, C.c_void_p,
                                          C.POINTER(C.c_long)]
        L.oracle_pool_near_ties.restype = C.c_long
        L.oracle_pool_near_ties.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p, C.c_int, C.c_double, C.c_long,
                                            C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_example_grad_routed.restype = C.c_double
        L.oracle_example_grad_routed.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p, C.c_int, C.c_long,
                                                 C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_philox4x32_10.restype = None
        L.oracle_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.oracle_noise.restype = None
        L.oracle_noise.argtypes = [C.c_uint64, C.c_long, C.c_void_p]
        L.oracle_dp_step.restype = C.c_int
        L.oracle_dp_step.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_double,
                                     C.c_double, C.c_uint64, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p,
                                     C.POINTER(C.c_long), C.c_void_p, C.c_void_p, C.c_int]
        L.oracle_sgd_step.restype = C.c_int
        L.oracle_sgd_step.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_double,
                                      C.c_double, C.c_uint64, C.c_double, C.c_void_p, C.c_int]
        L.oracle_sample_indices.restype = None
        L.oracle_sample_indices.argtypes = [C.c_uint64, C.c_long, C.c_int, C.c_void_p]
        L.oracle_train.restype = C.c_int
        L.oracle_train.argtypes = [C.POINTER(_Model), C.c_void_p, C.c_void_p, C.c_void_p, C.c_long, C.c_int, C.c_int,
                                   C.c_double, C.c_double, C.c_uint64, C.c_double, C.c_void_p, C.c_int]
        L.oracle_max_threads.restype = C.c_int
        _lib = L
    return _lib


def _to_c_model(m):
    layers = m["layers"]
    arr = (_Layer * len(layers))()
    for i, L in enumerate(layers):
        c = arr[i]
        c.kind = _KIND[L["kind"]]
        c.act = _ACT[L.get("act", "none")]
        if L["kind"] == "dense":
            c.d_in, c.d_out = L["d_in"], L["d_out"]
        elif L["kind"] == "conv2d":
            c.c_in, c.c_out, c.kh, c.kw, c.stride, c.pad = (L["c_in"], L["c_out"], L["kh"], L["kw"], L["stride"],
                                                            L["pad"])
        elif L["kind"] in ("maxpool2d", "avgpool2d"):
            c.kh = c.kw = L["k"]
            c.stride = L["stride"]
        elif L["kind"] == "embedding":
            c.vocab, c.dim = L["vocab"], L["dim"]
        elif L["kind"] in ("lstm_last", "lstm_seq"):
            c.d_in, c.d_out = L["d_in"], L["hidden"]
    cm = _Model()
    cm.n_layers = len(layers)
    cm.layers = C.cast(arr, C.POINTER(_Layer))
    inp = m["input"]
    if inp["kind"] == "image":
        cm.in_c, cm.in_h, cm.in_w, cm.seq_len = inp["c"], inp["h"], inp["w"], 0
    else:
        cm.in_c = cm.in_h = cm.in_w = 1
        cm.seq_len = inp["seq_len"]
    cm.n_classes = m["n_classes"]
    cm._keep = arr
    return cm


def _x_array(m, x):
    if m["input"]["kind"] == "image":
        return np.ascontiguousarray(x, dtype=np.float32)
    return np.ascontiguousarray(x, dtype=np.int32)


def num_params(m):
    cm = _to_c_model(m)
    return int(lib().oracle_num_params(C.byref(cm)))


def example_loss(m, theta64, x_i, y_i):
    """Loss of one example; theta64 is an fp64 parameter vector."""
    cm = _to_c_model(m)
    th = np.ascontiguousarray(theta64, dtype=np.float64)
    xi = _x_array(m, x_i)
    return float(lib().oracle_example_loss(C.byref(cm), th.ctypes.data, xi.ctypes.data, int(y_i)))


def example_grad(m, theta64, x_i, y_i):
    """(loss, g[P] fp64, tied pool windows) for one example."""
    cm = _to_c_model(m)
    th = np.ascontiguousarray(theta64, dtype=np.float64)
    xi = _x_array(m, x_i)
    g = np.empty(th.size, dtype=np.float64)
    ties = C.c_long(0)
    loss = lib().oracle_example_grad(C.byref(cm), th.ctypes.data, xi.ctypes.data, int(y_i), g.ctypes.data,
                                     C.byref(ties))
    return float(loss), g, int(ties.value)


def pool_near_ties(m, theta64, x_i, y_i, tau):
    """[(layer, out_idx, in_idx, gap)]: window elements of one example's max-pools that lie 0 < gap <= tau below
    their window's maximum (the elements an fp32 forward pass may legitimately pick instead), and, as
    (layer, unit, -1, |z|), the ReLU units of dense / convolution layers with 0 < |z| <= tau (whose subgradient an
    fp32 forward pass may legitimately take from the other side of zero)."""
    cm = _to_c_model(m)
    th = np.ascontiguousarray(theta64, dtype=np.float64)
    xi = _x_array(m, x_i)
    cap = 64
    while True:
        la, oi, ii = (np.empty(cap, dtype=np.int32) for _ in range(3))
        gp = np.empty(cap, dtype=np.float64)
        n = int(lib().oracle_pool_near_ties(C.byref(cm), th.ctypes.data, xi.ctypes.data, int(y_i), float(tau), cap,
                                            la.ctypes.data, oi.ctypes.data, ii.ctypes.data, gp.ctypes.data))
        if n <= cap:
            return [(int(la[k]), int(oi[k]), int(ii[k]), float(gp[k])) for k in range(n)]
        cap = n


def example_grad_routed(m, theta64, x_i, y_i, routes):
    """(loss, g[P] fp64) of one example with the max-pool windows in `routes` = [(layer, out_idx, in_idx), ...]
    sending their gradient to the named window element instead of the first maximum; a route (layer, unit, -1)
    gives that ReLU unit the subgradient of the other side of zero."""
    cm = _to_c_model(m)
    th = np.ascontiguousarray(theta64, dtype=np.float64)
    xi = _x_array(m, x_i)
    g = np.empty(th.size, dtype=np.float64)
    la = np.asarray([r[0] for r in routes], dtype=np.int32)
    oi = np.asarray([r[1] for r in routes], dtype=np.int32)
    ii = np.asarray([r[2] for r in routes], dtype=np.int32)
    loss = float(lib().oracle_example_grad_routed(C.byref(cm), th.ctypes.data, xi.ctypes.data, int(y_i), len(routes),
                                                  la.ctypes.data, oi.ctypes.data, ii.ctypes.data, g.ctypes.data))
    if loss != loss:
        raise ValueError("route outside a max-pool window, or no ReLU unit")
    return loss, g


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.empty(4, dtype=np.uint32)
    lib().oracle_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def noise(seed, n):
    """n standard normals (fp64) of the stream keyed by the 64-bit seed."""
    z = np.empty(int(n), dtype=np.float64)
    lib().oracle_noise(C.c_uint64(int(seed)), int(n), z.ctypes.data)
    return z


def dp_step(m, params, x, y, clip_c, sigma, seed, clip=True, n_threads=0):
    """One private step.  Returns dict(out fp32[P], norms fp64[B], clipped_sum fp64[P], ties, pool_margin fp64[B],
    abs_sum fp64[P] = sum_i |s_i g_i| coordinate by coordinate)."""
    cm = _to_c_model(m)
    th = np.ascontiguousarray(params, dtype=np.float32)
    xa = _x_array(m, x)
    ya = np.ascontiguousarray(y, dtype=np.int32)
    B = int(ya.shape[0])
    P = th.size
    out = np.empty(P, dtype=np.float32)
    norms = np.empty(B, dtype=np.float64)
    csum = np.empty(P, dtype=np.float64)
    ties = C.c_long(0)
    margin = np.empty(B, dtype=np.float64)
    mag = np.empty(P, dtype=np.float64)
    rc = lib().oracle_dp_step(C.byref(cm), th.ctypes.data, xa.ctypes.data, ya.ctypes.data, B, float(clip_c),
                              float(sigma), C.c_uint64(int(seed)), 1 if clip else 0, out.ctypes.data,
                              norms.ctypes.data, csum.ctypes.data, C.byref(ties), margin.ctypes.data, mag.ctypes.data,
                              int(n_threads))
    assert rc == 0
    return dict(out=out, norms=norms, clipped_sum=csum, ties=int(ties.value), pool_margin=margin, abs_sum=mag)


def sgd_step(m, params, x, y, clip_c, sigma, seed, lr, n_threads=0):
    """One private step followed by the parameter update: theta - (lr / B) * (clipped sum + sigma*C*z), fp32[P]."""
    cm = _to_c_model(m)
    th = np.ascontiguousarray(params, dtype=np.float32)
    xa = _x_array(m, x)
    ya = np.ascontiguousarray(y, dtype=np.int32)
    new = np.empty(th.size, dtype=np.float32)
    rc = lib().oracle_sgd_step(C.byref(cm), th.ctypes.data, xa.ctypes.data, ya.ctypes.data, int(ya.shape[0]),
                               float(clip_c), float(sigma), C.c_uint64(int(seed)), float(lr), new.ctypes.data,
                               int(n_threads))
    assert rc == 0
    return new


def sample_indices(seed, n, batch):
    """The minibatch of a step: `batch` indices into a dataset of n examples (int32)."""
    idx = np.empty(int(batch), dtype=np.int32)
    lib().oracle_sample_indices(C.c_uint64(int(seed) & (2**64 - 1)), int(n), int(batch), idx.ctypes.data)
    return idx


def train(m, params, data_x, data_y, steps, batch, clip_c, sigma, seed0, lr, n_threads=0):
    """`steps` iterations of draw / private step / update on the dataset (data_x, data_y); returns the parameters."""
    cm = _to_c_model(m)
    th = np.ascontiguousarray(params, dtype=np.float32)
    xa = _x_array(m, data_x)
    ya = np.ascontiguousarray(data_y, dtype=np.int32)
    new = np.empty(th.size, dtype=np.float32)
    rc = lib().oracle_train(C.byref(cm), th.ctypes.data, xa.ctypes.data, ya.ctypes.data, int(ya.shape[0]), int(steps),
                            int(batch), float(clip_c), float(sigma), C.c_uint64(int(seed0) & (2**64 - 1)), float(lr),
                            new.ctypes.data, int(n_threads))
    assert rc == 0
    return new


def max_threads():
    return int(lib().oracle_max_threads())
