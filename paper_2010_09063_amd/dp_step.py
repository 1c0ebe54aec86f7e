"""Thin ctypes binding of libdpstep.so: argument marshalling only.

Names mirror include/dp_step.h.  Tensors are torch CUDA tensors used purely as
device memory; every step of the path runs in the library's HIP kernels.  There
is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdpstep.so")

DP_OK, DP_EINVAL, DP_ENOMEM, DP_EHIP, DP_EUNSUPPORTED, DP_ETOOBIG = 0, -1, -2, -3, -4, -5
_KIND = {"dense": 0, "conv2d": 1, "maxpool2d": 2, "embedding": 3, "lstm_last": 4, "seq_mean": 5,
         "lstm_seq": 6, "avgpool2d": 7}
_ACT = {"none": 0, "relu": 1, "tanh": 2}

EXPORTS = ["dp_step_init", "dp_step_init_ex", "dp_step_validate", "dp_step_num_params", "dp_step_workspace_bytes", "dp_step", "dp_step_sgd", "dp_step_nonprivate",
           "dp_step_dense1_static", "dp_step_sample_indices", "dp_step_loop", "dp_step_last_norms", "dp_step_profile", "dp_step_profile_read", "dp_step_describe_plan", "dp_step_ceiling", "dp_step_strerror", "dp_step_free"]


class dp_layer_desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in ("kind", "act", "in_features", "out_features", "in_ch", "out_ch", "kh", "kw",
                                       "stride", "pad", "vocab", "embed_dim", "hidden")]


class dp_model_desc(C.Structure):
    _fields_ = [("n_layers", C.c_int), ("layers", C.POINTER(dp_layer_desc)), ("in_c", C.c_int), ("in_h", C.c_int),
                ("in_w", C.c_int), ("seq_len", C.c_int), ("n_classes", C.c_int)]


PLAN_OPTIONS = ("generic_conv", "no_minimal_filtering", "no_minimal_filtering_wgrad", "minimal_filtering_all",
                "no_pool_fusion", "no_gram", "no_stored_gradients", "no_columns", "no_specialised_waves",
                "specialised_waves_all", "conv_min_blocks", "gemm_plain_tiles", "no_fused_dense", "no_fused_cnn", "no_lstm_wgrad", "no_rows_gemm", "no_single_bucket", "no_small_gemm", "no_resident_weights", "no_side_stream", "no_first_layer_kernel")


class dp_plan_options(C.Structure):
    _fields_ = [(n, C.c_int) for n in PLAN_OPTIONS]


_lib = None


def load_library():
    """Loads libdpstep.so; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2010_09063_amd.build` "
                               "(or __graft_entry__.build()); there is no CPU fallback")
        L = C.CDLL(LIB_PATH)
        L.dp_step_init.restype = C.c_int
        L.dp_step_init.argtypes = [C.POINTER(dp_model_desc), C.c_int, C.c_void_p, C.POINTER(C.c_void_p)]
        L.dp_step_init_ex.restype = C.c_int
        L.dp_step_init_ex.argtypes = [C.POINTER(dp_model_desc), C.c_int, C.c_void_p, C.POINTER(dp_plan_options),
                                      C.POINTER(C.c_void_p)]
        L.dp_step_validate.restype = C.c_int
        L.dp_step_validate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.POINTER(C.c_int)]
        L.dp_step_num_params.restype = C.c_size_t
        L.dp_step_num_params.argtypes = [C.c_void_p]
        L.dp_step_workspace_bytes.restype = C.c_size_t
        L.dp_step_workspace_bytes.argtypes = [C.c_void_p]
        L.dp_step.restype = C.c_int
        L.dp_step.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_float,
                              C.c_uint64, C.c_void_p]
        L.dp_step_sgd.restype = C.c_int
        L.dp_step_sgd.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_float, C.c_float,
                                  C.c_uint64, C.c_float, C.c_void_p]
        L.dp_step_nonprivate.restype = C.c_int
        L.dp_step_nonprivate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.dp_step_dense1_static.restype = C.c_int
        L.dp_step_dense1_static.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_float,
                                            C.c_float, C.c_uint64, C.c_void_p, C.c_void_p, C.c_void_p]
        L.dp_step_sample_indices.restype = C.c_int
        L.dp_step_sample_indices.argtypes = [C.c_uint64, C.c_int64, C.c_int, C.c_void_p, C.c_void_p]
        L.dp_step_loop.restype = C.c_int
        L.dp_step_loop.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int, C.c_int,
                                   C.c_float, C.c_float, C.c_uint64, C.c_float]
        L.dp_step_last_norms.restype = C.c_int
        L.dp_step_last_norms.argtypes = [C.c_void_p, C.c_void_p]
        L.dp_step_profile.restype = C.c_int
        L.dp_step_profile.argtypes = [C.c_void_p, C.c_int]
        L.dp_step_profile_read.restype = C.c_int
        L.dp_step_profile_read.argtypes = [C.c_void_p, C.c_int, C.POINTER(C.c_char_p), C.POINTER(C.c_int),
                                           C.POINTER(C.c_float), C.c_int]
        L.dp_step_describe_plan.restype = C.c_int
        L.dp_step_describe_plan.argtypes = [C.c_void_p, C.c_char_p, C.c_size_t]
        L.dp_step_ceiling.restype = C.c_int
        L.dp_step_ceiling.argtypes = [C.c_int, C.c_void_p, C.POINTER(C.c_double)]
        L.dp_step_strerror.restype = C.c_char_p
        L.dp_step_strerror.argtypes = [C.c_int]
        L.dp_step_free.restype = None
        L.dp_step_free.argtypes = [C.c_void_p]
        _lib = L
    return _lib


class DpStepError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"dp_step status {code}: {load_library().dp_step_strerror(code).decode()}")


def _check(code):
    if code != DP_OK:
        raise DpStepError(code)


def model_desc(m):
    """dict description (see dp_workloads) -> (dp_model_desc, keepalive)."""
    layers = m["layers"]
    arr = (dp_layer_desc * len(layers))()
    for i, L in enumerate(layers):
        d = arr[i]
        d.kind = _KIND[L["kind"]]
        d.act = _ACT[L.get("act", "none")]
        if L["kind"] == "dense":
            d.in_features, d.out_features = L["d_in"], L["d_out"]
        elif L["kind"] == "conv2d":
            d.in_ch, d.out_ch, d.kh, d.kw, d.stride, d.pad = (L["c_in"], L["c_out"], L["kh"], L["kw"], L["stride"],
                                                              L["pad"])
        elif L["kind"] in ("maxpool2d", "avgpool2d"):
            d.kh = d.kw = L["k"]
            d.stride = L["stride"]
        elif L["kind"] == "embedding":
            d.vocab, d.embed_dim = L["vocab"], L["dim"]
        elif L["kind"] in ("lstm_last", "lstm_seq"):
            d.in_features, d.hidden = L["d_in"], L["hidden"]
    md = dp_model_desc()
    md.n_layers = len(layers)
    md.layers = C.cast(arr, C.POINTER(dp_layer_desc))
    inp = m["input"]
    if inp["kind"] == "image":
        md.in_c, md.in_h, md.in_w, md.seq_len = inp["c"], inp["h"], inp["w"], 0
    else:
        md.in_c = md.in_h = md.in_w = 1
        md.seq_len = inp["seq_len"]
    md.n_classes = m["n_classes"]
    return md, arr


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


# -- include/dp_step.h: dp_step_dense1_static (no context, no allocation)
def dp_step_dense1_static(params, x, y, batch, in_features, n_classes, C_, sigma, seed, out_grad, norms_out=None,
                          stream=None):
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(load_library().dp_step_dense1_static(_ptr(params), _ptr(x), _ptr(y), int(batch), int(in_features),
                                                int(n_classes), float(C_), float(sigma),
                                                C.c_uint64(int(seed) & (2**64 - 1)), _ptr(out_grad), _ptr(norms_out),
                                                C.c_void_p(st.cuda_stream)))


# -- dp_step_ceiling
def dp_step_ceiling(what, stream=None):
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    v = C.c_double(0.0)
    _check(load_library().dp_step_ceiling(int(what), C.c_void_p(st.cuda_stream), C.byref(v)))
    return float(v.value)


# -- dp_step_sample_indices
def dp_step_sample_indices(seed, n_examples, batch, indices, stream=None):
    import torch
    st = stream if stream is not None else torch.cuda.current_stream()
    _check(load_library().dp_step_sample_indices(C.c_uint64(int(seed) & (2**64 - 1)), int(n_examples), int(batch),
                                                 _ptr(indices), C.c_void_p(st.cuda_stream)))


class DpStep:
    """Owns one dp_ctx.  `stream` is a torch.cuda.Stream (default: the current one); keyword options are the fields
    of dp_plan_options (route switches for tests and A/B measurements)."""

    def __init__(self, m, max_batch, stream=None, **options):
        import torch
        self._lib = load_library()
        self._torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("dp_step needs a GPU (no CPU fallback)")
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        md, keep = model_desc(m)
        ctx = C.c_void_p(0)
        if options:
            opt = dp_plan_options()
            for k, v in options.items():
                if k not in PLAN_OPTIONS:
                    raise TypeError(f"unknown plan option {k!r}")
                setattr(opt, k, int(v))
            _check(self._lib.dp_step_init_ex(C.byref(md), int(max_batch), C.c_void_p(self.stream.cuda_stream),
                                             C.byref(opt), C.byref(ctx)))
        else:
            _check(self._lib.dp_step_init(C.byref(md), int(max_batch), C.c_void_p(self.stream.cuda_stream),
                                          C.byref(ctx)))
        self._ctx = ctx
        self.num_params = int(self._lib.dp_step_num_params(ctx))
        self.workspace_bytes = int(self._lib.dp_step_workspace_bytes(ctx))
        self.max_batch = int(max_batch)

    # -- include/dp_step.h: dp_step
    def dp_step(self, params, x, y, batch, C_, sigma, seed, out_grad):
        _check(self._lib.dp_step(self._ctx, _ptr(params), _ptr(x), _ptr(y), int(batch), float(C_), float(sigma),
                                 C.c_uint64(int(seed) & (2**64 - 1)), _ptr(out_grad)))

    # -- dp_step_sgd
    def dp_step_sgd(self, params, x, y, batch, C_, sigma, seed, lr, out_grad=None):
        _check(self._lib.dp_step_sgd(self._ctx, _ptr(params), _ptr(x), _ptr(y), int(batch), float(C_), float(sigma),
                                     C.c_uint64(int(seed) & (2**64 - 1)), float(lr),
                                     _ptr(out_grad) if out_grad is not None else None))

    # -- dp_step_loop
    def dp_step_loop(self, params, data_x, data_y, n_examples, steps, batch, C_, sigma, seed0, lr):
        _check(self._lib.dp_step_loop(self._ctx, _ptr(params), _ptr(data_x), _ptr(data_y), int(n_examples), int(steps),
                                      int(batch), float(C_), float(sigma), C.c_uint64(int(seed0) & (2**64 - 1)),
                                      float(lr)))

    # -- dp_step_nonprivate
    def dp_step_nonprivate(self, params, x, y, batch, out_grad):
        _check(self._lib.dp_step_nonprivate(self._ctx, _ptr(params), _ptr(x), _ptr(y), int(batch), _ptr(out_grad)))

    # -- dp_step_validate
    def dp_step_validate(self, x, y, batch):
        n = C.c_int(0)
        _check(self._lib.dp_step_validate(self._ctx, _ptr(x), _ptr(y), int(batch), C.byref(n)))
        return int(n.value)

    # -- dp_step_last_norms
    def dp_step_last_norms(self, norms_out):
        _check(self._lib.dp_step_last_norms(self._ctx, _ptr(norms_out)))

    # -- dp_step_profile / dp_step_profile_read
    def dp_step_profile(self, enable):
        _check(self._lib.dp_step_profile(self._ctx, 1 if enable else 0))

    def dp_step_profile_read(self, reset=True):
        cap = 64
        labels = (C.c_char_p * cap)()
        launches = (C.c_int * cap)()
        ms = (C.c_float * cap)()
        n = self._lib.dp_step_profile_read(self._ctx, cap, labels, launches, ms, 1 if reset else 0)
        if n < 0:
            raise DpStepError(n)
        return [(labels[i].decode(), int(launches[i]), float(ms[i])) for i in range(min(n, cap))]

    # -- dp_step_describe_plan
    def dp_step_describe_plan(self):
        buf = C.create_string_buffer(4096)
        _check(self._lib.dp_step_describe_plan(self._ctx, buf, 4096))
        plan = {}
        for item in buf.value.decode().split(";"):
            if item:
                li, rest = item.split(":")
                plan[int(li)] = dict(kv.split("=") for kv in rest.split(","))
        return plan

    # -- dp_step_free
    def dp_step_free(self):
        if self._ctx is not None and self._ctx.value:
            self._lib.dp_step_free(self._ctx)
        self._ctx = None

    def __del__(self):
        try:
            self.dp_step_free()
        except Exception:
            pass
