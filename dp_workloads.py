"""Seeded synthetic workloads for the private gradient step.

This module is the only thing the CPU oracle's tests and the HIP path share.  It
holds model *descriptions* (plain dicts), parameter counts/layout offsets and
seeded input generators.  It contains none of the method's arithmetic (no
forward pass, no gradients, no clipping, no noise).

Model description: {"input": {...}, "layers": [ {...}, ... ], "n_classes": k}

  input  {"kind": "image", "c": C, "h": H, "w": W}      fp32 x[B, C, H, W]
         {"kind": "tokens", "seq_len": T}               int32 x[B, T]
  layers {"kind": "dense", "d_in", "d_out", "act"}
         {"kind": "conv2d", "c_in", "c_out", "kh", "kw", "stride", "pad", "act"}
         {"kind": "maxpool2d", "k", "stride"}
         {"kind": "embedding", "vocab", "dim"}
         {"kind": "lstm_last", "d_in", "hidden"}
         {"kind": "seq_mean"}                           mean over the T steps of a sequence
  act    "none" | "relu" | "tanh"

Flat parameter layout (both implementations follow it): layers in order, each
weight tensor then its bias.  dense W[d_in][d_out], b[d_out]; conv
W[c_out][c_in][kh][kw], b[c_out]; embedding E[vocab][dim]; lstm W_ih[d_in][4H],
W_hh[H][4H], b[4H] with the 4H axis ordered i, f, g, o.

The first five named configurations reproduce the shapes of the paper's model
families (Section "Architectures", Appendix B) at the batch sizes, clip norm and
noise multiplier the benchmark fixes; the records of MNIST / CIFAR10 / IMDb /
Adult are not used, inputs are random with the same shapes and value ranges.
"""
from __future__ import annotations

import math
import numpy as np


def dense(d_in, d_out, act="none"):
    return {"kind": "dense", "d_in": int(d_in), "d_out": int(d_out), "act": act}


def conv2d(c_in, c_out, k, stride=1, pad=0, act="none", kw=None):
    return {"kind": "conv2d", "c_in": int(c_in), "c_out": int(c_out), "kh": int(k),
            "kw": int(k if kw is None else kw), "stride": int(stride), "pad": int(pad), "act": act}


def maxpool2d(k, stride):
    return {"kind": "maxpool2d", "k": int(k), "stride": int(stride)}


def embedding(vocab, dim):
    return {"kind": "embedding", "vocab": int(vocab), "dim": int(dim)}


def lstm_last(d_in, hidden):
    return {"kind": "lstm_last", "d_in": int(d_in), "hidden": int(hidden)}


def seq_mean():
    return {"kind": "seq_mean"}


def lstm_seq(d_in, hidden):
    """LSTM whose output is the hidden state of every time step, [T, hidden]."""
    return {"kind": "lstm_seq", "d_in": int(d_in), "hidden": int(hidden)}


def avgpool2d(k, stride):
    """Mean over k x k windows; k = stride = the whole plane is a global average pool."""
    return {"kind": "avgpool2d", "k": int(k), "stride": int(stride)}


def image_input(c, h=1, w=1):
    return {"kind": "image", "c": int(c), "h": int(h), "w": int(w)}


def token_input(seq_len):
    return {"kind": "tokens", "seq_len": int(seq_len)}


def model(inp, layers, n_classes):
    return {"input": inp, "layers": list(layers), "n_classes": int(n_classes)}


# --------------------------------------------------------------------------
# shape bookkeeping (integer arithmetic on shapes only)
# --------------------------------------------------------------------------

def conv_out(size, k, stride, pad):
    return (size + 2 * pad - k) // stride + 1


def layer_shapes(m):
    """Output shape of every layer: ("chw", C, H, W) or ("seq", T, D) or ("vec", D)."""
    inp = m["input"]
    cur = ("chw", inp["c"], inp["h"], inp["w"]) if inp["kind"] == "image" else ("tok", inp["seq_len"])
    out = []
    for L in m["layers"]:
        k = L["kind"]
        if k == "dense":
            n = cur[1] * cur[2] * cur[3] if cur[0] == "chw" else cur[1]
            assert n == L["d_in"], (cur, L)
            cur = ("vec", L["d_out"])
        elif k == "conv2d":
            assert cur[0] == "chw" and cur[1] == L["c_in"], (cur, L)
            cur = ("chw", L["c_out"], conv_out(cur[2], L["kh"], L["stride"], L["pad"]),
                   conv_out(cur[3], L["kw"], L["stride"], L["pad"]))
        elif k in ("maxpool2d", "avgpool2d"):
            assert cur[0] == "chw"
            cur = ("chw", cur[1], conv_out(cur[2], L["k"], L["stride"], 0),
                   conv_out(cur[3], L["k"], L["stride"], 0))
        elif k == "embedding":
            assert cur[0] == "tok"
            cur = ("seq", cur[1], L["dim"])
        elif k == "lstm_last":
            assert cur[0] == "seq" and cur[2] == L["d_in"], (cur, L)
            cur = ("vec", L["hidden"])
        elif k == "seq_mean":
            assert cur[0] == "seq", (cur, L)
            cur = ("vec", cur[2])
        elif k == "lstm_seq":
            assert cur[0] == "seq" and cur[2] == L["d_in"], (cur, L)
            cur = ("seq", cur[1], L["hidden"])
        else:
            raise ValueError(k)
        out.append(cur)
    assert cur in (("vec", m["n_classes"]), ("chw", m["n_classes"], 1, 1)), cur
    return out


def param_tensors(m):
    """[(layer_index, name, shape, offset)] in flat-layout order."""
    res, off = [], 0
    for li, L in enumerate(m["layers"]):
        k = L["kind"]
        if k == "dense":
            shapes = [("W", (L["d_in"], L["d_out"])), ("b", (L["d_out"],))]
        elif k == "conv2d":
            shapes = [("W", (L["c_out"], L["c_in"], L["kh"], L["kw"])), ("b", (L["c_out"],))]
        elif k == "embedding":
            shapes = [("E", (L["vocab"], L["dim"]))]
        elif k in ("lstm_last", "lstm_seq"):
            H = L["hidden"]
            shapes = [("W_ih", (L["d_in"], 4 * H)), ("W_hh", (H, 4 * H)), ("b", (4 * H,))]
        else:
            shapes = []
        for name, shp in shapes:
            res.append((li, name, shp, off))
            off += int(np.prod(shp))
    return res


def num_params(m):
    t = param_tensors(m)
    if not t:
        return 0
    li, name, shp, off = t[-1]
    return off + int(np.prod(shp))


# --------------------------------------------------------------------------
# seeded generators
# --------------------------------------------------------------------------

def init_params(m, rng, bias_scale=0.0):
    """Glorot-uniform weights; biases zero (benchmark) or U(-bias_scale, bias_scale)
    (parity tests use non-zero biases so that a dropped bias term is caught)."""
    theta = np.zeros(num_params(m), dtype=np.float32)
    for li, name, shp, off in param_tensors(m):
        n = int(np.prod(shp))
        L = m["layers"][li]
        if name == "b":
            v = rng.uniform(-bias_scale, bias_scale, size=n) if bias_scale > 0 else np.zeros(n)
        elif name == "E":
            v = rng.uniform(-0.05, 0.05, size=n)
        else:
            if L["kind"] == "conv2d":
                rf = L["kh"] * L["kw"]
                fan_in, fan_out = L["c_in"] * rf, L["c_out"] * rf
            else:
                fan_in, fan_out = shp[0], shp[1]
            lim = math.sqrt(6.0 / (fan_in + fan_out))
            v = rng.uniform(-lim, lim, size=n)
        theta[off:off + n] = v.astype(np.float32)
    return theta


def zipf_tokens(rng, vocab, exponent, shape):
    """Bounded Zipf: P(id = k-1) proportional to k^-exponent, k = 1..vocab (inverse CDF)."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-exponent)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    u = rng.random(size=shape)
    return np.minimum(np.searchsorted(cdf, u, side="left"), vocab - 1).astype(np.int32)


def make_inputs(m, batch, rng, x_dist="uniform", zipf_exponent=1.1):
    inp = m["input"]
    if inp["kind"] == "image":
        shp = (batch, inp["c"], inp["h"], inp["w"])
        if x_dist == "uniform":
            x = rng.random(size=shp).astype(np.float32)
        elif x_dist == "normal":
            x = rng.standard_normal(size=shp).astype(np.float32)
        else:
            raise ValueError(x_dist)
    else:
        vocab = m["layers"][0]["vocab"]
        x = zipf_tokens(rng, vocab, zipf_exponent, (batch, inp["seq_len"]))
    y = rng.integers(0, m["n_classes"], size=batch).astype(np.int32)
    return x, y


# --------------------------------------------------------------------------
# the five benchmark configurations
# --------------------------------------------------------------------------

def cfg1_logistic():
    return model(image_input(784), [dense(784, 10)], 10)


def cfg2_mlp():
    return model(image_input(784), [dense(784, 512, "relu"), dense(512, 10)], 10)


def cfg3_small_cnn():
    return model(image_input(1, 28, 28), [
        conv2d(1, 16, 8, stride=2, pad=3, act="tanh"), maxpool2d(2, 1),
        conv2d(16, 32, 4, stride=2, pad=0, act="tanh"), maxpool2d(2, 1),
        dense(512, 32, "tanh"), dense(32, 10)], 10)


def cfg4_cifar_cnn():
    L = []
    c_in = 3
    for width in (32, 64, 128):
        L += [conv2d(c_in, width, 3, 1, 1, "tanh"), conv2d(width, width, 3, 1, 1, "tanh"), maxpool2d(2, 2)]
        c_in = width
    L += [dense(128 * 4 * 4, 128, "tanh"), dense(128, 10)]
    return model(image_input(3, 32, 32), L, 10)


def cfg5_lstm(vocab=10000, seq_len=256, dim=100, hidden=100):
    return model(token_input(seq_len), [embedding(vocab, dim), lstm_last(dim, hidden), dense(hidden, 2)], 2)


def cfg6_embedding(vocab=10000, seq_len=256, dim=16):
    """The paper's embedding network (Appendix B): embedding, mean over the sequence, linear classifier."""
    return model(token_input(seq_len), [embedding(vocab, dim), seq_mean(), dense(dim, 2)], 2)


# The architectures exactly as Appendix B tabulates them (ReLU after every linear layer but the last,
# average pools, the LSTM returning its whole output sequence, vocabulary 10,004).  The MNIST table lists a
# third convolution and stride 1 for the second one, which cannot produce the 512 features its first fully
# connected layer takes; stride 2 and two convolutions do, and that is what cfg3 / paper_mnist_cnn use.
def paper_ffnn():
    return model(image_input(104), [dense(104, 50, "relu"), dense(50, 10)], 10)


def paper_mnist_cnn():
    return model(image_input(1, 28, 28), [
        conv2d(1, 16, 8, stride=2, pad=3, act="relu"), maxpool2d(2, 1),
        conv2d(16, 32, 4, stride=2, pad=0, act="relu"), maxpool2d(2, 1),
        dense(512, 32, "relu"), dense(32, 10)], 10)


def paper_cifar_cnn():
    L = []
    c_in = 3
    for width in (32, 64, 128):
        L += [conv2d(c_in, width, 3, 1, 1, "relu"), conv2d(width, width, 3, 1, 1, "relu"), avgpool2d(2, 2)]
        c_in = width
    L += [conv2d(128, 256, 3, 1, 1, "relu"), conv2d(256, 10, 3, 1, 1), avgpool2d(4, 4)]
    return model(image_input(3, 32, 32), L, 10)


def paper_embedding():
    return cfg6_embedding(vocab=10004)


def paper_lstm(vocab=10004, seq_len=256, dim=100, hidden=100):
    return model(token_input(seq_len), [embedding(vocab, dim), lstm_seq(dim, hidden), seq_mean(),
                                        dense(hidden, 2)], 2)


CONFIGS = {
    "cfg1_logistic": dict(build=cfg1_logistic, batch=256, x_dist="uniform"),
    "cfg2_mlp": dict(build=cfg2_mlp, batch=512, x_dist="uniform"),
    "cfg3_small_cnn": dict(build=cfg3_small_cnn, batch=1024, x_dist="uniform"),
    "cfg4_cifar_cnn": dict(build=cfg4_cifar_cnn, batch=1024, x_dist="normal"),
    "cfg5_lstm": dict(build=cfg5_lstm, batch=512, x_dist="uniform"),
    "cfg6_embedding": dict(build=cfg6_embedding, batch=512, x_dist="uniform"),
    # Appendix B architectures at the largest batch size of the paper's sweep
    "paper_ffnn": dict(build=paper_ffnn, batch=256, x_dist="uniform"),
    "paper_mnist_cnn": dict(build=paper_mnist_cnn, batch=256, x_dist="uniform"),
    "paper_cifar_cnn": dict(build=paper_cifar_cnn, batch=256, x_dist="normal"),
    "paper_embedding": dict(build=paper_embedding, batch=256, x_dist="uniform"),
    "paper_lstm": dict(build=paper_lstm, batch=256, x_dist="uniform"),
}
CLIP_C = 1.0
SIGMA = 1.1


def make_workload(name, batch=None, seed=0, bias_scale=0.0):
    """x, y, params drawn in that order from numpy default_rng(seed)."""
    c = CONFIGS[name]
    m = c["build"]()
    B = c["batch"] if batch is None else int(batch)
    rng = np.random.default_rng(seed)
    x, y = make_inputs(m, B, rng, x_dist=c["x_dist"])
    theta = init_params(m, rng, bias_scale=bias_scale)
    return dict(name=name, model=m, batch=B, x=x, y=y, params=theta, C=CLIP_C, sigma=SIGMA, seed=seed)


# small models used by parity tests: same layer kinds, sizes chosen so that a run
# spans several kernel tiles and leaves ragged tails.
def tiny_models():
    return {
        "tiny_dense": model(image_input(5), [dense(5, 4, "relu"), dense(4, 3)], 3),
        "tiny_dense_tanh": model(image_input(6), [dense(6, 5, "tanh"), dense(5, 4, "relu"), dense(4, 3)], 3),
        "tiny_conv": model(image_input(2, 5, 5), [
            conv2d(2, 3, 3, stride=2, pad=1, act="tanh"), maxpool2d(2, 1), dense(3 * 2 * 2, 3)], 3),
        "tiny_conv2": model(image_input(2, 7, 6), [
            conv2d(2, 3, 3, stride=1, pad=1, act="tanh"), conv2d(3, 4, 2, stride=1, pad=0, act="relu"),
            maxpool2d(2, 2), dense(4 * 3 * 2, 5, "tanh"), dense(5, 3)], 3),
        # 3x3 stride-1 convolutions with channel counts that exercise the LDS-staged kernels:
        # ragged channel groups (20, 40, 70), a non-square image, pad 1 (all direct kernels) and
        # pad 0 (direct forward / backward-data, generic weight gradient)
        "tiny_conv3": model(image_input(3, 9, 8), [
            conv2d(3, 20, 3, stride=1, pad=1, act="tanh"), conv2d(20, 40, 3, stride=1, pad=1, act="tanh"),
            conv2d(40, 70, 3, stride=1, pad=1, act="tanh"), conv2d(70, 24, 3, stride=1, pad=0, act="tanh"),
            maxpool2d(2, 2), dense(24 * 3 * 3, 3)], 3),
        # more than 128 output channels: the weight-gradient kernels take them in slices of 128 (here 128 + 2)
        "tiny_conv_wide": model(image_input(3, 4, 4), [
            conv2d(3, 20, 3, stride=1, pad=1, act="relu"), conv2d(20, 130, 3, stride=1, pad=1, act="tanh"),
            avgpool2d(2, 2), dense(130 * 2 * 2, 3)], 3),
        # 8x8 and 4x4 planes with enough channels that the per-example norm goes through Gram matrices; channel
        # counts that are no multiples of the 32-plane chunk
        "tiny_conv_gram": model(image_input(3, 8, 8), [
            conv2d(3, 40, 3, stride=1, pad=1, act="relu"), conv2d(40, 100, 3, stride=1, pad=1, act="tanh"),
            avgpool2d(2, 2), conv2d(100, 70, 3, stride=1, pad=1, act="tanh"), dense(70 * 4 * 4, 3)], 3),
        # 16x16 planes: the norm pass stores the per-example gradients and the clipped sum is a weighted sum of them;
        # ragged channel blocks (20 and 40 input channels) in the kernels for up to 32 and up to 64 output channels
        "tiny_conv_store": model(image_input(5, 16, 16), [
            conv2d(5, 20, 3, stride=1, pad=1, act="tanh"), conv2d(20, 40, 3, stride=1, pad=1, act="relu"),
            conv2d(40, 24, 3, stride=1, pad=1, act="tanh"), maxpool2d(2, 2), dense(24 * 8 * 8, 3)], 3),
        # a strided, non-square filter in the middle of the network (backward-data through columns + gather)
        "tiny_conv_stride": model(image_input(2, 9, 8), [
            conv2d(2, 3, 3, stride=1, pad=1, act="tanh"), conv2d(3, 5, 4, stride=2, pad=1, act="relu", kw=3),
            conv2d(5, 4, 3, stride=3, pad=2, act="tanh"), dense(4 * 2 * 2, 3)], 3),
        "tiny_lstm": model(token_input(5), [embedding(7, 3), lstm_last(3, 4), dense(4, 2)], 2),
        "tiny_emb": model(token_input(6), [embedding(7, 3), seq_mean(), dense(3, 2)], 2),
        "tiny_lstm_seq": model(token_input(5), [embedding(7, 3), lstm_seq(3, 4), seq_mean(), dense(4, 2)], 2),
        # average pools between and after convolutions; the last one is global and yields the logits
        "tiny_avgpool": model(image_input(2, 8, 8), [
            conv2d(2, 5, 3, stride=1, pad=1, act="relu"), avgpool2d(2, 2),
            conv2d(5, 3, 3, stride=1, pad=1), avgpool2d(4, 4)], 3),
        "tiny_avgpool_dense": model(image_input(2, 7, 6), [
            conv2d(2, 4, 3, stride=1, pad=1, act="tanh"), avgpool2d(3, 2), dense(4 * 3 * 2, 3)], 3),
    }
