"""PyTorch-CPU autograd model built from the same dict description.

Used only to pin the oracle: it is a library routine (autograd over torch's own
linear / conv2d / max_pool2d / avg_pool2d / embedding / nn.LSTM), independent of the oracle's
explicit backprop.  fp64 throughout.
"""
import numpy as np
import torch
import torch.nn.functional as F

import dp_workloads as W


def _act(name, t):
    if name == "relu":
        return torch.relu(t)
    if name == "tanh":
        return torch.tanh(t)
    return t


def split_params(m, theta):
    """theta: 1-D torch tensor (requires_grad ok) -> {(layer, name): view}."""
    out = {}
    for li, name, shp, off in W.param_tensors(m):
        n = int(np.prod(shp))
        out[(li, name)] = theta[off:off + n].reshape(shp)
    return out


def logits(m, theta, x):
    """x: torch tensor [B, ...] (float64 images or int64 tokens)."""
    p = split_params(m, theta)
    h = x
    for li, L in enumerate(m["layers"]):
        k = L["kind"]
        if k == "dense":
            h = h.reshape(h.shape[0], -1)
            h = _act(L["act"], h @ p[(li, "W")] + p[(li, "b")])
        elif k == "conv2d":
            h = _act(L["act"], F.conv2d(h, p[(li, "W")], p[(li, "b")], stride=L["stride"], padding=L["pad"]))
        elif k == "maxpool2d":
            h = F.max_pool2d(h, L["k"], L["stride"])
        elif k == "embedding":
            h = F.embedding(h, p[(li, "E")])
        elif k == "avgpool2d":
            h = F.avg_pool2d(h, L["k"], L["stride"])
        elif k in ("lstm_last", "lstm_seq"):
            H = L["hidden"]
            lstm = torch.nn.LSTM(L["d_in"], H, batch_first=True).double()
            # torch: weight_ih_l0 [4H, D] with rows ordered i, f, g, o; two biases that add.
            params = {"weight_ih_l0": p[(li, "W_ih")].t(), "weight_hh_l0": p[(li, "W_hh")].t(),
                      "bias_ih_l0": p[(li, "b")], "bias_hh_l0": torch.zeros(4 * H, dtype=torch.float64)}
            out, _ = torch.func.functional_call(lstm, params, (h,))
            h = out if k == "lstm_seq" else out[:, -1, :]
        elif k == "seq_mean":
            h = h.mean(dim=1)
    return h.reshape(h.shape[0], -1)


def to_torch_x(m, x):
    if m["input"]["kind"] == "image":
        return torch.from_numpy(np.asarray(x, dtype=np.float64))
    return torch.from_numpy(np.asarray(x, dtype=np.int64))


def per_example_grads(m, theta64, x, y):
    """[B, P] fp64 gradients of each example's own cross-entropy (batch of one at a time)."""
    xt = to_torch_x(m, x)
    yt = torch.from_numpy(np.asarray(y, dtype=np.int64))
    G = []
    for i in range(xt.shape[0]):
        th = torch.tensor(np.asarray(theta64, dtype=np.float64), requires_grad=True)
        loss = F.cross_entropy(logits(m, th, xt[i:i + 1]), yt[i:i + 1], reduction="sum")
        (g,) = torch.autograd.grad(loss, th)
        G.append(g.numpy())
    return np.stack(G)


def summed_grad(m, theta64, x, y):
    """Gradient of the batch's summed loss from one batched backward."""
    xt = to_torch_x(m, x)
    yt = torch.from_numpy(np.asarray(y, dtype=np.int64))
    th = torch.tensor(np.asarray(theta64, dtype=np.float64), requires_grad=True)
    loss = F.cross_entropy(logits(m, th, xt), yt, reduction="sum")
    (g,) = torch.autograd.grad(loss, th)
    return g.numpy()
