"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI binding."""
import math

import numpy as np


def run_gpu(m, params, x, y, C, sigma, seed, private=True, max_batch=None, want_norms=True, stepper=None):
    import torch
    from paper_2010_09063_amd import DpStep
    B = int(len(y))
    dev = torch.device("cuda:0")
    st = stepper if stepper is not None else DpStep(m, max_batch or max(B, 1))
    P = st.num_params
    tp = torch.from_numpy(np.ascontiguousarray(params, dtype=np.float32)).to(dev)
    xdt = np.float32 if m["input"]["kind"] == "image" else np.int32
    tx = torch.from_numpy(np.ascontiguousarray(x, dtype=xdt)).to(dev) if B > 0 else None
    ty = torch.from_numpy(np.ascontiguousarray(y, dtype=np.int32)).to(dev) if B > 0 else None
    out = torch.full((P,), float("nan"), dtype=torch.float32, device=dev)
    norms = None
    if private:
        st.dp_step(tp, tx, ty, B, C, sigma, seed, out)
        if want_norms and B > 0:
            tn = torch.empty(B, dtype=torch.float32, device=dev)
            st.dp_step_last_norms(tn)
            torch.cuda.synchronize()
            norms = tn.cpu().numpy()
    else:
        st.dp_step_nonprivate(tp, tx, ty, B, out)
    torch.cuda.synchronize()
    res = out.cpu().numpy()
    if stepper is None:
        st.dp_step_free()
    return res, norms


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


POOL_MARGIN = 1e-5


def clear_pool_examples(m, params, x, y, oracle_step, tau=POOL_MARGIN):
    """Max-pool routes a window's gradient to its maximum; the kernel decides that in fp32,
    the oracle in fp64.  Where the two largest values of a window differ by rounding-level
    amounts either choice is a valid (sub)gradient and the two sides may legitimately differ.
    Parity is therefore checked on examples all of whose windows have a clear maximum (gap
    > tau in the oracle's forward pass): the others are replaced by clear ones (cycled), so
    the batch keeps its size.  Returns (x, y, number of examples replaced)."""
    if not any(L["kind"] == "maxpool2d" for L in m["layers"]) or len(y) == 0:
        return x, y, 0
    mg = oracle_step(m, params, x, y, 1.0, 0.0, 0, clip=False)["pool_margin"]
    clear = np.flatnonzero(mg > tau)
    assert clear.size > 0, "no example with a clear pool maximum"
    if clear.size == len(y):
        return x, y, 0
    idx = np.arange(len(y))
    bad = np.flatnonzero(mg <= tau)
    idx[bad] = clear[np.arange(bad.size) % clear.size]
    return x[idx], y[idx], int(bad.size)
