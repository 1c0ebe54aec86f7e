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
