"""The allocation-free entry point dp_step_dense1_static against dp_step on the same one-layer model (and against
the oracle), two calls in a row on the one static scratch array, the second with a smaller input."""
import numpy as np
import pytest

import dp_workloads as W
from oracle import dpsgd_oracle as O
from tests.gpu_util import TOL, rel_l2

pytestmark = pytest.mark.gpu


def _one_call(d_in, n_classes, batch, seed, sigma):
    import torch
    from paper_2010_09063_amd import DpStep, dp_step_dense1_static
    m = W.model(W.image_input(d_in), [W.dense(d_in, n_classes)], n_classes)
    rng = np.random.default_rng(seed)
    x, y = W.make_inputs(m, batch, rng)
    theta = W.init_params(m, rng, bias_scale=0.3)
    norms_ref = O.dp_step(m, theta, x, y, 1.0, 0.0, 0)["norms"]
    Cc = float(np.median(norms_ref))
    dev = torch.device("cuda:0")
    tp, tx, ty = (torch.from_numpy(a).to(dev) for a in (theta, x.reshape(batch, -1), y))
    got = torch.full((theta.size,), float("nan"), device=dev)
    gn = torch.full((batch,), float("nan"), device=dev)
    dp_step_dense1_static(tp, tx, ty, batch, d_in, n_classes, Cc, sigma, 1234, got, gn)
    st = DpStep(m, batch)
    want = torch.empty(theta.size, device=dev)
    wn = torch.empty(batch, device=dev)
    st.dp_step(tp, tx, ty, batch, Cc, sigma, 1234, want)
    st.dp_step_last_norms(wn)
    torch.cuda.synchronize()
    st.dp_step_free()
    got, want, gn, wn = got.cpu().numpy(), want.cpu().numpy(), gn.cpu().numpy(), wn.cpu().numpy()
    ref = O.dp_step(m, theta, x, y, Cc, sigma, 1234)
    print(f"static entry d_in={d_in} classes={n_classes} B={batch}: vs dp_step {rel_l2(got, want):.2e}, "
          f"vs oracle {rel_l2(got, ref['out']):.2e}", flush=True)
    assert np.isfinite(got).all() and np.isfinite(gn).all()
    assert rel_l2(got, want) <= 1e-6 and np.allclose(gn, wn, rtol=1e-6)
    assert rel_l2(got, ref["out"]) <= TOL and np.allclose(gn, norms_ref, rtol=1e-4)


def test_static_entry_two_calls_second_smaller():
    _one_call(784, 10, 256, seed=5, sigma=0.0)   # the logistic-regression configuration
    _one_call(100, 3, 37, seed=6, sigma=1.1)     # smaller in every dimension: what the first call left must not show


def test_static_entry_rejects_what_does_not_fit():
    import torch
    from paper_2010_09063_amd import DpStepError, dp_step_dense1_static
    dev = torch.device("cuda:0")
    p = torch.zeros(2049 * 17, device=dev)
    x = torch.zeros(4 * 2048, device=dev)
    y = torch.zeros(4, dtype=torch.int32, device=dev)
    for d_in, k in ((1024, 10), (784, 17)):
        with pytest.raises(DpStepError) as e:
            dp_step_dense1_static(p, x, y, 4, d_in, k, 1.0, 0.0, 0, p)
        assert e.value.code == -5
    with pytest.raises(DpStepError) as e:
        dp_step_dense1_static(p, x, y, 4, 8, 3, -1.0, 0.0, 0, p)
    assert e.value.code == -1
    # an empty batch is pure noise
    out = torch.empty(9 * 3, device=dev)
    dp_step_dense1_static(p, None, None, 0, 8, 3, 1.0, 1.1, 7, out)
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy() - 1.1 * O.noise(7, 27)).max() <= 1e-5
