"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI binding, and compare its
result with the oracle tensor by tensor, over the whole batch, allowing for the two decisions that fp32 and
fp64 may legitimately take differently: the arg-max of a max-pool window whose two largest values differ by
less than the forward pass's rounding error, and the ReLU subgradient of a pre-activation closer to zero than
that error."""
import itertools
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

import dp_workloads as W
from oracle import dpsgd_oracle as O

TOL = 1e-4          # relative L2 of the aggregated gradient: the whole vector, and every parameter tensor
# Per tensor the bar is TOL * ||ref_t|| + ACC * ||abs_t||, abs_t = sum_i |s_i g_i| coordinate by coordinate (from the
# oracle).  The second term is what any fp32 summation is entitled to: the terms of a tensor may cancel (the clipped
# bias gradients of a small batch with mixed labels: sum of the terms' norms 1,800 times the norm of their sum), and
# the rounding error of the terms, about 1e-7 of each, does not cancel with them.  For a tensor whose terms do not
# cancel this adds 1 % to the bar.
ACC = 1e-6
NORM_RTOL = 1e-4    # per-example norms
# Two window elements closer than TAU may be ordered differently by an fp32 forward pass (and a ReLU pre-activation
# closer than TAU to zero may land on the other side of it): the kernels' forward
# error on unit-scale pre-activations is <= 3e-7 (direct convolution) to 2e-6 (minimal-filtering form) in the worst
# case, and both elements carry it.  Every flip the tests accept is printed with its gap (the largest seen at full
# size is 1.4e-7, on the CIFAR-shaped CNN); a flip at a gap above TAU is not a candidate and fails the comparison.
TAU = 2e-6
MAX_FLIPPED_FRACTION = 0.05


def run_gpu(m, params, x, y, C, sigma, seed, private=True, max_batch=None, want_norms=True, stepper=None,
            options=None):
    import torch
    from paper_2010_09063_amd import DpStep
    B = int(len(y))
    dev = torch.device("cuda:0")
    st = stepper if stepper is not None else DpStep(m, max_batch or max(B, 1), **(options or {}))
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


def tensor_errors(m, got, ref, mag=None):
    """[(label, error / bar)] for the whole vector (bar TOL * ||ref||) and for every parameter tensor (bar
    TOL * ||ref_t|| + ACC * ||mag_t||, mag = the oracle's abs_sum)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rows = [("all", float(np.linalg.norm(got - ref)) / (TOL * max(float(np.linalg.norm(ref)), 1e-300)))]
    for li, name, shp, off in W.param_tensors(m):
        n = int(np.prod(shp))
        r = ref[off:off + n]
        bar = TOL * float(np.linalg.norm(r)) + (ACC * float(np.linalg.norm(mag[off:off + n])) if mag is not None else 0.0)
        rows.append((f"L{li}.{name}", float(np.linalg.norm(got[off:off + n] - r)) / max(bar, 1e-300)))
    return rows


def assert_parity(m, got, ref, label, mag=None):
    """Aggregated gradient: relative L2 <= TOL on the whole vector AND every parameter tensor within its bar."""
    assert np.isfinite(got).all(), label
    rows = tensor_errors(m, got, ref, mag)
    worst = max(rows[1:], key=lambda r: r[1]) if len(rows) > 1 else rows[0]
    print(f"{label}: rel_l2 {rows[0][1] * TOL:.3e}; worst tensor {worst[0]} at {worst[1]:.3f} of its bar", flush=True)
    bad = [(n, f"{e:.3f}") for n, e in rows if e > 1.0]
    assert not bad, (label, bad)


class TieAwareOracle:
    """The oracle's step over the WHOLE batch, with every valid max-pool routing of the near-tied windows and every
    valid subgradient of the ReLU units whose pre-activation is within TAU of zero.

    For each example that has a window element within TAU of its window's maximum (or such a ReLU unit), the oracle
    computes the example's gradient for every combination of those windows' candidate elements and those units' two
    subgradients (all on the CPU, from the oracle's own forward pass).  `reference` then picks, per such example, the combination that best explains
    the GPU's aggregate, and returns the oracle's sum and norms under that routing; the caller holds the GPU
    to the usual tolerances against them.  Every example is therefore checked: a clear example against its
    unique gradient, a near-tied one against the closest member of its finite set of valid gradients."""

    def __init__(self, m, theta, x, y, margin, tau=TAU, max_combos=1024):
        self.m, self.theta, self.x, self.y, self.tau = m, theta, x, y, tau
        self.cands = {}  # example -> (g0, [(routes, g, gap)])
        decides = any(L["kind"] == "maxpool2d" or (L["kind"] in ("dense", "conv2d") and L.get("act") == "relu")
                      for L in m["layers"])
        if not decides or len(y) == 0:
            return
        th64 = np.asarray(theta, dtype=np.float64)
        near = [int(i) for i in np.flatnonzero(np.asarray(margin) <= tau)]

        def work(i):
            ent = O.pool_near_ties(m, th64, x[i], y[i], tau)
            wins = {}
            for l, oi, ii, gap in ent:
                wins.setdefault((l, oi), []).append((ii, gap))
            opts = [[None] + [(l, oi, ii, gap) for ii, gap in alts] for (l, oi), alts in sorted(wins.items())]
            n_combos = math.prod(len(o) for o in opts)
            assert n_combos <= max_combos, (f"example {i}: {len(opts)} near-tied pool windows / ReLU units ({n_combos} routings): "
                                            "degenerate test input (saturated activations?)")
            g0 = O.example_grad(m, th64, x[i], y[i])[1]
            out = []
            for combo in itertools.product(*opts):
                routes = [c for c in combo if c is not None]
                if routes:
                    g = O.example_grad_routed(m, th64, x[i], y[i], [r[:3] for r in routes])[1]
                    out.append((routes, g, max(r[3] for r in routes)))
            return i, g0, out

        with ThreadPoolExecutor(8) as ex:
            for i, g0, out in ex.map(work, near):
                self.cands[i] = (g0, out)

    @property
    def n_near(self):
        return len(self.cands)

    def reference(self, ref, C, got, clip=True):
        """ref: the oracle's dp_step result at this C (first-maximum routing).  Returns (clipped_sum, norms,
        flips) under the valid routing closest to `got`; flips = [(example, largest gap among its re-routed
        windows)]."""
        csum = np.array(ref["clipped_sum"], dtype=np.float64)
        norms = np.array(ref["norms"], dtype=np.float64)
        if not self.cands:
            return csum, norms, []

        def scale(n):
            return C / n if (clip and n > C) else 1.0

        R = np.asarray(got, dtype=np.float64) - csum
        choice = {i: -1 for i in self.cands}
        deltas = {}
        for i, (g0, cl) in self.cands.items():
            n0 = float(np.linalg.norm(g0))
            deltas[i] = [scale(float(np.linalg.norm(g))) * g - scale(n0) * g0 for _, g, _ in cl]
        for _ in range(2):  # coordinate descent on ||got - (csum + sum of chosen deltas)||
            for i, dl in deltas.items():
                cur = dl[choice[i]] if choice[i] >= 0 else None
                Ri = R + cur if cur is not None else R
                best, best_score = -1, 0.0
                for a, d in enumerate(dl):
                    score = float(d @ d) - 2.0 * float(Ri @ d)
                    if score < best_score:
                        best, best_score = a, score
                if best != choice[i]:
                    R = Ri - dl[best] if best >= 0 else Ri
                    choice[i] = best
        flips = []
        for i, a in choice.items():
            if a >= 0:
                csum += deltas[i][a]
                norms[i] = float(np.linalg.norm(self.cands[i][1][a][1]))
                flips.append((i, self.cands[i][1][a][2]))
        return csum, norms, flips


def check_step(m, theta, x, y, C, ref, label, tie=None, private=True, stepper=None, options=None):
    """One GPU step against the oracle result `ref` (same C), whole batch, every tensor, every norm."""
    out, gn = run_gpu(m, theta, x, y, C if private else 1.0, 0.0, 0, private=private, stepper=stepper,
                      options=options)
    if tie is None:
        tie = TieAwareOracle(m, theta, x, y, ref["pool_margin"])
    csum, norms, flips = tie.reference(ref, C, out, clip=private)
    if tie.n_near:
        print(f"{label}: {tie.n_near} of {len(y)} examples have a pool window with a gap <= {tie.tau:g}; the GPU "
              f"routed {len(flips)} of them to the runner-up (largest gap {max([g for _, g in flips], default=0):.2e})",
              flush=True)
    assert len(flips) <= max(1, MAX_FLIPPED_FRACTION * len(y)), (label, len(flips))
    assert_parity(m, out, csum, label, ref["abs_sum"])
    if private and len(y) > 0:
        assert np.allclose(gn, norms, rtol=NORM_RTOL, atol=1e-7), label
    return out, gn, norms
