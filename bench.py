#!/usr/bin/env python3
"""Benchmark of the private gradient step on one MI355X.

A step is one dp_step call (forward, backward-data, per-example norms, clip
factors, clipped sums, Philox noise) over one synthetic batch already resident
in HBM.  Prints ONE JSON line: private examples/s for the headline workload,
the same-run non-private step time and ratio, the roofline of the dominant
kernel (timed with HIP events on the library's stream) and the CPU oracle timed
on a bounded sample of the same workload.
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import dp_workloads as W  # noqa: E402

PEAK_MFMA_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
DEFAULT_WORKLOAD = "cfg4_cifar_cnn"


# algorithmic flops per example of the private step as the survey of the method prices it (forward, backward-data,
# per-example norms, clipped sum, each in its textbook direct form; dense norms by the norm identity)
SURVEY_FLOPS_PER_EXAMPLE = {"cfg1_logistic": 31.4e3 + 1.6e3, "cfg2_mlp": 1.64e6, "cfg3_small_cnn": 2.89e6,
                            "cfg4_cifar_cnn": 297e6, "cfg5_lstm": 164e6}
MF = 16.0 / 36.0  # multiplies of the minimal-filtering form per multiply of the direct form


def label_work(m, B, plan=None):
    """Work per kernel label for one step: {label: (algorithmic flops, algorithmic bytes, executed flops)}.
    Algorithmic flops: 2*M*N*K of the operation the route computes (a Gram-matrix norm is priced as Gram matrices, a
    weighted sum of stored gradients as a weighted sum; a convolution in minimal-filtering form is priced as the
    direct form it equals).  Executed flops: the multiplies the route really issues (minimal-filtering form: 16/36 of
    the direct form).  Bytes: compulsory HBM traffic (operands read once, result written once).  `plan` is the
    library's own description of its routes (dp_step_describe_plan)."""
    plan = plan or {}
    shapes = W.layer_shapes(m)
    inp = m["input"]
    cur = ("chw", inp["c"], inp["h"], inp["w"]) if inp["kind"] == "image" else ("tok", inp["seq_len"])
    out = {}

    def add(label, flops, nbytes, executed=None, layer=None):
        ex = flops if executed is None else executed
        for key in (label, f"{label}#{li if layer is None else layer}"):   # per kernel kind and per (kind, layer)
            f, b, e = out.get(key, (0.0, 0.0, 0.0))
            out[key] = (f + flops, b + nbytes, e + ex)

    for li, L in enumerate(m["layers"]):
        o = shapes[li]
        k = L["kind"]
        r = plan.get(li, {})
        if r.get("fwd") == "fused-net":
            # the whole network in one launch (cnn_small_fused): forward, backward-data and ONE weight-gradient
            # contraction per layer (the example's gradient serves the norm and, scaled, the clipped sum)
            if k == "dense":
                fl, pc = 2.0 * B * L["d_in"] * L["d_out"], L["d_in"] * L["d_out"] + L["d_out"]
            else:
                fl = 2.0 * B * o[1] * cur[1] * L["kh"] * L["kw"] * o[2] * o[3]
                pc = o[1] * cur[1] * L["kh"] * L["kw"] + o[1]
            nb = 4.0 * (B * int(np.prod(cur[1:])) if li == 0 else 0) + 4.0 * pc * (1 + min(B, 256))
            for key in ("cnn_small_fused",):
                f, b, e = out.get(key, (0.0, 0.0, 0.0))
                out[key] = (f + fl * (3 if li > 0 else 2), b + nb, e + fl * (3 if li > 0 else 2))
            cur = o
            continue
        if k == "dense":
            di, do = L["d_in"], L["d_out"]
            fl = 2.0 * B * di * do
            if r.get("fwd") == "fused" and li == 0:   # one-layer model: forward, loss, norm, clip factor and partial sums in one launch
                add("dense1_fused", 2 * fl + 2.0 * B * (di + do), 4.0 * (B * di + di * do + (B // 4) * (di + 1) * do))
            elif r.get("fwd") == "fused" and r.get("sum") == "joint":
                # logit layer of a two-layer model: forward, backward-data and both norms in one launch; its clipped
                # sum rides in the hidden layer's launch (s * delta in rows of 16 floats)
                add("dense2_mid", 2 * fl + 2.0 * B * (di + do), 4.0 * (3 * B * di + di * do + 16 * B))
                add("dense_clipped_sum", fl, 4.0 * (B * di + 16 * B + di * do), layer=li - 1)
            elif r.get("fwd") == "fused":  # the same with the logit layer's partial clipped sums written by that launch
                add("dense2_mid", 3 * fl + 2.0 * B * (di + do), 4.0 * (3 * B * di + di * do + (B // 4) * (di + 1) * do))
            elif r.get("norm") == "fused":  # hidden layer of the same model: its two batch-wide contractions remain
                add("dense_fwd", fl, 4.0 * (B * di + di * do + B * do))
                add("dense_clipped_sum", fl, 4.0 * (B * di + B * do + di * do))
            elif r.get("fwd") == "head":  # logit layer of a deeper network: forward, backward-data and both dense norms in one launch
                add("dense2_head", 2 * fl + 2.0 * B * (di + do), 4.0 * (3 * B * di + di * do + B * do))
                if r.get("sum") == "joint":  # its clipped sum rides in the hidden layer's launch (delta in rows of 16 floats)
                    add("dense_clipped_sum", fl, 4.0 * (B * di + 16 * B + di * do), layer=li - 1)
                else:
                    add("dense_clipped_sum", fl, 4.0 * (B * di + B * do + di * do))
            else:
                add("dense_fwd", fl, 4.0 * (B * di + di * do + B * do))
                if li > 0:
                    add("dense_bwd_data", fl, 4.0 * (B * do + di * do + 2 * B * di))
                if r.get("norm") == "head":  # hidden layer of that head: its norm (one pass over its input) is taken by the same launch
                    add("dense2_head", 2.0 * B * (di + do), 4.0 * B * di)
                else:
                    add("dense_norm", 2.0 * B * (di + do), 4.0 * B * (di + do))
                add("dense_clipped_sum", fl, 4.0 * (B * di + B * do + di * do))
        elif k == "conv2d":
            C_, H_, W_ = cur[1], cur[2], cur[3]
            D_, OH, OW = o[1], o[2], o[3]
            ckk = C_ * L["kh"] * L["kw"]
            fl = 2.0 * B * D_ * ckk * OH * OW
            xin, xout, wts = B * C_ * H_ * W_, B * D_ * OH * OW, D_ * ckk
            mf = lambda route: MF if route.startswith("mf") else 1.0
            fwd_route = r.get("fwd", "")
            if fwd_route.endswith("+maxpool"):    # pooled plane + arg-max byte instead of the plane before the pool
                out_bytes = 5.0 * (xout // 4)
            elif fwd_route.endswith("+avgpool"):  # both planes
                out_bytes = 4.0 * (xout + xout // 4)
            else:
                out_bytes = 4.0 * xout
            add("conv_fwd", fl, 4.0 * (xin + wts) + out_bytes, fl * mf(fwd_route))
            if li > 0:
                add("conv_bwd_data", fl, 4.0 * (xout + wts + 2 * xin), fl * mf(r.get("bwd", "")))
            Pp = OH * OW
            norm, sm = r.get("norm", "direct"), r.get("sum", "direct")
            store = norm.endswith("+store")
            nfl = 2.0 * B * Pp * Pp * (ckk + D_) if norm == "gram" else fl
            add("conv_wgrad_norm", nfl, 4.0 * (xin + xout + (B * (wts + D_) if store else 0)), nfl * mf(norm))
            if sm == "weighted":
                add("conv_weighted_sum", 2.0 * B * (wts + D_), 4.0 * (B * (wts + D_) + wts + D_))
            else:
                add("conv_clipped_sum", fl, 4.0 * (xin + xout + wts), fl * mf(sm))
        elif k == "maxpool2d":
            n_in, n_out = B * cur[1] * cur[2] * cur[3], B * o[1] * o[2] * o[3]
            add("maxpool_fwd", 0.0, 4.0 * n_in + 5.0 * n_out)
            add("maxpool_bwd", 0.0, 4.0 * n_in + 9.0 * n_out)  # writes the plane; reads pooled gradient, pooled plane, arg-max byte
        elif k == "avgpool2d":
            n_in, n_out = B * cur[1] * cur[2] * cur[3], B * o[1] * o[2] * o[3]
            add("avgpool_fwd", 1.0 * n_in, 4.0 * (n_in + n_out))
            add("avgpool_bwd", 1.0 * n_in, 4.0 * (2 * n_in + n_out))
        elif k == "embedding":
            T, D_ = inp["seq_len"], L["dim"]
            add("emb_gather", 0.0, 4.0 * B * T * (2 * D_ + 1))
            add("emb_norm", 2.0 * B * T * D_, 4.0 * B * T * (D_ + 1))
            add("emb_bucket", 0.0, 4.0 * (4 * B * T + 4 * L["vocab"]))  # counting sort: tokens read 3x, list written
            add("emb_scatter", 2.0 * B * T * D_, 4.0 * (B * T * (D_ + 1) + L["vocab"] * D_))
        elif k == "seq_mean":
            T, D_ = cur[1], cur[2]
            add("seq_mean_fwd", 1.0 * B * T * D_, 4.0 * B * (T * D_ + D_))
            add("seq_mean_bwd", 1.0 * B * T * D_, 4.0 * B * (T * D_ + D_))
        elif k in ("lstm_last", "lstm_seq"):
            T, Din, H = cur[1], L["d_in"], L["hidden"]
            G = 4 * H
            add("lstm_xproj", 2.0 * B * T * Din * G, 4.0 * (B * T * G + Din * G))
            add("lstm_fwd", 2.0 * B * T * H * G, 4.0 * B * T * (2 * G + 2 * H))
            add("lstm_bwd", 2.0 * B * T * H * G, 4.0 * B * T * (2 * G + H))
            pc = (Din + H + 1) * G
            store = r.get("sum", "weighted" if T >= 128 else "generic") == "weighted"
            add("lstm_wgrad_norm", 2.0 * B * T * (Din + H) * G, 4.0 * (B * T * (G + H + Din) + (B * pc if store else 0)))
            add("lstm_dx", 2.0 * B * T * Din * G, 4.0 * B * T * (G + Din))
            if store:
                add("lstm_weighted_sum", 2.0 * B * pc, 4.0 * (B * pc + pc))
            else:
                add("lstm_clipped_sum", 2.0 * B * T * (Din + H) * G, 4.0 * B * T * (G + H + Din))
        cur = o
    P = W.num_params(m)
    out["finalize_noise"] = (0.0, 8.0 * P, 0.0)
    return out


def step_flops(m, B, plan=None, executed=False):
    """Flops of one private step summed over its kernels: of the routes taken (algorithmic), or as issued."""
    w = label_work(m, B, plan)
    return sum((e if executed else f) for lab, (f, _, e) in w.items() if "#" not in lab)


def time_steps(fn, steps, warmup):
    import torch
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(warmup + i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def per_call_ms(fn, stream, calls):
    """Each call timed on its own with a pair of events on the library's stream: (median, p10, p90) in ms."""
    import torch
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(calls)]
    for i, (e0, e1) in enumerate(ev):
        e0.record(stream)
        fn(i)
        e1.record(stream)
    torch.cuda.synchronize()
    t = sorted(e0.elapsed_time(e1) for e0, e1 in ev)
    pick = lambda q: t[min(len(t) - 1, int(q * len(t)))]
    return pick(0.5), pick(0.1), pick(0.9)


def run_workload(name, steps, warmup, profile, batch=None, loop=True):
    import torch
    from paper_2010_09063_amd import DpStep
    wl = W.make_workload(name, batch=batch, seed=0)
    m, B = wl["model"], wl["batch"]
    dev = torch.device("cuda:0")
    st = DpStep(m, B)
    plan = st.dp_step_describe_plan()
    tp = torch.from_numpy(wl["params"]).to(dev)
    tx = torch.from_numpy(wl["x"]).to(dev)
    ty = torch.from_numpy(wl["y"]).to(dev)
    out = torch.empty(st.num_params, dtype=torch.float32, device=dev)
    Cc, sigma = wl["C"], wl["sigma"]

    ms_priv = time_steps(lambda i: st.dp_step(tp, tx, ty, B, Cc, sigma, i, out), steps, warmup)
    assert bool(torch.isfinite(out).all()), "non-finite gradient"
    ms_np = time_steps(lambda i: st.dp_step_nonprivate(tp, tx, ty, B, out), steps, warmup)
    res = dict(workload=name, batch=B, params=st.num_params, ms_private=ms_priv, ms_nonprivate=ms_np,
               examples_per_s=B / (ms_priv * 1e-3), ratio=ms_priv / ms_np, workspace_mb=st.workspace_bytes / 2**20,
               tflops=step_flops(m, B, plan) / (ms_priv * 1e-3) / 1e12,
               tflops_executed=step_flops(m, B, plan, executed=True) / (ms_priv * 1e-3) / 1e12)
    if name in SURVEY_FLOPS_PER_EXAMPLE:
        res["tflops_survey_accounting"] = SURVEY_FLOPS_PER_EXAMPLE[name] * B / (ms_priv * 1e-3) / 1e12
    if loop:
        # the same step inside dp_step_loop (draw from the batch as the dataset, step, update): one host call for all
        # steps, so what is timed is the launch chain itself without the per-call cost of the Python binding
        tq = tp.clone()
        st.dp_step_loop(tq, tx, ty, B, warmup, B, Cc, sigma, 0, 0.0)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        st.dp_step_loop(tq, tx, ty, B, steps, B, Cc, sigma, warmup, 0.0)
        torch.cuda.synchronize()
        res["loop_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / steps
    if profile:
        med, p10, p90 = per_call_ms(lambda i: st.dp_step(tp, tx, ty, B, Cc, sigma, i, out), st.stream, max(steps, 100))
        res["per_call_ms"] = dict(median=med, p10=p10, p90=p90, calls=max(steps, 100))
        # the same K steps again with every kernel launch bracketed by HIP events on the library's stream
        st.dp_step_profile(True)
        ms_prof = time_steps(lambda i: st.dp_step(tp, tx, ty, B, Cc, sigma, i, out), steps, 0)
        rows = st.dp_step_profile_read(reset=True)
        st.dp_step_profile(False)
        work = label_work(m, B, plan)

        def table(items):
            out = []
            for label, (launches, ms) in items.items():
                if launches == 0:
                    continue
                fl, by, ex = work.get(label, (0.0, 0.0, 0.0))
                per_step_ms = ms / steps
                sec = per_step_ms * 1e-3
                out.append(dict(kernel=label, launches_per_step=launches / steps, ms_per_step=per_step_ms,
                                avg_launch_us=1e3 * ms / launches,
                                tflops=(fl / sec / 1e12) if sec > 0 else 0.0,
                                tflops_executed=(ex / sec / 1e12) if sec > 0 else 0.0,
                                gbs=(by / sec / 1e9) if sec > 0 else 0.0,
                                hbm_frac=(by / sec / 1e9 / PEAK_HBM_GBS) if sec > 0 else 0.0,
                                flops_per_step=fl, bytes_per_step=by, executed_per_step=ex))
            out.sort(key=lambda r: -r["ms_per_step"])
            return out

        per_layer = {label: (launches, ms) for label, launches, ms in rows}
        per_kind = {}
        for label, launches, ms in rows:  # the library labels launches "<kind>#<layer>"
            k = label.split("#")[0]
            a, b = per_kind.get(k, (0, 0.0))
            per_kind[k] = (a + launches, b + ms)
        res["ms_private_profiled"] = ms_prof
        res["kernels"] = table(per_kind)
        res["kernels_per_layer"] = table(per_layer)
        res["launches_per_step"] = sum(l for _, l, _ in rows) / steps
        res["plan"] = plan
    st.dp_step_free()
    return res, wl


def cpu_baseline(wl, budget_s=12.0, threads=0):
    """The oracle as it stands on the host cores, on a bounded sample of the same workload."""
    from oracle import dpsgd_oracle as O
    m = wl["model"]
    cores = threads if threads > 0 else O.max_threads()
    n0 = min(wl["batch"], max(cores, 2 * cores if wl["batch"] >= 2 * cores else cores))
    t0 = time.perf_counter()
    O.dp_step(m, wl["params"], wl["x"][:n0], wl["y"][:n0], wl["C"], wl["sigma"], 0, n_threads=threads)
    dt = time.perf_counter() - t0
    rate = n0 / dt
    n = int(min(wl["batch"], max(n0, (rate * budget_s) // cores * cores)))
    t0 = time.perf_counter()
    O.dp_step(m, wl["params"], wl["x"][:n], wl["y"][:n], wl["C"], wl["sigma"], 0, n_threads=threads)
    dt = time.perf_counter() - t0
    return dict(value=n / dt, unit="examples/s", cores=cores, kind="oracle",
                sample=f"first {n} of {wl['batch']} examples of {wl['name']}, one step, {dt:.1f} s wall, "
                       f"gcc -O2 -fopenmp fp64 loop oracle")


def max_batch_fit(name, budgets_gb=(12.0, 288.0)):
    """Largest batch whose workspace + inputs + parameters fit a memory budget (the paper's Section 4 table lists the
    largest batch that runs in 12 GB): the workspace is linear in the batch (activations, backprops, stored
    per-example gradients) plus a fixed part (split-K partials, re-laid weights), so two contexts give the line."""
    from paper_2010_09063_amd import DpStep
    wl = W.make_workload(name, batch=2, seed=0)
    m = wl["model"]
    b1, b2 = 64, 256
    w1 = DpStep(m, b1); ws1 = w1.workspace_bytes; w1.dp_step_free()
    w2 = DpStep(m, b2); ws2 = w2.workspace_bytes; w2.dp_step_free()
    slope = (ws2 - ws1) / (b2 - b1)
    fixed = ws1 - slope * b1
    in_bytes = wl["x"][0].nbytes + 4
    P = wl["params"].size
    out = dict(workload=name, workspace_bytes_per_example=round(slope), workspace_fixed_mb=round(fixed / 2**20, 1))
    # the kernels index an activation tensor of the whole batch with 32-bit offsets
    shapes = W.layer_shapes(m)
    biggest = max(int(np.prod(sh[1:])) for sh in shapes)
    out["index_limit_batch"] = int((2**31 - 1) // max(biggest, 1))
    for gb in budgets_gb:
        fit = int((gb * 2**30 - fixed - 8.0 * P) // (slope + in_bytes))
        out[f"max_batch_{int(gb)}gb"] = max(0, min(fit, out["index_limit_batch"]))
    return out


def hbm_traffic(workload, label):
    """HBM bytes per launch of the kernel behind `label` ("<kind>#<layer>"), from the rocprofv3 --pmc runs summarised
    under profiles/ (FETCH_SIZE and WRITE_SIZE, already scaled by what a plain copy of known size reads); None when
    that launch has not been measured."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            t = json.load(f)
        e = t[workload][label]
        return float(e["fetch_bytes"]) + float(e["write_bytes"]), e.get("kernel")
    except (OSError, KeyError, ValueError, TypeError):
        return None, None


def rnd(d, keys=None):
    return {k: (round(v, 4) if isinstance(v, float) else v) for k, v in d.items() if keys is None or k in keys}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD, choices=sorted(W.CONFIGS))
    ap.add_argument("--batch", type=int, default=None, help="batch size of the main workload (default: the configuration's own)")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the short runs of the other configurations, the batch-size sweep, the memory study and the ceilings")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baselines")
    ap.add_argument("--kernels", action="store_true", help="print the per-kernel table to stderr")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also run the workload at batch sizes 16 ... 4096 (workspace bytes, examples/s, ratio)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (reference point for rocprofv3 --pmc byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (nothing in it uses a second); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible (the HIP path has no CPU fallback)", file=sys.stderr)
        sys.exit(3)
    from paper_2010_09063_amd import dp_step_ceiling

    if a.calib_copy:
        src = torch.ones(64 * 2**20, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    res, wl = run_workload(a.workload, a.steps, a.warmup, profile=True, batch=a.batch)
    kern = res["kernels"]
    # roofline of the dominant kernel: the single launch (kernel kind, layer) with the largest share of the step
    dom = res["kernels_per_layer"][0]
    mfma_bound = dom["flops_per_step"] > 0 and dom["flops_per_step"] / max(dom["bytes_per_step"], 1.0) > 20.0
    lps = max(dom["launches_per_step"], 1e-9)
    sec = dom["avg_launch_us"] * 1e-6
    traffic, hip_kernel = hbm_traffic(a.workload, dom["kernel"])
    if mfma_bound:
        ach = dom["flops_per_step"] / lps / sec / 1e12
        ach_ex = dom["executed_per_step"] / lps / sec / 1e12
        roof = dict(bound="mfma", achieved=ach, peak=PEAK_MFMA_FP32_TFLOPS, unit="TFLOP/s",
                    frac=ach / PEAK_MFMA_FP32_TFLOPS, traffic=traffic,
                    # the multiplies the launch really issues (a minimal-filtering route issues 16 where the direct
                    # form it is priced as has 36): this is the figure that says how busy the matrix units are
                    executed_flops_per_launch=dom["executed_per_step"] / lps, achieved_executed=ach_ex,
                    frac_executed=ach_ex / PEAK_MFMA_FP32_TFLOPS)
        if ach_ex < ach * 0.99:
            roof["note"] = ("frac divides the algorithmic (direct-form) flops by the peak; the route does fewer multiplies, "
                            "so frac overstates utilisation and may pass 1: frac_executed is the utilisation figure")
    else:
        ach = dom["bytes_per_step"] / lps / sec / 1e9
        roof = dict(bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s", frac=ach / PEAK_HBM_GBS,
                    traffic=traffic)
    layer = int(dom["kernel"].split("#")[1]) if "#" in dom["kernel"] else None
    roof.update(kernel=dom["kernel"], hip_kernel=hip_kernel, route=res["plan"].get(layer), avg_launch_us=dom["avg_launch_us"],
                launches_per_step=dom["launches_per_step"],
                algorithmic_flops_per_launch=dom["flops_per_step"] / lps,
                algorithmic_bytes_per_launch=dom["bytes_per_step"] / lps,
                share_of_step=dom["ms_per_step"] / max(res["ms_private_profiled"], 1e-9),
                traffic_source="profiles/hbm_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                               "scaled by a plain copy; not re-measured by this run)")
    # the whole step three ways: flops as the survey of the method prices them (direct forms everywhere), flops of
    # the routes taken (Gram norms, weighted sums of stored gradients), and the multiplies really issued
    acc = dict(tflops_routes=res["tflops"], frac_routes=res["tflops"] / PEAK_MFMA_FP32_TFLOPS,
               tflops_executed=res["tflops_executed"], frac_executed=res["tflops_executed"] / PEAK_MFMA_FP32_TFLOPS,
               launches_per_step=res["launches_per_step"],
               note="frac_executed is the utilisation of the fp32 matrix peak; the other two price work the routes avoid")
    if "tflops_survey_accounting" in res:
        acc.update(tflops_survey_accounting=res["tflops_survey_accounting"],
                   frac_survey_accounting=res["tflops_survey_accounting"] / PEAK_MFMA_FP32_TFLOPS)
    if a.kernels:
        for r in res["kernels_per_layer"]:
            print(f"  {r['kernel']:22s} {r['avg_launch_us']:9.1f} us {r['tflops']:8.2f} TFLOP/s (executed {r['tflops_executed']:7.2f}) "
                  f"{r['gbs']:9.1f} GB/s", file=sys.stderr)
        for r in kern:
            print(f"{r['kernel']:20s} {r['launches_per_step']:5.1f}/step {r['ms_per_step']*1e3:10.1f} us/step "
                  f"{r['tflops']:8.2f} TFLOP/s {r['gbs']:9.1f} GB/s", file=sys.stderr)

    others, sweeps, fits, ceilings = [], {}, [], None
    if not a.no_others:
        for name in sorted(W.CONFIGS):
            if name == a.workload:
                continue
            r, _ = run_workload(name, max(10, a.steps // 2), max(3, a.warmup // 2), profile=False)
            others.append(rnd(r))
        # batch sizes of the paper's Section 3 figures on the two large configurations
        for name in ("cfg4_cifar_cnn", "cfg5_lstm"):
            rows = []
            for bsz in (16, 32, 64, 128, 256):
                r, _ = run_workload(name, 20, 5, profile=False, batch=bsz, loop=False)
                rows.append(rnd(r, ("batch", "ms_private", "ms_nonprivate", "examples_per_s", "ratio", "workspace_mb")))
            sweeps[name] = rows
        fits = [max_batch_fit(name) for name in ("cfg1_logistic", "cfg2_mlp", "cfg3_small_cnn", "cfg4_cifar_cnn", "cfg5_lstm")]
        ceilings = dict(copy_gbs=dp_step_ceiling(0), mfma_fp32_tflops=dp_step_ceiling(1), empty_launch_us=dp_step_ceiling(2),
                        nominal=dict(hbm_gbs=PEAK_HBM_GBS, mfma_fp32_tflops=PEAK_MFMA_FP32_TFLOPS),
                        what="plain 256 MiB device copy (read + written); register-only v_mfma_f32_32x32x2_f32 loop; "
                             "1000 empty launches back to back")

    sweep = []
    if a.batch_sweep:
        for bsz in (16, 32, 64, 128, 256, 512, 1024, 2048, 4096):
            r, _ = run_workload(a.workload, max(10, a.steps // 2), max(3, a.warmup // 2), profile=False, batch=bsz, loop=False)
            sweep.append(rnd(r, ("batch", "ms_private", "ms_nonprivate", "examples_per_s", "ratio", "workspace_mb")))
            print(f"  B={bsz:5d}  {r['ms_private']:8.3f} ms  {r['examples_per_s']:12.0f} ex/s  ratio {r['ratio']:.3f}  "
                  f"workspace {r['workspace_mb']:9.1f} MB", file=sys.stderr)

    cpu, cpus = None, []
    if not a.no_cpu:
        cpu = cpu_baseline(wl)
        if not a.no_others:
            # the oracle on all five configurations (bounded samples), and on one thread for the three small ones
            for name in ("cfg1_logistic", "cfg2_mlp", "cfg3_small_cnn", "cfg4_cifar_cnn", "cfg5_lstm"):
                w2 = wl if name == a.workload and a.batch is None else W.make_workload(name, seed=0)
                e = dict(workload=name, **(cpu if w2 is wl else cpu_baseline(w2, budget_s=2.5)))
                if name in ("cfg1_logistic", "cfg2_mlp", "cfg3_small_cnn"):
                    e["one_thread_examples_per_s"] = cpu_baseline(w2, budget_s=1.0, threads=1)["value"]
                cpus.append(rnd(e))

    line = {
        "metric": "private examples/sec per DPSGD step on 1 MI355X; private/non-private step ratio",
        "value": res["examples_per_s"], "unit": "examples/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": res["ms_private"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": a.workload, "batch": res["batch"], "params": res["params"], "C": wl["C"],
                   "sigma": wl["sigma"], "inputs": "resident in HBM"},
        "nonprivate_ms_per_step": res["ms_nonprivate"], "private_over_nonprivate": res["ratio"],
        "loop_ms_per_step": res.get("loop_ms_per_step"),
        "per_call_ms": rnd(res.get("per_call_ms", {})),
        "roofline": roof,
        "step_accounting": acc,
        "ceilings": ceilings,
        "cpu_baseline": cpu,
        "cpu_baselines": cpus,
        "kernels": [rnd(r, ("kernel", "launches_per_step", "ms_per_step", "tflops", "tflops_executed", "gbs", "hbm_frac")) for r in kern],
        "kernels_per_layer": [rnd(r, ("kernel", "avg_launch_us", "tflops", "tflops_executed", "gbs", "hbm_frac"))
                              for r in res["kernels_per_layer"][:16]],
        "plan": {str(k): v for k, v in res["plan"].items()},
        "other_workloads": others,
        "batch_sweep_paper_sizes": sweeps,
        "max_batch_fit": fits,
    }
    if sweep:
        line["batch_sweep"] = sweep
    print(json.dumps(line))


if __name__ == "__main__":
    main()
