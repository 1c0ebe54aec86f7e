"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element on
the same seeded inputs.  Bar: relative L2 <= 1e-4 on the aggregated fp32 gradient at
sigma = 0; <= 1e-5 absolute on the noise term for the same Philox stream."""
import math

import numpy as np
import pytest

import dp_workloads as W
from oracle import dpsgd_oracle as O
from tests.gpu_util import TOL, TieAwareOracle, assert_parity, check_step, rel_l2, run_gpu

pytestmark = pytest.mark.gpu

TINY = W.tiny_models()


def _case(m, batch, seed, x_dist="normal", bias=0.3, scale=1.0, zipf=0.3):
    rng = np.random.default_rng(seed)
    x, y = W.make_inputs(m, batch, rng, x_dist=x_dist, zipf_exponent=zipf)
    theta = W.init_params(m, rng, bias_scale=bias) * np.float32(scale)
    return x, y, theta


def _check_all_regimes(m, x, y, theta, label, stepper=None, options=None):
    """Whole batch, every parameter tensor, every per-example norm, in the three clipping regimes and for the
    non-private sum (max-pool windows tied at rounding level: see tests/gpu_util.py)."""
    ref_inf = O.dp_step(m, theta, x, y, math.inf, 0.0, 0)
    tie = TieAwareOracle(m, theta, x, y, ref_inf["pool_margin"])
    n0 = ref_inf["norms"]
    regimes = [math.inf, float(np.median(n0)), 0.1 * float(n0.min())]
    for Cc in regimes:
        ref = ref_inf if math.isinf(Cc) else O.dp_step(m, theta, x, y, Cc, 0.0, 0)
        out, gn, norms = check_step(m, theta, x, y, Cc, ref, f"{label} C={Cc:.4g}", tie=tie, stepper=stepper,
                                    options=options)
        if not math.isinf(Cc):
            s = np.minimum(1.0, Cc / gn.astype(np.float64))
            assert np.all(s * norms <= Cc * (1 + 1e-5))
    ref_np = O.dp_step(m, theta, x, y, 1.0, 0.0, 0, clip=False)
    check_step(m, theta, x, y, 1.0, ref_np, f"{label} non-private", tie=tie, private=False, stepper=stepper,
               options=options)


@pytest.mark.parametrize("name", sorted(TINY))
@pytest.mark.parametrize("batch", [1, 7, 70])
def test_tiny_models(name, batch):
    m = TINY[name]
    scale = 4.0 if m["input"]["kind"] == "tokens" else 1.0
    x, y, theta = _case(m, batch, seed=11 + batch, scale=scale)
    _check_all_regimes(m, x, y, theta, f"{name}/B{batch}")


# real layer shapes, batches that span several tiles and leave a ragged tail
REDUCED = {"cfg1_logistic": 100, "cfg2_mlp": 77, "cfg3_small_cnn": 37, "cfg4_cifar_cnn": 5, "cfg5_lstm": 6,
           "cfg6_embedding": 45, "paper_ffnn": 100, "paper_mnist_cnn": 37, "paper_cifar_cnn": 5, "paper_embedding": 45,
           "paper_lstm": 6}


@pytest.mark.parametrize("name", sorted(REDUCED))
def test_benchmark_architectures_reduced_batch(name):
    wl = W.make_workload(name, batch=REDUCED[name], seed=2, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], name)


@pytest.mark.parametrize("name", ["cfg1_logistic", "cfg2_mlp", "cfg3_small_cnn", "cfg5_lstm", "cfg6_embedding",
                                  "cfg4_cifar_cnn", "paper_ffnn", "paper_mnist_cnn", "paper_embedding", "paper_lstm",
                                  "paper_cifar_cnn"])
def test_benchmark_full_size(name):
    """Full configured batch, benchmark launch configuration (C = 1, then a C that clips about half): every
    example takes part in the comparison."""
    wl = W.make_workload(name, seed=0)
    m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    ref = O.dp_step(m, theta, x, y, wl["C"], 0.0, 0)
    # ReLU outputs tie at 0 inside pool windows; ReLU'(0) = 0 stops the gradient whichever element wins
    assert ref["ties"] == 0 or name == "paper_mnist_cnn"
    tie = TieAwareOracle(m, theta, x, y, ref["pool_margin"])
    print(f"{name} full: clipped={(ref['norms'] > wl['C']).mean():.2f}", flush=True)
    check_step(m, theta, x, y, wl["C"], ref, f"{name} full C={wl['C']}", tie=tie)
    Cmed = float(np.median(ref["norms"]))
    ref2 = O.dp_step(m, theta, x, y, Cmed, 0.0, 0)
    out2, _, _ = check_step(m, theta, x, y, Cmed, ref2, f"{name} full C=median", tie=tie)
    assert np.linalg.norm(out2) <= len(y) * Cmed * (1 + 1e-5)


@pytest.mark.parametrize("name,batch", [("tiny_dense", 5), ("tiny_lstm", 3), ("cfg3_small_cnn", 16), ("cfg5_lstm", 2)])
def test_noise_term(name, batch):
    if name in TINY:
        m = TINY[name]
        x, y, theta = _case(m, batch, seed=5)
    else:
        wl = W.make_workload(name, batch=batch, seed=5)
        m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    Cc, sigma = 1.0, 1.1
    for seed in (0, 0x1234567887654321):
        out0, _ = run_gpu(m, theta, x, y, Cc, 0.0, seed)
        out1, _ = run_gpu(m, theta, x, y, Cc, sigma, seed)
        z = O.noise(seed, theta.size)
        err = np.abs((out1.astype(np.float64) - out0.astype(np.float64)) - sigma * Cc * z).max()
        print(f"{name} seed={seed:#x} noise abs err {err:.2e}", flush=True)
        assert err <= 1e-5
        ref = O.dp_step(m, theta, x, y, Cc, sigma, seed)
        assert np.abs(out1.astype(np.float64) - ref["out"]).max() <= 1e-5 + 1e-4 * np.abs(ref["out"]).max()
        # empty batch: pure noise
        outz, _ = run_gpu(m, theta, x[:0], y[:0], Cc, sigma, seed, max_batch=4)
        assert np.abs(outz - sigma * Cc * z).max() <= 1e-5


def test_context_reuse_and_smaller_batches():
    """One context serves batches of different sizes, private and non-private, in any order."""
    from paper_2010_09063_amd import DpStep
    m = W.cfg3_small_cnn()
    st = DpStep(m, 48)
    for batch in (48, 5, 33):
        wl = W.make_workload("cfg3_small_cnn", batch=batch, seed=batch, bias_scale=0.1)
        ref = O.dp_step(m, wl["params"], wl["x"], wl["y"], 0.5, 0.0, 0)
        tie = TieAwareOracle(m, wl["params"], wl["x"], wl["y"], ref["pool_margin"])
        check_step(m, wl["params"], wl["x"], wl["y"], 0.5, ref, f"reuse/B{batch}", tie=tie, stepper=st)
        refn = O.dp_step(m, wl["params"], wl["x"], wl["y"], 0.5, 0.0, 0, clip=False)
        check_step(m, wl["params"], wl["x"], wl["y"], 0.5, refn, f"reuse/B{batch} non-private", tie=tie,
                   private=False, stepper=st)
    st.dp_step_free()


def test_context_reuse_with_minimal_filtering_kernels():
    """One context planned for the largest batch serves smaller ones: the minimal-filtering kernels (forward,
    backward-data with the pool in the epilogue, weight gradients) size their grids and split counts from the batch
    of the call, the plan from the batch of the context."""
    from paper_2010_09063_amd import DpStep
    m = W.model(W.image_input(32, 16, 16), [
        W.conv2d(32, 32, 3, stride=1, pad=1, act="tanh"), W.conv2d(32, 64, 3, stride=1, pad=1, act="tanh"),
        W.maxpool2d(2, 2), W.conv2d(64, 64, 3, stride=1, pad=1, act="relu"), W.avgpool2d(2, 2),
        W.dense(64 * 4 * 4, 3)], 3)
    st = DpStep(m, 9, minimal_filtering_all=1)
    for batch in (9, 2, 7, 1):
        x, y, theta = _case(m, batch, seed=50 + batch)
        ref = O.dp_step(m, theta, x, y, 5.0, 0.0, 0)
        tie = TieAwareOracle(m, theta, x, y, ref["pool_margin"])
        check_step(m, theta, x, y, 5.0, ref, f"reuse-mf/B{batch}", tie=tie, stepper=st)
        refn = O.dp_step(m, theta, x, y, 5.0, 0.0, 0, clip=False)
        check_step(m, theta, x, y, 5.0, refn, f"reuse-mf/B{batch} non-private", tie=tie, private=False, stepper=st)
    st.dp_step_free()


def test_argument_errors():
    import torch
    from paper_2010_09063_amd import DpStep, DpStepError
    m = TINY["tiny_dense"]
    st = DpStep(m, 4)
    dev = torch.device("cuda:0")
    p = torch.zeros(st.num_params, device=dev)
    x = torch.zeros(4, 5, device=dev)
    y = torch.zeros(4, dtype=torch.int32, device=dev)
    o = torch.zeros(st.num_params, device=dev)
    for args in [(p, x, y, 5, 1.0, 0.0, 0, o), (p, x, y, 4, 0.0, 0.0, 0, o), (p, x, y, 4, -1.0, 0.0, 0, o),
                 (p, x, y, 4, 1.0, -0.1, 0, o), (p, x, y, 4, float("nan"), 0.0, 0, o),
                 (p, x, y, 4, float("inf"), 1.0, 0, o), (None, x, y, 4, 1.0, 0.0, 0, o), (p, None, y, 4, 1.0, 0.0, 0, o)]:
        with pytest.raises(DpStepError) as e:
            st.dp_step(*args)
        assert e.value.code == -1
    st.dp_step_free()
    bad = W.model(W.image_input(5), [W.dense(6, 3)], 3)
    with pytest.raises(DpStepError):
        DpStep(bad, 4)


def test_generic_convolution_path_matches_too():
    """generic_conv keeps 3x3 stride-1 convolutions on the functor contraction (the path every other kernel size /
    stride takes); gemm_plain_tiles picks its tiles without the padding-waste rule."""
    opt = dict(generic_conv=1)
    m = TINY["tiny_conv3"]
    x, y, theta = _case(m, 9, seed=21)
    _check_all_regimes(m, x, y, theta, "tiny_conv3/generic", options=opt)
    wl = W.make_workload("cfg4_cifar_cnn", batch=3, seed=4, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/generic", options=opt)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/generic, plain tiles",
                       options=dict(generic_conv=1, gemm_plain_tiles=1))
    wl = W.make_workload("cfg5_lstm", batch=5, seed=4, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg5/plain tiles", options=dict(gemm_plain_tiles=1))


def test_many_examples_per_workgroup():
    """Batches large enough that a workgroup of the convolution norm kernels walks through several examples (here
    three): what one example's reduction leaves in LDS must not reach the next one.  16x16 planes, so the norm pass
    also stores the per-example gradients that the clipped sum is formed from; the first-layer (flattened) kernel,
    the 32-channel-block kernel with at most 32 output channels (their waves share a cross-wave area) and the one
    for up to 64 output channels."""
    m = W.model(W.image_input(3, 16, 16), [
        W.conv2d(3, 16, 3, stride=1, pad=1, act="tanh"), W.conv2d(16, 24, 3, stride=1, pad=1, act="tanh"),
        W.conv2d(24, 40, 3, stride=1, pad=1, act="tanh"), W.dense(40 * 16 * 16, 3)], 3)
    x, y, theta = _case(m, 1100, seed=31)
    ref = O.dp_step(m, theta, x, y, math.inf, 0.0, 0)
    Cc = float(np.median(ref["norms"]))
    ref_c = O.dp_step(m, theta, x, y, Cc, 0.0, 0)
    out, gn = run_gpu(m, theta, x, y, Cc, 0.0, 0)
    err = np.abs(gn / ref["norms"] - 1.0).max()
    print(f"many examples per workgroup: rel_l2={rel_l2(out, ref_c['clipped_sum']):.3e} max norm err {err:.2e}", flush=True)
    assert err <= 2e-5
    assert rel_l2(out, ref_c["clipped_sum"]) <= TOL


def test_recompute_routes_match_too():
    """With the Gram norms, the stored-gradient route and the column route of strided backward-data switched off,
    the library takes the routes it otherwise keeps for shapes those do not cover (direct per-example contraction
    for the norm, a second contraction for the clipped sum, the gathering backward-data contraction)."""
    opt = dict(no_gram=1, no_stored_gradients=1, no_columns=1)
    for name, batch in (("tiny_conv_gram", 9), ("tiny_conv_store", 6), ("tiny_conv_stride", 11), ("tiny_lstm_seq", 5)):
        m = TINY[name]
        x, y, theta = _case(m, batch, seed=41, scale=4.0 if m["input"]["kind"] == "tokens" else 1.0)
        _check_all_regimes(m, x, y, theta, f"{name}/recompute", options=opt)
    wl = W.make_workload("cfg4_cifar_cnn", batch=3, seed=4, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/recompute", options=opt)
    m = W.paper_lstm(vocab=300, seq_len=140, dim=20, hidden=24)  # 140 steps: above the stored-gradient threshold
    rng = np.random.default_rng(9)
    x, y = W.make_inputs(m, 4, rng)
    theta = W.init_params(m, rng, bias_scale=0.2) * np.float32(3)
    _check_all_regimes(m, x, y, theta, "lstm_seq/T140/recompute", options=opt)


def test_minimal_filtering_route():
    """Forward and backward-data of the pad-1 3x3 convolutions through the F(2x2, 3x3) kernel at sizes the oracle
    covers element by element (the library keeps that kernel for launches that fill the chip; here it is forced):
    4x4, 8x8 and 16x16 planes, channel counts that are no multiples of the 8-channel chunk or of the 32 / 64 output
    channels of a workgroup, more than 64 output channels (several channel blocks), batches that end inside a
    workgroup's 32 tiles, a 3-channel first layer.  (The full-size cases run it wherever the library selects it.)
    The benchmark-shaped cases also take the weight-gradient kernels of the same family: per-example norm pass with
    stored gradients on 16- and 32-wide planes, clipped sums on 8x8 planes, and the batch sums of the non-private
    step; the last part switches the whole family off at full batch."""
    cases = (("tiny_conv_gram", 9), ("tiny_conv_store", 6), ("tiny_conv_wide", 13), ("tiny_conv_wide", 1))
    opt = dict(minimal_filtering_all=1)
    for name, batch in cases:
        m = TINY[name]
        x, y, theta = _case(m, batch, seed=43)
        _check_all_regimes(m, x, y, theta, f"{name}/minimal-filtering", options=opt)
    # 32x32 planes with 64 output channels per workgroup, forward (8 -> 40) and backward-data (16 -> 40)
    m = W.model(W.image_input(8, 32, 32), [
        W.conv2d(8, 40, 3, stride=1, pad=1, act="tanh"), W.conv2d(40, 16, 3, stride=1, pad=1, act="tanh"),
        W.avgpool2d(8, 8), W.dense(16 * 4 * 4, 3)], 3)
    x, y, theta = _case(m, 3, seed=44)
    _check_all_regimes(m, x, y, theta, "planes32/minimal-filtering", options=opt)
    wl = W.make_workload("cfg4_cifar_cnn", batch=3, seed=4, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/minimal-filtering", options=opt)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/minimal-filtering, pools apart",
                       options=dict(minimal_filtering_all=1, no_pool_fusion=1))
    wl = W.make_workload("paper_cifar_cnn", batch=5, seed=6, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "paper_cifar/minimal-filtering", options=opt)
    # 32 -> 32 channels without the persistent kernel that keeps the transformed weights in registers
    wl = W.make_workload("cfg4_cifar_cnn", batch=3, seed=4, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/minimal-filtering, per-group kernel",
                       options=dict(minimal_filtering_all=1, no_resident_weights=1))
    # full batch with that route switched off: the direct kernels in the launch shapes of the benchmark batch
    wl = W.make_workload("cfg4_cifar_cnn", seed=0)
    m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    ref = O.dp_step(m, theta, x, y, wl["C"], 0.0, 0)
    check_step(m, theta, x, y, wl["C"], ref, "cfg4 full batch, direct kernels", options=dict(no_minimal_filtering=1))


def test_first_layer_forward_kernel():
    """The persistent forward and per-example weight-gradient kernels of an RGB first layer (3x3, pad 1, 32-wide planes):
    3, 2 and 1 input channels, 32 and fewer output channels, planes of 8 (forward only), 16 and 32 rows, both
    activations, batches that give a workgroup one tile / example and several with a shorter run for the last
    workgroup; then the same layer on the generic direct kernels."""
    for cin, d, h, act, batch in ((3, 32, 32, "relu", 3), (3, 20, 16, "tanh", 5), (1, 7, 8, "relu", 9), (2, 32, 32, "tanh", 300),
                                  (3, 32, 16, "relu", 1100)):
        m = W.model(W.image_input(cin, h, 32), [
            W.conv2d(cin, d, 3, stride=1, pad=1, act=act), W.avgpool2d(8, 8), W.dense(d * (h // 8) * 4, 3)], 3)
        x, y, theta = _case(m, batch, seed=cin + d)
        _check_all_regimes(m, x, y, theta, f"first layer {cin}->{d}/H{h}/{act}/B{batch}")
    wl = W.make_workload("cfg4_cifar_cnn", batch=4, seed=5, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/first layer on the direct kernel",
                       options=dict(no_first_layer_kernel=1))


def test_resident_weight_minimal_filtering_kernel():
    """The persistent F(2x2, 3x3) kernel for 32 input and at most 32 output channels (weights in registers, a run of
    tile groups per workgroup): 32-wide planes with forward into 32 channels with the fused pool, forward into 20
    channels on 16-wide planes, backward-data into 8 and into 32 channels (through tanh and ReLU); batches that give a
    workgroup one group, two groups, and three with a shorter run for the last workgroup."""
    m = W.model(W.image_input(8, 32, 32), [
        W.conv2d(8, 32, 3, stride=1, pad=1, act="tanh"), W.conv2d(32, 32, 3, stride=1, pad=1, act="relu"),
        W.maxpool2d(2, 2), W.conv2d(32, 20, 3, stride=1, pad=1, act="tanh"), W.avgpool2d(4, 4), W.dense(20 * 4 * 4, 3)], 3)
    for batch in (2, 65, 130):
        x, y, theta = _case(m, batch, seed=batch)
        _check_all_regimes(m, x, y, theta, f"planes32 8->32->32->20/B{batch}", options=dict(minimal_filtering_all=1))
    m = W.model(W.image_input(32, 16, 16), [
        W.conv2d(32, 32, 3, stride=1, pad=1, act="relu"), W.conv2d(32, 32, 3, stride=1, pad=1, act="tanh"),
        W.maxpool2d(2, 2), W.dense(32 * 8 * 8, 3)], 3)
    for batch in (3, 514):
        x, y, theta = _case(m, batch, seed=batch)
        _check_all_regimes(m, x, y, theta, f"planes16 32->32->32/B{batch}", options=dict(minimal_filtering_all=1))
    # wider layers take the same kernel once per block of 32 output channels: 64 (two full blocks) and 40 (the second
    # block partly empty), forward; backward-data from 64 channels does not (its channel loop is longer)
    m = W.model(W.image_input(32, 16, 16), [
        W.conv2d(32, 64, 3, stride=1, pad=1, act="relu"), W.conv2d(64, 32, 3, stride=1, pad=1, act="tanh"),
        W.conv2d(32, 40, 3, stride=1, pad=1, act="tanh"), W.maxpool2d(2, 2), W.dense(40 * 8 * 8, 3)], 3)
    for batch in (3, 300):
        x, y, theta = _case(m, batch, seed=batch)
        _check_all_regimes(m, x, y, theta, f"planes16 32->64->32->40/B{batch}", options=dict(minimal_filtering_all=1))


def test_weight_gradients_in_minimal_filtering_form():
    """Weight-gradient kernels of the F(3x3, 2x2) family at shapes the benchmark configurations do not have: 32
    output channels on 16x16 planes (norm pass with stored gradients, and the batch sum of the non-private step), 64
    on 16x16, and on 8x8 planes a layer whose norm does not come from Gram matrices, with one block of 64 output
    channels; then the same network with these routes switched off."""
    m = W.model(W.image_input(32, 16, 16), [
        W.conv2d(32, 32, 3, stride=1, pad=1, act="tanh"), W.conv2d(32, 64, 3, stride=1, pad=1, act="tanh"),
        W.maxpool2d(2, 2), W.conv2d(64, 64, 3, stride=1, pad=1, act="relu"), W.avgpool2d(2, 2),
        W.dense(64 * 4 * 4, 3)], 3)
    x, y, theta = _case(m, 5, seed=46)
    _check_all_regimes(m, x, y, theta, "planes16x16+8x8/weight gradients")


def test_weight_gradients_direct_kernels_on_the_same_network():
    m = W.model(W.image_input(32, 16, 16), [
        W.conv2d(32, 32, 3, stride=1, pad=1, act="tanh"), W.conv2d(32, 64, 3, stride=1, pad=1, act="tanh"),
        W.maxpool2d(2, 2), W.conv2d(64, 64, 3, stride=1, pad=1, act="relu"), W.avgpool2d(2, 2),
        W.dense(64 * 4 * 4, 3)], 3)
    x, y, theta = _case(m, 5, seed=46)
    _check_all_regimes(m, x, y, theta, "planes16x16+8x8/direct weight gradients",
                       options=dict(no_minimal_filtering_wgrad=1))


def _wide_conv_net():
    # 8x8 planes, 128 output channels: the weight-gradient kernels with 144 accumulator registers per lane
    return W.model(W.image_input(32, 8, 8), [
        W.conv2d(32, 128, 3, stride=1, pad=1, act="tanh"), W.conv2d(128, 128, 3, stride=1, pad=1, act="tanh"),
        W.conv2d(128, 64, 3, stride=1, pad=1, act="tanh"), W.dense(64 * 8 * 8, 3)], 3)


@pytest.mark.parametrize("opt", [dict(no_gram=1, no_minimal_filtering=1),
                                 dict(no_gram=1, no_minimal_filtering=1, no_specialised_waves=1),
                                 dict(no_gram=1, no_minimal_filtering=1, specialised_waves_all=1),
                                 dict(no_gram=1, no_minimal_filtering=1, specialised_waves_all=1, no_stored_gradients=1)],
                         ids=["ws-wide-only", "no-ws", "ws-all", "ws-all-recompute"])
def test_specialised_wave_weight_gradients(opt):
    """The weight-gradient kernel whose waves split into staging and multiplying ones (norm and clipped-sum modes),
    for the 128-channel layers it is planned for, switched off, and forced for every width; batches that give a
    workgroup several examples and a ragged last run."""
    m = _wide_conv_net()
    for batch in (3, 70):
        x, y, theta = _case(m, batch, seed=60 + batch)
        _check_all_regimes(m, x, y, theta, f"wide conv/B{batch}/{sorted(opt)}", options=opt)
    if "specialised_waves_all" in opt:
        m = TINY["tiny_conv_store"]
        x, y, theta = _case(m, 6, seed=61)
        _check_all_regimes(m, x, y, theta, f"tiny_conv_store/{sorted(opt)}", options=opt)


def test_remaining_route_switches():
    """conv_min_blocks (tile narrowing of the direct forward kernel, both extremes) and no_fused_dense (a one-layer
    model on the generic kernels)."""
    m = TINY["tiny_conv3"]
    x, y, theta = _case(m, 9, seed=21)
    for mb in (1, 1 << 20):
        _check_all_regimes(m, x, y, theta, f"tiny_conv3/min_blocks={mb}", options=dict(conv_min_blocks=mb, no_minimal_filtering=1))
    wl = W.make_workload("cfg1_logistic", batch=100, seed=2, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg1/generic kernels", options=dict(no_fused_dense=1))
    # deeper networks that end in two dense layers take one launch for logits, loss gradient, both dense norms and the
    # hidden layer's backprop; the same switch keeps them on the generic kernels
    for name, batch in (("cfg4_cifar_cnn", 5), ("cfg6_embedding", 45), ("paper_lstm", 7)):
        wl = W.make_workload(name, batch=batch, seed=3, bias_scale=0.2)
        _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], f"{name}/dense head on the generic kernels",
                           options=dict(no_fused_dense=1))
        # the head's batch-wide contractions (hidden layer forward, both clipped sums in one launch with the clip
        # factors applied while delta is staged) on the split-K kernels instead
        _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], f"{name}/dense head, split-K contractions",
                           options=dict(no_small_gemm=1))
    # the embedding's counting sort as three launches with per-workgroup LDS histograms (the default for batches of
    # more than 2^15 steps; smaller ones take the single-workgroup kernel)
    for name, batch in (("cfg6_embedding", 45), ("cfg5_lstm", 6)):
        wl = W.make_workload(name, batch=batch, seed=2, bias_scale=0.2)
        _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], f"{name}/three-launch buckets",
                           options=dict(no_single_bucket=1))
        # the same lists built in line on the caller's stream (by default they are built beside the forward pass)
        _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], f"{name}/buckets on the caller's stream",
                           options=dict(no_side_stream=1))


def test_one_layer_models_of_other_widths():
    """The fused softmax-regression kernel at class counts that pad to 4, 10 and 15 lanes, feature counts below one
    wave's share and at the limit, batches that end inside a group of four and that give a workgroup several groups."""
    for d_in, k, batch in ((5, 2, 7), (9, 4, 1), (1023, 10, 33), (300, 15, 1100), (784, 10, 1026)):
        m = W.model(W.image_input(d_in), [W.dense(d_in, k)], k)
        x, y, theta = _case(m, batch, seed=d_in)
        _check_all_regimes(m, x, y, theta, f"dense {d_in}->{k}/B{batch}")


def test_two_layer_models_of_other_widths():
    """The fused kernel of two-dense-layer models: hidden widths below one wave's share, not a multiple of four, at
    the limit; both activations; class counts that pad to 4, 10 and 15 lanes; a hidden layer wide enough that its
    forward product is split over K and one that is not; batches with a ragged last group and several groups per
    workgroup; then the same models on the generic kernels."""
    cases = ((7, 5, 3, "tanh", 9), (784, 512, 10, "relu", 37), (64, 1023, 10, "tanh", 6), (300, 50, 15, "relu", 1100),
             (2000, 33, 2, "tanh", 70),
             # widths in whole groups of four floats take the kernel that splits K inside the workgroup: ragged 32 x 32
             # tiles in both directions, K below one slice, K that ends inside a slice, K of several slices per wave
             (100, 36, 4, "tanh", 70), (8, 4, 2, "relu", 5), (1000, 68, 10, "relu", 333))
    for d_in, H, k, act, batch in cases:
        m = W.model(W.image_input(d_in), [W.dense(d_in, H, act=act), W.dense(H, k)], k)
        x, y, theta = _case(m, batch, seed=H)
        _check_all_regimes(m, x, y, theta, f"dense {d_in}->{H}->{k}/{act}/B{batch}")
    wl = W.make_workload("cfg2_mlp", batch=77, seed=2, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg2/generic kernels", options=dict(no_fused_dense=1))
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg2/split-K contraction", options=dict(no_small_gemm=1))
    m = W.model(W.image_input(37), [W.dense(37, 45, act="tanh"), W.dense(45, 3)], 3)
    x, y, theta = _case(m, 70, seed=5)
    _check_all_regimes(m, x, y, theta, "dense 37->45->3/split-K contraction", options=dict(no_small_gemm=1))


def test_deeper_dense_stacks():
    """Three and four dense layers: the last two run in the head kernel.  Widths in whole groups of four floats take
    the small contraction for the hidden layer's forward product and for both clipped sums (clip factors applied to
    delta as it is staged: the layers below contribute to the norm, so most examples are clipped), at batches with a
    ragged last tile; odd widths keep the split-K kernels, and every tensor boundary then falls inside a Philox block
    of the final write."""
    from paper_2010_09063_amd import DpStep
    cases = (((64, 48, 36, 10), "tanh", 45), ((100, 64, 128, 32, 4), "relu", 133), ((37, 45, 33, 7, 3), "tanh", 21),
             ((784, 256, 128, 10), "relu", 300))
    for widths, act, batch in cases:
        layers = [W.dense(a, b, act=act) for a, b in zip(widths[:-2], widths[1:-1])] + [W.dense(widths[-2], widths[-1])]
        m = W.model(W.image_input(widths[0]), layers, widths[-1])
        x, y, theta = _case(m, batch, seed=widths[1])
        _check_all_regimes(m, x, y, theta, f"dense {'->'.join(map(str, widths))}/{act}/B{batch}")
        st = DpStep(m, batch)
        plan = st.dp_step_describe_plan()
        st.dp_step_free()
        last = plan[max(plan)]
        assert last["fwd"] == "head" and (last["sum"] == "joint") == (widths[-3] % 4 == 0 and widths[-2] % 4 == 0), plan
    widths = (100, 64, 128, 32, 4)
    layers = [W.dense(a, b, act="tanh") for a, b in zip(widths[:-2], widths[1:-1])] + [W.dense(widths[-2], widths[-1])]
    m = W.model(W.image_input(widths[0]), layers, widths[-1])
    x, y, theta = _case(m, 57, seed=3)
    _check_all_regimes(m, x, y, theta, "dense stack/split-K contractions", options=dict(no_small_gemm=1))


def test_seeded_random_architectures():
    """Architectures drawn from a seeded generator, within the documented limits: dense stacks of two to four layers
    (widths in whole groups of four floats or not, up to 900 inputs, 2 to 14 classes) and pad-1 3x3 convolution
    stacks on 8-, 16- and 32-wide planes with max- and average-pools between them (3 to 64 channels, one or two dense
    layers at the end), each with the planner's own routes or with the minimal-filtering kernels forced."""
    rng = np.random.default_rng(2024)
    for it in range(14):
        depth = int(rng.integers(2, 5))
        mult4 = rng.random() < 0.7
        def width(lo, hi):
            w = int(rng.integers(lo, hi))
            return max(4, (w // 4) * 4) if mult4 else w
        widths = [width(4, 900)] + [width(4, 300) for _ in range(depth - 1)] + [int(rng.integers(2, 15))]
        act = ["tanh", "relu"][int(rng.integers(0, 2))]
        batch = int(rng.integers(1, 400))
        layers = [W.dense(a, b, act=act) for a, b in zip(widths[:-2], widths[1:-1])] + [W.dense(widths[-2], widths[-1])]
        m = W.model(W.image_input(widths[0]), layers, widths[-1])
        x, y, theta = _case(m, batch, seed=it)
        _check_all_regimes(m, x, y, theta, f"random dense {widths} {act} B{batch}")
    rng = np.random.default_rng(77)
    for it in range(12):
        plane = int(rng.choice([8, 16, 32]))
        chans = [int(rng.choice([3, 8, 16, 32]))]
        layers, h = [], plane
        for _ in range(int(rng.integers(2, 5))):
            co = int(rng.choice([8, 20, 32, 40, 64] if plane * plane * max(chans) <= 32768 else [8, 16, 32]))
            layers.append(W.conv2d(chans[-1], co, 3, stride=1, pad=1, act=["tanh", "relu"][int(rng.integers(0, 2))]))
            chans.append(co)
            if h >= 8 and rng.random() < 0.6:
                layers.append(W.maxpool2d(2, 2) if rng.random() < 0.75 else W.avgpool2d(2, 2))
                h //= 2
        feat, k = chans[-1] * h * h, int(rng.integers(2, 11))
        if rng.random() < 0.5:
            hid = int(rng.choice([16, 30, 64]))
            layers += [W.dense(feat, hid, act="tanh"), W.dense(hid, k)]
        else:
            layers += [W.dense(feat, k)]
        m = W.model(W.image_input(chans[0], plane, plane), layers, k)
        batch = int(rng.integers(1, 40))
        opts = [None, dict(minimal_filtering_all=1)][int(rng.integers(0, 2))]
        x, y, theta = _case(m, batch, seed=it)
        _check_all_regimes(m, x, y, theta, f"random conv {it}: plane {plane}, channels {chans}, B{batch}", options=opts)


def test_small_cnn_layer_by_layer_and_fused():
    """The MNIST-shaped CNN takes one fused launch by default; no_fused_cnn keeps it on the per-layer kernels.  Both
    routes at batches below, at and above one example per workgroup (a workgroup of the fused kernel walks through
    several examples from batch 257 on), both activation sets."""
    for name in ("cfg3_small_cnn", "paper_mnist_cnn"):
        for batch in (1, 37, 300):
            wl = W.make_workload(name, batch=batch, seed=batch, bias_scale=0.2)
            _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], f"{name}/B{batch}/fused")
        wl = W.make_workload(name, batch=37, seed=2, bias_scale=0.2)
        _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], f"{name}/B37/layer by layer", options=dict(no_fused_cnn=1))
    # parameters that are not 16-byte aligned: the fused kernel reads weight rows with 16-byte loads, so the step
    # takes the per-layer route
    import torch
    from paper_2010_09063_amd import DpStep
    dev = torch.device("cuda:0")
    wl = W.make_workload("cfg3_small_cnn", batch=9, seed=3, bias_scale=0.2)
    m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    ref = O.dp_step(m, theta, x, y, 0.7, 0.0, 0)
    st = DpStep(m, 9)
    pbuf = torch.zeros(theta.size + 1, device=dev)
    pbuf[1:] = torch.from_numpy(theta).to(dev)
    out = torch.empty(theta.size, device=dev)
    st.dp_step(pbuf[1:], torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev), 9, 0.7, 0.0, 0, out)
    torch.cuda.synchronize()
    tie = TieAwareOracle(m, theta, x, y, ref["pool_margin"])
    csum, _, _ = tie.reference(ref, 0.7, out.cpu().numpy())
    assert_parity(m, out.cpu().numpy(), csum, "cfg3/unaligned parameters", ref["abs_sum"])
    st.dp_step_free()


def test_side_stream_and_validate():
    """A context on a non-default stream (its init-time fills must be ordered before the first step), and the debug
    range check of labels and token ids."""
    import torch
    from paper_2010_09063_amd import DpStep
    dev = torch.device("cuda:0")
    side = torch.cuda.Stream()
    wl = W.make_workload("cfg4_cifar_cnn", batch=4, seed=3, bias_scale=0.2)
    m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    ref = O.dp_step(m, theta, x, y, 0.5, 0.0, 0)
    tp, tx, ty = (torch.from_numpy(a).to(dev) for a in (theta, x, y))
    out = torch.empty(theta.size, device=dev)
    torch.cuda.synchronize()
    st = DpStep(m, 4, stream=side)
    st.dp_step(tp, tx, ty, 4, 0.5, 0.0, 0, out)   # enqueued right after init, on the side stream
    side.synchronize()
    tie = TieAwareOracle(m, theta, x, y, ref["pool_margin"])
    csum, _, _ = tie.reference(ref, 0.5, out.cpu().numpy())
    assert_parity(m, out.cpu().numpy(), csum, "side stream", ref["abs_sum"])
    assert st.dp_step_validate(tx, ty, 4) == 0
    bad_y = ty.clone()
    bad_y[1], bad_y[3] = 10, -1
    assert st.dp_step_validate(tx, bad_y, 4) == 2
    st.dp_step_free()
    wl = W.make_workload("cfg5_lstm", batch=3, seed=3)
    st = DpStep(wl["model"], 3)
    tx, ty = torch.from_numpy(wl["x"]).to(dev), torch.from_numpy(wl["y"]).to(dev)
    assert st.dp_step_validate(tx, ty, 3) == 0
    tx[0, 5], tx[2, 255], tx[1, 0] = 10000, -7, 9999
    ty[0] = 2
    assert st.dp_step_validate(tx, ty, 3) == 3
    assert st.dp_step_validate(None, None, 0) == 0
    st.dp_step_free()


def test_long_sequence_stored_gradients():
    """Sequences of 128 steps and more: the LSTM norm contraction stores each example's gradient and the clipped sum
    is a weighted sum of the rows (both LSTM variants)."""
    rng = np.random.default_rng(10)
    for build in (W.paper_lstm, W.cfg5_lstm):
        m = build(vocab=300, seq_len=140, dim=20, hidden=24)
        x, y = W.make_inputs(m, 7, rng)
        theta = W.init_params(m, rng, bias_scale=0.2) * np.float32(3)
        _check_all_regimes(m, x, y, theta, f"{build.__name__}/T140")


@pytest.mark.parametrize("seq_len", [300, 700, 1024])
def test_long_token_sequences(seq_len):
    """Sequences above 256 and above 512 steps: the per-example sort of the embedding norm holds two or four keys
    per thread (few distinct tokens, so every example has long runs of duplicates to add before squaring)."""
    m = W.cfg6_embedding(vocab=37, seq_len=seq_len, dim=12)
    rng = np.random.default_rng(seq_len)
    x, y = W.make_inputs(m, 9, rng, zipf_exponent=0.7)
    theta = W.init_params(m, rng, bias_scale=0.2) * np.float32(4)
    _check_all_regimes(m, x, y, theta, f"embedding/T{seq_len}")


def test_large_vocabulary_embedding_path():
    """Vocabularies above the LDS-histogram limit take the plain-atomic bucket kernels."""
    m = W.cfg5_lstm(vocab=20000, seq_len=24, dim=20, hidden=33)
    rng = np.random.default_rng(8)
    x, y = W.make_inputs(m, 11, rng)
    theta = W.init_params(m, rng, bias_scale=0.2) * np.float32(3)
    _check_all_regimes(m, x, y, theta, "lstm/V20000/H33")


@pytest.mark.parametrize("build", [W.cfg5_lstm, W.paper_lstm], ids=["last", "seq"])
@pytest.mark.parametrize("hidden", [7, 64, 128])
def test_lstm_hidden_sizes(hidden, build):
    m = build(vocab=50, seq_len=9, dim=12, hidden=hidden)
    rng = np.random.default_rng(hidden)
    x, y = W.make_inputs(m, 5, rng, zipf_exponent=0.5)
    theta = W.init_params(m, rng, bias_scale=0.2) * np.float32(3)
    _check_all_regimes(m, x, y, theta, f"lstm/H{hidden}")


def test_lstm_weight_gradient_routes():
    """The per-example LSTM weight gradient on 16x16 MFMA blocks (one example per two workgroups) at shapes other
    than the benchmark's: one and two column halves, row counts that end inside a block, sequences shorter than one
    chunk of 32 steps, ending inside a chunk, and of several chunks (with and without stored gradients); then the
    benchmark shape on the generic contraction."""
    rng = np.random.default_rng(12)
    for build in (W.cfg5_lstm, W.paper_lstm):
        for dim, hidden, T, batch in ((12, 8, 5, 7), (20, 24, 140, 4), (100, 100, 70, 3), (36, 52, 33, 5), (4, 104, 64, 2)):
            m = build(vocab=60, seq_len=T, dim=dim, hidden=hidden)
            x, y = W.make_inputs(m, batch, rng, zipf_exponent=0.5)
            theta = W.init_params(m, rng, bias_scale=0.2) * np.float32(3)
            _check_all_regimes(m, x, y, theta, f"{build.__name__}/D{dim}/H{hidden}/T{T}")
    wl = W.make_workload("cfg5_lstm", batch=6, seed=2, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg5/generic weight gradient", options=dict(no_lstm_wgrad=1))
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg5/generic projections", options=dict(no_rows_gemm=1))


def test_unaligned_device_pointers():
    """params / x that are not 16-byte aligned fall back to scalar operand staging."""
    import torch
    from paper_2010_09063_amd import DpStep
    for name, batch in (("cfg2_mlp", 33), ("tiny_conv3", 6)):
        if name in TINY:
            m = TINY[name]
            x, y, theta = _case(m, batch, seed=3)
        else:
            wl = W.make_workload(name, batch=batch, seed=3, bias_scale=0.2)
            m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
        ref = O.dp_step(m, theta, x, y, 0.7, 0.0, 0)
        tie = TieAwareOracle(m, theta, x, y, ref["pool_margin"])
        dev = torch.device("cuda:0")
        st = DpStep(m, batch)
        pbuf = torch.zeros(theta.size + 1, device=dev)
        xbuf = torch.zeros(x.size + 1, device=dev)
        pbuf[1:] = torch.from_numpy(theta).to(dev)
        xbuf[1:] = torch.from_numpy(x.reshape(-1)).to(dev)
        tp, tx = pbuf[1:], xbuf[1:]
        assert tp.data_ptr() % 16 != 0 and tx.data_ptr() % 16 != 0
        ty = torch.from_numpy(y).to(dev)
        out = torch.empty(theta.size, device=dev)
        st.dp_step(tp, tx, ty, batch, 0.7, 0.0, 0, out)
        torch.cuda.synchronize()
        csum, _, _ = tie.reference(ref, 0.7, out.cpu().numpy())
        assert_parity(m, out.cpu().numpy(), csum, f"unaligned/{name}", ref["abs_sum"])
        st.dp_step_free()


def test_repeatable_and_profile_hook():
    """Two calls give bit-identical results (fixed reduction order; no float atomics outside the
    embedding's hot tokens), and the per-kernel timing hook reports every launch."""
    import torch
    from paper_2010_09063_amd import DpStep
    wl = W.make_workload("cfg3_small_cnn", batch=64, seed=9)
    m = wl["model"]
    dev = torch.device("cuda:0")
    st = DpStep(m, 64, no_fused_cnn=1)   # layer by layer, so that every kernel kind shows up in the table
    tp = torch.from_numpy(wl["params"]).to(dev)
    tx = torch.from_numpy(wl["x"]).to(dev)
    ty = torch.from_numpy(wl["y"]).to(dev)
    o1 = torch.empty(st.num_params, device=dev)
    o2 = torch.empty(st.num_params, device=dev)
    st.dp_step(tp, tx, ty, 64, 1.0, 1.1, 7, o1)
    st.dp_step_profile(True)
    st.dp_step(tp, tx, ty, 64, 1.0, 1.1, 7, o2)
    rows = st.dp_step_profile_read()
    st.dp_step_profile(False)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2)
    names = {r[0].split("#")[0] for r in rows}
    assert {"conv_fwd", "conv_wgrad_norm", "conv_clipped_sum", "dense_fwd", "clip_factor", "finalize_noise"} <= names
    assert all(r[1] >= 1 and r[2] > 0 for r in rows)
    # a different seed changes the noise, the same seed does not
    st.dp_step(tp, tx, ty, 64, 1.0, 1.1, 8, o2)
    torch.cuda.synchronize()
    assert not torch.equal(o1, o2)
    st.dp_step_free()


@pytest.mark.parametrize("name,batch,opt", [("cfg4_cifar_cnn", None, {}), ("paper_cifar_cnn", None, {}), ("cfg2_mlp", None, {}),
                                            ("cfg1_logistic", None, {}), ("cfg5_lstm", 64, {}), ("wide", 70, dict(no_gram=1, no_minimal_filtering=1)),
                                            ("cfg3_small_cnn", None, {}), ("cfg3_small_cnn", None, dict(no_fused_cnn=1))],
                         ids=["cfg4", "paper_cifar", "cfg2", "cfg1", "cfg5-dense-tensors", "wide-ws", "cfg3", "cfg3-layerwise"])
def test_bit_identical_repeats_at_full_batch(name, batch, opt):
    """Every reduction of the step runs in a fixed order: two steps on the same inputs agree bit for bit, at the
    benchmark batch (the embedding tensor excepted: the chunks of a hot token meet through fp32 atomics)."""
    import torch
    from paper_2010_09063_amd import DpStep
    dev = torch.device("cuda:0")
    if name == "wide":
        m = _wide_conv_net()
        x, y, theta = _case(m, batch, seed=3)
    else:
        wl = W.make_workload(name, batch=batch, seed=0)
        m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    B = len(y)
    st = DpStep(m, B, **opt)
    tp, tx, ty = (torch.from_numpy(a).to(dev) for a in (theta, x, y))
    outs = []
    for rep in range(3):
        o = torch.empty(st.num_params, device=dev)
        st.dp_step(tp, tx, ty, B, 1.0, 1.1, 5, o)
        outs.append(o)
    torch.cuda.synchronize()
    lo = 0
    for li, tname, shp, off in W.param_tensors(m):
        n = int(np.prod(shp))
        if tname != "E":
            assert torch.equal(outs[0][off:off + n], outs[1][off:off + n]) and torch.equal(outs[0][off:off + n], outs[2][off:off + n]), (name, li, tname)
    st.dp_step_free()


@pytest.mark.gpu
@pytest.mark.parametrize("name,batch", [("tiny_dense", 9), ("tiny_conv3", 5), ("tiny_lstm", 4), ("tiny_emb", 7),
                                        ("tiny_lstm_seq", 6), ("tiny_avgpool", 8), ("cfg3_small_cnn", 33)])
def test_fused_sgd_update(name, batch):
    """dp_step_sgd: the update of Section 1 item 4 fused into the final write, against the oracle's step."""
    import torch
    from paper_2010_09063_amd import DpStep
    if name in TINY:
        m = TINY[name]
        x, y, theta = _case(m, batch, seed=21)
    else:
        wl = W.make_workload(name, batch=batch, seed=21, bias_scale=0.2)
        m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    norms = O.dp_step(m, theta, x, y, 1.0, 0.0, 0)["norms"]
    # a step small enough that the parameters stay in the regime they were drawn for (a large one saturates every
    # tanh, and a saturated plane is one big near-tie for the pool that follows it)
    Cc, sigma, seed = float(np.median(norms)), 0.7, 77
    lr = 0.01 * batch / Cc

    def want_after(th, sd, noised_sum):
        """The oracle's updated parameters; where the GPU routed a near-tied pool window to the runner-up, the
        oracle's aggregate under that (equally valid) routing takes the place of the first-maximum one."""
        want = O.sgd_step(m, th, x, y, Cc, sigma, sd, lr).astype(np.float64)
        ref = O.dp_step(m, th, x, y, Cc, 0.0, 0)
        tie = TieAwareOracle(m, th, x, y, ref["pool_margin"])
        if tie.n_near:
            z = O.noise(sd, th.size)
            csum, _, flips = tie.reference(ref, Cc, noised_sum - sigma * Cc * z)
            want = want - lr / batch * (csum - ref["clipped_sum"])
        return want

    dev = torch.device("cuda:0")
    st = DpStep(m, batch)
    tp = torch.from_numpy(theta.copy()).to(dev)
    tx, ty = torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev)
    out = torch.empty(st.num_params, dtype=torch.float32, device=dev)
    st.dp_step_sgd(tp, tx, ty, batch, Cc, sigma, seed, lr, out)
    torch.cuda.synchronize()
    got, g = tp.cpu().numpy(), out.cpu().numpy()
    want = want_after(theta, seed, g.astype(np.float64))
    upd_got, upd_want = got.astype(np.float64) - theta, want - theta
    print(f"{name}: update rel_l2 {rel_l2(upd_got, upd_want):.2e}", flush=True)
    assert rel_l2(g, -upd_want * batch / lr) <= 2e-4   # the noised sum is still delivered
    assert rel_l2(upd_got, upd_want) <= 2e-4          # fp32 subtraction on top of the 1e-4 bar of the sum
    # a second call without out_grad continues from the updated parameters
    st.dp_step_sgd(tp, tx, ty, batch, Cc, sigma, seed + 1, lr)
    torch.cuda.synchronize()
    got2 = tp.cpu().numpy().astype(np.float64)
    want2 = want_after(got, seed + 1, (got - got2) * batch / lr)
    assert rel_l2(got2 - got, want2 - got) <= 2e-4
    st.dp_step_free()


def test_minibatch_draw_is_bit_exact():
    """dp_step_sample_indices against the oracle's draw: integer work, compared bit for bit."""
    import torch
    from paper_2010_09063_amd import dp_step_sample_indices
    dev = torch.device("cuda:0")
    for seed, n, batch in ((0, 60000, 1024), (0x1234567887654321, 2**31 - 1, 777), (5, 1, 6), (7, 3, 1), (9, 50000, 0)):
        idx = torch.full((max(batch, 1),), -1, dtype=torch.int32, device=dev)
        dp_step_sample_indices(seed, n, batch, idx)
        torch.cuda.synchronize()
        assert np.array_equal(idx.cpu().numpy()[:batch], O.sample_indices(seed, n, batch))


@pytest.mark.parametrize("name,n,batch,steps", [("tiny_dense", 50, 8, 4), ("tiny_lstm", 30, 5, 3), ("tiny_emb", 40, 7, 3),
                                                ("tiny_avgpool", 30, 6, 3), ("cfg1_logistic", 300, 64, 5),
                                                ("cfg2_mlp", 200, 33, 3)])
def test_training_loop(name, n, batch, steps):
    """dp_step_loop: draw, private step and update, `steps` times with no host work in between, against the oracle's
    loop (models without max-pools, so every step has one valid result)."""
    import torch
    from paper_2010_09063_amd import DpStep
    if name in TINY:
        m = TINY[name]
        x, y, theta = _case(m, n, seed=31, scale=4.0 if m["input"]["kind"] == "tokens" else 1.0)
    else:
        wl = W.make_workload(name, batch=n, seed=31, bias_scale=0.2)
        m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    norms = O.dp_step(m, theta, x, y, 1.0, 0.0, 0)["norms"]
    Cc, sigma, seed0 = float(np.median(norms)), 0.7, 2**33 + 5
    lr = 0.02 * batch / Cc
    want = O.train(m, theta, x, y, steps, batch, Cc, sigma, seed0, lr).astype(np.float64)
    dev = torch.device("cuda:0")
    st = DpStep(m, batch)
    tp = torch.from_numpy(theta.copy()).to(dev)
    tx, ty = torch.from_numpy(x).to(dev), torch.from_numpy(y).to(dev)
    st.dp_step_loop(tp, tx, ty, n, steps, batch, Cc, sigma, seed0, lr)
    torch.cuda.synchronize()
    got = tp.cpu().numpy().astype(np.float64)
    err = rel_l2(got - theta, want - theta)
    print(f"{name}: {steps} steps, total update rel_l2 {err:.2e}", flush=True)
    assert err <= 3e-4   # every step within the 1e-4 bar of its own sum, carried through the following steps
    # the loop is dp_step_sgd on the drawn examples: one more step by hand from where the loop stopped
    idx = O.sample_indices(seed0 + steps, n, batch)
    nxt = O.sgd_step(m, got.astype(np.float32), x[idx], y[idx], Cc, sigma, seed0 + steps, lr).astype(np.float64)
    st.dp_step_loop(tp, tx, ty, n, 1, batch, Cc, sigma, seed0 + steps, lr)
    torch.cuda.synchronize()
    assert rel_l2(tp.cpu().numpy().astype(np.float64) - got, nxt - got) <= 2e-4
    st.dp_step_free()
