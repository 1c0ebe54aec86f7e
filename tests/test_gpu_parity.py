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


def _check_all_regimes(m, x, y, theta, label, stepper=None):
    """Whole batch, every parameter tensor, every per-example norm, in the three clipping regimes and for the
    non-private sum (max-pool windows tied at rounding level: see tests/gpu_util.py)."""
    ref_inf = O.dp_step(m, theta, x, y, math.inf, 0.0, 0)
    tie = TieAwareOracle(m, theta, x, y, ref_inf["pool_margin"])
    n0 = ref_inf["norms"]
    regimes = [math.inf, float(np.median(n0)), 0.1 * float(n0.min())]
    for Cc in regimes:
        ref = ref_inf if math.isinf(Cc) else O.dp_step(m, theta, x, y, Cc, 0.0, 0)
        out, gn, norms = check_step(m, theta, x, y, Cc, ref, f"{label} C={Cc:.4g}", tie=tie, stepper=stepper)
        if not math.isinf(Cc):
            s = np.minimum(1.0, Cc / gn.astype(np.float64))
            assert np.all(s * norms <= Cc * (1 + 1e-5))
    ref_np = O.dp_step(m, theta, x, y, 1.0, 0.0, 0, clip=False)
    check_step(m, theta, x, y, 1.0, ref_np, f"{label} non-private", tie=tie, private=False, stepper=stepper)


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


def test_context_reuse_with_minimal_filtering_kernels(monkeypatch):
    """One context planned for the largest batch serves smaller ones: the minimal-filtering kernels (forward,
    backward-data with the pool in the epilogue, weight gradients) size their grids and split counts from the batch
    of the call, the plan from the batch of the context."""
    from paper_2010_09063_amd import DpStep
    monkeypatch.setenv("DP_STEP_WINO_ALL", "1")
    m = W.model(W.image_input(32, 16, 16), [
        W.conv2d(32, 32, 3, stride=1, pad=1, act="tanh"), W.conv2d(32, 64, 3, stride=1, pad=1, act="tanh"),
        W.maxpool2d(2, 2), W.conv2d(64, 64, 3, stride=1, pad=1, act="relu"), W.avgpool2d(2, 2),
        W.dense(64 * 4 * 4, 3)], 3)
    st = DpStep(m, 9)
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


def test_generic_convolution_path_matches_too(monkeypatch):
    """DP_STEP_GENERIC_CONV=1 keeps 3x3 stride-1 convolutions on the functor contraction
    (the path every other kernel size / stride takes)."""
    monkeypatch.setenv("DP_STEP_GENERIC_CONV", "1")
    m = TINY["tiny_conv3"]
    x, y, theta = _case(m, 9, seed=21)
    _check_all_regimes(m, x, y, theta, "tiny_conv3/generic")
    wl = W.make_workload("cfg4_cifar_cnn", batch=3, seed=4, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/generic")


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


def test_recompute_routes_match_too(monkeypatch):
    """With the Gram norms, the stored-gradient route and the column route of strided backward-data switched off,
    the library takes the routes it otherwise keeps for shapes those do not cover (direct per-example contraction
    for the norm, a second contraction for the clipped sum, the gathering backward-data contraction)."""
    monkeypatch.setenv("DP_STEP_NO_GRAM", "1")
    monkeypatch.setenv("DP_STEP_NO_GSTORE", "1")
    monkeypatch.setenv("DP_STEP_NO_COLS", "1")
    for name, batch in (("tiny_conv_gram", 9), ("tiny_conv_store", 6), ("tiny_conv_stride", 11), ("tiny_lstm_seq", 5)):
        m = TINY[name]
        x, y, theta = _case(m, batch, seed=41, scale=4.0 if m["input"]["kind"] == "tokens" else 1.0)
        _check_all_regimes(m, x, y, theta, f"{name}/recompute")
    wl = W.make_workload("cfg4_cifar_cnn", batch=3, seed=4, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/recompute")
    m = W.paper_lstm(vocab=300, seq_len=140, dim=20, hidden=24)  # 140 steps: above the stored-gradient threshold
    rng = np.random.default_rng(9)
    x, y = W.make_inputs(m, 4, rng)
    theta = W.init_params(m, rng, bias_scale=0.2) * np.float32(3)
    _check_all_regimes(m, x, y, theta, "lstm_seq/T140/recompute")


def test_minimal_filtering_route(monkeypatch):
    """Forward and backward-data of the pad-1 3x3 convolutions through the F(2x2, 3x3) kernel at sizes the oracle
    covers element by element (the library keeps that kernel for launches that fill the chip; here it is forced):
    4x4, 8x8 and 16x16 planes, channel counts that are no multiples of the 8-channel chunk or of the 32 / 64 output
    channels of a workgroup, more than 64 output channels (several channel blocks), batches that end inside a
    workgroup's 32 tiles, a 3-channel first layer.  (The full-size cases run it wherever the library selects it.)
    The benchmark-shaped cases also take the weight-gradient kernels of the same family: per-example norm pass with
    stored gradients on 16- and 32-wide planes, clipped sums on 8x8 planes, and the batch sums of the non-private
    step; the last part switches the whole family off at full batch."""
    cases = (("tiny_conv_gram", 9), ("tiny_conv_store", 6), ("tiny_conv_wide", 13), ("tiny_conv_wide", 1))
    monkeypatch.setenv("DP_STEP_WINO_ALL", "1")
    for name, batch in cases:
        m = TINY[name]
        x, y, theta = _case(m, batch, seed=43)
        _check_all_regimes(m, x, y, theta, f"{name}/minimal-filtering")
    # 32x32 planes with 64 output channels per workgroup, forward (8 -> 40) and backward-data (16 -> 40)
    m = W.model(W.image_input(8, 32, 32), [
        W.conv2d(8, 40, 3, stride=1, pad=1, act="tanh"), W.conv2d(40, 16, 3, stride=1, pad=1, act="tanh"),
        W.avgpool2d(8, 8), W.dense(16 * 4 * 4, 3)], 3)
    x, y, theta = _case(m, 3, seed=44)
    _check_all_regimes(m, x, y, theta, "planes32/minimal-filtering")
    wl = W.make_workload("cfg4_cifar_cnn", batch=3, seed=4, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "cfg4/minimal-filtering")
    wl = W.make_workload("paper_cifar_cnn", batch=5, seed=6, bias_scale=0.2)
    _check_all_regimes(wl["model"], wl["x"], wl["y"], wl["params"], "paper_cifar/minimal-filtering")
    # full batch with that route switched off: the direct kernels in the launch shapes of the benchmark batch
    monkeypatch.delenv("DP_STEP_WINO_ALL")
    monkeypatch.setenv("DP_STEP_NO_WINO", "1")
    wl = W.make_workload("cfg4_cifar_cnn", seed=0)
    m, x, y, theta = wl["model"], wl["x"], wl["y"], wl["params"]
    ref = O.dp_step(m, theta, x, y, wl["C"], 0.0, 0)
    check_step(m, theta, x, y, wl["C"], ref, "cfg4 full batch, direct kernels")


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


def test_weight_gradients_direct_kernels_on_the_same_network(monkeypatch):
    monkeypatch.setenv("DP_STEP_NO_WINO_WG", "1")
    m = W.model(W.image_input(32, 16, 16), [
        W.conv2d(32, 32, 3, stride=1, pad=1, act="tanh"), W.conv2d(32, 64, 3, stride=1, pad=1, act="tanh"),
        W.maxpool2d(2, 2), W.conv2d(64, 64, 3, stride=1, pad=1, act="relu"), W.avgpool2d(2, 2),
        W.dense(64 * 4 * 4, 3)], 3)
    x, y, theta = _case(m, 5, seed=46)
    _check_all_regimes(m, x, y, theta, "planes16x16+8x8/direct weight gradients")


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
    st = DpStep(m, 64)
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
