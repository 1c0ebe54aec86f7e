"""Pins for the CPU oracle: every check here is against something other than the
oracle itself -- published known answers, finite differences, PyTorch-CPU autograd,
closed forms and invariants of the method (paper, Section 1, DPSGD items 2-3)."""
import math
import os

import numpy as np
import pytest

import dp_workloads as W
from oracle import dpsgd_oracle as O
from tests import torch_ref as TR

GOLD = os.path.join(os.path.dirname(__file__), "golden")
TINY = W.tiny_models()


def _tiny_case(name, batch, seed=3, bias=0.3):
    m = TINY[name]
    rng = np.random.default_rng(seed)
    x, y = W.make_inputs(m, batch, rng, x_dist="normal" if m["input"]["kind"] == "image" else "uniform",
                         zipf_exponent=0.3)
    theta = W.init_params(m, rng, bias_scale=bias)
    if m["input"]["kind"] == "tokens":  # larger embeddings so that the LSTM is not near-linear
        theta = theta * 4
    return m, x, y, theta


# ----------------------------------------------------------------- architecture wiring

def test_param_counts():
    # 26,010 and the LSTM formula are the counts the paper prints (Section 3, architectures paragraph).
    assert O.num_params(W.cfg1_logistic()) == 7850
    assert O.num_params(W.cfg2_mlp()) == 407050
    assert O.num_params(W.cfg3_small_cnn()) == 26010
    assert O.num_params(W.cfg4_cifar_cnn()) == 550570
    assert O.num_params(W.cfg5_lstm()) == 1080602
    assert O.num_params(W.cfg5_lstm(vocab=10004)) == 1081002
    for name, m in list(TINY.items()):
        assert O.num_params(m) == W.num_params(m)


# ----------------------------------------------------------------- Philox and the normal transform

def test_philox_known_answers():
    n = 0
    for line in open(os.path.join(GOLD, "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(t, 16) for t in line.split()]
        out = O.philox4x32_10(v[:4], v[4:6])
        assert [int(o) for o in out] == v[6:]
        n += 1
    assert n == 3


def test_philox_python_bigint_twin():
    # second, independently written implementation (Python integers)
    def ref(ctr, key):
        c, k = list(ctr), list(key)
        for _ in range(10):
            p0, p1 = 0xD2511F53 * c[0], 0xCD9E8D57 * c[2]
            c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & 0xFFFFFFFF, (p0 >> 32) ^ c[3] ^ k[1], p0 & 0xFFFFFFFF]
            k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
        return c
    rng = np.random.default_rng(0)
    for _ in range(200):
        ctr = [int(v) for v in rng.integers(0, 2**32, size=4)]
        key = [int(v) for v in rng.integers(0, 2**32, size=2)]
        assert [int(o) for o in O.philox4x32_10(ctr, key)] == ref(ctr, key)


def test_noise_layout_matches_philox_blocks():
    # coordinate j uses block j // 4, key = (seed lo, seed hi), counter = (block, 0, 0, 0)
    seed = (0x12345678 << 32) | 0x9ABCDEF0
    z = O.noise(seed, 11)
    for blk in range(3):
        r = O.philox4x32_10([blk, 0, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        u = [((int(v) >> 9) + 0.5) / 2**23 for v in r]
        exp = [math.sqrt(-2 * math.log(u[0])) * math.cos(2 * math.pi * u[1]),
               math.sqrt(-2 * math.log(u[0])) * math.sin(2 * math.pi * u[1]),
               math.sqrt(-2 * math.log(u[2])) * math.cos(2 * math.pi * u[3]),
               math.sqrt(-2 * math.log(u[2])) * math.sin(2 * math.pi * u[3])]
        for q in range(4):
            j = blk * 4 + q
            if j < 11:
                assert abs(z[j] - exp[q]) < 1e-12


def test_noise_is_standard_normal():
    from scipy import stats
    n = 4_000_000
    z = O.noise(7, n)
    assert abs(z.mean()) < 4 / math.sqrt(n)
    assert abs(z.var() - 1) < 0.01
    assert np.abs(z).max() <= math.sqrt(2 * 24 * math.log(2)) + 1e-9  # smallest uniform is 2^-24
    assert abs(np.corrcoef(z[:-1], z[1:])[0, 1]) < 4 / math.sqrt(n)
    ks = stats.kstest(z[:500_000], "norm")
    assert ks.pvalue > 1e-3
    # streams of different seeds are different, same seed is reproducible
    assert np.array_equal(O.noise(7, 64), z[:64])
    assert not np.allclose(O.noise(8, 64), z[:64])


# ----------------------------------------------------------------- per-example gradients

@pytest.mark.parametrize("name", sorted(TINY))
def test_gradient_vs_finite_differences(name):
    m, x, y, theta = _tiny_case(name, 3)
    th = theta.astype(np.float64)
    for i in range(x.shape[0]):
        _, g, _ = O.example_grad(m, th, x[i], y[i])
        # every coordinate of small models; for larger ones a seeded sample that covers every tensor
        if th.size <= 400:
            idx = np.arange(th.size)
        else:
            rs = np.random.default_rng(i)
            idx = np.unique(np.concatenate(
                [off + rs.integers(0, int(np.prod(shp)), size=24) for _, _, shp, off in W.param_tensors(m)]))
        num = np.zeros(idx.size)
        eps = 1e-6
        for k, j in enumerate(idx):
            tp, tm = th.copy(), th.copy()
            tp[j] += eps
            tm[j] -= eps
            num[k] = (O.example_loss(m, tp, x[i], y[i]) - O.example_loss(m, tm, x[i], y[i])) / (2 * eps)
        assert np.linalg.norm(g[idx] - num) <= 1e-6 * max(1.0, np.linalg.norm(num)), name
        assert np.linalg.norm(g) > 0


@pytest.mark.parametrize("name", sorted(TINY))
def test_gradient_vs_torch_autograd_tiny(name):
    m, x, y, theta = _tiny_case(name, 4)
    th = theta.astype(np.float64)
    G = TR.per_example_grads(m, th, x, y)
    for i in range(x.shape[0]):
        _, g, _ = O.example_grad(m, th, x[i], y[i])
        assert np.linalg.norm(g - G[i]) <= 1e-10 * max(1.0, np.linalg.norm(G[i]))


def _reduced(name):
    """The five benchmark architectures at their real layer shapes, small batch
    (the LSTM with a shorter sequence so that the loop oracle stays fast)."""
    if name in ("cfg5_lstm", "paper_lstm"):
        m = (W.cfg5_lstm if name == "cfg5_lstm" else W.paper_lstm)(vocab=300, seq_len=12, dim=100, hidden=100)
        rng = np.random.default_rng(1)
        x, y = W.make_inputs(m, 3, rng)
        theta = W.init_params(m, rng, bias_scale=0.2)
        return m, x, y, theta
    wl = W.make_workload(name, batch=3, seed=1, bias_scale=0.2)
    return wl["model"], wl["x"], wl["y"], wl["params"]


@pytest.mark.parametrize("name", sorted(W.CONFIGS))
def test_gradient_vs_torch_autograd_benchmark_shapes(name):
    m, x, y, theta = _reduced(name)
    th = theta.astype(np.float64)
    G = TR.per_example_grads(m, th, x, y)
    for i in range(x.shape[0]):
        _, g, ties = O.example_grad(m, th, x[i], y[i])
        # max-pool windows of ReLU outputs tie at 0, where ReLU'(0) = 0 stops the gradient whichever element wins
        assert ties == 0 or name == "paper_mnist_cnn"
        assert np.linalg.norm(g - G[i]) <= 1e-10 * max(1.0, np.linalg.norm(G[i]))


# ----------------------------------------------------------------- the step

@pytest.mark.parametrize("name", sorted(TINY))
def test_no_clip_no_noise_is_the_summed_gradient(name):
    m, x, y, theta = _tiny_case(name, 6)
    r = O.dp_step(m, theta, x, y, math.inf, 0.0, 0)
    ref = TR.summed_grad(m, theta.astype(np.float64), x, y)
    assert np.linalg.norm(r["clipped_sum"] - ref) <= 1e-10 * np.linalg.norm(ref)
    assert np.array_equal(r["out"], r["clipped_sum"].astype(np.float32))
    # the non-private switch gives the same thing even with a tiny C
    r2 = O.dp_step(m, theta, x, y, 1e-3, 0.0, 0, clip=False)
    assert np.array_equal(r2["out"], r["out"])


@pytest.mark.parametrize("name", sorted(TINY))
def test_batch_of_one_is_a_single_clipped_gradient(name):
    m, x, y, theta = _tiny_case(name, 1)
    G = TR.per_example_grads(m, theta.astype(np.float64), x, y)[0]
    n = np.linalg.norm(G)
    for Cc in (0.5 * n, 2.0 * n):
        r = O.dp_step(m, theta, x, y, Cc, 0.0, 0)
        exp = G * min(1.0, Cc / n)
        assert np.linalg.norm(r["clipped_sum"] - exp) <= 1e-10 * np.linalg.norm(exp)
        assert abs(r["norms"][0] - n) <= 1e-10 * n


@pytest.mark.parametrize("name", sorted(TINY))
def test_clip_invariants(name):
    m, x, y, theta = _tiny_case(name, 8)
    B = x.shape[0]
    G = TR.per_example_grads(m, theta.astype(np.float64), x, y)
    norms = np.linalg.norm(G, axis=1)
    r0 = O.dp_step(m, theta, x, y, math.inf, 0.0, 0)
    assert np.allclose(r0["norms"], norms, rtol=1e-10)
    # (a) each clipped gradient has norm <= C; (b) the whole sum has norm <= B*C
    Cmed = float(np.median(norms))
    r = O.dp_step(m, theta, x, y, Cmed, 0.0, 0)
    s = np.minimum(1.0, Cmed / norms)
    assert np.all(np.linalg.norm(G * s[:, None], axis=1) <= Cmed * (1 + 1e-12))
    assert np.linalg.norm(r["clipped_sum"]) <= B * Cmed * (1 + 1e-12)
    exp = (G * s[:, None]).sum(0)
    assert np.linalg.norm(r["clipped_sum"] - exp) <= 1e-10 * np.linalg.norm(exp)
    assert (s < 1).any() and (s == 1).any()
    # (c) C above every norm: nothing is clipped
    r = O.dp_step(m, theta, x, y, float(norms.max()) * 1.01, 0.0, 0)
    assert np.allclose(r["clipped_sum"], r0["clipped_sum"], rtol=1e-12, atol=0)
    # (d) C below every norm: the result is linear in C
    Clow = 0.1 * float(norms.min())
    ra = O.dp_step(m, theta, x, y, Clow, 0.0, 0)["clipped_sum"]
    rb = O.dp_step(m, theta, x, y, 2 * Clow, 0.0, 0)["clipped_sum"]
    assert np.linalg.norm(rb - 2 * ra) <= 1e-12 * np.linalg.norm(rb)


def test_batch_order_invariance_and_thread_count():
    m, x, y, theta = _tiny_case("tiny_conv2", 9)
    perm = np.random.default_rng(0).permutation(9)
    a = O.dp_step(m, theta, x, y, 0.7, 0.0, 0, n_threads=1)["clipped_sum"]
    b = O.dp_step(m, theta, x[perm], y[perm], 0.7, 0.0, 0, n_threads=3)["clipped_sum"]
    assert np.linalg.norm(a - b) <= 1e-12 * np.linalg.norm(a)


def test_noise_term_of_the_step():
    m, x, y, theta = _tiny_case("tiny_dense", 5)
    P = theta.size
    seed, Cc, sigma = 1234567890123, 0.8, 1.1
    r0 = O.dp_step(m, theta, x, y, Cc, 0.0, seed)
    r1 = O.dp_step(m, theta, x, y, Cc, sigma, seed)
    z = O.noise(seed, P)
    exp = (r0["clipped_sum"] + sigma * Cc * z).astype(np.float32)
    assert np.array_equal(r1["out"], exp)
    # empty batch: pure noise
    r2 = O.dp_step(m, theta, x[:0], y[:0], Cc, sigma, seed)
    assert np.array_equal(r2["out"], (sigma * Cc * z).astype(np.float32))


def test_logistic_closed_form():
    # W = 0, b = 0: softmax is uniform, delta = 1/10 - onehot, ||delta||^2 = 0.9,
    # ||g_i|| = sqrt(0.9 (||x_i||^2 + 1)) and the step is sum_i (C/||g_i||) [x_i; 1] (x) delta_i.
    wl = W.make_workload("cfg1_logistic", batch=16, seed=5)
    m, x, y = wl["model"], wl["x"].reshape(16, 784), wl["y"]
    theta = np.zeros(7850, dtype=np.float32)
    r = O.dp_step(m, theta, x, y, 1.0, 0.0, 0)
    xd = x.astype(np.float64)
    delta = np.full((16, 10), 0.1)
    delta[np.arange(16), y] -= 1.0
    n = np.sqrt(0.9 * ((xd ** 2).sum(1) + 1))
    assert np.allclose(r["norms"], n, rtol=1e-12)
    s = np.minimum(1.0, 1.0 / n)
    gW = np.einsum("bi,bo->io", xd * s[:, None], delta)
    gb = (delta * s[:, None]).sum(0)
    exp = np.concatenate([gW.ravel(), gb])
    assert np.linalg.norm(r["clipped_sum"] - exp) <= 1e-12 * np.linalg.norm(exp)


def test_dense_norm_identity():
    # Section 1 (per-example norms for fully-connected layers): ||a (x) delta||_F = ||a|| ||delta||.
    m, x, y, theta = _tiny_case("tiny_dense_tanh", 4)
    th = theta.astype(np.float64)
    for i in range(4):
        _, g, _ = O.example_grad(m, th, x[i], y[i])
        total = 0.0
        acts = [x[i].reshape(-1).astype(np.float64)]
        # recompute activations with numpy to get ||a|| for each layer
        for li, name, shp, off in W.param_tensors(m):
            if name == "W":
                Wm = th[off:off + shp[0] * shp[1]].reshape(shp)
                b = th[off + shp[0] * shp[1]: off + shp[0] * shp[1] + shp[1]]
                z = acts[-1] @ Wm + b
                act = m["layers"][li]["act"]
                acts.append(np.tanh(z) if act == "tanh" else np.maximum(z, 0) if act == "relu" else z)
                gW = g[off:off + shp[0] * shp[1]]
                gb = g[off + shp[0] * shp[1]: off + shp[0] * shp[1] + shp[1]]
                # delta is the bias gradient
                assert abs(np.linalg.norm(gW) - np.linalg.norm(acts[-2]) * np.linalg.norm(gb)) <= 1e-12
                total += (np.linalg.norm(acts[-2]) ** 2 + 1) * np.linalg.norm(gb) ** 2
        assert abs(math.sqrt(total) - np.linalg.norm(g)) <= 1e-12


def test_embedding_duplicates_are_summed_before_the_norm():
    m = TINY["tiny_lstm"]
    rng = np.random.default_rng(2)
    theta = (W.init_params(m, rng, bias_scale=0.3) * 4).astype(np.float64)
    E = 7 * 3
    x_same = np.full(5, 2, dtype=np.int32)
    _, g, _ = O.example_grad(m, theta, x_same, 1)
    gE = g[:E].reshape(7, 3)
    assert np.count_nonzero(np.abs(gE).sum(1)) == 1          # one row holds the sum over all steps
    x_distinct = np.array([0, 1, 2, 3, 4], dtype=np.int32)
    _, g2, _ = O.example_grad(m, theta, x_distinct, 1)
    assert np.count_nonzero(np.abs(g2[:E].reshape(7, 3)).sum(1)) == 5
    G = TR.per_example_grads(m, theta, np.stack([x_same, x_distinct]), np.array([1, 1]))
    assert np.allclose(G[0], g, atol=1e-12) and np.allclose(G[1], g2, atol=1e-12)


def test_embedding_mean_pool_norm_closed_form():
    """Embedding network (Appendix B): with a mean over T steps every step receives g/T, so row v of the embedding
    gradient is (count_v / T) g and its squared norm sum_v (count_v / T)^2 |g|^2, whatever the classifier does."""
    m = W.model(W.token_input(9), [W.embedding(6, 4), W.seq_mean(), W.dense(4, 3)], 3)
    rng = np.random.default_rng(3)
    theta = W.init_params(m, rng, bias_scale=0.3).astype(np.float64)
    tok = np.array([0, 2, 2, 5, 2, 0, 1, 5, 5], dtype=np.int32)
    _, g, _ = O.example_grad(m, theta, tok, 1)
    gE = g[:24].reshape(6, 4)
    counts = np.bincount(tok, minlength=6).astype(np.float64)
    # rows are parallel to one vector u = g_pooled / T: recover it from the row of token 1 (count 1)
    u = gE[1]
    assert np.allclose(gE, counts[:, None] * u[None, :], rtol=1e-12, atol=1e-15)
    assert np.isclose((gE ** 2).sum(), (counts ** 2).sum() * (u ** 2).sum(), rtol=1e-12)
    # and u is W delta / T with delta = softmax - onehot of the classifier on the mean embedding
    E, Wd, bd = theta[:24].reshape(6, 4), theta[24:36].reshape(4, 3), theta[36:39]
    z = E[tok].mean(axis=0) @ Wd + bd
    p = np.exp(z - z.max()); p /= p.sum()
    delta = p - np.eye(3)[1]
    assert np.allclose(u, Wd @ delta / 9.0, rtol=1e-12, atol=1e-15)


def test_global_average_pool_closed_form():
    """CIFAR10 network's last two layers (Appendix B): a 1x1 convolution followed by a global average pool is a
    linear classifier on the plane-mean of the input, so dL/dW = (softmax - onehot) outer mean_p x and
    dL/db = softmax - onehot."""
    m = W.model(W.image_input(3, 4, 4), [W.conv2d(3, 4, 1), W.avgpool2d(4, 4)], 4)
    rng = np.random.default_rng(5)
    theta = W.init_params(m, rng, bias_scale=0.3).astype(np.float64)
    x = rng.standard_normal((3, 4, 4))
    _, g, _ = O.example_grad(m, theta, x.astype(np.float32), 2)
    x = x.astype(np.float32).astype(np.float64)
    Wc, b = theta[:12].reshape(4, 3), theta[12:16]
    xm = x.mean(axis=(1, 2))
    z = Wc @ xm + b
    p = np.exp(z - z.max()); p /= p.sum()
    delta = p - np.eye(4)[2]
    assert np.allclose(g[:12].reshape(4, 3), np.outer(delta, xm), rtol=1e-12, atol=1e-15)
    assert np.allclose(g[12:16], delta, rtol=1e-12, atol=1e-15)


def test_conv_norm_from_gram_matrices():
    """Squared norm of a convolution's per-example gradient from two P x P Gram matrices:
    ||sum_p delta_p (x) patch_p||^2 + ||sum_p delta_p||^2 = sum_{p,q} (delta_p . delta_q)(patch_p . patch_q + 1).
    With one 3x3 / pad-1 convolution under a global average pool, delta_p = (softmax - onehot) / P for every
    pixel, so the right-hand side needs only numpy's im2col of the input."""
    Cin, D, Hh = 3, 4, 4
    m = W.model(W.image_input(Cin, Hh, Hh), [W.conv2d(Cin, D, 3, stride=1, pad=1), W.avgpool2d(Hh, Hh)], D)
    rng = np.random.default_rng(12)
    theta = W.init_params(m, rng, bias_scale=0.3).astype(np.float64)
    x = rng.standard_normal((Cin, Hh, Hh)).astype(np.float32)
    _, g, _ = O.example_grad(m, theta, x, 1)
    xp = np.pad(x.astype(np.float64), ((0, 0), (1, 1), (1, 1)))
    patches = np.stack([xp[:, i:i + 3, j:j + 3].reshape(-1) for i in range(Hh) for j in range(Hh)])  # [P, 9C]
    Wc, b = theta[:D * Cin * 9].reshape(D, Cin * 9), theta[D * Cin * 9:]
    z = (patches @ Wc.T + b).mean(axis=0)
    p = np.exp(z - z.max()); p /= p.sum()
    delta = np.tile((p - np.eye(D)[1]) / (Hh * Hh), (Hh * Hh, 1))                                      # [P, D]
    Gx, Gd = patches @ patches.T, delta @ delta.T
    assert np.isclose((g ** 2).sum(), (Gd * (Gx + 1.0)).sum(), rtol=1e-12)
    # and the gradient itself, for good measure
    assert np.allclose(g[:D * Cin * 9].reshape(D, Cin * 9), delta.T @ patches, rtol=1e-11, atol=1e-14)


def test_average_pool_spreads_the_gradient_evenly():
    """An average pool with window k and stride k followed by a dense layer: every input pixel of a window gets
    1/k^2 of that window's gradient, so the first layer's bias gradient (sum over pixels of the backpropagated
    signal, identity activation) equals the per-channel sum of the pooled gradient."""
    m = W.model(W.image_input(1, 4, 4), [W.conv2d(1, 2, 1), W.avgpool2d(2, 2), W.dense(8, 3)], 3)
    rng = np.random.default_rng(6)
    theta = W.init_params(m, rng, bias_scale=0.3).astype(np.float64)
    x = rng.random((1, 4, 4)).astype(np.float32)
    _, g, _ = O.example_grad(m, theta, x, 0)
    Wc, bc = theta[0:2], theta[2:4]
    Wd, bd = theta[4:28].reshape(8, 3), theta[28:31]
    a = Wc[:, None, None] * x.astype(np.float64) + bc[:, None, None]              # [2,4,4]
    pooled = a.reshape(2, 2, 2, 2, 2).mean(axis=(2, 4))                           # [2,2,2]
    z = pooled.reshape(-1) @ Wd + bd
    p = np.exp(z - z.max()); p /= p.sum()
    delta = p - np.eye(3)[0]
    dpool = (Wd @ delta).reshape(2, 2, 2)
    assert np.allclose(g[2:4], dpool.sum(axis=(1, 2)), rtol=1e-12, atol=1e-15)
    # weight of the 1x1 convolution: sum_p x_p * dpool[window(p)] / 4
    up = np.repeat(np.repeat(dpool, 2, axis=1), 2, axis=2) / 4.0
    assert np.allclose(g[0:2], (up * x.astype(np.float64)).sum(axis=(1, 2)), rtol=1e-12, atol=1e-15)


def test_lstm_sequence_output_of_one_step_is_the_last_state():
    """With T = 1 the sequence output followed by the mean over steps is the last-state LSTM."""
    rng = np.random.default_rng(8)
    m_seq = W.model(W.token_input(1), [W.embedding(5, 3), W.lstm_seq(3, 4), W.seq_mean(), W.dense(4, 2)], 2)
    m_last = W.model(W.token_input(1), [W.embedding(5, 3), W.lstm_last(3, 4), W.dense(4, 2)], 2)
    theta = W.init_params(m_seq, rng, bias_scale=0.3).astype(np.float64)
    tok = np.array([3], dtype=np.int32)
    _, g1, _ = O.example_grad(m_seq, theta, tok, 1)
    _, g2, _ = O.example_grad(m_last, theta, tok, 1)
    assert np.array_equal(g1, g2)


def test_lstm_sequence_mean_of_identical_steps():
    """Sequence output + mean over steps: with W_hh = 0 and the forget gate shut (its input weights zero, its bias
    -50, sigmoid(-50) ~ 2e-22) a step sees only its own token, so on a sequence of T identical tokens every h_t is
    the h of the one-token sequence, the mean is that h, the loss is the one-token loss, and each of the T steps
    contributes 1/T of the one-token gradient: the two gradients agree outside W_hh (whose gradient pairs a step
    with its predecessor, which the one-token sequence does not have)."""
    rng = np.random.default_rng(9)
    T = 4
    layers = [W.embedding(5, 3), W.lstm_seq(3, 4), W.seq_mean(), W.dense(4, 2)]
    m, m1 = W.model(W.token_input(T), layers, 2), W.model(W.token_input(1), layers, 2)
    theta = W.init_params(m, rng, bias_scale=0.3).astype(np.float64)
    off = {(li, n): (o, int(np.prod(s))) for li, n, s, o in W.param_tensors(m)}
    o, n = off[(1, "W_hh")]
    theta[o:o + n] = 0.0
    ob, _ = off[(1, "b")]
    theta[ob + 4:ob + 8] = -50.0
    oi, ni = off[(1, "W_ih")]
    Wih = theta[oi:oi + ni].reshape(3, 16)
    Wih[:, 4:8] = 0.0
    theta[oi:oi + ni] = Wih.reshape(-1)
    _, gT, _ = O.example_grad(m, theta, np.full(T, 2, dtype=np.int32), 0)
    _, g1, _ = O.example_grad(m1, theta, np.array([2], dtype=np.int32), 0)
    keep = np.ones(theta.size, dtype=bool)
    keep[o:o + n] = False
    assert np.allclose(gT[keep], g1[keep], rtol=1e-9, atol=1e-14)
    assert np.linalg.norm(g1[keep]) > 0 and np.linalg.norm(gT[o:o + n]) > 0 and not g1[o:o + n].any()


@pytest.mark.parametrize("name", ["tiny_dense_tanh", "tiny_conv2", "tiny_lstm", "tiny_emb", "tiny_lstm_seq",
                                  "tiny_avgpool"])
def test_sgd_step_reduces_to_plain_sgd(name):
    """Section 1, item 4 after items 2-3: with no clipping and no noise the private update is one step of ordinary
    SGD on the mean loss (torch.optim.SGD on an independent autograd model)."""
    import torch
    m = TINY[name]
    rng = np.random.default_rng(17)
    x, y = W.make_inputs(m, 6, rng)
    theta = W.init_params(m, rng, bias_scale=0.3)
    lr = 0.37
    new = O.sgd_step(m, theta, x, y, float("inf"), 0.0, 0, lr)
    G = TR.per_example_grads(m, theta.astype(np.float64), x, y)   # [B, P] from autograd
    t = torch.nn.Parameter(torch.from_numpy(theta.astype(np.float64)))
    opt = torch.optim.SGD([t], lr=lr)
    t.grad = torch.from_numpy(G.mean(axis=0))
    opt.step()
    assert np.allclose(new, t.detach().numpy().astype(np.float32), rtol=0, atol=2e-7)
    # and with clipping + noise it is theta - lr/B * out of the step itself
    ref = O.dp_step(m, theta, x, y, 0.5, 1.1, 9)
    new2 = O.sgd_step(m, theta, x, y, 0.5, 1.1, 9, lr)
    z = O.noise(9, theta.size)
    want = theta.astype(np.float64) - lr / 6 * (ref["clipped_sum"] + 1.1 * 0.5 * z)
    assert np.array_equal(new2, want.astype(np.float32))


# ----------------------------------------------------------------- max-pool margins and routing (test aids of the oracle)

def _pool_model():
    # 2x2x6 image -> 1x1 convolution to 2 channels, tanh -> 2x2 / stride-2 max-pool (3 windows a channel) -> fc 2
    return W.model(W.image_input(2, 2, 6), [W.conv2d(2, 2, 1, act="tanh"), W.maxpool2d(2, 2), W.dense(6, 2)], 2)


def _pool_case():
    m = _pool_model()
    e = 2.0 ** -20
    # v = sum of the two input planes; its windows (columns 0-1, 2-3, 4-5): clear maximum; runner-up 2^-20 below
    # the maximum; exact tie.  All values are dyadic, so the sums are exact, and tied pixels differ in their planes.
    v = np.array([[0.125, 0.875, 0.5 + e, 0.25, 0.75, 0.75],
                  [0.3125, 0.25, 0.5, 0.125, 0.75, 0.375]])
    p0 = np.array([[0.0625, 0.5, 0.125, 0.125, 0.25, 0.5],
                   [0.25, 0.125, 0.375, 0.0625, 0.375, 0.125]])
    x = np.stack([p0, v - p0])[None].astype(np.float32)
    assert np.array_equal(x[0, 0].astype(np.float64) + x[0, 1], v)
    theta = np.zeros(O.num_params(m), dtype=np.float32)
    theta[0:2], theta[2:4] = 1.0, 0.5        # channel 0 = tanh(v), channel 1 = tanh(v / 2): both keep the order of v
    theta[6:18] = np.linspace(-0.4, 0.5, 12)  # dense weights
    return m, x, np.array([1], dtype=np.int32), theta


def test_pool_margin_on_three_hand_built_windows():
    m, x, y, theta = _pool_case()
    r = O.dp_step(m, theta, x, y, 1.0, 0.0, 0, clip=False)
    # smallest non-zero gap over both channels: tanh(0.5 (0.5 + e)) - tanh(0.25), the second channel's middle window
    want = math.tanh(0.5 * (0.5 + 2.0 ** -20)) - math.tanh(0.25)
    assert want < math.tanh(0.5 + 2.0 ** -20) - math.tanh(0.5)
    assert r["pool_margin"][0] == pytest.approx(want, rel=1e-9)
    assert r["ties"] == 2   # the third window of either channel holds 0.7 twice
    ent = O.pool_near_ties(m, theta.astype(np.float64), x[0], y[0], 1e-5)
    # one runner-up per channel, in the middle window (pool output 1 / 4), element (row 1, column 2) of that channel
    assert [(l, oi, ii) for l, oi, ii, _ in ent] == [(1, 1, 8), (1, 4, 12 + 8)]
    assert ent[0][3] == pytest.approx(math.tanh(0.5 + 2.0 ** -20) - math.tanh(0.5), rel=1e-9)
    assert O.pool_near_ties(m, theta.astype(np.float64), x[0], y[0], 1e-8) == []
    with pytest.raises(ValueError):
        O.example_grad_routed(m, theta.astype(np.float64), x[0], y[0], [(1, 1, 0)])  # element of another window


def test_routed_gradient_equals_the_gradient_after_a_nudge():
    """Routing a near-tied window to its runner-up gives the gradient of the input in which that runner-up has been
    nudged past the maximum (up to the size of the nudge), and differs from the first-maximum gradient."""
    m, x, y, theta = _pool_case()
    th64 = theta.astype(np.float64)
    ent = O.pool_near_ties(m, th64, x[0], y[0], 1e-5)
    routes = [e[:3] for e in ent]
    g_first = O.example_grad(m, th64, x[0], y[0])[1]
    g_routed = O.example_grad_routed(m, th64, x[0], y[0], routes)[1]
    x2 = x.copy()
    x2[0, 0, 1, 2] += 2.0 ** -18            # v at (row 1, column 2) now exceeds (row 0, column 2) in both channels
    g_nudged = O.example_grad(m, th64, x2[0], y[0])[1]
    assert np.abs(g_routed - g_nudged).max() <= 1e-5 * np.abs(g_nudged).max()
    assert np.abs(g_routed - g_first).max() >= 1e-3 * np.abs(g_first).max()
    assert np.array_equal(O.example_grad_routed(m, th64, x[0], y[0], [])[1], g_first)


def _relu_case():
    # fc 3 -> 3 with ReLU, then fc 3 -> 2.  Dyadic inputs and weights: the hidden pre-activations are exactly
    # (0.75, 2^-24, -2^-24): one clear unit, one just above zero, one just below.
    m = W.model(W.image_input(3), [W.dense(3, 3, act="relu"), W.dense(3, 2)], 2)
    e = 2.0 ** -24
    x = np.array([[1.0, 0.5, 0.25]], dtype=np.float32)
    theta = np.zeros(O.num_params(m), dtype=np.float32)
    W1 = np.array([[0.5, 0.0, 0.0], [0.5, 0.0, 0.0], [0.0, 0.0, 0.0]])   # [d_in][d_out]
    theta[0:9] = W1.reshape(-1)
    theta[9:12] = [0.0, e, -e]                                            # b1
    theta[12:18] = [0.5, -0.25, 0.125, 0.75, -0.5, 0.25]                  # W2 [3][2]
    theta[18:20] = [0.125, -0.125]
    return m, x, np.array([0], dtype=np.int32), theta


def test_relu_units_next_to_zero_are_listed_and_flipped():
    """A ReLU pre-activation within tau of zero is a decision like a near-tied pool window.  Hand-built case with
    pre-activations (0.75, +2^-24, -2^-24): the margin is 2^-24, both small units are listed, and flipping one
    gives the gradient of the input in which its bias has been nudged across zero."""
    m, x, y, theta = _relu_case()
    th64 = theta.astype(np.float64)
    r = O.dp_step(m, theta, x, y, 1.0, 0.0, 0, clip=False)
    assert r["pool_margin"][0] == 2.0 ** -24
    ent = O.pool_near_ties(m, th64, x[0], y[0], 1e-6)
    assert [(l, oi, ii) for l, oi, ii, _ in ent] == [(0, 1, -1), (0, 2, -1)]
    assert [g for *_, g in ent] == [2.0 ** -24, 2.0 ** -24]
    assert O.pool_near_ties(m, th64, x[0], y[0], 1e-8) == []
    g0 = O.example_grad(m, th64, x[0], y[0])[1]
    # unit 1 (z = +2^-24, subgradient 1) switched off: the gradient after its bias is nudged below zero
    g_off = O.example_grad_routed(m, th64, x[0], y[0], [(0, 1, -1)])[1]
    th2 = th64.copy(); th2[10] = -2.0 ** -24
    g_nudged = O.example_grad(m, th2, x[0], y[0])[1]
    assert np.abs(g_off - g_nudged).max() <= 1e-6
    assert g_off[10] == 0.0 and g0[10] != 0.0          # its bias gradient: delta_1 * 1 before, * 0 after
    # unit 2 (z = -2^-24, subgradient 0) switched on: the gradient after its bias is nudged above zero
    g_on = O.example_grad_routed(m, th64, x[0], y[0], [(0, 2, -1)])[1]
    th3 = th64.copy(); th3[11] = 2.0 ** -24
    g_nudged = O.example_grad(m, th3, x[0], y[0])[1]
    assert np.abs(g_on - g_nudged).max() <= 1e-6
    assert g_on[11] != 0.0 and g0[11] == 0.0
    # closed form of the hidden bias gradients: delta_1[j] = relu'(z_j) * sum_k W2[j][k] (softmax_k - onehot_k)
    a1 = np.array([0.75, 2.0 ** -24, 0.0])
    logits = a1 @ th64[12:18].reshape(3, 2) + th64[18:20]
    p = np.exp(logits - logits.max()); p /= p.sum()
    d2 = p - np.array([1.0, 0.0])
    back = th64[12:18].reshape(3, 2) @ d2
    assert np.allclose(g0[9:12], back * np.array([1.0, 1.0, 0.0]), rtol=1e-12, atol=0)
    assert np.allclose(g_on[9:12], back * np.array([1.0, 1.0, 1.0]), rtol=1e-12, atol=0)
    assert np.allclose(g_off[9:12], back * np.array([1.0, 0.0, 0.0]), rtol=1e-12, atol=0)
    with pytest.raises(ValueError):
        O.example_grad_routed(m, th64, x[0], y[0], [(1, 0, -1)])   # the logit layer has no ReLU


def test_abs_sum_is_the_sum_of_term_magnitudes():
    """abs_sum (the yardstick of the per-tensor tolerance) against the per-example gradients: sum_i |s_i g_i|."""
    m, x, y, theta = _tiny_case("tiny_conv2", 6)
    th64 = theta.astype(np.float64)
    n0 = O.dp_step(m, theta, x, y, math.inf, 0.0, 0)["norms"]
    Cc = float(np.median(n0))
    r = O.dp_step(m, theta, x, y, Cc, 0.0, 0)
    want = np.zeros(theta.size)
    for i in range(6):
        g = O.example_grad(m, th64, x[i], y[i])[1]
        want += np.abs(g) * min(1.0, Cc / np.linalg.norm(g))
    assert np.allclose(r["abs_sum"], want, rtol=1e-12, atol=0)
    assert np.all(r["abs_sum"] >= np.abs(r["clipped_sum"]) * (1 - 1e-12))
    one = O.dp_step(m, theta, x[:1], y[:1], Cc, 0.0, 0)
    assert np.allclose(one["abs_sum"], np.abs(one["clipped_sum"]), rtol=1e-15, atol=0)


# ----------------------------------------------------------------- minibatch draw and the training loop (Section 1, items 1 and 4)

def test_sample_indices_against_the_philox_words():
    """Index k = (word k%4 of block (k/4, 0, 1, 0) times n) >> 32, written out with Python integers on top of the
    Philox function the known-answer vectors pin; the blocks differ from the noise stream's (third counter word)."""
    for seed, n, batch in ((0, 60000, 37), (0x1234567887654321, 2**31 - 1, 9), (5, 1, 6), (7, 3, 1000)):
        got = O.sample_indices(seed, n, batch)
        key = [seed & 0xffffffff, seed >> 32]
        want = [(int(O.philox4x32_10([k // 4, 0, 1, 0], key)[k % 4]) * n) >> 32 for k in range(batch)]
        assert got.tolist() == want
        assert got.min() >= 0 and got.max() < n
    assert not np.array_equal(O.philox4x32_10([0, 0, 1, 0], [0, 0]), O.philox4x32_10([0, 0, 0, 0], [0, 0]))
    # uniform over the range: every cell of a 16-cell histogram within 5 sigma of its expectation
    idx = O.sample_indices(11, 1600, 160000)
    h = np.bincount(idx // 100, minlength=16)
    assert np.all(np.abs(h - 10000) < 5 * math.sqrt(10000 * 15 / 16))
    assert len(np.unique(O.sample_indices(11, 10**6, 1000))) > 990   # with replacement: a few repeats at most


def test_train_is_the_chain_of_draw_step_update():
    m, x, y, theta = _tiny_case("tiny_conv2", 40)
    Cc, sigma, lr, B, seed0 = 0.8, 0.9, 0.3, 6, 2**40 + 3
    got = O.train(m, theta, x, y, 3, B, Cc, sigma, seed0, lr)
    cur = theta
    for t in range(3):
        idx = O.sample_indices(seed0 + t, len(y), B)
        cur = O.sgd_step(m, cur, x[idx], y[idx], Cc, sigma, seed0 + t, lr)
    assert np.array_equal(got, cur)
    assert not np.array_equal(got, theta)
    assert np.array_equal(O.train(m, theta, x, y, 0, B, Cc, sigma, seed0, lr), theta)
