"""Pins of the oracle's training step of the query model (Eq. 1 + Adam): gradients against central
finite differences of the loss, the loss against scipy's relative entropy, the stationary point
f_q = T, Adam's first step in closed form, and convergence on a target the model can realise."""
import numpy as np
from scipy.special import rel_entr, softmax

from oracle import train_ref as tr


def _problem(seed, R=9, d=6, hidden=7, B=5):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((R, d))
    T = rng.random((R, B)) ** 3
    T[0, 1] = 0.0                                           # an exact zero in the target
    T /= T.sum(axis=1, keepdims=True)
    W1 = rng.standard_normal((hidden, d)) / np.sqrt(d)
    b1 = 0.1 * rng.standard_normal(hidden)
    W2 = rng.standard_normal((B, hidden)) / np.sqrt(hidden)
    b2 = 0.1 * rng.standard_normal(B)
    return x, T, [W1, b1, W2, b2]


def test_loss_is_the_mean_relative_entropy():
    x, T, P = _problem(1)
    loss, _ = tr.loss_and_grads(x, T, *P)
    z = np.maximum(x @ P[0].T + P[1], 0) @ P[2].T + P[3]
    want = rel_entr(T, softmax(z, axis=1)).sum() / x.shape[0]
    np.testing.assert_allclose(loss, want, rtol=1e-12)
    assert loss > 0


def test_gradients_against_finite_differences():
    x, T, P = _problem(2)
    _, grads = tr.loss_and_grads(x, T, *P)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for i, (p, g) in enumerate(zip(P, grads)):
        assert p.shape == g.shape
        flat = p.reshape(-1)
        for j in rng.choice(flat.size, size=min(12, flat.size), replace=False):
            keep = flat[j]
            flat[j] = keep + eps
            lp, _ = tr.loss_and_grads(x, T, *P)
            flat[j] = keep - eps
            lm, _ = tr.loss_and_grads(x, T, *P)
            flat[j] = keep
            np.testing.assert_allclose(g.reshape(-1)[j], (lp - lm) / (2 * eps), rtol=2e-5, atol=1e-9,
                                       err_msg=f"parameter tensor {i}, entry {j}")


def test_zero_loss_and_gradient_when_the_model_equals_the_target():
    x, T, P = _problem(3)
    T = np.clip(T, 1e-3, None)
    T /= T.sum(axis=1, keepdims=True)
    # hidden units off (large negative bias): logits = b2; one shared target row realised by b2 = log T
    T[:] = T[0]
    P[1][:] = -100.0
    P[3][:] = np.log(T[0])
    loss, grads = tr.loss_and_grads(x, T, *P)
    assert abs(loss) < 1e-14
    for g in grads:
        assert np.abs(g).max() < 1e-15


def test_dead_relu_rows_pass_no_gradient_to_the_first_layer():
    x, T, P = _problem(4)
    P[1][:] = -100.0
    _, (dW1, db1, dW2, db2) = tr.loss_and_grads(x, T, *P)
    assert not dW1.any() and not db1.any() and not dW2.any() and db2.any()


def test_adam_first_step_and_convergence():
    rng = np.random.default_rng(5)
    p = rng.standard_normal(20)
    g = rng.standard_normal(20)
    new, m, v = tr.adam_update(p, g, np.zeros(20), np.zeros(20), 1, lr=0.01, eps=1e-12)
    # t = 1: mhat = g, vhat = g^2, so the step is lr * sign(g)
    np.testing.assert_allclose(new, p - 0.01 * np.sign(g), rtol=1e-9)
    np.testing.assert_allclose(m, 0.1 * g)
    np.testing.assert_allclose(v, 0.001 * g * g)
    # a target produced by a model of the same shape is learned: the loss falls by a large factor
    x, _, P_true = _problem(6, R=64)
    T = softmax(np.maximum(x @ P_true[0].T + P_true[1], 0) @ P_true[2].T + P_true[3], axis=1)
    _, _, P0 = _problem(7, R=64)
    params = tuple(p[None] for p in P0)
    zeros = tuple(np.zeros_like(p) for p in params)
    moments = (zeros, tuple(np.zeros_like(p) for p in params))
    first = None
    for t in range(1, 401):
        loss, params, moments = tr.train_step(x[None], T[None], params, moments, t, lr=0.02)
        first = loss[0] if first is None else first
    assert loss[0] < 0.05 * first


# ------------------------------------------------------------------ batch normalisation (Section 6.1)
def _problem_bn(seed, R=11, d=6, hidden=7, B=5):
    x, T, (W1, b1, W2, b2) = _problem(seed, R, d, hidden, B)
    rng = np.random.default_rng(seed + 100)
    gamma = 1.0 + 0.3 * rng.standard_normal(hidden)
    beta = 0.2 * rng.standard_normal(hidden)
    return x, T, [W1, b1, gamma, beta, W2, b2]


def test_bn_gradients_against_finite_differences():
    x, T, P = _problem_bn(5)
    _, grads, _ = tr.loss_and_grads_bn(x, T, *P)
    rng = np.random.default_rng(0)
    eps = 1e-6
    for i, (p, g) in enumerate(zip(P, grads)):
        assert p.shape == g.shape
        flat = p.reshape(-1)
        for j in rng.choice(flat.size, size=min(12, flat.size), replace=False):
            keep = flat[j]
            flat[j] = keep + eps
            lp = tr.loss_and_grads_bn(x, T, *P)[0]
            flat[j] = keep - eps
            lm = tr.loss_and_grads_bn(x, T, *P)[0]
            flat[j] = keep
            np.testing.assert_allclose(g.reshape(-1)[j], (lp - lm) / (2 * eps), rtol=5e-5, atol=2e-9,
                                       err_msg=f"parameter tensor {i}, entry {j}")
    # a shift of the first layer's bias is removed by the normalisation: its gradient vanishes
    assert np.abs(grads[1]).max() < 1e-12


def test_bn_against_torch_batch_norm_and_autograd():
    import torch
    import torch.nn.functional as F
    x, T, P = _problem_bn(6, R=16)
    loss, grads, (mu, var) = tr.loss_and_grads_bn(x, T, *P, eps=1e-5)
    tp = [torch.tensor(p, dtype=torch.float64, requires_grad=True) for p in P]
    tx, tT = torch.tensor(x), torch.tensor(T)
    run_mean = torch.zeros(7, dtype=torch.float64)
    run_var = torch.ones(7, dtype=torch.float64)
    a = F.linear(tx, tp[0], tp[1])
    y = F.batch_norm(a, run_mean, run_var, tp[2], tp[3], training=True, momentum=0.1, eps=1e-5)
    logp = F.log_softmax(F.linear(torch.relu(y), tp[4], tp[5]), dim=1)
    tl = F.kl_div(logp, tT, reduction="batchmean")
    tl.backward()
    np.testing.assert_allclose(loss, tl.item(), rtol=1e-12)
    for g, t in zip(grads, tp):
        np.testing.assert_allclose(g, t.grad.numpy(), rtol=1e-9, atol=1e-13)
    rm, rv = tr.running_stats_update(np.zeros(7), np.ones(7), mu, var, 16, 0.1)
    np.testing.assert_allclose(rm, run_mean.numpy(), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(rv, run_var.numpy(), rtol=1e-12)


def test_folded_model_is_the_normalised_model_at_inference():
    x, T, P = _problem_bn(7)
    W1, b1, gamma, beta, W2, b2 = P
    rng = np.random.default_rng(3)
    run_mean, run_var = rng.standard_normal(7), 0.5 + rng.random(7)
    W1f, b1f = tr.fold_batch_norm(W1, b1, gamma, beta, run_mean, run_var, 1e-5)
    _, _, z_folded, _ = tr.forward(x, W1f, b1f, W2, b2)
    a = x @ W1.T + b1
    y = gamma * (a - run_mean) / np.sqrt(run_var + 1e-5) + beta
    z = np.maximum(y, 0) @ W2.T + b2
    np.testing.assert_allclose(z_folded, z, rtol=1e-12, atol=1e-13)
    # with the batch's own statistics (divisor R) the folded model reproduces the training-mode forward
    _, mu, var, _, _, z_train, _ = tr.forward_bn(x, *P)
    W1b, b1b = tr.fold_batch_norm(W1, b1, gamma, beta, mu, var, 1e-5)
    np.testing.assert_allclose(tr.forward(x, W1b, b1b, W2, b2)[2], z_train, rtol=1e-11, atol=1e-12)
