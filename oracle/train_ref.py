"""CPU oracle of one training step of the query model f_q (arXiv 2502.08246, Section 4 "Query
assignment function", Eq. 1; Appendix "Training details": Adam).

TEST INFRASTRUCTURE ONLY: plain numpy in float64, the definition written out.  It shares no code
with the GPU path; only the tests (and a benchmark's baseline leg) import it.

Model (Section 6.1; BASELINE's configurations use no batch-norm): z = W2 relu(W1 x + b1) + b2,
f_q(x) = softmax(z).  Loss (Eq. 1), with T = the rows of A * H_k (bucket attention mass):
    L = 1/R * sum_r sum_b T[r,b] * (log T[r,b] - log f_q(x_r)[b]),      0 * log 0 = 0
i.e. the Kullback-Leibler divergence of the rows, averaged over the batch.  Its gradient with respect
to the logits is (sum_b T[r,b]) * f_q(x_r) - T[r,:], divided by R; the rest is the chain rule.
The derivative of relu at 0 is taken as 0.

With batch normalisation (the model of Section 6.1: two layers, batch normalisation, ReLU) the hidden
layer is h = relu(gamma * (a - mean_r a) / sqrt(var_r a + eps) + beta) with the statistics of the batch
(variance with divisor R); running statistics follow the usual exponential average with the variance
estimate of divisor R - 1; at inference the normalisation with the running statistics is an affine map
and folds into W1 and b1.  The paper names the layer and gives no constants: eps = 1e-5 and momentum 0.1
are this build's reading.

Parity pins (tests/test_oracle_train.py): central finite differences of the loss for every
parameter tensor, scipy's relative entropy for the loss, zero loss and zero gradient at f_q = T,
the first Adam step against its closed form, and convergence on a realisable target; for the
batch-norm variant finite differences again, torch's batch_norm with autograd, and the folded
inference model against the normalised one.
"""
from __future__ import annotations

import numpy as np


def forward(x, W1, b1, W2, b2):
    """x [R,d] -> pre-activations a [R,hidden], hidden h, logits z [R,B], log-probabilities logp [R,B]."""
    a = x @ W1.T + b1
    h = np.maximum(a, 0.0)
    z = h @ W2.T + b2
    zmax = z.max(axis=1, keepdims=True)
    logp = z - zmax - np.log(np.exp(z - zmax).sum(axis=1, keepdims=True))
    return a, h, z, logp


def loss_and_grads(x, T, W1, b1, W2, b2):
    """One weight set: x [R,d], T [R,B] -> loss, (dW1, db1, dW2, db2), all float64."""
    x, T, W1, b1, W2, b2 = (np.asarray(v, dtype=np.float64) for v in (x, T, W1, b1, W2, b2))
    R = x.shape[0]
    a, h, z, logp = forward(x, W1, b1, W2, b2)
    pos = T > 0
    loss = float((T[pos] * (np.log(T[pos]) - logp[pos])).sum() / R)
    g = (np.exp(logp) * T.sum(axis=1, keepdims=True) - T) / R
    dW2 = g.T @ h
    db2 = g.sum(axis=0)
    da = (g @ W2) * (a > 0)
    dW1 = da.T @ x
    db1 = da.sum(axis=0)
    return loss, (dW1, db1, dW2, db2)


def forward_bn(x, W1, b1, gamma, beta, W2, b2, eps=1e-5):
    """Training-mode forward.  -> a [R,hidden], its batch mean and variance (divisor R), the normalised
    ahat, y = gamma ahat + beta, logits z, log-probabilities logp."""
    a = x @ W1.T + b1
    mu = a.mean(axis=0)
    var = ((a - mu) ** 2).mean(axis=0)
    ahat = (a - mu) / np.sqrt(var + eps)
    y = gamma * ahat + beta
    z = np.maximum(y, 0.0) @ W2.T + b2
    zmax = z.max(axis=1, keepdims=True)
    logp = z - zmax - np.log(np.exp(z - zmax).sum(axis=1, keepdims=True))
    return a, mu, var, ahat, y, z, logp


def loss_and_grads_bn(x, T, W1, b1, gamma, beta, W2, b2, eps=1e-5):
    """One weight set with batch normalisation: -> loss, (dW1, db1, dgamma, dbeta, dW2, db2), (mean, var)."""
    x, T, W1, b1, gamma, beta, W2, b2 = (np.asarray(v, dtype=np.float64) for v in (x, T, W1, b1, gamma, beta, W2, b2))
    R = x.shape[0]
    a, mu, var, ahat, y, z, logp = forward_bn(x, W1, b1, gamma, beta, W2, b2, eps)
    pos = T > 0
    loss = float((T[pos] * (np.log(T[pos]) - logp[pos])).sum() / R)
    g = (np.exp(logp) * T.sum(axis=1, keepdims=True) - T) / R
    h = np.maximum(y, 0.0)
    dW2 = g.T @ h
    db2 = g.sum(axis=0)
    dy = (g @ W2) * (y > 0)
    dgamma = (dy * ahat).sum(axis=0)
    dbeta = dy.sum(axis=0)
    # a enters ahat directly, through the batch mean and through the batch variance
    da = gamma / np.sqrt(var + eps) * (dy - dbeta / R - ahat * dgamma / R)
    dW1 = da.T @ x
    db1 = da.sum(axis=0)
    return loss, (dW1, db1, dgamma, dbeta, dW2, db2), (mu, var)


def running_stats_update(run_mean, run_var, mu, var, R, momentum=0.1):
    """Exponential averages of the batch statistics; the variance enters with divisor R - 1."""
    return (1.0 - momentum) * run_mean + momentum * mu, (1.0 - momentum) * run_var + momentum * var * R / (R - 1.0)


def fold_batch_norm(W1, b1, gamma, beta, run_mean, run_var, eps=1e-5):
    """Inference: gamma (W1 x + b1 - mean) / sqrt(var + eps) + beta = W1' x + b1'."""
    s = gamma / np.sqrt(run_var + eps)
    return W1 * s[:, None], (b1 - run_mean) * s + beta


def adam_update(p, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """Adam (Kingma & Ba), step number t >= 1: returns the new parameter and moments."""
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** t)
    vhat = v / (1.0 - beta2 ** t)
    return p - lr * mhat / (np.sqrt(vhat) + eps), m, v


def train_step(x, T, params, moments, t, lr, beta1=0.9, beta2=0.999, eps=1e-8):
    """All weight sets.  x [Hw,R,d], T [Hw,R,B]; params = (W1 [Hw,hidden,d], b1 [Hw,hidden], W2 [Hw,B,hidden],
    b2 [Hw,B]); moments = (m, v), each a tuple shaped like params.  Returns loss [Hw] (before the update),
    new params, new moments."""
    Hw = x.shape[0]
    params = [np.array(p, dtype=np.float64) for p in params]
    m = [np.array(p, dtype=np.float64) for p in moments[0]]
    v = [np.array(p, dtype=np.float64) for p in moments[1]]
    loss = np.empty(Hw, dtype=np.float64)
    for w in range(Hw):
        loss[w], grads = loss_and_grads(x[w], T[w], *(p[w] for p in params))
        for i, g in enumerate(grads):
            params[i][w], m[i][w], v[i][w] = adam_update(params[i][w], g, m[i][w], v[i][w], t, lr, beta1, beta2, eps)
    return loss, tuple(params), (tuple(m), tuple(v))
