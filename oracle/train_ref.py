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

Parity pins (tests/test_oracle_train.py): central finite differences of the loss for every
parameter tensor, scipy's relative entropy for the loss, zero loss and zero gradient at f_q = T,
the first Adam step against its closed form, and convergence on a realisable target.
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
