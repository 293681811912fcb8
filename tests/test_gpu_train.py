"""GPU parity of the query-model training calls against the float64 oracle (oracle/train_ref.py):
loss and the four gradient tensors of query_model_loss_grads, the Adam update, a short run of
training steps, and bit-for-bit reproducibility.
Tolerances (fp32 sums of up to R or B terms against float64): loss 1e-5 relative; gradients
|gpu - ref| <= 1e-4 * max|ref| + 1e-4 |ref|; Adam: second moment 2e-6 relative, first moment 4e-7 of its two terms, the step 2e-4 relative."""
import numpy as np
import pytest
import torch

from oracle import train_ref as tr

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
# hyper-parameters as the fp32 numbers the C call receives, so that both sides start from the same values
LR, B1, B2, EPS = (float(np.float32(v)) for v in (1e-3, 0.9, 0.999, 1e-8))


@pytest.fixture(scope="module")
def saap():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: the -m gpu tests need a real device")
    import paper_2502_08246_amd as lib
    lib.load_library()
    return lib


def problem(seed, Hw, R, d, hidden, B, dtype=torch.float32):
    g = torch.Generator(device="cpu").manual_seed(seed)
    x = torch.randn(Hw, R, d, generator=g).to(dtype)
    T = torch.rand(Hw, R, B, generator=g) ** 4
    T[:, 0, 0] = 0.0
    T = T / T.sum(-1, keepdim=True)
    W1 = torch.randn(Hw, hidden, d, generator=g) / d ** 0.5
    b1 = 0.1 * torch.randn(Hw, hidden, generator=g)
    W2 = torch.randn(Hw, B, hidden, generator=g) / hidden ** 0.5
    b2 = 0.1 * torch.randn(Hw, B, generator=g)
    return x, T, (W1, b1, W2, b2)


def to_dev(ts):
    return tuple(t.to(DEV).contiguous() for t in ts)


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


@pytest.mark.parametrize("Hw,R,d,hidden,B,dtype", [
    (2, 70, 128, 64, 37, torch.float32), (1, 129, 128, 96, 200, torch.bfloat16), (3, 33, 40, 17, 5, torch.float32),
    (1, 300, 128, 512, 1024, torch.float32),
])
def test_loss_and_gradients(saap, Hw, R, d, hidden, B, dtype):
    x, T, params = problem(3, Hw, R, d, hidden, B, dtype)
    loss, grads = saap.query_model_loss_grads(x.to(DEV), T.to(DEV), to_dev(params))
    torch.cuda.synchronize()
    for w in range(Hw):
        want_loss, want = tr.loss_and_grads(f64(x[w]), f64(T[w]), *(f64(p[w]) for p in params))
        np.testing.assert_allclose(float(loss[w]), want_loss, rtol=1e-5)
        for name, g, r in zip(("dW1", "db1", "dW2", "db2"), grads, want):
            got = f64(g[w])
            lim = 1e-4 * np.abs(r).max() + 1e-4 * np.abs(r)
            assert (np.abs(got - r) <= lim).all(), f"{name}[{w}]: max err {np.abs(got - r).max():.3e} of {np.abs(r).max():.3e}"


def test_adam_update(saap):
    g = torch.Generator(device="cpu").manual_seed(9)
    n = 10_007
    p, grad = torch.randn(n, generator=g), torch.randn(n, generator=g) * torch.logspace(-8, 2, n)
    m, v = 0.1 * torch.randn(n, generator=g), torch.rand(n, generator=g) * 1e-3
    dp, dg, dm, dv = (t.to(DEV) for t in (p, grad, m, v))
    for step in (1, 2, 7):
        want_p, want_m, want_v = tr.adam_update(f64(dp), f64(dg), f64(dm), f64(dv), step, LR, B1, B2, EPS)
        before, m_old = f64(dp), f64(dm)
        saap.adam_update(dp, dg, dm, dv, step, LR, B1, B2, EPS)
        torch.cuda.synchronize()
        # the first moment is a sum of two terms that may cancel: the bound is relative to the terms
        assert (np.abs(f64(dm) - want_m) <= 4e-7 * (np.abs(m_old) + np.abs(f64(dg)))).all()
        np.testing.assert_allclose(f64(dv), want_v, rtol=2e-6, atol=1e-30)
        # the parameter itself is compared through its change (the step is small against the value)
        err = np.abs((f64(dp) - before) - (want_p - before))
        assert (err <= 2e-4 * np.abs(want_p - before) + 1.5e-7 * (1 + np.abs(before))).all()   # + one rounding of p


def test_training_steps_follow_the_oracle_and_are_reproducible(saap):
    Hw, R, d, hidden, B = 2, 64, 128, 32, 19
    x, T, params = problem(5, Hw, R, d, hidden, B)
    lr, steps = float(np.float32(3e-3)), 5

    def run():
        P = to_dev(tuple(p.clone() for p in params))
        M = tuple(torch.zeros_like(p) for p in P)
        V = tuple(torch.zeros_like(p) for p in P)
        losses = []
        dx, dT = x.to(DEV), T.to(DEV)
        for t in range(1, steps + 1):
            loss, grads = saap.query_model_loss_grads(dx, dT, P)
            for p, g, m, v in zip(P, grads, M, V):
                saap.adam_update(p, g, m, v, t, lr, B1, B2, EPS)
            losses.append(loss.clone())
        torch.cuda.synchronize()
        return torch.stack(losses), P

    losses, P = run()
    losses2, P2 = run()
    assert torch.equal(losses, losses2) and all(torch.equal(a, b) for a, b in zip(P, P2))
    rp = tuple(f64(p) for p in params)
    mom = (tuple(np.zeros_like(p) for p in rp), tuple(np.zeros_like(p) for p in rp))
    want = []
    for t in range(1, steps + 1):
        l, rp, mom = tr.train_step(f64(x), f64(T), rp, mom, t, lr, B1, B2, EPS)
        want.append(l)
    np.testing.assert_allclose(f64(losses), np.stack(want), rtol=2e-4)
    assert (f64(losses)[-1] < f64(losses)[0]).all()
    # Adam's first steps have the size lr whatever the gradient, so parameters are compared with an absolute bound
    for a, b in zip(P, rp):
        assert np.abs(f64(a) - b).max() < 0.05 * lr * steps


def test_training_argument_checks(saap):
    x, T, params = problem(7, 1, 8, 16, 8, 4)
    with pytest.raises(ValueError):
        saap.query_model_loss_grads(x.to(DEV), T[:, :, :3].contiguous().to(DEV), to_dev(params))
    with pytest.raises(TypeError):
        saap.query_model_loss_grads(x.to(DEV), T.to(DEV), to_dev(tuple(p.to(torch.bfloat16) for p in params)))
    p = torch.zeros(4, device=DEV)
    with pytest.raises(saap.SaapError):
        saap.adam_update(p, p.clone(), p.clone(), p.clone(), 0, 1e-3)


def test_training_driver_learns_on_a_small_workload(saap):
    """The whole procedure (targets from bucket_attention_mass, training steps, evaluation through
    classify_queries + select_buckets) on a small workload: the loss falls and the trained lists capture
    more attention mass than those of the random-init model."""
    from paper_2502_08246_amd import train_query_model
    from synth import gen
    cfg = gen.CONFIGS["cfg1_llama8b_128k"].replace(S=1, Hq=4, Hkv=2, N=6000, B=32, nprobe=4, hidden=64)
    for batch_norm in (False, True):
        rep = train_query_model.train(cfg, train_queries=256, eval_queries=32, steps=150, batch=256, lr=3e-3, seed=3,
                                      batch_norm=batch_norm)
        first, last = rep["loss"][0][1], rep["loss"][-1][1]
        assert last < 0.8 * first, (batch_norm, rep["loss"])
        cap = rep["captured_attention_mass"]
        assert cap["trained"] > cap["random_init"] + 0.02, (batch_norm, cap)
        assert cap["best_possible"] >= cap["trained"]


# ------------------------------------------------------------------ batch normalisation (Section 6.1)
@pytest.mark.parametrize("Hw,R,d,hidden,B,dtype", [
    (2, 70, 128, 64, 37, torch.float32), (1, 129, 128, 96, 200, torch.bfloat16), (3, 33, 40, 17, 5, torch.float32),
    (1, 300, 128, 512, 1024, torch.float32),
])
def test_bn_loss_gradients_and_running_statistics(saap, Hw, R, d, hidden, B, dtype):
    """Tolerances as for the plain model; the gradient of b1 is zero in exact arithmetic (the normalisation
    removes a shift), so it is bounded against the size of its terms, the gradient of beta."""
    x, T, params = problem(13, Hw, R, d, hidden, B, dtype)
    g = torch.Generator(device="cpu").manual_seed(14)
    gamma = 1.0 + 0.3 * torch.randn(Hw, hidden, generator=g)
    beta = 0.2 * torch.randn(Hw, hidden, generator=g)
    run_mean, run_var = torch.randn(Hw, hidden, generator=g), 0.5 + torch.rand(Hw, hidden, generator=g)
    mom, eps = float(np.float32(0.1)), float(np.float32(1e-5))
    d_rm, d_rv = run_mean.to(DEV), run_var.to(DEV)
    loss, grads, gg, gb = saap.query_model_bn_loss_grads(x.to(DEV), T.to(DEV), to_dev(params), gamma.to(DEV), beta.to(DEV),
                                                         d_rm, d_rv, mom, eps)
    torch.cuda.synchronize()
    for w in range(Hw):
        W1, b1, W2, b2 = (f64(p[w]) for p in params)
        want_loss, want, (mu, var) = tr.loss_and_grads_bn(f64(x[w]), f64(T[w]), W1, b1, f64(gamma[w]), f64(beta[w]), W2, b2, eps)
        np.testing.assert_allclose(float(loss[w]), want_loss, rtol=1e-5)
        got = dict(dW1=grads[0], db1=grads[1], dgamma=gg, dbeta=gb, dW2=grads[2], db2=grads[3])
        for name, r in zip(("dW1", "db1", "dgamma", "dbeta", "dW2", "db2"), want):
            a = f64(got[name][w])
            scale = np.abs(want[3]).max() if name == "db1" else np.abs(r).max()
            lim = 1e-4 * scale + 1e-4 * np.abs(r)
            assert (np.abs(a - r) <= lim).all(), f"{name}[{w}]: max err {np.abs(a - r).max():.3e} of {scale:.3e}"
        rm, rv = tr.running_stats_update(f64(run_mean[w]), f64(run_var[w]), mu, var, R, mom)
        np.testing.assert_allclose(f64(d_rm[w]), rm, rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(f64(d_rv[w]), rv, rtol=1e-5)
    # without running statistics the same gradients, bit for bit
    loss2, grads2, gg2, gb2 = saap.query_model_bn_loss_grads(x.to(DEV), T.to(DEV), to_dev(params), gamma.to(DEV), beta.to(DEV),
                                                             None, None, mom, eps)
    torch.cuda.synchronize()
    assert torch.equal(loss, loss2) and torch.equal(gg, gg2) and all(torch.equal(a, b) for a, b in zip(grads, grads2))


@pytest.mark.parametrize("out_dtype", [torch.float32, torch.bfloat16])
def test_fold_batch_norm_and_inference(saap, out_dtype):
    """The folded weights against the oracle's, and classify_queries on them against the oracle's normalised
    model with the running statistics (bf16: the weights are compared after the same rounding)."""
    Hw, hidden, d, B, S = 2, 96, 128, 48, 3
    _, _, (W1, b1, W2, b2) = problem(17, Hw, 4, d, hidden, B)
    g = torch.Generator(device="cpu").manual_seed(18)
    gamma = 1.0 + 0.3 * torch.randn(Hw, hidden, generator=g)
    beta = 0.2 * torch.randn(Hw, hidden, generator=g)
    run_mean, run_var = 0.3 * torch.randn(Hw, hidden, generator=g), 0.5 + torch.rand(Hw, hidden, generator=g)
    eps = float(np.float32(1e-5))
    W1f, b1f = saap.fold_batch_norm(*to_dev((W1, b1, gamma, beta, run_mean, run_var)), eps=eps, out_dtype=out_dtype)
    torch.cuda.synchronize()
    assert W1f.dtype == out_dtype
    for w in range(Hw):
        rW, rb = tr.fold_batch_norm(f64(W1[w]), f64(b1[w]), f64(gamma[w]), f64(beta[w]), f64(run_mean[w]), f64(run_var[w]), eps)
        np.testing.assert_allclose(f64(b1f[w]), rb, rtol=2e-6, atol=1e-7)
        if out_dtype == torch.float32:
            np.testing.assert_allclose(f64(W1f[w]), rW, rtol=2e-6, atol=1e-9)
        else:
            np.testing.assert_allclose(f64(W1f[w]), rW, rtol=2.0 ** -8, atol=1e-9)   # half a bf16 step
    # inference through classify_queries: logits of the folded model = the normalised model
    xq = torch.randn(S, Hw * 2, d, generator=g).to(out_dtype)
    W2d = W2.to(out_dtype)
    logits = saap.classify_queries(xq.to(DEV), W1f, b1f, W2d.to(DEV), b2.to(DEV), Hw, output_kind=saap.LOGITS)
    torch.cuda.synchronize()
    for hq in range(Hw * 2):
        w = hq // 2
        a = f64(xq[:, hq]) @ f64(W1f[w]).T + f64(b1f[w])              # the weights as stored (rounded for bf16)
        want = np.maximum(a, 0) @ f64(W2d[w]).T + f64(b2[w])
        np.testing.assert_allclose(f64(logits[:, hq]), want, rtol=1e-4, atol=2e-4)
        if out_dtype == torch.float32:                                # and against the definition with the statistics
            a0 = f64(xq[:, hq]) @ f64(W1[w]).T + f64(b1[w])
            y = f64(gamma[w]) * (a0 - f64(run_mean[w])) / np.sqrt(f64(run_var[w]) + eps) + f64(beta[w])
            np.testing.assert_allclose(f64(logits[:, hq]), np.maximum(y, 0) @ f64(W2[w]).T + f64(b2[w]), rtol=1e-4, atol=2e-4)
