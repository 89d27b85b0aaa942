"""Pins for the oracle's training objective (Eq. 5, Eq. 7, Eq. 9 as weights, AdamW): closed forms,
finite differences of the loss, torch autograd / torch.optim.AdamW in fp64 as library routines."""
import math

import numpy as np
import pytest
import torch

import oracle


def _close(a, b, atol=1e-12, rtol=0.0):
    return np.allclose(a, b, rtol=rtol, atol=atol)


def _head(seed, d=7, d_h=5, K=6):
    rng = np.random.default_rng(seed)
    return oracle.TrainHead(w1=rng.normal(0, d ** -0.5, (d_h, d)), b1=rng.normal(0, 0.3, d_h),
                            w2=rng.normal(0, d_h ** -0.5, (K, d_h)), b2=rng.normal(0, 0.3, K),
                            centers=np.linspace(10.0, 400.0, K))


def _batch(seed, B=9, d=7, K=6):
    rng = np.random.default_rng(seed)
    return rng.normal(size=(B, d)), rng.integers(0, K, size=B), rng.uniform(5.0, 450.0, size=B)


def test_soft_label_closed_forms():
    K = 20
    for i in (0, 7, 19):
        p = oracle.soft_label(i, K)
        assert abs(p.sum() - 1.0) < 1e-15 and int(np.argmax(p)) == i
        for j in range(K - 1):                      # neighbours differ by a factor e, away from the peak
            r = p[j + 1] / p[j]
            assert abs(r - (math.e if j < i else 1 / math.e)) < 1e-12
    # interior bin of a wide grid: Z = 1 + 2 sum_{k>=1} e^-k (truncated) -> p_i = tanh(1/2) as K grows
    p = oracle.soft_label(50, 101)
    assert abs(p[50] - math.tanh(0.5)) < 1e-12
    assert oracle.soft_label(0, 1).tolist() == [1.0]
    with pytest.raises(ValueError):
        oracle.soft_label(6, 6)


def _torch_loss(x, bins, y, h, lam, weight=None):
    t = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64, requires_grad=True)
    w1, b1, w2, b2 = t(h.w1), t(h.b1), t(h.w2), t(h.b2)
    xt, c = torch.tensor(x), torch.tensor(h.centers)
    z = torch.relu(xt @ w1.T + b1) @ w2.T + b2
    logp = torch.log_softmax(z, dim=1)
    K = z.shape[1]
    idx = torch.arange(K, dtype=torch.float64)
    soft = torch.softmax(-(idx[None, :] - torch.tensor(bins, dtype=torch.float64)[:, None]).abs(), dim=1)
    ce = -(soft * logp).sum(1)
    yhat = (logp.exp() * c).sum(1)
    mse = (yhat - torch.tensor(y)) ** 2
    wgt = torch.full((x.shape[0],), 1.0 / x.shape[0], dtype=torch.float64) if weight is None else torch.tensor(weight)
    loss = (wgt * (lam * ce + (1 - lam) * mse)).sum()
    loss.backward()
    return loss.item(), (wgt * ce).sum().item(), (wgt * mse).sum().item(), [p.grad.numpy() for p in (w1, b1, w2, b2)]


@pytest.mark.parametrize("lam", [0.95, 0.3])
def test_loss_and_gradients_match_torch_autograd(lam):
    h = _head(1)
    x, bins, y = _batch(2)
    wgt = np.random.default_rng(3).uniform(0.01, 0.2, size=x.shape[0])
    for weight in (None, wgt):
        loss, gs = oracle.head_loss_grad(x, bins, y, h, lam, weight)
        tl, tce, tmse, tg = _torch_loss(x, bins, y, h, lam, weight)
        assert abs(loss[0] - tl) < 1e-10 * max(1, abs(tl)) and abs(loss[1] - tce) < 1e-12 and abs(loss[2] - tmse) < 1e-8
        for g, t in zip(gs, tg):
            assert _close(g, t, atol=1e-9 * max(1.0, np.abs(t).max()))


def test_gradients_match_finite_differences():
    h = _head(4)
    x, bins, y = _batch(5, B=4)
    lam = 0.8
    _, gs = oracle.head_loss_grad(x, bins, y, h, lam)
    rng = np.random.default_rng(0)
    for arr, g in zip(h.params(), gs):
        flat = arr.reshape(-1)
        for idx in rng.choice(flat.size, size=min(6, flat.size), replace=False):
            old = flat[idx]
            eps = 1e-6
            flat[idx] = old + eps
            lp = oracle.head_loss_grad(x, bins, y, h, lam)[0][0]
            flat[idx] = old - eps
            lm = oracle.head_loss_grad(x, bins, y, h, lam)[0][0]
            flat[idx] = old
            fd = (lp - lm) / (2 * eps)
            assert abs(fd - g.reshape(-1)[idx]) < 1e-5 * max(1.0, abs(fd)), (idx, fd, g.reshape(-1)[idx])


def test_loss_special_cases():
    h = _head(6)
    x, bins, y = _batch(7)
    # lambda = 1: pure cross-entropy, the target length does not matter
    a = oracle.head_loss_grad(x, bins, y, h, 1.0)
    b = oracle.head_loss_grad(x, bins, y + 100.0, h, 1.0)
    assert a[0][0] == b[0][0] and all(np.array_equal(p, q) for p, q in zip(a[1], b[1]))
    # explicit uniform weights equal the default mean over the batch
    u = oracle.head_loss_grad(x, bins, y, h, 0.5, np.full(x.shape[0], 1.0 / x.shape[0]))
    v = oracle.head_loss_grad(x, bins, y, h, 0.5)
    assert _close(u[0], v[0], atol=1e-13) and all(_close(p, q, atol=1e-13) for p, q in zip(u[1], v[1]))
    # lambda = 0 with every prediction on target: zero loss and zero gradient
    from_pred = oracle.predict(x, oracle.Head(h.w1, h.w2, h.b1.astype(np.float32), h.b2.astype(np.float32), h.centers))
    h32 = oracle.TrainHead(h.w1, h.b1.astype(np.float32).astype(np.float64), h.w2,
                           h.b2.astype(np.float32).astype(np.float64), h.centers)
    l, g = oracle.head_loss_grad(x, bins, from_pred, h32, 0.0)
    assert l[0] < 1e-20 and all(np.abs(q).max() < 1e-9 for q in g)
    # cross-entropy is bounded below by the soft label's own entropy
    ent = np.mean([-(oracle.soft_label(i, 6) * np.log(oracle.soft_label(i, 6))).sum() for i in bins])
    assert a[0][1] >= ent - 1e-12


def test_eq9_weights_average_each_sequence_over_its_steps():
    # two sequences with 3 and 1 steps: weights 1/(N T_seq) reproduce the mean of per-sequence means
    h = _head(8)
    x, bins, y = _batch(9, B=4)
    wgt = np.array([1 / 6, 1 / 6, 1 / 6, 1 / 2])
    total = oracle.head_loss_grad(x, bins, y, h, 0.95, wgt)[0][0]
    per = [oracle.head_loss_grad(x[i:i + 1], bins[i:i + 1], y[i:i + 1], h, 0.95)[0][0] for i in range(4)]
    assert abs(total - 0.5 * (np.mean(per[:3]) + per[3])) < 1e-13


def test_adamw_matches_torch_and_first_step_closed_form():
    rng = np.random.default_rng(10)
    w0 = rng.normal(size=50)
    grads = [rng.normal(size=50) * s for s in (1.0, 0.1, 3.0, 1e-9)]
    lr, b1, b2, eps, wd = 2e-5, 0.9, 0.999, 1e-8, 0.01
    w, m, v = w0.copy(), np.zeros(50), np.zeros(50)
    tw = torch.tensor(w0.copy(), requires_grad=True)
    opt = torch.optim.AdamW([tw], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    for t, g in enumerate(grads, 1):
        oracle.adamw_step(w, m, v, np.ascontiguousarray(g), lr, b1, b2, eps, wd, t)
        tw.grad = torch.tensor(g.copy())
        opt.step()
        assert _close(w, tw.detach().numpy(), atol=1e-15)
        if t == 1:
            assert _close(w, w0 - lr * wd * w0 - lr * g / (np.abs(g) + eps), atol=1e-15)


def test_train_step_reduces_the_loss():
    h = _head(11, d=12, d_h=16, K=8)
    x, bins, y = _batch(12, B=32, d=12, K=8)
    y = h.centers[bins] + np.random.default_rng(1).normal(0, 3, size=32)
    first = oracle.train_step(x, bins, y, h, lr=1e-2, weight_decay=0.0)[0]
    for _ in range(60):
        last = oracle.train_step(x, bins, y, h, lr=1e-2, weight_decay=0.0)[0]
    assert last < 0.8 * first and h.t == 61
