"""Pins for the reference AdamW update and learning-rate schedule."""
import math

import numpy as np

import oracle


def test_first_step_closed_form():
    g = np.array([0.3, -2.0, 1e-3, 5.0])
    w = np.array([1.0, -1.0, 0.5, 2.0])
    lr, eps, wd = 1e-2, 1e-8, 0.1
    w1, m1, v1 = oracle.adamw_update(w, g, np.zeros(4), np.zeros(4), 1, lr, 0.9, 0.95, eps, wd)
    # bias correction makes m_hat = g and v_hat = g^2 at t = 1
    expect = w - lr * (g / (np.abs(g) + eps) + wd * w)
    assert np.max(np.abs(w1 - expect)) < 1e-15
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.05 * g * g)


def test_zero_grad_no_decay_is_identity_and_decay_is_decoupled():
    w = np.array([1.0, -3.0])
    w1, m1, v1 = oracle.adamw_update(w, np.zeros(2), np.zeros(2), np.zeros(2), 1, 1e-3, 0.9, 0.95, 1e-8, 0.0)
    assert np.array_equal(w1, w) and not m1.any() and not v1.any()
    w2, _, _ = oracle.adamw_update(w, np.zeros(2), np.zeros(2), np.zeros(2), 1, 1e-3, 0.9, 0.95, 1e-8, 0.1)
    assert np.max(np.abs(w2 - w * (1 - 1e-4))) < 1e-15        # pure shrink, no moment involved


def test_second_step_by_hand():
    g1, g2 = 2.0, -1.0
    b1, b2, lr, eps = 0.9, 0.95, 0.1, 1e-8
    w, m, v = np.array([1.0]), np.zeros(1), np.zeros(1)
    w, m, v = oracle.adamw_update(w, np.array([g1]), m, v, 1, lr, b1, b2, eps, 0.0)
    w, m, v = oracle.adamw_update(w, np.array([g2]), m, v, 2, lr, b1, b2, eps, 0.0)
    m2 = b1 * (1 - b1) * g1 + (1 - b1) * g2
    v2 = b2 * (1 - b2) * g1 ** 2 + (1 - b2) * g2 ** 2
    step2 = (m2 / (1 - b1 ** 2)) / (math.sqrt(v2 / (1 - b2 ** 2)) + eps)
    assert abs(w[0] - (1.0 - lr * g1 / (abs(g1) + eps) - lr * step2)) < 1e-14


def test_matches_torch_adamw_over_several_steps():
    import torch
    rs = np.random.default_rng(0)
    w0 = rs.standard_normal(50)
    p = torch.tensor(w0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=2e-5, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    w, m, v = w0.copy(), np.zeros(50), np.zeros(50)
    for t in range(1, 6):
        g = rs.standard_normal(50)
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        w, m, v = oracle.adamw_update(w, g, m, v, t, 2e-5, 0.9, 0.95, 1e-8, 0.1)
    assert np.max(np.abs(w - p.detach().numpy())) < 1e-12


def test_cosine_schedule_shape():
    total, peak = 200, 2e-4
    lrs = [oracle.cosine_lr(s, total, peak) for s in range(total)]
    assert abs(max(lrs) - peak) < 1e-15 and lrs.index(max(lrs)) == 9       # 5 % of 200 = 10 warm-up steps
    assert all(lrs[i] < lrs[i + 1] for i in range(9))
    assert all(lrs[i] >= lrs[i + 1] for i in range(9, total - 1))
    assert lrs[-1] < 1e-3 * peak * 5
