"""Pins for the oracle's parameter update rules (CPU only).

Each rule is checked against something other than itself: the library optimisers of torch where the two
definitions coincide (epsilon = 0), closed forms for a constant gradient (which fix where epsilon sits and
the bias correction), explicit sums for the asynchronous accumulators, and the paper's own statement that the
multi-step rule reduces to plain Adam for a single learner.
"""
import numpy as np
import torch

from oracle import update_rules as up


def _grads(seed, steps, n):
    r = np.random.default_rng(seed)
    return [r.standard_normal(n) * 10.0 ** r.uniform(-3, 1, size=n) for _ in range(steps)]


# ---------------- RMSProp ----------------
def test_rmsprop_matches_library_when_eps_is_zero():
    # with eps = 0 "inside the root" and "outside the root" coincide, so torch's routine is a valid check
    n, lr, rho = 40, 7e-4, 0.99
    gs = _grads(0, 6, n)
    th0 = np.random.default_rng(1).standard_normal(n)
    p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.RMSprop([p], lr=lr, alpha=rho, eps=0.0, momentum=0.0, centered=False)
    th, acc = th0.copy(), np.zeros(n)
    for g in gs:
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, acc = up.rmsprop_step(th, acc, g, lr, rho, 0.0)
    np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_rmsprop_constant_gradient_closed_form():
    # accu_k = g^2 (1 - rho^k); theta_K = theta_0 - sum_k lr g / sqrt(accu_k + eps): eps sits inside the root
    g, lr, rho, eps, K = np.array([0.5, -2.0, 1e-3]), 1e-2, 0.9, 1e-6, 7
    th, acc = np.zeros(3), np.zeros(3)
    for _ in range(K):
        th, acc = up.rmsprop_step(th, acc, g, lr, rho, eps)
    want = np.zeros(3)
    for k in range(1, K + 1):
        want -= lr * g / np.sqrt(g * g * (1 - rho ** k) + eps)
    np.testing.assert_allclose(acc, g * g * (1 - rho ** K), rtol=1e-13)
    np.testing.assert_allclose(th, want, rtol=1e-13)
    # eps outside the root would give a measurably different answer for the small-gradient entry
    other = -sum(lr * g[2] / (np.sqrt(g[2] ** 2 * (1 - rho ** k)) + eps) for k in range(1, K + 1))
    assert abs(other - th[2]) > 1e-3 * abs(th[2])


def test_rmsprop_zero_gradient_leaves_theta_and_decays_accu():
    th, acc = up.rmsprop_step(np.array([1.0, -3.0]), np.array([4.0, 0.25]), np.zeros(2), 0.1, 0.9, 1e-6)
    np.testing.assert_array_equal(th, [1.0, -3.0])
    np.testing.assert_allclose(acc, [3.6, 0.225], rtol=1e-15)


# ---------------- Adam ----------------
def test_adam_matches_library_when_eps_is_zero():
    # torch scales eps by the second bias correction and the paper's form does not; at eps = 0 they coincide
    n, r, b1, b2 = 50, 4.2e-4, 0.9, 0.999
    gs = _grads(2, 8, n)
    th0 = np.random.default_rng(3).standard_normal(n)
    p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([p], lr=r, betas=(b1, b2), eps=0.0)
    th, m, v = th0.copy(), np.zeros(n), np.zeros(n)
    for t, g in enumerate(gs, start=1):
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v, _ = up.adam_step(th, m, v, g, t, r, b1, b2, 0.0)
    np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(m, opt.state[p]["exp_avg"].numpy(), rtol=1e-12)
    np.testing.assert_allclose(v, opt.state[p]["exp_avg_sq"].numpy(), rtol=1e-12)


def test_adam_constant_gradient_closed_form():
    # m_t = g (1 - b1^t), v_t = g^2 (1 - b2^t)  =>  s_t = r g sqrt(1 - b2^t) / (|g| sqrt(1 - b2^t) + eps)
    g, r, b1, b2, eps = np.array([3.0, -0.02, 1e-5]), 1e-3, 0.9, 0.999, 0.01 / 256
    th, m, v = np.zeros(3), np.zeros(3), np.zeros(3)
    want = np.zeros(3)
    for t in range(1, 6):
        th, m, v, s = up.adam_step(th, m, v, g, t, r, b1, b2, eps)
        c2 = np.sqrt(1 - b2 ** t)
        s_want = r * g * c2 / (np.abs(g) * c2 + eps)
        np.testing.assert_allclose(s, s_want, rtol=1e-12)
        want -= s_want
    np.testing.assert_allclose(th, want, rtol=1e-12)
    np.testing.assert_allclose(m, g * (1 - b1 ** 5), rtol=1e-13)
    np.testing.assert_allclose(v, g * g * (1 - b2 ** 5), rtol=1e-13)
    # large gradients step by about r, gradients far below eps by about r |g| c2 / eps
    assert abs(abs(s[0]) - r) < 1e-3 * r
    assert abs(s[2]) < 0.05 * r


def test_adam_scale_first_step():
    # t = 1: a = r sqrt(1 - b2) / (1 - b1)
    np.testing.assert_allclose(up.adam_scale(1, 2e-3, 0.9, 0.999), 2e-3 * np.sqrt(1e-3) / 0.1, rtol=1e-12)


# ---------------- multi-step asynchronous Adam ----------------
def test_async_accumulators_are_the_explicit_sums():
    n, r, b1, b2, eps = 12, 3e-4, 0.9, 0.999, 1e-5
    gs = _grads(4, 5, n)
    th0 = np.random.default_rng(5).standard_normal(n)
    L = up.AsyncAdamLearner(th0, np.zeros(n), np.zeros(n))
    steps = []
    th, m, v = th0.copy(), np.zeros(n), np.zeros(n)
    for t, g in enumerate(gs, start=1):
        up.async_adam_local_step(L, g, r, b1, b2, eps)
        th, m, v, s = up.adam_step(th, m, v, g, t, r, b1, b2, eps)
        steps.append(s)
    K = len(gs)
    np.testing.assert_allclose(L.a_g, sum(b1 ** (K - 1 - i) * gs[i] for i in range(K)), rtol=1e-13)
    np.testing.assert_allclose(L.a_g2, sum(b2 ** (K - 1 - i) * gs[i] ** 2 for i in range(K)), rtol=1e-13)
    np.testing.assert_allclose(L.a_s, sum(steps), rtol=1e-13)
    np.testing.assert_allclose(L.theta, th, rtol=1e-14)      # the local rules are plain Adam
    assert L.n == K and L.t == K


def test_async_single_learner_reduces_to_adam():
    # the appendix states this reduction; n local steps then one merge == n plain Adam steps on the central state
    n, r, b1, b2, eps = 30, 4e-4, 0.9, 0.999, 1e-6
    th0 = np.random.default_rng(6).standard_normal(n)
    th_c, m_c, v_c = th0.copy(), np.zeros(n), np.zeros(n)
    L = up.AsyncAdamLearner(th0, np.zeros(n), np.zeros(n))
    th, m, v = th0.copy(), np.zeros(n), np.zeros(n)
    t = 0
    for rounds, nloc in enumerate((1, 3, 4)):
        for g in _grads(10 + rounds, nloc, n):
            t += 1
            up.async_adam_local_step(L, g, r, b1, b2, eps)
            th, m, v, _ = up.adam_step(th, m, v, g, t, r, b1, b2, eps)
        th_c, m_c, v_c = up.async_adam_merge(L, th_c, m_c, v_c, b1, b2)
        np.testing.assert_allclose(th_c, th, rtol=1e-12, atol=1e-15)
        np.testing.assert_allclose(m_c, m, rtol=1e-12, atol=1e-18)
        np.testing.assert_allclose(v_c, v, rtol=1e-12, atol=1e-18)
        for loc, cen in ((L.theta, th_c), (L.m, m_c), (L.v, v_c)):
            np.testing.assert_array_equal(loc, cen)
        assert L.n == 0 and not L.a_g.any() and not L.a_g2.any() and not L.a_s.any()


def test_async_two_learners_merge_is_additive_in_steps():
    # two learners start from the same central state and merge one after the other: the central parameters
    # move by the sum of both learners' steps, and the central moments decay by beta^n per merge
    n, r, b1, b2, eps = 9, 1e-3, 0.9, 0.99, 1e-4
    th0 = np.random.default_rng(7).standard_normal(n)
    m0 = np.random.default_rng(8).standard_normal(n) * 0.1
    v0 = np.random.default_rng(9).random(n) * 0.1
    A = up.AsyncAdamLearner(th0, m0, v0)
    Bl = up.AsyncAdamLearner(th0, m0, v0)
    ga, gb = _grads(20, 2, n), _grads(21, 3, n)
    for g in ga:
        up.async_adam_local_step(A, g, r, b1, b2, eps)
    for g in gb:
        up.async_adam_local_step(Bl, g, r, b1, b2, eps)
    sa, sb = A.a_s.copy(), Bl.a_s.copy()
    aga, agb = A.a_g.copy(), Bl.a_g.copy()
    th_c, m_c, v_c = up.async_adam_merge(A, th0, m0, v0, b1, b2)
    th_c, m_c, v_c = up.async_adam_merge(Bl, th_c, m_c, v_c, b1, b2)
    np.testing.assert_allclose(th_c, th0 - sa - sb, rtol=1e-13)
    np.testing.assert_allclose(m_c, b1 ** 3 * (b1 ** 2 * m0 + (1 - b1) * aga) + (1 - b1) * agb, rtol=1e-13)
    np.testing.assert_array_equal(Bl.theta, th_c)
    assert not np.array_equal(A.theta, th_c)          # A still holds the values of its own merge
