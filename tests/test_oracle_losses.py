"""Pins for the oracle's objectives and their gradients (CPU only)."""
import os

import numpy as np
import pytest
from scipy.special import logsumexp

from oracle import nature_cnn as orc


def _fd(f, x, h=1e-6):
    """Central finite differences of scalar f at array x."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        g[i] = (f(xp) - f(xm)) / (2 * h)
    return g


def _ac_inputs(seed=0, B=6, A=5):
    r = np.random.default_rng(seed)
    return dict(logits=r.standard_normal((B, A)) * 1.5, value=r.standard_normal(B),
                action=r.integers(0, A, size=B), adv=r.standard_normal(B), ret=r.standard_normal(B))


# ---------------- softmax / entropy ----------------
def test_log_softmax_properties():
    r = np.random.default_rng(1)
    z = r.standard_normal((7, 18)) * 3
    lp = orc.log_softmax(z)
    np.testing.assert_allclose(np.exp(lp).sum(axis=1), 1.0, atol=1e-14)
    np.testing.assert_allclose(lp, z - logsumexp(z, axis=1, keepdims=True), atol=1e-13)   # library routine
    np.testing.assert_allclose(orc.log_softmax(z + 123.0), lp, atol=1e-12)               # shift invariance
    # large logits do not overflow
    assert np.isfinite(orc.log_softmax(np.array([[1000.0, 0.0, -1000.0]]))).all()


def test_entropy_closed_forms():
    for A in (2, 6, 18):
        np.testing.assert_allclose(orc.entropy(orc.log_softmax(np.zeros((1, A)))), np.log(A), atol=1e-14)
    # two-point distribution p, 1-p
    p = 0.3
    z = np.log(np.array([[p, 1 - p]]))
    np.testing.assert_allclose(orc.entropy(orc.log_softmax(z)), -(p * np.log(p) + (1 - p) * np.log(1 - p)), atol=1e-14)


def test_greedy_lowest_index_on_ties():
    assert orc.greedy(np.array([[1.0, 3.0, 3.0, 2.0]]))[0] == 1
    np.testing.assert_allclose(orc.top2_gap(np.array([[1.0, 3.0, 2.5]])), 0.5)


# ---------------- A2C ----------------
def test_a2c_value_by_hand():
    # one sample, two actions, logits (0, ln 3): p = (1/4, 3/4)
    logits = np.array([[0.0, np.log(3.0)]])
    out = orc.a2c_loss_value(logits, np.array([2.0]), np.array([1]), np.array([2.0]), np.array([0.5]))
    H = -(0.25 * np.log(0.25) + 0.75 * np.log(0.75))
    assert np.isclose(out["policy"], -np.log(0.75) * 2.0)
    assert np.isclose(out["value"], 1.5 ** 2)
    assert np.isclose(out["entropy"], H)
    assert np.isclose(out["total"], -np.log(0.75) * 2.0 + 0.5 * 2.25 - 0.01 * H)


def test_a2c_grad_matches_finite_differences():
    d = _ac_inputs(2)
    dz, dv = orc.a2c_loss_grad(**d)
    f_z = lambda z: orc.a2c_loss_value(z, d["value"], d["action"], d["adv"], d["ret"])["total"]
    f_v = lambda v: orc.a2c_loss_value(d["logits"], v, d["action"], d["adv"], d["ret"])["total"]
    np.testing.assert_allclose(dz, _fd(f_z, d["logits"]), atol=1e-8)
    np.testing.assert_allclose(dv, _fd(f_v, d["value"]), atol=1e-8)
    np.testing.assert_allclose(dz.sum(axis=1), 0.0, atol=1e-15)        # softmax rows: gradients sum to 0
    np.testing.assert_allclose(dv, (d["value"] - d["ret"]) / len(dv), atol=1e-15)


def test_a2c_entropy_term_sign():
    """A uniform policy maximises entropy: its entropy gradient vanishes, and a
    peaked policy is pushed towards uniform (the taken logit's gradient is > 0
    for the loss, i.e. descent lowers the largest logit) with zero advantage."""
    z = np.array([[3.0, 0.0, 0.0]])
    dz, _ = orc.a2c_loss_grad(z, np.zeros(1), np.array([0]), np.zeros(1), np.zeros(1))
    assert dz[0, 0] > 0 and dz[0, 1] < 0
    dz, _ = orc.a2c_loss_grad(np.zeros((1, 3)), np.zeros(1), np.array([0]), np.zeros(1), np.zeros(1))
    np.testing.assert_allclose(dz, 0.0, atol=1e-16)


# ---------------- PPO ----------------
def test_ppo_grad_matches_finite_differences_away_from_kinks():
    d = _ac_inputs(3, B=12)
    lp = orc.log_softmax(d["logits"])[np.arange(12), d["action"]]
    r = np.random.default_rng(30)
    old = lp + r.choice([-0.2, -0.04, 0.04, 0.2], size=12)     # rho in {1.22, 1.04, .96, .82}: both branches
    dz, dv = orc.ppo_loss_grad(**d, old_logp=old)
    f_z = lambda z: orc.ppo_loss_value(z, d["value"], d["action"], d["adv"], d["ret"], old)["total"]
    np.testing.assert_allclose(dz, _fd(f_z, d["logits"]), atol=1e-8)
    rho = np.exp(lp - old)
    act = orc.ppo_active(rho, d["adv"])
    assert act.any() and (~act).any()


def test_ppo_reduces_to_a2c_policy_gradient():
    """With old = current policy and no clipping in reach, rho = 1 and the
    surrogate's gradient equals the advantage-weighted log-likelihood gradient."""
    d = _ac_inputs(4)
    lp = orc.log_softmax(d["logits"])[np.arange(6), d["action"]]
    dz_p, dv_p = orc.ppo_loss_grad(**d, old_logp=lp, clip_eps=1e9)
    dz_a, dv_a = orc.a2c_loss_grad(**d)
    np.testing.assert_allclose(dz_p, dz_a, atol=1e-15)
    np.testing.assert_allclose(dv_p, dv_a, atol=1e-15)
    # and the surrogate's value is then -mean(adv)
    v = orc.ppo_loss_value(**d, old_logp=lp)
    assert np.isclose(v["policy"], -d["adv"].mean())


def test_ppo_clip_cases_by_hand():
    # one sample, rho = 1.5 (> 1+eps): positive advantage -> clipped, zero policy gradient, value 1.1 A
    z = np.zeros((1, 2))
    lp = np.log(0.5)
    old = np.array([lp - np.log(1.5)])
    for adv, want_val, active in [(2.0, -1.1 * 2.0, False), (-2.0, 1.5 * 2.0, True)]:
        v = orc.ppo_loss_value(z, np.zeros(1), np.array([0]), np.array([adv]), np.zeros(1), old)
        assert np.isclose(v["policy"], want_val)
        dz, _ = orc.ppo_loss_grad(z, np.zeros(1), np.array([0]), np.array([adv]), np.zeros(1), old,
                                  entropy_coef=0.0)
        assert (np.abs(dz).max() > 0) == active
    # boundary is inclusive: rho exactly 1+eps with A>0 still passes gradient
    assert orc.ppo_active(np.array([1.1]), np.array([1.0]), 0.1)[0]
    assert orc.ppo_active(np.array([0.9]), np.array([-1.0]), 0.1)[0]


# ---------------- C51 ----------------
def _golden(path):
    out = {}
    for line in open(path):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            out[k] = np.array([float(t) for t in v])
    return out


def test_c51_projection_hand_worked(golden_dir):
    g = _golden(os.path.join(golden_dir, "c51_projection_n3.txt"))
    p = np.array([[0.2, 0.3, 0.5]])
    m = orc.c51_project(p, np.array([0.25]), np.array([0.0]), gamma=0.5, v_min=-1.0, v_max=1.0)
    np.testing.assert_allclose(m[0], g["m"], atol=1e-15)
    m = orc.c51_project(p, np.array([0.25]), np.array([1.0]), gamma=0.5, v_min=-1.0, v_max=1.0)
    np.testing.assert_allclose(m[0], g["m_done"], atol=1e-15)


def _rand_dist(r, B, N=51):
    p = r.random((B, N)) ** 3
    return p / p.sum(axis=1, keepdims=True)


def test_c51_projection_mass_and_mean():
    r = np.random.default_rng(5)
    B = 64
    p = _rand_dist(r, B)
    rew = r.integers(-1, 2, size=B).astype(np.float64)
    done = (r.random(B) < 0.3).astype(np.float64)
    m = orc.c51_project(p, rew, done)
    np.testing.assert_allclose(m.sum(axis=1), 1.0, atol=1e-13)
    assert (m >= 0).all()
    # no clipping happens for |r| <= 1, gamma = .99 on [-10,10] only if |r + .99 z| <= 10: z in +-10 -> 9.9+1 > 10.
    # so test mean preservation on a narrower distribution (atoms 5..45 only)
    q = np.zeros_like(p)
    q[:, 5:46] = p[:, 5:46]
    q /= q.sum(axis=1, keepdims=True)
    z = orc.c51_support()
    mq = orc.c51_project(q, rew, done)
    np.testing.assert_allclose(mq @ z, rew + 0.99 * (1 - done) * (q @ z), atol=1e-12)


def test_c51_projection_special_cases():
    r = np.random.default_rng(6)
    p = _rand_dist(r, 4)
    z = orc.c51_support()
    # identity: r = 0, gamma = 1, not terminal
    np.testing.assert_allclose(orc.c51_project(p, np.zeros(4), np.zeros(4), gamma=1.0), p, atol=1e-15)
    # terminal with r = 0: everything on the atom z_25 = 0 exactly (the case a floor/ceil scatter drops)
    m = orc.c51_project(p, np.zeros(4), np.ones(4))
    want = np.zeros_like(p)
    want[:, 25] = 1.0
    np.testing.assert_allclose(m, want, atol=1e-13)
    assert z[25] == 0.0
    # terminal, r = 1: split between z = 0.8 (atom 27) and 1.2 (atom 28), mean 1
    m = orc.c51_project(p, np.ones(4), np.ones(4))
    np.testing.assert_allclose(m[:, 27], 0.5, atol=1e-12)
    np.testing.assert_allclose(m[:, 28], 0.5, atol=1e-12)
    np.testing.assert_allclose(m @ z, 1.0, atol=1e-12)
    # clipping: huge reward puts everything on the last atom
    m = orc.c51_project(p, np.full(4, 100.0), np.zeros(4))
    np.testing.assert_allclose(m[:, -1], 1.0, atol=1e-13)


def test_c51_gather_equals_scatter_form():
    r = np.random.default_rng(7)
    B = 16
    p = _rand_dist(r, B)
    rew = r.standard_normal(B) * 0.7          # non-integer positions
    done = (r.random(B) < 0.2).astype(np.float64)
    np.testing.assert_allclose(orc.c51_project(p, rew, done), orc.c51_project_scatter(p, rew, done), atol=1e-13)


def test_c51_target_picks_best_expected_value():
    r = np.random.default_rng(8)
    B, A, N = 5, 4, 51
    z = r.standard_normal((B, A, N))
    z[2, 3, 45:] += 6.0                       # action 3 of sample 2 gets mass on high atoms
    t = orc.c51_target(z, np.zeros(B), np.zeros(B), gamma=1.0)
    assert t["a_star"][2] == 3
    p = np.exp(orc.log_softmax(z))
    np.testing.assert_allclose(t["q"], (p * orc.c51_support()).sum(axis=2), atol=1e-13)
    np.testing.assert_allclose(t["m"], p[np.arange(B), t["a_star"]], atol=1e-14)   # identity projection


def test_c51_target_with_a_given_next_action():
    """The next action handed in replaces the argmax and nothing else: with gamma = 1, r = 0 the projection is the
    identity, so m is that action's distribution; handing in the argmax itself changes nothing."""
    r = np.random.default_rng(18)
    B, A, N = 6, 5, 51
    z = r.standard_normal((B, A, N))
    p = np.exp(orc.log_softmax(z))
    own = orc.c51_target(z, np.zeros(B), np.zeros(B), gamma=1.0)
    same = orc.c51_target(z, np.zeros(B), np.zeros(B), gamma=1.0, a_star=own["a_star"])
    np.testing.assert_array_equal(same["m"], own["m"])
    pick = (own["a_star"] + np.array([0, 1, 0, 2, 0, 0])) % A
    t = orc.c51_target(z, np.zeros(B), np.zeros(B), gamma=1.0, a_star=pick)
    np.testing.assert_array_equal(t["a_star"], pick)
    np.testing.assert_allclose(t["m"], p[np.arange(B), pick], atol=1e-14)
    unchanged = pick == own["a_star"]
    np.testing.assert_array_equal(t["m"][unchanged], own["m"][unchanged])
    assert (np.abs(t["m"][~unchanged] - own["m"][~unchanged]).max(axis=1) > 1e-3).all()
    np.testing.assert_array_equal(t["q"], own["q"])                   # the action values themselves do not depend on it


def test_c51_loss_grad_matches_finite_differences():
    r = np.random.default_rng(9)
    B, A, N = 3, 4, 7
    z = r.standard_normal((B, A, N))
    a = r.integers(0, A, size=B)
    m = _rand_dist(r, B, N)
    d = orc.c51_loss_grad(z, a, m)
    f = lambda zz: orc.c51_loss_value(zz, a, m)["total"]
    np.testing.assert_allclose(d, _fd(f, z), atol=1e-8)
    for n in range(B):
        for k in range(A):
            if k != a[n]:
                assert (d[n, k] == 0).all()
        assert abs(d[n, a[n]].sum()) < 1e-15
    # cross-entropy of a distribution with itself is its entropy
    lp = orc.log_softmax(z)[np.arange(B), a]
    v = orc.c51_loss_value(z, a, np.exp(lp))
    assert np.isclose(v["total"], orc.entropy(lp).mean())
