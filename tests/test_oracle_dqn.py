"""Pins for the oracle's DQN objective, dueling aggregation and action selection (CPU only)."""
import numpy as np
import pytest

from oracle import nature_cnn as orc


def _fd(f, x, h=1e-6):
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        i = it.multi_index
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        g[i] = (f(xp) - f(xm)) / (2 * h)
    return g


# ---------------- DQN target and loss ----------------
def test_dqn_hand_example():
    # Q(s) = [1, 2], a = 0, r = 1, gamma = 0.5, Q(s'; theta-) = [3, 0]  =>  y = 2.5, loss = 2.25, dL/dQ[0] = -3
    q, qn = np.array([[1.0, 2.0]]), np.array([[3.0, 0.0]])
    y = orc.dqn_target(qn, [1.0], [0], 0.5)
    np.testing.assert_allclose(y, [2.5])
    assert orc.dqn_loss_value(q, [0], y)["total"] == pytest.approx(2.25)
    np.testing.assert_allclose(orc.dqn_loss_grad(q, [0], y), [[-3.0, 0.0]])


def test_dqn_terminal_and_double():
    qn_t = np.array([[3.0, 0.0], [3.0, 0.0], [1.0, 4.0]])
    qn_o = np.array([[0.0, 5.0], [0.0, 5.0], [2.0, 1.0]])
    # terminal transition: y = r
    np.testing.assert_allclose(orc.dqn_target(qn_t, [1.0, 1.0, 1.0], [0, 1, 0], 0.9), [1 + 2.7, 1.0, 1 + 3.6])
    # Double-DQN: the online values pick the action, the target values price it
    np.testing.assert_allclose(orc.dqn_target(qn_t, [1.0, 1.0, 1.0], [0, 1, 0], 0.9, qn_o), [1.0 + 0.0, 1.0, 1 + 0.9])
    # ties go to the lowest index
    np.testing.assert_allclose(orc.dqn_target(np.array([[2.0, 2.0]]), [0.0], [0], 1.0, np.array([[7.0, 7.0]])), [2.0])
    # a next action handed in replaces the argmax (of either network) and is priced by the target values
    np.testing.assert_allclose(orc.dqn_target(qn_t, [1.0, 1.0, 1.0], [0, 1, 0], 0.9, a_star=[1, 0, 0]), [1.0, 1.0, 1 + 0.9])
    np.testing.assert_allclose(orc.dqn_target(qn_t, [1.0, 1.0, 1.0], [0, 1, 0], 0.9, qn_o, a_star=[0, 0, 1]),
                               [1 + 2.7, 1.0, 1 + 3.6])


def test_dqn_grad_matches_finite_differences_and_brute_force():
    r = np.random.default_rng(0)
    B, A = 7, 5
    q, a, y = r.standard_normal((B, A)), r.integers(0, A, B), r.standard_normal(B)
    g = orc.dqn_loss_grad(q, a, y)
    np.testing.assert_allclose(g, _fd(lambda x: orc.dqn_loss_value(x, a, y)["total"], q), atol=1e-8)
    brute = sum((y[n] - q[n, a[n]]) ** 2 for n in range(B)) / B
    assert orc.dqn_loss_value(q, a, y)["total"] == pytest.approx(brute, rel=1e-14)
    assert (g != 0).sum() <= B                       # only the taken actions carry gradient


# ---------------- dueling aggregation ----------------
def test_dueling_hand_example_and_invariants():
    np.testing.assert_allclose(orc.dueling_aggregate([[1.0, 2.0, 3.0]], [1.0]), [[0.0, 1.0, 2.0]])
    r = np.random.default_rng(1)
    adv, val = r.standard_normal((6, 4)), r.standard_normal(6)
    q = orc.dueling_aggregate(adv, val)
    np.testing.assert_allclose(q.mean(axis=1), val, atol=1e-14)                       # mean_a Q = V
    np.testing.assert_allclose(orc.dueling_aggregate(adv + 3.7, val), q, atol=1e-13)  # advantage shift invariance
    np.testing.assert_array_equal(orc.greedy(q), orc.greedy(adv))                    # same ranking as the advantages


def test_dueling_grad_is_the_adjoint():
    r = np.random.default_rng(2)
    adv, val, dq = r.standard_normal((5, 6)), r.standard_normal(5), r.standard_normal((5, 6))
    dadv, dval = orc.dueling_aggregate_grad(dq)
    f = lambda a_, v_: float((orc.dueling_aggregate(a_, v_) * dq).sum())
    np.testing.assert_allclose(dadv, _fd(lambda x: f(x, val), adv), atol=1e-8)
    np.testing.assert_allclose(dval, _fd(lambda x: f(adv, x), val), atol=1e-8)


# ---------------- action selection ----------------
def test_categorical_draw_inverse_cdf():
    p = np.array([[0.2, 0.0, 0.5, 0.3]])
    for u, want in [(0.0, 0), (0.1999, 0), (0.2, 2), (0.6999, 2), (0.7, 3), (0.9999, 3)]:
        assert orc.sample_categorical(p, np.array([u]))[0] == want, u
    # a zero-probability action is never drawn; frequencies over a fine grid of u reproduce the probabilities
    u = (np.arange(10000) + 0.5) / 10000
    draws = orc.sample_categorical(np.repeat(p, u.size, axis=0), u)
    np.testing.assert_allclose(np.bincount(draws, minlength=4) / u.size, p[0], atol=1e-4)
    # rounding that leaves the total below u falls back to the last action
    assert orc.sample_categorical(np.array([[0.5, 0.4999999]]), np.array([0.99999999]))[0] == 1


def test_epsilon_greedy():
    q = np.array([[0.0, 2.0, 2.0, 1.0]] * 4)
    u = np.array([0.05, 0.0999, 0.1, 0.9])
    u2 = np.array([0.0, 0.76, 0.99, 0.3])
    np.testing.assert_array_equal(orc.epsilon_greedy(q, u, u2, 0.1), [0, 3, 1, 1])    # explore, explore, greedy, greedy
    np.testing.assert_array_equal(orc.epsilon_greedy(q, u, u2, 0.0), [1, 1, 1, 1])
    assert orc.epsilon_greedy(q[:1], np.array([0.0]), np.array([0.99999999]), 1.0)[0] == 3


# ---------------- network level ----------------
TINY = orc.Geometry(in_ch=2, in_h=12, in_w=12, convs=((3, 4, 2, 0), (4, 3, 1, 0)), hidden=6)


def test_dueling_network_is_the_pv_network_recombined():
    # the two heads share one flat layout: Q = value + logits - mean(logits) of the same parameters
    r = np.random.default_rng(3)
    sp_d, sp_p = orc.NetSpec(5, "duel", geometry=TINY), orc.NetSpec(5, "pv", geometry=TINY)
    assert orc.param_count(sp_d) == orc.param_count(sp_p)
    flat = r.standard_normal(orc.param_count(sp_d)) * 0.3
    obs = r.integers(0, 256, size=(4, 2, 12, 12), dtype=np.uint8)
    cd = orc.forward(orc.unflatten(flat, sp_d), obs, sp_d)
    cp = orc.forward(orc.unflatten(flat, sp_p), obs, sp_p)
    want = cp["value"][:, None] + cp["logits"] - cp["logits"].mean(axis=1, keepdims=True)
    np.testing.assert_allclose(cd["q"], want, atol=1e-13)


@pytest.mark.parametrize("head,double_q", [("q", False), ("q", True), ("duel", True)])
def test_dqn_step_gradient_matches_finite_differences(head, double_q):
    r = np.random.default_rng(4)
    spec = orc.NetSpec(3, head, geometry=TINY)
    n = orc.param_count(spec)
    flat, tflat = r.standard_normal(n) * 0.4, r.standard_normal(n) * 0.4
    B = 5
    batch = dict(obs=r.integers(0, 256, size=(B, 2, 12, 12), dtype=np.uint8),
                 next_obs=r.integers(0, 256, size=(B, 2, 12, 12), dtype=np.uint8),
                 action=r.integers(0, 3, B), reward=r.standard_normal(B), done=np.array([0, 1, 0, 0, 0]))
    hyp = orc.Hyper(gamma=0.9, double_q=double_q)
    out = orc.train_step_grads(flat, batch, "dqn", spec, hyp, flat_target_params=tflat)
    y = out["target"]                                       # a constant of the step

    def loss(x):
        c = orc.forward(orc.unflatten(x, spec), batch["obs"], spec)
        return orc.dqn_loss_value(c["q"], batch["action"], y)["total"]

    idx = r.choice(n, size=60, replace=False)
    fd = np.zeros(60)
    for j, i in enumerate(idx):
        xp, xm = flat.copy(), flat.copy()
        xp[i] += 1e-6
        xm[i] -= 1e-6
        fd[j] = (loss(xp) - loss(xm)) / 2e-6
    np.testing.assert_allclose(out["flat"][idx], fd, rtol=2e-5, atol=1e-8)
    assert y[1] == batch["reward"][1]                       # the terminal transition does not bootstrap


@pytest.mark.parametrize("head,kind,double_q", [("q", "dqn", False), ("duel", "dqn", True), ("c51", "c51", False)])
def test_step_with_a_given_next_action(head, kind, double_q):
    """train_step_grads with the next actions handed in: its own greedy actions reproduce the step bit for bit,
    and changing one sample's next action changes the step exactly as if only that sample's target had changed
    (every objective is a batch mean: the two-sample batch's gradient is the mean of the one-sample gradients)."""
    r = np.random.default_rng(14)
    spec = orc.NetSpec(3, head, num_atoms=5, geometry=TINY) if head == "c51" else orc.NetSpec(3, head, geometry=TINY)
    n = orc.param_count(spec)
    flat, tflat = r.standard_normal(n) * 0.4, r.standard_normal(n) * 0.4
    B = 2
    batch = dict(obs=r.integers(0, 256, size=(B, 2, 12, 12), dtype=np.uint8),
                 next_obs=r.integers(0, 256, size=(B, 2, 12, 12), dtype=np.uint8),
                 action=r.integers(0, 3, B), reward=r.standard_normal(B), done=np.zeros(B, dtype=np.uint8))
    hyp = orc.Hyper(gamma=0.9, double_q=double_q, v_min=-2.0, v_max=2.0)
    step = lambda b, na=None: orc.train_step_grads(flat, b, kind, spec, hyp, flat_target_params=tflat, next_action=na)
    own = step(batch)
    sel_params = flat if double_q else tflat
    c = orc.forward(orc.unflatten(sel_params, spec), batch["next_obs"], spec)
    if head == "c51":
        p = np.exp(orc.log_softmax(c["atom_logits"]))
        want_q = p @ orc.c51_support(5, -2.0, 2.0)
    else:
        want_q = c["q"]
    np.testing.assert_allclose(own["select_q"], want_q, atol=1e-13)
    np.testing.assert_array_equal(own["next_action"], orc.greedy(want_q))
    same = step(batch, own["next_action"])
    np.testing.assert_array_equal(same["flat"], own["flat"])
    other = own["next_action"].copy()
    other[1] = (other[1] + 1) % 3
    changed = step(batch, other)
    np.testing.assert_array_equal(changed["next_action"], other)
    one = lambda i, na: step({k: v[i:i + 1] for k, v in batch.items()}, na[i:i + 1])["flat"]
    np.testing.assert_allclose(changed["flat"], 0.5 * (one(0, other) + one(1, other)), atol=1e-12)
    np.testing.assert_allclose(one(0, other), one(0, own["next_action"]), atol=0)
    assert np.abs(one(1, other) - one(1, own["next_action"])).max() > 1e-6
