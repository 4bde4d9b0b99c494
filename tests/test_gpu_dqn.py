"""GPU parity of the action-value heads, the DQN objective and the action draws, through the C ABI."""
import numpy as np
import pytest

import workloads as wl
from oracle import nature_cnn as orc
from tests.gpu_util import GpuNet, check_grads, per_tensor, tol_check, train_c51_or_dqn

pytestmark = pytest.mark.gpu


def _dqn_batch(B, A, seed=7):
    b = wl.c51_batch(5, B=B)
    b["action"] = (b["action"] % A).astype(np.int32)
    b["done"][: min(B, 3)] = 1
    return b


@pytest.mark.parametrize("head,A,B", [("q", 18, 70), ("duel", 18, 70), ("q", 1, 5), ("duel", 31, 33), ("q", 6, 1)])
def test_action_value_inference(head, A, B):
    flat = wl.he_normal_params(A, head, seed=2500 + A, bias_std=0.05)
    obs = wl.rect_frames(B, seed=1500 + A)
    spec = orc.NetSpec(A, head)
    ref = orc.forward(orc.unflatten(flat, spec), obs, spec)["q"]
    out = GpuNet(A, head, flat).forward(obs)
    tol_check(out["q"], ref, "q")
    tol_check(out["value"], ref.max(axis=1), "max q")
    clear = orc.top2_gap(ref) > 1e-2
    np.testing.assert_array_equal(out["greedy"][clear], orc.greedy(ref)[clear])
    np.testing.assert_array_equal(out["greedy"], np.argmax(out["q"], axis=1))      # self-consistent everywhere


@pytest.mark.parametrize("head,double_q,B", [("q", 0, 150), ("q", 1, 150), ("duel", 1, 150), ("duel", 0, 3)])
def test_dqn_gradients(head, double_q, B):
    A = 18
    flat = wl.he_normal_params(A, head, seed=2600, bias_std=0.02)
    tflat = wl.he_normal_params(A, head, seed=3600, bias_std=0.02)
    batch = _dqn_batch(B, A)
    spec = orc.NetSpec(A, head)
    net = GpuNet(A, head, flat, double_q=double_q)
    dW, loss, ref, _ = train_c51_or_dqn(net, orc, flat, tflat, batch, "dqn", spec, hyper=orc.Hyper(double_q=bool(double_q)))
    got, want = per_tensor(dW, A, head), per_tensor(ref["flat"], A, head)
    check_grads(got, want, "dqn %s double=%d B=%d" % (head, double_q, B))
    assert abs(loss[0] - ref["loss"]["total"]) <= 1e-2 * abs(ref["loss"]["total"]) + 1e-3
    assert loss[1] == pytest.approx(loss[0]) and loss[2] == 0 and loss[3] == 0
    # most of this batch is decided by clear margins, so the equality part of the greedy rule is exercised
    assert (orc.top2_gap(ref["select_q"]) > 1e-2).mean() > 0.9


def test_categorical_draw_matches_the_oracle():
    A, B = 18, 300
    flat = wl.he_normal_params(A, "pv", seed=2700, bias_std=0.05)
    obs = wl.rect_frames(B, seed=1700)
    un = wl.action_uniforms(B, seed=1)
    spec = orc.NetSpec(A, "pv")
    cache = orc.forward(orc.unflatten(flat, spec), obs, spec)
    probs = np.exp(orc.log_softmax(cache["logits"]))
    want = orc.sample_categorical(probs, un["u"])
    act, logp = GpuNet(A, "pv", flat).act(obs, un["u"], un["u2"], want_logp=True)
    assert ((act >= 0) & (act < A)).all()
    # the draw is a threshold decision on the CDF, as the greedy action is one on the logits: it is compared
    # where u is clear of every CDF boundary by 5e-3 (the greedy rule's top-2 gap of 1e-2, half for each side:
    # a boundary moves by no more than the logits' error); elsewhere either neighbour is a correct draw
    cdf = np.cumsum(probs, axis=1)
    margin = np.abs(cdf - un["u"][:, None].astype(np.float64)).min(axis=1)
    clear = margin > 5e-3
    assert clear.mean() > 0.75
    np.testing.assert_array_equal(act[clear], want[clear])
    near = ~clear
    assert (np.abs(act[near].astype(int) - want[near]) <= 1).all()
    lp_ref = orc.log_softmax(cache["logits"])[np.arange(B), act]
    tol_check(logp, lp_ref, "log pi(drawn action)")
    assert len(np.unique(act)) > 5                                   # a real spread of actions, not one mode


@pytest.mark.parametrize("head", ["q", "duel", "c51"])
def test_epsilon_greedy_draw(head):
    A, B, eps = 18, 200, 0.3
    flat = wl.he_normal_params(A, head, seed=2800, bias_std=0.05)
    obs = wl.rect_frames(B, seed=1800)
    un = wl.action_uniforms(B, seed=2)
    spec = orc.NetSpec(A, head)
    cache = orc.forward(orc.unflatten(flat, spec), obs, spec)
    if head == "c51":
        p = np.exp(orc.log_softmax(cache["atom_logits"]))
        q = (p * orc.c51_support(51, -10.0, 10.0)).sum(axis=-1)
    else:
        q = cache["q"]
    want = orc.epsilon_greedy(q, un["u"], un["u2"], float(np.float32(eps)))    # the C ABI takes epsilon as fp32
    act, _ = GpuNet(A, head, flat).act(obs, un["u"], un["u2"], epsilon=eps)
    explore = un["u"] < np.float32(eps)
    assert 0.15 < explore.mean() < 0.45
    np.testing.assert_array_equal(act[explore], want[explore])          # random actions are exact integer work
    clear = ~explore & (orc.top2_gap(q) > 1e-2)
    np.testing.assert_array_equal(act[clear], want[clear])
    assert ((act >= 0) & (act < A)).all()
    # epsilon = 0 is pure greedy, epsilon = 1 pure random
    act0, _ = GpuNet(A, head, flat).act(obs, un["u"], un["u2"], epsilon=0.0)
    np.testing.assert_array_equal(act0[orc.top2_gap(q) > 1e-2], orc.greedy(q)[orc.top2_gap(q) > 1e-2])
    act1, _ = GpuNet(A, head, flat).act(obs, un["u"], un["u2"], epsilon=1.0)
    np.testing.assert_array_equal(act1, np.minimum((un["u2"].astype(np.float64) * A).astype(int), A - 1))
