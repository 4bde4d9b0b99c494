"""GPU parity of the parameter update rules against the fp64 oracle, through the C ABI.

Tolerance: every rule is a handful of fp32 operations per element and step, each rounded to 2^-24 relative,
and the state carries the error forward, so after K steps a state entry differs from the fp64 result by at
most about 10 K 2^-24 of its own size (theta: of |theta| + |s|).  The tests allow 2e-6 K relative to the
tensor's largest entry plus, elementwise, 1e-5 relative to the entry itself.
"""
import numpy as np
import pytest
import torch

import paper_1803_02811_amd as arn
import workloads as wl
from oracle import nature_cnn as orc
from oracle import update_rules as up
from tests.gpu_util import DEV, GpuNet, check_grads, per_tensor, tol_check

pytestmark = pytest.mark.gpu

SIZES = [1, 3, 4, 1003, 262147]          # single element, a ragged tail only, one vector, ragged, many blocks


def _dev(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(DEV)


def _close(got, ref, name, K):
    got = got.cpu().numpy().astype(np.float64)
    ref = np.asarray(ref, np.float64)
    assert np.isfinite(got).all(), name
    scale = float(np.abs(ref).max())
    bound = 2e-6 * K * scale + 1e-5 * np.abs(ref) + 1e-30
    bad = np.abs(got - ref) > bound
    assert not bad.any(), f"{name}: {int(bad.sum())} entries off, worst {np.abs(got - ref).max():.3e} (scale {scale:.3e})"


@pytest.mark.parametrize("n", SIZES)
def test_rmsprop_steps(n):
    K, lr, rho, eps = 5, 7e-4, 0.99, 1e-6
    inp = wl.update_rule_inputs(n, K, seed=n % 97)
    th, acc = inp["theta"].astype(np.float64), np.zeros(n)
    d_th, d_acc = _dev(inp["theta"]), torch.zeros(n, dtype=torch.float32, device=DEV)
    for g in inp["grads"]:
        arn.rmsprop_update(d_th, _dev(g), d_acc, lr=lr, rho=rho, eps=eps)
        th, acc = up.rmsprop_step(th, acc, g, np.float32(lr), np.float32(rho), np.float32(eps))
    torch.cuda.synchronize()
    _close(d_th, th, "theta", K)
    _close(d_acc, acc, "accu", K)


@pytest.mark.parametrize("n", SIZES)
def test_adam_steps(n):
    K, r, b1, b2, eps = 6, 4.2e-4, 0.9, 0.999, 0.01 / 256
    inp = wl.update_rule_inputs(n, K, seed=100 + n % 97)
    th, m, v = inp["theta"].astype(np.float64), np.zeros(n), np.zeros(n)
    d_th = _dev(inp["theta"])
    d_m, d_v = (torch.zeros(n, dtype=torch.float32, device=DEV) for _ in range(2))
    for t, g in enumerate(inp["grads"], start=1):
        arn.adam_update(d_th, _dev(g), d_m, d_v, t=t, r=r, beta1=b1, beta2=b2, eps=eps)
        th, m, v, _ = up.adam_step(th, m, v, g, t, np.float32(r), np.float32(b1), np.float32(b2), np.float32(eps))
    torch.cuda.synchronize()
    _close(d_th, th, "theta", K)
    _close(d_m, m, "m", K)
    _close(d_v, v, "v", K)


@pytest.mark.parametrize("n", [1, 1003, 262147])
def test_async_adam_two_learners(n):
    """Two learners take 2 and 3 local steps from the same central state and merge one after the other."""
    r, b1, b2, eps = 3e-4, 0.9, 0.999, 1e-5
    f = np.float32
    ia, ib = wl.update_rule_inputs(n, 2, seed=200), wl.update_rule_inputs(n, 3, seed=201)
    th0 = ia["theta"]
    zeros = lambda: torch.zeros(n, dtype=torch.float32, device=DEV)
    cen = dict(theta=_dev(th0), m=zeros(), v=zeros())
    th_c, m_c, v_c = th0.astype(np.float64), np.zeros(n), np.zeros(n)
    learners = []
    for inp in (ia, ib):
        L = up.AsyncAdamLearner(th0, np.zeros(n), np.zeros(n))
        D = dict(theta=_dev(th0), m=zeros(), v=zeros(), a_g=zeros(), a_g2=zeros(), a_s=zeros())
        for t, g in enumerate(inp["grads"], start=1):
            arn.async_adam_local_step(D["theta"], _dev(g), D["m"], D["v"], D["a_g"], D["a_g2"], D["a_s"], t=t, r=r,
                                      beta1=b1, beta2=b2, eps=eps)
            up.async_adam_local_step(L, g, f(r), f(b1), f(b2), f(eps))
        torch.cuda.synchronize()
        for name in ("theta", "m", "v", "a_g", "a_g2", "a_s"):
            _close(D[name], getattr(L, name), "local " + name, len(inp["grads"]))
        learners.append((L, D, len(inp["grads"])))
    for L, D, nloc in learners:
        arn.async_adam_merge(cen["theta"], cen["m"], cen["v"], D["theta"], D["m"], D["v"], D["a_g"], D["a_g2"],
                             D["a_s"], n_local=nloc, beta1=b1, beta2=b2)
        th_c, m_c, v_c = up.async_adam_merge(L, th_c, m_c, v_c, f(b1), f(b2))
        torch.cuda.synchronize()
        _close(cen["theta"], th_c, "central theta", 6)
        _close(cen["m"], m_c, "central m", 6)
        _close(cen["v"], v_c, "central v", 6)
        for name in ("theta", "m", "v"):
            assert torch.equal(D[name], cen[name]), name            # local copies take the central values
        for name in ("a_g", "a_g2", "a_s"):
            assert not D[name].any(), name


def test_single_learner_merge_equals_plain_adam_on_the_gpu():
    """n local steps + merge from one learner give the central state plain Adam would have reached."""
    n, r, b1, b2, eps = 50021, 4e-4, 0.9, 0.999, 1e-6
    inp = wl.update_rule_inputs(n, 4, seed=300)
    zeros = lambda: torch.zeros(n, dtype=torch.float32, device=DEV)
    plain = dict(theta=_dev(inp["theta"]), m=zeros(), v=zeros())
    cen = dict(theta=_dev(inp["theta"]), m=zeros(), v=zeros())
    D = dict(theta=_dev(inp["theta"]), m=zeros(), v=zeros(), a_g=zeros(), a_g2=zeros(), a_s=zeros())
    for t, g in enumerate(inp["grads"], start=1):
        dg = _dev(g)
        arn.adam_update(plain["theta"], dg, plain["m"], plain["v"], t=t, r=r, beta1=b1, beta2=b2, eps=eps)
        arn.async_adam_local_step(D["theta"], dg, D["m"], D["v"], D["a_g"], D["a_g2"], D["a_s"], t=t, r=r,
                                  beta1=b1, beta2=b2, eps=eps)
    assert torch.equal(D["theta"], plain["theta"])               # same arithmetic, same bits
    arn.async_adam_merge(cen["theta"], cen["m"], cen["v"], D["theta"], D["m"], D["v"], D["a_g"], D["a_g2"], D["a_s"],
                         n_local=4, beta1=b1, beta2=b2)
    torch.cuda.synchronize()
    for name in ("theta", "m", "v"):
        _close(cen[name], plain[name].cpu().numpy(), name, 8)


@pytest.mark.parametrize("head", ["pv", "c51"])
def test_update_with_repack_matches_separate_prepare(head):
    """The packed copy written by the update call is byte-identical to arn_weights_prepare of the new theta."""
    A = 18
    flat = wl.he_normal_params(A, head, seed=2400)
    net = GpuNet(A, head, flat)
    n = flat.size
    inp = wl.update_rule_inputs(n, 1, seed=400)
    g = _dev(inp["grads"][0] * 100.0)
    for rule in ("rmsprop", "adam", "adam_local", "adam_merge"):
        th = _dev(flat)
        packed = torch.zeros(arn.packed_bytes(net.cfg), dtype=torch.uint8, device=DEV)
        s1, s2, a1, a2, a3 = (torch.zeros(n, dtype=torch.float32, device=DEV) for _ in range(5))
        if rule == "rmsprop":
            arn.rmsprop_update(th, g, s1, lr=1e-3, rho=0.99, eps=1e-6, cfg=net.cfg, w_packed=packed)
        elif rule == "adam":
            arn.adam_update(th, g, s1, s2, t=1, r=1e-3, beta1=0.9, beta2=0.999, eps=1e-5, cfg=net.cfg, w_packed=packed)
        elif rule == "adam_local":
            arn.async_adam_local_step(th, g, s1, s2, a1, a2, a3, t=1, r=1e-3, beta1=0.9, beta2=0.999, eps=1e-5,
                                      cfg=net.cfg, w_packed=packed)
        else:
            # a local step without the re-pack, then the merge re-packs the learner's new theta (= the new central one)
            arn.async_adam_local_step(th, g, s1, s2, a1, a2, a3, t=1, r=1e-3, beta1=0.9, beta2=0.999, eps=1e-5)
            th_c = _dev(flat)
            m_c, v_c = (torch.zeros(n, dtype=torch.float32, device=DEV) for _ in range(2))
            arn.async_adam_merge(th_c, m_c, v_c, th, s1, s2, a1, a2, a3, n_local=1, beta1=0.9, beta2=0.999,
                                 cfg=net.cfg, w_packed=packed)
            torch.cuda.synchronize()
            assert torch.equal(th, th_c) and not a1.any() and not a3.any()
        torch.cuda.synchronize()
        assert not torch.equal(th, _dev(flat))
        want = torch.zeros_like(packed)
        arn.weights_prepare(net.cfg, th, want)
        torch.cuda.synchronize()
        assert torch.equal(packed, want), rule


def test_one_learner_iteration_gradient_update_gradient():
    """Steps 1-3 of the synchronous procedure on one GPU: gradient, Adam update with repack, gradient again,
    against the same chain in the oracle."""
    k, B, A = 3, 96, 18
    flat = wl.he_normal_params(A, "pv", seed=2000 + k)
    net = GpuNet(A, "pv", flat)
    batch = wl.actor_critic_batch(k, B=B)
    spec = orc.NetSpec(A, "pv")
    r, b1, b2, eps = 4.2e-4, 0.9, 0.999, 0.01 / B          # appendix "Experiment Details": epsilon = 0.01 / batch
    f = np.float32
    # oracle chain
    g0 = orc.train_step_grads(flat, batch, "a2c", spec)
    zero = np.zeros(flat.size)
    th1, _, _, _ = up.adam_step(flat.astype(np.float64), zero, zero, g0["flat"], 1, f(r), f(b1), f(b2), f(eps))
    g1 = orc.train_step_grads(th1, batch, "a2c", spec)
    # GPU: its own gradient drives its own update ...
    th = _dev(flat)
    m, v = (torch.zeros(flat.size, dtype=torch.float32, device=DEV) for _ in range(2))
    dW0, _ = net.train(batch, "a2c")
    tol_check(dW0, g0["flat"], "gradient before the update")
    arn.adam_update(th, _dev(dW0), m, v, t=1, r=r, beta1=b1, beta2=b2, eps=eps)
    # first step: s = r g / (|g| + eps / sqrt(1 - beta2)), whose slope in g is at most r sqrt(1 - beta2) / eps,
    # so the gradient's error bar carries over to theta with that factor
    slope = r * np.sqrt(1 - b2) / eps
    dg = np.abs(dW0.astype(np.float64) - g0["flat"]).max()
    got_th = th.cpu().numpy().astype(np.float64)
    assert np.abs(got_th - th1).max() <= slope * dg + 1e-6 * np.abs(th1).max()
    assert np.abs(th1 - flat).max() > 0.5 * r               # the update moved the parameters
    # ... and the second gradient, taken with the weights the update call re-packed.  The map from a gradient
    # error to the next gradient is ill-conditioned at this batch size (ReLU masks flip, V - ret changes
    # sign), so the step that feeds the second gradient uses the oracle's first gradient on both sides.
    th = _dev(flat)
    m.zero_(), v.zero_()
    arn.adam_update(th, _dev(g0["flat"]), m, v, t=1, r=r, beta1=b1, beta2=b2, eps=eps, cfg=net.cfg,
                    w_packed=net.packed)
    dW1, loss1 = net.train(batch, "a2c")
    assert np.abs(g1["flat"] - g0["flat"]).max() > 0.2 * np.abs(g0["flat"]).max()     # a different gradient
    got, want = per_tensor(dW1, A, "pv"), per_tensor(g1["flat"], A, "pv")
    check_grads(got, want, "gradient after the update")
    assert abs(loss1[0] - g1["loss"]["total"]) < 1e-2 * abs(g1["loss"]["total"]) + 1e-3
