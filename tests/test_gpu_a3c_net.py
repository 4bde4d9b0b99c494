"""GPU parity for the 2-convolution policy-gradient network of appendix "Atari Frame Processing" (104x80 frames,
16 filters 8x8/4, 32 filters 4x4/2 padded by 1 -> 12x9, 256 hidden units; cfg.geometry = ARN_GEOM_A3C): inference
outputs and every gradient tensor against the CPU oracle's own 2-convolution network, through the C ABI.  Same bars
as everywhere: max|err| <= 1e-2 max|ref| + 1e-3 per tensor, 2e-2 max|ref| per gradient tensor, greedy actions equal
wherever the top-2 gap exceeds 1e-2."""
import numpy as np
import pytest

import workloads as wl
from oracle import nature_cnn as orc

pytestmark = pytest.mark.gpu
FRAME = wl.PAPER_FRAME


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    from tests import gpu_util
    return gpu_util


def _spec(A, head):
    return orc.NetSpec(A, head, geometry=orc.A3C_104x80)


def _grads(gu, dW, ref_flat, A, head):
    got, want = wl.split_params(dW, A, head, net="a3c"), wl.split_params(ref_flat, A, head, net="a3c")
    return gu.check_grads(got, want, "2-convolution network %s" % head)


@pytest.mark.parametrize("B,frames", [(1, "uniform"), (19, "uniform"), (70, "rects"), (300, "rects")])
def test_forward(gu, B, frames):
    A = 6 if frames == "uniform" else 18
    flat = wl.he_normal_params(A, "pv", 2201, bias_std=0.1, net="a3c")
    obs = wl.uniform_frames(B, 1201, FRAME) if frames == "uniform" else wl.rect_frames(B, 1202, frame=FRAME)
    spec = _spec(A, "pv")
    ref = orc.forward(orc.unflatten(flat, spec), obs, spec)
    out = gu.GpuNet(A, "pv", flat, geometry="a3c").forward(obs)
    pol = orc.policy_outputs(ref)
    gu.tol_check(out["logits"], ref["logits"], "logits")
    gu.tol_check(out["value"], ref["value"], "value")
    gu.tol_check(out["probs"], pol["probs"], "probs")
    decided = orc.top2_gap(ref["logits"]) > 1e-2
    np.testing.assert_array_equal(out["greedy"][decided], pol["greedy"][decided])
    np.testing.assert_array_equal(out["greedy"], np.argmax(out["logits"], axis=1))


@pytest.mark.parametrize("kind,B", [("a2c", 150), ("ppo", 90), ("a2c", 3), ("a2c", 515)])
def test_actor_critic_gradients(gu, kind, B):
    A = 18
    flat = wl.he_normal_params(A, "pv", 2203, bias_std=0.1, net="a3c")
    batch = wl.actor_critic_batch(3 if kind == "a2c" else 4, B=B, normalise_adv=(kind == "ppo"), frame=FRAME)
    spec = _spec(A, "pv")
    if kind == "ppo":
        ref_fwd = orc.forward(orc.unflatten(flat, spec), batch["obs"], spec)
        noisy = ref_fwd["logits"] + wl.logit_noise(4, B, A)
        batch["old_logp"] = orc.log_softmax(noisy)[np.arange(B), batch["action"]].astype(np.float32)
    ref = orc.train_step_grads(flat, batch, kind, spec)
    dW, loss = gu.GpuNet(A, "pv", flat, geometry="a3c").train(batch, kind)
    _grads(gu, dW, ref["flat"], A, "pv")
    for i, k in enumerate(["total", "policy", "value", "entropy"]):
        gu.tol_check(loss[i:i + 1], np.array([ref["loss"][k]]), "loss." + k)


def test_full_size_a2c_b2048(gu):
    """The batch size the benchmark line times."""
    A, B = 18, 2048
    flat = wl.he_normal_params(A, "pv", 2003, net="a3c")
    batch = wl.actor_critic_batch(3, B=B, frame=FRAME)
    ref = orc.train_step_grads(flat, batch, "a2c", _spec(A, "pv"))
    dW, loss = gu.GpuNet(A, "pv", flat, geometry="a3c").train(batch, "a2c")
    _grads(gu, dW, ref["flat"], A, "pv")
    gu.tol_check(loss[:1], np.array([ref["loss"]["total"]]), "loss.total")


def test_categorical_head_and_action_values_on_the_small_network(gu):
    """The other heads ride on the same embedding: a categorical step and a dueling Double-DQN step."""
    A, B = 6, 40
    for head, kind, hyper, cfgkw in (("c51", "c51", orc.Hyper(), {}), ("duel", "dqn", orc.Hyper(double_q=True), dict(double_q=1))):
        flat = wl.he_normal_params(A, head, 2205, bias_std=0.1, net="a3c")
        tflat = wl.he_normal_params(A, head, 3205, bias_std=0.1, net="a3c")
        batch = wl.c51_batch(5, B=B, frame=FRAME)
        batch["action"] = (batch["action"] % A).astype(np.int32)
        batch["done"][:3] = 1
        spec = _spec(A, head)
        net = gu.GpuNet(A, head, flat, geometry="a3c", **cfgkw)
        dW, loss, ref, _ = gu.train_c51_or_dqn(net, orc, flat, tflat, batch, kind, spec, hyper=hyper)
        _grads(gu, dW, ref["flat"], A, head)
        gu.tol_check(loss[:1], np.array([ref["loss"]["total"]]), "loss.total " + head)


def test_update_with_repack_on_the_small_network(gu):
    """An Adam step on the small network's flat vector with the re-pack asked for equals a separate prepare."""
    import torch
    import paper_1803_02811_amd as arn
    A = 18
    flat = wl.he_normal_params(A, "pv", 2207, net="a3c")
    net = gu.GpuNet(A, "pv", flat, geometry="a3c")
    n = flat.size
    th = torch.from_numpy(flat.copy()).to(gu.DEV)
    g = torch.from_numpy((wl.update_rule_inputs(n, 1, seed=401)["grads"][0] * 100.0).astype(np.float32)).to(gu.DEV)
    m, v = (torch.zeros(n, dtype=torch.float32, device=gu.DEV) for _ in range(2))
    packed = torch.zeros(arn.packed_bytes(net.cfg), dtype=torch.uint8, device=gu.DEV)
    arn.adam_update(th, g, m, v, t=1, r=1e-3, beta1=0.9, beta2=0.999, eps=1e-5, cfg=net.cfg, w_packed=packed)
    want = torch.zeros_like(packed)
    arn.weights_prepare(net.cfg, th, want)
    torch.cuda.synchronize()
    assert torch.equal(packed, want)
