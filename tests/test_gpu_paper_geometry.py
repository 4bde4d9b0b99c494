"""GPU parity for the paper's own frame size and padding (appendix "Atari Frame Processing": 104x80
frames, conv2 and conv3 padded by 1, feature maps 25x19 -> 12x9 -> 12x9, fc 6912 -> 512): inference
outputs and every gradient tensor against the CPU oracle on the same seeded inputs, through the C ABI.
Same bar as the 84x84 tests: max|err| <= 1e-2 max|ref| + 1e-3 per tensor; greedy actions equal
wherever the top-2 gap exceeds 1e-2."""
import numpy as np
import pytest

import workloads as wl
from oracle import nature_cnn as orc

pytestmark = pytest.mark.gpu

FRAME = wl.PAPER_FRAME
FC = wl.FC_INPUTS[FRAME]


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    from tests import gpu_util
    return gpu_util


def _spec(A, head):
    return orc.NetSpec(A, head, geometry=orc.PAPER_104x80)


def _net(gu, A, head, flat, **kw):
    return gu.GpuNet(A, head, flat, geometry="paper", **kw)


def _compare_grads(gu, dW, ref_flat, A, head, loss, ref_loss, keys):
    got, ref = gu.per_tensor(dW, A, head, fc_inputs=FC), gu.per_tensor(ref_flat, A, head, fc_inputs=FC)
    gu.check_grads(got, ref, "104x80 %s" % head)
    for i, k in enumerate(keys):
        if k is not None:
            gu.tol_check(loss[i:i + 1], np.array([ref_loss[k]]), f"loss.{k}")


def test_sizes_follow_the_appendix(gu):
    import paper_1803_02811_amd as arn
    cfg = arn.Config(18, geometry=arn.ARN_GEOM_PAPER)
    spec = _spec(18, "pv")
    assert spec.geometry.feature_shape() == (64, 12, 9)
    assert arn.param_count(cfg) == orc.param_count(spec) == sum(int(np.prod(s)) for _, s in wl.param_shapes(18, "pv", fc_inputs=FC))


@pytest.mark.parametrize("B,frames", [(1, "uniform"), (19, "uniform"), (70, "rects")])
def test_forward(gu, B, frames):
    """Logits, value, probabilities and greedy action; single-sample, ragged and multi-tile batches."""
    A = 6 if frames == "uniform" else 18
    flat = wl.he_normal_params(A, "pv", 2101, bias_std=0.1, fc_inputs=FC)
    obs = wl.uniform_frames(B, 1101, FRAME) if frames == "uniform" else wl.rect_frames(B, 1102, frame=FRAME)
    spec = _spec(A, "pv")
    ref = orc.forward(orc.unflatten(flat, spec), obs, spec)
    out = _net(gu, A, "pv", flat).forward(obs)
    pol = orc.policy_outputs(ref)
    gu.tol_check(out["logits"], ref["logits"], "logits")
    gu.tol_check(out["value"], ref["value"], "value")
    gu.tol_check(out["probs"], pol["probs"], "probs")
    decided = orc.top2_gap(ref["logits"]) > 1e-2
    np.testing.assert_array_equal(out["greedy"][decided], pol["greedy"][decided])
    np.testing.assert_array_equal(out["greedy"], np.argmax(out["logits"], axis=1))


@pytest.mark.parametrize("kind,B", [("a2c", 150), ("ppo", 90), ("a2c", 3)])
def test_actor_critic_gradients(gu, kind, B):
    """A2C / PPO objective and every parameter gradient; the padded convolutions' gradients included."""
    A = 18
    flat = wl.he_normal_params(A, "pv", 2103, bias_std=0.1, fc_inputs=FC)
    batch = wl.actor_critic_batch(3 if kind == "a2c" else 4, B=B, normalise_adv=(kind == "ppo"), frame=FRAME)
    spec = _spec(A, "pv")
    if kind == "ppo":
        ref_fwd = orc.forward(orc.unflatten(flat, spec), batch["obs"], spec)
        noisy = ref_fwd["logits"] + wl.logit_noise(4, B, A)
        batch["old_logp"] = orc.log_softmax(noisy)[np.arange(B), batch["action"]].astype(np.float32)
    ref = orc.train_step_grads(flat, batch, kind, spec)
    dW, loss = _net(gu, A, "pv", flat).train(batch, kind)
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])


def test_c51_gradients(gu):
    A, B = 18, 60
    flat = wl.he_normal_params(A, "c51", 2105, bias_std=0.1, fc_inputs=FC)
    tflat = wl.he_normal_params(A, "c51", 3105, bias_std=0.1, fc_inputs=FC)
    batch = wl.c51_batch(5, B=B, frame=FRAME)
    batch["done"][:3] = 1
    batch["reward"][0] = 0.0
    spec = _spec(A, "c51")
    dW, loss, ref, _ = gu.train_c51_or_dqn(_net(gu, A, "c51", flat), orc, flat, tflat, batch, "c51", spec)
    _compare_grads(gu, dW, ref["flat"], A, "c51", loss, ref["loss"], ["total", "ce", None, None])


def test_double_dqn_dueling_gradients(gu):
    A, B = 18, 60
    flat = wl.he_normal_params(A, "duel", 2106, bias_std=0.1, fc_inputs=FC)
    tflat = wl.he_normal_params(A, "duel", 3106, bias_std=0.1, fc_inputs=FC)
    batch = wl.c51_batch(5, B=B, frame=FRAME)
    spec = _spec(A, "duel")
    net = _net(gu, A, "duel", flat, double_q=1)
    dW, loss, ref, _ = gu.train_c51_or_dqn(net, orc, flat, tflat, batch, "dqn", spec, hyper=orc.Hyper(double_q=True))
    _compare_grads(gu, dW, ref["flat"], A, "duel", loss, ref["loss"], ["total", None, None, None])


def test_gradients_bit_reproducible_and_mean_of_shards(gu):
    """Fixed summation order, and the data-parallel rule (section "Synchronous Multi-GPU Optimization")."""
    A, B = 18, 256
    flat = wl.he_normal_params(A, "pv", 2103, fc_inputs=FC)
    batch = wl.actor_critic_batch(3, B=B, frame=FRAME)
    net = _net(gu, A, "pv", flat)
    d1, l1 = net.train(batch, "a2c")
    d2, l2 = net.train(batch, "a2c")
    assert d1.tobytes() == d2.tobytes() and l1.tobytes() == l2.tobytes()
    halves = [net.train({k: v[s] for k, v in batch.items()}, "a2c")[0] for s in (slice(0, 128), slice(128, 256))]
    mean = 0.5 * (halves[0] + halves[1])
    assert np.abs(d1 - mean).max() <= 2e-3 * np.abs(mean).max() + 1e-6


def test_full_size_a2c_b2048(gu):
    """The A2C step at the batch size the benchmark times (B=2048), every gradient tensor against the oracle."""
    A, B = 18, 2048
    flat = wl.he_normal_params(A, "pv", 2003, fc_inputs=FC)
    batch = wl.actor_critic_batch(3, B=B, frame=FRAME)
    ref = orc.train_step_grads(flat, batch, "a2c", _spec(A, "pv"))
    dW, loss = _net(gu, A, "pv", flat).train(batch, "a2c")
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])


@pytest.mark.parametrize("fill", [0, 255])
def test_constant_frames(gu, fill):
    """Black and saturated frames: with zero biases a black frame gives pre-activations of exactly zero
    everywhere (ReLU derivative 0 there), and the padded borders must contribute nothing."""
    A, B = 6, 5
    flat = wl.he_normal_params(A, "pv", 2107, bias_std=0.0 if fill == 0 else 0.1, fc_inputs=FC)
    r = np.random.default_rng(fill)
    batch = dict(obs=np.full((B,) + FRAME, fill, dtype=np.uint8), action=r.integers(0, A, size=B).astype(np.int32),
                 adv=r.standard_normal(B).astype(np.float32), ret=r.standard_normal(B).astype(np.float32))
    ref = orc.train_step_grads(flat, batch, "a2c", _spec(A, "pv"))
    dW, loss = _net(gu, A, "pv", flat).train(batch, "a2c")
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])
    if fill == 0:
        got = gu.per_tensor(dW, A, "pv", fc_inputs=FC)
        for name in ("conv1.W", "conv1.b", "conv2.W", "conv3.W", "fc.W"):
            assert not got[name].any(), name


def test_bad_geometry_is_rejected(gu):
    import paper_1803_02811_amd as arn
    cfg = arn.Config(18, geometry=3)
    assert arn.param_count(cfg) == 0 and arn.workspace_bytes(cfg, 16, arn.ARN_MODE_FORWARD) == 0
