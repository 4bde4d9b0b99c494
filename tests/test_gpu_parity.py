"""GPU parity: the HIP path through the C ABI against the CPU oracle, element
by element on the same seeded inputs.  Bar: max|err| <= 1e-2 max|ref| + 1e-3
per output tensor; greedy actions equal wherever the top-2 gap exceeds 1e-2."""
import numpy as np
import pytest

import workloads as wl
from oracle import nature_cnn as orc

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gu():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a device"
    from tests import gpu_util
    return gpu_util


def _oracle_forward(flat, obs, A, head):
    spec = orc.NetSpec(A, head)
    return orc.forward(orc.unflatten(flat, spec), obs, spec), spec


@pytest.mark.parametrize("B", [1, 16, 37, 64, 85, 86, 130])
def test_forward_uniform_frames(gu, B):
    """Workload 1 (B=16, A=6, uniform frames) plus ragged and single-sample batches."""
    flat = wl.he_normal_params(6, "pv", 2001, bias_std=0.0 if B == 16 else 0.1)
    obs = wl.uniform_frames(B, 1001)
    ref, _ = _oracle_forward(flat, obs, 6, "pv")
    out = gu.GpuNet(6, "pv", flat).forward(obs)
    gu.tol_check(out["logits"], ref["logits"], "logits")
    gu.tol_check(out["value"], ref["value"], "value")


def test_inference_structured_frames_b256(gu):
    """Workload 2: probabilities, greedy action and value for 256 simulators."""
    flat = wl.he_normal_params(18, "pv", 2002)
    obs = wl.frames_for(2)
    ref, _ = _oracle_forward(flat, obs, 18, "pv")
    out = gu.GpuNet(18, "pv", flat).forward(obs)
    pol = orc.policy_outputs(ref)
    gu.tol_check(out["logits"], ref["logits"], "logits")
    gu.tol_check(out["probs"], pol["probs"], "probs")
    gu.tol_check(out["value"], ref["value"], "value")
    np.testing.assert_allclose(out["probs"].sum(axis=1), 1.0, atol=1e-5)
    decided = orc.top2_gap(ref["logits"]) > 1e-2
    assert decided.sum() > 200
    np.testing.assert_array_equal(out["greedy"][decided], pol["greedy"][decided])
    # the kernel's own argmax is the lowest-index maximum of its own logits
    np.testing.assert_array_equal(out["greedy"], np.argmax(out["logits"], axis=1))


def _compare_grads(gu, dW, ref_flat, A, head, loss, ref_loss, keys):
    got, ref = gu.per_tensor(dW, A, head), gu.per_tensor(ref_flat, A, head)
    report = gu.check_grads(got, ref, "%s A=%d" % (head, A))
    for i, k in enumerate(keys):
        if k is not None:
            gu.tol_check(loss[i:i + 1], np.array([ref_loss[k]]), f"loss.{k}")
    return report


@pytest.mark.parametrize("kind,B", [("a2c", 200), ("ppo", 200), ("a2c", 3)])
def test_actor_critic_gradients(gu, kind, B):
    """A2C / PPO loss and every parameter gradient, ragged batch over several tiles."""
    A = 18
    flat = wl.he_normal_params(A, "pv", 2003, bias_std=0.1)
    batch = wl.actor_critic_batch(3 if kind == "a2c" else 4, B=B, normalise_adv=(kind == "ppo"))
    spec = orc.NetSpec(A, "pv")
    if kind == "ppo":
        ref_fwd = orc.forward(orc.unflatten(flat, spec), batch["obs"], spec)
        noisy = ref_fwd["logits"] + wl.logit_noise(4, B, A)
        batch["old_logp"] = orc.log_softmax(noisy)[np.arange(B), batch["action"]].astype(np.float32)
    ref = orc.train_step_grads(flat, batch, kind, spec)
    dW, loss = gu.GpuNet(A, "pv", flat).train(batch, kind)
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])


@pytest.mark.parametrize("B", [150, 2])
def test_c51_gradients(gu, B):
    """Categorical DQN step: target forward, projection, cross-entropy, all gradients."""
    A = 18
    flat = wl.he_normal_params(A, "c51", 2005, bias_std=0.1)
    tflat = wl.he_normal_params(A, "c51", 3005, bias_std=0.1)
    batch = wl.c51_batch(5, B=B)
    batch["done"][: min(B, 3)] = 1            # terminal transitions present (reward 0 hits an atom exactly)
    batch["reward"][0] = 0.0
    spec = orc.NetSpec(A, "c51")
    dW, loss, ref, _ = gu.train_c51_or_dqn(gu.GpuNet(A, "c51", flat), orc, flat, tflat, batch, "c51", spec)
    _compare_grads(gu, dW, ref["flat"], A, "c51", loss, ref["loss"], ["total", "ce", None, None])


def test_c51_gradients_peaked_distributions(gu):
    """A categorical step whose head gradients are O(1e-1): a small batch, an online head whose weights are
    scaled up so that its predicted distributions are peaked, and many terminal transitions (targets of one or
    two atoms).  Here the absolute term of the stated bar carries nothing: the comparison is relative."""
    A, B = 18, 24
    flat = wl.he_normal_params(A, "c51", 2015, bias_std=0.1)
    parts = wl.split_params(flat, A, "c51")
    parts["c51.W"] *= 6.0                          # views into flat: the head's logits spread over several nats
    tflat = wl.he_normal_params(A, "c51", 3015, bias_std=0.1)
    batch = wl.c51_batch(5, B=B)
    batch["done"][::2] = 1
    spec = orc.NetSpec(A, "c51")
    dW, loss, ref, _ = gu.train_c51_or_dqn(gu.GpuNet(A, "c51", flat), orc, flat, tflat, batch, "c51", spec)
    want = gu.per_tensor(ref["flat"], A, "c51")
    assert np.abs(want["c51.W"]).max() > 0.1 and np.abs(want["c51.b"]).max() > 0.02
    _compare_grads(gu, dW, ref["flat"], A, "c51", loss, ref["loss"], ["total", "ce", None, None])


def test_c51_inference_outputs(gu):
    """Atom probabilities, expected values and greedy action of the categorical head."""
    A, B = 18, 40
    flat = wl.he_normal_params(A, "c51", 2005)
    obs = wl.frames_for(5, B)
    ref, _ = _oracle_forward(flat, obs, A, "c51")
    out = gu.GpuNet(A, "c51", flat).forward(obs)
    gu.tol_check(out["logits"], ref["atom_logits"], "atom_logits")
    p = np.exp(orc.log_softmax(ref["atom_logits"]))
    q = p @ orc.c51_support()
    gu.tol_check(out["probs"], p, "atom_probs")
    gu.tol_check(out["value"], q, "q")
    decided = orc.top2_gap(q) > 1e-2
    np.testing.assert_array_equal(out["greedy"][decided], orc.greedy(q)[decided])


def test_gradients_bit_reproducible(gu):
    A, B = 18, 300
    flat = wl.he_normal_params(A, "pv", 2003)
    batch = wl.actor_critic_batch(3, B=B)
    net = gu.GpuNet(A, "pv", flat)
    d1, l1 = net.train(batch, "a2c")
    d2, l2 = net.train(batch, "a2c")
    assert d1.tobytes() == d2.tobytes() and l1.tobytes() == l2.tobytes()


def test_full_batch_gradient_is_mean_of_shards(gu):
    """Data-parallel rule (section "Synchronous Multi-GPU Optimization") on the GPU path."""
    A, B = 18, 512
    flat = wl.he_normal_params(A, "pv", 2003)
    batch = wl.actor_critic_batch(3, B=B)
    net = gu.GpuNet(A, "pv", flat)
    full, lf = net.train(batch, "a2c")
    halves = [net.train({k: v[s] for k, v in batch.items()}, "a2c") for s in (slice(0, 256), slice(256, 512))]
    mean = 0.5 * (halves[0][0] + halves[1][0])
    scale = np.abs(mean).max()
    assert np.abs(full - mean).max() <= 2e-3 * scale + 1e-6
    assert abs(lf[0] - 0.5 * (halves[0][1][0] + halves[1][1][0])) < 1e-5


@pytest.mark.parametrize("geometry", ["84", "paper"])
def test_outputs_do_not_depend_on_the_batch_they_are_in(gu, geometry):
    """Small batches deal a sample's position tiles to several workgroups and cut the fc contraction
    differently; a sample's outputs must not change with the batch it is computed in (beyond fp32 rounding
    of the differently ordered fc sums)."""
    A = 18
    frame = wl.FRAME if geometry == "84" else wl.PAPER_FRAME
    flat = wl.he_normal_params(A, "pv", 2002, bias_std=0.1, fc_inputs=wl.FC_INPUTS[frame])
    obs = wl.rect_frames(300, 1002, frame=frame)
    net = gu.GpuNet(A, "pv", flat, geometry=geometry)
    full = net.forward(obs)
    for B in (1, 5, 16, 64, 129):
        part = net.forward(obs[:B])
        np.testing.assert_allclose(part["logits"], full["logits"][:B], atol=2e-5, rtol=0)
        np.testing.assert_allclose(part["value"], full["value"][:B], atol=2e-5, rtol=0)


# ---------------------------------------------------------------------------
# Full workload sizes, in the launch configuration the benchmark times.
# The oracle needs a few seconds per case on the GPU machine's host cores.
# ---------------------------------------------------------------------------
def test_full_size_a2c_b2048(gu):
    """Workload 3 as benchmarked: B=2048 A2C step, every gradient tensor and the loss against the oracle."""
    A, B = 18, 2048
    flat = wl.he_normal_params(A, "pv", 2003)
    batch = wl.actor_critic_batch(3, B=B)
    spec = orc.NetSpec(A, "pv")
    ref = orc.train_step_grads(flat, batch, "a2c", spec)
    dW, loss = gu.GpuNet(A, "pv", flat).train(batch, "a2c")
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])


@pytest.mark.parametrize("copies", [4096, 16384])
def test_largest_batches(gu, copies):
    """B = 2^18 and B = 2^20 (the largest batch the library accepts): element and byte offsets into every
    activation tensor pass 2^31 and 2^32.  The batch is `copies` copies of 64 distinct samples (tiled on the
    device), so every copy's forward outputs must repeat the first copy's bits, the first copy must match the
    oracle, and the batch-mean gradient must be the oracle's gradient of the 64."""
    import torch
    import paper_1803_02811_amd as arn
    A, base = 18, 64
    B = base * copies
    flat = wl.he_normal_params(A, "pv", 2003, bias_std=0.05)
    small = wl.actor_critic_batch(3, B=base)
    spec = orc.NetSpec(A, "pv")
    ref = orc.train_step_grads(flat, small, "a2c", spec)
    net = gu.GpuNet(A, "pv", flat)
    dev = net.device_batch(small)
    big = {k: v.repeat(copies, *([1] * (v.dim() - 1))).contiguous() for k, v in dev.items()}
    assert big["obs"].shape == (B, 4, 84, 84) and big["obs"].numel() > 2 ** 31
    logits = torch.empty(B, A, dtype=torch.float32, device=gu.DEV)
    value = torch.empty(B, dtype=torch.float32, device=gu.DEV)
    arn.policy_forward(net.cfg, net.packed, big["obs"], logits, value, None, None,
                       workspace=net.workspace(B, arn.ARN_MODE_FORWARD))
    torch.cuda.synchronize()
    lg, vl = logits.view(copies, base, A), value.view(copies, base)
    assert bool((lg == lg[:1]).all()) and bool((vl == vl[:1]).all())
    gu.tol_check(lg[0].cpu().numpy(), ref["cache"]["logits"], "logits")
    gu.tol_check(vl[0].cpu().numpy(), ref["cache"]["value"], "value")
    del logits, value, lg, vl
    net._ws.clear()
    dW, loss = net.train(None, "a2c", dev_batch=big)
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])
    net._ws.clear()
    del big
    torch.cuda.empty_cache()


def test_full_size_ppo_b4096(gu):
    """Workload 4: B=4096 PPO-clip step on uniform frames, old log-probs from perturbed oracle logits."""
    A, B = 18, 4096
    flat = wl.he_normal_params(A, "pv", 2004)
    batch = wl.actor_critic_batch(4, B=B, normalise_adv=True)
    spec = orc.NetSpec(A, "pv")
    fwd = orc.forward(orc.unflatten(flat, spec), batch["obs"], spec)
    noisy = fwd["logits"] + wl.logit_noise(4, B, A)
    batch["old_logp"] = orc.log_softmax(noisy)[np.arange(B), batch["action"]].astype(np.float32)
    ref = orc.train_step_grads(flat, batch, "ppo", spec)
    rho = np.exp(orc.log_softmax(fwd["logits"])[np.arange(B), batch["action"]] - batch["old_logp"])
    assert (~orc.ppo_active(rho, batch["adv"])).sum() > 20           # the clipped branch is exercised
    dW, loss = gu.GpuNet(A, "pv", flat).train(batch, "ppo")
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])


def test_full_size_c51_b8192(gu):
    """Workload 5: B=8192 categorical step (target forward, projection, cross-entropy, all gradients)."""
    A, B = 18, 8192
    flat = wl.he_normal_params(A, "c51", 2005)
    tflat = wl.he_normal_params(A, "c51", 3005)
    batch = wl.c51_batch(5, B=B)
    spec = orc.NetSpec(A, "c51")
    assert batch["done"].sum() > 20
    dW, loss, ref, _ = gu.train_c51_or_dqn(gu.GpuNet(A, "c51", flat), orc, flat, tflat, batch, "c51", spec)
    _compare_grads(gu, dW, ref["flat"], A, "c51", loss, ref["loss"], ["total", "ce", None, None])
    # properties that hold at any size: gradient of the categorical head's bias sums to zero per action
    got = gu.per_tensor(dW, A, "c51")
    assert np.abs(got["c51.b"].reshape(A, 51).sum(axis=1)).max() < 1e-4


# ---------------------------------------------------------------------------
# Edge and degenerate configurations
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("A", [1, 2, 31])
def test_policy_head_extreme_action_counts(gu, A):
    """Smallest and largest supported policy heads (A = 1: a single action, zero entropy)."""
    B = 9
    flat = wl.he_normal_params(A, "pv", 2100 + A, bias_std=0.1)
    r = np.random.default_rng(A)
    batch = dict(obs=wl.rect_frames(B, 1300 + A), action=r.integers(0, A, size=B).astype(np.int32),
                 adv=r.standard_normal(B).astype(np.float32), ret=r.standard_normal(B).astype(np.float32))
    spec = orc.NetSpec(A, "pv")
    ref = orc.train_step_grads(flat, batch, "a2c", spec)
    net = gu.GpuNet(A, "pv", flat)
    out = net.forward(batch["obs"])
    gu.tol_check(out["logits"], ref["cache"]["logits"], "logits")
    gu.tol_check(out["value"], ref["cache"]["value"], "value")
    np.testing.assert_allclose(out["probs"].sum(axis=1), 1.0, atol=1e-5)
    dW, loss = net.train(batch, "a2c")
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])
    if A == 1:
        assert abs(loss[3]) < 1e-6 and abs(loss[1]) < 1e-6      # one action: no entropy, log pi = 0


@pytest.mark.parametrize("A,atoms,vmin,vmax", [(3, 21, -5.0, 5.0), (1, 2, 0.0, 1.0), (18, 64, -10.0, 10.0)])
def test_c51_other_supports(gu, A, atoms, vmin, vmax):
    """Categorical head with other action counts, atom counts (2 and the maximum 64) and supports."""
    B = 12
    flat = wl.he_normal_params(A, "c51", 2200 + atoms, num_atoms=atoms, bias_std=0.1)
    tflat = wl.he_normal_params(A, "c51", 3200 + atoms, num_atoms=atoms, bias_std=0.1)
    r = np.random.default_rng(atoms)
    obs, nxt = wl.rect_frames(B, 1400 + atoms, with_next=True)
    batch = dict(obs=obs, next_obs=nxt, action=r.integers(0, A, size=B).astype(np.int32),
                 reward=r.integers(-1, 2, size=B).astype(np.float32), done=(r.random(B) < 0.3).astype(np.uint8))
    spec = orc.NetSpec(A, "c51", num_atoms=atoms)
    hyper = orc.Hyper(v_min=vmin, v_max=vmax, gamma=0.9)
    net = gu.GpuNet(A, "c51", flat, num_atoms=atoms, v_min=vmin, v_max=vmax, gamma=0.9)
    dW, loss, ref, _ = gu.train_c51_or_dqn(net, orc, flat, tflat, batch, "c51", spec, hyper=hyper)
    got, want = wl.split_params(dW, A, "c51", atoms), wl.split_params(ref["flat"], A, "c51", atoms)
    gu.check_grads(got, want, "c51 A=%d atoms=%d" % (A, atoms))
    gu.tol_check(loss[:1], np.array([ref["loss"]["total"]]), "loss")


def test_black_frames_exact_zero_preactivations(gu):
    """All-black frames with zero biases: conv1 pre-activations are exactly 0 and the ReLU
    derivative there is 0, so nothing reaches conv1's parameters (and the oracle agrees)."""
    A, B = 6, 5
    flat = wl.he_normal_params(A, "pv", 2300)
    r = np.random.default_rng(5)
    batch = dict(obs=np.zeros((B, 4, 84, 84), dtype=np.uint8), action=r.integers(0, A, size=B).astype(np.int32),
                 adv=r.standard_normal(B).astype(np.float32), ret=r.standard_normal(B).astype(np.float32))
    spec = orc.NetSpec(A, "pv")
    ref = orc.train_step_grads(flat, batch, "a2c", spec)
    dW, loss = gu.GpuNet(A, "pv", flat).train(batch, "a2c")
    got = gu.per_tensor(dW, A, "pv")
    assert (got["conv1.W"] == 0).all() and (got["conv1.b"] == 0).all()
    assert (ref["grads"]["conv1.W"] == 0).all()
    _compare_grads(gu, dW, ref["flat"], A, "pv", loss, ref["loss"], ["total", "policy", "value", "entropy"])


@pytest.mark.parametrize("geometry,B", [("84", 515), ("paper", 515), ("84", 1), ("paper", 1), ("84", 257), ("84", 4099)])
def test_gradients_with_short_and_single_sample_workgroups(gu, geometry, B):
    """The sample-resident backward kernels give each workgroup a contiguous range of samples: 515 = 171 x 3 + 2
    leaves the last workgroup short (and makes the fused conv1 backward pipeline three samples per workgroup),
    257 gives ranges of two with a single sample at the end, 1 is one workgroup with nothing to prefetch; 4099 is
    past the size from which the head kernel takes sixteen samples per workgroup, with three in its last one."""
    A = 18
    frame = wl.FRAME if geometry == "84" else wl.PAPER_FRAME
    fc_in = wl.FC_INPUTS[frame]
    flat = wl.he_normal_params(A, "pv", 2011, bias_std=0.1, fc_inputs=fc_in)
    batch = wl.actor_critic_batch(3, B=B, frame=frame)
    spec = orc.NetSpec(A, "pv") if geometry == "84" else orc.NetSpec(A, "pv", geometry=orc.PAPER_104x80)
    ref = orc.train_step_grads(flat, batch, "a2c", spec)
    dW, loss = gu.GpuNet(A, "pv", flat, geometry=geometry).train(batch, "a2c")
    got, want = gu.per_tensor(dW, A, "pv", fc_inputs=fc_in), gu.per_tensor(ref["flat"], A, "pv", fc_inputs=fc_in)
    gu.check_grads(got, want, "%s B=%d" % (geometry, B))
    gu.tol_check(loss[:1], np.array([ref["loss"]["total"]]), "loss.total")


def test_saturated_frames_and_large_batch_tail(gu):
    """All-255 frames (largest pixel sums) and a batch that leaves ragged tails in every kernel."""
    A, B = 18, 259
    flat = wl.he_normal_params(A, "pv", 2301, bias_std=0.05)
    obs = np.full((B, 4, 84, 84), 255, dtype=np.uint8)
    obs[1::2] = wl.uniform_frames((B + 1) // 2, 1501)[: B // 2 + B % 2][: len(obs[1::2])]
    ref, _ = _oracle_forward(flat, obs, A, "pv")
    out = gu.GpuNet(A, "pv", flat).forward(obs)
    gu.tol_check(out["logits"], ref["logits"], "logits")
    gu.tol_check(out["value"], ref["value"], "value")


def test_single_stream_mode_gives_the_same_bits(gu, tmp_path):
    """ARN_SINGLE_STREAM=1 keeps every kernel on the caller's stream; the fixed summation order makes the
    gradient bit-identical to the two-stream run.  The switch is read once per process, hence the child."""
    import os
    import subprocess
    import sys
    A, B = 18, 70
    flat = wl.he_normal_params(A, "pv", 2003)
    batch = wl.actor_critic_batch(3, B=B)
    dW, loss = gu.GpuNet(A, "pv", flat).train(batch, "a2c")
    out = tmp_path / "dw.npy"
    code = (
        "import sys, numpy as np\n"
        f"sys.path.insert(0, {os.path.dirname(os.path.dirname(os.path.abspath(__file__)))!r})\n"
        "import workloads as wl\n"
        "from tests import gpu_util as gu\n"
        f"flat = wl.he_normal_params({A}, 'pv', 2003)\n"
        f"dW, loss = gu.GpuNet({A}, 'pv', flat).train(wl.actor_critic_batch(3, B={B}), 'a2c')\n"
        f"np.save({str(out)!r}, np.concatenate([dW, loss]))\n")
    env = dict(os.environ, ARN_SINGLE_STREAM="1")
    subprocess.run([sys.executable, "-c", code], check=True, env=env, timeout=110)
    other = np.load(out)
    assert np.array_equal(other[:-4], dW) and np.array_equal(other[-4:], loss)
