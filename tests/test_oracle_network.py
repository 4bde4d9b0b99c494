"""Pins for the oracle's whole-network forward and backward (CPU only)."""
import numpy as np
import pytest

import workloads as wl
from oracle import nature_cnn as orc

SMALL = orc.Geometry(in_ch=2, in_h=20, in_w=20, convs=((3, 4, 2, 0), (4, 3, 1, 0), (4, 2, 1, 0)), hidden=6)
# a small non-square stack padded like the paper's own (appendix "Atari Frame Processing": no padding on the first
# layer, padding 1 on a stride-2 4x4 and on a stride-1 3x3 layer)
SMALL_PADDED = orc.Geometry(in_ch=2, in_h=22, in_w=18, convs=((3, 4, 2, 0), (4, 4, 2, 1), (4, 3, 1, 1)), hidden=6)


# a small 2-convolution stack shaped like the policy-gradient network of the same appendix (second layer padded by 1)
SMALL_TWO_CONV = orc.Geometry(in_ch=2, in_h=22, in_w=18, convs=((3, 4, 2, 0), (5, 4, 2, 1)), hidden=7)


def _rand_params(spec, seed, bias=True):
    r = np.random.default_rng(seed)
    out = {}
    for name, shp in orc.param_layout(spec):
        if name.endswith(".W"):
            out[name] = r.standard_normal(shp) * np.sqrt(2.0 / np.prod(shp[1:]))
        else:
            out[name] = r.standard_normal(shp) * (0.3 if bias else 0.0)
    return out


def test_param_counts_and_layout():
    assert orc.param_count(orc.NetSpec(6, "pv")) == 1_687_719
    assert orc.param_count(orc.NetSpec(18, "pv")) == 1_693_875
    assert orc.param_count(orc.NetSpec(18, "c51")) == 2_155_062
    # the shared shape table (interface) and the oracle's own agree
    for A, head in [(6, "pv"), (18, "pv"), (18, "c51")]:
        assert orc.param_layout(orc.NetSpec(A, head)) == wl.param_shapes(A, head)
    spec = orc.NetSpec(6, "pv")
    flat = np.arange(orc.param_count(spec), dtype=np.float64)
    p = orc.unflatten(flat, spec)
    assert p["conv1.W"][0, 0, 0, 1] == 1 and p["conv1.b"][0] == 8192
    assert p["fc.W"][1, 0] == flat[8224 + 32832 + 36928 + 3136]
    np.testing.assert_array_equal(orc.flatten(p, spec), flat)


def test_forward_shapes_and_flatten_order():
    spec = orc.NetSpec(6, "pv")
    params = orc.unflatten(wl.he_normal_params(6, "pv", seed=1), spec)
    obs = wl.uniform_frames(2, seed=2)
    c = orc.forward(params, obs, spec)
    assert c["act1"].shape == (2, 32, 20, 20) and c["act2"].shape == (2, 64, 9, 9)
    assert c["act3"].shape == (2, 64, 7, 7) and c["h"].shape == (2, 512)
    assert c["logits"].shape == (2, 6) and c["value"].shape == (2,)
    # fc input index is c*49 + y*7 + x: rebuild one hidden unit with explicit loops
    acc = params["fc.b"][3]
    for ch in range(64):
        for y in range(7):
            for x in range(7):
                acc += params["fc.W"][3, ch * 49 + y * 7 + x] * c["act3"][1, ch, y, x]
    assert np.isclose(c["pre_fc"][1, 3], acc, atol=1e-12)
    assert c["x"].max() <= 1.0 and c["x"].min() >= 0.0
    assert np.isclose(c["x"][0, 0, 0, 0], obs[0, 0, 0, 0] / 255.0)


def test_forward_first_layer_against_explicit_window():
    spec = orc.NetSpec(6, "pv")
    params = orc.unflatten(wl.he_normal_params(6, "pv", seed=3, bias_std=0.1), spec)
    obs = wl.uniform_frames(1, seed=4)
    c = orc.forward(params, obs, spec)
    oy, ox, co = 7, 13, 5
    win = obs[0, :, 4 * oy:4 * oy + 8, 4 * ox:4 * ox + 8].astype(np.float64) / 255.0
    want = (win * params["conv1.W"][co]).sum() + params["conv1.b"][co]
    assert np.isclose(c["pre1"][0, co, oy, ox], want, atol=1e-12)
    assert np.isclose(c["act1"][0, co, oy, ox], max(want, 0.0), atol=1e-12)


def test_paper_geometry_forward_against_explicit_windows():
    """Appendix "Atari Frame Processing": 104x80 frames, no padding on the first layer, padding 1 on the second
    and third: the feature maps are 25x19, 12x9, 12x9 and border outputs see zeros outside the map.  One
    corner and one interior output of conv2 and conv3 and one hidden unit are rebuilt with explicit loops."""
    spec = orc.NetSpec(6, "pv", geometry=orc.PAPER_104x80)
    fc_in = wl.FC_INPUTS[wl.PAPER_FRAME]
    params = orc.unflatten(wl.he_normal_params(6, "pv", seed=5, bias_std=0.1, fc_inputs=fc_in), spec)
    obs = wl.uniform_frames(1, seed=6, frame=wl.PAPER_FRAME)
    c = orc.forward(params, obs, spec)
    assert c["act1"].shape == (1, 32, 25, 19) and c["act2"].shape == (1, 64, 12, 9) and c["act3"].shape == (1, 64, 12, 9)
    assert c["h"].shape == (1, 512) and params["fc.W"].shape == (512, 6912)

    def window_sum(inp, W, b, k, stride, pad, co, oy, ox):
        acc = b[co]
        for ci in range(inp.shape[0]):
            for ky in range(k):
                for kx in range(k):
                    y, x = oy * stride - pad + ky, ox * stride - pad + kx
                    if 0 <= y < inp.shape[1] and 0 <= x < inp.shape[2]:
                        acc += W[co, ci, ky, kx] * inp[ci, y, x]
        return acc

    for (oy, ox) in [(0, 0), (11, 8), (5, 4)]:
        want2 = window_sum(c["act1"][0], params["conv2.W"], params["conv2.b"], 4, 2, 1, 7, oy, ox)
        assert np.isclose(c["pre2"][0, 7, oy, ox], want2, atol=1e-12)
        want3 = window_sum(c["act2"][0], params["conv3.W"], params["conv3.b"], 3, 1, 1, 9, oy, ox)
        assert np.isclose(c["pre3"][0, 9, oy, ox], want3, atol=1e-12)
    acc = params["fc.b"][3]
    for ch in range(64):
        for y in range(12):
            for x in range(9):
                acc += params["fc.W"][3, ch * 108 + y * 9 + x] * c["act3"][0, ch, y, x]
    assert np.isclose(c["pre_fc"][0, 3], acc, atol=1e-12)


def test_two_convolution_network_sizes_and_forward_against_explicit_loops():
    """The policy-gradient network of appendix "Atari Frame Processing": 104x80 frames, first layer 25x19, second
    layer padded by 1 -> the 12x9 map the appendix states; outputs rebuilt with explicit window sums."""
    g = orc.A3C_104x80
    assert g.feature_shape() == (32, 12, 9) and wl.A3C_FC_INPUTS == 32 * 12 * 9
    assert orc.out_size(104, 8, 4) == 25 and orc.out_size(80, 8, 4) == 19
    assert orc.out_size(25, 4, 2, 1) == 12 and orc.out_size(19, 4, 2, 1) == 9
    spec = orc.NetSpec(6, "pv", geometry=g)
    assert orc.param_layout(spec) == wl.param_shapes(6, "pv", net="a3c")
    assert orc.param_count(spec) == 16 * 256 + 16 + 32 * 256 + 32 + 256 * 3456 + 256 + 7 * 256 + 7
    params = orc.unflatten(wl.he_normal_params(6, "pv", seed=5, bias_std=0.1, net="a3c"), spec)
    obs = wl.uniform_frames(1, seed=6, frame=wl.PAPER_FRAME)
    c = orc.forward(params, obs, spec)
    assert c["act1"].shape == (1, 16, 25, 19) and c["act2"].shape == (1, 32, 12, 9) and "act3" not in c
    assert c["h"].shape == (1, 256)
    x = obs[0].astype(np.float64) / 255.0
    # conv1, one output: window rows 4 oy .. 4 oy + 7
    oy, ox, co = 24, 18, 9
    want = (x[:, 4 * oy:4 * oy + 8, 4 * ox:4 * ox + 8] * params["conv1.W"][co]).sum() + params["conv1.b"][co]
    assert np.isclose(c["pre1"][0, co, oy, ox], want, atol=1e-12)
    # conv2 at a corner and at an edge: taps that fall into the padding contribute nothing
    a1 = np.zeros((16, 27, 21))
    a1[:, 1:26, 1:20] = c["act1"][0]
    for (oy, ox, co) in [(0, 0, 3), (11, 8, 31), (5, 0, 17)]:
        want = (a1[:, 2 * oy:2 * oy + 4, 2 * ox:2 * ox + 4] * params["conv2.W"][co]).sum() + params["conv2.b"][co]
        assert np.isclose(c["pre2"][0, co, oy, ox], want, atol=1e-12)
    # fc input index is c*108 + y*9 + x over the second layer's map
    acc = params["fc.b"][5]
    for ch in range(32):
        for y in range(12):
            for xx in range(9):
                acc += params["fc.W"][5, ch * 108 + y * 9 + xx] * c["act2"][0, ch, y, xx]
    assert np.isclose(c["pre_fc"][0, 5], acc, atol=1e-12)


def _total_loss(flat, spec, batch, kind, tflat=None):
    params = orc.unflatten(flat, spec)
    c = orc.forward(params, batch["obs"], spec)
    if kind == "a2c":
        return orc.a2c_loss_value(c["logits"], c["value"], batch["action"], batch["adv"], batch["ret"])["total"]
    if kind == "ppo":
        return orc.ppo_loss_value(c["logits"], c["value"], batch["action"], batch["adv"], batch["ret"],
                                  batch["old_logp"])["total"]
    t = orc.forward(orc.unflatten(tflat, spec), batch["next_obs"], spec)
    m = orc.c51_target(t["atom_logits"], batch["reward"], batch["done"])["m"]
    return orc.c51_loss_value(c["atom_logits"], batch["action"], m)["total"]


@pytest.mark.parametrize("kind,geometry", [("a2c", SMALL), ("ppo", SMALL), ("c51", SMALL), ("a2c", SMALL_PADDED),
                                           ("c51", SMALL_PADDED), ("a2c", SMALL_TWO_CONV), ("ppo", SMALL_TWO_CONV)])
def test_whole_backward_by_finite_differences(kind, geometry):
    """Central differences of the scalar loss on a sample of coordinates of every
    tensor, small geometries (one of them padded and non-square), non-zero biases, B = 3."""
    r = np.random.default_rng(21)
    A = 4
    spec = orc.NetSpec(A, "c51" if kind == "c51" else "pv", num_atoms=5, geometry=geometry)
    frame = (2, geometry.in_h, geometry.in_w)
    flat = orc.flatten(_rand_params(spec, 22), spec)
    tflat = orc.flatten(_rand_params(spec, 23), spec)
    B = 3
    obs = r.integers(0, 256, size=(B,) + frame, dtype=np.uint8)
    batch = dict(obs=obs, action=r.integers(0, A, size=B), adv=r.standard_normal(B), ret=r.standard_normal(B))
    if kind == "ppo":
        c = orc.forward(orc.unflatten(flat, spec), obs, spec)
        lp = orc.log_softmax(c["logits"])[np.arange(B), batch["action"]]
        batch["old_logp"] = lp + np.array([0.05, -0.05, 0.3])
    if kind == "c51":
        batch.update(next_obs=r.integers(0, 256, size=(B,) + frame, dtype=np.uint8),
                     reward=np.array([1.0, -1.0, 0.0]), done=np.array([0, 0, 1], dtype=np.uint8))
    out = orc.train_step_grads(flat, batch, kind, spec, flat_target_params=tflat)
    g = out["flat"]
    assert np.isclose(out["loss"]["total"], _total_loss(flat, spec, batch, kind, tflat))
    # sample coordinates from every tensor
    o, checked = 0, 0
    for name, shp in orc.param_layout(spec):
        n = int(np.prod(shp))
        for i in r.choice(n, size=min(n, 6), replace=False):
            h = 1e-5
            fp, fm = flat.copy(), flat.copy()
            fp[o + i] += h
            fm[o + i] -= h
            fd = (_total_loss(fp, spec, batch, kind, tflat) - _total_loss(fm, spec, batch, kind, tflat)) / (2 * h)
            assert abs(fd - g[o + i]) < 1e-7 + 1e-5 * abs(fd), (name, i, fd, g[o + i])
            checked += 1
        o += n
    assert checked > 40


def test_relu_derivative_at_zero_is_zero():
    """A black frame with zero biases gives pre-activations of exactly 0 in conv1;
    nothing may flow back through them."""
    spec = orc.NetSpec(4, "pv", geometry=SMALL)
    params = _rand_params(spec, 31, bias=False)
    obs = np.zeros((1, 2, 20, 20), dtype=np.uint8)
    c = orc.forward(params, obs, spec)
    assert (c["pre1"] == 0).all()
    g = orc.backward(params, c, spec, dlogits=np.ones((1, 4)), dvalue=np.ones(1))
    assert (g["conv1.b"] == 0).all() and (g["conv1.W"] == 0).all()
    assert (g["pi.b"] == 1).all()


def test_batch_gradient_is_mean_of_shard_gradients():
    """Data-parallel rule (section "Synchronous Multi-GPU Optimization"): the
    full-batch gradient equals the average of the gradients of equal shards."""
    spec = orc.NetSpec(6, "pv")
    flat = wl.he_normal_params(6, "pv", seed=41, bias_std=0.05)
    r = np.random.default_rng(42)
    B = 8
    batch = dict(obs=wl.rect_frames(B, 43), action=r.integers(0, 6, size=B), adv=r.standard_normal(B),
                 ret=r.standard_normal(B))
    full = orc.train_step_grads(flat, batch, "a2c", spec)
    halves = [orc.train_step_grads(flat, {k: v[s] for k, v in batch.items()}, "a2c", spec)
              for s in (slice(0, 4), slice(4, 8))]
    mean = 0.5 * (halves[0]["flat"] + halves[1]["flat"])
    np.testing.assert_allclose(full["flat"], mean, atol=1e-12 * np.abs(mean).max() + 1e-15)
    assert np.isclose(full["loss"]["total"], 0.5 * (halves[0]["loss"]["total"] + halves[1]["loss"]["total"]))
    # permutation invariance over samples
    perm = r.permutation(B)
    shuf = orc.train_step_grads(flat, {k: v[perm] for k, v in batch.items()}, "a2c", spec)
    np.testing.assert_allclose(shuf["flat"], full["flat"], atol=1e-12 * np.abs(mean).max() + 1e-15)


def test_workload_generators_are_seeded_and_shaped():
    a = wl.rect_frames(3, 5)
    b = wl.rect_frames(3, 5)
    np.testing.assert_array_equal(a, b)
    assert a.dtype == np.uint8 and a.shape == (3, 4, 84, 84)
    assert (a == 0).mean() > 0.2                     # black background survives
    obs, nxt = wl.rect_frames(2, 6, with_next=True)
    np.testing.assert_array_equal(obs[:, 1:], nxt[:, :3])   # a real frame-stack transition
    batch = wl.c51_batch(5, B=64)
    assert set(np.unique(batch["reward"])) <= {-1.0, 0.0, 1.0}
    assert batch["done"].dtype == np.uint8
    w = wl.he_normal_params(18, "pv", seed=2003)
    assert w.dtype == np.float32 and w.size == 1_693_875
    p = wl.split_params(w, 18, "pv")
    assert abs(p["fc.W"].std() - np.sqrt(2 / 3136)) < 1e-3 and (p["fc.b"] == 0).all()
    ac = wl.actor_critic_batch(4, B=128, normalise_adv=True)
    assert abs(ac["adv"].mean()) < 1e-6 and abs(ac["adv"].std() - 1) < 1e-3
