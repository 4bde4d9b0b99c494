"""Seeded synthetic inputs shaped like the paper's Atari workloads.

This module serves both the CPU oracle's tests and the GPU library's tests and
benchmark.  It contains only random-number draws and array layout -- none of
the network's or the objectives' arithmetic -- so that neither side can inherit
a mistake from the other through it.

The paper measures on Atari-2600 frames from the Arcade Learning Environment
(section "Experiments"); the emulator, its ROMs and recorded frames are not
available here, so the arrays below stand in for them: uint8 stacks of four
84x84 frames, batches of (simulators x horizon) samples, 6 or 18 actions, 51
atoms.  Network throughput does not depend on pixel values.

Seeds: inputs 1000+k, weights 2000+k, target weights 3000+k for workload k.
"""
from __future__ import annotations

from typing import Dict, List, Sequence, Tuple

import numpy as np

FRAME = (4, 84, 84)
# the frame size of the paper's own runs (appendix "Atari Frame Processing": 104x80, convolutions padded so
# that the feature map is 12x9) and the fc input sizes that go with the two frame sizes
PAPER_FRAME = (4, 104, 80)
FC_INPUTS = {FRAME: 64 * 7 * 7, PAPER_FRAME: 64 * 12 * 9}

WORKLOADS = {
    1: dict(name="fwd_b16", B=16, A=6, head="pv", kind="forward", frames="uniform"),
    2: dict(name="infer_b256", B=256, A=18, head="pv", kind="forward", frames="rects"),
    3: dict(name="a2c_b2048", B=2048, A=18, head="pv", kind="a2c", frames="rects"),
    4: dict(name="ppo_b4096", B=4096, A=18, head="pv", kind="ppo", frames="uniform"),
    5: dict(name="c51_b8192", B=8192, A=18, head="c51", kind="c51", frames="rects"),
}


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def uniform_frames(B: int, seed: int, frame: Tuple[int, int, int] = FRAME) -> np.ndarray:
    """uint8 [B,4,H,W], every pixel i.i.d. uniform on 0..255."""
    return rng(seed).integers(0, 256, size=(B,) + tuple(frame), dtype=np.uint8)


def rect_frames(B: int, seed: int, with_next: bool = False, frame: Tuple[int, int, int] = FRAME):
    """Smooth structured stacks: black background, 4..12 random rectangles of
    side 4..32 and intensity 1..255 (later ones overwrite earlier ones); frame f
    of a stack is frame 0 translated by f*(dx,dy), dx,dy in +-{1,2,3}, zero
    filled.  With `with_next`, also returns the stack one step later: frames
    1..3 followed by frame 0 translated by 4*(dx,dy).
    """
    g = rng(seed)
    C, H, W = frame
    obs = np.zeros((B, C, H, W), dtype=np.uint8)
    nxt = np.zeros((B, C, H, W), dtype=np.uint8) if with_next else None
    for n in range(B):
        base = np.zeros((H, W), dtype=np.uint8)
        for _ in range(int(g.integers(4, 13))):
            h, w = int(g.integers(4, 33)), int(g.integers(4, 33))
            y, x = int(g.integers(0, H - h + 1)), int(g.integers(0, W - w + 1))
            base[y:y + h, x:x + w] = int(g.integers(1, 256))
        dx = int(g.integers(1, 4)) * (1 if g.integers(0, 2) else -1)
        dy = int(g.integers(1, 4)) * (1 if g.integers(0, 2) else -1)
        frames = [_shift(base, f * dy, f * dx) for f in range(5 if with_next else 4)]
        obs[n] = np.stack(frames[:4])
        if with_next:
            nxt[n] = np.stack(frames[1:5])
    return (obs, nxt) if with_next else obs


def _shift(img: np.ndarray, dy: int, dx: int) -> np.ndarray:
    H, W = img.shape
    out = np.zeros_like(img)
    ys, yd = (slice(0, H - dy), slice(dy, H)) if dy >= 0 else (slice(-dy, H), slice(0, H + dy))
    xs, xd = (slice(0, W - dx), slice(dx, W)) if dx >= 0 else (slice(-dx, W), slice(0, W + dx))
    out[yd, xd] = img[ys, xs]
    return out


# fc inputs of the 2-convolution policy-gradient network on 104x80 frames (32 channels x 12 x 9)
A3C_FC_INPUTS = 32 * 12 * 9


def param_shapes(num_actions: int, head: str, num_atoms: int = 51,
                 fc_inputs: int = FC_INPUTS[FRAME], net: str = "nature") -> List[Tuple[str, Tuple[int, ...]]]:
    """Canonical flat order of the parameter vector (interface, fixed by the C header).  net = "nature": the
    3-convolution network (fc_inputs selects the frame size); net = "a3c": the 2-convolution network on 104x80
    frames (16 and 32 filters, 256 hidden units)."""
    if net == "a3c":
        hid = 256
        out = [("conv1.W", (16, 4, 8, 8)), ("conv1.b", (16,)),
               ("conv2.W", (32, 16, 4, 4)), ("conv2.b", (32,)),
               ("fc.W", (hid, A3C_FC_INPUTS)), ("fc.b", (hid,))]
    elif net == "nature":
        hid = 512
        out = [("conv1.W", (32, 4, 8, 8)), ("conv1.b", (32,)),
               ("conv2.W", (64, 32, 4, 4)), ("conv2.b", (64,)),
               ("conv3.W", (64, 64, 3, 3)), ("conv3.b", (64,)),
               ("fc.W", (hid, fc_inputs)), ("fc.b", (hid,))]
    else:
        raise ValueError(net)
    if head == "pv":
        out += [("pi.W", (num_actions, hid)), ("pi.b", (num_actions,)), ("v.W", (1, hid)), ("v.b", (1,))]
    elif head == "c51":
        out += [("c51.W", (num_actions * num_atoms, hid)), ("c51.b", (num_actions * num_atoms,))]
    elif head == "q":
        out += [("q.W", (num_actions, hid)), ("q.b", (num_actions,))]
    elif head == "duel":
        out += [("adv.W", (num_actions, hid)), ("adv.b", (num_actions,)), ("val.W", (1, hid)), ("val.b", (1,))]
    else:
        raise ValueError(head)
    return out


def he_normal_params(num_actions: int, head: str, seed: int, num_atoms: int = 51,
                     bias_std: float = 0.0, fc_inputs: int = FC_INPUTS[FRAME], net: str = "nature") -> np.ndarray:
    """Flat fp32 vector: every weight tensor ~ N(0, 2/fan_in); biases 0, or
    N(0, bias_std^2) when a test wants the bias paths exercised."""
    g = rng(seed)
    parts = []
    for name, shp in param_shapes(num_actions, head, num_atoms, fc_inputs, net):
        if name.endswith(".W"):
            fan_in = int(np.prod(shp[1:]))
            parts.append(g.standard_normal(shp).reshape(-1) * np.sqrt(2.0 / fan_in))
        else:
            parts.append(g.standard_normal(shp).reshape(-1) * bias_std)
    return np.concatenate(parts).astype(np.float32)


def split_params(flat: np.ndarray, num_actions: int, head: str, num_atoms: int = 51,
                 fc_inputs: int = FC_INPUTS[FRAME], net: str = "nature") -> Dict[str, np.ndarray]:
    out, o = {}, 0
    for name, shp in param_shapes(num_actions, head, num_atoms, fc_inputs, net):
        n = int(np.prod(shp))
        out[name] = flat[o:o + n].reshape(shp)
        o += n
    assert o == flat.size
    return out


def frames_for(k: int, B: int | None = None, with_next: bool = False, frame: Tuple[int, int, int] = FRAME):
    w = WORKLOADS[k]
    B = w["B"] if B is None else B
    if w["frames"] == "uniform":
        if with_next:
            return uniform_frames(B, 1000 + k, frame), uniform_frames(B, 1500 + k, frame)
        return uniform_frames(B, 1000 + k, frame)
    return rect_frames(B, 1000 + k, with_next=with_next, frame=frame)


def actor_critic_batch(k: int, B: int | None = None, normalise_adv: bool = False,
                       frame: Tuple[int, int, int] = FRAME) -> dict:
    """obs, action ~ U{0..A-1}, adv ~ N(0,1) (optionally standardised over the
    batch with population std + 1e-8), ret ~ N(0,1)."""
    w = WORKLOADS[k]
    B = w["B"] if B is None else B
    g = rng(1100 + k)
    adv = g.standard_normal(B)
    if normalise_adv:
        adv = (adv - adv.mean()) / (adv.std() + 1e-8)
    return {"obs": frames_for(k, B, frame=frame),
            "action": g.integers(0, w["A"], size=B).astype(np.int32),
            "adv": adv.astype(np.float32),
            "ret": g.standard_normal(B).astype(np.float32)}


def logit_noise(k: int, B: int, A: int, std: float = 0.05) -> np.ndarray:
    """N(0, std^2) perturbation added to current logits to fabricate the
    sampling policy's logits for the PPO workload (the caller applies it)."""
    return rng(1200 + k).standard_normal((B, A)) * std


def c51_batch(k: int = 5, B: int | None = None, frame: Tuple[int, int, int] = FRAME) -> dict:
    """obs / next_obs (a real frame-stack transition), action ~ U{0..17},
    reward ~ U{-1,0,1}, done ~ Bernoulli(0.01)."""
    w = WORKLOADS[k]
    B = w["B"] if B is None else B
    g = rng(1100 + k)
    obs, nxt = frames_for(k, B, with_next=True, frame=frame)
    return {"obs": obs, "next_obs": nxt,
            "action": g.integers(0, w["A"], size=B).astype(np.int32),
            "reward": g.integers(-1, 2, size=B).astype(np.float32),
            "done": (g.random(B) < 0.01).astype(np.uint8)}


def update_rule_inputs(n: int, steps: int, seed: int) -> dict:
    """Inputs for the parameter-update rules: a parameter vector and `steps` gradient vectors, all exactly
    representable in fp32.  Gradient magnitudes spread over five decades per entry, as gradients of a deep
    network do across layers; a few entries are exactly zero (dead units).  Seeds: 4000 + seed."""
    r = rng(4000 + seed)
    theta = (r.standard_normal(n) * 0.05).astype(np.float32)
    grads = []
    for _ in range(steps):
        g = r.standard_normal(n) * 10.0 ** r.uniform(-6.0, -1.0, size=n)
        g[r.random(n) < 0.01] = 0.0
        grads.append(g.astype(np.float32))
    return dict(theta=theta, grads=grads)


def action_uniforms(B: int, seed: int) -> dict:
    """The two uniform [0,1) numbers per sample that action selection consumes (u: the categorical draw or
    the explore/exploit coin; u2: which random action), as fp32.  Seeds: 5000 + seed."""
    r = rng(5000 + seed)
    return {"u": r.random(B).astype(np.float32), "u2": r.random(B).astype(np.float32)}
