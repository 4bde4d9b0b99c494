"""TEST INFRASTRUCTURE ONLY -- slow, plain CPU oracle for the Nature-CNN hot path.

What this file is
-----------------
A direct, fp64 statement of what the GPU library has to compute: the forward
pass of the Atari "Nature" convolutional network on uint8 frame stacks, the
three training objectives the paper trains it with, and the gradient of each
objective with respect to every parameter.  It exists to check the GPU path and
to be timed beside it as a CPU baseline.  Only tests, the smoke check and the
CPU-baseline leg of the benchmark may import it.  It shares no code with the
GPU library and neither imports the other.

Where each piece comes from
---------------------------
* Network: the paper's appendix "Atari Frame Processing" names it only as the
  standard 3-convolutional-layer network; the shape (84x84x4 input, 8x8/4 x32,
  4x4/2 x64, 3x3/1 x64, fc 512, ReLU after every hidden layer) is the
  well-known one and is fixed by this build's workload statement.  The paper's
  own geometry (104x80 frames, padding 1 on conv2/conv3, 12x9 feature map) is
  available through `Geometry` and is used as a pin for the output-size rule.
* A2C objective: section "RL Algorithm Background", the advantage actor-critic
  gradient E[grad log pi(a|s) A]; value regression and entropy bonus as in the
  actor-critic method the paper cites, with coefficients 0.5 and 0.01.
* PPO objective: same section, the clipped surrogate
  E[min(rho A, clip(rho, 1-eps, 1+eps) A)].
* Categorical DQN: same section (one sentence); the projected distributional
  Bellman target is the algorithm of the distributional-RL paper it cites.

* DQN objective: same section, E[(y - Q(a|s))^2] with y = r + gamma max_a Q(a|s';theta-);
  Double-DQN (the online network picks the action, the target network values it) and the
  dueling aggregation Q = V + A - mean(A) are the rules of the two publications that
  section cites for the epsilon-Rainbow agent.
* Action selection: the sampler returns actions, not logits (section "Synchronized
  Sampling"): a categorical draw for policy-gradient agents, epsilon-greedy for Q-learning
  agents.  The uniform random numbers are inputs, so that both sides draw the same action.

Readings taken where the paper is silent (each also listed in the design notes)
* cross-correlation (no kernel flip); pixel scaling x = u8/255;
* ReLU derivative at 0 is 0 (mask = pre > 0);
* every loss term is a mean over the batch; entropy uses natural log;
* advantages, returns, old log-probs and C51 targets are constants;
* PPO clip boundaries are inclusive; argmax ties go to the lowest index;
* DQN: squared error exactly as printed (no 1/2, no Huber clipping), mean over the batch;
  the target is a constant; y = r where the transition is terminal; the dueling network
  shares the 512-unit hidden layer between its value and advantage outputs;
* categorical draw = inverse CDF: the first action whose cumulative probability exceeds u;
  epsilon-greedy: u < epsilon takes action floor(u2 * A), otherwise the greedy action;
* C51: the target network both selects and evaluates the next action; the
  projection is the triangular-kernel (gather) form, which conserves mass even
  when a shifted atom lands exactly on a support point.

Parity pins: see tests/test_oracle_*.py.  Not pinned by anything outside this
repository: agreement with the authors' own (unpublished) network outputs --
"parity unpinned" for that, since the paper prints no worked numeric example.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass, field
from typing import Dict, List, Tuple

import numpy as np

from . import build as _build

_lib = None


def _conv_lib():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        dp = ctypes.POINTER(ctypes.c_double)
        i = ctypes.c_int
        lib.orc_conv2d_forward.argtypes = [dp, dp, dp, dp, i, i, i, i, i, i, i, i]
        lib.orc_conv2d_input_grad.argtypes = [dp, dp, dp, i, i, i, i, i, i, i, i]
        lib.orc_conv2d_weight_grad.argtypes = [dp, dp, dp, dp, i, i, i, i, i, i, i, i]
        lib.orc_out_size.argtypes = [i, i, i, i]
        lib.orc_out_size.restype = i
        lib.orc_num_threads.restype = i
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the C loops will use (OpenMP default for this process)."""
    return int(_conv_lib().orc_num_threads())


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _c(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


# --------------------------------------------------------------------------
# convolution layer (C loops)
# --------------------------------------------------------------------------
def out_size(h: int, k: int, s: int, pad: int = 0) -> int:
    """floor((h + 2 pad - k) / s) + 1."""
    return int(_conv_lib().orc_out_size(h, k, s, pad))


def conv2d(x, W, b, stride: int, pad: int = 0) -> np.ndarray:
    """pre[n,co,oy,ox] = b[co] + sum W[co,ci,ky,kx] x[n,ci,oy*s+ky-pad,ox*s+kx-pad]."""
    x, W = _c(x), _c(W)
    N, Cin, H, Wd = x.shape
    Cout, Cin2, k, k2 = W.shape
    assert Cin == Cin2 and k == k2
    b = _c(b if b is not None else np.zeros(Cout))
    OH, OW = out_size(H, k, stride, pad), out_size(Wd, k, stride, pad)
    pre = np.empty((N, Cout, OH, OW), dtype=np.float64)
    _conv_lib().orc_conv2d_forward(_p(x), _p(W), _p(b), _p(pre), N, Cin, H, Wd, Cout, k, stride, pad)
    return pre


def conv2d_input_grad(x_shape, W, dpre, stride: int, pad: int = 0) -> np.ndarray:
    W, dpre = _c(W), _c(dpre)
    N, Cin, H, Wd = x_shape
    Cout, _, k, _ = W.shape
    dx = np.empty((N, Cin, H, Wd), dtype=np.float64)
    _conv_lib().orc_conv2d_input_grad(_p(W), _p(dpre), _p(dx), N, Cin, H, Wd, Cout, k, stride, pad)
    return dx


def conv2d_weight_grad(x, dpre, k: int, stride: int, pad: int = 0):
    x, dpre = _c(x), _c(dpre)
    N, Cin, H, Wd = x.shape
    Cout = dpre.shape[1]
    dW = np.empty((Cout, Cin, k, k), dtype=np.float64)
    db = np.empty((Cout,), dtype=np.float64)
    _conv_lib().orc_conv2d_weight_grad(_p(x), _p(dpre), _p(dW), _p(db), N, Cin, H, Wd, Cout, k, stride, pad)
    return dW, db


# --------------------------------------------------------------------------
# network description and flat parameter vector
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Geometry:
    """Input size and the conv stack as (Cout, k, stride, pad) tuples."""
    in_ch: int = 4
    in_h: int = 84
    in_w: int = 84
    convs: Tuple[Tuple[int, int, int, int], ...] = ((32, 8, 4, 0), (64, 4, 2, 0), (64, 3, 1, 0))
    hidden: int = 512

    def feature_shape(self) -> Tuple[int, int, int]:
        c, h, w = self.in_ch, self.in_h, self.in_w
        for (co, k, s, p) in self.convs:
            c, h, w = co, out_size(h, k, s, p), out_size(w, k, s, p)
        return c, h, w


NATURE_84 = Geometry()
# the paper's own frame size and padding (appendix "Atari Frame Processing")
PAPER_104x80 = Geometry(in_h=104, in_w=80, convs=((32, 8, 4, 0), (64, 4, 2, 1), (64, 3, 1, 1)))
# the 2-convolutional-layer network the same appendix names for the policy-gradient runs.  The paper gives no filter
# counts; they are those of the publication it cites for that network (the asynchronous actor-critic paper):
# 16 filters 8x8 stride 4, 32 filters 4x4 stride 2, 256 hidden units.  On 104x80 frames the first layer gives 25x19
# and the second, padded by 1 as the appendix says, the 12x9 map it states.
A3C_104x80 = Geometry(in_h=104, in_w=80, convs=((16, 8, 4, 0), (32, 4, 2, 1)), hidden=256)


@dataclass(frozen=True)
class NetSpec:
    num_actions: int = 18
    head: str = "pv"            # "pv" = policy logits + value, "c51" = categorical, "q" = scalar Q-values,
                                # "duel" = advantage rows + a value row combined into Q-values
    num_atoms: int = 51
    geometry: Geometry = field(default_factory=Geometry)


def param_layout(spec: NetSpec) -> List[Tuple[str, Tuple[int, ...]]]:
    """Canonical order of the flat fp32 parameter / gradient vector."""
    g = spec.geometry
    out: List[Tuple[str, Tuple[int, ...]]] = []
    cin = g.in_ch
    for i, (co, k, s, p) in enumerate(g.convs, start=1):
        out += [(f"conv{i}.W", (co, cin, k, k)), (f"conv{i}.b", (co,))]
        cin = co
    c, h, w = g.feature_shape()
    out += [("fc.W", (g.hidden, c * h * w)), ("fc.b", (g.hidden,))]
    if spec.head == "pv":
        out += [("pi.W", (spec.num_actions, g.hidden)), ("pi.b", (spec.num_actions,)),
                ("v.W", (1, g.hidden)), ("v.b", (1,))]
    elif spec.head == "c51":
        n = spec.num_actions * spec.num_atoms
        out += [("c51.W", (n, g.hidden)), ("c51.b", (n,))]
    elif spec.head == "q":
        out += [("q.W", (spec.num_actions, g.hidden)), ("q.b", (spec.num_actions,))]
    elif spec.head == "duel":
        out += [("adv.W", (spec.num_actions, g.hidden)), ("adv.b", (spec.num_actions,)),
                ("val.W", (1, g.hidden)), ("val.b", (1,))]
    else:
        raise ValueError(spec.head)
    return out


def param_count(spec: NetSpec) -> int:
    return int(sum(int(np.prod(s)) for _, s in param_layout(spec)))


def unflatten(flat, spec: NetSpec) -> Dict[str, np.ndarray]:
    flat = np.asarray(flat)
    assert flat.ndim == 1 and flat.size == param_count(spec)
    out, o = {}, 0
    for name, shp in param_layout(spec):
        n = int(np.prod(shp))
        out[name] = flat[o:o + n].astype(np.float64).reshape(shp)
        o += n
    return out


def flatten(params: Dict[str, np.ndarray], spec: NetSpec) -> np.ndarray:
    return np.concatenate([np.asarray(params[name], dtype=np.float64).reshape(-1)
                           for name, _ in param_layout(spec)])


# --------------------------------------------------------------------------
# forward
# --------------------------------------------------------------------------
def forward(params: Dict[str, np.ndarray], obs_u8: np.ndarray, spec: NetSpec) -> dict:
    """Whole network on a batch of uint8 frame stacks [B,C,H,W].

    Returns every intermediate (`x`, `pre1..3`, `act1..3`, `pre_fc`, `h`) plus
    `logits` [B,A] and `value` [B]   (head "pv"), or
    `atom_logits` [B,A,atoms]       (head "c51").
    """
    g = spec.geometry
    obs_u8 = np.asarray(obs_u8)
    assert obs_u8.dtype == np.uint8 and obs_u8.shape[1:] == (g.in_ch, g.in_h, g.in_w)
    cache = {"x": obs_u8.astype(np.float64) / 255.0}
    a = cache["x"]
    for i, (co, k, s, p) in enumerate(g.convs, start=1):
        pre = conv2d(a, params[f"conv{i}.W"], params[f"conv{i}.b"], s, p)
        a = np.maximum(pre, 0.0)
        cache[f"pre{i}"], cache[f"act{i}"] = pre, a
    B = obs_u8.shape[0]
    flat = a.reshape(B, -1)                       # index c*(h*w) + y*w + x
    pre_fc = flat @ params["fc.W"].T + params["fc.b"]
    h = np.maximum(pre_fc, 0.0)
    cache["pre_fc"], cache["h"] = pre_fc, h
    if spec.head == "pv":
        cache["logits"] = h @ params["pi.W"].T + params["pi.b"]
        cache["value"] = (h @ params["v.W"].T + params["v.b"])[:, 0]
    elif spec.head == "c51":
        z = h @ params["c51.W"].T + params["c51.b"]
        cache["atom_logits"] = z.reshape(B, spec.num_actions, spec.num_atoms)
    elif spec.head == "q":
        cache["q"] = h @ params["q.W"].T + params["q.b"]
    elif spec.head == "duel":
        cache["adv"] = h @ params["adv.W"].T + params["adv.b"]
        cache["val"] = (h @ params["val.W"].T + params["val.b"])[:, 0]
        cache["q"] = dueling_aggregate(cache["adv"], cache["val"])
    else:
        raise ValueError(spec.head)
    return cache


def dueling_aggregate(adv: np.ndarray, val: np.ndarray) -> np.ndarray:
    """Q[n,a] = V[n] + A[n,a] - mean_a A[n,a]."""
    adv = np.asarray(adv, dtype=np.float64)
    return np.asarray(val, dtype=np.float64)[:, None] + adv - adv.mean(axis=1, keepdims=True)


def dueling_aggregate_grad(dq: np.ndarray):
    """Gradients at (A, V) of a scalar whose gradient at Q is dq."""
    dq = np.asarray(dq, dtype=np.float64)
    return dq - dq.mean(axis=1, keepdims=True), dq.sum(axis=1)


def sample_categorical(probs: np.ndarray, u: np.ndarray) -> np.ndarray:
    """Inverse-CDF draw: the first index whose cumulative probability exceeds u (the last one if rounding
    leaves the total below u)."""
    probs = np.asarray(probs, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    cdf = np.cumsum(probs, axis=1)
    idx = (cdf > u[:, None]).argmax(axis=1)
    none = ~(cdf > u[:, None]).any(axis=1)
    idx[none] = probs.shape[1] - 1
    return idx.astype(np.int32)


def epsilon_greedy(q: np.ndarray, u: np.ndarray, u2: np.ndarray, epsilon: float) -> np.ndarray:
    """u < epsilon: the uniformly random action floor(u2 * A); otherwise the lowest-index greedy action."""
    q = np.asarray(q, dtype=np.float64)
    A = q.shape[1]
    rand = np.minimum((np.asarray(u2, dtype=np.float64) * A).astype(np.int64), A - 1)
    return np.where(np.asarray(u, dtype=np.float64) < epsilon, rand, greedy(q)).astype(np.int32)


def log_softmax(z: np.ndarray) -> np.ndarray:
    """Along the last axis, with the row maximum subtracted first."""
    z = np.asarray(z, dtype=np.float64)
    s = z - z.max(axis=-1, keepdims=True)
    return s - np.log(np.exp(s).sum(axis=-1, keepdims=True))


def entropy(logp: np.ndarray) -> np.ndarray:
    """H = -sum p log p (natural log) along the last axis."""
    return -(np.exp(logp) * logp).sum(axis=-1)


def greedy(z: np.ndarray) -> np.ndarray:
    """Lowest-index argmax along the last axis (numpy's argmax rule)."""
    return np.argmax(z, axis=-1).astype(np.int32)


def top2_gap(z: np.ndarray) -> np.ndarray:
    """Largest minus second-largest entry along the last axis (infinite for a single entry)."""
    s = np.sort(np.asarray(z, dtype=np.float64), axis=-1)
    if s.shape[-1] < 2:
        return np.full(s.shape[:-1], np.inf)
    return s[..., -1] - s[..., -2]


def policy_outputs(cache: dict) -> dict:
    """What action selection needs: probabilities, greedy action, value."""
    logp = log_softmax(cache["logits"])
    return {"probs": np.exp(logp), "greedy": greedy(cache["logits"]), "value": cache["value"]}


# --------------------------------------------------------------------------
# objectives (value of the loss, then its gradient at the network outputs)
# --------------------------------------------------------------------------
def a2c_loss_value(logits, value, action, adv, ret, value_coef=0.5, entropy_coef=0.01) -> dict:
    """L = -mean(log pi(a) adv) + c_v mean((V - ret)^2) - c_e mean(H)."""
    logp = log_softmax(logits)
    B = logp.shape[0]
    lp_a = logp[np.arange(B), action]
    pol = -np.mean(lp_a * adv)
    val = np.mean((value - ret) ** 2)
    ent = np.mean(entropy(logp))
    return {"total": pol + value_coef * val - entropy_coef * ent,
            "policy": pol, "value": val, "entropy": ent}


def _entropy_grad(logp: np.ndarray) -> np.ndarray:
    """d(-H)/dz for one row: p (log p + H)."""
    p = np.exp(logp)
    return p * (logp + entropy(logp)[:, None])


def a2c_loss_grad(logits, value, action, adv, ret, value_coef=0.5, entropy_coef=0.01):
    """(dL/dlogits [B,A], dL/dvalue [B]) of `a2c_loss_value`; adv and ret are constants."""
    logp = log_softmax(logits)
    B, A = logp.shape
    p = np.exp(logp)
    onehot = np.zeros((B, A))
    onehot[np.arange(B), action] = 1.0
    dz = (-adv[:, None] * (onehot - p) + entropy_coef * _entropy_grad(logp)) / B
    dv = value_coef * 2.0 * (value - ret) / B
    return dz, dv


def ppo_loss_value(logits, value, action, adv, ret, old_logp, clip_eps=0.1,
                   value_coef=0.5, entropy_coef=0.01) -> dict:
    """L = -mean(min(rho A, clip(rho,1-eps,1+eps) A)) + c_v mean((V-ret)^2) - c_e mean(H)."""
    logp = log_softmax(logits)
    B = logp.shape[0]
    rho = np.exp(logp[np.arange(B), action] - old_logp)
    surr = np.minimum(rho * adv, np.clip(rho, 1.0 - clip_eps, 1.0 + clip_eps) * adv)
    pol = -np.mean(surr)
    val = np.mean((value - ret) ** 2)
    ent = np.mean(entropy(logp))
    return {"total": pol + value_coef * val - entropy_coef * ent,
            "policy": pol, "value": val, "entropy": ent}


def ppo_active(rho, adv, clip_eps=0.1) -> np.ndarray:
    """True where the unclipped branch carries the gradient (boundaries inclusive)."""
    return ((adv >= 0) & (rho <= 1.0 + clip_eps)) | ((adv < 0) & (rho >= 1.0 - clip_eps))


def ppo_loss_grad(logits, value, action, adv, ret, old_logp, clip_eps=0.1,
                  value_coef=0.5, entropy_coef=0.01):
    logp = log_softmax(logits)
    B, A = logp.shape
    p = np.exp(logp)
    rho = np.exp(logp[np.arange(B), action] - old_logp)
    w = np.where(ppo_active(rho, adv, clip_eps), adv * rho, 0.0)   # d surr / d logp[a]
    onehot = np.zeros((B, A))
    onehot[np.arange(B), action] = 1.0
    dz = (-w[:, None] * (onehot - p) + entropy_coef * _entropy_grad(logp)) / B
    dv = value_coef * 2.0 * (value - ret) / B
    return dz, dv


def c51_support(num_atoms=51, v_min=-10.0, v_max=10.0) -> np.ndarray:
    return v_min + (v_max - v_min) / (num_atoms - 1) * np.arange(num_atoms, dtype=np.float64)


def c51_project(p_next, reward, done, gamma=0.99, v_min=-10.0, v_max=10.0) -> np.ndarray:
    """Project the shifted/shrunk distribution back onto the fixed support.

    p_next [B,N] is the next-state distribution of the chosen action on atoms
    z_j.  Each atom moves to T_j = clip(r + gamma (1-done) z_j, v_min, v_max)
    and gives its mass to the support points within one spacing, linearly:
        m_i = sum_j p_next[j] * max(0, 1 - |T_j - z_i| / delta).
    """
    p_next = np.asarray(p_next, dtype=np.float64)
    B, N = p_next.shape
    z = c51_support(N, v_min, v_max)
    delta = (v_max - v_min) / (N - 1)
    m = np.empty((B, N))
    step = 1024
    for s in range(0, B, step):
        e = min(B, s + step)
        T = np.clip(reward[s:e, None] + gamma * (1.0 - done[s:e, None]) * z[None, :], v_min, v_max)
        tri = np.maximum(0.0, 1.0 - np.abs(T[:, :, None] - z[None, None, :]) / delta)   # [b,j,i]
        m[s:e] = np.einsum("bj,bji->bi", p_next[s:e], tri)
    return m


def c51_project_scatter(p_next, reward, done, gamma=0.99, v_min=-10.0, v_max=10.0) -> np.ndarray:
    """The floor/ceil scatter form of the same projection (cross-check only).

    Written as explicit Python loops; when a shifted atom lands exactly on a
    support point the whole mass goes there.
    """
    p_next = np.asarray(p_next, dtype=np.float64)
    B, N = p_next.shape
    z = c51_support(N, v_min, v_max)
    delta = (v_max - v_min) / (N - 1)
    m = np.zeros((B, N))
    for n in range(B):
        for j in range(N):
            T = min(max(reward[n] + gamma * (1.0 - done[n]) * z[j], v_min), v_max)
            b = (T - v_min) / delta
            lo, hi = int(np.floor(b)), int(np.ceil(b))
            if lo == hi:
                m[n, lo] += p_next[n, j]
            else:
                m[n, lo] += p_next[n, j] * (hi - b)
                m[n, hi] += p_next[n, j] * (b - lo)
    return m


def c51_target(atom_logits_next, reward, done, gamma=0.99, v_min=-10.0, v_max=10.0, a_star=None) -> dict:
    """Target distribution from the target network's outputs on next states.

    p = softmax over atoms; Q[a] = sum_j z_j p[a,j]; a* = lowest-index argmax Q;
    m = projection of p[a*].  Also returns the top-2 gap of Q for graders.
    `a_star` given: the next action is taken from it instead of the argmax (a grader that accepts either of two
    next actions whose values tie within its margin evaluates the step for the one under test).
    """
    B, A, N = atom_logits_next.shape
    p = np.exp(log_softmax(atom_logits_next))
    q = p @ c51_support(N, v_min, v_max)
    a_star = greedy(q) if a_star is None else np.asarray(a_star, dtype=np.int64)
    m = c51_project(p[np.arange(B), a_star], np.asarray(reward, dtype=np.float64),
                    np.asarray(done, dtype=np.float64), gamma, v_min, v_max)
    return {"m": m, "a_star": a_star, "q": q, "q_gap": top2_gap(q)}


def c51_loss_value(atom_logits, action, m) -> dict:
    """L = -mean_n sum_i m[n,i] log p(theta)[n, a_n, i]."""
    B = atom_logits.shape[0]
    logp = log_softmax(atom_logits)[np.arange(B), action]
    ce = -np.mean((m * logp).sum(axis=1))
    return {"total": ce, "ce": ce}


def c51_loss_grad(atom_logits, action, m) -> np.ndarray:
    """dL/d atom_logits [B,A,N]: (p - m sum(m))/B on the taken action's row, 0 elsewhere.

    With sum(m) = 1 this is (p - m)/B.
    """
    B = atom_logits.shape[0]
    p = np.exp(log_softmax(atom_logits)[np.arange(B), action])
    d = np.zeros_like(atom_logits, dtype=np.float64)
    d[np.arange(B), action] = (p * m.sum(axis=1, keepdims=True) - m) / B
    return d


# --------------------------------------------------------------------------
# backward through the network
# --------------------------------------------------------------------------
# --------------------------------------------------------------------------
# DQN objective (section "RL Algorithm Background")
# --------------------------------------------------------------------------
def dqn_target(q_next_target, reward, done, gamma: float, q_next_online=None, a_star=None) -> np.ndarray:
    """y = r + gamma (1 - done) Q(a*|s'; theta-), with a* = argmax of the target network's values, or of
    the online network's values on s' when `q_next_online` is given (Double-DQN); `a_star` given: that action
    instead of the argmax (see c51_target)."""
    qt = np.asarray(q_next_target, dtype=np.float64)
    if a_star is None:
        sel = greedy(qt if q_next_online is None else np.asarray(q_next_online, dtype=np.float64))
    else:
        sel = np.asarray(a_star, dtype=np.int64)
    boot = qt[np.arange(qt.shape[0]), sel]
    live = 1.0 - np.asarray(done, dtype=np.float64)
    return np.asarray(reward, dtype=np.float64) + gamma * live * boot


def dqn_loss_value(q, action, y) -> dict:
    """mean_n (y_n - Q[n, a_n])^2."""
    q = np.asarray(q, dtype=np.float64)
    td = np.asarray(y, dtype=np.float64) - q[np.arange(q.shape[0]), np.asarray(action)]
    return {"total": float(np.mean(td * td)), "td": float(np.mean(td * td))}


def dqn_loss_grad(q, action, y) -> np.ndarray:
    """d loss / d Q: 2 (Q[n,a_n] - y_n) / B at the taken action, zero elsewhere (y is a constant)."""
    q = np.asarray(q, dtype=np.float64)
    B = q.shape[0]
    rows = np.arange(B)
    a = np.asarray(action)
    g = np.zeros_like(q)
    g[rows, a] = 2.0 * (q[rows, a] - np.asarray(y, dtype=np.float64)) / B
    return g


def backward(params: Dict[str, np.ndarray], cache: dict, spec: NetSpec, *, dlogits=None,
             dvalue=None, datom_logits=None, dq=None) -> Dict[str, np.ndarray]:
    """Chain rule from gradients at the heads to every parameter (layout = params)."""
    g = spec.geometry
    grads: Dict[str, np.ndarray] = {}
    h = cache["h"]
    B = h.shape[0]
    if spec.head == "pv":
        grads["pi.W"] = dlogits.T @ h
        grads["pi.b"] = dlogits.sum(axis=0)
        grads["v.W"] = dvalue[None, :] @ h
        grads["v.b"] = np.array([dvalue.sum()])
        dh = dlogits @ params["pi.W"] + dvalue[:, None] * params["v.W"]
    elif spec.head == "c51":
        dz = datom_logits.reshape(B, -1)
        grads["c51.W"] = dz.T @ h
        grads["c51.b"] = dz.sum(axis=0)
        dh = dz @ params["c51.W"]
    elif spec.head == "q":
        grads["q.W"] = dq.T @ h
        grads["q.b"] = dq.sum(axis=0)
        dh = dq @ params["q.W"]
    else:
        dadv, dval = dueling_aggregate_grad(dq)
        grads["adv.W"] = dadv.T @ h
        grads["adv.b"] = dadv.sum(axis=0)
        grads["val.W"] = dval[None, :] @ h
        grads["val.b"] = np.array([dval.sum()])
        dh = dadv @ params["adv.W"] + dval[:, None] * params["val.W"]
    dpre_fc = dh * (cache["pre_fc"] > 0)
    nconv = len(g.convs)
    feat = cache[f"act{nconv}"]
    grads["fc.W"] = dpre_fc.T @ feat.reshape(B, -1)
    grads["fc.b"] = dpre_fc.sum(axis=0)
    da = (dpre_fc @ params["fc.W"]).reshape(feat.shape)
    for i in range(nconv, 0, -1):
        co, k, s, p = g.convs[i - 1]
        dpre = da * (cache[f"pre{i}"] > 0)
        x_in = cache[f"act{i-1}"] if i > 1 else cache["x"]
        grads[f"conv{i}.W"], grads[f"conv{i}.b"] = conv2d_weight_grad(x_in, dpre, k, s, p)
        if i > 1:
            da = conv2d_input_grad(x_in.shape, params[f"conv{i}.W"], dpre, s, p)
    return grads


@dataclass
class Hyper:
    clip_eps: float = 0.1
    value_coef: float = 0.5
    entropy_coef: float = 0.01
    gamma: float = 0.99
    v_min: float = -10.0
    v_max: float = 10.0
    double_q: bool = False


def train_step_grads(flat_params, batch: dict, loss_kind: str, spec: NetSpec,
                     hyper: Hyper = Hyper(), flat_target_params=None, next_action=None) -> dict:
    """Forward, objective and backward for one batch.

    batch keys -- a2c: obs, action, adv, ret; ppo: + old_logp;
    c51, dqn: obs, action, next_obs, reward, done (and `flat_target_params`).
    `next_action` (c51, dqn): bootstrap from these next actions instead of the greedy ones (see c51_target).
    Returns {"loss": {...}, "grads": {name: array}, "flat": flat gradient, ...}; c51 and dqn also
    "select_q" [B,A], the action values the greedy next action is the argmax of, and "next_action" [B].
    """
    params = unflatten(flat_params, spec)
    cache = forward(params, batch["obs"], spec)
    out = {"cache": cache}
    if loss_kind == "a2c":
        args = (cache["logits"], cache["value"], batch["action"], _c(batch["adv"]), _c(batch["ret"]))
        kw = dict(value_coef=hyper.value_coef, entropy_coef=hyper.entropy_coef)
        out["loss"] = a2c_loss_value(*args, **kw)
        dz, dv = a2c_loss_grad(*args, **kw)
        grads = backward(params, cache, spec, dlogits=dz, dvalue=dv)
        out["dlogits"], out["dvalue"] = dz, dv
    elif loss_kind == "ppo":
        args = (cache["logits"], cache["value"], batch["action"], _c(batch["adv"]), _c(batch["ret"]),
                _c(batch["old_logp"]))
        kw = dict(clip_eps=hyper.clip_eps, value_coef=hyper.value_coef, entropy_coef=hyper.entropy_coef)
        out["loss"] = ppo_loss_value(*args, **kw)
        dz, dv = ppo_loss_grad(*args, **kw)
        grads = backward(params, cache, spec, dlogits=dz, dvalue=dv)
        out["dlogits"], out["dvalue"] = dz, dv
    elif loss_kind == "c51":
        tparams = unflatten(flat_target_params, spec)
        tcache = forward(tparams, batch["next_obs"], spec)
        tgt = c51_target(tcache["atom_logits"], batch["reward"], batch["done"],
                         hyper.gamma, hyper.v_min, hyper.v_max, a_star=next_action)
        out["target"] = tgt
        out["select_q"], out["next_action"] = tgt["q"], tgt["a_star"]
        out["loss"] = c51_loss_value(cache["atom_logits"], batch["action"], tgt["m"])
        d = c51_loss_grad(cache["atom_logits"], batch["action"], tgt["m"])
        grads = backward(params, cache, spec, datom_logits=d)
        out["datom_logits"] = d
    elif loss_kind == "dqn":
        tparams = unflatten(flat_target_params, spec)
        q_next_t = forward(tparams, batch["next_obs"], spec)["q"]
        q_next_o = forward(params, batch["next_obs"], spec)["q"] if hyper.double_q else None
        y = dqn_target(q_next_t, batch["reward"], batch["done"], hyper.gamma, q_next_o, a_star=next_action)
        out["target"] = y
        out["select_q"] = q_next_t if q_next_o is None else q_next_o
        out["next_action"] = greedy(out["select_q"]) if next_action is None else np.asarray(next_action, dtype=np.int64)
        out["loss"] = dqn_loss_value(cache["q"], batch["action"], y)
        d = dqn_loss_grad(cache["q"], batch["action"], y)
        grads = backward(params, cache, spec, dq=d)
        out["dq"] = d
    else:
        raise ValueError(loss_kind)
    out["grads"] = grads
    out["flat"] = flatten(grads, spec)
    return out
