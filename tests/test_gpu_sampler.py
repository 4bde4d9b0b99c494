"""The sampler's side of the GPU path as a tested component (section "Synchronized Sampling"): the simulators are
split into two groups that alternate, each group's observations go host -> device, through arn_policy_act, and its
actions device -> host, on a stream of its own, while the other group's request is in flight.  Checked against the
oracle's draws and, bit for bit, against one call that serves all simulators as a single group.  Also the case the
header promises for arn_train_step_grads: two calls issued back to back from one thread on two caller streams."""
import numpy as np
import pytest

import workloads as wl
from oracle import nature_cnn as orc

pytestmark = pytest.mark.gpu

A, N_SIMS, ROUNDS = 18, 256, 4


class _Group:
    """Pinned host buffers, device buffers, workspace and stream of one group of simulators."""

    def __init__(self, torch, arn, gu, cfg, n):
        self.n = n
        self.stream = torch.cuda.Stream()            # default priority
        self.h_obs = torch.empty((n, 4, 84, 84), dtype=torch.uint8).pin_memory()
        self.h_u = torch.empty(n, dtype=torch.float32).pin_memory()
        self.h_act = torch.empty(n, dtype=torch.int32).pin_memory()
        self.h_logp = torch.empty(n, dtype=torch.float32).pin_memory()
        self.d_obs = torch.empty((n, 4, 84, 84), dtype=torch.uint8, device=gu.DEV)
        self.d_u = torch.empty(n, dtype=torch.float32, device=gu.DEV)
        self.d_u2 = torch.zeros(n, dtype=torch.float32, device=gu.DEV)
        self.d_act = torch.empty(n, dtype=torch.int32, device=gu.DEV)
        self.d_logp = torch.empty(n, dtype=torch.float32, device=gu.DEV)
        self.ws = torch.empty(arn.workspace_bytes(cfg, n, arn.ARN_MODE_FORWARD), dtype=torch.uint8, device=gu.DEV)
        self.done = torch.cuda.Event()

    def issue(self, torch, arn, cfg, packed, obs_np, u_np):
        """Host hand-over of one environment step: frames and random numbers in, actions and log-probabilities out."""
        self.h_obs.copy_(torch.from_numpy(obs_np))
        self.h_u.copy_(torch.from_numpy(u_np))
        with torch.cuda.stream(self.stream):
            self.d_obs.copy_(self.h_obs, non_blocking=True)
            self.d_u.copy_(self.h_u, non_blocking=True)
            arn.policy_act(cfg, packed, self.d_obs, self.d_u, self.d_u2, self.d_act, self.d_logp, workspace=self.ws,
                           stream=self.stream)
            self.h_act.copy_(self.d_act, non_blocking=True)
            self.h_logp.copy_(self.d_logp, non_blocking=True)
            self.done.record(self.stream)

    def collect(self):
        self.done.synchronize()
        return self.h_act.numpy().copy(), self.h_logp.numpy().copy()


def test_alternating_groups_match_the_oracle_and_the_single_group():
    import torch
    import paper_1803_02811_amd as arn
    from tests import gpu_util as gu
    flat = wl.he_normal_params(A, "pv", seed=2900, bias_std=0.05)
    net = gu.GpuNet(A, "pv", flat)
    spec = orc.NetSpec(A, "pv")
    params = orc.unflatten(flat, spec)
    half = N_SIMS // 2
    frames = [wl.rect_frames(N_SIMS, seed=1900 + r) for r in range(ROUNDS)]           # the frames change every step
    unif = [wl.action_uniforms(N_SIMS, seed=10 + r)["u"] for r in range(ROUNDS)]
    groups = [_Group(torch, arn, gu, net.cfg, half), _Group(torch, arn, gu, net.cfg, N_SIMS - half)]
    spans = [slice(0, half), slice(half, N_SIMS)]
    got_act = np.full((ROUNDS, N_SIMS), -1, dtype=np.int32)
    got_logp = np.full((ROUNDS, N_SIMS), np.nan, dtype=np.float32)
    # steady state of the alternation: a group's next request is issued as soon as its actions are back, while
    # the other group's request is still in flight
    for g, sp in zip(groups, spans):
        g.issue(torch, arn, net.cfg, net.packed, frames[0][sp], unif[0][sp])
    for r in range(ROUNDS):
        for g, sp in zip(groups, spans):
            got_act[r, sp], got_logp[r, sp] = g.collect()
            if r + 1 < ROUNDS:
                g.issue(torch, arn, net.cfg, net.packed, frames[r + 1][sp], unif[r + 1][sp])
    torch.cuda.synchronize()
    n_clear = 0
    for r in range(ROUNDS):
        # one group of all simulators, device-resident inputs: the same bits
        one_act, one_logp = net.act(frames[r], unif[r], np.zeros(N_SIMS, dtype=np.float32), want_logp=True)
        assert np.array_equal(got_act[r], one_act), "round %d: two-group actions differ from the one-group call" % r
        assert np.array_equal(got_logp[r], one_logp), "round %d: log-probabilities differ" % r
        # the oracle's draw wherever u is clear of every CDF boundary by 5e-3 (the greedy rule's gap of 1e-2, half
        # for each side of a boundary)
        cache = orc.forward(params, frames[r], spec)
        logp = orc.log_softmax(cache["logits"])
        probs = np.exp(logp)
        want = orc.sample_categorical(probs, unif[r])
        margin = np.abs(np.cumsum(probs, axis=1) - unif[r][:, None].astype(np.float64)).min(axis=1)
        clear = margin > 5e-3
        n_clear += int(clear.sum())
        np.testing.assert_array_equal(got_act[r][clear], want[clear])
        assert (np.abs(got_act[r][~clear].astype(int) - want[~clear]) <= 1).all()
        gu.tol_check(got_logp[r], logp[np.arange(N_SIMS), got_act[r]], "log pi(drawn action), round %d" % r)
    assert n_clear > 0.75 * ROUNDS * N_SIMS
    assert len({tuple(a) for a in got_act}) == ROUNDS            # the rounds really saw different frames


def test_two_gradient_steps_back_to_back_on_two_streams():
    """Two arn_train_step_grads calls issued one after the other from this thread on two caller streams (the
    library's side stream and events are shared between them): each gives the bits of the same call made alone."""
    import torch
    import paper_1803_02811_amd as arn
    from tests import gpu_util as gu
    B = 300
    flat = wl.he_normal_params(A, "pv", 2003, bias_std=0.05)
    net = gu.GpuNet(A, "pv", flat)
    batches = [wl.actor_critic_batch(3, B=B), wl.actor_critic_batch(4, B=B)]
    alone = [net.train(b, "a2c") for b in batches]
    assert not np.array_equal(alone[0][0], alone[1][0])
    dev = [net.device_batch(b) for b in batches]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ws = [torch.empty(arn.workspace_bytes(net.cfg, B, arn.ARN_MODE_TRAIN), dtype=torch.uint8, device=gu.DEV) for _ in range(2)]
    for rep in range(3):
        dW = [torch.full((net.nparam,), float("nan"), dtype=torch.float32, device=gu.DEV) for _ in range(2)]
        loss = [torch.empty(4, dtype=torch.float32, device=gu.DEV) for _ in range(2)]
        torch.cuda.synchronize()
        for i in range(2):
            arn.train_step_grads(net.cfg, net.packed, dev[i], "a2c", dW[i], loss[i], workspace=ws[i], stream=streams[i])
        for i in range(2):
            streams[i].synchronize()        # each caller stream alone orders the whole call, side-stream work included
            assert np.array_equal(dW[i].cpu().numpy(), alone[i][0]), (rep, i)
            assert np.array_equal(loss[i].cpu().numpy(), alone[i][1]), (rep, i)
