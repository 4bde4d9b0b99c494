"""HIP-graph capture of the inference and gradient calls: every replay must equal the eager result.

The library launches only kernels and (in the gradient step) event record / wait pairs between the caller's
stream and its own side stream, all of which can be captured; it issues no memset and allocates nothing.
Replays are interleaved with eager work and synchronisations, and each is compared bit for bit."""
import numpy as np
import pytest
import torch

import paper_1803_02811_amd as arn
import workloads as wl
from tests.gpu_util import DEV, GpuNet

pytestmark = pytest.mark.gpu


def test_policy_forward_graph_replays_equal_eager():
    A, B = 18, 48
    net = GpuNet(A, "pv", wl.he_normal_params(A, "pv", seed=2900, bias_std=0.05))
    frames = [wl.rect_frames(B, seed=1900 + i) for i in range(3)]
    obs = torch.from_numpy(frames[0]).to(DEV)
    ws = net.workspace(B, arn.ARN_MODE_FORWARD)
    logits = torch.empty(B, A, dtype=torch.float32, device=DEV)
    value = torch.empty(B, dtype=torch.float32, device=DEV)
    greedy = torch.empty(B, dtype=torch.int32, device=DEV)

    def call(stream=None):
        arn.policy_forward(net.cfg, net.packed, obs, logits, value, None, greedy, workspace=ws, stream=stream)

    eager = []
    for f in frames:
        obs.copy_(torch.from_numpy(f))
        call()
        torch.cuda.synchronize()
        eager.append((logits.clone(), value.clone(), greedy.clone()))

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        call(side)                                   # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        call(torch.cuda.current_stream())
    for rep in range(2):
        for f, want in zip(frames, eager):
            obs.copy_(torch.from_numpy(f))
            logits.zero_(), value.zero_(), greedy.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(logits, want[0]) and torch.equal(value, want[1]) and torch.equal(greedy, want[2])
            call()                                   # eager work between the replays
            torch.cuda.synchronize()


def test_train_step_graph_replays_equal_eager():
    """The gradient step forks to and joins from the library's side stream inside the call; captured, the side
    stream's work becomes part of the graph."""
    A, B = 18, 64
    net = GpuNet(A, "pv", wl.he_normal_params(A, "pv", seed=2901, bias_std=0.05))
    batches = [wl.actor_critic_batch(3, B=B), wl.actor_critic_batch(4, B=B)]
    dev = net.device_batch(batches[0])
    ws = net.workspace(B, arn.ARN_MODE_TRAIN)
    dW = torch.empty(net.nparam, dtype=torch.float32, device=DEV)
    loss = torch.empty(4, dtype=torch.float32, device=DEV)

    def load(b):
        nb = net.device_batch(b)
        for k in dev:
            dev[k].copy_(nb[k])

    def call(stream=None):
        arn.train_step_grads(net.cfg, net.packed, dev, "a2c", dW, loss, workspace=ws, stream=stream)

    eager = []
    for b in batches:
        load(b)
        call()
        torch.cuda.synchronize()
        eager.append((dW.clone(), loss.clone()))

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(torch.cuda.current_stream())
    for rep in range(2):
        for b, want in zip(batches, eager):
            load(b)
            dW.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(dW, want[0]) and torch.equal(loss, want[1])
            call()
            torch.cuda.synchronize()
