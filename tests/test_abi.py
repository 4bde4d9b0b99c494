"""CPU-only checks of the C ABI: the library loads, exports every symbol the
header declares, sizes agree with the oracle's layout, and argument errors are
caught on the host before anything touches a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1803_02811_amd as arn
from oracle import nature_cnn as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(arn.lib_path()):
        from paper_1803_02811_amd import build
        build.build()
    return arn.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "arn.h")).read()
    declared = set(re.findall(r"\b(arn_[a-z_]+)\s*\(", header))
    assert {"arn_policy_forward", "arn_train_step_grads", "arn_weights_prepare", "arn_param_count",
            "arn_packed_bytes", "arn_workspace_bytes", "arn_status_string"} <= declared
    for name in declared:
        assert hasattr(lib, name), name


def test_param_counts_match_the_oracle_layout(lib):
    for A, head, okind in [(6, arn.ARN_HEAD_PV, "pv"), (18, arn.ARN_HEAD_PV, "pv"), (18, arn.ARN_HEAD_C51, "c51")]:
        assert arn.param_count(arn.Config(A, head)) == orc.param_count(orc.NetSpec(A, okind))
    assert arn.param_count(arn.Config(18, arn.ARN_HEAD_PV)) == 1_693_875
    assert arn.param_count(arn.Config(18, arn.ARN_HEAD_C51)) == 2_155_062


def test_paper_geometry_sizes(lib):
    """Appendix "Atari Frame Processing": 104x80 frames, conv2/conv3 padded by 1 -> 12x9 feature map, fc 6912 -> 512."""
    for A, head, okind in [(18, arn.ARN_HEAD_PV, "pv"), (18, arn.ARN_HEAD_C51, "c51"), (6, arn.ARN_HEAD_DUEL, "duel")]:
        cfg = arn.Config(A, head, geometry=arn.ARN_GEOM_PAPER)
        assert arn.param_count(cfg) == orc.param_count(orc.NetSpec(A, okind, geometry=orc.PAPER_104x80))
    cfg = arn.Config(18, geometry=arn.ARN_GEOM_PAPER)
    assert arn.param_count(cfg) == 1_693_875 + 512 * (6912 - 3136)
    assert arn.packed_bytes(cfg) > arn.packed_bytes(arn.Config(18))
    assert arn.workspace_bytes(cfg, 64, arn.ARN_MODE_TRAIN) > arn.workspace_bytes(arn.Config(18), 64, arn.ARN_MODE_TRAIN)
    bad = arn.Config(18, geometry=3)
    assert arn.param_count(bad) == 0 and arn.packed_bytes(bad) == 0
    assert arn.workspace_bytes(bad, 64, arn.ARN_MODE_FORWARD) == 0
    fake = ctypes.c_void_p(1 << 20)
    assert lib.arn_weights_prepare(ctypes.byref(bad), fake, fake, None) == -2


def test_two_convolution_network_sizes(lib):
    """ARN_GEOM_A3C: the flat vector is the small network's own (oracle layout), whatever the kernels embed it in."""
    for A, head, okind in [(18, arn.ARN_HEAD_PV, "pv"), (6, arn.ARN_HEAD_PV, "pv"), (18, arn.ARN_HEAD_C51, "c51"),
                           (4, arn.ARN_HEAD_Q, "q"), (9, arn.ARN_HEAD_DUEL, "duel")]:
        cfg = arn.Config(A, head, geometry=arn.ARN_GEOM_A3C)
        assert arn.param_count(cfg) == orc.param_count(orc.NetSpec(A, okind, geometry=orc.A3C_104x80))
    cfg = arn.Config(18, geometry=arn.ARN_GEOM_A3C)
    assert arn.param_count(cfg) == 897_328 + 18 * 256 + 18 + 256 + 1
    big = arn.Config(18, geometry=arn.ARN_GEOM_PAPER)
    assert arn.packed_bytes(cfg) >= arn.packed_bytes(big) + 4 * arn.param_count(big)
    assert arn.workspace_bytes(cfg, 64, arn.ARN_MODE_TRAIN) >= arn.workspace_bytes(big, 64, arn.ARN_MODE_TRAIN) + 4 * arn.param_count(big)
    assert arn.workspace_bytes(cfg, 64, arn.ARN_MODE_FORWARD) == arn.workspace_bytes(big, 64, arn.ARN_MODE_FORWARD)


def test_sizes_and_bad_configs(lib):
    cfg = arn.Config(18, arn.ARN_HEAD_PV)
    assert arn.packed_bytes(cfg) > 2 * 1_693_875          # bf16 copies of every matrix
    f16, f256 = arn.workspace_bytes(cfg, 16, arn.ARN_MODE_FORWARD), arn.workspace_bytes(cfg, 256, arn.ARN_MODE_FORWARD)
    assert 0 < f16 < f256
    assert arn.workspace_bytes(cfg, 256, arn.ARN_MODE_TRAIN) > f256
    assert arn.workspace_bytes(cfg, 0, arn.ARN_MODE_FORWARD) == 0
    assert arn.workspace_bytes(cfg, 16, 7) == 0
    for bad in [arn.Config(0, arn.ARN_HEAD_PV), arn.Config(32, arn.ARN_HEAD_PV), arn.Config(19, arn.ARN_HEAD_C51),
                arn.Config(18, arn.ARN_HEAD_C51, num_atoms=1), arn.Config(18, 5),
                arn.Config(18, arn.ARN_HEAD_C51, v_min=1.0, v_max=1.0)]:
        assert arn.param_count(bad) == 0 and arn.packed_bytes(bad) == 0
    # the gradient workspace is a fixed function of B (fixed split counts => reproducible sums)
    assert arn.workspace_bytes(cfg, 2048, arn.ARN_MODE_TRAIN) == arn.workspace_bytes(cfg, 2048, arn.ARN_MODE_TRAIN)


def test_argument_errors_are_reported_on_the_host(lib):
    """Null / misaligned pointers, bad kinds and short workspaces return error codes without any launch."""
    cfg = arn.Config(18, arn.ARN_HEAD_PV)
    c = ctypes.byref(cfg)
    fake = ctypes.c_void_p(0x1000)                 # aligned, never dereferenced on these paths
    odd = ctypes.c_void_p(0x1001)
    EINVAL, ESHAPE, EKIND, EWORKSPACE = -1, -2, -3, -4
    assert lib.arn_weights_prepare(None, fake, fake, None) == EINVAL
    assert lib.arn_weights_prepare(c, None, fake, None) == EINVAL
    assert lib.arn_weights_prepare(c, fake, odd, None) == EINVAL
    assert lib.arn_weights_prepare(ctypes.byref(arn.Config(18, 9)), fake, fake, None) == EKIND
    assert lib.arn_weights_prepare(ctypes.byref(arn.Config(40, arn.ARN_HEAD_PV)), fake, fake, None) == ESHAPE
    big = 1 << 40
    assert lib.arn_policy_forward(c, fake, fake, 0, fake, fake, None, None, fake, big, None) == EINVAL
    assert lib.arn_policy_forward(c, fake, None, 4, fake, fake, None, None, fake, big, None) == EINVAL
    assert lib.arn_policy_forward(c, fake, fake, 4, fake, None, None, None, fake, big, None) == EINVAL   # PV needs value
    assert lib.arn_policy_forward(c, fake, fake, 4, fake, fake, None, None, fake, 16, None) == EWORKSPACE
    batch = arn.binding._Batch(*([0x1000] * 9))
    b = ctypes.byref(batch)
    assert lib.arn_train_step_grads(c, fake, b, 4, 9, fake, fake, fake, big, None) == EKIND
    assert lib.arn_train_step_grads(c, fake, b, 4, arn.ARN_LOSS_C51, fake, fake, fake, big, None) == ESHAPE
    assert lib.arn_train_step_grads(c, fake, b, 4, arn.ARN_LOSS_A2C, fake, fake, fake, 64, None) == EWORKSPACE
    assert lib.arn_train_step_grads(c, fake, None, 4, arn.ARN_LOSS_A2C, fake, fake, fake, big, None) == EINVAL
    nob = arn.binding._Batch(*([0x1000] * 2 + [None] * 7))
    assert lib.arn_train_step_grads(c, fake, ctypes.byref(nob), 4, arn.ARN_LOSS_A2C, fake, fake, fake, big,
                                    None) == EINVAL
    assert "workspace" in arn.status_string(EWORKSPACE)


def test_action_value_heads_and_act_argument_errors(lib):
    q = arn.Config(18, arn.ARN_HEAD_Q)
    duel = arn.Config(18, arn.ARN_HEAD_DUEL)
    pv = arn.Config(18, arn.ARN_HEAD_PV)
    assert arn.param_count(q) == orc.param_count(orc.NetSpec(18, "q")) == 1_693_362
    assert arn.param_count(duel) == arn.param_count(pv) == orc.param_count(orc.NetSpec(18, "duel"))
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    EINVAL, ESHAPE, EKIND = -1, -2, -3
    big = 1 << 40
    cq, cp = ctypes.byref(q), ctypes.byref(pv)
    # action-value heads have no probabilities
    assert lib.arn_policy_forward(cq, fake, fake, 4, fake, fake, fake, None, fake, big, None) == ESHAPE
    assert lib.arn_policy_forward(cq, fake, fake, 4, fake, None, None, None, fake, big, None) == EINVAL   # max Q required
    # dqn needs an action-value head and vice versa
    batch = arn.binding._Batch(*([0x1000] * 9))
    b = ctypes.byref(batch)
    assert lib.arn_train_step_grads(cp, fake, b, 4, arn.ARN_LOSS_DQN, fake, fake, fake, big, None) == ESHAPE
    assert lib.arn_train_step_grads(cq, fake, b, 4, arn.ARN_LOSS_A2C, fake, fake, fake, big, None) == ESHAPE
    nonext = arn.binding._Batch(*([0x1000] * 5 + [None] * 4))
    assert lib.arn_train_step_grads(cq, fake, ctypes.byref(nonext), 4, arn.ARN_LOSS_DQN, fake, fake, fake, big,
                                    None) == EINVAL
    # the optional next-action output must be 16-byte aligned when given (checked before anything is launched)
    badnext = arn.binding._Batch(*([0x1000] * 9 + [0x1004]))
    assert lib.arn_train_step_grads(cq, fake, ctypes.byref(badnext), 4, arn.ARN_LOSS_DQN, fake, fake, fake, big,
                                    None) == EINVAL
    # arn_policy_act
    assert lib.arn_policy_act(cp, fake, fake, 4, None, fake, 0.0, fake, None, fake, big, None) == EINVAL      # u
    assert lib.arn_policy_act(cp, fake, fake, 4, fake, None, 0.0, None, None, fake, big, None) == EINVAL      # action
    assert lib.arn_policy_act(cq, fake, fake, 4, fake, None, 0.1, fake, None, fake, big, None) == EINVAL      # u2
    assert lib.arn_policy_act(cq, fake, fake, 4, fake, fake, 1.5, fake, None, fake, big, None) == EINVAL      # epsilon
    assert lib.arn_policy_act(cq, fake, fake, 4, fake, fake, 0.1, fake, fake, fake, big, None) == ESHAPE      # logp
    assert lib.arn_policy_act(cp, fake, fake, 4, fake, None, 0.0, fake, odd, fake, big, None) == EINVAL
    assert lib.arn_policy_act(cp, fake, fake, 4, fake, None, 0.0, fake, None, fake, 16, None) == -4


def test_update_rule_argument_errors(lib):
    cfg = arn.Config(18, arn.ARN_HEAD_PV)
    c = ctypes.byref(cfg)
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1004)
    EINVAL, ESHAPE = -1, -2
    n = arn.param_count(cfg)
    assert lib.arn_rmsprop_update(0, fake, fake, fake, 1e-3, 0.9, 1e-6, None, None, None) == EINVAL
    assert lib.arn_rmsprop_update(8, fake, odd, fake, 1e-3, 0.9, 1e-6, None, None, None) == EINVAL
    assert lib.arn_rmsprop_update(8, fake, fake, fake, 1e-3, 1.0, 1e-6, None, None, None) == EINVAL   # rho = 1
    assert lib.arn_rmsprop_update(8, fake, fake, fake, 1e-3, 0.9, -1.0, None, None, None) == EINVAL
    assert lib.arn_rmsprop_update(n - 1, fake, fake, fake, 1e-3, 0.9, 1e-6, c, fake, None) == ESHAPE  # repack needs n
    assert lib.arn_rmsprop_update(n, fake, fake, fake, 1e-3, 0.9, 1e-6, None, fake, None) == EINVAL   # ... and cfg
    assert lib.arn_adam_update(8, fake, fake, fake, fake, 0, 1e-3, 0.9, 0.999, 1e-5, None, None, None) == EINVAL
    assert lib.arn_adam_update(8, fake, fake, None, fake, 1, 1e-3, 0.9, 0.999, 1e-5, None, None, None) == EINVAL
    assert lib.arn_adam_update(8, fake, fake, fake, fake, 1, 1e-3, 1.5, 0.999, 1e-5, None, None, None) == EINVAL
    assert lib.arn_async_adam_local_step(8, fake, fake, fake, fake, fake, None, fake, 1, 1e-3, 0.9, 0.999, 1e-5,
                                         None, None, None) == EINVAL
    other = ctypes.c_void_p(0x2000)
    assert lib.arn_async_adam_merge(8, fake, fake, fake, fake, other, other, other, other, other, 1, 0.9, 0.999,
                                    None, None, None) == EINVAL      # theta_c aliases theta
    assert lib.arn_async_adam_merge(8, fake, fake, fake, other, other, other, other, other, other, -1, 0.9, 0.999,
                                    None, None, None) == EINVAL


def test_binding_fails_loudly_without_the_library(monkeypatch, tmp_path):
    """No CPU fallback: a missing libarn.so is an error, not a silent detour."""
    monkeypatch.setenv("ARN_LIBRARY", str(tmp_path / "nope.so"))
    monkeypatch.setattr(arn.binding, "_LIB", None)
    with pytest.raises(RuntimeError):
        arn.load_library()
    monkeypatch.delenv("ARN_LIBRARY")
    monkeypatch.setattr(arn.binding, "_LIB", None)


def test_product_path_does_not_import_the_oracle():
    for root, _, files in os.walk(os.path.join(ROOT, "paper_1803_02811_amd")):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".cpp")):
                text = open(os.path.join(root, f)).read()
                assert "oracle" not in text, f


def test_static_scratch_entry_point_rejects_on_the_host(lib):
    """arn_policy_forward_static: same argument checks as arn_policy_forward, and a batch whose forward workspace
    exceeds the library's static buffer is refused (ARN_ESTATIC) before anything is launched."""
    header = open(os.path.join(ROOT, "include", "arn.h")).read()
    m = re.search(r"#define ARN_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", header)
    assert m and int(m.group(1)) << int(m.group(2)) == arn.STATIC_SCRATCH_BYTES
    cfg = arn.Config(18, arn.ARN_HEAD_PV)
    c = ctypes.byref(cfg)
    fake, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x1001)
    fn = lib.arn_policy_forward_static
    assert fn(None, fake, fake, 4, fake, fake, None, None, None) == -1
    assert fn(c, fake, fake, 0, fake, fake, None, None, None) == -1
    assert fn(c, fake, odd, 4, fake, fake, None, None, None) == -1
    assert fn(c, fake, fake, 4, fake, None, None, None, None) == -1          # the policy/value head needs `value`
    assert arn.workspace_bytes(cfg, 256, arn.ARN_MODE_FORWARD) <= arn.STATIC_SCRATCH_BYTES      # the documented example
    too_big = 256
    while arn.workspace_bytes(cfg, too_big, arn.ARN_MODE_FORWARD) <= arn.STATIC_SCRATCH_BYTES:
        too_big *= 2
    assert fn(c, fake, fake, too_big, fake, fake, None, None, None) == -7
    assert b"static" in lib.arn_status_string(-7)
