"""MI355X-native Nature-CNN hot path (policy inference and training gradients).

Thin binding over the C ABI in include/arn.h; every step runs in the HIP
kernels of libarn.so.  Importing the package does not load the library;
the first call does, and fails loudly if it has not been built.
"""
from .binding import (STATIC_SCRATCH_BYTES, policy_forward_static, ARN_GEOM_84, ARN_GEOM_PAPER, ARN_GEOM_A3C, GEOMETRIES, ARN_HEAD_C51, ARN_HEAD_DUEL, ARN_HEAD_PV, ARN_HEAD_Q, ARN_LOSS_DQN, HEAD_KINDS, policy_act, profile_null, ARN_LOSS_A2C, ARN_LOSS_C51, ARN_LOSS_PPO, ARN_MODE_FORWARD,
                      ARN_MODE_TRAIN, ArnError, Config, lib_path, load_library, packed_bytes, param_count,
                      policy_forward, profile_collect, profile_enable, status_string, train_step_grads, weights_prepare,
                      workspace_bytes, rmsprop_update, adam_update, async_adam_local_step, async_adam_merge)

__all__ = [
    "STATIC_SCRATCH_BYTES", "policy_forward_static", "ARN_GEOM_84", "ARN_GEOM_PAPER", "ARN_GEOM_A3C", "GEOMETRIES", "ARN_HEAD_DUEL", "ARN_HEAD_Q", "ARN_LOSS_DQN", "HEAD_KINDS", "policy_act", "profile_null", "ARN_HEAD_C51", "ARN_HEAD_PV", "ARN_LOSS_A2C", "ARN_LOSS_C51", "ARN_LOSS_PPO", "ARN_MODE_FORWARD",
    "ARN_MODE_TRAIN", "ArnError", "Config", "lib_path", "load_library", "packed_bytes", "param_count",
    "policy_forward", "profile_collect", "profile_enable", "status_string", "train_step_grads", "weights_prepare",
    "workspace_bytes", "rmsprop_update", "adam_update", "async_adam_local_step", "async_adam_merge",
]
