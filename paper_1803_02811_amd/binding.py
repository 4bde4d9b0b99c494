"""ctypes binding for libarn.so: same names as the C entry points, argument
marshalling only.  Tensors are torch device tensors used purely as memory."""
from __future__ import annotations

import ctypes
import os
from typing import Optional

ARN_HEAD_PV, ARN_HEAD_C51, ARN_HEAD_Q, ARN_HEAD_DUEL = 0, 1, 2, 3
ARN_LOSS_A2C, ARN_LOSS_PPO, ARN_LOSS_C51, ARN_LOSS_DQN = 0, 1, 2, 3
ARN_MODE_FORWARD, ARN_MODE_TRAIN = 0, 1
ARN_GEOM_84, ARN_GEOM_PAPER, ARN_GEOM_A3C = 0, 1, 2
LOSS_KINDS = {"a2c": ARN_LOSS_A2C, "ppo": ARN_LOSS_PPO, "c51": ARN_LOSS_C51, "dqn": ARN_LOSS_DQN}
HEAD_KINDS = {"pv": ARN_HEAD_PV, "c51": ARN_HEAD_C51, "q": ARN_HEAD_Q, "duel": ARN_HEAD_DUEL}
GEOMETRIES = {"84": ARN_GEOM_84, "paper": ARN_GEOM_PAPER, "a3c": ARN_GEOM_A3C}


class Config(ctypes.Structure):
    """Mirror of arn_config."""
    _fields_ = [("num_actions", ctypes.c_int32), ("head_kind", ctypes.c_int32), ("num_atoms", ctypes.c_int32),
                ("v_min", ctypes.c_float), ("v_max", ctypes.c_float), ("gamma", ctypes.c_float),
                ("clip_eps", ctypes.c_float), ("value_coef", ctypes.c_float), ("entropy_coef", ctypes.c_float),
                ("double_q", ctypes.c_int32), ("geometry", ctypes.c_int32)]

    def __init__(self, num_actions=18, head_kind=ARN_HEAD_PV, num_atoms=51, v_min=-10.0, v_max=10.0, gamma=0.99,
                 clip_eps=0.1, value_coef=0.5, entropy_coef=0.01, double_q=0, geometry=ARN_GEOM_84):
        super().__init__(num_actions, head_kind, num_atoms, v_min, v_max, gamma, clip_eps, value_coef, entropy_coef,
                         int(double_q), int(geometry))


class _Batch(ctypes.Structure):
    """Mirror of arn_batch."""
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("obs", "action", "adv", "ret", "old_logp", "next_obs", "reward", "done", "w_target_packed",
                 "next_action")]


class ArnError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} ({status})")


_LIB = None


def lib_path() -> str:
    """In-tree libarn.so, or the library named by the ARN_LIBRARY environment variable."""
    return os.environ.get("ARN_LIBRARY") or os.path.join(os.path.dirname(os.path.abspath(__file__)), "libarn.so")


def load_library():
    """Load libarn.so (built by paper_1803_02811_amd.build); no fallback exists."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: run `python -m paper_1803_02811_amd.build` first")
        lib = ctypes.CDLL(path)
        vp, cp = ctypes.c_void_p, ctypes.POINTER(Config)
        lib.arn_status_string.restype = ctypes.c_char_p
        lib.arn_status_string.argtypes = [ctypes.c_int]
        for name in ("arn_param_count", "arn_packed_bytes"):
            getattr(lib, name).restype = ctypes.c_size_t
            getattr(lib, name).argtypes = [cp]
        lib.arn_workspace_bytes.restype = ctypes.c_size_t
        lib.arn_workspace_bytes.argtypes = [cp, ctypes.c_int, ctypes.c_int]
        lib.arn_weights_prepare.restype = ctypes.c_int
        lib.arn_weights_prepare.argtypes = [cp, vp, vp, vp]
        lib.arn_policy_forward.restype = ctypes.c_int
        lib.arn_policy_forward.argtypes = [cp, vp, vp, ctypes.c_int, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.arn_policy_forward_static.restype = ctypes.c_int
        lib.arn_policy_forward_static.argtypes = [cp, vp, vp, ctypes.c_int, vp, vp, vp, vp, vp]
        lib.arn_policy_act.restype = ctypes.c_int
        lib.arn_policy_act.argtypes = [cp, vp, vp, ctypes.c_int, vp, vp, ctypes.c_float, vp, vp, vp, ctypes.c_size_t, vp]
        lib.arn_train_step_grads.restype = ctypes.c_int
        lib.arn_train_step_grads.argtypes = [cp, vp, ctypes.POINTER(_Batch), ctypes.c_int, ctypes.c_int, vp, vp, vp,
                                             ctypes.c_size_t, vp]
        f, i64, sz = ctypes.c_float, ctypes.c_int64, ctypes.c_size_t
        lib.arn_rmsprop_update.restype = ctypes.c_int
        lib.arn_rmsprop_update.argtypes = [sz, vp, vp, vp, f, f, f, cp, vp, vp]
        lib.arn_adam_update.restype = ctypes.c_int
        lib.arn_adam_update.argtypes = [sz, vp, vp, vp, vp, i64, f, f, f, f, cp, vp, vp]
        lib.arn_async_adam_local_step.restype = ctypes.c_int
        lib.arn_async_adam_local_step.argtypes = [sz, vp, vp, vp, vp, vp, vp, vp, i64, f, f, f, f, cp, vp, vp]
        lib.arn_async_adam_merge.restype = ctypes.c_int
        lib.arn_async_adam_merge.argtypes = [sz, vp, vp, vp, vp, vp, vp, vp, vp, vp, ctypes.c_int, f, f, cp, vp, vp]
        lib.arn_profile_enable.restype = ctypes.c_int
        lib.arn_profile_enable.argtypes = [ctypes.c_int]
        lib.arn_profile_null.restype = ctypes.c_int
        lib.arn_profile_null.argtypes = [vp]
        lib.arn_profile_collect.restype = ctypes.c_int
        lib.arn_profile_collect.argtypes = [ctypes.c_char_p, ctypes.POINTER(ctypes.c_float), ctypes.c_int]
        _LIB = lib
    return _LIB


def status_string(status: int) -> str:
    return load_library().arn_status_string(int(status)).decode()


def param_count(cfg: Config) -> int:
    return int(load_library().arn_param_count(ctypes.byref(cfg)))


def packed_bytes(cfg: Config) -> int:
    return int(load_library().arn_packed_bytes(ctypes.byref(cfg)))


def workspace_bytes(cfg: Config, B: int, mode: int) -> int:
    return int(load_library().arn_workspace_bytes(ctypes.byref(cfg), int(B), int(mode)))


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream) or None
    return int(getattr(stream, "cuda_stream", stream)) or None


def _check(status: int, where: str):
    if status != 0:
        raise ArnError(status, where)


def weights_prepare(cfg: Config, w_fp32, w_packed, stream=None) -> None:
    _check(load_library().arn_weights_prepare(ctypes.byref(cfg), _ptr(w_fp32), _ptr(w_packed), _stream(stream)),
           "arn_weights_prepare")


def policy_forward(cfg: Config, w_packed, obs, logits, value=None, probs=None, greedy=None, *, workspace,
                   stream=None) -> None:
    B = int(obs.shape[0])
    _check(load_library().arn_policy_forward(
        ctypes.byref(cfg), _ptr(w_packed), _ptr(obs), B, _ptr(logits), _ptr(value), _ptr(probs), _ptr(greedy),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)), "arn_policy_forward")


STATIC_SCRATCH_BYTES = 32 << 20   # ARN_STATIC_SCRATCH_BYTES of the header


def policy_forward_static(cfg: Config, w_packed, obs, logits, value=None, probs=None, greedy=None, *, stream=None) -> None:
    B = int(obs.shape[0])
    _check(load_library().arn_policy_forward_static(
        ctypes.byref(cfg), _ptr(w_packed), _ptr(obs), B, _ptr(logits), _ptr(value), _ptr(probs), _ptr(greedy),
        _stream(stream)), "arn_policy_forward_static")


def policy_act(cfg: Config, w_packed, obs, u, u2, action, logp=None, *, epsilon=0.0, workspace, stream=None) -> None:
    B = int(obs.shape[0])
    _check(load_library().arn_policy_act(
        ctypes.byref(cfg), _ptr(w_packed), _ptr(obs), B, _ptr(u), _ptr(u2), float(epsilon), _ptr(action), _ptr(logp),
        _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream)), "arn_policy_act")


def train_step_grads(cfg: Config, w_packed, batch: dict, loss_kind, dW, loss, *, workspace, stream=None) -> None:
    """batch: dict of device tensors keyed like arn_batch's fields (missing = NULL); "next_action" is an output."""
    kind = LOSS_KINDS[loss_kind] if isinstance(loss_kind, str) else int(loss_kind)
    b = _Batch(*[_ptr(batch.get(n)) for n, _ in _Batch._fields_])
    B = int(batch["obs"].shape[0])
    _check(load_library().arn_train_step_grads(
        ctypes.byref(cfg), _ptr(w_packed), ctypes.byref(b), B, kind, _ptr(dW), _ptr(loss), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _stream(stream)), "arn_train_step_grads")


def _cfg_ref(cfg):
    return None if cfg is None else ctypes.byref(cfg)


def rmsprop_update(theta, g, accu, *, lr, rho, eps, cfg: Optional[Config] = None, w_packed=None, stream=None) -> None:
    _check(load_library().arn_rmsprop_update(
        theta.numel(), _ptr(theta), _ptr(g), _ptr(accu), lr, rho, eps, _cfg_ref(cfg), _ptr(w_packed),
        _stream(stream)), "arn_rmsprop_update")


def adam_update(theta, g, m, v, *, t, r, beta1, beta2, eps, cfg: Optional[Config] = None, w_packed=None,
                stream=None) -> None:
    _check(load_library().arn_adam_update(
        theta.numel(), _ptr(theta), _ptr(g), _ptr(m), _ptr(v), int(t), r, beta1, beta2, eps, _cfg_ref(cfg),
        _ptr(w_packed), _stream(stream)), "arn_adam_update")


def async_adam_local_step(theta, g, m, v, a_g, a_g2, a_s, *, t, r, beta1, beta2, eps, cfg: Optional[Config] = None,
                          w_packed=None, stream=None) -> None:
    _check(load_library().arn_async_adam_local_step(
        theta.numel(), _ptr(theta), _ptr(g), _ptr(m), _ptr(v), _ptr(a_g), _ptr(a_g2), _ptr(a_s), int(t), r, beta1,
        beta2, eps, _cfg_ref(cfg), _ptr(w_packed), _stream(stream)), "arn_async_adam_local_step")


def async_adam_merge(theta_c, m_c, v_c, theta, m, v, a_g, a_g2, a_s, *, n_local, beta1, beta2,
                     cfg: Optional[Config] = None, w_packed=None, stream=None) -> None:
    _check(load_library().arn_async_adam_merge(
        theta.numel(), _ptr(theta_c), _ptr(m_c), _ptr(v_c), _ptr(theta), _ptr(m), _ptr(v), _ptr(a_g), _ptr(a_g2),
        _ptr(a_s), int(n_local), beta1, beta2, _cfg_ref(cfg), _ptr(w_packed), _stream(stream)),
        "arn_async_adam_merge")


def profile_enable(on: bool) -> None:
    load_library().arn_profile_enable(1 if on else 0)


def profile_null(stream=None) -> None:
    load_library().arn_profile_null(_stream(stream))


def profile_collect(cap: int = 4096):
    """[(kernel name, milliseconds)] in launch order for the launches recorded since enabling."""
    names = ctypes.create_string_buffer(cap * 32)
    ms = (ctypes.c_float * cap)()
    n = load_library().arn_profile_collect(names, ms, cap)
    return [(names.raw[i * 32:(i + 1) * 32].split(b"\0", 1)[0].decode(), float(ms[i])) for i in range(n)]
