"""TEST INFRASTRUCTURE ONLY -- slow, plain CPU oracle for the parameter update rules.

What this file is
-----------------
fp64 numpy statements of the three update rules the paper's learners apply to the
flat parameter vector after a gradient has been computed.  Only tests, the smoke
check and the CPU-baseline leg of the benchmark may import it; it shares no code
with the GPU library and neither imports the other.

Where each rule comes from
--------------------------
* RMSProp: appendix "Experiment Details" (A2C) and the appendix on update rules,
  which says: no momentum, squared gradients accumulated directly, and points to
  the `rmsprop` routine of a public library for the exact form.  That form is
      accu <- rho*accu + (1-rho)*g^2 ;  theta <- theta - lr*g / sqrt(accu + eps)
  (epsilon inside the square root).
* Adam: appendix "Update Rule for Multi-Step Asynchronous Adam", first block of
  equations (t, a, m, v, s, theta), all state zero-initialised.
* Multi-step asynchronous Adam: same appendix, second block (local accumulators
  a_g, a_g2, a_s) and third block (merge into the central parameters, which carry
  a tilde in the paper and the suffix `_c` here), n = number of local steps since
  the last merge.

Readings taken (each also listed in the design notes)
* The step formula is printed without an operator between sqrt(v) and epsilon;
  it is read as s = a*m / (sqrt(v) + eps), the standard rule of the optimiser the
  appendix cites.
* t is the learner's own step counter and is not touched by a merge.
* The merge assigns the new central values to the local copies as well, then
  clears the accumulators, in the order the equations are printed.

Parity pins: tests/test_oracle_updates.py.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


def rmsprop_step(theta, accu, g, lr, rho, eps):
    """One RMSProp step without momentum; returns (theta, accu) as new fp64 arrays."""
    theta = np.asarray(theta, np.float64)
    accu = np.asarray(accu, np.float64)
    g = np.asarray(g, np.float64)
    accu = rho * accu + (1.0 - rho) * g * g
    theta = theta - lr * g / np.sqrt(accu + eps)
    return theta, accu


def adam_scale(t, r, beta1, beta2):
    """a = r * sqrt(1 - beta2^t) / (1 - beta1^t) for step count t >= 1 (after the increment)."""
    return r * np.sqrt(1.0 - beta2 ** t) / (1.0 - beta1 ** t)


def adam_step(theta, m, v, g, t, r, beta1, beta2, eps):
    """One Adam step.  `t` is the step count after the increment (1 for the first step).

    Returns (theta, m, v, s) as new fp64 arrays; s is the step that was subtracted.
    """
    theta = np.asarray(theta, np.float64)
    g = np.asarray(g, np.float64)
    a = adam_scale(t, r, beta1, beta2)
    m = beta1 * np.asarray(m, np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, np.float64) + (1.0 - beta2) * g * g
    s = a * m / (np.sqrt(v) + eps)
    return theta - s, m, v, s


@dataclass
class AsyncAdamLearner:
    """Local state of one learner of the multi-step asynchronous rule."""
    theta: np.ndarray
    m: np.ndarray
    v: np.ndarray
    a_g: np.ndarray = field(default=None)
    a_g2: np.ndarray = field(default=None)
    a_s: np.ndarray = field(default=None)
    t: int = 0
    n: int = 0     # local steps since the last merge

    def __post_init__(self):
        self.theta = np.array(self.theta, np.float64)
        self.m = np.array(self.m, np.float64)
        self.v = np.array(self.v, np.float64)
        for name in ("a_g", "a_g2", "a_s"):
            if getattr(self, name) is None:
                setattr(self, name, np.zeros_like(self.theta))


def async_adam_local_step(L: AsyncAdamLearner, g, r, beta1, beta2, eps):
    """A local Adam step plus the three local accumulations."""
    g = np.asarray(g, np.float64)
    L.t += 1
    L.theta, L.m, L.v, s = adam_step(L.theta, L.m, L.v, g, L.t, r, beta1, beta2, eps)
    L.a_g = beta1 * L.a_g + g
    L.a_g2 = beta2 * L.a_g2 + g * g
    L.a_s = L.a_s + s
    L.n += 1


def async_adam_merge(L: AsyncAdamLearner, theta_c, m_c, v_c, beta1, beta2):
    """Apply learner L's accumulated steps to the central values; returns the new (theta_c, m_c, v_c).

    The learner's local copies take the same new values and its accumulators are cleared.
    """
    n = L.n
    theta_c = np.asarray(theta_c, np.float64) - L.a_s
    m_c = beta1 ** n * np.asarray(m_c, np.float64) + (1.0 - beta1) * L.a_g
    v_c = beta2 ** n * np.asarray(v_c, np.float64) + (1.0 - beta2) * L.a_g2
    L.theta, L.m, L.v = theta_c.copy(), m_c.copy(), v_c.copy()
    L.a_g = np.zeros_like(L.a_g)
    L.a_g2 = np.zeros_like(L.a_g2)
    L.a_s = np.zeros_like(L.a_s)
    L.n = 0
    return theta_c, m_c, v_c
