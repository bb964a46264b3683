"""CPU oracle for the sparse feed-forward verification (Sec. 3.4, Eq. 10-14).

TEST INFRASTRUCTURE ONLY: plain numpy in fp64, imported by tests and by the bench's CPU leg, never
by the product, and sharing no code with the HIP path.

  activation     sigma of Eq. 10: SiLU  z / (1 + exp(-z))  (the gate of SwiGLU) or GELU
                 0.5 z (1 + erf(z / sqrt 2)).
  gate           Eq. 10:  h = sigma(W_gate x + b_gate), per token.
  dense_ffn      Eq. 11:  y = W_down (h * (W_up x + b_up)) + b_down.
  inactive       Eq. 12:  S = { i : |h_i| < tau }, per token.
  sparse_ffn     Eq. 13-14, written with index sets as the equations are: per token, the channels
                 outside S are gathered from W_up, b_up, h and from the columns of W_down.

Readings: Eq. 13 writes x with the channel superscript, but x lives in the model dimension, not
in the hidden one: the whole x enters the up projection; likewise b_down of Eq. 14 (a vector of
the model dimension) is added whole.  Every draft token has its own set S (h depends on the
token).  The comparison of Eq. 12 is strict (|h| = tau stays active).  w_down_t is W_down
transposed: [d_ff][d_model].
"""
from __future__ import annotations

from typing import Optional, Tuple

import numpy as np
from scipy.special import erf

from .svf_oracle import _f64


def activation(z: np.ndarray, act: str) -> np.ndarray:
    if act == "silu":
        return z / (1.0 + np.exp(-z))
    if act == "gelu":
        return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))
    raise ValueError("unknown activation")


def _bias(b, n):
    return np.zeros(n) if b is None else _f64(b)


def gate(x, w_gate, b_gate, act: str) -> np.ndarray:
    """h [M][d_ff] (Eq. 10)."""
    wg = _f64(w_gate)
    return activation(_f64(x) @ wg.T + _bias(b_gate, wg.shape[0]), act)


def dense_ffn(x, w_gate, w_up, w_down_t, b_gate=None, b_up=None, b_down=None, act: str = "silu") -> np.ndarray:
    """y [M][d_model] (Eq. 10-11)."""
    wu, wd = _f64(w_up), _f64(w_down_t)
    h = gate(x, w_gate, b_gate, act)
    up = _f64(x) @ wu.T + _bias(b_up, wu.shape[0])
    return (h * up) @ wd + _bias(b_down, wd.shape[1])


def inactive(h: np.ndarray, tau: float) -> np.ndarray:
    """bool [M][d_ff]: channel i of token m belongs to S (Eq. 12)."""
    return np.abs(h) < tau


def sparse_ffn(x, w_gate, w_up, w_down_t, b_gate=None, b_up=None, b_down=None, act: str = "silu",
               tau: float = 0.0, active: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(y [M][d_model], active bool [M][d_ff], h [M][d_ff]) by Eq. 12-14.  `active` overrides
    the set of Eq. 12 (the complement of S) when given."""
    xf, wu, wd = _f64(x), _f64(w_up), _f64(w_down_t)
    bu, bd = _bias(b_up, wu.shape[0]), _bias(b_down, wd.shape[1])
    h = gate(x, w_gate, b_gate, act)
    act_set = ~inactive(h, tau) if active is None else np.asarray(active, dtype=bool)
    y = np.empty((xf.shape[0], wd.shape[1]))
    for m in range(xf.shape[0]):
        keep = np.flatnonzero(act_set[m])                 # the channels outside S
        h_up = h[m, keep] * (wu[keep] @ xf[m] + bu[keep])  # Eq. 13
        y[m] = wd[keep].T @ h_up + bd                       # Eq. 14
    return y, act_set, h
