"""Host side of the global rigid transform of a dynamic frame (Eq. 9: x_c = R (x + T)).

The device reduces the step's position gradient to M = sum_i g_i (x_i + T)^T (3x3) and
b = sum_i g_i (3), where g_i is dL/dx_c of point i (neus2_rigid_bwd).  What is left is a
handful of 3x3 products on the host: the rotation matrix of the axis-angle parameters, and
the chain rule from (M, b) to the six parameters.
"""
from __future__ import annotations

import numpy as np


def _skew(w: np.ndarray) -> np.ndarray:
    return np.array([[0.0, -w[2], w[1]], [w[2], 0.0, -w[0]], [-w[1], w[0], 0.0]])


def rotation(omega) -> np.ndarray:
    """R = exp([omega]_x) = I + a K + b K^2 with a = sin(t)/t, b = (1 - cos t)/t^2, t = |omega|."""
    w = np.asarray(omega, dtype=np.float64)
    t2 = float(w @ w)
    K = _skew(w)
    if t2 < 1e-16:
        return np.eye(3) + K + 0.5 * (K @ K)
    t = np.sqrt(t2)
    return np.eye(3) + (np.sin(t) / t) * K + ((1.0 - np.cos(t)) / t2) * (K @ K)


def rotation_derivatives(omega):
    """dR/domega_k for k = 0, 1, 2 in closed form (derivative of the formula above)."""
    w = np.asarray(omega, dtype=np.float64)
    t2 = float(w @ w)
    K = _skew(w)
    K2 = K @ K
    out = []
    if t2 < 1e-12:                       # a -> 1 - t^2/6, b -> 1/2 - t^2/24
        a, b, da, db = 1.0, 0.5, -1.0 / 3.0, -1.0 / 12.0        # da, db: derivative with respect to t^2, times 2
    else:
        t = np.sqrt(t2)
        a, b = np.sin(t) / t, (1.0 - np.cos(t)) / t2
        da = (np.cos(t) - a) / t2          # (1/t) da/dt
        db = (a - 2.0 * b) / t2            # (1/t) db/dt
    for k in range(3):
        e = np.zeros(3)
        e[k] = 1.0
        E = _skew(e)
        out.append(a * E + b * (E @ K + K @ E) + w[k] * (da * K + db * K2))
    return out


def transform_gradient(omega, shift, M, b):
    """(dL/domega [3], dL/dT [3]) from the device's M and b.
    x_c = R (x + T):  dL/dT = R^T b,  dL/domega_k = sum_ij (dR/domega_k)_ij M_ij."""
    R = rotation(omega)
    M = np.asarray(M, dtype=np.float64).reshape(3, 3)
    d_omega = np.array([float(np.sum(dR * M)) for dR in rotation_derivatives(omega)])
    return d_omega, R.T @ np.asarray(b, dtype=np.float64)
