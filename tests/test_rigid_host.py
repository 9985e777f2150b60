"""Host-side rigid-transform helpers of the package against the oracle's (Eq. 9)."""
import numpy as np

from oracle import neus2_oracle as o
from paper_2212_05231_amd import rigid


def test_rotation_and_its_derivative():
    rng = np.random.default_rng(0)
    for omega in (np.zeros(3), np.array([1e-9, 0.0, 0.0]), np.array([0.3, -0.2, 0.1]), rng.normal(size=3) * 2.0):
        R = rigid.rotation(omega)
        np.testing.assert_allclose(R @ R.T, np.eye(3), atol=1e-12)
        np.testing.assert_allclose(R, o.rotation_from_axis_angle(omega), atol=1e-12)
        M = rng.normal(size=(3, 3))
        b = rng.normal(size=3)
        d_omega, d_T = rigid.transform_gradient(omega, np.zeros(3), M, b)
        np.testing.assert_allclose(d_omega, o.axis_angle_gradient(omega, M), atol=1e-7)
        np.testing.assert_allclose(d_T, R.T @ b, atol=1e-12)


def test_transform_gradient_by_finite_differences_of_a_point_loss():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(20, 3))
    g = rng.normal(size=(20, 3))                  # dL/dx_c of a linear loss L = sum g . x_c
    omega, T = np.array([0.2, 0.5, -0.4]), np.array([0.1, -0.3, 0.05])
    loss = lambda w, t: float(np.sum(g * ((x + t) @ rigid.rotation(w).T)))
    M = g.T @ (x + T)
    d_omega, d_T = rigid.transform_gradient(omega, T, M, g.sum(axis=0))
    h = 1e-6
    for k in range(3):
        e = np.zeros(3)
        e[k] = h
        assert abs((loss(omega + e, T) - loss(omega - e, T)) / (2 * h) - d_omega[k]) < 1e-6
        assert abs((loss(omega, T + e) - loss(omega, T - e)) / (2 * h) - d_T[k]) < 1e-6
