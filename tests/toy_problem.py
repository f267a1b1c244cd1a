"""Synthetic strongly convex least-squares problem for the end-to-end tests (not a test itself).

f_i(w) = 0.5 (a_i^T w - y_i)^2 with E[a a^T] = diag(eig), eig in [mu, L]: every f is smooth, the
mean is mu-strongly convex (Assumptions 1-3 of Sec. 2 hold on a bounded region).  Gradients are
computed in numpy fp32 on the host so that the oracle-driven and the library-driven loops see the
same numbers.
"""
import numpy as np


def make_problem(d=256, n=4096, seed=0, mu=0.1, L=1.0, noise=0.1):
    rng = np.random.default_rng(seed)
    eig = np.linspace(mu, L, d)
    A = (rng.standard_normal((n, d)) * np.sqrt(eig)).astype(np.float32)
    w_true = rng.standard_normal(d).astype(np.float32)
    y = (A @ w_true + noise * rng.standard_normal(n).astype(np.float32)).astype(np.float32)
    w_star = np.linalg.lstsq(A.astype(np.float64), y.astype(np.float64), rcond=None)[0]
    return A, y, w_star


def loss(A, y, w):
    r = A.astype(np.float64) @ np.asarray(w, np.float64) - y
    return 0.5 * float(np.mean(r * r))


def minibatch_grad(A, y, w, idx):
    Ab = A[idx]
    r = (Ab @ w - y[idx]).astype(np.float32)
    return ((Ab.T @ r) / np.float32(len(idx))).astype(np.float32)


def schedule(t, eta0=0.1, K0=30):
    """Epoch t: fixed learning rate eta_t, K_t inner steps; eta decreases and K_t grows (Sec. 2.2)."""
    return np.float32(eta0 / (1 + 0.5 * t)), int(K0 * (1 + 0.5 * t))
