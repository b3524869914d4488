"""Floating-point counterparts of the integer ops (float64 numpy), for tolerance tests.

Each function is the textbook definition applied to *dequantised* inputs (teacher forcing): the
integer result, dequantised, must agree with it within the tolerance the test states.
"""
import numpy as np
from scipy.special import erf


def gelu(x):
    x = np.asarray(x, dtype=np.float64)
    return x * 0.5 * (1.0 + erf(x / np.sqrt(2.0)))


def hgelu(x):
    """Eq. 6: x ReLU6(1.702 x + 3) / 6."""
    x = np.asarray(x, dtype=np.float64)
    return x * np.clip(1.702 * x + 3.0, 0.0, 6.0) / 6.0


def sigmoid_gelu(x):
    """Eq. 5: x sigma(1.702 x)."""
    x = np.asarray(x, dtype=np.float64)
    return x / (1.0 + np.exp(-1.702 * x))


def softmax(x):
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - x.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def layernorm(x, gamma, beta):
    x = np.asarray(x, dtype=np.float64)
    mu = x.mean(axis=-1, keepdims=True)
    sd = np.sqrt(((x - mu) ** 2).mean(axis=-1, keepdims=True))
    return (x - mu) / sd * gamma + beta


def linear(x, w_int, s_w, bias_int, S_in):
    """x real [T,K]; weights w_int*s_w[n]; bias at scale S_in*s_w[n]."""
    W = w_int.astype(np.float64) * s_w[:, None]
    return x @ W.T + bias_int.astype(np.float64) * (S_in * s_w)
