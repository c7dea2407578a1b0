"""Plain float64 Adam step with decoupled weight decay, and bf16 rounding.

Test infrastructure only (see package docstring).

Follows the paper's mixed-precision definition (Sec. 2.1 "Mixed precision"): the
optimizer converts the half-precision gradient to full precision, descales it, and
updates the full-precision master copy theta with two state variables per parameter
(Sec. 5.2); the half-precision copy theta_16 is then the rounded master copy.  The
update itself is Kingma & Ba's Adam with bias correction, epsilon added to the root of
the corrected second moment, and Loshchilov & Hutter's decoupled decay applied to the
pre-update theta (the paper names Adam/AdamW and its hyper-parameters in Sec. 6.1 and
prints no formula).
"""
import numpy as np


def bf16_round(x):
    """Round float values to the nearest bfloat16 (ties to even); returns float32.

    Works on the float32 bit pattern: bf16 keeps the top 16 bits."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = ((bits + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    out = rounded.astype(np.uint32).view(np.float32)
    return np.where(np.isnan(f), f, out).reshape(np.shape(x))


def adam_step(theta, m, v, g16, lr, beta1, beta2, eps, weight_decay, step, grad_scale):
    """One Adam step on arrays of any shape.

    theta, m, v: fp32 master state (values used exactly, arithmetic in float64).
    g16: the half-precision gradient values.  step: t >= 1.
    Returns (theta', m', v') in float64 and theta16' = bf16(fp32(theta')) as float32."""
    theta = np.asarray(theta, np.float64)
    m = np.asarray(m, np.float64)
    v = np.asarray(v, np.float64)
    g = np.float64(grad_scale) * np.asarray(g16, np.float64)
    m1 = beta1 * m + (1.0 - beta1) * g
    v1 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m1 / (1.0 - np.float64(beta1) ** step)
    vhat = v1 / (1.0 - np.float64(beta2) ** step)
    theta1 = theta - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * theta)
    return theta1, m1, v1, bf16_round(theta1.astype(np.float32))
