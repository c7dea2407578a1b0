"""Plain float64 Adam step with decoupled weight decay, rounding to the two 16-bit formats, and the
dynamic loss scaler.

Test infrastructure only (see package docstring).

Follows the paper's mixed-precision definition (Sec. 2.1 "Mixed precision"): the
optimizer converts the half-precision gradient to full precision, descales it, and
updates the full-precision master copy theta with two state variables per parameter
(Sec. 5.2); the half-precision copy theta_16 is then the rounded master copy.  The
update itself is Kingma & Ba's Adam with bias correction, epsilon added to the root of
the corrected second moment, and Loshchilov & Hutter's decoupled decay applied to the
pre-update theta (the paper names Adam/AdamW and its hyper-parameters in Sec. 6.1 and
prints no formula).

Loss scale (same section): the loss is multiplied by a scaling factor S so that small half-precision
gradients do not underflow; the optimizer descales.  The paper does not say how S is chosen.  Reading
taken here, the usual dynamic scheme (Micikevicius et al. 2018, Sec. 3.2): if any gradient value of a batch
is infinite or NaN, the batch is dropped (no state changes) and S is multiplied by `backoff`; after
`growth_interval` batches in a row without such a value S is multiplied by `growth`.
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


def fp16_round(x):
    """Round float values to the nearest IEEE half precision value (ties to even, overflow to infinity beyond
    65504 + half a step, gradual underflow below 2^-14); returns float32.  numpy's own conversion."""
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float32).astype(np.float16).astype(np.float32)


def half_round(x, half="bf16"):
    return fp16_round(x) if half == "fp16" else bf16_round(x)


def adam_step(theta, m, v, g16, lr, beta1, beta2, eps, weight_decay, step, grad_scale, half="bf16"):
    """One Adam step on arrays of any shape.

    theta, m, v: fp32 master state (values used exactly, arithmetic in float64).
    g16: the half-precision gradient values.  step: t >= 1.  half: the 16-bit format, "bf16" or "fp16".
    Returns (theta', m', v') in float64 and theta16' = half(fp32(theta')) as float32."""
    theta = np.asarray(theta, np.float64)
    m = np.asarray(m, np.float64)
    v = np.asarray(v, np.float64)
    g = np.float64(grad_scale) * np.asarray(g16, np.float64)
    m1 = beta1 * m + (1.0 - beta1) * g
    v1 = beta2 * v + (1.0 - beta2) * g * g
    mhat = m1 / (1.0 - np.float64(beta1) ** step)
    vhat = v1 / (1.0 - np.float64(beta2) ** step)
    theta1 = theta - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * theta)
    return theta1, m1, v1, half_round(theta1.astype(np.float32), half)


def nonfinite_count(g):
    """Number of infinite or NaN values in g."""
    return int(np.count_nonzero(~np.isfinite(np.asarray(g, np.float64))))


def loss_scaled_adam_step(scaler, theta, m, v, g16, lr, beta1, beta2, eps, weight_decay, step, grad_scale,
                          other_nonfinite=0, half="bf16"):
    """One optimizer step under the dynamic loss scale.

    scaler: dict with scale, growth, backoff, growth_interval, good_steps; g16: the gradients of a loss that was
    multiplied by scaler["scale"].  Returns (scaler', theta', m', v', theta16' or None, skipped)."""
    sc = dict(scaler)
    if nonfinite_count(g16) + int(other_nonfinite) != 0:
        sc["scale"] = sc["scale"] * sc["backoff"]
        sc["good_steps"] = 0
        return sc, np.asarray(theta, np.float64), np.asarray(m, np.float64), np.asarray(v, np.float64), None, True
    t1, m1, v1, t16 = adam_step(theta, m, v, g16, lr, beta1, beta2, eps, weight_decay, step,
                                grad_scale / sc["scale"], half)
    sc["good_steps"] += 1
    if sc["good_steps"] >= sc["growth_interval"]:
        sc["scale"] = sc["scale"] * sc["growth"]
        sc["good_steps"] = 0
    return sc, t1, m1, v1, t16, False
