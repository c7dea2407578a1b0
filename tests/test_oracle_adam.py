"""Pins for the fp64 Adam oracle and its bf16 rounding."""
import math
import numpy as np
import pytest

from oracle import adam_step, bf16_round


def test_first_step_is_sign_update():
    """t = 1, m = v = 0: bias correction gives mhat = g, vhat = g^2, so
    theta' = theta - lr * g / (|g| + eps)."""
    g = np.array([0.5, -2.0, 1e-3, -1e-6])
    th = np.array([1.0, -1.0, 0.25, 3.0])
    lr, eps = 1e-2, 1e-8
    t1, m1, v1, _ = adam_step(th, 0 * th, 0 * th, g, lr, 0.9, 0.999, eps, 0.0, 1, 1.0)
    assert np.allclose(t1, th - lr * g / (np.abs(g) + eps), rtol=1e-14)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)


def test_zero_gradient_zero_state_leaves_theta():
    th = np.array([0.3, -0.7])
    t1, m1, v1, _ = adam_step(th, 0 * th, 0 * th, 0 * th, 1e-3, 0.9, 0.95, 1e-8, 0.0, 5, 1.0)
    assert np.array_equal(t1, th) and not m1.any() and not v1.any()


def test_hand_computed_scalar_example():
    """theta=1, m=0.1, v=0.04, g16=0.5, grad_scale=2 -> g=1; beta=(0.5,0.5), t=2,
    lr=0.1, eps=0, wd=0.1:
      m' = 0.05+0.5 = 0.55 ; v' = 0.02+0.5 = 0.52
      mhat = 0.55/0.75 ; vhat = 0.52/0.75
      theta' = 1 - 0.1*( mhat/sqrt(vhat) + 0.1*1 )"""
    t1, m1, v1, _ = adam_step(1.0, 0.1, 0.04, 0.5, 0.1, 0.5, 0.5, 0.0, 0.1, 2, 2.0)
    mhat = 0.55 / 0.75
    vhat = 0.52 / 0.75
    assert abs(float(m1) - 0.55) < 1e-15 and abs(float(v1) - 0.52) < 1e-15
    assert abs(float(t1) - (1 - 0.1 * (mhat / math.sqrt(vhat) + 0.1))) < 1e-15


def test_constant_gradient_converges_to_unit_steps():
    """Constant g: mhat -> g and vhat -> g^2 exactly at every step (bias correction),
    so each step moves theta by -lr*sign(g) (eps = 0)."""
    th, m, v = np.array([0.0]), np.array([0.0]), np.array([0.0])
    for t in range(1, 30):
        th, m, v, _ = adam_step(th, m, v, np.array([-0.25]), 1e-2, 0.9, 0.99, 0.0, 0.0, t, 1.0)
        assert abs(th[0] - 1e-2 * t) < 1e-12


def test_against_torch_adamw_fp64_many_steps():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    n = 64
    th0 = rng.standard_normal(n)
    p = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.01)
    th, m, v = th0.copy(), np.zeros(n), np.zeros(n)
    for t in range(1, 8):
        g = rng.standard_normal(n)
        p.grad = torch.tensor(g)
        opt.step()
        th, m, v, _ = adam_step(th, m, v, g, 3e-3, 0.9, 0.95, 1e-8, 0.01, t, 1.0)
        assert np.allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_bf16_round_ties_to_even_and_library():
    torch = pytest.importorskip("torch")
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1 and 1 + 2^-7 -> even (1.0)
    assert bf16_round(np.float32(1 + 2 ** -8)) == np.float32(1.0)
    # 1 + 3*2^-8 is halfway between 1+2^-7 (odd mantissa) and 1+2^-6 (even) -> 1+2^-6
    assert bf16_round(np.float32(1 + 3 * 2 ** -8)) == np.float32(1 + 2 ** -6)
    assert bf16_round(np.float32(1 + 2 ** -8 + 2 ** -20)) == np.float32(1 + 2 ** -7)
    a = (np.random.default_rng(1).standard_normal(50000) * 10).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.bfloat16).float().numpy()
    assert np.array_equal(bf16_round(a), ref)
    th, _, _, th16 = adam_step(a[:100], 0 * a[:100], 0 * a[:100], a[100:200], 1e-3, 0.9, 0.95, 1e-8, 0.0, 1, 1.0)
    assert np.array_equal(th16, torch.from_numpy(th.astype(np.float32)).to(torch.bfloat16).float().numpy())


def test_fp16_round_closed_forms_and_library():
    """IEEE half precision: 10 fraction bits, ties to even, gradual underflow, overflow to infinity."""
    import torch
    from oracle import fp16_round
    assert fp16_round(np.float32(1 + 2 ** -11)) == np.float32(1.0)                 # tie -> even (down)
    assert fp16_round(np.float32(1 + 3 * 2 ** -11)) == np.float32(1 + 2 ** -9)     # tie -> even (up)
    assert fp16_round(np.float32(1 + 2 ** -11 + 2 ** -20)) == np.float32(1 + 2 ** -10)
    assert fp16_round(np.float32(65504.0)) == np.float32(65504.0)                   # largest finite value
    assert fp16_round(np.float32(65519.0)) == np.float32(65504.0)
    assert np.isinf(fp16_round(np.float32(65520.0)))                                # half a step beyond: infinity
    assert fp16_round(np.float32(2.0 ** -24)) == np.float32(2.0 ** -24)            # smallest subnormal
    assert fp16_round(np.float32(2.0 ** -25)) == 0.0                                # tie with zero -> even
    assert fp16_round(np.float32(1.5 * 2.0 ** -24)) == np.float32(2.0 ** -23)      # tie between subnormals -> even
    assert fp16_round(np.float32(-2.9e-8)) == 0.0 and fp16_round(np.float32(-3.0e-8)) == np.float32(-(2.0 ** -24))  # either side of half the smallest
    rng = np.random.default_rng(3)
    a = (rng.standard_normal(20000) * np.exp(rng.uniform(-20, 12, 20000))).astype(np.float32)
    ref = torch.from_numpy(a).to(torch.float16).float().numpy()
    assert np.array_equal(fp16_round(a), ref)


def test_adam_step_theta16_in_either_format():
    th = np.array([1.0 + 2.0 ** -9, 70000.0], np.float32)
    z = np.zeros_like(th)
    _, _, _, t_bf = adam_step(th, z, z, z, 0.0, 0.9, 0.999, 1e-8, 0.0, 1, 1.0)
    _, _, _, t_fp = adam_step(th, z, z, z, 0.0, 0.9, 0.999, 1e-8, 0.0, 1, 1.0, half="fp16")
    assert t_bf[0] == np.float32(1.0) and t_fp[0] == np.float32(1.0 + 2.0 ** -9)   # bf16 tie -> even; exact in fp16
    assert t_bf[1] == np.float32(70144.0) and np.isinf(t_fp[1])


def test_loss_scaler_policy_worked_example():
    """Dynamic loss scale by hand: S = 8, growth 2 after 2 good batches, backoff 1/2.
    good, good (-> 16), overflow (-> 8, skipped, state untouched), good, NaN elsewhere (-> 4), good, good (-> 8)."""
    from oracle import loss_scaled_adam_step, nonfinite_count
    assert nonfinite_count([1.0, np.inf, -np.inf, np.nan, 0.0]) == 3
    sc = dict(scale=8.0, growth=2.0, backoff=0.5, growth_interval=2, good_steps=0)
    th, m, v = np.array([1.0, -2.0]), np.zeros(2), np.zeros(2)
    hyper = (1e-2, 0.9, 0.99, 1e-8, 0.0)
    true_g = np.array([0.25, -0.5])
    scales, skips, step = [], [], 1
    for k, (bad_here, bad_other) in enumerate([(0, 0), (0, 0), (1, 0), (0, 0), (0, 2), (0, 0), (0, 0)]):
        g = true_g * sc["scale"]
        if bad_here:
            g = g.copy(); g[0] = np.inf
        before = (th.copy(), m.copy(), v.copy())
        s_used = sc["scale"]
        sc, th2, m2, v2, t16, skipped = loss_scaled_adam_step(sc, th, m, v, g, *hyper, step, 1.0, other_nonfinite=bad_other)
        if skipped:
            assert t16 is None and all(np.array_equal(a, b) for a, b in zip(before, (th2, m2, v2)))
        else:
            # descaling gives back the true gradient whatever S was: same result as a plain step on true_g
            r = adam_step(th, m, v, true_g, *hyper, step, 1.0)
            assert np.allclose(th2, r[0], rtol=0, atol=1e-15) and np.allclose(v2, r[2], rtol=0, atol=1e-18)
            step += 1
        th, m, v = th2, m2, v2
        scales.append(sc["scale"]); skips.append(skipped); assert s_used > 0
    assert scales == [8.0, 16.0, 8.0, 8.0, 4.0, 4.0, 8.0]
    assert skips == [False, False, True, False, True, False, False]
    assert sc["good_steps"] == 0
