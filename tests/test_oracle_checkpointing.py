"""Pins for the oracle's activation checkpointing (Sec. 5.1): regeneration must not change
any result, only what is kept; Eq. 1 and the stride rule are checked against closed forms
and hand-worked cases."""
import math
import numpy as np
import pytest

from oracle import transformer as T

EPS = 1e-5


def _rand_layers(rng, L, h, f, scale=0.3):
    def n(*s):
        return rng.standard_normal(s)
    return [{"ln1_g": 1 + 0.2 * n(h), "ln1_b": 0.2 * n(h), "w_qkv": scale * n(h, 3 * h), "b_qkv": 0.1 * n(3 * h),
             "w_o": scale * n(h, h), "b_o": 0.1 * n(h), "ln2_g": 1 + 0.2 * n(h), "ln2_b": 0.2 * n(h),
             "w_fc1": scale * n(h, f), "b_fc1": 0.1 * n(f), "w_fc2": scale * n(f, h), "b_fc2": 0.1 * n(h)}
            for _ in range(L)]


@pytest.mark.parametrize("ac", [1, 2, 3, 6])
def test_checkpointed_pass_equals_the_plain_pass(ac):
    """The plain backward pass is pinned to finite differences and to an independent autograd
    elsewhere; regenerating activations from kept tensors must reproduce it exactly."""
    rng = np.random.default_rng(5)
    L, h, a = 6, 8, 2
    layers = _rand_layers(rng, L, h, 4 * h)
    x, dy = rng.standard_normal((2, 5, h)), rng.standard_normal((2, 5, h))
    z, caches = T.stage_forward(x, layers, a, EPS)
    dx, grads = T.stage_backward(dy, caches, layers, a)
    live = []
    zc, kept = T.stage_forward_checkpointed(x, layers, a, EPS, ac)
    dxc, gradsc = T.stage_backward_checkpointed(dy, kept, layers, a, EPS, ac, live_log=live)
    assert np.array_equal(z, zc)
    assert np.allclose(dx, dxc, rtol=0, atol=1e-13)
    for l in range(L):
        for name in T.PARAM_NAMES:
            assert np.allclose(grads[l][name], gradsc[l][name], rtol=0, atol=1e-12), (l, name)
    # what is kept: L/ac tensors, the inputs of layers 0, ac, 2ac, ...; never more than ac layers regenerated
    assert len(kept) == L // ac
    inputs = [x]
    for p in layers[:-1]:
        inputs.append(T.layer_forward(inputs[-1], p, a, EPS)[0])
    for j, t in enumerate(kept):
        assert np.array_equal(t, inputs[j * ac])
    assert live == [ac] * (L // ac)


def test_checkpointed_gradient_against_central_differences():
    """Direct check of the regenerating pass: d<dy, stage(x)>/dtheta for a few entries of a first-layer and a
    last-layer weight, and for the input."""
    rng = np.random.default_rng(6)
    L, h, a, ac = 4, 8, 2, 2
    layers = _rand_layers(rng, L, h, 4 * h)
    x, dy = rng.standard_normal((1, 6, h)), rng.standard_normal((1, 6, h))
    _, kept = T.stage_forward_checkpointed(x, layers, a, EPS, ac)
    dx, grads = T.stage_backward_checkpointed(dy, kept, layers, a, EPS, ac)

    def loss():
        return float((T.stage_forward(x, layers, a, EPS)[0] * dy).sum())

    e = 1e-6
    for l, name, idx in [(0, "w_qkv", (3, 17)), (0, "ln1_g", (2,)), (1, "w_fc1", (5, 9)), (3, "w_fc2", (20, 1)),
                         (2, "b_o", (4,))]:
        t = layers[l][name]
        old = t[idx]
        t[idx] = old + e; up = loss()
        t[idx] = old - e; dn = loss()
        t[idx] = old
        assert math.isclose((up - dn) / (2 * e), grads[l][name][idx], rel_tol=2e-6, abs_tol=1e-8), (l, name)
    old = x[0, 2, 3]
    x[0, 2, 3] = old + e; up = loss()
    x[0, 2, 3] = old - e; dn = loss()
    x[0, 2, 3] = old
    assert math.isclose((up - dn) / (2 * e), dx[0, 2, 3], rel_tol=2e-6, abs_tol=1e-8)


def test_stride_must_divide_the_layer_count():
    rng = np.random.default_rng(7)
    layers = _rand_layers(rng, 4, 8, 32)
    with pytest.raises(ValueError):
        T.stage_forward_checkpointed(rng.standard_normal((1, 4, 8)), layers, 2, EPS, 3)


def test_activation_memory_formula_and_its_minimum():
    """Eq. 1 = N/ac + 1 + ac whatever G_inter; by calculus its minimum over real ac is at sqrt(N), value
    2 sqrt(N) + 1."""
    for N, G in [(16, 1), (36, 2), (64, 4), (144, 12)]:
        r = math.isqrt(N)
        assert T.activation_memory(N, G, r) == 2 * r + 1
        for ac in range(1, N + 1):
            assert math.isclose(T.activation_memory(N, G, ac), N / ac + 1 + ac)
            assert T.activation_memory(N, G, ac) >= 2 * r + 1
    # hand-worked: N = 48 layers on 6 GPUs, ac = 4: 6 * (48 / 24) + 1 + 4 = 17
    assert T.activation_memory(48, 6, 4) == 17


def test_stride_rule_hand_worked_cases():
    """Factor of the per-GPU layer count closest to sqrt(N) (Sec. 5.1)."""
    # N = 48, 6 GPUs: 8 layers per GPU, factors 1 2 4 8, sqrt(48) = 6.93 -> 8
    assert T.checkpoint_stride(48, 6) == 8
    # N = 48, 12 GPUs: 4 per GPU, factors 1 2 4 -> 4
    assert T.checkpoint_stride(48, 12) == 4
    # N = 36 on one GPU: sqrt = 6 is a factor
    assert T.checkpoint_stride(36, 1) == 6
    # N = 96, 4 GPUs: 24 per GPU, factors 1 2 3 4 6 8 12 24, sqrt(96) = 9.80 -> 8 (1.80 away; 12 is 2.20 away)
    assert T.checkpoint_stride(96, 4) == 8
    # N = 24 on one GPU: sqrt = 4.90; 4 (0.90 away) beats 6 (1.10 away)
    assert T.checkpoint_stride(24, 1) == 4
    for N, G in [(48, 6), (96, 4), (24, 1), (60, 5)]:
        ac = T.checkpoint_stride(N, G)
        assert (N // G) % ac == 0
