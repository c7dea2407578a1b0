"""Pins for the fp64 transformer oracle: every check here compares the oracle with
something other than itself -- finite differences, closed forms, special cases, a naive
loop, or an independent library autograd."""
import math
import numpy as np
import pytest

import oracle
from oracle import transformer as T
from paper_2110_13005_amd.inputs import StageShape, make_stage_inputs

EPS = 1e-5


def _rand_layers(rng, L, h, f, scale=0.3):
    layers = []
    for _ in range(L):
        layers.append({
            "ln1_g": 1 + 0.2 * rng.standard_normal(h), "ln1_b": 0.2 * rng.standard_normal(h),
            "w_qkv": scale * rng.standard_normal((h, 3 * h)), "b_qkv": 0.1 * rng.standard_normal(3 * h),
            "w_o": scale * rng.standard_normal((h, h)), "b_o": 0.1 * rng.standard_normal(h),
            "ln2_g": 1 + 0.2 * rng.standard_normal(h), "ln2_b": 0.2 * rng.standard_normal(h),
            "w_fc1": scale * rng.standard_normal((h, f)), "b_fc1": 0.1 * rng.standard_normal(f),
            "w_fc2": scale * rng.standard_normal((f, h)), "b_fc2": 0.1 * rng.standard_normal(h),
        })
    return layers


# ------------------------------------------------------------ finite differences
@pytest.mark.parametrize("L,h,a,s,b", [(1, 16, 2, 8, 1), (2, 16, 2, 8, 2), (2, 12, 3, 5, 2)])
def test_all_gradients_match_central_differences(L, h, a, s, b):
    """Scalar loss l = sum(z * dy); every parameter gradient and dx against central
    differences in fp64 (a dropped term, wrong sign or transposed operand fails)."""
    rng = np.random.default_rng(7)
    layers = _rand_layers(rng, L, h, 4 * h)
    x = rng.standard_normal((b, s, h))
    dy = rng.standard_normal((b, s, h))

    def loss():
        z, _ = T.stage_forward(x, layers, a, EPS)
        return float((z * dy).sum())

    z, caches = T.stage_forward(x, layers, a, EPS)
    dx, grads = T.stage_backward(dy, caches, layers, a)
    step = 1e-5
    pick = np.random.default_rng(3)

    def check(arr, ana, n_probe):
        flat = arr.reshape(-1)
        aflat = ana.reshape(-1)
        idx = pick.choice(flat.size, size=min(n_probe, flat.size), replace=False)
        num = np.empty(len(idx))
        for j, i in enumerate(idx):
            old = flat[i]
            flat[i] = old + step
            lp = loss()
            flat[i] = old - step
            lm = loss()
            flat[i] = old
            num[j] = (lp - lm) / (2 * step)
        err = np.linalg.norm(num - aflat[idx]) / max(np.linalg.norm(num), 1e-30)
        assert err < 1e-6, err

    check(x, dx, 40)
    for li in range(L):
        for name in T.PARAM_NAMES:
            check(layers[li][name], grads[li][name], 12)


# --------------------------------------------------------------------- softmax
def test_softmax_rows_mask_and_closed_forms():
    rng = np.random.default_rng(0)
    b, s, a, d = 2, 9, 3, 4
    q, k, v = (rng.standard_normal((b, s, a * d)) for _ in range(3))
    o, P = T.causal_attention_fwd(q, k, v, a)
    assert np.allclose(P.sum(-1), 1.0, atol=1e-14)
    iu = np.triu_indices(s, 1)
    assert (P[..., iu[0], iu[1]] == 0).all()           # masked entries exactly zero
    assert (P[..., 0, 0] == 1).all()                   # row 0 attends to itself only
    # first token's output is its own value vector
    assert np.allclose(o[:, 0, :], v[:, 0, :], atol=1e-14)
    # equal scores (q = 0): row i is uniform 1/(i+1); output = running mean of v
    o0, P0 = T.causal_attention_fwd(np.zeros_like(q), k, v, a)
    for i in range(s):
        assert np.allclose(P0[..., i, :i + 1], 1.0 / (i + 1), atol=1e-15)
    assert np.allclose(o0, np.cumsum(v, axis=1) / np.arange(1, s + 1)[None, :, None], atol=1e-13)


def test_softmax_scale_is_inverse_sqrt_head_dim():
    """Two keys with a known score gap: P = sigmoid(gap / sqrt(d))."""
    d = 16
    q = np.zeros((1, 2, d)); k = np.zeros((1, 2, d)); v = np.zeros((1, 2, d))
    q[0, 1, 0] = 3.0
    k[0, 0, 0] = 2.0          # score(1,0) = 6/sqrt(16) = 1.5 ; score(1,1) = 0
    _, P = T.causal_attention_fwd(q, k, v, 1)
    assert abs(P[0, 0, 1, 0] - 1 / (1 + math.exp(-1.5))) < 1e-15


def test_attention_matches_per_query_loop():
    """Brute force on a tiny input: explicit python loops over heads, queries, keys."""
    rng = np.random.default_rng(5)
    b, s, a, d = 1, 6, 2, 3
    q, k, v = (rng.standard_normal((b, s, a * d)) for _ in range(3))
    o, _ = T.causal_attention_fwd(q, k, v, a)
    ref = np.zeros_like(o)
    for hd in range(a):
        sl = slice(hd * d, (hd + 1) * d)
        for i in range(s):
            sc = [sum(q[0, i, sl][t] * k[0, j, sl][t] for t in range(d)) / math.sqrt(d) for j in range(i + 1)]
            mx = max(sc)
            e = [math.exp(x - mx) for x in sc]
            Z = sum(e)
            for j in range(i + 1):
                ref[0, i, sl] += e[j] / Z * v[0, j, sl]
    assert np.allclose(o, ref, atol=1e-13)


# ------------------------------------------------------------------- LayerNorm
def test_layernorm_moments_and_constant_row():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((4, 7, 32)) * 3 + 2
    out, xhat, rstd = T.layernorm_fwd(x, np.ones(32), np.zeros(32), EPS)
    assert np.allclose(out.mean(-1), 0, atol=1e-13)
    var = x.var(-1)
    assert np.allclose(out.var(-1), var / (var + EPS), rtol=1e-12)
    beta = rng.standard_normal(32)
    outc, _, _ = T.layernorm_fwd(np.full((2, 32), 5.0), 1 + rng.standard_normal(32), beta, EPS)
    assert np.array_equal(outc, np.broadcast_to(beta, (2, 32)))
    # hand example: x = [1, 3], eps = 0 -> xhat = [-1, 1]
    o2, _, _ = T.layernorm_fwd(np.array([[1.0, 3.0]]), np.array([2.0, 3.0]), np.array([0.5, -0.5]), 0.0)
    assert np.allclose(o2, [[-1.5, 2.5]], atol=1e-15)


# ------------------------------------------------------------------------ GeLU
def test_gelu_against_math_erf_and_known_values():
    xs = np.linspace(-6, 6, 241)
    ref = np.array([0.5 * x * (1 + math.erf(x / math.sqrt(2))) for x in xs])
    assert np.allclose(T.gelu(xs), ref, atol=1e-15)
    assert T.gelu(np.array([0.0]))[0] == 0.0
    assert abs(T.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15   # Phi(1)
    assert abs(T.gelu(np.array([10.0]))[0] - 10.0) < 1e-12
    assert abs(T.gelu_grad(np.array([0.0]))[0] - 0.5) < 1e-15
    num = (T.gelu(xs + 1e-6) - T.gelu(xs - 1e-6)) / 2e-6
    assert np.allclose(T.gelu_grad(xs), num, atol=1e-8)


# -------------------------------------------------------------- special cases
def test_seq_len_one_reduces_to_linear_maps():
    """s = 1: attention returns v, so the layer is two LayerNorms and four linear maps."""
    rng = np.random.default_rng(2)
    h, a = 8, 2
    p = _rand_layers(rng, 1, h, 4 * h)[0]
    x = rng.standard_normal((3, 1, h))
    z, _ = T.layer_forward(x, p, a, EPS)

    def ln(t, g, b):
        mu = t.mean(-1, keepdims=True)
        return g * (t - mu) / np.sqrt(t.var(-1, keepdims=True) + EPS) + b
    u = ln(x, p["ln1_g"], p["ln1_b"])
    vv = u @ p["w_qkv"][:, 2 * h:] + p["b_qkv"][2 * h:]
    y = x + vv @ p["w_o"] + p["b_o"]
    pre = ln(y, p["ln2_g"], p["ln2_b"]) @ p["w_fc1"] + p["b_fc1"]
    g = np.array([[0.5 * t * (1 + math.erf(t / math.sqrt(2))) for t in row] for row in pre.reshape(-1, 4 * h)]).reshape(pre.shape)
    assert np.allclose(z, y + g @ p["w_fc2"] + p["b_fc2"], atol=1e-13)


def test_zero_output_projections_give_residual_identity():
    rng = np.random.default_rng(4)
    h, a = 8, 2
    p = _rand_layers(rng, 1, h, 4 * h)[0]
    for n in ("w_o", "b_o", "w_fc2", "b_fc2"):
        p[n] = np.zeros_like(p[n])
    x = rng.standard_normal((2, 5, h)); dy = rng.standard_normal((2, 5, h))
    z, c = T.layer_forward(x, p, a, EPS)
    assert np.array_equal(z, x)
    dx, _ = T.layer_backward(dy, c, p, a)
    assert np.array_equal(dx, dy)


def test_linear_map_against_naive_triple_loop_and_layout():
    """Weights are [in, out]; Q/K/V thirds and head-contiguous columns."""
    rng = np.random.default_rng(6)
    h, a, s = 4, 2, 3
    p = _rand_layers(rng, 1, h, 4 * h)[0]
    x = rng.standard_normal((1, s, h))
    _, c = T.layer_forward(x, p, a, EPS)
    u = c["u"]
    for name, off in (("q", 0), ("k", h), ("v", 2 * h)):
        ref = np.zeros((s, h))
        for i in range(s):
            for o_ in range(h):
                acc = p["b_qkv"][off + o_]
                for k_ in range(h):
                    acc += u[0, i, k_] * p["w_qkv"][k_, off + o_]
                ref[i, o_] = acc
        assert np.allclose(c[name][0], ref, atol=1e-14)


def test_heads_are_independent_column_blocks():
    """Changing K columns of head 1 must not change head 0's output columns."""
    rng = np.random.default_rng(8)
    b, s, a, d = 1, 5, 2, 4
    q, k, v = (rng.standard_normal((b, s, a * d)) for _ in range(3))
    o1, _ = T.causal_attention_fwd(q, k, v, a)
    k2 = k.copy(); k2[:, 2, d:] += 1.0   # one key row (a uniform shift would cancel in softmax)
    o2, _ = T.causal_attention_fwd(q, k2, v, a)
    assert np.array_equal(o1[..., :d], o2[..., :d])
    assert not np.allclose(o1[..., d:], o2[..., d:])


def test_causality_prefix_property():
    """Outputs at tokens < n depend only on inputs at tokens < n."""
    rng = np.random.default_rng(9)
    layers = _rand_layers(rng, 2, 8, 32)
    x = rng.standard_normal((2, 10, 8))
    z, _ = T.stage_forward(x, layers, 2, EPS)
    zp, _ = T.stage_forward(x[:, :4], layers, 2, EPS)
    assert np.allclose(z[:, :4], zp, atol=1e-13)


# ------------------------------------------------------- third opinion: autograd
def test_layer_against_torch_cpu_fp64_autograd():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(10)
    L, h, a, s, b = 2, 24, 3, 7, 2
    layers = _rand_layers(rng, L, h, 4 * h)
    x = rng.standard_normal((b, s, h)); dy = rng.standard_normal((b, s, h))
    tl = [{k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()} for p in layers]
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    cur = tx
    for p in tl:
        u = F.layer_norm(cur, (h,), p["ln1_g"], p["ln1_b"], EPS)
        qkv = F.linear(u, p["w_qkv"].T, p["b_qkv"])
        q, k, v = (t.reshape(b, s, a, h // a).transpose(1, 2) for t in qkv.split(h, dim=-1))
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(1, 2).reshape(b, s, h)
        y = cur + F.linear(o, p["w_o"].T, p["b_o"])
        w = F.layer_norm(y, (h,), p["ln2_g"], p["ln2_b"], EPS)
        cur = y + F.linear(F.gelu(F.linear(w, p["w_fc1"].T, p["b_fc1"])), p["w_fc2"].T, p["b_fc2"])
    (cur * torch.tensor(dy)).sum().backward()
    z, caches = T.stage_forward(x, layers, a, EPS)
    dx, grads = T.stage_backward(dy, caches, layers, a)
    assert np.allclose(z, cur.detach().numpy(), atol=1e-11)
    assert np.allclose(dx, tx.grad.numpy(), atol=1e-10)
    for li in range(L):
        for n in T.PARAM_NAMES:
            assert np.allclose(grads[li][n], tl[li][n].grad.numpy(), atol=1e-10), (li, n)


# ------------------------------------------------------------ grad accumulation
def test_microbatch_sum_equals_concatenated_batch():
    """Batch rows are independent: summing per-microbatch gradients equals the gradient of
    one microbatch holding all rows."""
    rng = np.random.default_rng(11)
    layers = _rand_layers(rng, 2, 8, 32)
    xs = [rng.standard_normal((2, 6, 8)) for _ in range(3)]
    dys = [rng.standard_normal((2, 6, 8)) for _ in range(3)]
    outs, dxs, tot = T.stage_batch(xs, dys, layers, 2, EPS)
    z, c = T.stage_forward(np.concatenate(xs), layers, 2, EPS)
    dx, g = T.stage_backward(np.concatenate(dys), c, layers, 2)
    assert np.allclose(np.concatenate(outs), z, atol=1e-13)
    assert np.allclose(np.concatenate(dxs), dx, atol=1e-12)
    for li in range(2):
        for n in T.PARAM_NAMES:
            assert np.allclose(tot[li][n], g[li][n], atol=1e-11)


def test_tiny_config_runs_and_is_finite():
    sh = StageShape(2, 64, 4, 16, 2, 2)
    layers, xs, dys = make_stage_inputs(sh, seed=0, perturb=True)
    outs, dxs, tot = oracle.stage_batch(xs, dys, layers, sh.n_heads, EPS)
    assert all(np.isfinite(o).all() for o in outs + dxs)
    assert outs[0].shape == (2, 16, 64)
