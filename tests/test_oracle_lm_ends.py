"""Pins for the oracle's first-stage and last-stage parts (embedding; final LayerNorm, LM head,
cross-entropy with the loss pre-divided by the number of microbatches, Sec. 4.2)."""
import math
import numpy as np
import pytest

from oracle import lm_ends as E
from oracle import transformer as T

EPS = 1e-5


def _head(rng, h, V):
    return 1 + 0.2 * rng.standard_normal(h), 0.2 * rng.standard_normal(h), 0.5 * rng.standard_normal((h, V))


def test_loss_closed_forms():
    rng = np.random.default_rng(0)
    b, s, h, V, M = 2, 5, 8, 11, 4
    x = rng.standard_normal((b, s, h))
    tg = rng.integers(0, V, (b, s))
    g, bt, W = _head(rng, h, V)
    # a zero head gives equal logits: every token costs log V
    loss, c = E.head_loss_forward(x, g, bt, 0 * W, tg, EPS, M)
    assert math.isclose(loss, math.log(V) / M, rel_tol=1e-14)
    # a head that puts a huge logit on every target makes the loss vanish (4 tokens, h = 8: an exact fit exists)
    xs, tgs = x[:1, :4], tg[:1, :4]
    a = T.layernorm_fwd(xs, g, bt, EPS)[0]
    big = np.zeros((1, 4, V)); np.put_along_axis(big, tgs[..., None], 50.0, axis=-1)
    Wfit = np.linalg.lstsq(a.reshape(-1, h), big.reshape(-1, V), rcond=None)[0]
    assert np.allclose(a.reshape(-1, h) @ Wfit, big.reshape(-1, V), atol=1e-8)
    assert E.head_loss_forward(xs, g, bt, Wfit, tgs, EPS, 1)[0] < 1e-15
    # one token, hand-worked: logits (0, log 2, log 3) -> p = (1/6, 2/6, 3/6); target 1 -> loss = log 3
    logits = np.array([0.0, math.log(2), math.log(3)])
    x1 = np.array([[[1.0, -1.0]]])                  # LayerNorm(gain 1, shift 0) -> (1, -1) up to eps
    a1 = T.layernorm_fwd(x1, np.ones(2), np.zeros(2), 1e-12)[0][0, 0]
    W1 = np.linalg.lstsq(np.array([a1, [1.0, 1.0]]), np.array([logits, [0, 0, 0]]), rcond=None)[0]
    loss1, c1 = E.head_loss_forward(x1, np.ones(2), np.zeros(2), W1, np.array([[1]]), 1e-12, 1)
    assert math.isclose(loss1, math.log(3), rel_tol=1e-9)
    dx1, gr1 = E.head_loss_backward(c1, np.ones(2), W1, np.array([[1]]), 1)
    # dL/dlogits = p - onehot = (1/6, -4/6, 3/6); dW = a^T dlogits
    assert np.allclose(gr1["w_head"], np.outer(a1, [1 / 6, -4 / 6, 3 / 6]), atol=1e-9)


def test_pre_division_makes_microbatch_losses_sum_to_the_batch_mean():
    """Sec. 4.2: with every microbatch's loss divided by M, the sum over microbatches is the mean token loss of
    the whole batch, and the summed gradients are its gradients."""
    rng = np.random.default_rng(1)
    b, s, h, V, M = 2, 4, 8, 13, 3
    g, bt, W = _head(rng, h, V)
    xs = [rng.standard_normal((b, s, h)) for _ in range(M)]
    tgs = [rng.integers(0, V, (b, s)) for _ in range(M)]
    tot, dW = 0.0, 0.0
    dxs = []
    for x, tg in zip(xs, tgs):
        loss, c = E.head_loss_forward(x, g, bt, W, tg, EPS, M)
        dx, gr = E.head_loss_backward(c, g, W, tg, M)
        tot += loss; dW = dW + gr["w_head"]; dxs.append(dx)
    lossb, cb = E.head_loss_forward(np.concatenate(xs), g, bt, W, np.concatenate(tgs), EPS, 1)
    dxb, grb = E.head_loss_backward(cb, g, W, np.concatenate(tgs), 1)
    assert math.isclose(tot, lossb, rel_tol=1e-13)
    assert np.allclose(dW, grb["w_head"], atol=1e-14)
    assert np.allclose(np.concatenate(dxs), dxb, atol=1e-14)


def test_head_gradients_against_central_differences_and_invariants():
    rng = np.random.default_rng(2)
    b, s, h, V, M = 2, 3, 6, 9, 2
    x = rng.standard_normal((b, s, h))
    tg = rng.integers(0, V, (b, s))
    g, bt, W = _head(rng, h, V)
    loss, c = E.head_loss_forward(x, g, bt, W, tg, EPS, M)
    dx, gr = E.head_loss_backward(c, g, W, tg, M)
    e = 1e-6
    for arr, grad in ((x, dx), (g, gr["lnf_g"]), (bt, gr["lnf_b"]), (W, gr["w_head"])):
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + e; up = E.head_loss_forward(x, g, bt, W, tg, EPS, M)[0]
            arr[i] = old - e; dn = E.head_loss_forward(x, g, bt, W, tg, EPS, M)[0]
            arr[i] = old
            assert math.isclose((up - dn) / (2 * e), grad[i], rel_tol=2e-6, abs_tol=2e-9), i
    # each token's logit gradient sums to zero over the vocabulary, so dW's columns sum to zero along V
    assert np.allclose(gr["w_head"].sum(axis=1), 0, atol=1e-15)
    # LayerNorm removes the mean and the scale of x: dx is orthogonal to the all-ones vector and to x - mean
    assert np.allclose(dx.sum(axis=-1), 0, atol=1e-14)
    xc = x - x.mean(-1, keepdims=True)           # (exactly so only for eps = 0: the residue is of order eps / var)
    assert np.all(np.abs((dx * xc).sum(-1)) <= 1e-4 * np.linalg.norm(dx, axis=-1) * np.linalg.norm(xc, axis=-1))


def test_loss_against_torch_cross_entropy():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(3)
    b, s, h, V, M = 2, 6, 8, 17, 4
    x = rng.standard_normal((b, s, h)); tg = rng.integers(0, V, (b, s))
    g, bt, W = _head(rng, h, V)
    loss, c = E.head_loss_forward(x, g, bt, W, tg, EPS, M)
    dx, gr = E.head_loss_backward(c, g, W, tg, M)
    tx = torch.tensor(x, requires_grad=True); tW = torch.tensor(W, requires_grad=True)
    tgam = torch.tensor(g, requires_grad=True); tbet = torch.tensor(bt, requires_grad=True)
    a = torch.nn.functional.layer_norm(tx, (h,), tgam, tbet, EPS)
    tl = torch.nn.functional.cross_entropy((a @ tW).reshape(-1, V), torch.tensor(tg).reshape(-1)) / M
    tl.backward()
    assert math.isclose(loss, tl.item(), rel_tol=1e-12)
    assert np.allclose(dx, tx.grad.numpy(), atol=1e-13)
    assert np.allclose(gr["w_head"], tW.grad.numpy(), atol=1e-13)
    assert np.allclose(gr["lnf_g"], tgam.grad.numpy(), atol=1e-13)
    assert np.allclose(gr["lnf_b"], tbet.grad.numpy(), atol=1e-13)


def test_embedding_forward_and_backward():
    rng = np.random.default_rng(4)
    V, h, s_max = 7, 4, 6
    wte, wpe = rng.standard_normal((V, h)), rng.standard_normal((s_max, h))
    tokens = np.array([[3, 3, 0, 6, 3], [1, 0, 0, 2, 6]])
    x = E.embedding_forward(tokens, wte, wpe)
    assert x.shape == (2, 5, h)
    assert np.array_equal(x[0, 1], wte[3] + wpe[1]) and np.array_equal(x[1, 4], wte[6] + wpe[4])
    # with every dx row equal to r, a table row receives (number of uses) * r; unused rows get nothing
    r = rng.standard_normal(h)
    dwte, dwpe = E.embedding_backward(np.broadcast_to(r, (2, 5, h)), tokens, V, s_max)
    uses = np.bincount(tokens.ravel(), minlength=V)
    assert np.allclose(dwte, uses[:, None] * r) and not dwte[4].any() and not dwte[5].any()
    assert np.allclose(dwpe[:5], 2 * r) and not dwpe[5].any()
    # general dx: the pair is the adjoint of the forward map: <dx, E(wte, wpe)> = <dwte, wte> + <dwpe, wpe>
    dx = rng.standard_normal((2, 5, h))
    dwte, dwpe = E.embedding_backward(dx, tokens, V, s_max)
    assert math.isclose((dx * x).sum(), (dwte * wte).sum() + (dwpe * wpe).sum(), rel_tol=1e-12)


def test_whole_model_through_both_ends_against_central_differences():
    """Embedding -> two transformer layers -> head and loss: the gradient that reaches the tables through the
    whole chain."""
    rng = np.random.default_rng(5)
    V, h, a, s, b, M = 11, 8, 2, 4, 2, 2
    wte, wpe = 0.5 * rng.standard_normal((V, h)), 0.5 * rng.standard_normal((s, h))
    g, bt, W = _head(rng, h, V)

    def n(*sh):
        return rng.standard_normal(sh)
    layers = [{"ln1_g": 1 + 0.2 * n(h), "ln1_b": 0.2 * n(h), "w_qkv": 0.3 * n(h, 3 * h), "b_qkv": 0.1 * n(3 * h),
               "w_o": 0.3 * n(h, h), "b_o": 0.1 * n(h), "ln2_g": 1 + 0.2 * n(h), "ln2_b": 0.2 * n(h),
               "w_fc1": 0.3 * n(h, 4 * h), "b_fc1": 0.1 * n(4 * h), "w_fc2": 0.3 * n(4 * h, h), "b_fc2": 0.1 * n(h)}
              for _ in range(2)]
    tokens, tg = rng.integers(0, V, (b, s)), rng.integers(0, V, (b, s))

    def loss():
        z = T.stage_forward(E.embedding_forward(tokens, wte, wpe), layers, a, EPS)[0]
        return E.head_loss_forward(z, g, bt, W, tg, EPS, M)[0]

    z, caches = T.stage_forward(E.embedding_forward(tokens, wte, wpe), layers, a, EPS)
    _, c = E.head_loss_forward(z, g, bt, W, tg, EPS, M)
    dz, _ = E.head_loss_backward(c, g, W, tg, M)
    dx, _ = T.stage_backward(dz, caches, layers, a)
    dwte, dwpe = E.embedding_backward(dx, tokens, V, s)
    e = 1e-6
    for arr, grad in ((wte, dwte), (wpe, dwpe)):
        for i in [(int(tokens[0, 0]), 1), (int(tokens[1, 2]), 5), (2, 3)] if arr is wte else [(0, 0), (3, 7)]:
            old = arr[i]
            arr[i] = old + e; up = loss()
            arr[i] = old - e; dn = loss()
            arr[i] = old
            assert math.isclose((up - dn) / (2 * e), grad[i], rel_tol=5e-6, abs_tol=1e-9), i
