"""Plain float64 definition of what the first and the last pipeline stage add to a stage of
transformer layers: token + position embedding in front, final LayerNorm, LM head and
cross-entropy loss behind.

Test infrastructure only (see package docstring).

Alg. 2 treats the two ends specially: the first stage turns a microbatch of the input batch
into activations (its Forward consumes token ids), the last stage computes the loss and
starts the backward pass at once ("Backward(1)": the loss is the scalar whose gradient is 1).
Sec. 4.2 pre-divides the loss by the number of microbatches of the batch, so that the
gradients accumulated over microbatches are those of the batch-mean loss.  Sec. 6.1 fixes the
vocabulary at 51200 and Eq. 3 counts the LM head as 6*b*s*h*V FLOPs (the V/16lh term).

The paper prints no equations for these parts; the reading taken here is the GPT one its
models follow: learned token and position tables added together, a LayerNorm in front of the
head, a head matrix [h, V] of its own (on a pipeline the table and the head sit on different
GPUs; tying them needs a collective and is not modelled), token-mean cross-entropy.
"""
import numpy as np

from .transformer import layernorm_fwd, layernorm_bwd

_F = np.float64


# ------------------------------------------------------------------ first stage
def embedding_forward(tokens, wte, wpe):
    """tokens: int [b,s]; wte: [V,h]; wpe: [s_max,h].  x[b,i,:] = wte[tokens[b,i]] + wpe[i]."""
    tokens = np.asarray(tokens)
    s = tokens.shape[1]
    return np.asarray(wte, _F)[tokens] + np.asarray(wpe, _F)[None, :s, :]


def embedding_backward(dx, tokens, vocab, s_max):
    """Returns (dwte [V,h], dwpe [s_max,h]): every use of a table row adds its dx row."""
    dx = np.asarray(dx, _F)
    tokens = np.asarray(tokens)
    b, s, h = dx.shape
    dwte = np.zeros((vocab, h), _F)
    for bi in range(b):
        for i in range(s):
            dwte[tokens[bi, i]] += dx[bi, i]
    dwpe = np.zeros((s_max, h), _F)
    dwpe[:s] = dx.sum(axis=0)
    return dwte, dwpe


# ------------------------------------------------------------------- last stage
def head_loss_forward(x, lnf_g, lnf_b, w_head, targets, eps, n_microbatches):
    """x: [b,s,h] output of the last transformer layer; targets: int [b,s].

    a = LN(x); logits = a W_head; per token loss = log sum_v exp(logit_v) - logit_target;
    loss = mean over the microbatch's tokens / n_microbatches.  Returns (loss, cache)."""
    x = np.asarray(x, _F)
    a, xhat, rstd = layernorm_fwd(x, np.asarray(lnf_g, _F), np.asarray(lnf_b, _F), eps)
    logits = a @ np.asarray(w_head, _F)
    m = logits.max(axis=-1, keepdims=True)
    lse = m[..., 0] + np.log(np.exp(logits - m).sum(axis=-1))
    tgt = np.take_along_axis(logits, np.asarray(targets)[..., None], axis=-1)[..., 0]
    token_loss = lse - tgt
    loss = token_loss.mean() / n_microbatches
    cache = dict(a=a, xhat=xhat, rstd=rstd, logits=logits, lse=lse, token_loss=token_loss)
    return loss, cache


def head_loss_backward(cache, lnf_g, w_head, targets, n_microbatches):
    """Backward(1): gradient of the loss above.  Returns (dx, dict of lnf_g, lnf_b, w_head gradients)."""
    c = cache
    logits = c["logits"]
    b, s, V = logits.shape
    p = np.exp(logits - c["lse"][..., None])
    onehot = np.zeros_like(p)
    np.put_along_axis(onehot, np.asarray(targets)[..., None], 1.0, axis=-1)
    dlogits = (p - onehot) / (b * s * n_microbatches)
    a2 = c["a"].reshape(-1, c["a"].shape[-1])
    gr = {"w_head": a2.T @ dlogits.reshape(-1, V)}
    da = dlogits @ np.asarray(w_head, _F).T
    dx, gr["lnf_g"], gr["lnf_b"] = layernorm_bwd(da, c["xhat"], c["rstd"], np.asarray(lnf_g, _F))
    return dx, gr
