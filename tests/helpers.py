"""Shared helpers of the GPU parity tests: host <-> device plumbing, the error metric, the bounds of the benchmark
definition, drivers for a batch through a stage, and wrappers of the embedding / head handles."""
import numpy as np

from oracle import lm_ends as OE
from oracle import transformer as OT
from paper_2110_13005_amd import binding as B
from paper_2110_13005_amd.stage import view_bf16

FWD_TOL, GRAD_TOL, ADAM_TOL = 2e-2, 3e-2, 1e-6   # forward, gradients, Adam master state (relative)
EPS = 1e-5                                      # LayerNorm epsilon of every test


def rel_fro(got, ref):
    """||got - ref||_F / ||ref||_F ; if ref is all zero, got must be too."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    n = np.linalg.norm(ref)
    if n == 0:
        return 0.0 if np.linalg.norm(got) == 0 else np.inf
    return float(np.linalg.norm(got - ref) / n)


ELEM_ULP = 2.0 ** -8      # twice the relative rounding error of bfloat16 (half precision rounds finer)
_elem_report = []         # (label, factor) of every element-wise check, printed at the end under AXONN_TEST_REPORT=1


def elem_factor(got, ref, axis=-1):
    """Smallest c with |got - ref| <= c * 2^-8 * (|ref| + s) for every element, where s is the root mean square of
    ref along `axis` (None: of the whole tensor): the error of each element in units of one 16-bit rounding of
    its own magnitude plus that of a typical element of its row (the scale of the sums an element was formed
    from, which is what a rounded intermediate or a cancellation leaves behind)."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    if axis is None or ref.ndim == 0:
        s = np.sqrt(np.mean(ref * ref))
    else:
        s = np.sqrt(np.mean(ref * ref, axis=axis, keepdims=True))
    # plus a floor of 2^-16 of the tensor's typical element, for rows that are exactly zero in the reference (the
    # first query's dq: a single key, no gradient) and come out as a few ulps of fp32 noise
    den = ELEM_ULP * (np.abs(ref) + s) + ELEM_ULP ** 2 * np.sqrt(np.mean(ref * ref))
    err = np.abs(got - ref)
    with np.errstate(divide="ignore", invalid="ignore"):
        f = np.where(den > 0, err / den, np.where(err > 0, np.inf, 0.0))
    return float(f.max())


def parity(got, ref, tol, c, axis=-1, label=""):
    """The two bounds of a parity check: relative Frobenius error below `tol` (the metric of the benchmark
    definition) and every single element within c roundings (elem_factor): one wrong element or one wrong row of a
    ragged tile passes the first and fails the second."""
    e = rel_fro(got, ref)
    f = elem_factor(got, ref, axis)
    _elem_report.append((label, f, c, e))
    assert e < tol, (label, "rel_fro", e, tol)
    assert f <= c, (label, "element-wise factor", f, c)
    return e


def dev_bf16(a):
    """float32 numpy array holding values of the selected 16-bit element type (bfloat16 or half precision) -> cuda
    tensor of that type."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(B.torch_elem_dtype()).cuda()


def round_elem(x):
    """The oracle's rounding to the library's 16-bit element type."""
    import oracle
    return oracle.half_round(x, B.ELEM)


def dev_f32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host(t):
    """cuda tensor (bf16 or fp32) -> float64 numpy."""
    return t.float().cpu().numpy().astype(np.float64)


def run_direct(stage, xs, dys, order=None):
    """All forwards then all backwards (or a given order of (kind, mb)) on the null stream."""
    import torch
    M = len(xs)
    X = [dev_bf16(x) for x in xs]
    DY = [dev_bf16(d) for d in dys]
    Y = [torch.zeros_like(X[0]) for _ in range(M)]
    DX = [torch.zeros_like(X[0]) for _ in range(M)]
    stage.zero_grad()
    if order is None:
        order = [(0, i) for i in range(M)] + [(1, i) for i in range(M)]
    for kind, i in order:
        if kind == 0:
            stage.forward(i, X[i], Y[i])
        else:
            stage.backward(i, DY[i], DX[i])
    torch.cuda.synchronize()
    return [host(y) for y in Y], [host(d) for d in DX], stage.grads_numpy()


def check_batch(outs, dxs, grads, ref, fwd_tol=FWD_TOL, grad_tol=GRAD_TOL, elem_c=24.0):
    r_outs, r_dxs, r_tot = ref
    worst = {"fwd": 0.0, "dx": 0.0, "grad": 0.0}
    worst_f = 0.0
    for o, r in zip(outs, r_outs):
        worst["fwd"] = max(worst["fwd"], rel_fro(o.reshape(r.shape), r))
        worst_f = max(worst_f, elem_factor(o.reshape(r.shape), r))
    for o, r in zip(dxs, r_dxs):
        worst["dx"] = max(worst["dx"], rel_fro(o.reshape(r.shape), r))
        worst_f = max(worst_f, elem_factor(o.reshape(r.shape), r))
    for li, g in enumerate(grads):
        for name, arr in g.items():
            e = rel_fro(arr, r_tot[li][name])
            assert e <= grad_tol, ("layer%d.%s" % (li, name), e)
            worst["grad"] = max(worst["grad"], e)
            worst_f = max(worst_f, elem_factor(arr, r_tot[li][name], axis=None))
    # Element-wise: a stage output has passed through 5 rounded tensors per layer and a softmax; its error is a sum
    # of that many roundings, each of the size of a typical element of its row, and a gradient adds the backward
    # chain's.  elem_c roundings bound every single element (measured worst over the stage tests: 11.3).
    _elem_report.append(("check_batch", worst_f, elem_c, max(worst.values())))
    assert worst_f <= elem_c, ("element-wise factor", worst_f, elem_c)
    assert worst["fwd"] <= fwd_tol, worst
    assert worst["dx"] <= grad_tol, worst
    return worst


def schedules(M, P):
    """Valid message orders for a middle stage (warm-up depth w, then one-forward-one-backward,
    then drain), as lists of (kind, mb)."""
    out = {}
    for w in sorted({1, max(1, P // 2), P}):
        order, f, b = [], 0, 0
        while f < min(w, M):
            order.append((0, f)); f += 1
        while b < M:
            order.append((1, b)); b += 1
            if f < M:
                order.append((0, f)); f += 1
        out["warmup%d" % w] = order
    return out


def dev_i32(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


class EmbedHandle:
    def __init__(self, vocab, h, s, b, wte, wpe):
        import torch
        self.h = B.axonn_embed_create(0, vocab, h, s, b)
        p, g, n = B.axonn_embed_buffers(self.h)
        assert n == (vocab + s) * h
        self.params, self.grads = view_bf16(p, n), view_bf16(g, n)
        self.params[:vocab * h] = dev_bf16(wte).reshape(-1)
        self.params[vocab * h:] = dev_bf16(wpe).reshape(-1)
        self.vocab, self.hid, self.s = vocab, h, s
        torch.cuda.synchronize()

    def grads_numpy(self):
        g = host(self.grads)
        return g[:self.vocab * self.hid].reshape(self.vocab, self.hid), g[self.vocab * self.hid:].reshape(self.s, self.hid)

    def close(self):
        self.params = self.grads = None
        B.axonn_embed_destroy(self.h)


class HeadHandle:
    def __init__(self, vocab, h, T, M, lnf_g, lnf_b, w_head):
        import torch
        self.h = B.axonn_head_create(0, vocab, h, T, M, EPS)
        p, g, n = B.axonn_head_buffers(self.h)
        assert n == 2 * h + h * vocab
        self.params, self.grads = view_bf16(p, n), view_bf16(g, n)
        self.params[:h] = dev_bf16(lnf_g); self.params[h:2 * h] = dev_bf16(lnf_b)
        self.params[2 * h:] = dev_bf16(w_head).reshape(-1)
        self.vocab, self.hid = vocab, h
        torch.cuda.synchronize()

    def grads_numpy(self):
        g = host(self.grads)
        h = self.hid
        return {"lnf_g": g[:h], "lnf_b": g[h:2 * h], "w_head": g[2 * h:].reshape(h, self.vocab)}

    def close(self):
        self.params = self.grads = None
        B.axonn_head_destroy(self.h)


def oracle_model(tokens, targets, wte, wpe, layers, g, bt, W, n_heads, M):
    l64 = [{k: np.asarray(v, np.float64) for k, v in p.items()} for p in layers]
    losses, tot = [], None
    for tk, tg in zip(tokens, targets):
        z, caches = OT.stage_forward(OE.embedding_forward(tk, wte, wpe), l64, n_heads, EPS)
        loss, c = OE.head_loss_forward(z, g, bt, W, tg, EPS, M)
        dz, gh = OE.head_loss_backward(c, g, W, tg, M)
        dx, gl = OT.stage_backward(dz, caches, l64, n_heads)
        dte, dpe = OE.embedding_backward(dx, tk, wte.shape[0], wpe.shape[0])
        cur = dict(layers=gl, head=gh, wte=dte, wpe=dpe)
        losses.append(loss)
        if tot is None:
            tot = cur
        else:
            tot["wte"] += dte; tot["wpe"] += dpe
            for k in gh:
                tot["head"][k] += gh[k]
            for a, b_ in zip(tot["layers"], gl):
                for k in a:
                    a[k] += b_[k]
    return losses, tot


