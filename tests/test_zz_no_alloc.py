"""axonn_layernorm_bwd_noalloc (the entry point for callers that cannot allocate device memory) against
axonn_layernorm_bwd, through the C ABI: two calls in a row on the same device, the second on a smaller
input, so that stale partial sums of the first call would show; then a non-default stream; then the size
limit.  The two entry points run the same kernels, so the results must be bit-identical, and the existing
one is in turn checked against the oracle (here once more, to the bounds of the operation tests)."""
import numpy as np
import pytest

from oracle import transformer as OT
from paper_2110_13005_amd import binding as B
from helpers import dev_bf16, host, rel_fro

pytestmark = pytest.mark.gpu
TOL = 5e-3


def _inputs(T, h, seed):
    import oracle
    rng = np.random.default_rng(seed)

    def draw(shape, std=1.0, shift=0.0):
        return oracle.half_round((rng.standard_normal(shape) * std + shift).astype(np.float32), B.ELEM).astype(np.float32)

    return dict(x=draw((T, h), 2.0, 0.5), g=draw((h,), 0.2, 1.0), b=draw((h,), 0.2), dout=draw((T, h)),
                res=draw((T, h)))


def _run_pair(T, h, seed, with_res, stream=None):
    import torch
    a = _inputs(T, h, seed)
    X, G, Bt, DO, RG = (dev_bf16(a[k]) for k in ("x", "g", "b", "dout", "res"))
    et = B.torch_elem_dtype()
    out = torch.empty(T, h, dtype=et, device="cuda")
    stats = torch.empty(T, 2, dtype=torch.float32, device="cuda")
    B.axonn_layernorm_fwd(T, h, X, G, Bt, 1e-5, out, stats)
    torch.cuda.synchronize()
    res = RG if with_res else None
    ws = torch.empty(2 * ((T + 63) // 64) * h, dtype=torch.float32, device="cuda")
    dx0 = torch.empty(T, h, dtype=et, device="cuda")
    dg0 = torch.empty(h, dtype=torch.float32, device="cuda"); db0 = torch.empty_like(dg0)
    B.axonn_layernorm_bwd(T, h, DO, X, stats, G, res, dx0, dg0, db0, ws)
    dx1 = torch.full((T, h), 7.0, dtype=et, device="cuda")
    dg1 = torch.full((h,), 7.0, dtype=torch.float32, device="cuda"); db1 = torch.full_like(dg1, -7.0)
    torch.cuda.synchronize()
    B.axonn_layernorm_bwd_noalloc(T, h, DO, X, stats, G, res, dx1, dg1, db1, stream)
    torch.cuda.synchronize()
    assert torch.equal(dx0, dx1) and torch.equal(dg0, dg1) and torch.equal(db0, db1), (T, h)
    # and the pair against the oracle
    x64 = a["x"].astype(np.float64)
    _, xhat, rstd = OT.layernorm_fwd(x64, a["g"].astype(np.float64), a["b"].astype(np.float64), 1e-5)
    dxr, dgr, dbr = OT.layernorm_bwd(a["dout"].astype(np.float64), xhat, rstd, a["g"].astype(np.float64))
    if with_res:
        dxr = dxr + a["res"]
    assert rel_fro(host(dx1), dxr) < TOL
    assert rel_fro(host(dg1), dgr) < 1e-4 and rel_fro(host(db1), dbr) < 1e-4


def test_noalloc_two_calls_second_smaller():
    _run_pair(1000, 2056, seed=1, with_res=True)      # ragged: 16 row blocks, 5 column blocks of 512
    _run_pair(72, 520, seed=2, with_res=False)        # smaller: 2 row blocks; the scratch still holds call 1
    _run_pair(2048, 5120, seed=3, with_res=True)      # the 12B stage's shape


def test_noalloc_on_a_side_stream():
    import torch
    s = torch.cuda.Stream()
    _run_pair(256, 1024, seed=4, with_res=True, stream=s)


def test_noalloc_rejects_sizes_beyond_the_buffer():
    import torch
    T, h = 64 * 65, 16384                             # 2 * 65 * 16384 floats > 2 * 64 * 16384
    t = torch.empty(8, dtype=torch.float32, device="cuda")
    with pytest.raises(B.AxonnError) as e:
        B.axonn_layernorm_bwd_noalloc(T, h, t, t, t, t, None, t, t, t)
    assert e.value.status == B.AXONN_EUNSUPPORTED and "scratch" in str(e.value)
    with pytest.raises(B.AxonnError):
        B.axonn_layernorm_bwd_noalloc(8, 16392, t, t, t, t, None, t, t, t)
