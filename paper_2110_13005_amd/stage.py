"""Convenience wrapper around the stage handle: owns the torch views of the library's flat
parameter / gradient buffers and moves named tensors in and out.  Plumbing only -- every
computation is a call into libaxonn_stage.so."""
import ctypes

import numpy as np

from . import binding as B


def _view(ptr, n, dtype):
    """torch tensor aliasing `n` elements of device memory at `ptr` (no copy, no ownership)."""
    import torch
    itemsize = torch.empty((), dtype=dtype).element_size()

    class _Holder:
        __cuda_array_interface__ = {
            "shape": (n * itemsize,), "typestr": "|u1", "data": (ptr, False), "version": 3}
    return torch.as_tensor(_Holder(), device="cuda").view(dtype)


def view_bf16(ptr, n):
    """torch view (the library's 16-bit element type) of `n` elements of library-owned device memory at `ptr`."""
    return _view(ptr, n, B.torch_elem_dtype())


class Stage:
    def __init__(self, shape, pipeline_limit=None, ln_eps=1e-5, device=0, grad_accum_fp32=1,
                 n_microbatches=None, wgrad_group=0, qkv_input_split=0, ckpt_stride=0):
        import torch
        self.shape = shape
        self.cfg = B.make_config(shape, pipeline_limit, ln_eps, device, grad_accum_fp32, n_microbatches, wgrad_group,
                                 qkv_input_split, ckpt_stride)
        self.handle = B.axonn_stage_create(self.cfg)
        self.n_params = B.axonn_stage_param_count(self.handle)
        self.layout = {}
        for i in range(B.axonn_stage_num_tensors(self.handle)):
            name, off, dims = B.axonn_stage_param_layout(self.handle, i)
            self.layout[name] = (off, dims)
        self.params = _view(B.axonn_stage_params(self.handle), self.n_params, B.torch_elem_dtype())
        self.grads = _view(B.axonn_stage_grads(self.handle), self.n_params, B.torch_elem_dtype())

    def close(self):
        if self.handle:
            self.params = self.grads = None
            B.axonn_stage_destroy(self.handle)
            self.handle = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def tensor(self, name, grad=False):
        off, dims = self.layout[name]
        n = int(np.prod(dims))
        return (self.grads if grad else self.params)[off:off + n].view(*dims)

    def load_params(self, layers):
        """layers: list of dicts name -> float32 numpy array of values representable in the element type."""
        import torch
        for li, p in enumerate(layers):
            for name, arr in p.items():
                t = torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).to(B.torch_elem_dtype())
                self.tensor("layer%d.%s" % (li, name)).copy_(t)
        torch.cuda.synchronize()

    def grads_numpy(self):
        """list of dicts name -> float64 numpy array."""
        out = [dict() for _ in range(self.shape.n_layers)]
        for name in self.layout:
            l, short = name.split(".")
            out[int(l[5:])][short] = self.tensor(name, grad=True).float().cpu().numpy().astype(np.float64)
        return out

    # thin pass-throughs
    def zero_grad(self, stream=None):
        B.axonn_stage_zero_grad(self.handle, stream)

    def forward(self, mb_id, x, y, stream=None):
        B.axonn_stage_forward(self.handle, mb_id, x, y, stream)

    def backward(self, mb_id, dy, dx, stream=None):
        B.axonn_stage_backward(self.handle, mb_id, dy, dx, stream)

    def post(self, kind, mb_id, payload, result, ready_event=None, targets=None, loss=None, done_event=None):
        B.axonn_stage_post(self.handle, kind, mb_id, payload, result, ready_event, targets, loss, done_event)

    def poll(self, n_streams=2, stream=None):
        return B.axonn_stage_poll(self.handle, n_streams, stream)

    def run(self, n_streams=2, stream=None):
        B.axonn_stage_run(self.handle, n_streams, stream)

    def join(self, stream=None):
        B.axonn_stage_join(self.handle, stream)

    def synchronize(self):
        B.axonn_stage_synchronize(self.handle)
