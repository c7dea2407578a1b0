"""ctypes binding of libaxonn_stage.so: argument marshalling only.

Every function has the name and argument order of its C declaration in
include/axonn_stage.h.  Device buffers may be passed as torch tensors (their
`data_ptr()` is taken) or as integer addresses; streams as `torch.cuda.Stream`,
integer handles or None.  A negative status raises AxonnError with the library's
message.  There is no fallback: if the shared library has not been built, loading
fails with an error that says how to build it.
"""
import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
# The library exists in two builds of the same sources: bfloat16 (default) or IEEE half precision as the
# 16-bit element type, each a shared library of its own with the same C ABI.  AXONN_ELEM chooses the one a
# process starts with; select_elem() switches at run time (both can be loaded, and a stage, embedding, head or
# optimizer handle keeps going to the library that created it).
_LIB_FILES = {"bf16": "libaxonn_stage.so", "fp16": "libaxonn_stage_fp16.so"}
ELEM = os.environ.get("AXONN_ELEM", "bf16")
if ELEM not in _LIB_FILES:
    raise ValueError("AXONN_ELEM must be bf16 or fp16, not %r" % ELEM)
_IMPORT_ELEM = ELEM
LIB_PATH = os.path.join(_HERE, _LIB_FILES[ELEM])     # of the element type at import; may be pointed elsewhere before load()


def select_elem(elem):
    """Makes `elem` ("bf16" or "fp16") the element type of everything created from now on: the library that
    handle-free calls go to, torch_elem_dtype(), and the rounding of the synthetic inputs."""
    global ELEM
    if elem not in _LIB_FILES:
        raise ValueError("element type must be bf16 or fp16, not %r" % elem)
    ELEM = elem
    from . import inputs
    inputs.ELEM = elem


def torch_elem_dtype():
    """torch dtype of the selected 16-bit element type."""
    import torch
    return torch.bfloat16 if ELEM == "bf16" else torch.float16

AXONN_OK, AXONN_EINVAL, AXONN_ESTATE, AXONN_ENOMEM, AXONN_EHIP, AXONN_EUNSUPPORTED = 0, -1, -2, -3, -4, -5
EPI_BIAS, EPI_BIAS_RES, EPI_BIAS_GELU, EPI_DGELU, EPI_ACC_F32, EPI_ACC_BF16 = range(6)


class AxonnError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("axonn status %d: %s" % (status, message))
        self.status = status


class axonn_stage_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_heads", C.c_int32),
                ("ffn_hidden", C.c_int32), ("seq_len", C.c_int32), ("microbatch_size", C.c_int32),
                ("n_microbatches", C.c_int32), ("pipeline_limit", C.c_int32), ("ln_eps", C.c_float),
                ("device", C.c_int32), ("grad_accum_fp32", C.c_int32), ("wgrad_group", C.c_int32),
                ("qkv_input_split", C.c_int32), ("ckpt_stride", C.c_int32)]


class axonn_loss_scaler(C.Structure):
    _fields_ = [("scale", C.c_float), ("growth", C.c_float), ("backoff", C.c_float),
                ("growth_interval", C.c_int32), ("good_steps", C.c_int32)]


class axonn_msg(C.Structure):
    _fields_ = [("kind", C.c_int32), ("mb_id", C.c_int32), ("payload_dev", C.c_void_p),
                ("result_dev", C.c_void_p), ("ready_event", C.c_void_p),
                ("targets_dev", C.c_void_p), ("loss_dev", C.c_void_p), ("done_event", C.c_void_p)]


_vp, _i32, _i64, _u64, _f, _d = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64, C.c_float, C.c_double
_PROTOTYPES = {
    "axonn_pinned_alloc": [C.POINTER(_vp), _u64],
    "axonn_pinned_free": [_vp],
    "axonn_stage_create": [C.POINTER(axonn_stage_config), C.POINTER(_vp)],
    "axonn_stage_destroy": [_vp],
    "axonn_stage_param_count": [_vp, C.POINTER(_u64)],
    "axonn_stage_num_tensors": [_vp, C.POINTER(_i32)],
    "axonn_stage_param_layout": [_vp, _i32, C.POINTER(C.c_char_p), C.POINTER(_u64), C.POINTER(_i32), C.POINTER(_i64)],
    "axonn_stage_params": [_vp, C.POINTER(_vp)],
    "axonn_stage_grads": [_vp, C.POINTER(_vp)],
    "axonn_stage_zero_grad": [_vp, _vp],
    "axonn_stage_device_bytes": [_vp, C.POINTER(_u64)],
    "axonn_stage_forward": [_vp, _i32, _vp, _vp, _vp],
    "axonn_stage_backward": [_vp, _i32, _vp, _vp, _vp],
    "axonn_stage_post": [_vp, C.POINTER(axonn_msg)],
    "axonn_stage_run": [_vp, _i32, _vp],
    "axonn_stage_poll": [_vp, _i32, _vp, C.POINTER(_i32), C.POINTER(_i32)],
    "axonn_stage_join": [_vp, _vp],
    "axonn_stage_set_message_wait": [_vp, _d],
    "axonn_stage_synchronize": [_vp],
    "axonn_stage_dispatch_log": [_vp, C.POINTER(_i32), _i32, C.POINTER(_i32)],
    "axonn_embed_create": [_i32, _i32, _i32, _i32, _i32, C.POINTER(_vp)],
    "axonn_embed_destroy": [_vp],
    "axonn_embed_buffers": [_vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_u64)],
    "axonn_embed_zero_grad": [_vp],
    "axonn_embed_forward": [_vp, _vp, _vp, _vp],
    "axonn_embed_backward": [_vp, _vp, _vp, _vp],
    "axonn_head_create": [_i32, _i32, _i32, _i32, _i32, _f, C.POINTER(_vp)],
    "axonn_head_destroy": [_vp],
    "axonn_head_buffers": [_vp, C.POINTER(_vp), C.POINTER(_vp), C.POINTER(_u64)],
    "axonn_head_zero_grad": [_vp],
    "axonn_head_forward_backward": [_vp, _vp, _vp, _vp, _vp, _vp],
    "axonn_stage_attach_ends": [_vp, _vp, _vp],
    "axonn_offload_adam_create": [_i32, _u64, _u64, _vp, _vp, _vp, _vp, _vp, C.POINTER(_vp)],
    "axonn_offload_adam_destroy": [_vp],
    "axonn_offload_adam_step": [_vp, _d, _d, _d, _d, _d, _i64, _d, _vp],
    "axonn_offload_adam_device_bytes": [_vp, C.POINTER(_u64)],
    "axonn_stage_optimizer_attach": [_vp, _vp, _vp, _vp, _u64, _u64],
    "axonn_stage_optimizer_step": [_vp, _d, _d, _d, _d, _d, _i64, _d, _vp],
    "axonn_stage_optimizer_step_overlapped": [_vp, _d, _d, _d, _d, _d, _i64, _d, _i32, _vp],
    "axonn_count_nonfinite": [_vp, _u64, _vp, _vp],
    "axonn_stage_count_nonfinite_grads": [_vp, _vp, C.POINTER(_u64)],
    "axonn_stage_optimizer_step_scaled": [_vp, _d, _d, _d, _d, _d, _i64, _d, C.POINTER(axonn_loss_scaler), _u64, _vp,
                                          C.POINTER(_i32)],
    "axonn_head_set_loss_scale": [_vp, _f],
    "axonn_gemm_bf16": [_i32, _i32, _i32, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _i64,
                        _vp, _i64, _i32, _vp],
    "axonn_gemm_wgrad_colsum": [_i32, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _vp, _vp, _i32, _vp],
    "axonn_layernorm_fwd": [_i64, _i64, _vp, _vp, _vp, _f, _vp, _vp, _vp],
    "axonn_layernorm_bwd": [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp],
    "axonn_layernorm_bwd_noalloc": [_i64, _i64, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp],
    "axonn_colsum": [_i64, _i64, _vp, _i64, _vp, _vp, _vp],
    "axonn_attention_fwd": [_i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp],
    "axonn_attention_bwd": [_i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp],
    "axonn_profile_enable": [_i32],
    "axonn_profile_num_categories": [C.POINTER(_i32)],
    "axonn_profile_category_name": [_i32, C.POINTER(C.c_char_p)],
    "axonn_profile_collect": [C.POINTER(C.c_double), C.POINTER(_i64), _i32],
    "axonn_host_link_probe": [_i32, _u64, _i32, C.POINTER(_d)],
    "axonn_tuning": [_i32, _i64],
    "axonn_adam_bucket": [_u64, _vp, _vp, _vp, _vp, _vp, _d, _d, _d, _d, _d, _i64, _d, _vp],
}
EXPORTED_SYMBOLS = ["axonn_last_error", "axonn_element_type"] + sorted(_PROTOTYPES)

_libs = {}      # element type -> loaded library
_owner = {}     # address of a handle -> the library that created it


def load(elem=None):
    """The shared library of `elem` (default: the selected element type), loaded once.  Raises if it has not been
    built."""
    e = elem or ELEM
    lib = _libs.get(e)
    if lib is None:
        path = LIB_PATH if e == _IMPORT_ELEM else os.path.join(_HERE, _LIB_FILES[e])
        if not os.path.exists(path):
            raise ImportError("%s not found: build it with `python -m paper_2110_13005_amd.build`" % path)
        # torch brings its own HIP runtime; it must be the one already in the process when this
        # library's dependency on libamdhip64 is resolved, or the two runtimes do not share devices,
        # streams and allocations
        import torch  # noqa: F401
        lib = C.CDLL(path)          # RTLD_LOCAL: the two builds export the same names and must not see each other's
        lib.axonn_last_error.restype = C.c_char_p
        lib.axonn_last_error.argtypes = []
        for name, args in _PROTOTYPES.items():
            fn = getattr(lib, name)
            fn.restype = C.c_int
            fn.argtypes = args
        lib.axonn_element_type.restype = C.c_int32
        lib.axonn_element_type.argtypes = []
        want = 0 if e == "bf16" else 1
        if lib.axonn_element_type() != want:
            raise ImportError("%s was built for element type %d, %s needs %d: rebuild"
                              % (path, lib.axonn_element_type(), e, want))
        _libs[e] = lib
    return lib


def _ptr(x):
    """torch tensor / numpy array / int / None -> address."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "ctypes"):
        return x.ctypes.data
    if isinstance(x, C.c_void_p):
        return x.value
    raise TypeError("cannot take the address of %r" % type(x))


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream  # torch.cuda.Stream


def _addr(h):
    if isinstance(h, int):
        return h
    if isinstance(h, C.c_void_p):
        return h.value
    return None


_HANDLE_CALLS = ("axonn_stage_", "axonn_embed_", "axonn_head_", "axonn_offload_adam_")


def _call(name, *args):
    """Calls `name` in the library that owns the handle in the first argument, or in the selected one; a non-zero
    status raises with that library's message."""
    lib = None
    if args and name.startswith(_HANDLE_CALLS) and not name.endswith("_create"):
        lib = _owner.get(_addr(args[0]))
    if lib is None:
        lib = load()
    status = getattr(lib, name)(*args)
    if status != 0:
        raise AxonnError(status, lib.axonn_last_error().decode())


def _created(handle):
    _owner[_addr(handle)] = load()
    return handle


def axonn_last_error():
    return load().axonn_last_error().decode()


def axonn_pinned_alloc(nbytes):
    out = _vp()
    _call("axonn_pinned_alloc", C.byref(out), nbytes)
    return out.value


def axonn_pinned_free(host):
    _call("axonn_pinned_free", _ptr(host))


def axonn_stage_create(cfg):
    out = _vp()
    _call("axonn_stage_create", C.byref(cfg), C.byref(out))
    return _created(out.value)


def axonn_stage_destroy(st):
    _call("axonn_stage_destroy", st)
    _owner.pop(_addr(st), None)


def axonn_stage_param_count(st):
    n = _u64()
    _call("axonn_stage_param_count", st, C.byref(n))
    return n.value


def axonn_stage_num_tensors(st):
    n = _i32()
    _call("axonn_stage_num_tensors", st, C.byref(n))
    return n.value


def axonn_stage_param_layout(st, idx):
    name, off, rank = C.c_char_p(), _u64(), _i32()
    dims = (_i64 * 4)()
    _call("axonn_stage_param_layout", st, idx, C.byref(name), C.byref(off), C.byref(rank), dims)
    return name.value.decode(), off.value, tuple(dims[i] for i in range(rank.value))


def axonn_stage_params(st):
    p = _vp()
    _call("axonn_stage_params", st, C.byref(p))
    return p.value


def axonn_stage_grads(st):
    p = _vp()
    _call("axonn_stage_grads", st, C.byref(p))
    return p.value


def axonn_stage_zero_grad(st, stream=None):
    _call("axonn_stage_zero_grad", st, _stream(stream))


def axonn_stage_device_bytes(st):
    b = (_u64 * 6)()
    _call("axonn_stage_device_bytes", st, b)
    return list(b)


def axonn_stage_forward(st, mb_id, x, y, stream=None):
    _call("axonn_stage_forward", st, mb_id, _ptr(x), _ptr(y), _stream(stream))


def axonn_stage_backward(st, mb_id, dy, dx, stream=None):
    _call("axonn_stage_backward", st, mb_id, _ptr(dy), _ptr(dx), _stream(stream))


def _event(ev):
    return ev if (ev is None or isinstance(ev, int)) else ev.cuda_event


def axonn_stage_post(st, kind, mb_id, payload, result, ready_event=None, targets=None, loss=None, done_event=None):
    """ready_event / done_event: hipEvent_t handles (int) or torch.cuda.Event objects that have been recorded at
    least once (torch creates the underlying event at the first record)."""
    m = axonn_msg(kind, mb_id, _ptr(payload), _ptr(result), _event(ready_event), _ptr(targets), _ptr(loss),
                  _event(done_event))
    _call("axonn_stage_post", st, C.byref(m))


def axonn_stage_poll(st, n_streams=2, stream=None):
    """(messages dispatched by this call, messages the batch still expects)."""
    n, r = _i32(), _i32()
    _call("axonn_stage_poll", st, n_streams, _stream(stream), C.byref(n), C.byref(r))
    return n.value, r.value


def axonn_embed_create(device, vocab, hidden, seq_len, microbatch_size):
    out = _vp()
    _call("axonn_embed_create", device, vocab, hidden, seq_len, microbatch_size, C.byref(out))
    return _created(out)


def axonn_embed_destroy(e):
    _call("axonn_embed_destroy", e)
    _owner.pop(_addr(e), None)


def _buffers(name, handle):
    p, g, n = _vp(), _vp(), _u64()
    _call(name, handle, C.byref(p), C.byref(g), C.byref(n))
    return p.value, g.value, n.value


def axonn_embed_buffers(e):
    """(params pointer, grads pointer, element count)."""
    return _buffers("axonn_embed_buffers", e)


def axonn_embed_zero_grad(e):
    _call("axonn_embed_zero_grad", e)


def axonn_embed_forward(e, tokens, x, stream=None):
    _call("axonn_embed_forward", e, _ptr(tokens), _ptr(x), _stream(stream))


def axonn_embed_backward(e, tokens, dx, stream=None):
    _call("axonn_embed_backward", e, _ptr(tokens), _ptr(dx), _stream(stream))


def axonn_head_create(device, vocab, hidden, tokens_per_microbatch, n_microbatches, ln_eps=1e-5):
    out = _vp()
    _call("axonn_head_create", device, vocab, hidden, tokens_per_microbatch, n_microbatches, ln_eps, C.byref(out))
    return _created(out)


def axonn_head_destroy(hd):
    _call("axonn_head_destroy", hd)
    _owner.pop(_addr(hd), None)


def axonn_head_buffers(hd):
    """(params pointer, grads pointer, element count)."""
    return _buffers("axonn_head_buffers", hd)


def axonn_head_zero_grad(hd):
    _call("axonn_head_zero_grad", hd)


def axonn_head_forward_backward(hd, x, targets, loss, dx, stream=None):
    _call("axonn_head_forward_backward", hd, _ptr(x), _ptr(targets), _ptr(loss), _ptr(dx), _stream(stream))


def axonn_stage_attach_ends(st, embed=None, head=None):
    _call("axonn_stage_attach_ends", st, embed, head)


def axonn_stage_run(st, n_streams=2, stream=None):
    _call("axonn_stage_run", st, n_streams, _stream(stream))


def axonn_stage_join(st, stream=None):
    _call("axonn_stage_join", st, _stream(stream))


def axonn_stage_synchronize(st):
    _call("axonn_stage_synchronize", st)


def axonn_stage_dispatch_log(st, capacity=4096):
    buf = (_i32 * capacity)()
    n = _i32()
    _call("axonn_stage_dispatch_log", st, buf, capacity, C.byref(n))
    return [(buf[i] // 2, buf[i] % 2) for i in range(n.value)]


def axonn_offload_adam_create(device, n, bucket_elems, param16, grad16, host_master, host_m, host_v):
    out = _vp()
    _call("axonn_offload_adam_create", device, n, bucket_elems, _ptr(param16), _ptr(grad16),
          _ptr(host_master), _ptr(host_m), _ptr(host_v), C.byref(out))
    return _created(out.value)


def axonn_offload_adam_destroy(opt):
    _call("axonn_offload_adam_destroy", opt)
    _owner.pop(_addr(opt), None)


def axonn_offload_adam_step(opt, lr, beta1, beta2, eps, weight_decay, step, grad_scale, stream=None):
    _call("axonn_offload_adam_step", opt, lr, beta1, beta2, eps, weight_decay, step, grad_scale, _stream(stream))


def axonn_offload_adam_device_bytes(opt):
    b = _u64()
    _call("axonn_offload_adam_device_bytes", opt, C.byref(b))
    return b.value


def axonn_stage_optimizer_attach(st, host_master, host_m, host_v, n, bucket_elems):
    _call("axonn_stage_optimizer_attach", st, _ptr(host_master), _ptr(host_m), _ptr(host_v), n, bucket_elems)


def axonn_stage_optimizer_step(st, lr, beta1, beta2, eps, weight_decay, step, grad_scale, stream=None):
    _call("axonn_stage_optimizer_step", st, lr, beta1, beta2, eps, weight_decay, step, grad_scale, _stream(stream))


def axonn_stage_optimizer_step_overlapped(st, lr, beta1, beta2, eps, weight_decay, step, grad_scale, chunk_buckets,
                                          stream=None):
    _call("axonn_stage_optimizer_step_overlapped", st, lr, beta1, beta2, eps, weight_decay, step, grad_scale,
                                                        chunk_buckets, _stream(stream))


def axonn_element_type():
    return load().axonn_element_type()


def axonn_count_nonfinite(x, n, workspace, stream=None):
    _call("axonn_count_nonfinite", _ptr(x), n, _ptr(workspace), _stream(stream))


def axonn_stage_count_nonfinite_grads(st, stream=None):
    out = _u64()
    _call("axonn_stage_count_nonfinite_grads", st, _stream(stream), C.byref(out))
    return out.value


def axonn_stage_optimizer_step_scaled(st, lr, beta1, beta2, eps, weight_decay, step, grad_scale, scaler,
                                      other_nonfinite=0, stream=None):
    """scaler: an axonn_loss_scaler, updated in place.  Returns True if the step was skipped."""
    skipped = _i32()
    _call("axonn_stage_optimizer_step_scaled", st, lr, beta1, beta2, eps, weight_decay, step, grad_scale,
                                                    C.byref(scaler), other_nonfinite, _stream(stream),
                                                    C.byref(skipped))
    return bool(skipped.value)


def axonn_head_set_loss_scale(head, loss_scale):
    _call("axonn_head_set_loss_scale", head, loss_scale)


def axonn_gemm_bf16(a_kcontig, b_kcontig, epilogue, M, N, K, A, lda, B, ldb, Cmat, ldc, bias=None, res=None,
                    ld_res=0, aux=None, ld_aux=0, accumulate=0, stream=None):
    _call("axonn_gemm_bf16", a_kcontig, b_kcontig, epilogue, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(Cmat),
                                  ldc, _ptr(bias), _ptr(res), ld_res, _ptr(aux), ld_aux, accumulate, _stream(stream))


def axonn_gemm_wgrad_colsum(epilogue, M, N, K, A, lda, B, ldb, Cmat, ldc, colsum, workspace, accumulate=0, stream=None):
    _call("axonn_gemm_wgrad_colsum", epilogue, M, N, K, _ptr(A), lda, _ptr(B), ldb, _ptr(Cmat), ldc, _ptr(colsum),
                                          _ptr(workspace), accumulate, _stream(stream))


def axonn_layernorm_fwd(T, h, x, gamma, beta, eps, out, stats, stream=None):
    _call("axonn_layernorm_fwd", T, h, _ptr(x), _ptr(gamma), _ptr(beta), eps, _ptr(out), _ptr(stats), _stream(stream))


def axonn_layernorm_bwd(T, h, dout, x, stats, gamma, res_grad, dx, dgamma, dbeta, workspace, stream=None):
    _call("axonn_layernorm_bwd", T, h, _ptr(dout), _ptr(x), _ptr(stats), _ptr(gamma), _ptr(res_grad), _ptr(dx),
                                      _ptr(dgamma), _ptr(dbeta), _ptr(workspace), _stream(stream))


def axonn_layernorm_bwd_noalloc(T, h, dout, x, stats, gamma, res_grad, dx, dgamma, dbeta, stream=None):
    _call("axonn_layernorm_bwd_noalloc", T, h, _ptr(dout), _ptr(x), _ptr(stats), _ptr(gamma), _ptr(res_grad),
                                              _ptr(dx), _ptr(dgamma), _ptr(dbeta), _stream(stream))


def axonn_colsum(T, N, y, ldy, out, workspace, stream=None):
    _call("axonn_colsum", T, N, _ptr(y), ldy, _ptr(out), _ptr(workspace), _stream(stream))


def axonn_attention_fwd(b, s, n_heads, head_dim, qkv, o, lse, stream=None):
    _call("axonn_attention_fwd", b, s, n_heads, head_dim, _ptr(qkv), _ptr(o), _ptr(lse), _stream(stream))


def axonn_attention_bwd(b, s, n_heads, head_dim, qkv, o, lse, dout, dqkv, delta_ws, stream=None):
    _call("axonn_attention_bwd", b, s, n_heads, head_dim, _ptr(qkv), _ptr(o), _ptr(lse), _ptr(dout), _ptr(dqkv),
                                      _ptr(delta_ws), _stream(stream))


def axonn_adam_bucket(n, theta, m, v, grad16, param16, lr, beta1, beta2, eps, weight_decay, step, grad_scale,
                      stream=None):
    _call("axonn_adam_bucket", n, _ptr(theta), _ptr(m), _ptr(v), _ptr(grad16), _ptr(param16), lr, beta1, beta2,
                                    eps, weight_decay, step, grad_scale, _stream(stream))


TUNE_GEMM_COPY_MASK, TUNE_GEMM_BIG_MIN_TILES, TUNE_GEMM_TILE_N = 0, 1, 2


def axonn_tuning(knob, value):
    _call("axonn_tuning", knob, value)


def axonn_host_link_probe(device, n_bytes, reps):
    """(host-to-device alone, device-to-host alone, each way with both running) in GB/s."""
    out = (_d * 3)()
    _call("axonn_host_link_probe", device, n_bytes, reps, out)
    return out[0], out[1], out[2]


def axonn_stage_set_message_wait(st, seconds):
    _call("axonn_stage_set_message_wait", st, seconds)


def axonn_profile_enable(on):
    _call("axonn_profile_enable", 1 if on else 0)


def axonn_profile_num_categories():
    n = _i32()
    _call("axonn_profile_num_categories", C.byref(n))
    return n.value


def axonn_profile_category_name(idx):
    name = C.c_char_p()
    _call("axonn_profile_category_name", idx, C.byref(name))
    return name.value.decode()


def axonn_profile_collect():
    """-> {category: (total_ms, launches)}"""
    n = axonn_profile_num_categories()
    ms = (C.c_double * n)()
    cnt = (_i64 * n)()
    _call("axonn_profile_collect", ms, cnt, n)
    return {axonn_profile_category_name(i): (ms[i], cnt[i]) for i in range(n)}


def make_config(shape, pipeline_limit=None, ln_eps=1e-5, device=0, grad_accum_fp32=1, n_microbatches=None,
                wgrad_group=0, qkv_input_split=0, ckpt_stride=0):
    """axonn_stage_config from a `inputs.StageShape`."""
    M = shape.n_microbatches if n_microbatches is None else n_microbatches
    return axonn_stage_config(shape.n_layers, shape.hidden, shape.n_heads, shape.ffn, shape.seq_len,
                              shape.microbatch_size, M, M if pipeline_limit is None else pipeline_limit,
                              ln_eps, device, grad_accum_fp32, wgrad_group, qkv_input_split, ckpt_stride)
